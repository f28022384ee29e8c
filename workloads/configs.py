"""The benchmark / parity workloads: shapes, dtypes, cache parameters, value recipe."""
from __future__ import annotations

from dataclasses import dataclass, replace


@dataclass(frozen=True)
class Workload:
    name: str
    index: int            # 1..6, enters the seed
    layers: int
    batch: int
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    dtype: str            # "fp32" | "fp16" | "bf16"
    prompt: int           # N
    decode_steps: int
    sink: int             # k
    window: int           # w
    segment: int          # s
    keep: int             # survivors per segment
    evict_every: int      # T
    old_stride: int       # s^ ; 1 = survivors persist, 0 = paper default floor((s+1)/2)
    n_obs: int            # prompt queries observed for prefill scoring
    key_scale_sigma: float = 0.0   # per-token lognormal(0, sigma) key scale, shared across heads
    planted_frac: float = 0.0      # fraction of prompt keys that get +3u (u shared with queries)
    clusters: int = 0              # >0: keys/queries drawn around this many topic means per head
    cluster_noise: float = 0.3
    threshold_total: bool = False  # T bounds old + new tokens (the reading of the Parameter Estimation theorem)

    @property
    def group(self) -> int:
        return self.n_q_heads // self.n_kv_heads

    @property
    def max_context(self) -> int:
        return self.prompt + self.decode_steps

    def scaled(self, **kw) -> "Workload":
        """A copy with some fields replaced (reduced sizes for fast tests)."""
        return replace(self, **kw)


WORKLOADS = {
    "tiny": Workload("tiny", 1, 1, 1, 8, 8, 64, "fp32", 512, 256, 4, 64, 16, 1, 16, 1, 512,
                     planted_frac=0.05),
    "llama7b_layer": Workload("llama7b_layer", 2, 1, 8, 32, 32, 128, "fp16", 4096, 512, 4, 1024, 32, 4, 32, 1, 256,
                              key_scale_sigma=0.5),
    "llama7b_full": Workload("llama7b_full", 3, 32, 16, 32, 32, 128, "bf16", 16384, 256, 4, 2048, 64, 8, 64, 1, 256,
                             key_scale_sigma=0.5, planted_frac=0.02),
    "gqa8b_layer": Workload("gqa8b_layer", 4, 1, 4, 32, 8, 128, "bf16", 32768, 256, 4, 4096, 64, 8, 64, 1, 256,
                            key_scale_sigma=0.5),
    "long131k": Workload("long131k", 5, 1, 1, 32, 32, 128, "bf16", 131072, 128, 4, 8192, 128, 16, 128, 1, 256,
                         clusters=50),
    # The paper's own parameterisation on config 2's shape: stride 5, old tokens re-sampled with
    # s^ = floor((s+1)/2) = 3 at every eviction, T bounding old + new tokens and set by the Parameter
    # Estimation theorem (T / w = 26/6 = 4.33 for s = 5, w = 256), one survivor per segment.
    "llama7b_layer_paper": Workload("llama7b_layer_paper", 6, 1, 8, 32, 32, 128, "fp16", 4096, 1536, 4, 256, 5, 1,
                                    1109, 0, 256, key_scale_sigma=0.5, threshold_total=True),
}


def get_workload(name: str) -> Workload:
    if name not in WORKLOADS:
        raise KeyError(f"unknown workload {name!r}; choose from {sorted(WORKLOADS)}")
    return WORKLOADS[name]

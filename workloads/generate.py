"""Seeded generators for prompt and decode-step tensors of a :class:`Workload`.

Only random draws, scaling and dtype casts happen here; no attention, scoring or eviction arithmetic.
The same tensor (wherever it was generated) is handed to the GPU library and, widened exactly to
float64, to the CPU oracle, so both sides see identical bits.
"""
from __future__ import annotations

import torch

from .configs import Workload

_DTYPES = {"fp32": torch.float32, "fp16": torch.float16, "bf16": torch.bfloat16}


def torch_dtype(wl: Workload) -> torch.dtype:
    return _DTYPES[wl.dtype]


def seed_for(wl: Workload, layer: int = 0, stream: int = 0) -> int:
    return 0xB0220000 + 1000 * wl.index + layer + 500 * stream


def _gen(device, seed):
    g = torch.Generator(device=device)
    g.manual_seed(seed)
    return g


def _structure(wl: Workload, layer: int, device):
    """Per-head structure shared by prompt and decode draws: planted direction u and cluster means."""
    g = _gen(device, seed_for(wl, layer, stream=2))
    B, Hkv, D = wl.batch, wl.n_kv_heads, wl.head_dim
    u = torch.randn(B, Hkv, D, generator=g, device=device)
    u = u / u.norm(dim=-1, keepdim=True)
    means = None
    if wl.clusters > 0:
        means = torch.randn(B, Hkv, wl.clusters, D, generator=g, device=device)
    return u, means


def prompt_inputs(wl: Workload, layer: int = 0, device="cpu"):
    """Prompt K, V ``[B,Hkv,N,D]`` and the last ``n_obs`` prompt queries ``[B,Hq,n_obs,D]`` in ``wl.dtype``."""
    device = torch.device(device)
    g = _gen(device, seed_for(wl, layer, stream=0))
    B, Hq, Hkv, D, N, G = wl.batch, wl.n_q_heads, wl.n_kv_heads, wl.head_dim, wl.prompt, wl.group
    dt = torch_dtype(wl)
    u, means = _structure(wl, layer, device)
    K = torch.empty(B, Hkv, N, D, dtype=dt, device=device)
    V = torch.empty(B, Hkv, N, D, dtype=dt, device=device)
    for b in range(B):                                     # one batch row at a time bounds the fp32 temporaries
        k = torch.randn(Hkv, N, D, generator=g, device=device)
        if means is not None:
            cid = torch.randint(0, wl.clusters, (Hkv, N), generator=g, device=device)
            k = torch.gather(means[b], 1, cid[..., None].expand(Hkv, N, D)) + wl.cluster_noise * k
        if wl.key_scale_sigma > 0:
            z = torch.randn(N, generator=g, device=device)
            k = k * torch.exp(wl.key_scale_sigma * z)[None, :, None]
        if wl.planted_frac > 0:
            planted = torch.rand(Hkv, N, generator=g, device=device) < wl.planted_frac
            k = k + 3.0 * planted[..., None] * u[b][:, None, :]
        K[b] = k.to(dt)
        V[b] = torch.randn(Hkv, N, D, generator=g, device=device).to(dt)
    n_obs = min(wl.n_obs, N)
    q = _queries(wl, g, u, means, n_obs, device)           # [n_obs,B,Hq,D]
    q_obs = q.permute(1, 2, 0, 3).contiguous().to(dt)
    return {"K": K, "V": V, "q_obs": q_obs}


def _queries(wl, g, u, means, count, device):
    B, Hq, Hkv, D, G = wl.batch, wl.n_q_heads, wl.n_kv_heads, wl.head_dim, wl.group
    q = torch.randn(count, B, Hq, D, generator=g, device=device)
    if means is not None:
        cid = torch.randint(0, wl.clusters, (count, B, Hq), generator=g, device=device)
        mq = means.repeat_interleave(G, dim=1)             # [B,Hq,C,D]
        picked = torch.gather(mq[None].expand(count, B, Hq, wl.clusters, D), 3,
                              cid[..., None, None].expand(count, B, Hq, 1, D)).squeeze(3)
        q = picked + wl.cluster_noise * q
    if wl.planted_frac > 0:
        q = q + 3.0 * u.repeat_interleave(G, dim=1)[None]
    return q


def decode_inputs(wl: Workload, layer: int = 0, device="cpu", steps: int | None = None):
    """Per-step q ``[steps,B,Hq,D]`` and new k, v ``[steps,B,Hkv,D]`` in ``wl.dtype``."""
    device = torch.device(device)
    steps = wl.decode_steps if steps is None else steps
    g = _gen(device, seed_for(wl, layer, stream=1))
    B, Hkv, D = wl.batch, wl.n_kv_heads, wl.head_dim
    dt = torch_dtype(wl)
    u, means = _structure(wl, layer, device)
    q = _queries(wl, g, u, means, steps, device)
    k = torch.randn(steps, B, Hkv, D, generator=g, device=device)
    if means is not None:
        cid = torch.randint(0, wl.clusters, (steps, B, Hkv), generator=g, device=device)
        picked = torch.gather(means[None].expand(steps, B, Hkv, wl.clusters, D), 3,
                              cid[..., None, None].expand(steps, B, Hkv, 1, D)).squeeze(3)
        k = picked + wl.cluster_noise * k
    if wl.key_scale_sigma > 0:
        z = torch.randn(steps, B, generator=g, device=device)
        k = k * torch.exp(wl.key_scale_sigma * z)[:, :, None, None]
    v = torch.randn(steps, B, Hkv, D, generator=g, device=device)
    return {"q": q.to(dt).contiguous(), "k": k.to(dt).contiguous(), "v": v.to(dt).contiguous()}

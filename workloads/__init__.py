"""Seeded synthetic decode workloads (inputs only -- none of the method's arithmetic lives here).

These stand in for the paper's LLaMA2 / XSUM / CNN-DailyMail / Wikitext / multi-document-QA runs,
whose weights and data are not available: only the tensor shapes, dtypes, value distributions and
cache parameters of those runs are reproduced.
"""
from .configs import WORKLOADS, Workload, get_workload
from .generate import decode_inputs, prompt_inputs, seed_for

__all__ = ["WORKLOADS", "Workload", "get_workload", "prompt_inputs", "decode_inputs", "seed_for"]

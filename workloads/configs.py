"""The five seeded workloads (shapes only) the build is measured and checked on.

Shapes follow the geometries the paper evaluates (Llama-3.1-8B, a 70B-class
GQA-8 layer, Qwen-2.5-7B; page size 32; budget 2048 with sink = window = 512;
tau 0.8 for long input and 0.9 for long generation -- Sec. 5.3 "Setup" and
App. A).  Values are synthetic: the paper's datasets and weights are not used.
"""
from __future__ import annotations

import dataclasses
import math


@dataclasses.dataclass(frozen=True)
class Workload:
    name: str
    n_layers: int
    batch: int
    n_q_heads: int
    n_kv_heads: int
    dtype: str            # "fp16" | "bf16"
    ctx: int              # tokens cached before the first decode step
    budget: int           # B, tokens
    sink: int             # S, tokens
    window: int           # W, tokens
    tau: float            # correction threshold
    steps: int            # decode steps (one token appended per step)
    rho: float            # adjacent-step query correlation
    q_noise: float        # coefficient of the fresh N(0,1) term in the query recurrence
    seed: int
    placement: int = 0    # 0: whole KV in HBM, 1: whole KV in a pinned host pool
    shift_every: int = 0  # >0: every this many steps the query is a fresh draw
    head_dim: int = 128
    page_size: int = 32

    @property
    def group(self) -> int:
        return self.n_q_heads // self.n_kv_heads

    @property
    def k_pages(self) -> int:
        """Selectable pages per KV head: (B - S - W) / p."""
        return (self.budget - self.sink - self.window) // self.page_size

    @property
    def max_ctx(self) -> int:
        p = self.page_size
        return ((self.ctx + self.steps + p - 1) // p) * p

    def scaled(self, **kw) -> "Workload":
        return dataclasses.replace(self, **kw)


def _noise(rho: float) -> float:
    return math.sqrt(1.0 - rho * rho)


WORKLOADS = {
    # correctness case the oracle finishes in seconds (fp16, cache-resident)
    "c1": Workload("c1", 1, 1, 32, 8, "fp16", 4096, 512, 32, 32, 0.8, 64, 0.9, 0.44, 0),
    # headline: Llama-3-8B shape, 32K context, KV resident in HBM
    "c2": Workload("c2", 32, 1, 32, 8, "bf16", 32768, 2048, 512, 512, 0.8, 256, 0.9, _noise(0.9), 1),
    # hybrid placement: KV in pinned host memory, recall on a side stream
    "c3": Workload("c3", 32, 4, 32, 8, "bf16", 131072, 2048, 512, 512, 0.8, 128, 0.8, _noise(0.8), 2,
                   placement=1),
    # 70B-class layer shape, GQA 8
    "c4": Workload("c4", 80, 1, 64, 8, "bf16", 65536, 4096, 512, 512, 0.8, 128, 0.9, _noise(0.9), 3),
    # long generation: G = 7, context grows 2048 -> 34816, topic shift every 1024 steps
    "c5": Workload("c5", 28, 1, 28, 4, "bf16", 2048, 2048, 512, 512, 0.9, 32768, 0.7, _noise(0.7), 4,
                   shift_every=1024),
    # the paper's long-generation scenario (Sec. 5.3 "Setup": 600 tokens in, 16K out, B = 2048, S = W = 512,
    # tau = 0.9) on the Llama-3.1-8B shape with the KV pool in host memory; rho inside the similarity range the
    # paper reports (Table 8), so that a part of the heads is corrected each step as in its Table 9
    "longgen": Workload("longgen", 32, 1, 32, 8, "bf16", 600, 2048, 512, 512, 0.9, 16384, 0.93, _noise(0.93), 5,
                        placement=1),
}


def get_workload(name: str) -> Workload:
    return WORKLOADS[name.lower()]

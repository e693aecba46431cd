"""The five workload shapes the build is measured and tested on.

Shapes follow LLaMA-3-8B / Mistral-7B attention layers (32 query heads, 8 KV
heads, head_dim 128) and the paper's VQ settings "d<n>m256" (Sec. 4, Baselines):
sub-vector dim 4 / 8 / 16 with 256 centroids = 2 / 1 / 0.5 bit per element.
The anchor budget is 1 % of the context (Sec. 4, parameter settings; the paper's
own example is 82 anchors for an 8192-token context, App. G).
"""
from __future__ import annotations

import math
from dataclasses import dataclass


def anchor_count(n_ctx: int, ratio: float = 0.01) -> int:
    """Number of FP16 anchor tokens for a context of n_ctx tokens: ceil(ratio*n)."""
    return int(math.ceil(ratio * n_ctx - 1e-9))


@dataclass(frozen=True)
class Workload:
    name: str
    B: int
    N: int
    d_sub: int
    seed: int
    Nq_select: int  # query rows used by anchor selection (N = prefill form)
    Hq: int = 32
    Hkv: int = 8
    D: int = 128
    C: int = 256
    description: str = ""

    @property
    def M(self) -> int:
        return self.D // self.d_sub

    @property
    def G(self) -> int:
        return self.Hq // self.Hkv

    @property
    def k(self) -> int:
        return anchor_count(self.N)

    @property
    def scale(self) -> float:
        return 1.0 / math.sqrt(self.D)

    @property
    def bits_per_element(self) -> float:
        return math.log2(self.C) / self.d_sub


CONFIGS = {
    "cfg0": Workload("cfg0", B=1, N=4096, d_sub=8, seed=0, Nq_select=4096,
                     description="tiny decode step, 1-bit VQ, 41 anchors"),
    "cfg1": Workload("cfg1", B=1, N=32768, d_sub=4, seed=1, Nq_select=32768,
                     description="LLaMA3-8B-shaped decode layer, 2-bit VQ, 328 anchors"),
    "cfg2": Workload("cfg2", B=4, N=131072, d_sub=8, seed=2, Nq_select=32,
                     description="long-context batched decode, 1-bit VQ, 1311 anchors per sequence"),
    "cfg3": Workload("cfg3", B=1, N=32768, d_sub=8, seed=3, Nq_select=32768,
                     description="prefill encode + anchor selection over a 32768-token prompt"),
    "cfg4": Workload("cfg4", B=1, N=840000, d_sub=16, seed=4, Nq_select=32,
                     description="Mistral-7B-shaped 840K context, 0.5-bit VQ, 8400 anchors, re-selection"),
}

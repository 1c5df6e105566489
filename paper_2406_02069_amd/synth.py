"""Seeded synthetic inputs shaped like the paper's workloads.

This module serves both the tests (which feed the same bits to the CPU oracle
and to the HIP library) and the benchmark.  It holds none of the method's
arithmetic: only random draws, the planted structure (attention sink, needle
keys, per-channel outlier scales, ragged lengths) and the shapes of the five
workloads (LLaMA-3-8B / 70B and Mistral-7B head geometry, 8k-32k contexts,
cache sizes 64-2048, alpha 8-64, beta 20; Sec. 5.1 and the ablations of the
paper).  The datasets and trained weights of the paper's experiments are not
used; these tensors stand in for them.
"""
from __future__ import annotations

import dataclasses
from typing import List, Optional, Tuple

import numpy as np
import torch

BASE_SEED = 240602069

POOL_NONE, POOL_MAX, POOL_AVG = 0, 1, 2


@dataclasses.dataclass(frozen=True)
class Workload:
    name: str
    index: int            # position in the configs list; enters the seed
    B: int
    L: int
    Hq: int
    Hkv: int
    d: int
    N: int
    alpha: int
    avg_budgets: Tuple[int, ...]
    beta: int
    pool: int
    pool_w: int
    sink: bool = False
    needles: int = 0
    needle_depths: str = "spaced"      # "spaced": >= 8 apart in [64, N-alpha-64); "uniform": U[0,1)*(N-alpha)
    channel_outliers: bool = False     # keys scaled per channel by LogNormal(0,1)
    ragged_min: Optional[int] = None   # per-sequence lengths ~ U{ragged_min..N}

    @property
    def G(self) -> int:
        return self.Hq // self.Hkv

    def scaled(self, **kw) -> "Workload":
        """Same structure at another size (tests that must finish on a CPU)."""
        return dataclasses.replace(self, **kw)


WORKLOADS: List[Workload] = [
    Workload("tiny-mha", 0, B=1, L=4, Hq=8, Hkv=8, d=64, N=1024, alpha=8, avg_budgets=(128,), beta=20,
             pool=POOL_MAX, pool_w=7, sink=True),
    Workload("llama3-8b-8k", 1, B=1, L=32, Hq=32, Hkv=8, d=128, N=8192, alpha=8, avg_budgets=(128,), beta=20,
             pool=POOL_MAX, pool_w=7, sink=True, needles=16),
    Workload("llama3-8b-32k", 2, B=1, L=32, Hq=32, Hkv=8, d=128, N=32768, alpha=32,
             avg_budgets=(128, 64, 512, 2048), beta=20, pool=POOL_AVG, pool_w=5, sink=True, needles=16),
    Workload("mistral-7b-ragged", 3, B=8, L=32, Hq=32, Hkv=8, d=128, N=16384, alpha=16, avg_budgets=(256,),
             beta=20, pool=POOL_MAX, pool_w=7, channel_outliers=True, ragged_min=8192),
    Workload("llama3-70b-32k", 4, B=1, L=80, Hq=64, Hkv=8, d=128, N=32768, alpha=64, avg_budgets=(128,), beta=20,
             pool=POOL_MAX, pool_w=7, sink=True, needles=16, needle_depths="uniform"),
]


# Beside the five configurations above: multi-head attention (G = 1, so only alpha = 8 query rows share a head's keys)
# at a long context, the shape on which padding the query rows to a 32-row MFMA tile wastes the most exponentials.
# A measurement shape (bench.py --config 5), not one of the parity configurations.
EXTRA_WORKLOADS: List[Workload] = [
    Workload("mha-32k", 5, B=1, L=8, Hq=32, Hkv=32, d=128, N=32768, alpha=8, avg_budgets=(128,), beta=20,
             pool=POOL_MAX, pool_w=7, sink=True, needles=16),
]


def _seed(w: Workload, layer: int, stream: int) -> int:
    return (BASE_SEED + w.index) * 1_000_003 + layer * 101 + stream


def seq_lens(w: Workload) -> Optional[np.ndarray]:
    """Valid lengths n_b of the batch (None: every sequence has N tokens).  Same for all layers."""
    if w.ragged_min is None:
        return None
    rs = np.random.RandomState((BASE_SEED + w.index) % (2**31))
    lo = min(w.ragged_min, w.N)
    return rs.randint(lo, w.N + 1, size=w.B).astype(np.int32)


def needle_plan(w: Workload, layer: int, lens: Optional[np.ndarray]):
    """[(b, g, position, h, t)]: key (b,g,position) is set to 2*Q_win[b,h,t]."""
    if w.needles <= 0:
        return []
    rs = np.random.RandomState(_seed(w, layer, 7) % (2**31))
    plan = []
    for b in range(w.B):
        n = int(lens[b]) if lens is not None else w.N
        npre = n - w.alpha
        pos: List[int] = []
        if w.needle_depths == "uniform":
            while len(pos) < w.needles and len(pos) < max(npre - 1, 0):
                p = int(rs.random_sample() * npre)
                if 0 < p < npre and p not in pos:
                    pos.append(p)
        else:
            lo, hi = (64, npre - 64) if npre > 64 * 2 + 8 * w.needles * 4 else (1, npre)
            tries = 0
            while len(pos) < w.needles and tries < 100000:
                tries += 1
                p = int(rs.randint(lo, max(hi, lo + 1)))
                if all(abs(p - o) >= 8 for o in pos) and p < npre:
                    pos.append(p)
        for i, p in enumerate(pos):
            g = i % w.Hkv
            h = g * w.G + (i // w.Hkv) % w.G
            t = i % w.alpha
            plan.append((b, g, p, h, t))
    return plan


def make_layer(w: Workload, layer: int, device="cpu"):
    """Q_win [B,Hq,alpha,d], K, V [B,Hkv,N,d] (bf16, contiguous, on `device`) of one layer.

    Returns (Q_win, K, V, lens) with lens an int32 numpy array or None."""
    dev = torch.device(device)
    g = torch.Generator(device=dev)
    lens = seq_lens(w)

    def normal(shape, stream):
        g.manual_seed(_seed(w, layer, stream))
        return torch.randn(shape, generator=g, device=dev, dtype=torch.float32)

    Q = normal((w.B, w.Hq, w.alpha, w.d), 1).to(torch.bfloat16)
    Kf = normal((w.B, w.Hkv, w.N, w.d), 2)
    if w.channel_outliers:
        g.manual_seed(_seed(w, layer, 4))
        s = torch.exp(torch.randn((1, w.Hkv, 1, w.d), generator=g, device=dev, dtype=torch.float32))
        Kf = Kf * s
    K = Kf.to(torch.bfloat16)
    del Kf
    V = normal((w.B, w.Hkv, w.N, w.d), 3).to(torch.bfloat16)
    if w.sink:
        K[:, :, 0, :] = K[:, :, 0, :] * 8
    for (b, gg, p, h, t) in needle_plan(w, layer, lens):
        K[b, gg, p, :] = Q[b, h, t, :] * 2
    if lens is not None:
        nan = torch.tensor(float("nan"), dtype=torch.bfloat16, device=dev)
        for b in range(w.B):
            K[b, :, int(lens[b]):, :] = nan
            V[b, :, int(lens[b]):, :] = nan
    return Q.contiguous(), K.contiguous(), V.contiguous(), lens

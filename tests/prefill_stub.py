"""Stand-in for the prefill attention kernel that would hand its softmax statistics to pkv_compress_layers_lse.

Not part of the compression path: it produces an INPUT of that entry point (like synth.py produces Q, K, V) with
plain torch ops, in fp64, rounded once to fp32.  Tests and the benchmark call it outside any timed region.
"""
from __future__ import annotations

import math
from typing import Optional

import torch


def window_lse(Q_win: torch.Tensor, K: torch.Tensor, seq_lens=None) -> torch.Tensor:
    """ln sum_{i <= n_b - alpha + t} exp(q_{b,h,t} . k_{b,g(h),i} / sqrt(d)) for every window query.

    Q_win [B,Hq,alpha,d], K [B,Hkv,N,d] (bf16); seq_lens: None or B ints.  Returns fp32 [B,Hq,alpha] on K's
    device; rows of sequences shorter than the window are NaN (such sequences are kept whole, never scored)."""
    B, Hq, alpha, d = Q_win.shape
    Hkv, N = K.shape[1], K.shape[2]
    G = Hq // Hkv
    out = torch.full((B, Hq, alpha), float("nan"), dtype=torch.float64, device=K.device)
    for b in range(B):
        n = N if seq_lens is None else int(seq_lens[b])
        if n < alpha:
            continue
        pos = torch.arange(n, device=K.device)[None, :]
        last = (n - alpha + torch.arange(alpha, device=K.device)).repeat(G)[:, None]   # row r = h * alpha + t
        for g in range(Hkv):
            q = Q_win[b, g * G:(g + 1) * G].reshape(G * alpha, d).double()
            logits = (q @ K[b, g, :n].double().T) / math.sqrt(d)
            logits = logits.masked_fill(pos > last, float("-inf"))
            out[b, g * G:(g + 1) * G] = torch.logsumexp(logits, dim=1).reshape(G, alpha)
    return out.float()

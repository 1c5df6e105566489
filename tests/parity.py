"""Comparison of one layer's HIP result with the CPU oracle (shared by the GPU tests and the smoke check).

Protocol (fp32 device scores vs. fp64 oracle scores):
  * pooled scores agree within 1e-4 relative (+1e-30 absolute: fp32 flushes below its normal range);
  * the device's kept set is exactly the top-k (value desc, position asc) of the device's own scores,
    followed by the window -- checked with the oracle's selection routine, bit for bit;
  * the kept set equals the oracle's bit for bit, unless the oracle scores within 1e-5 relative of its k-th
    value (the cut) take at least two distinct values (a near-tie that fp32 cannot resolve; with max pooling
    the plateaus of two neighbouring sources can adjoin at the cut, so that the k-th and (k+1)-th values are
    equal and the next distinct one is a hair away); then the two sets may differ only in positions inside
    that band.  A band with a single value is an exact tie: the lower position wins, on both sides alike;
  * K_out / V_out rows are bit copies of K / V at the device's kept positions, and equal the oracle's
    K_out / V_out bit for bit whenever the kept sets agree.
"""
from __future__ import annotations

import numpy as np
import torch

from oracle import pkv_oracle

SCORE_RTOL = 1e-4
SCORE_FLOOR = 1e-30
TIE_RTOL = 1e-5


def bits(t: torch.Tensor) -> np.ndarray:
    return t.detach().cpu().contiguous().view(torch.int16).numpy().view(np.uint16)


def compare_layer(Q, K, V, k_l, alpha, pool, pool_w, lens, gpu, ref=None, check_scores=True):
    """gpu = (K_out, V_out, idx, count, scores) torch tensors from the library.  Returns a stats dict."""
    Kb, Vb = bits(K), bits(V)
    B, Hkv, N, d = Kb.shape
    if ref is None:
        ref = pkv_oracle.compress_layer(Q, K, V, k_l, alpha, pool, pool_w, seq_lens=lens)
    gK, gV = bits(gpu[0]), bits(gpu[1])
    gidx = gpu[2].cpu().numpy()
    gcount = gpu[3].cpu().numpy()
    gsc = gpu[4].cpu().numpy().astype(np.float64) if gpu[4] is not None else None
    stats = dict(units=0, near_tie_units=0, below_floor=0, max_rel_err=0.0)
    np.testing.assert_array_equal(gcount, ref["count"])
    for b in range(B):
        n = int(lens[b]) if lens is not None else N
        c = int(ref["count"][b])
        for g in range(Hkv):
            stats["units"] += 1
            gi = gidx[b, g]
            # rows beyond count: -1 / zeros
            assert np.all(gi[c:] == -1), (b, g)
            assert np.all(gK[b, g, c:] == 0) and np.all(gV[b, g, c:] == 0), (b, g)
            gi = gi[:c]
            assert np.all(np.diff(gi) > 0) if c > 1 else True, (b, g, "positions not ascending")
            assert c == 0 or (gi[0] >= 0 and gi[-1] < n), (b, g)
            # gathered rows are bit copies at the device's own indices
            np.testing.assert_array_equal(gK[b, g, :c], Kb[b, g, gi])
            np.testing.assert_array_equal(gV[b, g, :c], Vb[b, g, gi])
            ri = ref["idx"][b, g, :c]
            if k_l >= n:
                np.testing.assert_array_equal(gi, ri)
                continue
            npre, kk = n - alpha, k_l - alpha
            np.testing.assert_array_equal(gi[kk:], np.arange(npre, n))       # window kept, last
            rp = ref["pooled"][b, g, :npre]
            if gsc is not None:
                gp = gsc[b, g, :npre]
                if check_scores:
                    err = np.abs(gp - rp)
                    bad = err > SCORE_RTOL * np.abs(rp) + SCORE_FLOOR
                    assert not bad.any(), (b, g, int(bad.sum()), float((err / np.maximum(rp, 1e-300)).max()))
                    big = rp > SCORE_FLOOR / SCORE_RTOL
                    if big.any():
                        stats["max_rel_err"] = max(stats["max_rel_err"], float((err[big] / rp[big]).max()))
                    stats["below_floor"] += int((~big).sum())
                # selection is exact on the device's own scores
                own = pkv_oracle.topk(gp, kk)
                np.testing.assert_array_equal(gi[:kk], own)
            if np.array_equal(gi, ri):
                np.testing.assert_array_equal(gK[b, g, :c], ref["K_out"][b, g, :c])
                np.testing.assert_array_equal(gV[b, g, :c], ref["V_out"][b, g, :c])
                continue
            # sets differ: only allowed at an unresolved near-tie of the cut
            order = np.lexsort((np.arange(npre), -rp))
            vk, vk1 = rp[order[kk - 1]], rp[order[kk]]
            band = np.abs(rp - vk) <= TIE_RTOL * vk
            assert np.unique(rp[band]).size >= 2, (b, g, "kept set differs without a near-tie", vk, vk1)
            diff = np.setxor1d(gi[:kk], ri[:kk])
            assert np.all(band[diff]), (b, g, "difference outside the near-tie band")
            stats["near_tie_units"] += 1
    return stats

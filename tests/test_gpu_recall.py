"""Attention recall rate of the kept sets (pkv_attention_recall) vs. the CPU oracle's direct definition, for every
(sequence, KV head), on both scoring paths and both scoring variants."""
import numpy as np
import pytest
import torch

from oracle import pkv_oracle
from paper_2406_02069_amd import binding, synth
from tests import prefill_stub

pytestmark = pytest.mark.gpu
DEV = "cuda:0"
ATOL = 2e-5   # fp32 window scores (1e-5 relative of a mass <= alpha, divided by alpha) and their fp32 sums


def _rand(B, Hq, Hkv, d, N, alpha, seed, scale=1.0):
    g = torch.Generator(device=DEV).manual_seed(seed)
    Q = (torch.randn(B, Hq, alpha, d, generator=g, device=DEV) * scale).to(torch.bfloat16)
    K = torch.randn(B, Hkv, N, d, generator=g, device=DEV).to(torch.bfloat16)
    V = torch.randn(B, Hkv, N, d, generator=g, device=DEV).to(torch.bfloat16)
    return Q, K, V


def _check(Qs, Ks, Vs, k_ls, alpha, pool, pw, lens=None, use_lse=False):
    L = len(Ks)
    B, Hkv, N, d = Ks[0].shape
    G = Qs[0].shape[1] // Hkv
    lens_dev = None if lens is None else torch.from_numpy(np.asarray(lens, dtype=np.int32)).to(DEV)
    lses = [prefill_stub.window_lse(Qs[l], Ks[l], lens) for l in range(L)] if use_lse else None
    call = binding.LayersCall(Qs, Ks, Vs, k_ls, pool, pw, seq_lens=lens_dev, lse=lses)
    outs = call.run()
    rec = binding.attention_recall(call)
    torch.cuda.synchronize()
    worst = 0.0
    for l in range(L):
        idx = outs[l][2].cpu().numpy()
        count = outs[l][3].cpu().numpy()
        got = rec[l].cpu().numpy()
        for b in range(B):
            n = N if lens is None else int(lens[b])
            for g in range(Hkv):
                if k_ls[l] >= n:
                    assert got[b, g] == 1.0
                    continue
                want = pkv_oracle.attention_recall(Qs[l][b, g * G:(g + 1) * G], Ks[l][b, g, :n], idx[b, g, : count[b]])
                assert abs(got[b, g] - want) <= ATOL, (l, b, g, got[b, g], want)
                worst = max(worst, abs(got[b, g] - want))
    return worst


@pytest.mark.parametrize("path", ["resident", "stream"])
@pytest.mark.parametrize("use_lse", [False, True])
def test_recall_matches_the_definition(path, use_lse, monkeypatch):
    monkeypatch.setattr(binding, "DESC_FLAGS", binding.FLAG_STREAM_SCORING if path == "stream" else 0)
    alpha = 8
    Q, K, V = _rand(3, 8, 2, 128, 1300, alpha, seed=3, scale=2.0)
    lens = np.array([1300, 600, 5], dtype=np.int32)
    ks = [alpha, 40, 200, 700, 5000]
    L = len(ks)
    print("recall", path, use_lse, flush=True)
    _check([Q] * L, [K] * L, [V] * L, ks, alpha, synth.POOL_MAX, 7, lens=lens, use_lse=use_lse)


@pytest.mark.parametrize("path", ["resident", "stream"])
def test_recall_wide_groups_and_d64(path, monkeypatch):
    monkeypatch.setattr(binding, "DESC_FLAGS", binding.FLAG_STREAM_SCORING if path == "stream" else 0)
    for (d, Hq, Hkv, alpha, N) in [(64, 12, 4, 5, 900), (128, 64, 8, 32, 700), (64, 16, 2, 64, 500)]:
        print("recall geometry", path, d, Hq, Hkv, alpha, N, flush=True)
        Q, K, V = _rand(2, Hq, Hkv, d, N, alpha, seed=d + Hq)
        _check([Q, Q], [K, K], [V, V], [alpha + 30, alpha + 200], alpha, synth.POOL_AVG, 5)


def test_recall_grows_with_the_budget_and_more_layers_than_one_launch():
    alpha = 4
    Q, K, V = _rand(1, 4, 2, 64, 600, alpha, seed=8)
    ks = [alpha + 5 * i for i in range(50)]                  # 50 layers: two launches of the recall kernel
    call = binding.LayersCall([Q] * 50, [K] * 50, [V] * 50, ks, synth.POOL_NONE, 1)
    call.run()
    rec = torch.stack(binding.attention_recall(call)).cpu().numpy()   # [50, 1, 2]
    torch.cuda.synchronize()
    assert np.all(np.diff(rec, axis=0) >= -1e-6)             # un-pooled scores: nested kept sets, recall monotone
    assert rec[0].max() < rec[-1].min() <= 1.0

"""Contexts beyond 32k (the appendix discusses up to 128k): units that span 128, 256 or all 512 workgroups of the
persistent scoring kernel, prefixes too long for the in-LDS selection (radix select over keys in global memory),
the largest length the register-resident kernel takes (262 144) and one beyond it (streaming kernels).  HIP
library vs. CPU oracle, element by element, through the C ABI (needs an MI355X)."""
import numpy as np
import pytest
import torch

from oracle import pkv_oracle
from paper_2406_02069_amd import binding, synth
from tests import prefill_stub
from tests.parity import compare_layer

pytestmark = pytest.mark.gpu
DEV = "cuda:0"
B, HQ, HKV, D, ALPHA = 1, 8, 2, 128, 32   # G * alpha = 128 query rows per KV head, as in the 32k workload


def _layers(L, N, seed, B=B):
    g = torch.Generator(device=DEV).manual_seed(seed)
    Qs = [torch.randn(B, HQ, ALPHA, D, generator=g, device=DEV).to(torch.bfloat16) for _ in range(L)]
    Ks = [torch.randn(B, HKV, N, D, generator=g, device=DEV).to(torch.bfloat16) for _ in range(L)]
    Vs = [torch.randn(B, HKV, N, D, generator=g, device=DEV).to(torch.bfloat16) for _ in range(L)]
    for K, Q in zip(Ks, Qs):   # a sink and a few needles, so that the kept set is not all noise
        K[:, :, 0] *= 8
        for i, p in enumerate((N // 7, N // 3, N - ALPHA - 40)):
            K[0, i % HKV, p] = (Q[0, (i % HKV) * (HQ // HKV) + 1, 5 + i].float() * 2).to(torch.bfloat16)
    return Qs, Ks, Vs


# N -> parts of 512 keys per unit, workgroups per group, groups:
#   40000 -> 79, 128, 4 (49 workgroups of every group idle) | 100000 -> 196, 256, 2 | 131072 -> 256, 256, 2
#   200001 -> 391, 512, 1 (ragged last tile) | 262144 -> 512, 512, 1 (every workgroup one part)
@pytest.mark.parametrize("N", [40000, 100000, 131072, 200001, 262144])
def test_two_sweeps_long_context(N):
    L = 3   # 6 units: every group works through more than one
    Qs, Ks, Vs = _layers(L, N, seed=N % 1000)
    ks = [1200, ALPHA + 300, ALPHA + 17]
    outs = binding.compress_layers(Qs, Ks, Vs, ks, synth.POOL_MAX, 7, want_scores=True)
    torch.cuda.synchronize()
    for l in (0, L - 1):
        print("long context N", N, "layer", l, flush=True)
        st = compare_layer(Qs[l], Ks[l], Vs[l], ks[l], ALPHA, synth.POOL_MAX, 7, None, outs[l])
        assert st["near_tie_units"] <= 1
        kept = outs[l][2].cpu().numpy()
        assert 0 in kept[0, 0] and N // 7 in kept[0, 0] and N // 3 in kept[0, 1]


@pytest.mark.parametrize("N", [40000, 131072, 262144])
def test_ragged_batch_long_context(N):
    # sequence lengths differ: the arrival counter instead of the tagged exchange, parts beyond a sequence's end
    lens = np.array([N, (N * 5) // 8 + 3], dtype=np.int32)
    Qs, Ks, Vs = _layers(2, N, seed=7 + N % 1000, B=2)
    for K in Ks:
        K[1, :, int(lens[1]):] = float("nan")   # never read
    ks = [700, ALPHA + 50]
    outs = binding.compress_layers(Qs, Ks, Vs, ks, synth.POOL_AVG, 5, seq_lens=torch.from_numpy(lens).to(DEV),
                                   want_scores=True)
    torch.cuda.synchronize()
    for l in range(2):
        print("ragged long context N", N, "layer", l, flush=True)
        compare_layer(Qs[l], Ks[l], Vs[l], ks[l], ALPHA, synth.POOL_AVG, 5, lens, outs[l])


@pytest.mark.parametrize("N", [100000, 262144])
def test_supplied_denominators_long_context(N):
    Qs, Ks, Vs = _layers(2, N, seed=11 + N % 1000)
    lses = [prefill_stub.window_lse(Q, K, None) for Q, K in zip(Qs, Ks)]
    ks = [900, ALPHA + 64]
    outs = binding.compress_layers_lse(Qs, Ks, Vs, lses, ks, synth.POOL_MAX, 7, want_scores=True)
    torch.cuda.synchronize()
    for l in range(2):
        print("lse long context N", N, "layer", l, flush=True)
        ref = pkv_oracle.compress_layer(Qs[l], Ks[l], Vs[l], ks[l], ALPHA, synth.POOL_MAX, 7,
                                        lse=lses[l].cpu().numpy())
        compare_layer(Qs[l], Ks[l], Vs[l], ks[l], ALPHA, synth.POOL_MAX, 7, None, outs[l], ref=ref)


def test_beyond_the_resident_limit_streams():
    N = 270000   # more than 512 parts of 512 keys: the per-layer streaming kernels take over
    Qs, Ks, Vs = _layers(1, N, seed=3)
    out = binding.compress_layer(Qs[0], Ks[0], Vs[0], 500, synth.POOL_MAX, 7, want_scores=True)
    torch.cuda.synchronize()
    compare_layer(Qs[0], Ks[0], Vs[0], 500, ALPHA, synth.POOL_MAX, 7, None, out)


def _small(N, alpha, seed, B=1, Hq=2, Hkv=2, d=64):
    g = torch.Generator(device=DEV).manual_seed(seed)
    Q = torch.randn(B, Hq, alpha, d, generator=g, device=DEV).to(torch.bfloat16)
    K = torch.randn(B, Hkv, N, d, generator=g, device=DEV).to(torch.bfloat16)
    V = torch.randn(B, Hkv, N, d, generator=g, device=DEV).to(torch.bfloat16)
    return Q, K, V


@pytest.mark.parametrize("pool,pw", [(synth.POOL_NONE, 1), (synth.POOL_MAX, 63), (synth.POOL_AVG, 9), (synth.POOL_MAX, 3)])
def test_long_prefix_selection_edges(pool, pw):
    # the selection of prefixes beyond 32768 keys: smallest and largest budgets, a pool as wide as a tile's halo
    # allows, lengths around the tile size of the pooling (16384) and the per-wave ranges of the emission
    alpha = 8
    for N, k_ls in ((32768 + alpha + 1, (alpha + 1, 500)), (49152 + alpha, (alpha + 1, 49152 + alpha - 1)),
                    (40001, (alpha, 3000, 40000, 40001))):
        Q, K, V = _small(N, alpha, seed=N % 97 + pw)
        for k_l in k_ls:
            print("long selection", pool, pw, "N", N, "k_l", k_l, flush=True)
            out = binding.compress_layer(Q, K, V, k_l, pool, pw, want_scores=True)
            torch.cuda.synchronize()
            compare_layer(Q, K, V, k_l, alpha, pool, pw, None, out)


def test_long_prefix_with_equal_scores():
    # identical keys: every prefix key gets the same score, the cut falls inside one plateau that spans the whole
    # prefix, and the lowest positions win; then two plateaus (a block of keys that scores higher)
    alpha, N = 8, 36000
    Q, K, V = _small(N, alpha, seed=5)
    K[:] = K[:, :, :1]
    out = binding.compress_layer(Q, K, V, alpha + 1000, synth.POOL_NONE, 1, want_scores=True)
    torch.cuda.synchronize()
    compare_layer(Q, K, V, alpha + 1000, alpha, synth.POOL_NONE, 1, None, out)
    assert out[2][0, 0, :1000].cpu().tolist() == list(range(1000))
    K[:, :, 20000:20300] = (Q[:, :1, 3:4].float() * 0.5).to(torch.bfloat16)
    out = binding.compress_layer(Q, K, V, alpha + 1000, synth.POOL_NONE, 1, want_scores=True)
    torch.cuda.synchronize()
    compare_layer(Q, K, V, alpha + 1000, alpha, synth.POOL_NONE, 1, None, out)


def test_long_prefix_with_non_finite_scores_stays_in_bounds():
    alpha, N, k_l = 8, 40000, 300
    Q, K, V = _small(N, alpha, seed=6)
    K[0, 0, 1234] = float("nan")
    out = binding.compress_layer(Q, K, V, k_l, synth.POOL_MAX, 7, want_scores=True)
    torch.cuda.synchronize()
    idx = out[2].cpu().numpy()
    assert out[3].cpu().tolist() == [k_l]
    for g in range(2):
        row = idx[0, g]
        assert row.min() >= 0 and row.max() < N and np.all(np.diff(row) > 0), g
        assert row[-alpha:].tolist() == list(range(N - alpha, N)), g
    Kc = K.clone()
    Kc[0, 0, 1234] = 0
    ref = binding.compress_layer(Q, Kc, V, k_l, synth.POOL_MAX, 7, want_scores=True)
    torch.cuda.synchronize()
    assert np.array_equal(idx[0, 1], ref[2][0, 1].cpu().numpy())   # the other head is unaffected


@pytest.mark.parametrize("d,Hq,Hkv,alpha,N", [(64, 16, 2, 64, 70000),    # 512 query rows per KV head: four row blocks
                                              (128, 4, 4, 8, 50000),     # 8 rows: padded row tile, MHA
                                              (64, 6, 2, 37, 33000)])    # odd window, just beyond the in-LDS selection
def test_other_geometries_long_context(d, Hq, Hkv, alpha, N):
    g = torch.Generator(device=DEV).manual_seed(N + d)
    Q = torch.randn(1, Hq, alpha, d, generator=g, device=DEV).to(torch.bfloat16)
    K = torch.randn(1, Hkv, N, d, generator=g, device=DEV).to(torch.bfloat16)
    V = torch.randn(1, Hkv, N, d, generator=g, device=DEV).to(torch.bfloat16)
    k_l = alpha + 333
    out = binding.compress_layer(Q, K, V, k_l, synth.POOL_MAX, 7, want_scores=True)
    torch.cuda.synchronize()
    compare_layer(Q, K, V, k_l, alpha, synth.POOL_MAX, 7, None, out)
    lse = prefill_stub.window_lse(Q, K, None)
    out = binding.compress_layers_lse([Q], [K], [V], [lse], [k_l], synth.POOL_AVG, 5, want_scores=True)[0]
    torch.cuda.synchronize()
    ref = pkv_oracle.compress_layer(Q, K, V, k_l, alpha, synth.POOL_AVG, 5, lse=lse.cpu().numpy())
    compare_layer(Q, K, V, k_l, alpha, synth.POOL_AVG, 5, None, out, ref=ref)

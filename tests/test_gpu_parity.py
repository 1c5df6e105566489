"""HIP library vs. CPU oracle, element by element, through the C ABI (needs an MI355X)."""
import numpy as np
import pytest
import torch

from oracle import pkv_oracle
from paper_2406_02069_amd import binding, synth
from tests.parity import bits, compare_layer

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


@pytest.fixture(params=["resident", "stream"])
def score_path(request, monkeypatch):
    """Both scoring implementations: K held in registers (default) and the per-layer streaming kernels."""
    monkeypatch.setattr(binding, "DESC_FLAGS", binding.FLAG_STREAM_SCORING if request.param == "stream" else 0)
    return request.param


def _lens_dev(lens):
    return None if lens is None else torch.from_numpy(np.asarray(lens, dtype=np.int32)).to(DEV)


def _run_and_compare(w, layer, k_l, Q=None, K=None, V=None, lens=None, check_scores=True):
    if Q is None:
        Q, K, V, lens = synth.make_layer(w, layer, DEV)
    out = binding.compress_layer(Q, K, V, k_l, w.pool, w.pool_w, seq_lens=_lens_dev(lens), want_scores=True)
    torch.cuda.synchronize()
    return compare_layer(Q, K, V, k_l, w.alpha, w.pool, w.pool_w, lens, out, check_scores=check_scores), out


def _rand(B, Hq, Hkv, d, N, alpha, seed):
    g = torch.Generator(device=DEV).manual_seed(seed)
    Q = torch.randn(B, Hq, alpha, d, generator=g, device=DEV).to(torch.bfloat16)
    K = torch.randn(B, Hkv, N, d, generator=g, device=DEV).to(torch.bfloat16)
    V = torch.randn(B, Hkv, N, d, generator=g, device=DEV).to(torch.bfloat16)
    return Q, K, V


class _W:  # minimal stand-in for a workload in ad-hoc cases
    def __init__(self, alpha, pool, pool_w):
        self.alpha, self.pool, self.pool_w = alpha, pool, pool_w


def test_config0_tiny_mha_all_layers(score_path):
    w = synth.WORKLOADS[0]
    ks = binding.budgets(w.L, w.avg_budgets[0], w.beta, w.alpha)
    assert ks == [242, 166, 90, 14]
    for layer in range(w.L):
        print("config0 layer", layer, flush=True)
        st, _ = _run_and_compare(w, layer, ks[layer])
        assert st["units"] == 8


@pytest.mark.parametrize("cfg,N", [(1, 1500), (1, 4099), (2, 2500), (4, 1111)])
def test_scaled_configs_ragged_tiles(cfg, N, score_path):
    # several key tiles, several chunks, a ragged tail (N not a multiple of 32), every row-block shape
    w = synth.WORKLOADS[cfg].scaled(N=N, L=3)
    ks = binding.budgets(w.L, w.avg_budgets[0], w.beta, w.alpha)
    for layer in range(w.L):
        print("scaled config", cfg, "N", N, "layer", layer, flush=True)
        _run_and_compare(w, layer, ks[layer])


def test_config3_scaled_ragged_batch_with_nan_padding(score_path):
    w = synth.WORKLOADS[3].scaled(N=3000, ragged_min=700, B=4)
    ks = binding.budgets(w.L, w.avg_budgets[0], w.beta, w.alpha)
    for layer, k_l in ((0, ks[0]), (1, ks[-1]), (2, 900)):     # 900 > some n_b: those keep everything
        print("config3 scaled layer", layer, flush=True)
        st, out = _run_and_compare(w, layer, k_l)
        assert not torch.isnan(out[4]).any()


@pytest.mark.parametrize("d,Hq,Hkv,alpha", [(64, 8, 8, 8), (64, 16, 2, 8), (64, 12, 4, 5), (128, 4, 4, 1),
                                             (128, 28, 4, 16), (128, 64, 8, 64), (64, 6, 2, 37)])
def test_head_geometries(d, Hq, Hkv, alpha, score_path):
    Q, K, V = _rand(2, Hq, Hkv, d, 777, alpha, seed=d + Hq + alpha)
    for pool, pw in ((synth.POOL_MAX, 7), (synth.POOL_AVG, 5), (synth.POOL_NONE, 1), (synth.POOL_MAX, 63)):
        print("geometry", d, Hq, Hkv, alpha, pool, pw, flush=True)
        _run_and_compare(_W(alpha, pool, pw), 0, alpha + 100, Q, K, V)


def test_more_query_rows_per_kv_head_than_the_resident_kernels_hold():
    # G * alpha = 16 * 64 = 1024 > 512: the per-layer streaming kernels take the call whatever path is asked for,
    # eight 128-row blocks whose partial scores are added by the selection kernel
    alpha, N = 64, 3000
    Q, K, V = _rand(1, 32, 2, 128, N, alpha, seed=77)
    lens = np.array([N], dtype=np.int32)
    for pool, pw in ((synth.POOL_MAX, 7), (synth.POOL_AVG, 5)):
        st, _ = _run_and_compare(_W(alpha, pool, pw), 0, alpha + 150, Q, K, V)
        assert st["units"] == 2
        _run_and_compare(_W(alpha, pool, pw), 0, alpha + 150, Q, K, V, lens)


def test_edge_budgets_and_lengths(score_path):
    alpha = 8
    Q, K, V = _rand(3, 8, 2, 128, 300, alpha, seed=5)
    w = _W(alpha, synth.POOL_MAX, 7)
    for k_l in (alpha, alpha + 1, 299, 300, 301, 5000):        # window only ... full cache
        print("edge k_l", k_l, flush=True)
        _run_and_compare(w, 0, k_l, Q, K, V)
    lens = np.array([300, 3, 0], dtype=np.int32)               # n < alpha and n = 0
    for k_l in (alpha, 40):
        print("edge lens k_l", k_l, flush=True)
        _run_and_compare(w, 0, k_l, Q, K, V, lens)
    lens = np.array([alpha + 1, 41, 40], dtype=np.int32)       # single prefix token; n = k_l + 1; n = k_l
    _run_and_compare(w, 0, 40, Q, K, V, lens)


def test_exact_ties_lower_position_wins():
    # identical keys -> identical scores everywhere: the kept prefix must be 0..kk-1
    alpha, N = 4, 500
    Q, K, V = _rand(1, 4, 2, 64, N, alpha, seed=6)
    K[:] = K[:, :, :1, :]
    w = _W(alpha, synth.POOL_NONE, 1)
    st, out = _run_and_compare(w, 0, 54, Q, K, V)
    assert out[2][0, 0, :50].tolist() == list(range(50))
    # max-pool plateaus cut in the middle
    Q, K, V = _rand(1, 4, 1, 64, N, alpha, seed=7)
    K[0, 0, 200] = (Q[0, :, :].float().sum(dim=(0, 1)) * 2).to(torch.bfloat16)
    st, out = _run_and_compare(_W(alpha, synth.POOL_MAX, 7), 0, alpha + 4, Q, K, V)
    assert out[2][0, 0, :4].tolist() == [197, 198, 199, 200]


def test_strided_inputs_and_outputs():
    # K/V stored token-major [B, N, Hkv, d] and viewed head-major; outputs written into a larger buffer
    alpha, N, B, Hq, Hkv, d, k_l = 8, 600, 2, 8, 2, 128, 64
    g = torch.Generator(device=DEV).manual_seed(8)
    Q = torch.randn(B, alpha, Hq, d, generator=g, device=DEV).to(torch.bfloat16).permute(0, 2, 1, 3)
    K = torch.randn(B, N, Hkv, d, generator=g, device=DEV).to(torch.bfloat16).permute(0, 2, 1, 3)
    V = torch.randn(B, N, Hkv, d, generator=g, device=DEV).to(torch.bfloat16).permute(0, 2, 1, 3)
    big = torch.zeros(B, Hkv, k_l + 10, 2 * d, dtype=torch.bfloat16, device=DEV)
    K_out, V_out = big[:, :, :k_l, :d], big[:, :, :k_l, d:]
    _, _, idx, count, scores = binding.alloc_outputs(Q, K, k_l, want_scores=True)
    out = binding.compress_layer(Q, K, V, k_l, synth.POOL_MAX, 7, outputs=(K_out, V_out, idx, count, scores))
    torch.cuda.synchronize()
    compare_layer(Q, K, V, k_l, alpha, synth.POOL_MAX, 7, None, out)
    assert torch.all(big[:, :, k_l:] == 0)


def test_deterministic_and_inputs_untouched():
    w = synth.WORKLOADS[1].scaled(N=5000, L=1)
    Q, K, V, _ = synth.make_layer(w, 0, DEV)
    q0, k0, v0 = bits(Q).copy(), bits(K).copy(), bits(V).copy()
    a = binding.compress_layer(Q, K, V, 100, w.pool, w.pool_w, want_scores=True)
    b = binding.compress_layer(Q, K, V, 100, w.pool, w.pool_w, want_scores=True)
    torch.cuda.synchronize()
    for x, y in zip(a, b):
        assert torch.equal(x.view(torch.int32) if x.dtype == torch.float32 else x,
                           y.view(torch.int32) if y.dtype == torch.float32 else y)
    assert np.array_equal(bits(Q), q0) and np.array_equal(bits(K), k0) and np.array_equal(bits(V), v0)


def test_compress_layers_equals_per_layer_calls_and_budget_nesting():
    w = synth.WORKLOADS[2].scaled(N=3000, L=4)
    layers = [synth.make_layer(w, l, DEV) for l in range(w.L)]
    Qs, Ks, Vs = [x[0] for x in layers], [x[1] for x in layers], [x[2] for x in layers]
    prev = None
    for avg in (64, 128, 512):
        ks = binding.budgets(w.L, avg, w.beta, w.alpha)
        outs = binding.compress_layers(Qs, Ks, Vs, ks, w.pool, w.pool_w, want_scores=True)
        torch.cuda.synchronize()
        for l in range(w.L):
            single = binding.compress_layer(Qs[l], Ks[l], Vs[l], ks[l], w.pool, w.pool_w, want_scores=True)
            torch.cuda.synchronize()
            for x, y in zip(outs[l], single):
                assert torch.equal(x, y)
        compare_layer(Qs[0], Ks[0], Vs[0], ks[0], w.alpha, w.pool, w.pool_w, None, outs[0])
        # same scores, larger budget (layer 0 budgets grow with avg) => kept sets are nested
        cur = [set(outs[0][2][0, g].tolist()) for g in range(w.Hkv)]
        if prev is not None:
            assert all(p <= c for p, c in zip(prev, cur))
        prev = cur


def test_extreme_logits_take_the_exact_fallback(score_path):
    # Keys aligned with a window query and scaled x8 give logits near 8*|q|^2 ~ 1000: about 130 binary orders
    # above their neighbours' after the 1/sqrt(d) scaling, beyond what a fixed reference exponent can
    # carry in fp32.  Planted away from the first keys of a 128-key span, in the middle of the prefix and
    # inside the last, masked tile; also a strongly negative one (-8x).
    alpha, N, B, Hq, Hkv, d = 32, 2000, 2, 8, 2, 128
    Q, K, V = _rand(B, Hq, Hkv, d, N, alpha, seed=11)
    K[0, 0, 77] = (Q[0, 1, 3].float() * 8).to(torch.bfloat16)          # head group 0: query heads 0..3
    K[0, 0, 700] = (Q[0, 2, 31].float() * 8).to(torch.bfloat16)
    K[0, 1, 1] = (Q[0, 5, 0].float() * 8).to(torch.bfloat16)           # head group 1: query heads 4..7
    K[0, 1, N - alpha - 2] = (Q[0, 7, 30].float() * 8).to(torch.bfloat16)
    K[1, 0, 1300] = (Q[1, 0, 16].float() * -8).to(torch.bfloat16)
    K[1, 1, 515] = (Q[1, 6, 9].float() * 8).to(torch.bfloat16)
    for pool, pw in ((synth.POOL_AVG, 5), (synth.POOL_NONE, 1)):
        print("extreme logits", pool, pw, flush=True)
        st, out = _run_and_compare(_W(alpha, pool, pw), 0, alpha + 96, Q, K, V)
        kept = out[2].cpu().numpy()
        assert 77 in kept[0, 0] and 700 in kept[0, 0] and 1 in kept[0, 1] and 515 in kept[1, 1]


def test_non_finite_inputs_stay_in_bounds(score_path):
    # NaN / Inf in one head's keys make that head's scores NaN.  Whatever is kept there must still be a valid
    # selection (in range, ascending, window present, rows copied bit for bit); every other unit is unaffected.
    alpha, N, B, Hq, Hkv, d, k_l = 8, 1500, 2, 8, 2, 128, 72
    Q, K, V = _rand(B, Hq, Hkv, d, N, alpha, seed=12)
    w = _W(alpha, synth.POOL_MAX, 7)
    clean = binding.compress_layer(Q, K, V, k_l, w.pool, w.pool_w, want_scores=True)
    torch.cuda.synchronize()
    Kbad = K.clone()
    Kbad[0, 0, 100] = float("nan")
    Kbad[0, 0, 900, 5] = float("inf")
    Kbad[0, 0, 901, 6] = float("-inf")
    out = binding.compress_layer(Q, Kbad, V, k_l, w.pool, w.pool_w, want_scores=True)
    torch.cuda.synchronize()
    idx = out[2].cpu().numpy()
    assert out[3].cpu().tolist() == [k_l, k_l]
    for b in range(B):
        for g in range(Hkv):
            row = idx[b, g]
            assert row.min() >= 0 and row.max() < N and np.all(np.diff(row) > 0), (b, g)
            assert row[-alpha:].tolist() == list(range(N - alpha, N)), (b, g)
            sel = torch.from_numpy(row.astype(np.int64)).to(DEV)
            assert np.array_equal(bits(out[0][b, g]), bits(Kbad[b, g].index_select(0, sel)))
            assert np.array_equal(bits(out[1][b, g]), bits(V[b, g].index_select(0, sel)))
            if (b, g) != (0, 0):
                assert np.array_equal(row, clean[2][b, g].cpu().numpy()), (b, g)
                assert torch.equal(out[4][b, g], clean[4][b, g])


def test_probe_read_runs_and_leaves_the_buffer_alone():
    x = torch.arange(1 << 20, dtype=torch.int32, device=DEV)
    ref = x.clone()
    sink = torch.zeros(1, dtype=torch.int32, device=DEV)
    for n in (1 << 20, 4, 4096 + 4):                       # whole buffer, one 16-byte word, a ragged tail of the grid
        binding.probe_read(x[:n], sink)
    torch.cuda.synchronize()
    assert torch.equal(x, ref)


def test_all_layers_without_score_output_keep_the_same_tokens():
    # the benchmark's launch shape: one call over every layer, pooled scores kept in the workspace only
    w = synth.WORKLOADS[2].scaled(N=6000, L=5)
    layers = [synth.make_layer(w, l, DEV) for l in range(w.L)]
    Qs, Ks, Vs = [x[0] for x in layers], [x[1] for x in layers], [x[2] for x in layers]
    ks = binding.budgets(w.L, 128, w.beta, w.alpha)
    with_scores = binding.compress_layers(Qs, Ks, Vs, ks, w.pool, w.pool_w, want_scores=True)
    without = binding.compress_layers(Qs, Ks, Vs, ks, w.pool, w.pool_w, want_scores=False)
    torch.cuda.synchronize()
    for a, b in zip(with_scores, without):
        assert b[4] is None
        for x, y in zip(a[:4], b[:4]):
            assert torch.equal(x, y)


def test_given_up_wait_is_reported_through_the_counts(monkeypatch):
    # Forced from the host: with PKV_FLAG_NO_WAIT every workgroup that has to wait for its group gives up at
    # once.  The kernels still run to completion and stay in bounds; the caller sees count -1 and repeats the call.
    monkeypatch.setattr(binding, "DESC_FLAGS", 0)
    w = synth.WORKLOADS[2].scaled(N=5000, L=2)
    layers = [synth.make_layer(w, l, DEV) for l in range(w.L)]
    Qs, Ks, Vs = [x[0] for x in layers], [x[1] for x in layers], [x[2] for x in layers]
    ks = binding.budgets(w.L, 128, w.beta, w.alpha)
    monkeypatch.setattr(binding, "DESC_FLAGS", binding.FLAG_NO_WAIT)
    bad = binding.compress_layers(Qs, Ks, Vs, ks, w.pool, w.pool_w)
    torch.cuda.synchronize()
    for out in bad:
        assert out[3].cpu().tolist() == [-1] * w.B
        idx = out[2].cpu().numpy()
        assert idx.min() >= 0 and idx.max() < w.N
    monkeypatch.setattr(binding, "DESC_FLAGS", 0)
    good = binding.compress_layers(Qs, Ks, Vs, ks, w.pool, w.pool_w, want_scores=True)
    torch.cuda.synchronize()
    for l, out in enumerate(good):
        assert out[3].cpu().tolist() == [min(ks[l], w.N)] * w.B
        compare_layer(Qs[l], Ks[l], Vs[l], ks[l], w.alpha, w.pool, w.pool_w, None, out)


def test_more_layers_than_one_launch_holds(score_path):
    # 100 layers: the kernel-argument tables hold 96 (scoring) and 40 (select, gather) layers per launch, so the
    # call is split into several launches that share one workspace.
    L, alpha, N = 100, 8, 700
    w = _W(alpha, synth.POOL_MAX, 7)
    layers = [_rand(1, 8, 2, 64, N, alpha, seed=1000 + l) for l in range(L)]
    Qs, Ks, Vs = [x[0] for x in layers], [x[1] for x in layers], [x[2] for x in layers]
    ks = [alpha + 1 + (l * 7) % 90 for l in range(L)]
    outs = binding.compress_layers(Qs, Ks, Vs, ks, w.pool, w.pool_w, want_scores=True)
    torch.cuda.synchronize()
    for l in (0, 39, 40, 79, 80, 95, 96, 99):
        single = binding.compress_layer(Qs[l], Ks[l], Vs[l], ks[l], w.pool, w.pool_w, want_scores=True)
        torch.cuda.synchronize()
        for x, y in zip(outs[l], single):
            assert torch.equal(x, y), l
    compare_layer(Qs[96], Ks[96], Vs[96], ks[96], alpha, w.pool, w.pool_w, None, outs[96])

"""Pins of the oracle's selection (Sec. 4.2.2: top-k^l per head, instruction tokens always kept) and of the
gather (appendix "Details of Proposed Method"; ascending positions per the rotary-embedding appendix)."""
import numpy as np
import pytest
import torch

from oracle import pkv_oracle
from paper_2406_02069_amd import synth


def test_topk_brute_force_with_ties():
    rs = np.random.RandomState(0)
    for trial in range(200):
        n = int(rs.randint(1, 40))
        p = rs.randint(0, 5, size=n).astype(np.float64) / 4.0     # many exact ties
        kk = int(rs.randint(0, n + 1))
        got = pkv_oracle.topk(p, kk)
        order = sorted(range(n), key=lambda i: (-p[i], i))         # value desc, lower index first
        want = sorted(order[:kk])
        assert list(got) == want


def test_topk_nesting_and_threshold_property():
    rs = np.random.RandomState(1)
    p = rs.rand(500)
    prev = set()
    for kk in range(0, 501, 7):
        cur = set(int(i) for i in pkv_oracle.topk(p, kk))
        assert len(cur) == kk and prev <= cur
        if 0 < kk < 500:
            rest = [p[i] for i in range(500) if i not in cur]
            assert min(p[list(cur)]) >= max(rest)
        prev = cur
    with pytest.raises(ValueError):
        pkv_oracle.topk(p, 501)


def _run(Q, K, V, k_l, alpha, pool=synth.POOL_MAX, w=7, lens=None):
    return pkv_oracle.compress_layer(Q, K, V, k_l, alpha, pool, w, seq_lens=lens)


def _rand_layer(B, Hq, Hkv, d, N, alpha, seed):
    g = torch.Generator().manual_seed(seed)
    Q = torch.randn(B, Hq, alpha, d, generator=g).to(torch.bfloat16)
    K = torch.randn(B, Hkv, N, d, generator=g).to(torch.bfloat16)
    V = torch.randn(B, Hkv, N, d, generator=g).to(torch.bfloat16)
    return Q, K, V


def _bits(t):
    return t.contiguous().view(torch.int16).numpy().view(np.uint16)


def test_window_always_kept_rows_are_copies_positions_ascending():
    B, Hq, Hkv, d, N, alpha = 2, 4, 2, 64, 200, 8
    Q, K, V = _rand_layer(B, Hq, Hkv, d, N, alpha, 10)
    for k_l in (alpha, alpha + 1, 40, 199):
        out = _run(Q, K, V, k_l, alpha)
        idx = out["idx"]
        assert list(out["count"]) == [k_l] * B
        for b in range(B):
            for g in range(Hkv):
                assert list(idx[b, g, k_l - alpha:]) == list(range(N - alpha, N))      # instruction tokens
                assert np.all(np.diff(idx[b, g]) > 0)                                   # ascending, unique
                np.testing.assert_array_equal(out["K_out"][b, g], _bits(K)[b, g, idx[b, g]])
                np.testing.assert_array_equal(out["V_out"][b, g], _bits(V)[b, g, idx[b, g]])


def test_budget_at_least_n_keeps_the_whole_cache():
    B, Hq, Hkv, d, N, alpha = 1, 2, 2, 64, 50, 4
    Q, K, V = _rand_layer(B, Hq, Hkv, d, N, alpha, 11)
    for k_l in (50, 51, 400):
        out = _run(Q, K, V, k_l, alpha)
        assert out["idx"].shape[-1] == N and list(out["count"]) == [N]
        for g in range(Hkv):
            assert list(out["idx"][0, g]) == list(range(N))
            np.testing.assert_array_equal(out["K_out"][0, g], _bits(K)[0, g])
            np.testing.assert_array_equal(out["V_out"][0, g], _bits(V)[0, g])


def test_end_to_end_equals_stagewise_python_brute_force():
    # Whole layer vs. a test-side composition: library pooling + Python sort, on the oracle's own stage outputs.
    B, Hq, Hkv, d, N, alpha, k_l = 1, 4, 2, 64, 120, 4, 30
    Q, K, V = _rand_layer(B, Hq, Hkv, d, N, alpha, 12)
    G = Hq // Hkv
    for pool, w in ((synth.POOL_MAX, 7), (synth.POOL_AVG, 5), (synth.POOL_NONE, 1)):
        out = _run(Q, K, V, k_l, alpha, pool, w)
        for g in range(Hkv):
            _, s = pkv_oracle.window_scores(Q[0, g * G:(g + 1) * G], K[0, g])
            t = torch.from_numpy(s)[None, None]
            if pool == synth.POOL_MAX:
                p = torch.nn.functional.max_pool1d(t, w, 1, (w - 1) // 2)[0, 0].numpy()
            elif pool == synth.POOL_AVG:
                p = torch.nn.functional.avg_pool1d(t, w, 1, (w - 1) // 2)[0, 0].numpy()
            else:
                p = s
            np.testing.assert_allclose(out["pooled"][0, g, :N - alpha], p, rtol=1e-13)
            order = sorted(range(N - alpha), key=lambda i: (-out["pooled"][0, g, i], i))
            want = sorted(order[:k_l - alpha]) + list(range(N - alpha, N))
            assert list(out["idx"][0, g]) == want


def test_planted_needles_and_sink_are_selected():
    # Keys aligned with a window query collect that query's mass; with max-pool 7 each needle brings its
    # 3 neighbours on either side.  Budget 7*(needles+1) + alpha keeps every needle, the sink and all plateaus.
    w = synth.WORKLOADS[1].scaled(N=1024, L=1, needles=6)
    Q, K, V, lens = synth.make_layer(w, 0)
    plan = synth.needle_plan(w, 0, lens)
    assert len(plan) == 6
    k_l = 7 * 7 + w.alpha
    out = _run(Q, K, V, k_l, w.alpha, w.pool, w.pool_w)
    for (b, g, p, h, t) in plan:
        kept = set(int(i) for i in out["idx"][b, g])
        assert set(range(p - 3, p + 4)) <= kept
        pooled = out["pooled"][b, g]
        assert pooled[p] > 0.5 / w.G
    # a sink: key 0 made attractive for every query of the group
    w0 = w.scaled(needles=0, sink=False)
    Q, K2, V, _ = synth.make_layer(w0, 0)
    K2[0, 0, 0] = (Q[0, 0:w.G].float().sum(dim=(0, 1)) * 2).to(torch.bfloat16)
    out2 = _run(Q, K2, V, w.alpha + 4, w.alpha, w.pool, w.pool_w)
    assert out2["pooled"][0, 0, 0] > 0.5 * w.alpha
    assert list(out2["idx"][0, 0, :4]) == [0, 1, 2, 3]     # plateau of the sink, lower positions first


def test_ragged_batch_each_sequence_on_its_own():
    B, Hq, Hkv, d, N, alpha, k_l = 3, 4, 2, 64, 90, 4, 20
    Q, K, V = _rand_layer(B, Hq, Hkv, d, N, alpha, 13)
    lens = np.array([90, 37, 12], dtype=np.int32)            # last one: n_b <= k_l keeps everything
    Kn, Vn = K.clone(), V.clone()
    for b in range(B):
        Kn[b, :, lens[b]:] = float("nan")
        Vn[b, :, lens[b]:] = float("nan")
    out = _run(Q, Kn, Vn, k_l, alpha, lens=lens)
    assert list(out["count"]) == [20, 20, 12]
    for b in range(B):
        n = int(lens[b])
        solo = _run(Q[b:b + 1], K[b:b + 1, :, :n].contiguous(), V[b:b + 1, :, :n].contiguous(), k_l, alpha)
        c = int(out["count"][b])
        np.testing.assert_array_equal(out["idx"][b, :, :c], solo["idx"][0, :, :c])
        np.testing.assert_array_equal(out["K_out"][b, :, :c], solo["K_out"][0, :, :c])
        np.testing.assert_array_equal(out["V_out"][b, :, :c], solo["V_out"][0, :, :c])
        assert np.all(out["idx"][b, :, c:] == -1) and np.all(out["K_out"][b, :, c:] == 0)
        assert not np.isnan(out["pooled"][b]).any()          # padded rows were never read


def test_uniform_budget_nesting_across_a_budget_sweep():
    # Scores do not depend on the budget, so kept sets are nested as the budget grows.
    B, Hq, Hkv, d, N, alpha = 1, 4, 1, 64, 300, 8
    Q, K, V = _rand_layer(B, Hq, Hkv, d, N, alpha, 14)
    prev = None
    for k_l in (8, 16, 40, 100, 299):
        out = _run(Q, K, V, k_l, alpha, synth.POOL_AVG, 5)
        cur = set(int(i) for i in out["idx"][0, 0])
        assert prev is None or prev <= cur
        prev = cur


# ---- per-layer paged output (appendix "PyramidKV Implementation at vLLM") -------------------------------


def test_scatter_pages_hand_written_pool_image():
    # one sequence, one head, d = 2: five kept rows, pages of two slots, block table [3, 0, 2] into a pool of four
    # pages.  Rows 0,1 -> page 3; rows 2,3 -> page 0; row 4 -> page 2 slot 0; everything else keeps its old content.
    K_out = np.array([[[[10, 11], [20, 21], [30, 31], [40, 41], [50, 51], [0, 0]]]], dtype=np.uint16)
    V_out = K_out + 100
    pool = np.full((4, 1, 2, 2), 7, dtype=np.uint16)
    Kp, Vp = pkv_oracle.scatter_pages(K_out, V_out, np.array([5]), np.array([[3, 0, 2]]), 2, pool, pool)
    want = np.array([[[[30, 31], [40, 41]]], [[[7, 7], [7, 7]]], [[[50, 51], [7, 7]]], [[[10, 11], [20, 21]]]],
                    dtype=np.uint16)
    np.testing.assert_array_equal(Kp, want)
    np.testing.assert_array_equal(Vp, np.where(want == 7, 7, want + 100))
    np.testing.assert_array_equal(pool, 7)                           # the inputs are not modified


def test_scatter_pages_identity_table_and_heads():
    # pages numbered in order and as large as the budget: the pool is the compact cache, head by head
    rs = np.random.RandomState(3)
    B, Hkv, k_cap, d = 3, 2, 8, 4
    K_out = rs.randint(1, 60000, size=(B, Hkv, k_cap, d)).astype(np.uint16)
    V_out = rs.randint(1, 60000, size=(B, Hkv, k_cap, d)).astype(np.uint16)
    count = np.array([8, 5, 0])
    pool = np.zeros((B, Hkv, k_cap, d), dtype=np.uint16)
    Kp, Vp = pkv_oracle.scatter_pages(K_out, V_out, count, np.arange(B)[:, None], k_cap, pool, pool)
    for b in range(B):
        np.testing.assert_array_equal(Kp[b, :, : count[b]], K_out[b, :, : count[b]])
        np.testing.assert_array_equal(Vp[b, :, : count[b]], V_out[b, :, : count[b]])
        assert not Kp[b, :, count[b]:].any() and not Vp[b, :, count[b]:].any()


def test_scatter_pages_rejects_bad_tables():
    K_out = np.ones((1, 1, 4, 2), dtype=np.uint16)
    pool = np.zeros((2, 1, 2, 2), dtype=np.uint16)
    with pytest.raises(ValueError):
        pkv_oracle.scatter_pages(K_out, K_out, np.array([4]), np.array([[0, 2]]), 2, pool, pool)     # page 2 of 2
    with pytest.raises(ValueError):
        pkv_oracle.scatter_pages(K_out, K_out, np.array([4]), np.array([[0]]), 2, pool, pool)        # table too short

"""Pins of the oracle's window-score stage (Sec. 4.2.2, Eq. Al and Eq. att_score) and pooling."""
import math

import numpy as np
import pytest
import torch

from oracle import pkv_oracle


def _bf16(x: torch.Tensor) -> torch.Tensor:
    return x.to(torch.bfloat16)


def test_alpha1_reduces_to_library_softmax():
    # alpha = 1, one head: the score vector is the last query's attention row over all n keys,
    # restricted to the prefix -- a textbook softmax(q K^T / sqrt(d)).
    torch.manual_seed(0)
    for d in (64, 128):
        n = 300
        q = _bf16(torch.randn(1, 1, d))
        k = _bf16(torch.randn(n, d))
        s_head, s_mean = pkv_oracle.window_scores(q, k)
        ref = torch.softmax((k.double() @ q[0, 0].double()) / math.sqrt(d), dim=0)[: n - 1].numpy()
        np.testing.assert_allclose(s_mean, ref, rtol=1e-12, atol=0)
        np.testing.assert_allclose(s_head[0], ref, rtol=1e-12, atol=0)


def test_identical_keys_give_harmonic_closed_form():
    # All keys equal => every visible key gets the same attention.  Window query t sits at position
    # n-alpha+t and (causally) sees n-alpha+t+1 keys, so each prefix key receives
    # sum_t 1/(n-alpha+t+1) from one head; the group mean of identical heads is the same number.
    torch.manual_seed(1)
    for (G, alpha, n, d) in [(1, 4, 50, 64), (4, 8, 97, 128), (2, 1, 9, 64)]:
        q = _bf16(torch.randn(G, alpha, d))
        k = _bf16(torch.randn(1, d)).repeat(n, 1)
        s_head, s_mean = pkv_oracle.window_scores(q, k)
        want = sum(1.0 / (n - alpha + t + 1) for t in range(alpha))
        np.testing.assert_allclose(s_mean, np.full(n - alpha, want), rtol=1e-12)
        np.testing.assert_allclose(s_head, np.full((G, n - alpha), want), rtol=1e-12)


def test_rows_are_softmaxes_total_mass():
    # Each window query's attention sums to 1 over the keys it sees.  With window keys made
    # invisible in practice (logit very negative for every query) all mass lands on the prefix:
    # sum_i s^h_i = alpha for every head.
    torch.manual_seed(2)
    G, alpha, n, d = 3, 5, 200, 64
    q = _bf16(torch.rand(G, alpha, d) + 0.5)              # all-positive queries
    k = _bf16(torch.randn(n, d))
    k[n - alpha:] = _bf16(torch.full((alpha, d), -30.0))  # q.k << 0 for window keys
    s_head, s_mean = pkv_oracle.window_scores(q, k)
    np.testing.assert_allclose(s_head.sum(axis=1), np.full(G, float(alpha)), rtol=1e-9)
    np.testing.assert_allclose(s_mean.sum(), float(alpha), rtol=1e-9)


def test_causal_mask_inside_window():
    # One dominant key INSIDE the window at window offset j (position n-alpha+j).  Queries t >= j see
    # it and give it nearly all their mass; queries t < j do not see it and spread their mass.  So the
    # prefix receives (nearly) only the mass of the j queries in front of it: sum_i s_i ~= j.
    torch.manual_seed(3)
    alpha, n, d = 6, 120, 64
    for j in range(alpha):
        q = _bf16(torch.ones(1, alpha, d))
        k = _bf16(torch.zeros(n, d))
        k[n - alpha + j] = _bf16(torch.full((d,), 8.0))   # logit 8*64/8 = 64 vs 0
        _, s_mean = pkv_oracle.window_scores(q, k)
        assert abs(s_mean.sum() - sum((n - alpha) / (n - alpha + t + 1) for t in range(j))) < 1e-6


def test_group_mean_and_window_sum_linearity():
    torch.manual_seed(4)
    alpha, n, d = 4, 80, 64
    q1 = _bf16(torch.randn(1, alpha, d))
    k = _bf16(torch.randn(n, d))
    _, s1 = pkv_oracle.window_scores(q1, k)
    # duplicating the head (G = 1 -> 3) leaves the group mean unchanged
    _, s3 = pkv_oracle.window_scores(q1.repeat(3, 1, 1), k)
    np.testing.assert_allclose(s3, s1, rtol=1e-13)
    # two different heads: mean of the two single-head results
    q2 = _bf16(torch.randn(1, alpha, d))
    _, s2 = pkv_oracle.window_scores(q2, k)
    sh, s12 = pkv_oracle.window_scores(torch.cat([q1, q2]), k)
    np.testing.assert_allclose(s12, 0.5 * (s1 + s2), rtol=1e-13)
    np.testing.assert_allclose(sh[0], s1, rtol=1e-13)
    np.testing.assert_allclose(sh[1], s2, rtol=1e-13)


def test_attention_received_not_given():
    # A key aligned with one window query collects that query's whole mass: score ~ 1/G at that key.
    torch.manual_seed(5)
    G, alpha, n, d = 4, 8, 256, 128
    q = _bf16(torch.randn(G, alpha, d))
    k = _bf16(torch.randn(n, d))
    P = 100
    k[P] = q[2, 3] * 2
    _, s = pkv_oracle.window_scores(q, k)
    assert int(np.argmax(s)) == P
    assert 0.9 / G < s[P] < 1.6 / G


def test_brute_force_python_tiny():
    # Pure-Python restatement on a tiny case, no vector library involved.
    torch.manual_seed(6)
    G, alpha, n, d = 2, 3, 11, 4
    q = _bf16(torch.randn(G, alpha, d))
    k = _bf16(torch.randn(n, d))
    _, s = pkv_oracle.window_scores(q, k)
    ql, kl = q.float().tolist(), k.float().tolist()
    want = [0.0] * (n - alpha)
    for h in range(G):
        for t in range(alpha):
            p = n - alpha + t
            logit = [sum(ql[h][t][c] * kl[i][c] for c in range(d)) / math.sqrt(d) for i in range(p + 1)]
            Z = sum(math.exp(x) for x in logit)
            for i in range(n - alpha):
                want[i] += math.exp(logit[i]) / Z / G
    np.testing.assert_allclose(s, np.array(want), rtol=1e-12)


@pytest.mark.parametrize("w", [1, 3, 5, 7, 13])
def test_pool_matches_library_pooling(w):
    rs = np.random.RandomState(w)
    for length in (1, 2, 5, 64, 301):
        s = rs.rand(length)
        t = torch.from_numpy(s)[None, None]
        r = (w - 1) // 2
        ref_max = torch.nn.functional.max_pool1d(t, w, stride=1, padding=r)[0, 0].numpy() if length >= 1 else s
        ref_avg = torch.nn.functional.avg_pool1d(t, w, stride=1, padding=r, count_include_pad=True)[0, 0].numpy()
        np.testing.assert_array_equal(pkv_oracle.pool(pkv_oracle.POOL_MAX, w, s), ref_max)
        np.testing.assert_allclose(pkv_oracle.pool(pkv_oracle.POOL_AVG, w, s), ref_avg, rtol=1e-14)
        np.testing.assert_array_equal(pkv_oracle.pool(pkv_oracle.POOL_NONE, w, s), s)


def test_pool_closed_forms():
    c, length, w = 0.25, 20, 7
    r = (w - 1) // 2
    s = np.full(length, c)
    np.testing.assert_array_equal(pkv_oracle.pool(pkv_oracle.POOL_MAX, w, s), s)
    want = np.array([c * (min(i, r) + 1 + min(length - 1 - i, r)) / w for i in range(length)])
    np.testing.assert_allclose(pkv_oracle.pool(pkv_oracle.POOL_AVG, w, s), want, rtol=1e-14)
    # a single spike spreads to exactly w positions under max pooling
    s = np.zeros(length)
    s[9] = 1.0
    p = pkv_oracle.pool(pkv_oracle.POOL_MAX, w, s)
    assert list(np.nonzero(p)[0]) == list(range(9 - r, 9 + r + 1))
    with pytest.raises(ValueError):
        pkv_oracle.pool(pkv_oracle.POOL_MAX, 4, s)


# ---- supplied softmax denominators (one-sweep variant of Sec. 4.2.2's window attention) ---------------


def _library_lse(q, k, alpha):
    """ln sum_{i <= p} exp(q.k_i / sqrt(d)) per window row with a library routine (scipy), fp64."""
    from scipy.special import logsumexp

    G, _, d = q.shape
    n = k.shape[0]
    logits = (q.double().reshape(G * alpha, d) @ k.double().T).numpy() / math.sqrt(d)
    out = np.zeros(G * alpha)
    for r in range(G * alpha):
        p = n - alpha + r % alpha
        out[r] = logsumexp(logits[r, : p + 1])
    return out.reshape(G, alpha)


def test_supplied_exact_denominators_reproduce_the_softmax():
    torch.manual_seed(11)
    for (G, alpha, n, d) in [(1, 1, 40, 64), (4, 8, 130, 128), (2, 5, 77, 64)]:
        q = _bf16(torch.randn(G, alpha, d) * 2.0)
        k = _bf16(torch.randn(n, d))
        sh0, sm0 = pkv_oracle.window_scores(q, k)
        sh1, sm1 = pkv_oracle.window_scores(q, k, lse=_library_lse(q, k, alpha))
        np.testing.assert_allclose(sh1, sh0, rtol=1e-11)
        np.testing.assert_allclose(sm1, sm0, rtol=1e-11)


def test_supplied_denominator_single_visible_pair_closed_form():
    # alpha = 1, all keys orthogonal to the query: every logit is 0; with lse = ln(c) every prefix
    # key receives exactly 1/c whatever n is (nothing is renormalised).
    d, n = 64, 20
    q = torch.zeros(1, 1, d)
    q[0, 0, 0] = 1.0
    k = torch.zeros(n, d)
    k[:, 1] = 3.0
    for c in (2.0, 20.0, 0.5):
        _, sm = pkv_oracle.window_scores(_bf16(q), _bf16(k), lse=np.array([[math.log(c)]]))
        np.testing.assert_allclose(sm, np.full(n - 1, 1.0 / c), rtol=1e-14)


def test_shifted_denominator_scales_each_rows_share():
    # lse_r + delta_r multiplies row r's attention by exp(-delta_r): with one row per head and one
    # head, the whole score vector scales; with several rows the per-head sums are the delta-weighted
    # sums of the per-row softmaxes, which alpha = 1 heads expose one at a time.
    torch.manual_seed(12)
    G, n, d = 3, 90, 64
    q = _bf16(torch.randn(G, 1, d))
    k = _bf16(torch.randn(n, d))
    base = _library_lse(q, k, 1)
    sh0, _ = pkv_oracle.window_scores(q, k)
    delta = np.array([[0.7], [-1.3], [0.0]])
    sh1, sm1 = pkv_oracle.window_scores(q, k, lse=base + delta)
    np.testing.assert_allclose(sh1, sh0 * np.exp(-delta), rtol=1e-11)
    np.testing.assert_allclose(sm1, (sh0 * np.exp(-delta)).mean(axis=0), rtol=1e-11)


def test_layer_with_supplied_denominators_indexes_them_by_batch_head_row():
    # Full layer: every (b, head, t) row gets its own offset; only the matching layout of
    # lse [B, Hq, alpha] reproduces the per-head scaled scores computed stage-wise above.
    torch.manual_seed(13)
    B, Hq, Hkv, alpha, N, d = 2, 4, 2, 3, 60, 64
    G = Hq // Hkv
    Q = _bf16(torch.randn(B, Hq, alpha, d))
    K = _bf16(torch.randn(B, Hkv, N, d))
    V = _bf16(torch.randn(B, Hkv, N, d))
    rng = np.random.default_rng(5)
    lse = np.zeros((B, Hq, alpha), dtype=np.float32)
    for b in range(B):
        for g in range(Hkv):
            lse[b, g * G:(g + 1) * G] = _library_lse(Q[b, g * G:(g + 1) * G], K[b, g], alpha)
    lse += rng.uniform(-0.5, 0.5, size=lse.shape).astype(np.float32)
    out = pkv_oracle.compress_layer(Q, K, V, 16, alpha, pkv_oracle.POOL_NONE, 1, lse=lse)
    for b in range(B):
        for g in range(Hkv):
            _, sm = pkv_oracle.window_scores(Q[b, g * G:(g + 1) * G], K[b, g],
                                             lse=lse[b, g * G:(g + 1) * G].astype(np.float64))
            np.testing.assert_allclose(out["pooled"][b, g, : N - alpha], sm, rtol=1e-14)
            want = np.sort(np.argsort(-sm, kind="stable")[: 16 - alpha])
            np.testing.assert_array_equal(out["idx"][b, g, : 16 - alpha], want)


# ---- attention recall rate (appendix, "Attention Recall Rate Experiment") --------------------------------


def test_recall_is_one_when_everything_is_kept_and_drops_with_the_kept_set():
    torch.manual_seed(21)
    G, alpha, n, d = 2, 4, 60, 64
    q, k = _bf16(torch.randn(G, alpha, d)), _bf16(torch.randn(n, d))
    assert abs(pkv_oracle.attention_recall(q, k, np.arange(n)) - 1.0) < 1e-12
    r_half = pkv_oracle.attention_recall(q, k, np.arange(0, n, 2))
    r_rest = pkv_oracle.attention_recall(q, k, np.arange(1, n, 2))
    assert 0.0 < r_half < 1.0 and abs(r_half + r_rest - 1.0) < 1e-12          # a partition of the keys
    assert pkv_oracle.attention_recall(q, k, np.array([], dtype=np.int32)) == 0.0


def test_recall_of_the_window_alone_with_identical_keys():
    # identical keys: query t spreads its attention evenly over its n-alpha+t+1 visible keys, of which t+1 lie in
    # the window -> recall of "window only" = mean_t (t+1)/(n-alpha+t+1)
    G, alpha, n, d = 3, 5, 40, 64
    torch.manual_seed(22)
    q = _bf16(torch.randn(G, alpha, d))
    k = _bf16(torch.randn(1, d)).repeat(n, 1)
    want = np.mean([(t + 1) / (n - alpha + t + 1) for t in range(alpha)])
    got = pkv_oracle.attention_recall(q, k, np.arange(n - alpha, n))
    assert abs(got - want) < 1e-12


def test_recall_equals_window_mass_plus_scores_at_the_kept_prefix_positions():
    # ties the metric to the selection scores: sum of s_mean over kept prefix keys = (1/G) sum_h sum_t kept mass
    torch.manual_seed(23)
    G, alpha, n, d = 4, 6, 150, 64
    q, k = _bf16(torch.randn(G, alpha, d)), _bf16(torch.randn(n, d))
    _, s_mean = pkv_oracle.window_scores(q, k)
    kept_prefix = np.sort(np.random.default_rng(1).choice(n - alpha, size=30, replace=False))
    kept = np.concatenate([kept_prefix, np.arange(n - alpha, n)])
    want = (s_mean[kept_prefix].sum() + (alpha - s_mean.sum())) / alpha
    assert abs(pkv_oracle.attention_recall(q, k, kept) - want) < 1e-12

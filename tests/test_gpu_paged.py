"""Per-layer paged output (pkv_compress_layers_paged) vs. the CPU oracle: the pools equal the oracle's scatter of
the kept rows bit for bit, untouched slots keep their content, and the kept positions meet the usual parity bar."""
import numpy as np
import pytest
import torch

from oracle import pkv_oracle
from paper_2406_02069_amd import binding, synth
from tests import prefill_stub
from tests.parity import bits, compare_layer

pytestmark = pytest.mark.gpu
DEV = "cuda:0"
SENTINEL = 0x7E57  # bit pattern the pools are filled with beforehand


def _rand(B, Hq, Hkv, d, N, alpha, seed):
    g = torch.Generator(device=DEV).manual_seed(seed)
    Q = torch.randn(B, Hq, alpha, d, generator=g, device=DEV).to(torch.bfloat16)
    K = torch.randn(B, Hkv, N, d, generator=g, device=DEV).to(torch.bfloat16)
    V = torch.randn(B, Hkv, N, d, generator=g, device=DEV).to(torch.bfloat16)
    return Q, K, V


def _tables(rs, L, B, max_pages, num_pages):
    """Per layer: every sequence gets max_pages distinct pages, no page shared between sequences."""
    out = []
    for _ in range(L):
        perm = rs.permutation(num_pages)[: B * max_pages].astype(np.int32).reshape(B, max_pages)
        out.append(perm)
    return out


def _run_paged(Qs, Ks, Vs, k_ls, alpha, pool, pw, page_size, lens=None, use_lse=False, seed=0, spare_pages=3):
    L = len(Ks)
    B, Hkv, N, d = Ks[0].shape
    rs = np.random.RandomState(seed)
    max_pages = max((min(k, N) + page_size - 1) // page_size for k in k_ls)
    num_pages = B * max_pages + spare_pages
    tables = _tables(rs, L, B, max_pages, num_pages)
    fill = torch.full((num_pages, Hkv, page_size, d), SENTINEL, dtype=torch.int16, device=DEV).view(torch.bfloat16)
    Kp = [fill.clone() for _ in range(L)]
    Vp = [fill.clone() for _ in range(L)]
    tb = [torch.from_numpy(t).to(DEV) for t in tables]
    lens_dev = None if lens is None else torch.from_numpy(np.asarray(lens, dtype=np.int32)).to(DEV)
    lses = [prefill_stub.window_lse(Qs[l], Ks[l], lens) for l in range(L)] if use_lse else None
    outs = binding.compress_layers_paged(Qs, Ks, Vs, k_ls, pool, pw, Kp, Vp, tb, page_size, seq_lens=lens_dev,
                                         want_scores=True, lse=lses)
    torch.cuda.synchronize()
    sent = np.full((num_pages, Hkv, page_size, d), SENTINEL, dtype=np.uint16)
    for l in range(L):
        print("paged layer", l, "k_l", k_ls[l], "page", page_size, flush=True)
        gKp, gVp = bits(outs[l][0]), bits(outs[l][1])
        idx = outs[l][2].cpu().numpy()
        count = outs[l][3].cpu().numpy()
        k_cap = min(k_ls[l], N)
        # un-page the device's pools into the compact layout (rows beyond count: zero, as the compact call leaves them)
        cK = np.zeros((B, Hkv, k_cap, d), dtype=np.uint16)
        cV = np.zeros_like(cK)
        for b in range(B):
            for j in range(int(count[b])):
                pg = tables[l][b, j // page_size]
                cK[b, :, j] = gKp[pg, :, j % page_size]
                cV[b, :, j] = gVp[pg, :, j % page_size]
        compact = (torch.from_numpy(cK.view(np.int16)).view(torch.bfloat16), torch.from_numpy(cV.view(np.int16)).view(torch.bfloat16),
                   outs[l][2], outs[l][3], outs[l][4])
        ref = None
        if use_lse:
            ref = pkv_oracle.compress_layer(Qs[l], Ks[l], Vs[l], k_ls[l], alpha, pool, pw, seq_lens=lens,
                                            lse=np.nan_to_num(lses[l].cpu().numpy(), nan=0.0))
        compare_layer(Qs[l], Ks[l], Vs[l], k_ls[l], alpha, pool, pw, lens, compact, ref=ref)
        # the pools as a whole: the oracle's scatter of the rows at the device's kept positions, everything else untouched
        wK, wV = pkv_oracle.scatter_pages(cK, cV, count, tables[l], page_size, sent, sent)
        np.testing.assert_array_equal(gKp, wK)
        np.testing.assert_array_equal(gVp, wV)
        assert idx.shape == (B, Hkv, k_cap)


@pytest.mark.parametrize("page_size", [1, 16, 17, 128])
def test_page_sizes_and_budgets(page_size):
    alpha = 8
    Q, K, V = _rand(2, 8, 2, 128, 900, alpha, seed=page_size)
    ks = [200, 64, alpha, alpha + 1, 5000]          # last: more than N, everything kept
    L = len(ks)
    _run_paged([Q] * L, [K] * L, [V] * L, ks, alpha, synth.POOL_MAX, 7, page_size, seed=page_size)


def test_ragged_batch_d64_and_supplied_denominators():
    alpha = 5
    Q, K, V = _rand(4, 12, 4, 64, 700, alpha, seed=9)
    lens = np.array([700, 41, 3, 0], dtype=np.int32)
    for use_lse in (False, True):
        _run_paged([Q, Q], [K, K], [V, V], [40, 90], alpha, synth.POOL_AVG, 5, 16, lens=lens, use_lse=use_lse, seed=4)


def test_config1_scaled_all_layers():
    w = synth.WORKLOADS[1].scaled(N=3000, L=6)
    ks = binding.budgets(w.L, w.avg_budgets[0], w.beta, w.alpha)
    layers = [synth.make_layer(w, l, DEV) for l in range(w.L)]
    _run_paged([x[0] for x in layers], [x[1] for x in layers], [x[2] for x in layers], ks, w.alpha, w.pool, w.pool_w, 16,
               lens=layers[0][3], seed=2)


def test_bad_page_number_is_reported_and_never_written_through():
    alpha = 8
    Q, K, V = _rand(2, 4, 2, 128, 300, alpha, seed=1)
    page_size, k_l = 16, 64
    max_pages, num_pages = 4, 8
    tables = np.array([[0, 1, 2, 3], [4, 99, -5, 7]], dtype=np.int32)     # sequence 1: two bad entries
    fill = torch.full((num_pages, 2, page_size, 128), SENTINEL, dtype=torch.int16, device=DEV).view(torch.bfloat16)
    Kp, Vp = fill.clone(), fill.clone()
    outs = binding.compress_layers_paged([Q], [K], [V], [k_l], synth.POOL_MAX, 7, [Kp], [Vp],
                                         [torch.from_numpy(tables).to(DEV)], page_size)
    torch.cuda.synchronize()
    count = outs[0][3].cpu().numpy()
    assert count[0] == k_l and count[1] == -2
    gKp = bits(Kp)
    assert (gKp[[5, 6]] == SENTINEL).all()                                # pages no table names: untouched
    assert (gKp[[0, 1, 2, 3, 4, 7]] != SENTINEL).any(axis=(1, 2, 3)).all()  # the named ones were written


def test_more_layers_than_one_launch_holds():
    # 45 layers: the gather runs in two launches (40 layers per kernel-argument table), each with its own tables
    alpha = 4
    Q, K, V = _rand(2, 4, 2, 64, 400, alpha, seed=12)
    L = 45
    Qs = [Q.roll(l, dims=2).contiguous() for l in range(L)]
    ks = [alpha + 3 + (11 * l) % 70 for l in range(L)]
    _run_paged(Qs, [K] * L, [V] * L, ks, alpha, synth.POOL_MAX, 3, 8, seed=6)

"""Decoding attention over the compacted cache (pkv_decode_attention) vs. the CPU oracle, element by element: compact
and paged caches, ragged counts, both head dimensions, and end to end behind the compression calls."""
import numpy as np
import pytest
import torch

from oracle import pkv_oracle
from paper_2406_02069_amd import binding, synth
from tests.parity import bits

pytestmark = pytest.mark.gpu
DEV = "cuda:0"
# fp32 accumulation of <= 4096 products of bf16 values against fp64: relative to the scale of the values
RTOL, ATOL_SCALE = 1e-4, 2e-5


def _cmp(out, lse, Ks, Vs, q, count):
    ref, ref_lse = pkv_oracle.decode_attention(q, Ks, Vs, count)
    got = out.cpu().numpy().astype(np.float64)
    scale = float(Vs.float().abs().max())
    err = np.abs(got - ref)
    assert np.all(err <= RTOL * np.abs(ref) + ATOL_SCALE * scale), float(err.max())
    if lse is not None:
        gl = lse.cpu().numpy().astype(np.float64)
        fin = np.isfinite(ref_lse)
        assert np.array_equal(np.isneginf(gl), ~fin)
        np.testing.assert_allclose(gl[fin], ref_lse[fin], rtol=0, atol=2e-5 * np.maximum(1.0, np.abs(ref_lse[fin])).max())
    return float(err.max())


def _rand(B, Hq, Hkv, d, k_cap, seed, scale=1.0):
    g = torch.Generator(device=DEV).manual_seed(seed)
    q = (torch.randn(B, Hq, d, generator=g, device=DEV) * scale).to(torch.bfloat16)
    Ks = torch.randn(B, Hkv, k_cap, d, generator=g, device=DEV).to(torch.bfloat16)
    Vs = torch.randn(B, Hkv, k_cap, d, generator=g, device=DEV).to(torch.bfloat16)
    return q, Ks, Vs


@pytest.mark.parametrize("d,Hq,Hkv,k_cap", [(128, 32, 8, 128), (128, 8, 2, 1), (64, 8, 8, 333), (64, 12, 4, 40),
                                             (128, 64, 8, 2048), (128, 4, 4, 4096), (64, 16, 2, 777)])
def test_compact_cache_ragged_counts(d, Hq, Hkv, k_cap):
    B = 4
    q, Ks, Vs = _rand(B, Hq, Hkv, d, k_cap, seed=d + Hq + k_cap, scale=2.0)
    count = np.array([k_cap, max(k_cap // 3, 1), 1, 0], dtype=np.int32)
    Ks[1, :, count[1]:] = float("nan")                      # rows beyond count are never read
    Vs[1, :, count[1]:] = float("nan")
    print("decode compact", d, Hq, Hkv, k_cap, flush=True)
    out, lse = binding.decode_attention(q, Ks, Vs, torch.from_numpy(count).to(DEV), want_lse=True)
    torch.cuda.synchronize()
    assert not torch.isnan(out).any()
    Kc, Vc = Ks.clone(), Vs.clone()
    Kc[1, :, count[1]:] = 0
    Vc[1, :, count[1]:] = 0
    _cmp(out, lse, Kc, Vc, q, count)
    assert not out[3].any()                                  # empty cache: zero rows


def test_strided_compact_cache_and_error_counts():
    B, Hq, Hkv, d, k_cap = 3, 8, 2, 128, 100
    q, Ks, Vs = _rand(B, Hq, Hkv, d, k_cap, seed=5)
    big_k = torch.zeros(B, Hkv, k_cap + 7, d + 64, dtype=torch.bfloat16, device=DEV)
    big_v = torch.zeros_like(big_k)
    big_k[:, :, :k_cap, :d] = Ks
    big_v[:, :, :k_cap, :d] = Vs
    count = torch.tensor([100, -1, 5000], dtype=torch.int32, device=DEV)   # error code reads as empty, too large is clamped
    out, _ = binding.decode_attention(q, big_k[:, :, :k_cap, :d], big_v[:, :, :k_cap, :d], count)
    torch.cuda.synchronize()
    _cmp(out, None, Ks, Vs, q, np.array([100, 0, 100], dtype=np.int32))


@pytest.mark.parametrize("page_size", [1, 16, 17, 128])
def test_paged_cache_behind_the_paged_compression(page_size):
    # end to end: compress into page pools, then attend over them; reference: oracle compression + oracle attention
    alpha, k_l = 8, 150
    B, Hq, Hkv, d, N = 3, 8, 2, 128, 700
    g = torch.Generator(device=DEV).manual_seed(page_size)
    Q = torch.randn(B, Hq, alpha, d, generator=g, device=DEV).to(torch.bfloat16)
    K = torch.randn(B, Hkv, N, d, generator=g, device=DEV).to(torch.bfloat16)
    V = torch.randn(B, Hkv, N, d, generator=g, device=DEV).to(torch.bfloat16)
    lens = np.array([700, 90, 300], dtype=np.int32)
    max_pages = (k_l + page_size - 1) // page_size
    num_pages = B * max_pages + 2
    rs = np.random.RandomState(page_size)
    table = torch.from_numpy(rs.permutation(num_pages)[: B * max_pages].astype(np.int32).reshape(B, max_pages)).to(DEV)
    Kp = torch.full((num_pages, Hkv, page_size, d), float("nan"), dtype=torch.bfloat16, device=DEV)
    Vp = Kp.clone()
    outs = binding.compress_layers_paged([Q], [K], [V], [k_l], synth.POOL_MAX, 7, [Kp], [Vp], [table], page_size,
                                         seq_lens=torch.from_numpy(lens).to(DEV))
    count = outs[0][3]
    qd = torch.randn(B, Hq, d, generator=g, device=DEV).to(torch.bfloat16)
    out, lse = binding.decode_attention(qd, Kp, Vp, count, block_table=table, k_cap=k_l, want_lse=True)
    torch.cuda.synchronize()
    assert not torch.isnan(out).any()
    ref = pkv_oracle.compress_layer(Q, K, V, k_l, alpha, synth.POOL_MAX, 7, seq_lens=lens, want_pooled=False)
    np.testing.assert_array_equal(outs[0][2].cpu().numpy(), ref["idx"])       # same kept sets on this input
    Kc = torch.from_numpy(ref["K_out"].view(np.int16)).view(torch.bfloat16)
    Vc = torch.from_numpy(ref["V_out"].view(np.int16)).view(torch.bfloat16)
    _cmp(out, lse, Kc, Vc, qd, ref["count"])


def test_compact_cache_behind_compress_layer_and_bad_pages_count_as_absent():
    alpha, k_l = 8, 64
    B, Hq, Hkv, d, N = 2, 8, 2, 64, 500
    g = torch.Generator(device=DEV).manual_seed(3)
    Q = torch.randn(B, Hq, alpha, d, generator=g, device=DEV).to(torch.bfloat16)
    K = torch.randn(B, Hkv, N, d, generator=g, device=DEV).to(torch.bfloat16)
    V = torch.randn(B, Hkv, N, d, generator=g, device=DEV).to(torch.bfloat16)
    Ko, Vo, idx, count, _ = binding.compress_layer(Q, K, V, k_l, synth.POOL_AVG, 5)
    qd = torch.randn(B, Hq, d, generator=g, device=DEV).to(torch.bfloat16)
    out, _ = binding.decode_attention(qd, Ko, Vo, count)
    torch.cuda.synchronize()
    _cmp(out, None, Ko, Vo, qd, count.cpu().numpy())
    # paged view of the same rows with one bad table entry: its 16 rows drop out of the softmax
    P = 16
    pool_k = Ko.reshape(B, Hkv, k_l // P, P, d).permute(0, 2, 1, 3, 4).reshape(B * (k_l // P), Hkv, P, d).contiguous()
    pool_v = Vo.reshape(B, Hkv, k_l // P, P, d).permute(0, 2, 1, 3, 4).reshape(B * (k_l // P), Hkv, P, d).contiguous()
    table = torch.arange(B * (k_l // P), dtype=torch.int32, device=DEV).reshape(B, k_l // P).clone()
    table[1, 2] = 12345
    out2, _ = binding.decode_attention(qd, pool_k, pool_v, count, block_table=table, k_cap=k_l)
    torch.cuda.synchronize()
    keep = torch.ones(k_l, dtype=torch.bool)
    keep[2 * P:3 * P] = False
    Kc, Vc = Ko.clone(), Vo.clone()
    Kc[1, :, : k_l - P] = Ko[1][:, keep]
    Vc[1, :, : k_l - P] = Vo[1][:, keep]
    _cmp(out2, None, Kc, Vc, qd, np.array([k_l, k_l - P], dtype=np.int32))


# ---- all layers of a decoding step in one call (pkv_decode_attention_layers) ----

def _layers_case(B, Hq, Hkv, d, k_caps, seed, ragged=True):
    qs, Ks, Vs, counts = [], [], [], []
    rs = np.random.RandomState(seed)
    for l, k_cap in enumerate(k_caps):
        q, K, V = _rand(B, Hq, Hkv, d, k_cap, seed=seed * 1000 + l, scale=2.0)
        c = rs.randint(0, k_cap + 1, size=B).astype(np.int32) if ragged else np.full(B, k_cap, dtype=np.int32)
        c[0] = k_cap
        qs.append(q); Ks.append(K); Vs.append(V); counts.append(c)
    return qs, Ks, Vs, counts


@pytest.mark.parametrize("B,Hq,Hkv,d,k_caps", [
    (1, 32, 8, 128, [242, 166, 90, 14]),                      # a small pyramid at batch 1: one range per head
    (1, 32, 8, 128, [3963, 2730, 1500, 700, 133, 1]),         # a steep pyramid: 16 ... 1 ranges per head
    (3, 8, 2, 64, [4096, 33, 777, 128, 129]),
    (8, 32, 8, 128, [2048, 300]),
    (2, 8, 8, 64, list(range(1, 70, 2))),                     # 35 layers: more than one launch's table holds
])
def test_layers_call_compact_caches(B, Hq, Hkv, d, k_caps):
    qs, Ks, Vs, counts = _layers_case(B, Hq, Hkv, d, k_caps, seed=B + Hq + len(k_caps))
    print("decode layers", B, Hq, Hkv, d, k_caps[:6], flush=True)
    outs = binding.decode_attention_layers(qs, Ks, Vs, [torch.from_numpy(c).to(DEV) for c in counts], want_lse=True)
    torch.cuda.synchronize()
    for l, (out, lse) in enumerate(outs):
        _cmp(out, lse, Ks[l], Vs[l], qs[l], counts[l])
        # and the per-layer entry gives the same up to the order of the fp32 additions
        one, _ = binding.decode_attention(qs[l], Ks[l], Vs[l], torch.from_numpy(counts[l]).to(DEV))
        torch.cuda.synchronize()
        scale = float(Vs[l].float().abs().max())
        assert float((one - out).abs().max()) <= 4e-5 * scale


def test_layers_call_without_lse_and_strided_caches():
    B, Hq, Hkv, d = 2, 8, 2, 128
    k_caps = [100, 1000]
    qs, Ks, Vs, counts = _layers_case(B, Hq, Hkv, d, k_caps, seed=77)
    bigK = [torch.zeros(B, Hkv, k + 5, d + 64, dtype=torch.bfloat16, device=DEV) for k in k_caps]
    bigV = [torch.zeros_like(x) for x in bigK]
    for l, k in enumerate(k_caps):
        bigK[l][:, :, :k, :d] = Ks[l]
        bigV[l][:, :, :k, :d] = Vs[l]
    outs = binding.decode_attention_layers(qs, [x[:, :, :k, :d] for x, k in zip(bigK, k_caps)],
                                           [x[:, :, :k, :d] for x, k in zip(bigV, k_caps)],
                                           [torch.from_numpy(c).to(DEV) for c in counts])
    torch.cuda.synchronize()
    for l, (out, lse) in enumerate(outs):
        assert lse is None
        _cmp(out, None, Ks[l], Vs[l], qs[l], counts[l])


@pytest.mark.parametrize("page_size", [16, 17])
def test_layers_call_behind_the_paged_compression(page_size):
    # end to end over three layers with a pyramid of budgets: compress into per-layer page pools, attend over all
    # layers' pools in one call; reference: oracle compression + oracle attention per layer
    alpha, k_ls = 8, [600, 150, 40]
    B, Hq, Hkv, d, N = 2, 8, 2, 128, 900
    g = torch.Generator(device=DEV).manual_seed(100 + page_size)
    L = len(k_ls)
    Qs = [torch.randn(B, Hq, alpha, d, generator=g, device=DEV).to(torch.bfloat16) for _ in range(L)]
    Ks = [torch.randn(B, Hkv, N, d, generator=g, device=DEV).to(torch.bfloat16) for _ in range(L)]
    Vs = [torch.randn(B, Hkv, N, d, generator=g, device=DEV).to(torch.bfloat16) for _ in range(L)]
    lens = np.array([900, 333], dtype=np.int32)
    rs = np.random.RandomState(page_size)
    tables, Kp, Vp = [], [], []
    max_pages = (max(k_ls) + page_size - 1) // page_size     # the compression call takes one pool shape for all layers
    num_pages = B * max_pages + 3
    for k_l in k_ls:
        tables.append(torch.from_numpy(rs.permutation(num_pages)[: B * max_pages].astype(np.int32)
                                       .reshape(B, max_pages)).to(DEV))
        Kp.append(torch.full((num_pages, Hkv, page_size, d), float("nan"), dtype=torch.bfloat16, device=DEV))
        Vp.append(Kp[-1].clone())
    outs = binding.compress_layers_paged(Qs, Ks, Vs, k_ls, synth.POOL_MAX, 7, Kp, Vp, tables, page_size,
                                         seq_lens=torch.from_numpy(lens).to(DEV))
    qd = [torch.randn(B, Hq, d, generator=g, device=DEV).to(torch.bfloat16) for _ in range(L)]
    res = binding.decode_attention_layers(qd, Kp, Vp, [o[3] for o in outs], block_tables=tables, k_caps=k_ls,
                                          want_lse=True)
    torch.cuda.synchronize()
    for l in range(L):
        out, lse = res[l]
        assert not torch.isnan(out).any()
        ref = pkv_oracle.compress_layer(Qs[l], Ks[l], Vs[l], k_ls[l], alpha, synth.POOL_MAX, 7, seq_lens=lens,
                                        want_pooled=False)
        np.testing.assert_array_equal(outs[l][2].cpu().numpy(), ref["idx"])
        Kc = torch.from_numpy(ref["K_out"].view(np.int16)).view(torch.bfloat16)
        Vc = torch.from_numpy(ref["V_out"].view(np.int16)).view(torch.bfloat16)
        _cmp(out, lse, Kc, Vc, qd[l], ref["count"])

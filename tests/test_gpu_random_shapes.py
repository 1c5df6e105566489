"""Seeded random shapes through both scoring paths, each compared with the oracle element by element."""
import numpy as np
import pytest
import torch

from paper_2406_02069_amd import binding, synth
from tests.parity import compare_layer

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def _case(seed):
    rs = np.random.RandomState(seed)
    d = int(rs.choice([64, 128]))
    Hkv = int(rs.choice([1, 2, 4, 8]))
    G = int(rs.choice([1, 2, 4, 8]))
    alpha = int(rs.choice([1, 3, 8, 16, 32, 64]))
    if G * alpha > 512:                      # keep to shapes both paths accept
        G = 512 // alpha
    B = int(rs.choice([1, 2, 3]))
    N = int(rs.randint(alpha + 2, 2600))
    pool, pw = [(synth.POOL_NONE, 1), (synth.POOL_MAX, 3), (synth.POOL_MAX, 7), (synth.POOL_AVG, 5),
                (synth.POOL_AVG, 9), (synth.POOL_MAX, 31)][rs.randint(6)]
    k_l = int(rs.randint(alpha, min(N + 50, alpha + 400)))
    lens = None
    if rs.rand() < 0.5:
        lens = rs.randint(0, N + 1, size=B).astype(np.int32)
        lens[rs.randint(B)] = N              # at least one full-length sequence
    return d, Hkv, G, alpha, B, N, pool, pw, k_l, lens


@pytest.mark.parametrize("seed", range(60))
@pytest.mark.parametrize("path", ["resident", "stream"])
def test_random_shape(seed, path, monkeypatch):
    monkeypatch.setattr(binding, "DESC_FLAGS", binding.FLAG_STREAM_SCORING if path == "stream" else 0)
    d, Hkv, G, alpha, B, N, pool, pw, k_l, lens = _case(seed)
    print("case", seed, path, dict(d=d, Hkv=Hkv, G=G, alpha=alpha, B=B, N=N, pool=pool, pw=pw, k_l=k_l,
                                   lens=None if lens is None else lens.tolist()), flush=True)
    g = torch.Generator(device=DEV).manual_seed(5000 + seed)
    scale = 1.0 + 2.0 * (seed % 3)           # wider logit ranges in some cases
    Q = (torch.randn(B, Hkv * G, alpha, d, generator=g, device=DEV) * scale).to(torch.bfloat16)
    K = torch.randn(B, Hkv, N, d, generator=g, device=DEV).to(torch.bfloat16)
    V = torch.randn(B, Hkv, N, d, generator=g, device=DEV).to(torch.bfloat16)
    lens_dev = None if lens is None else torch.from_numpy(lens).to(DEV)
    out = binding.compress_layer(Q, K, V, k_l, pool, pw, seq_lens=lens_dev, want_scores=True)
    torch.cuda.synchronize()
    compare_layer(Q, K, V, k_l, alpha, pool, pw, lens, out)


@pytest.mark.parametrize("seed", range(8))
def test_random_ragged_batch_with_many_parts(seed):
    """Units of many parts (16 or more) in a ragged batch: the tagged exchange of the softmax statistics with parts that lie
    beyond the end of a shorter sequence (they take part with neutral statistics), several layers so that every
    group of workgroups works through more than one unit."""
    rs = np.random.RandomState(300 + seed)
    d = int(rs.choice([64, 128]))
    Hkv = int(rs.choice([1, 2, 4]))
    G = int(rs.choice([1, 4, 8]))
    alpha = int(rs.choice([8, 16, 32]))
    B = 3
    N = int(rs.randint(8192, 14000))
    L = int(rs.randint(2, 5))
    pool, pw = [(synth.POOL_MAX, 7), (synth.POOL_AVG, 5), (synth.POOL_NONE, 1)][rs.randint(3)]
    lens = np.array([N, rs.randint(alpha + 1, N), rs.choice([0, alpha - 1, 513, N // 2])], dtype=np.int32)
    lens = lens[rs.permutation(3)]
    ks = [int(rs.randint(alpha, 2000)) for _ in range(L)]
    print("ragged case", seed, dict(d=d, Hkv=Hkv, G=G, alpha=alpha, N=N, L=L, pool=pool, pw=pw, lens=lens.tolist(), ks=ks),
          flush=True)
    g = torch.Generator(device=DEV).manual_seed(900 + seed)
    Qs = [torch.randn(B, Hkv * G, alpha, d, generator=g, device=DEV).to(torch.bfloat16) for _ in range(L)]
    Ks = [torch.randn(B, Hkv, N, d, generator=g, device=DEV).to(torch.bfloat16) for _ in range(L)]
    Vs = [torch.randn(B, Hkv, N, d, generator=g, device=DEV).to(torch.bfloat16) for _ in range(L)]
    for K in Ks:
        for b in range(B):
            K[b, :, int(lens[b]):] = float("nan")   # never read
    outs = binding.compress_layers(Qs, Ks, Vs, ks, pool, pw, seq_lens=torch.from_numpy(lens).to(DEV), want_scores=True)
    torch.cuda.synchronize()
    for l in sorted({0, L - 1}):
        compare_layer(Qs[l], Ks[l], Vs[l], ks[l], alpha, pool, pw, lens, outs[l])

"""Contexts beyond 32k (the appendix discusses up to 128k): units that span 128, 256 or all 512 workgroups of the
persistent scoring kernel, prefixes too long for the in-LDS selection (radix select over keys in global memory),
the largest length the register-resident kernel takes (262 144) and one beyond it (streaming kernels).  HIP
library vs. CPU oracle, element by element, through the C ABI (needs an MI355X)."""
import numpy as np
import pytest
import torch

from oracle import pkv_oracle
from paper_2406_02069_amd import binding, prefill_stub, synth
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

"""Pins of the oracle's decoding attention over the compacted cache (Sec. 3: after compression the model attends
over the kept keys and values only)."""
import math

import numpy as np
import torch

from oracle import pkv_oracle


def _bf16(x):
    return x.to(torch.bfloat16)


def test_equals_library_softmax_attention():
    torch.manual_seed(0)
    for (B, Hq, Hkv, d, k_cap) in [(2, 8, 2, 64, 50), (1, 4, 4, 128, 33), (3, 6, 3, 64, 7)]:
        q = _bf16(torch.randn(B, Hq, d) * 2)
        Ks, Vs = _bf16(torch.randn(B, Hkv, k_cap, d)), _bf16(torch.randn(B, Hkv, k_cap, d))
        count = np.array([k_cap, max(k_cap // 2, 1), 1][:B], dtype=np.int32)
        out, lse = pkv_oracle.decode_attention(q, Ks, Vs, count)
        G = Hq // Hkv
        for b in range(B):
            n = int(count[b])
            for h in range(Hq):
                logits = (Ks[b, h // G, :n].double() @ q[b, h].double()) / math.sqrt(d)
                want = torch.softmax(logits, dim=0) @ Vs[b, h // G, :n].double()
                np.testing.assert_allclose(out[b, h], want.numpy(), rtol=1e-12, atol=1e-14)
                np.testing.assert_allclose(lse[b, h], torch.logsumexp(logits, dim=0).item(), rtol=1e-12)


def test_identical_keys_give_the_mean_of_the_values_and_one_key_its_value():
    torch.manual_seed(1)
    B, Hq, Hkv, d, k_cap = 1, 4, 2, 64, 20
    q = _bf16(torch.randn(B, Hq, d))
    Ks = _bf16(torch.randn(1, 1, 1, d)).expand(B, Hkv, k_cap, d).contiguous()
    Vs = _bf16(torch.randn(B, Hkv, k_cap, d))
    out, lse = pkv_oracle.decode_attention(q, Ks, Vs, np.array([k_cap]))
    for h in range(Hq):
        np.testing.assert_allclose(out[0, h], Vs[0, h // 2].double().mean(dim=0).numpy(), rtol=1e-12, atol=1e-14)
        logit = float(Ks[0, 0, 0].double() @ q[0, h].double()) / math.sqrt(d)
        assert abs(lse[0, h] - (logit + math.log(k_cap))) < 1e-12
    out1, _ = pkv_oracle.decode_attention(q, Ks, Vs, np.array([1]))
    for h in range(Hq):
        np.testing.assert_array_equal(out1[0, h], Vs[0, h // 2, 0].double().numpy())


def test_empty_cache_gives_zero_rows():
    q = _bf16(torch.randn(2, 2, 64))
    Ks = _bf16(torch.randn(2, 1, 4, 64))
    out, lse = pkv_oracle.decode_attention(q, Ks, Ks, np.array([0, 4]))
    assert not out[0].any() and np.all(np.isneginf(lse[0])) and out[1].any()

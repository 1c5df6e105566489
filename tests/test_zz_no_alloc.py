"""pkv_compress_layer_noalloc (the entry point for callers that cannot allocate) against pkv_compress_layer.

Both run the same kernels, the first on the library's built-in scratch buffer, the second on a caller workspace:
every output must be equal bit for bit.  Two calls in a row on the same device, the second with a smaller input,
so that the buffer still holds the first call's contents when the second starts; then once more against the
oracle."""
import pytest
import torch

from paper_2406_02069_amd import binding, synth
from tests.parity import compare_layer

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def _both(w, layer, k_l):
    Q, K, V, lens = synth.make_layer(w, layer, DEV)
    lens_dev = None if lens is None else torch.from_numpy(lens).to(DEV)
    want = binding.compress_layer(Q, K, V, k_l, w.pool, w.pool_w, seq_lens=lens_dev, want_scores=True)
    outs = binding.alloc_outputs(Q, K, k_l, want_scores=True)
    for t in outs[:4]:
        t.fill_(-7)           # stale contents must not survive
    torch.cuda.synchronize()
    got = binding.compress_layer_noalloc(Q, K, V, k_l, w.pool, w.pool_w, outs, seq_lens=lens_dev)
    torch.cuda.synchronize()
    for name, x, y in zip(("K_out", "V_out", "idx", "count", "scores"), got, want):
        assert torch.equal(x, y), (w.name, layer, name)
    return Q, K, V, lens, got


def test_noalloc_equals_the_workspace_entry_point_on_two_calls_in_a_row():
    # first call: a unit of 24 parts (tagged exchange, several groups); second call: a smaller input with units of
    # 3 parts (arrival counter), whose scratch regions overlap what the first call left behind
    big = synth.WORKLOADS[2].scaled(N=12000, L=2)
    small = synth.WORKLOADS[1].scaled(N=1500, L=2)
    _both(big, 0, 200)
    Q, K, V, lens, got = _both(small, 1, 90)
    compare_layer(Q, K, V, 90, small.alpha, small.pool, small.pool_w, lens, got)
    # and the other way round: large after small
    _both(big, 1, 64)


def test_noalloc_ragged_batch_and_streaming_kernels(monkeypatch):
    w = synth.WORKLOADS[3].scaled(N=3000, L=1, B=3, ragged_min=1200)
    _both(w, 0, 256)
    monkeypatch.setattr(binding, "DESC_FLAGS", binding.FLAG_STREAM_SCORING)
    _both(w, 0, 100)


def test_noalloc_rejects_what_does_not_fit():
    w = synth.WORKLOADS[1]
    Q = torch.zeros(8, w.Hq, w.alpha, w.d, dtype=torch.bfloat16, device=DEV)
    K = torch.zeros(8, w.Hkv, 65536, w.d, dtype=torch.bfloat16, device=DEV)
    outs = binding.alloc_outputs(Q, K, 128)
    with pytest.raises(binding.PkvError) as e:
        binding.compress_layer_noalloc(Q, K, K, 128, w.pool, w.pool_w, outs)
    assert e.value.status == binding.ERR_SCRATCH

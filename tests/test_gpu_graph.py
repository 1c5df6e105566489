"""The calls of the path recorded into a HIP graph and replayed: every launch goes to the caller's stream, nothing
allocates or synchronises, and the scratch is cleared by a kernel (not a memset node), so a captured step must give
the eager result on every replay, with eager work of the same library between the replays."""
import numpy as np
import pytest
import torch

from paper_2406_02069_amd import binding, synth

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def _same(a, b):
    for x, y in zip(a, b):
        for t, u in zip(x, y):
            if t is None or u is None:
                assert t is None and u is None
            else:
                assert torch.equal(t.view(torch.uint8) if t.dtype == torch.bfloat16 else t,
                                   u.view(torch.uint8) if u.dtype == torch.bfloat16 else u)


def _clone(outs):
    return [tuple(None if t is None else t.clone() for t in o) for o in outs]


@pytest.mark.parametrize("cfg,N,L", [(2, 9000, 3), (1, 3000, 4), (3, 9000, 2)])
def test_compress_layers_in_a_graph(cfg, N, L):
    w = synth.WORKLOADS[cfg].scaled(N=N, L=L, **({"ragged_min": 5000, "B": 3} if cfg == 3 else {}))
    ks = binding.budgets(w.L, w.avg_budgets[0], w.beta, w.alpha)
    lens = synth.seq_lens(w)
    lens_dev = None if lens is None else torch.from_numpy(lens).to(DEV)
    layers = [synth.make_layer(w, l, DEV) for l in range(w.L)]
    call = binding.LayersCall([x[0] for x in layers], [x[1] for x in layers], [x[2] for x in layers], ks, w.pool,
                              w.pool_w, seq_lens=lens_dev, want_scores=True)
    want = _clone(call.run())       # eager; also sets the per-device launch attributes before anything is recorded
    torch.cuda.synchronize()
    side = torch.cuda.Stream()      # default priority
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        with torch.cuda.graph(graph, stream=side):
            call.run()
    other = binding.LayersCall([x[0] for x in layers[:1]], [x[1] for x in layers[:1]], [x[2] for x in layers[:1]],
                               ks[:1], w.pool, w.pool_w, seq_lens=lens_dev)
    for rep in range(4):
        for o in call.outputs:      # poison what the replay must rewrite
            o[2].fill_(-7)
            o[3].fill_(-7)
        graph.replay()
        torch.cuda.synchronize()
        _same(call.outputs, want)
        other.run()                 # eager work of the library (its own workspace) between the replays
        torch.cuda.synchronize()
    first = binding.compress_layer(layers[0][0], layers[0][1], layers[0][2], ks[0], w.pool, w.pool_w, seq_lens=lens_dev)
    torch.cuda.synchronize()
    assert torch.equal(first[2], want[0][2]) and torch.equal(first[3], want[0][3])


def test_noalloc_entry_in_a_graph():
    # what the entry is for: a caller under graph capture, where no allocation is possible
    w = synth.WORKLOADS[1].scaled(N=6000, L=1)
    Q, K, V, _ = synth.make_layer(w, 0, DEV)
    k_l = 200
    want = _clone([binding.compress_layer(Q, K, V, k_l, w.pool, w.pool_w, want_scores=True)])
    outs = binding.alloc_outputs(Q, K, k_l, True)
    binding.compress_layer_noalloc(Q, K, V, k_l, w.pool, w.pool_w, outs)   # first call on the device: address look-up
    torch.cuda.synchronize()
    _same([outs], want)
    side = torch.cuda.Stream()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        with torch.cuda.graph(graph, stream=side):
            binding.compress_layer_noalloc(Q, K, V, k_l, w.pool, w.pool_w, outs)
    for rep in range(3):
        outs[2].fill_(-7)
        outs[3].fill_(-7)
        graph.replay()
        torch.cuda.synchronize()
        _same([outs], want)
        binding.compress_layer(Q, K, V, k_l + 8, w.pool, w.pool_w)   # eager work between the replays
        torch.cuda.synchronize()

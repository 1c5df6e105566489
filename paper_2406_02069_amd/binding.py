"""Thin Python binding of the C-ABI library libpkv (include/pkv.h).

Argument marshalling only: torch tensors supply device memory and the current
stream; every step of the method runs in the library's HIP kernels.  There is
no CPU fallback: if libpkv.so is missing or a call fails, an exception is raised.
Function names mirror the C entry points.
"""
from __future__ import annotations

import ctypes
import os
from typing import List, Optional, Sequence

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libpkv.so")

POOL_NONE, POOL_MAX, POOL_AVG = 0, 1, 2
OK, ERR_INVALID_ARG, ERR_UNSUPPORTED, ERR_WORKSPACE, ERR_HIP, ERR_SCRATCH = 0, 1, 2, 3, 4, 5
NOALLOC_SCRATCH_BYTES = 32 << 20   # PKV_NOALLOC_SCRATCH_BYTES of include/pkv.h

# pkv_layer_desc.flags (include/pkv_measure.h): test and measurement switches, 0 in production.  Descriptors made
# by this module carry DESC_FLAGS, which tests set to run the other scoring path or exchange.
FLAG_STREAM_SCORING, FLAG_COUNTER_EXCHANGE, FLAG_NO_WAIT = 1, 2, 4
DESC_FLAGS = 0

EXPORTS = ["pkv_budgets", "pkv_workspace_bytes", "pkv_compress_layer", "pkv_compress_layer_noalloc", "pkv_compress_layers",
           "pkv_compress_layers_lse", "pkv_compress_layers_paged", "pkv_compress_layers_profiled",
           "pkv_budgets_schedule", "pkv_attention_recall", "pkv_decode_attention", "pkv_decode_workspace_bytes", "pkv_decode_attention_layers",
           "pkv_decode_layers_workspace_bytes", "pkv_probe_read", "pkv_status_string"]


class PkvError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__(f"{where}: {status_string(status)} (status {status})")


class LayerDesc(ctypes.Structure):
    _fields_ = [(n, ctypes.c_int32) for n in
                ("B", "Hq", "Hkv", "d", "N", "alpha", "k_l", "pool", "pool_w", "flags")] + \
               [(n, ctypes.c_int64) for n in
                ("q_sb", "q_sh", "q_st", "kv_sb", "kv_sh", "kv_st", "o_sb", "o_sh", "o_st")]


class DecodeDesc(ctypes.Structure):
    _fields_ = [(n, ctypes.c_int32) for n in ("B", "Hq", "Hkv", "d", "k_cap", "page_size", "num_pages", "max_pages",
                                              "reserved", "reserved2")] + \
               [(n, ctypes.c_int64) for n in ("c_sb", "c_sh", "c_st")]


class PagedDesc(ctypes.Structure):
    _fields_ = [(n, ctypes.c_int32) for n in ("page_size", "num_pages", "max_pages", "reserved")]


_lib = None


def load() -> ctypes.CDLL:
    """Load libpkv.so (built in-tree by paper_2406_02069_amd.build).  Fails loudly if absent."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise FileNotFoundError(f"{LIB_PATH} not built: run `python -m paper_2406_02069_amd.build`")
        lib = ctypes.CDLL(LIB_PATH)
        vp, i32 = ctypes.c_void_p, ctypes.c_int32
        lib.pkv_budgets.argtypes = [i32, i32, i32, i32, vp]
        lib.pkv_budgets.restype = ctypes.c_int
        lib.pkv_workspace_bytes.argtypes = [ctypes.POINTER(LayerDesc), i32]
        lib.pkv_workspace_bytes.restype = ctypes.c_size_t
        lib.pkv_compress_layer.argtypes = [ctypes.POINTER(LayerDesc)] + [vp] * 10 + [ctypes.c_size_t, vp]
        lib.pkv_compress_layer.restype = ctypes.c_int
        lib.pkv_compress_layer_noalloc.argtypes = [ctypes.POINTER(LayerDesc)] + [vp] * 10
        lib.pkv_compress_layer_noalloc.restype = ctypes.c_int
        lib.pkv_compress_layers.argtypes = [i32, ctypes.POINTER(LayerDesc)] + [vp] * 10 + [ctypes.c_size_t, vp]
        lib.pkv_compress_layers.restype = ctypes.c_int
        lib.pkv_compress_layers_lse.argtypes = [i32, ctypes.POINTER(LayerDesc)] + [vp] * 11 + [ctypes.c_size_t, vp]
        lib.pkv_compress_layers_lse.restype = ctypes.c_int
        lib.pkv_compress_layers_paged.argtypes = [i32, ctypes.POINTER(LayerDesc)] + [vp] * 5 + \
            [ctypes.POINTER(PagedDesc)] + [vp] * 6 + [vp, ctypes.c_size_t, vp]
        lib.pkv_compress_layers_paged.restype = ctypes.c_int
        lib.pkv_budgets_schedule.argtypes = [i32, i32, i32, i32, i32, vp]
        lib.pkv_budgets_schedule.restype = ctypes.c_int
        lib.pkv_attention_recall.argtypes = [i32, ctypes.POINTER(LayerDesc), i32, vp, vp, vp, vp, ctypes.c_size_t, vp]
        lib.pkv_attention_recall.restype = ctypes.c_int
        lib.pkv_decode_attention.argtypes = [ctypes.POINTER(DecodeDesc)] + [vp] * 8 + [ctypes.c_size_t, vp]
        lib.pkv_decode_workspace_bytes.argtypes = [ctypes.POINTER(DecodeDesc)]
        lib.pkv_decode_workspace_bytes.restype = ctypes.c_size_t
        lib.pkv_decode_attention.restype = ctypes.c_int
        lib.pkv_decode_layers_workspace_bytes.argtypes = [i32, ctypes.POINTER(DecodeDesc)]
        lib.pkv_decode_layers_workspace_bytes.restype = ctypes.c_size_t
        lib.pkv_decode_attention_layers.argtypes = [i32, ctypes.POINTER(DecodeDesc)] + [vp] * 8 + [ctypes.c_size_t, vp]
        lib.pkv_decode_attention_layers.restype = ctypes.c_int
        lib.pkv_status_string.argtypes = [ctypes.c_int]
        lib.pkv_status_string.restype = ctypes.c_char_p
        _lib = lib
    return _lib


def status_string(status: int) -> str:
    return load().pkv_status_string(int(status)).decode()


def budgets(L: int, avg_budget: int, beta: int, alpha: int) -> List[int]:
    """pkv_budgets: per-layer cache sizes k_l (window included)."""
    out = (ctypes.c_int32 * max(L, 1))()
    rc = load().pkv_budgets(L, avg_budget, beta, alpha, ctypes.cast(out, ctypes.c_void_p))
    if rc != OK:
        raise PkvError(rc, "pkv_budgets")
    return [int(x) for x in out[:L]]


SCHEDULE_LINEAR, SCHEDULE_GEOMETRIC, SCHEDULE_UNIFORM = 0, 1, 2


def budgets_schedule(L: int, avg_budget: int, beta: int, alpha: int, schedule: int) -> List[int]:
    """pkv_budgets_schedule: linear (pkv_budgets), geometric or uniform per-layer budgets."""
    out = (ctypes.c_int32 * max(L, 1))()
    rc = load().pkv_budgets_schedule(L, avg_budget, beta, alpha, schedule, out)
    if rc != OK:
        raise PkvError(rc, "pkv_budgets_schedule")
    return [int(out[l]) for l in range(L)]


def _check_bf16(t: torch.Tensor, name: str):
    if t.dtype != torch.bfloat16 or t.dim() != 4 or t.stride(3) != 1:
        raise ValueError(f"{name}: need a 4-d bf16 tensor with a contiguous last dimension")


def make_desc(Q_win: torch.Tensor, K: torch.Tensor, k_l: int, pool: int, pool_w: int,
              K_out: Optional[torch.Tensor] = None) -> LayerDesc:
    B, Hq, alpha, d = Q_win.shape
    _, Hkv, N, _ = K.shape
    k_cap = min(int(k_l), N)
    if K_out is not None:
        o = (K_out.stride(0), K_out.stride(1), K_out.stride(2))
    else:
        o = (Hkv * k_cap * d, k_cap * d, d)
    return LayerDesc(B, Hq, Hkv, d, N, alpha, int(k_l), int(pool), int(pool_w), int(DESC_FLAGS),
                     Q_win.stride(0), Q_win.stride(1), Q_win.stride(2),
                     K.stride(0), K.stride(1), K.stride(2), o[0], o[1], o[2])


def workspace_bytes(desc: LayerDesc, L: int = 1) -> int:
    return int(load().pkv_workspace_bytes(ctypes.byref(desc), L))


def alloc_workspace(desc: LayerDesc, device, L: int = 1) -> torch.Tensor:
    nbytes = workspace_bytes(desc, L)
    if nbytes == 0:
        raise PkvError(ERR_INVALID_ARG, "pkv_workspace_bytes")
    return torch.empty(nbytes, dtype=torch.uint8, device=device)  # torch allocations are >= 256-byte aligned


def alloc_outputs(Q_win: torch.Tensor, K: torch.Tensor, k_l: int, want_scores: bool = False):
    B, Hq, alpha, d = Q_win.shape
    _, Hkv, N, _ = K.shape
    k_cap = min(int(k_l), N)
    dev = K.device
    K_out = torch.empty((B, Hkv, k_cap, d), dtype=torch.bfloat16, device=dev)
    V_out = torch.empty((B, Hkv, k_cap, d), dtype=torch.bfloat16, device=dev)
    idx = torch.empty((B, Hkv, k_cap), dtype=torch.int32, device=dev)
    count = torch.empty((B,), dtype=torch.int32, device=dev)
    scores = torch.zeros((B, Hkv, N), dtype=torch.float32, device=dev) if want_scores else None
    return K_out, V_out, idx, count, scores


def _p(t: Optional[torch.Tensor]):
    return None if t is None else ctypes.c_void_p(t.data_ptr())


def _stream_ptr(device) -> ctypes.c_void_p:
    return ctypes.c_void_p(torch.cuda.current_stream(device).cuda_stream)


def compress_layer(Q_win: torch.Tensor, K: torch.Tensor, V: torch.Tensor, k_l: int, pool: int, pool_w: int,
                   seq_lens: Optional[torch.Tensor] = None, outputs=None, workspace: Optional[torch.Tensor] = None,
                   want_scores: bool = False):
    """pkv_compress_layer on the current torch stream.  Returns (K_out, V_out, idx, count, scores)."""
    _check_bf16(Q_win, "Q_win"), _check_bf16(K, "K"), _check_bf16(V, "V")
    if V.shape != K.shape or V.stride() != K.stride():
        raise ValueError("K and V must have the same shape and strides")
    if outputs is None:
        outputs = alloc_outputs(Q_win, K, k_l, want_scores)
    K_out, V_out, idx, count, scores = outputs
    desc = make_desc(Q_win, K, k_l, pool, pool_w, K_out)
    if workspace is None:
        workspace = alloc_workspace(desc, K.device)
    if seq_lens is not None and (seq_lens.dtype != torch.int32 or not seq_lens.is_contiguous()):
        raise ValueError("seq_lens must be a contiguous int32 tensor")
    rc = load().pkv_compress_layer(ctypes.byref(desc), _p(Q_win), _p(K), _p(V), _p(seq_lens), _p(K_out), _p(V_out),
                                   _p(idx), _p(count), _p(scores), _p(workspace), workspace.numel(),
                                   _stream_ptr(K.device))
    if rc != OK:
        raise PkvError(rc, "pkv_compress_layer")
    return outputs


def compress_layer_noalloc(Q_win: torch.Tensor, K: torch.Tensor, V: torch.Tensor, k_l: int, pool: int, pool_w: int,
                           outputs, seq_lens: Optional[torch.Tensor] = None):
    """pkv_compress_layer_noalloc on the current torch stream: the library's built-in scratch buffer serves as the
    workspace, and nothing is allocated here either (the caller passes the output tensors of alloc_outputs)."""
    _check_bf16(Q_win, "Q_win"), _check_bf16(K, "K"), _check_bf16(V, "V")
    if V.shape != K.shape or V.stride() != K.stride():
        raise ValueError("K and V must have the same shape and strides")
    K_out, V_out, idx, count, scores = outputs
    desc = make_desc(Q_win, K, k_l, pool, pool_w, K_out)
    if seq_lens is not None and (seq_lens.dtype != torch.int32 or not seq_lens.is_contiguous()):
        raise ValueError("seq_lens must be a contiguous int32 tensor")
    rc = load().pkv_compress_layer_noalloc(ctypes.byref(desc), _p(Q_win), _p(K), _p(V), _p(seq_lens), _p(K_out),
                                           _p(V_out), _p(idx), _p(count), _p(scores), _stream_ptr(K.device))
    if rc != OK:
        raise PkvError(rc, "pkv_compress_layer_noalloc")
    return outputs


class LayersCall:
    """Pre-marshalled arguments of pkv_compress_layers, so that a timed loop only crosses the ABI."""

    def __init__(self, Q_win: Sequence[torch.Tensor], K: Sequence[torch.Tensor], V: Sequence[torch.Tensor],
                 k_ls: Sequence[int], pool: int, pool_w: int, seq_lens: Optional[torch.Tensor] = None,
                 want_scores: bool = False, lse: Optional[Sequence[torch.Tensor]] = None, paged=None):
        """paged: None, or (K_pages, V_pages, block_tables, page_size): per layer bf16 pools
        [num_pages, Hkv, page_size, d] and int32 tables [B, max_pages]; the kept rows then go into the pools
        (pkv_compress_layers_paged) and the first two entries of every output tuple are the layer's pools."""
        L = len(K)
        assert len(Q_win) == L and len(V) == L and len(k_ls) == L
        self.L = L
        self.inputs = (list(Q_win), list(K), list(V), seq_lens)
        self.outputs = [alloc_outputs(Q_win[l], K[l], k_ls[l], want_scores) for l in range(L)]
        self.descs = (LayerDesc * L)(*[make_desc(Q_win[l], K[l], k_ls[l], pool, pool_w, self.outputs[l][0])
                                        for l in range(L)])
        self.workspace = alloc_workspace(self.descs[0], K[0].device, L)
        arr = ctypes.c_void_p * L

        def ptrs(ts):
            return arr(*[None if t is None else t.data_ptr() for t in ts])

        self._args = [ptrs(Q_win), ptrs(K), ptrs(V), _p(seq_lens)] + \
                     [ptrs([o[i] for o in self.outputs]) for i in range(4)] + \
                     [ptrs([o[4] for o in self.outputs]) if want_scores else None]
        self.device = K[0].device
        self._lse = None
        if lse is not None:  # per layer: fp32 [B, Hq, alpha] contiguous, natural-log softmax denominators
            B, Hq, alpha, _ = Q_win[0].shape
            assert len(lse) == L
            for t in lse:
                assert t.dtype == torch.float32 and t.is_contiguous() and tuple(t.shape) == (B, Hq, alpha)
            self.inputs = self.inputs + (list(lse),)
            self._lse = ptrs(lse)

        self._paged = None
        if paged is not None:
            Kp, Vp, tables, page_size = paged
            assert len(Kp) == L and len(Vp) == L and len(tables) == L
            B, Hkv, d = K[0].shape[0], K[0].shape[1], K[0].shape[3]
            num_pages, max_pages = Kp[0].shape[0], tables[0].shape[1]
            for l in range(L):
                assert Kp[l].dtype == torch.bfloat16 and Kp[l].is_contiguous() and Vp[l].is_contiguous()
                assert tuple(Kp[l].shape) == (num_pages, Hkv, page_size, d) == tuple(Vp[l].shape)
                assert tables[l].dtype == torch.int32 and tables[l].is_contiguous()
                assert tuple(tables[l].shape) == (B, max_pages)
            self.inputs = self.inputs + (list(Kp), list(Vp), list(tables))
            self._paged = (PagedDesc(page_size, num_pages, max_pages, 0), ptrs(Kp), ptrs(Vp), ptrs(tables))
            self.outputs = [(Kp[l], Vp[l]) + tuple(o[2:]) for l, o in enumerate(self.outputs)]

    def run(self):
        tail = (_p(self.workspace), self.workspace.numel(), _stream_ptr(self.device))
        if self._paged is not None:
            a, (pd, kp, vp, tb) = self._args, self._paged
            rc = load().pkv_compress_layers_paged(self.L, self.descs, a[0], a[1], a[2], self._lse, a[3],
                                                  ctypes.byref(pd), kp, vp, tb, a[6], a[7], a[8], *tail)
            if rc != OK:
                raise PkvError(rc, "pkv_compress_layers_paged")
            return self.outputs
        if self._lse is not None:
            a = self._args
            rc = load().pkv_compress_layers_lse(self.L, self.descs, a[0], a[1], a[2], self._lse, *a[3:], *tail)
        else:
            rc = load().pkv_compress_layers(self.L, self.descs, *self._args, *tail)
        if rc != OK:
            raise PkvError(rc, "pkv_compress_layers_lse" if self._lse is not None else "pkv_compress_layers")
        return self.outputs


def attention_recall(call: "LayersCall") -> List[torch.Tensor]:
    """pkv_attention_recall right after call.run(): per layer fp32 [B, Hkv]."""
    B, Hkv = call.inputs[1][0].shape[0], call.inputs[1][0].shape[1]
    outs = [torch.empty(B, Hkv, dtype=torch.float32, device=call.device) for _ in range(call.L)]
    arr = ctypes.c_void_p * call.L
    rc = load().pkv_attention_recall(call.L, call.descs, 1 if call._lse is not None else 0, call._args[3],
                                     call._args[6], arr(*[t.data_ptr() for t in outs]), _p(call.workspace),
                                     call.workspace.numel(), _stream_ptr(call.device))
    if rc != OK:
        raise PkvError(rc, "pkv_attention_recall")
    return outs


def decode_attention(q: torch.Tensor, K_cache: torch.Tensor, V_cache: torch.Tensor, count: torch.Tensor,
                     block_table: Optional[torch.Tensor] = None, k_cap: Optional[int] = None, want_lse: bool = False,
                     out: Optional[torch.Tensor] = None, lse: Optional[torch.Tensor] = None,
                     workspace: Optional[torch.Tensor] = None):
    """pkv_decode_attention.  q bf16 [B,Hq,d]; compact cache: K_cache, V_cache bf16 [B,Hkv,k_cap,d] (any row strides);
    paged cache: pools [num_pages,Hkv,page_size,d], block_table int32 [B,max_pages] and k_cap given.
    Returns (out fp32 [B,Hq,d], lse fp32 [B,Hq] or None)."""
    assert q.dtype == torch.bfloat16 and q.dim() == 3 and q.is_contiguous() and count.dtype == torch.int32
    assert K_cache.dtype == torch.bfloat16 and V_cache.dtype == torch.bfloat16
    B, Hq, d = q.shape
    if block_table is None:
        Hkv, k_cap = K_cache.shape[1], K_cache.shape[2]
        assert K_cache.stride() == V_cache.stride() and K_cache.stride(3) == 1
        desc = DecodeDesc(B, Hq, Hkv, d, k_cap, 0, 0, 0, 0, 0, K_cache.stride(0), K_cache.stride(1), K_cache.stride(2))
    else:
        num_pages, Hkv, page_size, _ = K_cache.shape
        assert K_cache.is_contiguous() and V_cache.is_contiguous() and block_table.is_contiguous()
        assert block_table.dtype == torch.int32 and k_cap is not None
        desc = DecodeDesc(B, Hq, Hkv, d, k_cap, page_size, num_pages, block_table.shape[1], 0, 0, 0, 0, 0)
    if out is None:
        out = torch.empty(B, Hq, d, dtype=torch.float32, device=q.device)
    if want_lse and lse is None:
        lse = torch.empty(B, Hq, dtype=torch.float32, device=q.device)
    need = load().pkv_decode_workspace_bytes(ctypes.byref(desc))
    if workspace is None and need > 0:
        workspace = torch.empty(need, dtype=torch.uint8, device=q.device)
    rc = load().pkv_decode_attention(ctypes.byref(desc), q.data_ptr(), K_cache.data_ptr(), V_cache.data_ptr(),
                                     _p(block_table), count.data_ptr(), out.data_ptr(), _p(lse), _p(workspace),
                                     0 if workspace is None else workspace.numel(), _stream_ptr(q.device))
    if rc != OK:
        raise PkvError(rc, "pkv_decode_attention")
    return out, lse


class DecodeLayersCall:
    """pkv_decode_attention_layers over the caches of L layers, marshalled once and launched any number of times.
    qs[l] bf16 [B,Hq,d]; compact caches: K_caches[l], V_caches[l] bf16 [B,Hkv,k_cap_l,d] (any row strides); paged:
    pools [num_pages_l,Hkv,page_size,d] with block_tables[l] int32 [B,max_pages_l] and k_caps[l]; counts[l] int32 [B].
    outputs: list of (out fp32 [B,Hq,d], lse fp32 [B,Hq] or None)."""

    def __init__(self, qs, K_caches, V_caches, counts, block_tables=None, k_caps=None, want_lse=False):
        L = len(qs)
        B, Hq, d = qs[0].shape
        dev = qs[0].device
        descs = (DecodeDesc * L)()
        for l in range(L):
            q, K, V = qs[l], K_caches[l], V_caches[l]
            assert q.dtype == torch.bfloat16 and q.is_contiguous() and counts[l].dtype == torch.int32
            assert K.dtype == torch.bfloat16 and V.dtype == torch.bfloat16
            if block_tables is None:
                assert K.stride() == V.stride() and K.stride(3) == 1
                descs[l] = DecodeDesc(B, Hq, K.shape[1], d, K.shape[2], 0, 0, 0, 0, 0, K.stride(0), K.stride(1), K.stride(2))
            else:
                tb = block_tables[l]
                assert K.is_contiguous() and V.is_contiguous() and tb.is_contiguous() and tb.dtype == torch.int32
                descs[l] = DecodeDesc(B, Hq, K.shape[1], d, k_caps[l], K.shape[2], K.shape[0], tb.shape[1], 0, 0, 0, 0, 0)
        self.L, self.descs, self.dev = L, descs, dev
        self.keep = (qs, K_caches, V_caches, counts, block_tables)
        self.outputs = [(torch.empty(B, Hq, d, dtype=torch.float32, device=dev),
                         torch.empty(B, Hq, dtype=torch.float32, device=dev) if want_lse else None) for _ in range(L)]
        arr = ctypes.c_void_p * L
        self.a_q = arr(*[t.data_ptr() for t in qs])
        self.a_K = arr(*[t.data_ptr() for t in K_caches])
        self.a_V = arr(*[t.data_ptr() for t in V_caches])
        self.a_tb = None if block_tables is None else arr(*[t.data_ptr() for t in block_tables])
        self.a_cnt = arr(*[t.data_ptr() for t in counts])
        self.a_out = arr(*[o[0].data_ptr() for o in self.outputs])
        self.a_lse = arr(*[o[1].data_ptr() for o in self.outputs]) if want_lse else None
        need = load().pkv_decode_layers_workspace_bytes(L, descs)
        self.ws = torch.empty(max(need, 1), dtype=torch.uint8, device=dev) if need > 0 else None
        self.ws_bytes = need

    def run(self):
        rc = load().pkv_decode_attention_layers(self.L, self.descs, self.a_q, self.a_K, self.a_V, self.a_tb, self.a_cnt,
                                                self.a_out, self.a_lse, _p(self.ws), self.ws_bytes,
                                                _stream_ptr(self.dev))
        if rc != OK:
            raise PkvError(rc, "pkv_decode_attention_layers")
        return self.outputs


def decode_attention_layers(qs, K_caches, V_caches, counts, block_tables=None, k_caps=None, want_lse=False):
    """pkv_decode_attention_layers: one call for the caches of all layers.  Returns [(out, lse or None)] per layer."""
    return DecodeLayersCall(qs, K_caches, V_caches, counts, block_tables, k_caps, want_lse).run()


def compress_layers(Q_win, K, V, k_ls, pool, pool_w, seq_lens=None, want_scores=False):
    """pkv_compress_layers: all layers of one request batch.  Returns a list of per-layer output tuples."""
    return LayersCall(Q_win, K, V, k_ls, pool, pool_w, seq_lens, want_scores).run()


def compress_layers_lse(Q_win, K, V, lse, k_ls, pool, pool_w, seq_lens=None, want_scores=False):
    """pkv_compress_layers_lse: the same with the window queries' softmax denominators supplied per layer
    (fp32 [B, Hq, alpha] each)."""
    return LayersCall(Q_win, K, V, k_ls, pool, pool_w, seq_lens, want_scores, lse=lse).run()


def compress_layers_paged(Q_win, K, V, k_ls, pool, pool_w, K_pages, V_pages, block_tables, page_size,
                          seq_lens=None, want_scores=False, lse=None):
    """pkv_compress_layers_paged: kept rows written into per-layer page pools through per-layer block tables."""
    return LayersCall(Q_win, K, V, k_ls, pool, pool_w, seq_lens, want_scores, lse=lse,
                      paged=(K_pages, V_pages, block_tables, page_size)).run()


def probe_read(buf: torch.Tensor, sink: torch.Tensor) -> None:
    """pkv_probe_read: one streaming read of `buf` (contiguous, 16-byte multiple) on the current stream."""
    lib = load()
    lib.pkv_probe_read.argtypes = [ctypes.c_void_p, ctypes.c_size_t, ctypes.c_void_p, ctypes.c_void_p]
    lib.pkv_probe_read.restype = ctypes.c_int
    assert buf.is_contiguous() and sink.dtype == torch.int32
    rc = lib.pkv_probe_read(buf.data_ptr(), buf.numel() * buf.element_size(), sink.data_ptr(), _stream_ptr(buf.device))
    if rc != OK:
        raise PkvError(rc, "pkv_probe_read")


KERNEL_NAMES = ["score_stats", "score_finalize", "score_accum", "pool_select", "gather", "score_resident"]


class HipEvents:
    """A pool of timing-enabled HIP events (created through the HIP runtime that torch has loaded)."""

    def __init__(self, n: int):
        self.hip = ctypes.CDLL("libamdhip64.so.7")
        self.hip.hipEventCreate.argtypes = [ctypes.POINTER(ctypes.c_void_p)]
        self.hip.hipEventElapsedTime.argtypes = [ctypes.POINTER(ctypes.c_float), ctypes.c_void_p, ctypes.c_void_p]
        self.hip.hipEventDestroy.argtypes = [ctypes.c_void_p]
        self.n = n
        self.handles = (ctypes.c_void_p * n)()
        for i in range(n):
            ev = ctypes.c_void_p()
            if self.hip.hipEventCreate(ctypes.byref(ev)) != 0:
                raise RuntimeError("hipEventCreate failed")
            self.handles[i] = ev

    def elapsed_ms(self, i: int, j: int) -> float:
        ms = ctypes.c_float()
        rc = self.hip.hipEventElapsedTime(ctypes.byref(ms), self.handles[i], self.handles[j])
        if rc != 0:
            raise RuntimeError(f"hipEventElapsedTime failed ({rc})")
        return float(ms.value)

    def close(self):
        for i in range(self.n):
            self.hip.hipEventDestroy(self.handles[i])
        self.n = 0


def run_profiled(call: LayersCall, events: HipEvents):
    """pkv_compress_layers_profiled on the current stream.  Returns the kernel ids of the recorded intervals;
    after a stream synchronise, interval i lies between events i and i+1."""
    lib = load()
    if not hasattr(lib, "_prof_ready"):
        vp, i32 = ctypes.c_void_p, ctypes.c_int32
        lib.pkv_compress_layers_profiled.argtypes = [i32, ctypes.POINTER(LayerDesc)] + [vp] * 5 + \
            [ctypes.POINTER(PagedDesc), vp] + [vp] * 6 + \
            [ctypes.c_size_t, vp, vp, i32, vp, vp]
        lib.pkv_compress_layers_profiled.restype = ctypes.c_int
        lib._prof_ready = True
    ids = (ctypes.c_int32 * events.n)()
    used = ctypes.c_int32(0)
    a = call._args
    pd, kp, vp_, tb = call._paged if call._paged is not None else (None, a[4], a[5], None)
    rc = lib.pkv_compress_layers_profiled(call.L, call.descs, a[0], a[1], a[2], call._lse, a[3],
                                          None if pd is None else ctypes.byref(pd), tb, kp, vp_, a[6], a[7], a[8],
                                          _p(call.workspace),
                                          call.workspace.numel(), _stream_ptr(call.device), events.handles,
                                          events.n, ids, ctypes.byref(used))
    if rc != OK:
        raise PkvError(rc, "pkv_compress_layers_profiled")
    return [int(ids[i]) for i in range(used.value - 1)]

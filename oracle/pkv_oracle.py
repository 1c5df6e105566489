"""ctypes front end of the CPU oracle (oracle/pkv_oracle.c) -- TEST INFRASTRUCTURE ONLY.

Only tests, the smoke check and the benchmark's cpu_baseline leg may import
this module.  It holds no arithmetic of the method: it compiles the C file
with gcc, loads it and marshals numpy arrays.  bf16 tensors travel as their
raw 16-bit patterns (numpy uint16).
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from typing import Optional

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "pkv_oracle.c")
_LIB = os.path.join(_HERE, "libpkv_oracle.so")

POOL_NONE, POOL_MAX, POOL_AVG = 0, 1, 2

_lib = None


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (plain C, OpenMP over independent rows)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O2", "-std=c11", "-fopenmp", "-fPIC", "-shared", "-Wall", "-Wextra",
               "-o", _LIB, _SRC, "-lm"]
        subprocess.check_call(cmd)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        build()
        lib = ctypes.CDLL(_LIB)
        i32, p = ctypes.c_int32, ctypes.c_void_p
        lib.pkvo_budgets.argtypes = [i32, i32, i32, i32, p]
        lib.pkvo_window_scores.argtypes = [i32, i32, i32, i32, p, p, p, p]
        lib.pkvo_pool.argtypes = [i32, i32, i32, p, p]
        lib.pkvo_topk.argtypes = [i32, p, i32, p]
        lib.pkvo_window_scores_lse.argtypes = [i32, i32, i32, i32, p, p, p, p, p]
        lib.pkvo_compress_layer.argtypes = [i32] * 9 + [p] * 9
        lib.pkvo_compress_layer_lse.argtypes = [i32] * 9 + [p] * 10
        lib.pkvo_scatter_pages.argtypes = [i32] * 7 + [p] * 6
        lib.pkvo_scatter_pages.restype = ctypes.c_int
        lib.pkvo_decode_attention.argtypes = [i32] * 5 + [p] * 6
        lib.pkvo_decode_attention.restype = ctypes.c_int
        lib.pkvo_budgets_schedule.argtypes = [i32] * 5 + [p]
        lib.pkvo_budgets_schedule.restype = ctypes.c_int
        lib.pkvo_attention_recall.argtypes = [i32] * 4 + [p, p, p, i32, p]
        lib.pkvo_attention_recall.restype = ctypes.c_int
        for f in (lib.pkvo_budgets, lib.pkvo_window_scores, lib.pkvo_window_scores_lse, lib.pkvo_pool,
                  lib.pkvo_topk, lib.pkvo_compress_layer, lib.pkvo_compress_layer_lse,
                  lib.pkvo_num_threads):
            f.restype = ctypes.c_int
        _lib = lib
    return _lib


def _ptr(a: Optional[np.ndarray]):
    return None if a is None else a.ctypes.data_as(ctypes.c_void_p)


def _bits(a) -> np.ndarray:
    """Raw bf16 bit patterns as a contiguous uint16 numpy array.

    Accepts a numpy uint16 array or a torch bfloat16 tensor (any device)."""
    if isinstance(a, np.ndarray):
        assert a.dtype == np.uint16
        return np.ascontiguousarray(a)
    import torch  # only for the dtype view; no arithmetic

    assert a.dtype == torch.bfloat16
    return np.ascontiguousarray(a.detach().cpu().contiguous().view(torch.int16).numpy().view(np.uint16))


def num_threads() -> int:
    return int(_load().pkvo_num_threads())


def budgets(L: int, avg_budget: int, beta: int, alpha: int) -> np.ndarray:
    out = np.zeros(max(L, 1), dtype=np.int32)
    rc = _load().pkvo_budgets(L, avg_budget, beta, alpha, _ptr(out))
    if rc != 0:
        raise ValueError("pkvo_budgets: invalid arguments")
    return out[:L]


def window_scores(q, k, lse=None):
    """q: [G, alpha, d] bf16, k: [n, d] bf16 -> (s_head [G, n-alpha], s_mean [n-alpha]) fp64.

    lse: optional [G, alpha] float64, the supplied natural-log softmax denominators."""
    qb, kb = _bits(q), _bits(k)
    G, alpha, d = qb.shape
    n = kb.shape[0]
    assert kb.shape[1] == d
    s_head = np.zeros((G, n - alpha), dtype=np.float64)
    s_mean = np.zeros(n - alpha, dtype=np.float64)
    if lse is None:
        rc = _load().pkvo_window_scores(G, alpha, d, n, _ptr(qb), _ptr(kb), _ptr(s_head), _ptr(s_mean))
    else:
        lb = np.ascontiguousarray(lse, dtype=np.float64)
        assert lb.shape == (G, alpha)
        rc = _load().pkvo_window_scores_lse(G, alpha, d, n, _ptr(qb), _ptr(kb), _ptr(lb), _ptr(s_head),
                                            _ptr(s_mean))
    if rc != 0:
        raise ValueError("pkvo_window_scores: invalid arguments")
    return s_head, s_mean


def pool(kind: int, w: int, s: np.ndarray) -> np.ndarray:
    s = np.ascontiguousarray(s, dtype=np.float64)
    p = np.zeros_like(s)
    rc = _load().pkvo_pool(kind, w, s.shape[0], _ptr(s), _ptr(p))
    if rc != 0:
        raise ValueError("pkvo_pool: invalid arguments")
    return p


def topk(p: np.ndarray, kk: int) -> np.ndarray:
    p = np.ascontiguousarray(p, dtype=np.float64)
    idx = np.zeros(max(kk, 1), dtype=np.int32)
    rc = _load().pkvo_topk(p.shape[0], _ptr(p), kk, _ptr(idx))
    if rc != 0:
        raise ValueError("pkvo_topk: invalid arguments")
    return idx[:kk]


def compress_layer(Q_win, K, V, k_l: int, alpha: int, pool_kind: int, pool_w: int,
                   seq_lens=None, want_pooled: bool = True, lse=None):
    """One layer.  Q_win [B,Hq,alpha,d], K,V [B,Hkv,N,d] bf16 (torch) or uint16 bits (numpy).
    lse: optional [B,Hq,alpha] float32 supplied natural-log softmax denominators.

    Returns dict(K_out, V_out (uint16 bits [B,Hkv,k_cap,d]), idx [B,Hkv,k_cap] int32,
    count [B] int32, pooled [B,Hkv,N] float64 or None)."""
    qb, kb, vb = _bits(Q_win), _bits(K), _bits(V)
    B, Hq, a, d = qb.shape
    assert a == alpha
    _, Hkv, N, _ = kb.shape
    assert kb.shape == vb.shape and kb.shape[0] == B and kb.shape[3] == d
    k_cap = min(k_l, N)
    sl = None
    if seq_lens is not None:
        sl = np.ascontiguousarray(np.asarray(seq_lens, dtype=np.int32))
        assert sl.shape == (B,)
    K_out = np.zeros((B, Hkv, k_cap, d), dtype=np.uint16)
    V_out = np.zeros((B, Hkv, k_cap, d), dtype=np.uint16)
    idx = np.zeros((B, Hkv, k_cap), dtype=np.int32)
    count = np.zeros(B, dtype=np.int32)
    pooled = np.zeros((B, Hkv, N), dtype=np.float64) if want_pooled else None
    if lse is None:
        rc = _load().pkvo_compress_layer(B, Hq, Hkv, d, N, alpha, k_l, pool_kind, pool_w,
                                         _ptr(qb), _ptr(kb), _ptr(vb), _ptr(sl), _ptr(K_out), _ptr(V_out),
                                         _ptr(idx), _ptr(count), _ptr(pooled))
    else:
        lb = np.ascontiguousarray(lse, dtype=np.float32)
        assert lb.shape == (B, Hq, alpha)
        rc = _load().pkvo_compress_layer_lse(B, Hq, Hkv, d, N, alpha, k_l, pool_kind, pool_w,
                                             _ptr(qb), _ptr(kb), _ptr(vb), _ptr(sl), _ptr(lb), _ptr(K_out),
                                             _ptr(V_out), _ptr(idx), _ptr(count), _ptr(pooled))
    if rc != 0:
        raise ValueError("pkvo_compress_layer: invalid arguments")
    return dict(K_out=K_out, V_out=V_out, idx=idx, count=count, pooled=pooled)


def scatter_pages(K_out: np.ndarray, V_out: np.ndarray, count: np.ndarray, table: np.ndarray, page_size: int,
                  K_pages: np.ndarray, V_pages: np.ndarray):
    """Kept rows (K_out, V_out uint16 [B,Hkv,k_cap,d], count [B]) into copies of the page pools
    (uint16 [num_pages,Hkv,page_size,d]) through the block table (int32 [B,max_pages]).  Returns the new pools."""
    K_out, V_out = np.ascontiguousarray(K_out), np.ascontiguousarray(V_out)
    B, Hkv, k_cap, d = K_out.shape
    count = np.ascontiguousarray(count, dtype=np.int32)
    table = np.ascontiguousarray(table, dtype=np.int32)
    Kp, Vp = np.array(K_pages, dtype=np.uint16, order="C"), np.array(V_pages, dtype=np.uint16, order="C")
    num_pages = Kp.shape[0]
    assert Kp.shape == (num_pages, Hkv, page_size, d) == Vp.shape and table.shape[0] == B
    rc = _load().pkvo_scatter_pages(B, Hkv, d, k_cap, page_size, num_pages, table.shape[1], _ptr(K_out), _ptr(V_out),
                                    _ptr(count), _ptr(table), _ptr(Kp), _ptr(Vp))
    if rc != 0:
        raise ValueError(f"pkvo_scatter_pages: status {rc}")
    return Kp, Vp


SCHEDULE_LINEAR, SCHEDULE_GEOMETRIC, SCHEDULE_UNIFORM = 0, 1, 2


def budgets_schedule(L: int, avg_budget: int, beta: int, alpha: int, schedule: int) -> np.ndarray:
    out = np.zeros(max(L, 1), dtype=np.int32)
    rc = _load().pkvo_budgets_schedule(L, avg_budget, beta, alpha, schedule, _ptr(out))
    if rc != 0:
        raise ValueError("pkvo_budgets_schedule: invalid arguments")
    return out[:L]


def attention_recall(q, k, kept) -> float:
    """q: [G, alpha, d] bf16, k: [n, d] bf16 (the sequence's valid keys), kept: positions -> recall in [0, 1]."""
    qb, kb = _bits(q), _bits(k)
    G, alpha, d = qb.shape
    kept = np.ascontiguousarray(kept, dtype=np.int32)
    out = ctypes.c_double(0.0)
    rc = _load().pkvo_attention_recall(G, alpha, d, kb.shape[0], _ptr(qb), _ptr(kb), _ptr(kept), kept.shape[0],
                                       ctypes.byref(out))
    if rc != 0:
        raise ValueError("pkvo_attention_recall: invalid arguments")
    return float(out.value)


def decode_attention(q, Ks, Vs, count):
    """q [B,Hq,d], Ks, Vs [B,Hkv,k_cap,d] bf16 (torch) or uint16 bits, count [B] -> (out [B,Hq,d], lse [B,Hq]) fp64."""
    qb, kb, vb = _bits(q), _bits(Ks), _bits(Vs)
    B, Hq, d = qb.shape
    _, Hkv, k_cap, _ = kb.shape
    assert kb.shape == vb.shape == (B, Hkv, k_cap, d)
    count = np.ascontiguousarray(count, dtype=np.int32)
    out = np.zeros((B, Hq, d), dtype=np.float64)
    lse = np.zeros((B, Hq), dtype=np.float64)
    rc = _load().pkvo_decode_attention(B, Hq, Hkv, d, k_cap, _ptr(qb), _ptr(kb), _ptr(vb), _ptr(count), _ptr(out),
                                       _ptr(lse))
    if rc != 0:
        raise ValueError("pkvo_decode_attention: invalid arguments")
    return out, lse

"""Host-side checks of the C-ABI library: it loads, exports what include/pkv.h declares, computes the
budgets of Sec. 4.2.1 exactly like the oracle, and rejects bad arguments before any launch (no GPU needed)."""
import ctypes
import os
import re

import numpy as np
import pytest

from oracle import pkv_oracle
from paper_2406_02069_amd import binding

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)


def _declared():
    names = set()
    for header in ("pkv.h", "pkv_measure.h"):
        text = open(os.path.join(ROOT, "include", header)).read()
        text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
        names |= set(re.findall(r"\b(pkv_[a-z_]+)\s*\(", text))
    return sorted(names)


def test_library_loads_and_exports_every_declared_symbol():
    lib = binding.load()
    names = _declared()
    assert names == sorted(binding.EXPORTS)
    for n in names:
        assert getattr(lib, n) is not None


def test_status_strings():
    assert binding.status_string(0) == "ok"
    for s in range(1, 6):
        assert binding.status_string(s) not in ("ok", "unknown status")
    assert binding.status_string(99) == "unknown status"


def test_budgets_equal_oracle_on_golden_and_grid():
    with open(os.path.join(HERE, "golden", "budget_cases.txt")) as f:
        for line in f:
            if line.startswith("#"):
                continue
            head, tail = line.split(":")
            L, avg, beta, alpha = (int(x) for x in head.split())
            assert binding.budgets(L, avg, beta, alpha) == [int(x) for x in tail.split()]
    rs = np.random.RandomState(0)
    for _ in range(300):
        L = int(rs.randint(1, 100))
        alpha = int(rs.randint(0, 70))
        avg = alpha + int(rs.randint(0, 3000))
        beta = int(rs.randint(1, 40))
        assert binding.budgets(L, avg, beta, alpha) == list(pkv_oracle.budgets(L, avg, beta, alpha))


def test_budgets_reject_bad_arguments():
    for bad in [(0, 10, 20, 8), (4, 10, 0, 8), (4, 7, 20, 8), (4, 10, 20, -1)]:
        with pytest.raises(binding.PkvError) as e:
            binding.budgets(*bad)
        assert e.value.status == binding.ERR_INVALID_ARG
    assert binding.load().pkv_budgets(4, 128, 20, 8, None) == binding.ERR_INVALID_ARG


def _desc(**kw):
    base = dict(B=1, Hq=32, Hkv=8, d=128, N=4096, alpha=8, k_l=128, pool=1, pool_w=7, flags=0,
                q_sb=32 * 8 * 128, q_sh=8 * 128, q_st=128, kv_sb=8 * 4096 * 128, kv_sh=4096 * 128, kv_st=128,
                o_sb=8 * 128 * 128, o_sh=128 * 128, o_st=128)
    base.update(kw)
    return binding.LayerDesc(**base)


def _call(desc, ws_bytes=None, ws=0x10000, **ptr_overrides):
    lib = binding.load()
    p = dict(Q=0x1000, K=0x2000, V=0x3000, seq=None, Ko=0x4000, Vo=0x5000, idx=0x6000, cnt=0x7000, sc=None)
    p.update(ptr_overrides)
    if ws_bytes is None:
        ws_bytes = binding.workspace_bytes(desc)
    return lib.pkv_compress_layer(ctypes.byref(desc), p["Q"], p["K"], p["V"], p["seq"], p["Ko"], p["Vo"], p["idx"],
                                  p["cnt"], p["sc"], ws, ws_bytes, None)


def test_workspace_size_is_positive_and_budget_independent():
    a = binding.workspace_bytes(_desc(k_l=64))
    b = binding.workspace_bytes(_desc(k_l=4000))
    assert a == b > 0
    assert binding.workspace_bytes(_desc(Hq=30)) == 0        # Hq % Hkv != 0
    assert binding.workspace_bytes(_desc(d=96)) == 0          # unsupported head dim
    assert binding.workspace_bytes(_desc(), 0) == 0 and binding.workspace_bytes(_desc(), 1025) == 0
    assert binding.workspace_bytes(_desc(), 32) > a           # grows with the layer count


def test_compress_layer_rejects_bad_arguments_before_launching():
    I, U, W = binding.ERR_INVALID_ARG, binding.ERR_UNSUPPORTED, binding.ERR_WORKSPACE
    assert _call(_desc(Hq=30)) == I
    assert _call(_desc(k_l=4)) == I                 # budget smaller than the window
    assert _call(_desc(alpha=0, k_l=8)) == I
    assert _call(_desc(pool=7)) == I
    assert _call(_desc(pool_w=4)) == I
    assert _call(_desc(flags=8)) == I               # a bit outside PKV_FLAG_ALL
    assert _call(_desc(kv_st=130)) == I             # rows not 16-byte aligned
    assert _call(_desc(kv_st=64)) == I              # rows overlap
    assert _call(_desc(d=96, q_st=96, kv_st=96, o_st=96)) == U
    assert _call(_desc(alpha=72, k_l=128)) == U
    assert _call(_desc(pool_w=65)) == U
    good = _desc()
    assert _call(good, Q=None) == I
    assert _call(good, idx=None) == I
    assert _call(good, K=0x2004) == I               # misaligned pointer
    assert _call(good, ws=None) == W
    assert _call(good, ws=0x10010) == W             # not 256-byte aligned
    assert _call(good, ws_bytes=binding.workspace_bytes(good) - 1) == W


def test_compress_layers_rejects_mismatched_layers():
    lib = binding.load()
    descs = (binding.LayerDesc * 2)(_desc(), _desc(N=2048, kv_sh=2048 * 128, kv_sb=8 * 2048 * 128))
    arr = (ctypes.c_void_p * 2)(0x1000, 0x2000)
    rc = lib.pkv_compress_layers(2, descs, arr, arr, arr, None, arr, arr, arr, arr, None, 0x10000, 1 << 30, None)
    assert rc == binding.ERR_INVALID_ARG
    rc = lib.pkv_compress_layers(0, descs, arr, arr, arr, None, arr, arr, arr, arr, None, 0x10000, 1 << 30, None)
    assert rc == binding.ERR_INVALID_ARG


def test_probe_read_rejects_bad_arguments_before_any_launch():
    lib = binding.load()
    lib.pkv_probe_read.argtypes = [ctypes.c_void_p, ctypes.c_size_t, ctypes.c_void_p, ctypes.c_void_p]
    lib.pkv_probe_read.restype = ctypes.c_int
    assert lib.pkv_probe_read(None, 1024, 0x1000, None) == binding.ERR_INVALID_ARG      # no buffer
    assert lib.pkv_probe_read(0x1000, 1024, None, None) == binding.ERR_INVALID_ARG      # no sink
    assert lib.pkv_probe_read(0x1000, 0, 0x2000, None) == binding.ERR_INVALID_ARG       # empty
    assert lib.pkv_probe_read(0x1000, 1000, 0x2000, None) == binding.ERR_INVALID_ARG    # not a multiple of 16
    assert lib.pkv_probe_read(0x1008, 1024, 0x2000, None) == binding.ERR_INVALID_ARG    # misaligned buffer


def test_compress_layers_lse_rejects_missing_or_misaligned_denominators():
    lib = binding.load()
    descs = (binding.LayerDesc * 2)(_desc(), _desc())
    arr = (ctypes.c_void_p * 2)(0x1000, 0x2000)
    I = binding.ERR_INVALID_ARG

    def call(lse, ws_bytes=1 << 30):
        return lib.pkv_compress_layers_lse(2, descs, arr, arr, arr, lse, None, arr, arr, arr, arr, None,
                                           0x10000, ws_bytes, None)

    assert call(None) == I                                         # no table of denominators
    assert call((ctypes.c_void_p * 2)(0x1000, None)) == I          # a layer without them
    assert call((ctypes.c_void_p * 2)(0x1000, 0x2002)) == I        # not 4-byte aligned
    assert call(arr, ws_bytes=16) == binding.ERR_WORKSPACE         # valid so far: fails at the workspace check


def test_compress_layers_paged_rejects_inconsistent_paging():
    lib = binding.load()
    descs = (binding.LayerDesc * 2)(_desc(k_l=128), _desc(k_l=64))
    arr = (ctypes.c_void_p * 2)(0x1000, 0x2000)
    I = binding.ERR_INVALID_ARG

    def call(pd, tables=arr, ws_bytes=16):
        pdp = None if pd is None else ctypes.byref(pd)
        return lib.pkv_compress_layers_paged(2, descs, arr, arr, arr, None, None, pdp, arr, arr, tables, arr, arr,
                                             None, 0x10000, ws_bytes, None)

    assert call(None) == I                                              # no paging descriptor
    assert call(binding.PagedDesc(0, 8, 8, 0)) == I                     # page size
    assert call(binding.PagedDesc(16, 0, 8, 0)) == I                    # empty pool
    assert call(binding.PagedDesc(16, 8, 8, 1)) == I                    # reserved
    assert call(binding.PagedDesc(16, 64, 7, 0)) == I                   # 128 kept rows need 8 table entries
    assert call(binding.PagedDesc(16, 64, 8, 0), tables=None) == I      # no tables
    assert call(binding.PagedDesc(16, 64, 8, 0), tables=(ctypes.c_void_p * 2)(0x1000, 0x2002)) == I
    assert call(binding.PagedDesc(16, 64, 8, 0)) == binding.ERR_WORKSPACE   # valid so far


def _geometric_fractions(L, avg, beta, alpha):
    """Fractional parts of the real-valued geometric budgets, in 60-digit decimal arithmetic (test only)."""
    from decimal import Decimal, getcontext
    getcontext().prec = 60
    q = (-(Decimal(2 * beta - 1).ln()) / (L - 1)).exp()
    w = [q ** l for l in range(L)]
    tot = sum(w)
    r = [Decimal(L * (avg - alpha)) * x / tot for x in w]
    return [x - int(x) for x in r]


def test_budget_schedules_equal_oracle_on_a_grid():
    # The library evaluates the geometric schedule its own way (closed-form first term, running product), the oracle
    # with a power per layer; the integer budgets must agree, except that units may sit on other layers among layers
    # whose fractional parts lie within 1e-9 of each other (the largest-remainder rule cannot tell them apart in
    # double; e.g. L = 4, beta = 14 has q = 1/3 exactly and every fractional part equal to 1/2).
    swaps = 0
    for sched in (pkv_oracle.SCHEDULE_LINEAR, pkv_oracle.SCHEDULE_GEOMETRIC, pkv_oracle.SCHEDULE_UNIFORM):
        for L in (1, 2, 3, 4, 7, 28, 32, 40, 80, 126):
            for avg in (64, 96, 128, 256, 512, 2048, 777):
                for beta in (1, 2, 5, 14, 20):
                    for alpha in (0, 8, 32):
                        if avg < alpha:
                            continue
                        want = pkv_oracle.budgets_schedule(L, avg, beta, alpha, sched).tolist()
                        got = binding.budgets_schedule(L, avg, beta, alpha, sched)
                        if got == want:
                            continue
                        assert sched == pkv_oracle.SCHEDULE_GEOMETRIC, (sched, L, avg, beta, alpha)
                        diff = [(l, g - w) for l, (g, w) in enumerate(zip(got, want)) if g != w]
                        assert all(abs(d) == 1 for _, d in diff) and sum(d for _, d in diff) == 0, (L, avg, beta, alpha, diff)
                        fr = [_geometric_fractions(L, avg, beta, alpha)[l] for l, _ in diff]
                        assert max(fr) - min(fr) < 1e-9, (L, avg, beta, alpha, diff)
                        swaps += 1
    assert swaps <= 5
    with pytest.raises(binding.PkvError):
        binding.budgets_schedule(4, 128, 20, 8, 9)


def test_noalloc_entry_point_checks_its_arguments_and_the_scratch_limit():
    lib = binding.load()

    def call(desc, Q=0x1000):
        return lib.pkv_compress_layer_noalloc(ctypes.byref(desc), Q, 0x2000, 0x3000, None, 0x4000, 0x5000, 0x6000,
                                              0x7000, None, None)

    assert call(_desc(Hq=30)) == binding.ERR_INVALID_ARG
    assert call(_desc(d=96, q_st=96, kv_st=96, o_st=96)) == binding.ERR_UNSUPPORTED
    # 64 heads of 65536 keys need more scratch than the built-in buffer holds: refused before anything else happens
    big = _desc(B=8, N=65536, kv_sh=65536 * 128, kv_sb=8 * 65536 * 128)
    assert binding.workspace_bytes(big) > binding.NOALLOC_SCRATCH_BYTES
    assert call(big) == binding.ERR_SCRATCH
    assert binding.workspace_bytes(_desc()) <= binding.NOALLOC_SCRATCH_BYTES
    text = open(os.path.join(ROOT, "include", "pkv.h")).read()
    assert re.search(r"#define PKV_NOALLOC_SCRATCH_BYTES \(\(size_t\)32 << 20\)", text)


def test_attention_recall_rejects_bad_arguments():
    lib = binding.load()
    descs = (binding.LayerDesc * 2)(_desc(), _desc())
    arr = (ctypes.c_void_p * 2)(0x1000, 0x2000)
    I = binding.ERR_INVALID_ARG
    assert lib.pkv_attention_recall(2, descs, 0, None, None, arr, 0x10000, 1 << 30, None) == I
    assert lib.pkv_attention_recall(2, descs, 0, None, arr, (ctypes.c_void_p * 2)(0x1000, None), 0x10000, 1 << 30, None) == I
    assert lib.pkv_attention_recall(0, descs, 0, None, arr, arr, 0x10000, 1 << 30, None) == I
    assert lib.pkv_attention_recall(2, descs, 0, None, arr, arr, 0x10000, 16, None) == binding.ERR_WORKSPACE


def test_decode_attention_rejects_bad_arguments():
    lib = binding.load()
    I, U = binding.ERR_INVALID_ARG, binding.ERR_UNSUPPORTED

    def desc(**kw):
        base = dict(B=2, Hq=32, Hkv=8, d=128, k_cap=128, page_size=0, num_pages=0, max_pages=0, reserved=0, reserved2=0,
                    c_sb=8 * 128 * 128, c_sh=128 * 128, c_st=128)
        base.update(kw)
        return binding.DecodeDesc(**base)

    def call(d, q=0x1000, K=0x2000, V=0x3000, tb=None, cnt=0x4000, out=0x5000):
        return lib.pkv_decode_attention(ctypes.byref(d), q, K, V, tb, cnt, out, None, 0x10000, 1 << 30, None)

    assert call(desc(), q=None) == I and call(desc(), cnt=None) == I and call(desc(), out=None) == I
    assert call(desc(), K=0x2004) == I                                 # misaligned cache
    assert call(desc(Hq=30)) == I and call(desc(k_cap=0)) == I and call(desc(reserved=3)) == I
    assert call(desc(c_st=64)) == I and call(desc(c_sh=12)) == I        # rows overlap / not 16-byte aligned
    assert call(desc(page_size=16, num_pages=64, max_pages=8)) == I    # paged without a table
    assert call(desc(page_size=16, num_pages=64, max_pages=7), tb=0x6000) == I   # table too short for k_cap
    assert call(desc(d=96)) == U and call(desc(Hq=128)) == U and call(desc(k_cap=5000)) == U
    big = desc(k_cap=2048)                                              # small batch, long cache: split over key ranges
    need = lib.pkv_decode_workspace_bytes(ctypes.byref(big))
    assert need == 2 * 8 * 16 * (8 * 128 + 16) * 4                      # 16 key ranges
    assert lib.pkv_decode_workspace_bytes(ctypes.byref(desc(B=64))) == 0
    assert lib.pkv_decode_attention(ctypes.byref(big), 0x1000, 0x2000, 0x3000, None, 0x4000, 0x5000, None, 0x10000,
                                    need - 1, None) == binding.ERR_WORKSPACE


def test_decode_attention_layers_rejects_bad_arguments():
    lib = binding.load()
    I, U = binding.ERR_INVALID_ARG, binding.ERR_UNSUPPORTED

    def desc(**kw):
        base = dict(B=1, Hq=32, Hkv=8, d=128, k_cap=256, page_size=0, num_pages=0, max_pages=0, reserved=0, reserved2=0,
                    c_sb=8 * 256 * 128, c_sh=256 * 128, c_st=128)
        base.update(kw)
        return binding.DecodeDesc(**base)

    arr = lambda *v: (ctypes.c_void_p * len(v))(*v)
    good = arr(0x1000, 0x2000)

    def call(descs, q=good, K=good, V=good, tb=None, cnt=good, out=good, lse=None, ws=0x10000, ws_bytes=1 << 30):
        return lib.pkv_decode_attention_layers(len(descs), descs, q, K, V, tb, cnt, out, lse, ws, ws_bytes, None)

    two = (binding.DecodeDesc * 2)(desc(), desc(k_cap=4096, c_sb=8 * 4096 * 128, c_sh=4096 * 128))
    assert call(two, q=None) == I and call(two, out=None) == I and call(two, cnt=None) == I
    assert call(two, K=arr(0x1000, None)) == I and call(two, V=arr(0x1000, 0x2004)) == I
    assert lib.pkv_decode_attention_layers(0, two, good, good, good, None, good, good, None, 0x10000, 1 << 30, None) == I
    assert call((binding.DecodeDesc * 2)(desc(), desc(Hq=16))) == I            # the layers differ in their heads
    assert call((binding.DecodeDesc * 2)(desc(), desc(B=2))) == I
    assert call((binding.DecodeDesc * 2)(desc(), desc(d=96))) == U
    assert call((binding.DecodeDesc * 2)(desc(), desc(k_cap=5000))) == U
    paged = (binding.DecodeDesc * 2)(desc(page_size=16, num_pages=64, max_pages=16),
                                     desc(page_size=16, num_pages=64, max_pages=16))
    assert call(paged) == I and call(paged, tb=arr(0x6000, None)) == I          # paged without (all) tables
    # 8 heads x (256 + 4096) rows = 34 816 rows: 256-key ranges (the smallest), so 1 and 16 ranges per head; only
    # the layer with more than one range needs partial results
    need = lib.pkv_decode_layers_workspace_bytes(2, two)
    assert need == 8 * 16 * (8 * 128 + 16) * 4
    assert call(two, ws_bytes=need - 1) == binding.ERR_WORKSPACE and call(two, ws=None) == binding.ERR_WORKSPACE
    one = (binding.DecodeDesc * 1)(desc(k_cap=100, c_sb=8 * 100 * 128, c_sh=100 * 128))
    assert lib.pkv_decode_layers_workspace_bytes(1, one) == 0                   # a single range per head: no partials
    assert lib.pkv_decode_layers_workspace_bytes(2, (binding.DecodeDesc * 2)(desc(), desc(Hq=16))) == 0

"""CPU-only checks of the GPU library's host side: it loads, exports every symbol the header declares,
validates arguments before touching a device, and its decode constants do what the kernels rely on."""
import ctypes as C
import os
import re
from fractions import Fraction

import numpy as np
import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "iflow.h")


@pytest.fixture(scope="module")
def iflow():
    from paper_2401_08294_amd import build, iflow as mod
    if not os.path.exists(mod.LIB_PATH):
        build.build_lib()
    mod.lib()
    return mod


def declared_symbols():
    text = open(HEADER).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(iflow_[a-z0-9_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol(iflow):
    names = declared_symbols()
    assert {"iflow_quantize", "iflow_dequant", "iflow_qgemv", "iflow_qgemm", "iflow_packed_bytes",
            "iflow_unpack_logical"} <= set(names)
    L = iflow.lib()
    for n in names:
        assert hasattr(L, n), f"{n} is declared in iflow.h but not exported"
    assert iflow.layout_version() == 1


def test_binding_constants_are_the_headers(iflow):
    """The numbers the binding repeats from include/iflow.h (limits of the chained launch, where a launch leaves its clock stamps)."""
    import re
    defs = dict(re.findall(r"^#define (IFLOW_[A-Z_]+) (\d+)\s*$", open(HEADER).read(), flags=re.M))
    assert int(defs["IFLOW_CHAIN_MAX_PHASES"]) == iflow.CHAIN_MAX_PHASES
    assert int(defs["IFLOW_CHAIN_MAX_GROUP"]) == iflow.CHAIN_MAX_GROUP
    assert int(defs["IFLOW_CHAIN_MAX_MATRICES"]) == iflow.CHAIN_MAX_MATRICES
    assert int(defs["IFLOW_CHAIN_WS_CLOCKS"]) == iflow.CHAIN_WS_CLOCKS
    assert 4 * (iflow.CHAIN_WS_CLOCKS + 4) <= int(defs["IFLOW_CHAIN_WS_HEADER"])      # the stamps lie inside the workspace header


def test_format_queries_and_bit_budget(iflow):
    # Table 3: block sizes, levels (2^k, or 11 for Eq.3) and actual bits per weight
    expect = {"Q8_B32": (32, 256, 9), "Q8_B64": (64, 256, 8.5), "Q4_B32": (32, 16, 5), "Q4_B64": (64, 16, 4.5),
              "Q3H_B64": (64, 11, 4), "Q6_B64": (64, 64, 6.5), "Q5_B64": (64, 32, 5.5), "Q3_B32": (32, 8, 4),
              "Q2_B32": (32, 4, 3)}          # (the 2-bit format is not in Table 3: 2 bits + 32 header bits per 32 weights)
    for name, (bs, lv, bpw) in expect.items():
        f = iflow.FORMATS[name]
        assert iflow.format_block(f) == bs and iflow.format_levels(f) == lv
        for r, c in ((1, 64), (4096, 4096), (4096, 11008), (28672, 8192)):
            assert Fraction(iflow.packed_bytes(f, r, c) * 8, r * c) == Fraction(bpw)
    assert iflow.format_block(17) == -1 and iflow.format_levels(-1) == -1


def test_argument_validation_happens_before_any_launch(iflow):
    L = iflow.lib()
    sz = C.c_size_t(0)
    assert L.iflow_packed_bytes(4, 8, 100, C.byref(sz)) == iflow.ERR_SHAPE      # cols % 64 != 0
    assert L.iflow_packed_bytes(4, 0, 64, C.byref(sz)) == iflow.ERR_SHAPE
    assert L.iflow_packed_bytes(4, 8, 1 << 31, C.byref(sz)) == iflow.ERR_SHAPE
    assert L.iflow_packed_bytes(9, 8, 64, C.byref(sz)) == iflow.ERR_FORMAT
    assert L.iflow_packed_bytes(4, 8, 64, None) == iflow.ERR_NULL
    good = 0x10000                                                               # aligned, never dereferenced
    assert L.iflow_quantize(4, None, 8, 64, good, 256, None) == iflow.ERR_NULL
    assert L.iflow_quantize(4, good, 8, 64, good, 255, None) == iflow.ERR_SIZE
    assert L.iflow_quantize(4, good + 8, 8, 64, good, 256, None) == iflow.ERR_ALIGN
    assert L.iflow_quantize(4, good, 8, 32, good, 256, None) == iflow.ERR_SHAPE
    assert L.iflow_dequant(4, good, 8, 64, None, None) == iflow.ERR_NULL
    assert L.iflow_dequant(9, good, 8, 64, good, None) == iflow.ERR_FORMAT
    assert L.iflow_qgemv(4, good, 8, 64, good, good + 2, None) == iflow.ERR_ALIGN
    assert L.iflow_qgemm(4, good, 8, 64, good, 0, good, None) == iflow.ERR_SHAPE
    assert L.iflow_qgemm(4, good, 8, 64, None, 3, good, None) == iflow.ERR_NULL
    assert L.iflow_unpack_logical(4, good, 8, 64, good, good, None, None) == iflow.ERR_NULL
    for st in range(8):
        assert isinstance(iflow.status_string(st), str) and iflow.status_string(st)
    with pytest.raises(iflow.IflowError):
        iflow.packed_bytes(4, 3, 65)


def test_chain_validation_happens_before_any_launch(iflow):
    """iflow_qgemv_chain_plan: limits, aliasing rules and buffer sizes are checked on the host (no device call on any of
    these errors: this test runs without a GPU)."""
    L = iflow.lib()
    base = 0x100000                                                              # aligned, never dereferenced

    def call(fmt, counts, cols, x, packed, rows, y, ws=base * 64, ws_bytes=1 << 30, plan=base * 128, plan_bytes=1 << 30):
        nph, n = len(counts), len(rows)
        chain = iflow.Chain()
        return L.iflow_qgemv_chain_plan(fmt, nph, (C.c_int * max(nph, 1))(*counts), (C.c_int64 * max(nph, 1))(*cols),
                                        (C.c_void_p * max(nph, 1))(*x), (C.c_void_p * max(n, 1))(*packed),
                                        (C.c_int64 * max(n, 1))(*rows), (C.c_void_p * max(n, 1))(*y), plan, plan_bytes, ws, ws_bytes,
                                        None, C.byref(chain))

    x0, pk, y0, y1 = base, base * 2, base * 3, base * 4
    assert call(9, [1], [64], [x0], [pk], [8], [y0]) == iflow.ERR_FORMAT          # no such format
    assert call(7, [1], [65536 + 32], [x0], [pk], [8], [y0]) == iflow.ERR_SHAPE  # a bit-plane format: rows of at most 65536 columns
    assert call(5, [1], [96], [x0], [pk], [8], [y0]) == iflow.ERR_SHAPE          # cols % block (64)
    assert call(1, [1], [61440 + 64], [x0], [pk], [8], [y0]) == iflow.ERR_SHAPE  # 8-bit: a row's staged activations must fit LDS
    assert call(3, [1], [65536 + 64], [x0], [pk], [8], [y0]) == iflow.ERR_SHAPE
    assert call(3, [1], [96], [x0], [pk], [8], [y0]) == iflow.ERR_SHAPE          # cols % block (64)
    assert call(4, [], [], [], [], [], []) == iflow.ERR_SHAPE                    # no phase
    assert call(4, [1] * 1025, [64] * 1025, [x0] * 1025, [pk] * 1025, [8] * 1025, [y0 + 64 * i for i in range(1025)]) == iflow.ERR_SHAPE
    assert call(4, [5], [64], [x0], [pk] * 5, [8] * 5, [y0 + 64 * i for i in range(5)]) == iflow.ERR_SHAPE   # > 4 per phase
    assert call(4, [1], [100], [x0], [pk], [8], [y0]) == iflow.ERR_SHAPE         # cols % 64
    assert call(4, [1], [131072], [x0], [pk], [8], [y0]) == iflow.ERR_SHAPE      # cols > 65536
    assert call(4, [1], [64], [None], [pk], [8], [y0]) == iflow.ERR_NULL
    assert call(4, [1], [64], [x0 + 2], [pk], [8], [y0]) == iflow.ERR_ALIGN
    assert call(4, [1], [64], [y0], [pk], [8], [y0]) == iflow.ERR_SHAPE          # in place: x is this phase's own output
    # x of phase 1 = y of phase 0 is fine only if it is the whole vector (rows == cols) ...
    assert call(4, [1, 1], [64, 128], [x0, y0], [pk, pk], [64, 8], [y0, y1]) == iflow.ERR_SHAPE    # 64 rows feeding 128 columns
    assert call(4, [1, 1], [64, 64], [x0, y0 + 32], [pk, pk], [128, 8], [y0, y1]) == iflow.ERR_SHAPE   # the middle of an output
    # ... a launch input must not be overlapped by ANY output of the call, also not by a later phase's ...
    assert call(4, [1, 1, 1], [64, 64, 64], [x0, y1 + 4096, y0], [pk, pk, pk], [64, 64, 64], [y0, y0 + 4096, y1 + 4096]) == iflow.ERR_SHAPE
    # ... two outputs must not overlap ...
    assert call(4, [2], [64], [x0], [pk, pk], [64, 64], [y0, y0 + 64]) == iflow.ERR_SHAPE
    # ... and the workspace has to hold the hand-over words
    sz = C.c_size_t(0)
    assert L.iflow_qgemv_chain_workspace_bytes(2, (C.c_int64 * 2)(64, 8), C.byref(sz)) == iflow.OK
    assert sz.value == 4096 + 2 * 4096 * 4
    assert call(4, [1, 1], [64, 64], [x0, y0], [pk, pk], [64, 8], [y0, y1], ws_bytes=sz.value - 1) == iflow.ERR_SIZE
    assert call(4, [1, 1], [64, 64], [x0, y0], [pk, pk], [64, 8], [y0, y1], ws=None) == iflow.ERR_NULL
    assert L.iflow_qgemv_chain_plan_bytes(2, 2, C.byref(sz)) == iflow.OK and sz.value == 64 + 2 * (64 + 32) + 2 * 64
    assert call(4, [1, 1], [64, 64], [x0, y0], [pk, pk], [64, 8], [y0, y1], plan_bytes=sz.value - 1) == iflow.ERR_SIZE
    assert L.iflow_qgemv_chain_plan_bytes(0, 0, C.byref(sz)) == iflow.ERR_SHAPE
    assert L.iflow_qgemv_chain_plan_bytes(2, 5000, C.byref(sz)) == iflow.ERR_SHAPE
    assert call(4, [1, 1], [64, 64], [x0, y0], [pk, pk], [64, 8], [y0, y1], plan=base * 128 + 4) == iflow.ERR_ALIGN
    assert L.iflow_qgemv_chain_workspace_bytes(4097, (C.c_int64 * 4097)(*[8] * 4097), C.byref(sz)) == iflow.ERR_SHAPE
    assert L.iflow_qgemv_chain_check(None, None) == iflow.ERR_NULL
    assert L.iflow_qgemv_chain_launch(None, None) == iflow.ERR_NULL
    blank = iflow.Chain()
    blank.plan, blank.workspace = base, base * 2                                 # never filled by a plan call: refused by its magic word
    assert L.iflow_qgemv_chain_launch(C.byref(blank), None) == iflow.ERR_SHAPE


def test_fused_chain_validation_happens_before_any_launch(iflow):
    """iflow_qgemv_chain_plan_fused: the rules for gains, gated pairs and residuals, checked on the host."""
    L = iflow.lib()
    base = 0x100000

    def call(counts, cols, x, packed, rows, y, x_op=None, aux=None, eps=None, gated=None, residual=None):
        nph, n = len(counts), len(rows)
        chain = iflow.Chain()
        arr = lambda t, v, k: (t * k)(*v) if v is not None else None
        return L.iflow_qgemv_chain_plan_fused(4, nph, (C.c_int * nph)(*counts), (C.c_int64 * nph)(*cols), (C.c_void_p * nph)(*x),
                                              arr(C.c_int, x_op, nph), arr(C.c_void_p, aux, nph), arr(C.c_float, eps, nph),
                                              arr(C.c_int, gated, nph), (C.c_void_p * n)(*packed), (C.c_int64 * n)(*rows),
                                              arr(C.c_void_p, residual, n), (C.c_void_p * n)(*y), None, 1 << 20, base * 64, 1 << 30,
                                              None, C.byref(chain))

    x0, g0, pk, y0, y1, r0 = base, base + 0x1000, base * 2, base * 3, base * 4, base * 5
    ok_then_null = iflow.ERR_NULL                      # every check passed; the null plan pointer is what is reported
    assert call([1], [64], [x0], [pk], [8], [y0], x_op=[1], aux=[g0], eps=[1e-5]) == ok_then_null
    assert call([1], [64], [x0], [pk], [8], [y0], x_op=[1], aux=[None], eps=[1e-5]) == iflow.ERR_NULL
    assert call([1], [64], [x0], [pk], [8], [y0], x_op=[1], aux=[g0 + 2], eps=[1e-5]) == iflow.ERR_ALIGN
    assert call([1], [64], [x0], [pk], [8], [y0], x_op=[1], aux=[g0], eps=[-1.0]) == iflow.ERR_SHAPE
    assert call([1], [64], [x0], [pk], [8], [y0], x_op=[1], aux=[y0], eps=[0.0]) == iflow.ERR_SHAPE      # gains overlapped by an output
    assert call([1], [64], [x0], [pk], [8], [y0], x_op=[2], aux=[g0], eps=[0.0]) == iflow.ERR_SHAPE      # silu*mul is a gated phase's job
    # a gated phase: two matrices of equal size, one output
    assert call([2], [64], [x0], [pk, pk], [8, 8], [y0, None], gated=[1]) == ok_then_null
    assert call([2], [64], [x0], [pk, pk], [8, 8], [y0, y1], gated=[1]) == iflow.ERR_SHAPE
    assert call([2], [64], [x0], [pk, pk], [8, 16], [y0, None], gated=[1]) == iflow.ERR_SHAPE
    assert call([1], [64], [x0], [pk], [8], [y0], gated=[1]) == iflow.ERR_SHAPE
    assert call([2], [64], [x0], [pk, pk], [8, 8], [y0, None], gated=[0]) == iflow.ERR_NULL               # not gated: every matrix has an output
    assert call([2], [64], [x0], [pk, pk], [8, 8], [y0, None], gated=[1], residual=[r0, None]) == iflow.ERR_SHAPE
    # residuals: a launch input, or exactly an earlier phase's output
    assert call([1], [64], [x0], [pk], [8], [y0], residual=[r0]) == ok_then_null
    assert call([1], [64], [x0], [pk], [8], [y0], residual=[r0 + 2]) == iflow.ERR_ALIGN
    assert call([1], [64], [x0], [pk], [8], [y0], residual=[y0]) == iflow.ERR_SHAPE                       # its own output
    assert call([1, 1], [64, 64], [x0, x0], [pk, pk], [8, 8], [y0, y1], residual=[None, y0]) == ok_then_null
    assert call([1, 1], [64, 64], [x0, x0], [pk, pk], [16, 8], [y0, y1], residual=[None, y0]) == iflow.ERR_SHAPE   # another length
    assert call([1, 1], [64, 64], [x0, x0], [pk, pk], [8, 8], [y0, y1], residual=[y1, None]) == iflow.ERR_SHAPE    # a later phase's output


def test_binding_fails_loudly_without_the_library(monkeypatch):
    from paper_2401_08294_amd import iflow as mod
    monkeypatch.setattr(mod, "_lib", None)
    monkeypatch.setattr(mod, "LIB_PATH", os.path.join(ROOT, "no_such_dir", "libiflow.so"))
    with pytest.raises(RuntimeError):
        mod.lib()


def test_product_path_does_not_import_the_oracle():
    pkg = os.path.join(ROOT, "paper_2401_08294_amd")
    bad = re.compile(r"(^\s*(from|import)\s+oracle\b)|liboracle|iflow_oracle|orc_[a-z0-9_]+\s*\(", re.M)
    for dirpath, _, files in os.walk(pkg):
        for f in files:
            if f.endswith((".py", ".hip", ".h", ".cpp")):
                text = open(os.path.join(dirpath, f)).read()
                assert not bad.search(text), f"{f} reaches into the oracle"


# ---- the fp16 / u16 identities the Q3H decode relies on, checked for every code with exact arithmetic ----
def _fp16_round(v: Fraction) -> int:
    f = float(v)
    assert Fraction(f) == v
    return int(np.float64(f).astype(np.float16).view(np.uint16))


def test_q3h_packed_decode_identities():
    K1 = Fraction(1489, 1 << 14)          # fp16 nearest to 1/11
    K2 = Fraction(1863, 2)                # 931.5
    assert _fp16_round(K1) == 0x2DD1 and _fp16_round(K2) == 0x6347
    for c in range(121):
        hc = 0x6400 | c                                               # fp16 1024 + c
        h1 = _fp16_round((1024 + c) * K1 + K2)                        # one fused multiply-add
        assert h1 == 0x6401 + c // 11                                 # fp16 1025 + floor(c/11)
        h2 = (h1 * 0xFFF5 + hc) & 0xFFFF                              # packed u16 multiply-add by -11
        assert h2 == 0x17F5 + c % 11
        val = np.array([h2], np.uint16).view(np.float16)[0]
        assert Fraction(float(val)) == Fraction(2037 + c % 11, 1 << 20)


def test_q4_q8_magic_number_identities():
    for v in range(16):
        lo = np.array([0x6400 | v], np.uint16).view(np.float16)[0]
        hi = np.array([0x5400 | (v << 4)], np.uint16).view(np.float16)[0]
        assert float(lo) == 1024 + v and float(hi) == 64 + v
    for v in range(256):
        b = np.array([0x6400 | v], np.uint16).view(np.float16)[0]
        assert float(b) == 1024 + v


def test_fused_validation_happens_before_any_launch(iflow):
    """iflow_qgemv_fused: format, operand and overlap rules are checked on the host (no launch on any error)."""
    L = iflow.lib()
    base = 0x100000                                                              # aligned, never dereferenced

    def call(fmt, rows, cols, x, y, x_op=0, aux=None, eps=0.0, residual=None, packed=None):
        n = len(rows)
        res = None if residual is None else (C.c_void_p * n)(*residual)
        return L.iflow_qgemv_fused(fmt, n, (C.c_void_p * n)(*(packed or [base * 2] * n)), (C.c_int64 * n)(*rows), cols, x, x_op, aux,
                                   C.c_float(eps), res, (C.c_void_p * n)(*y), None)

    x, y0, y1, aux = base, base * 3, base * 4, base * 5
    assert call(9, [8], 64, x, [y0]) == iflow.ERR_FORMAT                         # no such format
    assert call(3, [8], 65536, x, [y0]) == iflow.ERR_SHAPE                       # 4-bit rows too long to stage in LDS
    assert call(4, [8], 64, x, [y0], x_op=7, aux=aux) == iflow.ERR_SHAPE         # unknown operation
    assert call(4, [8], 64, x, [y0], x_op=iflow.X_RMS_GAIN) == iflow.ERR_NULL    # gains missing
    assert call(4, [8], 64, x, [y0], x_op=iflow.X_PLAIN, aux=aux) == iflow.ERR_NULL   # a second operand nobody asked for
    assert call(4, [8], 64, x, [y0], x_op=iflow.X_RMS_GAIN, aux=aux, eps=-1.0) == iflow.ERR_SHAPE
    assert call(4, [8], 64, x, [y0], x_op=iflow.X_RMS_GAIN, aux=aux, eps=float("nan")) == iflow.ERR_SHAPE
    assert call(4, [8], 64, x, [y0], x_op=iflow.X_SILU_MUL, aux=aux + 2) == iflow.ERR_ALIGN
    assert call(4, [8], 100, x, [y0]) == iflow.ERR_SHAPE                         # columns not a multiple of the block
    assert call(4, [8] * 9, 64, x, [y0] * 9) == iflow.ERR_SHAPE                  # more than eight matrices
    assert call(4, [8], 64, x, [x + 16]) == iflow.ERR_SHAPE                      # output inside the activations
    assert call(4, [8], 64, x, [y0], x_op=iflow.X_SILU_MUL, aux=y0) == iflow.ERR_SHAPE    # output is the second operand
    assert call(4, [8], 64, x, [y0], residual=[y0 + 2]) == iflow.ERR_SHAPE       # residual shifted against its own output
    assert call(4, [8, 8], 64, x, [y0, y1], residual=[y1, None]) == iflow.ERR_SHAPE       # residual is another matrix's output
    assert call(4, [8], 64, x, [y0], residual=[y0 + 1]) == iflow.ERR_ALIGN


def test_gated_validation_happens_before_any_launch(iflow):
    L = iflow.lib()
    base = 0x100000

    def call(fmt=4, rows=8, cols=64, gate=base, up=base * 2, x=base * 3, y=base * 4, x_op=0, aux=None, eps=0.0):
        return L.iflow_qgemv_gated(fmt, gate, up, rows, cols, x, x_op, aux, C.c_float(eps), y, None)

    assert call(fmt=9) == iflow.ERR_FORMAT
    assert call(x_op=iflow.X_SILU_MUL, aux=base * 5) == iflow.ERR_SHAPE          # the gate is this call's own
    assert call(up=None) == iflow.ERR_NULL and call(y=None) == iflow.ERR_NULL
    assert call(x_op=iflow.X_RMS_GAIN) == iflow.ERR_NULL and call(aux=base * 5) == iflow.ERR_NULL
    assert call(x_op=iflow.X_RMS_GAIN, aux=base * 5, eps=-1.0) == iflow.ERR_SHAPE
    assert call(cols=100) == iflow.ERR_SHAPE and call(rows=0) == iflow.ERR_SHAPE
    assert call(up=base * 2 + 8) == iflow.ERR_ALIGN
    assert call(y=base * 3 + 64) == iflow.ERR_SHAPE                              # output inside the activations
    assert call(fmt=3, cols=65536) == iflow.ERR_SHAPE                            # 4-bit rows too long to stage in LDS


def test_attention_validation_happens_before_any_launch(iflow):
    L = iflow.lib()
    base = 0x100000

    def call(n_heads=32, n_kv=32, d=128, T=10, max_seq=64, scale=0.1, q=base, k=base * 2, v=base * 3, out=base * 4, ws=base * 5, ws_bytes=1 << 30):
        return L.iflow_attn_decode(q, k, v, n_heads, n_kv, d, T, max_seq, C.c_float(scale), out, ws, ws_bytes, None)

    assert call(d=96) == iflow.ERR_SHAPE and call(d=256) == iflow.ERR_SHAPE      # head dimensions 64 and 128
    assert call(n_heads=30, n_kv=4) == iflow.ERR_SHAPE                           # heads not a multiple of kv heads
    assert call(n_heads=1024, n_kv=8) == iflow.ERR_SHAPE                         # more than 512 heads
    assert call(n_heads=128, n_kv=128) == iflow.ERR_SHAPE                        # more than 64 kv heads
    assert call(T=0) == iflow.ERR_SHAPE and call(T=65) == iflow.ERR_SHAPE        # empty, or longer than the cache
    assert call(scale=0.0) == iflow.ERR_SHAPE and call(scale=float("nan")) == iflow.ERR_SHAPE
    assert call(q=None) == iflow.ERR_NULL and call(ws=None) == iflow.ERR_NULL
    assert call(k=base * 2 + 8) == iflow.ERR_ALIGN
    assert call(ws_bytes=1000) == iflow.ERR_SIZE
    assert iflow.attn_decode_workspace_bytes(32) == 32 * 64 * 130 * 4


def test_unpack_pair_codes_is_for_the_pair_format_only(iflow):
    L = iflow.lib()
    base = 0x100000
    assert L.iflow_unpack_pair_codes(3, base, 8, 64, base * 2, None) == iflow.ERR_FORMAT
    assert L.iflow_unpack_pair_codes(4, base, 8, 100, base * 2, None) == iflow.ERR_SHAPE
    assert L.iflow_unpack_pair_codes(4, base, 8, 64, None, None) == iflow.ERR_NULL
    assert L.iflow_unpack_pair_codes(4, base + 4, 8, 64, base * 2, None) == iflow.ERR_ALIGN


def test_batch_fused_validation_happens_before_any_launch(iflow):
    """iflow_qgemm_fused: batch size, operands and overlap rules are checked on the host (no launch on any error)."""
    L = iflow.lib()
    base = 0x100000

    def call(fmt=4, rows=128, cols=256, batch=4, x_op=0, aux=None, eps=0.0, res=None, pk=base, X=base * 2, Y=base * 3):
        return L.iflow_qgemm_fused(fmt, pk, rows, cols, X, batch, x_op, aux, C.c_float(eps), res, Y, None)

    assert call(fmt=9) == iflow.ERR_FORMAT
    assert call(batch=0) == iflow.ERR_SHAPE and call(batch=17) == iflow.ERR_SHAPE
    assert call(x_op=3) == iflow.ERR_SHAPE
    assert call(x_op=1) == iflow.ERR_NULL and call(x_op=0, aux=base * 4) == iflow.ERR_NULL      # aux if and only if an operation
    assert call(x_op=1, aux=base * 4, eps=-1.0) == iflow.ERR_SHAPE
    assert call(cols=100) == iflow.ERR_SHAPE and call(fmt=2, cols=96) == iflow.ERR_SHAPE        # 64-column groups, also for block 32
    assert call(X=None) == iflow.ERR_NULL and call(Y=None) == iflow.ERR_NULL
    assert call(X=base * 2 + 2) == iflow.ERR_ALIGN and call(res=base * 5 + 1) == iflow.ERR_ALIGN
    assert call(Y=base * 2 + 256) == iflow.ERR_SHAPE                                            # Y inside X
    assert call(x_op=2, aux=base * 3 - 4 * 256 * 2 + 16) == iflow.ERR_SHAPE                     # the end of aux [batch][cols] reaches into Y
    assert call(res=base * 3 + 64) == iflow.ERR_SHAPE                                           # residual overlaps Y, shifted


def test_rope_validation_happens_before_any_launch(iflow):
    L = iflow.lib()
    base = 0x100000

    def call(n_heads=32, n_kv=8, d=128, pos=5, max_seq=64, theta=10000.0, mode=0, q=base, k=base * 2, v=base * 3, kc=base * 4, vc=base * 5):
        return L.iflow_rope_append(q, k, v, n_heads, n_kv, d, pos, max_seq, C.c_float(theta), mode, kc, vc, None)

    assert call(d=8) == iflow.ERR_SHAPE and call(d=260) == iflow.ERR_SHAPE and call(d=100) == iflow.ERR_SHAPE   # 16..256, a multiple of 8
    assert call(n_heads=0) == iflow.ERR_SHAPE and call(n_kv=0) == iflow.ERR_SHAPE
    assert call(pos=-1) == iflow.ERR_SHAPE and call(pos=64) == iflow.ERR_SHAPE   # the row must exist
    assert call(max_seq=(1 << 20) + 1, pos=0) == iflow.ERR_SHAPE
    assert call(theta=1.0) == iflow.ERR_SHAPE and call(theta=float("nan")) == iflow.ERR_SHAPE
    assert call(mode=2) == iflow.ERR_SHAPE
    assert call(q=None) == iflow.ERR_NULL and call(vc=None) == iflow.ERR_NULL
    assert call(k=base * 2 + 2) == iflow.ERR_ALIGN


def test_decode_stack_validation_happens_before_any_launch(iflow):
    """iflow_decode_stack_*: the description is checked on the host, in the size query, in the plan call and at the launch."""
    L = iflow.lib()
    base = 0x100000
    fmt = iflow.FORMATS["Q3H_B64"]

    def desc(**change):
        args = dict(fmt=fmt, hidden=512, ffn=704, n_heads=4, n_kv_heads=2, max_seq=16, eps=1e-5, rope_base=10000.0, rope_pairing=1)
        layer = {n: base * (i + 8) for i, (n, _) in enumerate(iflow.DecodeLayer._fields_)}
        layer.update(change.pop("layer", {}))
        ptrs = dict(h_in=base, h_out=base * 2, scratch=base * 3)
        ptrs.update({k: change.pop(k) for k in list(change) if k in ptrs})
        args.update(change)
        return iflow.decode_stack(layers=[layer], **args, **ptrs)

    def sizes(**change):
        a, b, c = C.c_size_t(0), C.c_size_t(0), C.c_size_t(0)
        return L.iflow_decode_stack_sizes(C.byref(desc(**change)), C.byref(a), C.byref(b), C.byref(c))

    def plan(plan_ptr=base * 40, ws=base * 50, **change):
        return L.iflow_decode_stack_plan(C.byref(desc(**change)), plan_ptr, 1 << 30, ws, 1 << 30, None, C.byref(iflow.Chain()))

    assert sizes(fmt=99) == iflow.ERR_FORMAT
    assert sizes(head_dim=64) == iflow.ERR_SHAPE                                 # head dimension 128 only
    assert sizes(n_heads=6, n_kv_heads=2, hidden=768) == iflow.ERR_SHAPE         # 1 or an even number of query heads per kv head
    assert sizes(n_heads=4, n_kv_heads=3) == iflow.ERR_SHAPE
    assert sizes(hidden=640) == iflow.ERR_SHAPE                                  # hidden = n_heads * 128
    assert sizes(ffn=100) == iflow.ERR_SHAPE and sizes(ffn=0) == iflow.ERR_SHAPE and sizes(ffn=131072) == iflow.ERR_SHAPE
    assert sizes(max_seq=0) == iflow.ERR_SHAPE and sizes(max_seq=(1 << 20) + 1) == iflow.ERR_SHAPE
    assert sizes(rope_pairing=2) == iflow.ERR_SHAPE and sizes(rope_base=1.0) == iflow.ERR_SHAPE and sizes(eps=-1.0) == iflow.ERR_SHAPE
    assert L.iflow_decode_stack_sizes(None, None, None, None) == iflow.ERR_NULL
    d = desc()
    d.n_layers = 129
    assert L.iflow_decode_stack_sizes(C.byref(d), C.byref(C.c_size_t()), C.byref(C.c_size_t()), C.byref(C.c_size_t())) == iflow.ERR_SHAPE
    assert plan(h_in=None) == iflow.ERR_NULL and plan(scratch=None) == iflow.ERR_NULL and plan(plan_ptr=None) == iflow.ERR_NULL
    assert plan(layer={"wo": None}) == iflow.ERR_NULL and plan(layer={"v_cache": None}) == iflow.ERR_NULL
    assert plan(h_out=base * 2 + 8) == iflow.ERR_ALIGN and plan(layer={"norm2": base * 16 + 2}) == iflow.ERR_ALIGN
    assert plan(h_out=base + 512) == iflow.ERR_SHAPE                             # h_out inside h_in
    assert plan(h_in=base * 3 + 4096) == iflow.ERR_SHAPE                         # h_in inside the scratch buffer
    assert plan(layer={"k_cache": base * 3 + 1024}) == iflow.ERR_SHAPE           # a cache inside the scratch buffer
    assert plan(layer={"v_cache": base * 17 + 4096}) == iflow.ERR_SHAPE          # the two caches overlap (k_cache sits at base * 17)
    assert plan(layer={"norm1": base * 2}) == iflow.ERR_SHAPE                    # the gains are h_out
    chain = iflow.Chain(plan=base, workspace=base * 2, grid=256, max_strips=1, magic=0x69464C57, fused=1, format=fmt, lds_bytes=32768, max_seq=16)
    assert L.iflow_decode_stack_launch(None, 0, None) == iflow.ERR_NULL
    chain.magic = 0
    assert L.iflow_decode_stack_launch(C.byref(chain), 0, None) == iflow.ERR_SHAPE
    chain2 = iflow.Chain(plan=base, workspace=base * 2, grid=256, max_strips=1, magic=0x69464C57, fused=1, format=fmt, lds_bytes=32768, max_seq=16)
    for position in (-1, 16, 1 << 40):
        assert L.iflow_decode_stack_launch(C.byref(chain2), position, None) == iflow.ERR_SHAPE


def test_public_header_is_plain_c_and_cpp(tmp_path):
    """include/iflow.h is the boundary: it has to compile on its own as C99 and as C++11 (no HIP, no torch types)."""
    import shutil
    import subprocess
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    src = tmp_path / "use_header.c"
    src.write_text('#include "iflow.h"\nint main(void) { return (int)IFLOW_Q2_B32 + (int)IFLOW_ROPE_HALVES + (int)IFLOW_X_SILU_MUL; }\n')
    inc = os.path.join(root, "include")
    for cc, flags in (("gcc", ["-std=c99", "-pedantic", "-Wall", "-Wextra", "-Werror"]), ("g++", ["-x", "c++", "-std=c++11", "-pedantic", "-Wall", "-Werror"])):
        if shutil.which(cc) is None:
            pytest.skip(f"{cc} not installed")
        res = subprocess.run([cc] + flags + ["-I", inc, "-fsyntax-only", str(src)], capture_output=True, text=True, timeout=120)
        assert res.returncode == 0, res.stderr


def test_bench_refuses_more_than_one_gpu():
    """bench.py --gpus N with N above 1 exits with a message and runs nothing (one GPU only)."""
    import subprocess
    import sys
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    res = subprocess.run([sys.executable, os.path.join(root, "bench.py"), "--gpus", "2"], capture_output=True, text=True, timeout=120)
    assert res.returncode != 0
    assert "one GPU" in (res.stdout + res.stderr)
    assert not any(line.startswith("{") for line in res.stdout.splitlines())

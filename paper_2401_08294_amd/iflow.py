"""Thin ctypes binding over libiflow.so, with the same names as the C ABI in include/iflow.h.

Argument marshalling only: every step of the path runs in the library's HIP kernels.  PyTorch is used
by callers for device memory and streams; tensors are passed as `tensor.data_ptr()` and the stream as
`torch.cuda.current_stream().cuda_stream`.  There is no CPU fallback: if the library has not been built
(`python -m paper_2401_08294_amd.build` or `__graft_entry__.build()`), loading raises.
"""
from __future__ import annotations

import ctypes as C
import os

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libiflow.so")

Q8_B32, Q8_B64, Q4_B32, Q4_B64, Q3H_B64, Q6_B64, Q5_B64, Q3_B32, Q2_B32 = range(9)
FORMATS = {"Q8_B32": Q8_B32, "Q8_B64": Q8_B64, "Q4_B32": Q4_B32, "Q4_B64": Q4_B64, "Q3H_B64": Q3H_B64,
           "Q6_B64": Q6_B64, "Q5_B64": Q5_B64, "Q3_B32": Q3_B32, "Q2_B32": Q2_B32}
BITS_PER_WEIGHT = {Q8_B32: 9.0, Q8_B64: 8.5, Q4_B32: 5.0, Q4_B64: 4.5, Q3H_B64: 4.0, Q6_B64: 6.5, Q5_B64: 5.5, Q3_B32: 4.0,
                   Q2_B32: 3.0}

OK, ERR_NULL, ERR_FORMAT, ERR_SHAPE, ERR_SIZE, ERR_ALIGN, ERR_DEVICE, ERR_TIMEOUT = range(8)
CHAIN_MAX_PHASES, CHAIN_MAX_GROUP, CHAIN_MAX_MATRICES = 1024, 4, 4096
CHAIN_WS_CLOCKS = 8            # 32-bit word of the workspace where a chained launch leaves its clock stamps (IFLOW_CHAIN_WS_CLOCKS)
ATTN_STATIC_MAX_HEADS = 128


class Chain(C.Structure):
    """iflow_chain_t: what iflow_qgemv_chain_plan fills and iflow_qgemv_chain_launch takes (plain data)."""
    _fields_ = [("plan", C.c_void_p), ("workspace", C.c_void_p), ("grid", C.c_int32), ("max_strips", C.c_int32),
                ("magic", C.c_uint32), ("fused", C.c_uint32), ("format", C.c_int32), ("lds_bytes", C.c_int32),
                ("max_seq", C.c_int64)]


class DecodeLayer(C.Structure):
    """iflow_decode_layer_t: the device pointers of one decoder layer."""
    _fields_ = [(n, C.c_void_p) for n in ("wq", "wk", "wv", "wo", "w_gate", "w_up", "w_down", "norm1", "norm2", "k_cache", "v_cache")]


class DecodeStack(C.Structure):
    """iflow_decode_stack_t."""
    _fields_ = [("format", C.c_int), ("n_layers", C.c_int32), ("hidden", C.c_int32), ("ffn", C.c_int32), ("n_heads", C.c_int32),
                ("n_kv_heads", C.c_int32), ("head_dim", C.c_int32), ("max_seq", C.c_int64), ("eps", C.c_float), ("rope_base", C.c_float),
                ("rope_pairing", C.c_int32), ("layers", C.POINTER(DecodeLayer)), ("h_in", C.c_void_p), ("h_out", C.c_void_p),
                ("scratch", C.c_void_p)]


class IflowError(RuntimeError):
    def __init__(self, status: int, what: str):
        self.status = status
        super().__init__(f"{what}: {status_string(status)} (status {status})")


_lib = None


def lib():
    """Load libiflow.so (once).  Raises if it is missing: the product path has no fallback."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(f"{LIB_PATH} is missing: build it with __graft_entry__.build() "
                               "or `python -m paper_2401_08294_amd.build`")
        # PyTorch ships its own HIP runtime; import it first so that the library binds to that same
        # runtime (two runtimes in one process do not share devices, streams or memory).
        import torch  # noqa: F401
        L = C.CDLL(LIB_PATH)
        i64, p, sz = C.c_int64, C.c_void_p, C.c_size_t
        L.iflow_layout_version.restype = C.c_int
        L.iflow_status_string.restype = C.c_char_p
        L.iflow_status_string.argtypes = [C.c_int]
        L.iflow_last_hip_error.restype = C.c_int
        L.iflow_format_block.argtypes = [C.c_int]
        L.iflow_format_levels.argtypes = [C.c_int]
        L.iflow_packed_bytes.argtypes = [C.c_int, i64, i64, C.POINTER(sz)]
        L.iflow_quantize.argtypes = [C.c_int, p, i64, i64, p, sz, p]
        L.iflow_dequant.argtypes = [C.c_int, p, i64, i64, p, p]
        L.iflow_qgemv.argtypes = [C.c_int, p, i64, i64, p, p, p]
        L.iflow_qgemm.argtypes = [C.c_int, p, i64, i64, p, i64, p, p]
        L.iflow_unpack_logical.argtypes = [C.c_int, p, i64, i64, p, p, p, p]
        L.iflow_unpack_pair_codes.argtypes = [C.c_int, p, i64, i64, p, p]
        L.iflow_calibration_copy.argtypes = [p, p, sz, p]
        L.iflow_calibration_read.argtypes = [p, sz, p, p]
        L.iflow_qgemv_multi.argtypes = [C.c_int, C.c_int, C.POINTER(p), C.POINTER(i64), i64, p, C.POINTER(p), p]
        L.iflow_qgemv_gated.argtypes = [C.c_int, p, p, i64, i64, p, C.c_int, p, C.c_float, p, p]
        L.iflow_qgemv_fused.argtypes = [C.c_int, C.c_int, C.POINTER(p), C.POINTER(i64), i64, p, C.c_int, p, C.c_float,
                                        C.POINTER(p), C.POINTER(p), p]
        L.iflow_qgemm_fused.argtypes = [C.c_int, p, i64, i64, p, i64, C.c_int, p, C.c_float, p, p, p]
        L.iflow_attn_decode_workspace_bytes.argtypes = [C.c_int, C.POINTER(sz)]
        L.iflow_attn_decode.argtypes = [p, p, p, C.c_int, C.c_int, C.c_int, i64, i64, C.c_float, p, p, sz, p]
        L.iflow_attn_decode_static.argtypes = [p, p, p, C.c_int, C.c_int, C.c_int, i64, i64, C.c_float, p, p]
        L.iflow_rope_append.argtypes = [p, p, p, C.c_int, C.c_int, C.c_int, i64, i64, C.c_float, C.c_int, p, p, p]
        L.iflow_qgemv_chain_workspace_bytes.argtypes = [C.c_int, C.POINTER(i64), C.POINTER(sz)]
        L.iflow_qgemv_chain_plan_bytes.argtypes = [C.c_int, C.c_int, C.POINTER(sz)]
        L.iflow_qgemv_chain_plan.argtypes = [C.c_int, C.c_int, C.POINTER(C.c_int), C.POINTER(i64), C.POINTER(p), C.POINTER(p),
                                             C.POINTER(i64), C.POINTER(p), p, sz, p, sz, p, C.POINTER(Chain)]
        L.iflow_qgemv_chain_plan_fused.argtypes = [C.c_int, C.c_int, C.POINTER(C.c_int), C.POINTER(i64), C.POINTER(p), C.POINTER(C.c_int),
                                                   C.POINTER(p), C.POINTER(C.c_float), C.POINTER(C.c_int), C.POINTER(p), C.POINTER(i64),
                                                   C.POINTER(p), C.POINTER(p), p, sz, p, sz, p, C.POINTER(Chain)]
        L.iflow_qgemv_chain_launch.argtypes = [C.POINTER(Chain), p]
        L.iflow_qgemv_chain_check.argtypes = [C.POINTER(Chain), p]
        L.iflow_decode_stack_sizes.argtypes = [C.POINTER(DecodeStack), C.POINTER(sz), C.POINTER(sz), C.POINTER(sz)]
        L.iflow_decode_stack_plan.argtypes = [C.POINTER(DecodeStack), p, sz, p, sz, p, C.POINTER(Chain)]
        L.iflow_decode_stack_launch.argtypes = [C.POINTER(Chain), i64, p]
        _lib = L
    return _lib


def _ptr(t):
    """Device address of a torch tensor, or an integer address passed through."""
    return t if isinstance(t, int) or t is None else t.data_ptr()


def _stream(stream):
    if stream is None:
        import torch
        return torch.cuda.current_stream().cuda_stream
    return stream if isinstance(stream, int) else stream.cuda_stream


def _check(status: int, what: str):
    if status != OK:
        raise IflowError(status, what)


def layout_version() -> int:
    return lib().iflow_layout_version()


def status_string(status: int) -> str:
    return lib().iflow_status_string(status).decode()


def last_hip_error() -> int:
    return lib().iflow_last_hip_error()


def format_block(fmt: int) -> int:
    return lib().iflow_format_block(fmt)


def format_levels(fmt: int) -> int:
    return lib().iflow_format_levels(fmt)


def packed_bytes(fmt: int, rows: int, cols: int) -> int:
    out = C.c_size_t(0)
    _check(lib().iflow_packed_bytes(fmt, rows, cols, C.byref(out)), "iflow_packed_bytes")
    return int(out.value)


def quantize(fmt: int, w, rows: int, cols: int, packed, packed_capacity: int, stream=None) -> None:
    """w: fp32 [rows][cols] device tensor; packed: uint8 device tensor of at least packed_bytes()."""
    _check(lib().iflow_quantize(fmt, _ptr(w), rows, cols, _ptr(packed), packed_capacity, _stream(stream)), "iflow_quantize")


def dequant(fmt: int, packed, rows: int, cols: int, w16, stream=None) -> None:
    _check(lib().iflow_dequant(fmt, _ptr(packed), rows, cols, _ptr(w16), _stream(stream)), "iflow_dequant")


def qgemv(fmt: int, packed, rows: int, cols: int, x, y, stream=None) -> None:
    _check(lib().iflow_qgemv(fmt, _ptr(packed), rows, cols, _ptr(x), _ptr(y), _stream(stream)), "iflow_qgemv")


def qgemm(fmt: int, packed, rows: int, cols: int, X, batch: int, Y, stream=None) -> None:
    _check(lib().iflow_qgemm(fmt, _ptr(packed), rows, cols, _ptr(X), batch, _ptr(Y), _stream(stream)), "iflow_qgemm")


def unpack_logical(fmt: int, packed, rows: int, cols: int, levels, scale16, offset16, stream=None) -> None:
    _check(lib().iflow_unpack_logical(fmt, _ptr(packed), rows, cols, _ptr(levels), _ptr(scale16), _ptr(offset16),
                                      _stream(stream)), "iflow_unpack_logical")


def unpack_pair_codes(fmt: int, packed, rows: int, cols: int, codes, stream=None) -> None:
    """The 3.5-bit format's stored pair codes [rows][cols/2] (Eq.4), uint8."""
    _check(lib().iflow_unpack_pair_codes(fmt, _ptr(packed), rows, cols, _ptr(codes), _stream(stream)), "iflow_unpack_pair_codes")


def calibration_copy(src, dst, nbytes: int, stream=None) -> None:
    _check(lib().iflow_calibration_copy(_ptr(src), _ptr(dst), nbytes, _stream(stream)), "iflow_calibration_copy")


def calibration_read(src, nbytes: int, sink, stream=None) -> None:
    _check(lib().iflow_calibration_read(_ptr(src), nbytes, _ptr(sink), _stream(stream)), "iflow_calibration_read")


def qgemv_multi(fmt: int, packed_list, rows_list, cols: int, x, y_list, stream=None) -> None:
    """y_list[i] = W'_i x for matrices that share x and cols; one launch for Q3H."""
    n = len(packed_list)
    pk = (C.c_void_p * n)(*[_ptr(t) for t in packed_list])
    ys = (C.c_void_p * n)(*[_ptr(t) for t in y_list])
    rs = (C.c_int64 * n)(*[int(r) for r in rows_list])
    _check(lib().iflow_qgemv_multi(fmt, n, pk, rs, cols, _ptr(x), ys, _stream(stream)), "iflow_qgemv_multi")


X_PLAIN, X_RMS_GAIN, X_SILU_MUL = 0, 1, 2
ROPE_ADJACENT, ROPE_HALVES = 0, 1


def qgemv_fused(fmt: int, packed_list, rows_list, cols: int, x, y_list, x_op: int = X_PLAIN, aux=None, eps: float = 0.0,
                residual_list=None, stream=None) -> None:
    """qgemv_multi with rms normalization (aux = gains) or the silu-gated input (aux = second factor) in front of the
    product and an optional residual per matrix behind it, in the same launch."""
    n = len(packed_list)
    pk = (C.c_void_p * n)(*[_ptr(t) for t in packed_list])
    ys = (C.c_void_p * n)(*[_ptr(t) for t in y_list])
    rs = (C.c_int64 * n)(*[int(r) for r in rows_list])
    res = None
    if residual_list is not None:
        res = (C.c_void_p * n)(*[(_ptr(t) if t is not None else None) for t in residual_list])
    _check(lib().iflow_qgemv_fused(fmt, n, pk, rs, cols, _ptr(x), x_op, _ptr(aux) if aux is not None else None, eps, res, ys,
                                   _stream(stream)), "iflow_qgemv_fused")


def qgemm_fused(fmt: int, packed, rows: int, cols: int, X, batch: int, Y, x_op: int = X_PLAIN, aux=None, eps: float = 0.0,
                residual=None, stream=None) -> None:
    """qgemv_fused for 1..16 activation vectors X [batch][cols] -> Y [batch][rows]: rms normalization (aux = gains [cols]) or the
    silu-gated input (aux [batch][cols]) in front of the product, an optional residual [batch][rows] behind it."""
    _check(lib().iflow_qgemm_fused(fmt, _ptr(packed), rows, cols, _ptr(X), batch, x_op, _ptr(aux) if aux is not None else None, eps,
                                   _ptr(residual) if residual is not None else None, _ptr(Y), _stream(stream)), "iflow_qgemm_fused")


def qgemv_gated(fmt: int, packed_gate, packed_up, rows: int, cols: int, x, y, x_op: int = X_PLAIN, aux=None, eps: float = 0.0,
                stream=None) -> None:
    """y = silu(c W_gate' v) * (c W_up' v): a gated feed-forward's two first projections and its gate in one launch
    (v, c: x itself and 1, or the rms-normalized x with gains `aux`)."""
    _check(lib().iflow_qgemv_gated(fmt, _ptr(packed_gate), _ptr(packed_up), rows, cols, _ptr(x), x_op,
                                   _ptr(aux) if aux is not None else None, eps, _ptr(y), _stream(stream)), "iflow_qgemv_gated")


def attn_decode_workspace_bytes(n_heads: int) -> int:
    out = C.c_size_t(0)
    _check(lib().iflow_attn_decode_workspace_bytes(n_heads, C.byref(out)), "iflow_attn_decode_workspace_bytes")
    return int(out.value)


def attn_decode(q, k_cache, v_cache, n_heads: int, n_kv_heads: int, head_dim: int, seq_len: int, max_seq: int, scale: float, out,
                workspace, workspace_bytes: int, stream=None) -> None:
    """One decode step of grouped-query attention over an fp16 key/value cache [n_kv_heads][max_seq][head_dim]."""
    _check(lib().iflow_attn_decode(_ptr(q), _ptr(k_cache), _ptr(v_cache), n_heads, n_kv_heads, head_dim, seq_len, max_seq, scale,
                                   _ptr(out), _ptr(workspace), workspace_bytes, _stream(stream)), "iflow_attn_decode")


def attn_decode_static(q, k_cache, v_cache, n_heads: int, n_kv_heads: int, head_dim: int, seq_len: int, max_seq: int, scale: float,
                       out, stream=None) -> None:
    """attn_decode without a workspace argument: the partial results live in an array inside the library (no allocation)."""
    _check(lib().iflow_attn_decode_static(_ptr(q), _ptr(k_cache), _ptr(v_cache), n_heads, n_kv_heads, head_dim, seq_len, max_seq,
                                          scale, _ptr(out), _stream(stream)), "iflow_attn_decode_static")


def rope_append(q, k_new, v_new, n_heads: int, n_kv_heads: int, head_dim: int, position: int, max_seq: int, base: float,
                pair_mode: int, k_cache, v_cache, stream=None) -> None:
    """Rotary position embedding of one decode step: q rotated in place, rotated k_new and v_new written to row `position`
    of the caches [n_kv_heads][max_seq][head_dim]."""
    _check(lib().iflow_rope_append(_ptr(q), _ptr(k_new), _ptr(v_new), n_heads, n_kv_heads, head_dim, position, max_seq, base,
                                   pair_mode, _ptr(k_cache), _ptr(v_cache), _stream(stream)), "iflow_rope_append")


def qgemv_chain_workspace_bytes(rows_list) -> int:
    n = len(rows_list)
    rs = (C.c_int64 * n)(*[int(r) for r in rows_list])
    out = C.c_size_t(0)
    _check(lib().iflow_qgemv_chain_workspace_bytes(n, rs, C.byref(out)), "iflow_qgemv_chain_workspace_bytes")
    return int(out.value)


def _chain_arrays(phases):
    nph = len(phases)
    mats = [m for (_, _, ms) in phases for m in ms]
    n = len(mats)
    counts = (C.c_int * nph)(*[len(ms) for (_, _, ms) in phases])
    cols = (C.c_int64 * nph)(*[int(c) for (c, _, _) in phases])
    xs = (C.c_void_p * nph)(*[_ptr(x) for (_, x, _) in phases])
    pk = (C.c_void_p * n)(*[_ptr(m[0]) for m in mats])
    rs = (C.c_int64 * n)(*[int(m[1]) for m in mats])
    ys = (C.c_void_p * n)(*[_ptr(m[2]) for m in mats])
    return nph, counts, cols, xs, pk, rs, ys


def qgemv_chain_plan_bytes(phases) -> int:
    """Size of the plan.  `phases`: list of (cols, x, [(packed, rows, y), ...])."""
    out = C.c_size_t(0)
    _check(lib().iflow_qgemv_chain_plan_bytes(len(phases), sum(len(ph[2]) for ph in phases), C.byref(out)), "iflow_qgemv_chain_plan_bytes")
    return int(out.value)


def qgemv_chain_plan(fmt: int, phases, plan, plan_bytes: int, workspace, workspace_bytes: int, stream=None) -> Chain:
    """Compiles a chain of batch-1 products once.  `phases` is a list of (cols, x, [(packed, rows, y), ...]); x may be the y
    tensor of a matrix of an earlier phase.  `plan`, `workspace`: uint8 device tensors the chain keeps using."""
    nph, counts, cols, xs, pk, rs, ys = _chain_arrays(phases)
    chain = Chain()
    _check(lib().iflow_qgemv_chain_plan(fmt, nph, counts, cols, xs, pk, rs, ys, _ptr(plan), plan_bytes, _ptr(workspace),
                                        workspace_bytes, _stream(stream), C.byref(chain)), "iflow_qgemv_chain_plan")
    return chain


def qgemv_chain_plan_fused(fmt: int, phases, plan, plan_bytes: int, workspace, workspace_bytes: int, stream=None) -> Chain:
    """qgemv_chain_plan with the modules between the products.  `phases` is a list of (cols, x, mats, ops): mats a list of
    (packed, rows, y) or (packed, rows, y, residual) (y None for the up matrix of a gated pair), ops a dict with any of
    x_op (X_PLAIN / X_RMS_GAIN), aux (the gains), eps, gated (bool)."""
    nph, counts, cols, xs, pk, rs, ys = _chain_arrays([(c, x, ms) for (c, x, ms, _) in phases])
    mats = [m for (_, _, ms, _) in phases for m in ms]
    n = len(mats)
    x_op = (C.c_int * nph)(*[int(o.get("x_op", X_PLAIN)) for (_, _, _, o) in phases])
    aux = (C.c_void_p * nph)(*[_ptr(o.get("aux")) for (_, _, _, o) in phases])
    eps = (C.c_float * nph)(*[float(o.get("eps", 0.0)) for (_, _, _, o) in phases])
    gated = (C.c_int * nph)(*[int(bool(o.get("gated", False))) for (_, _, _, o) in phases])
    res = (C.c_void_p * n)(*[_ptr(m[3]) if len(m) > 3 else None for m in mats])
    chain = Chain()
    _check(lib().iflow_qgemv_chain_plan_fused(fmt, nph, counts, cols, xs, x_op, aux, eps, gated, pk, rs, res, ys, _ptr(plan), plan_bytes,
                                              _ptr(workspace), workspace_bytes, _stream(stream), C.byref(chain)), "iflow_qgemv_chain_plan_fused")
    return chain


def qgemv_chain_launch(chain: Chain, stream=None) -> None:
    _check(lib().iflow_qgemv_chain_launch(C.byref(chain), _stream(stream)), "iflow_qgemv_chain_launch")


def qgemv_chain_check(chain: Chain, stream=None) -> None:
    """Synchronises the stream; raises IflowError(ERR_TIMEOUT) if a chained launch gave up a wait."""
    _check(lib().iflow_qgemv_chain_check(C.byref(chain), _stream(stream)), "iflow_qgemv_chain_check")


def decode_stack(fmt: int, hidden: int, ffn: int, n_heads: int, n_kv_heads: int, max_seq: int, eps: float, rope_base: float,
                 rope_pairing: int, layers=(), n_layers=None, h_in=None, h_out=None, scratch=None, head_dim: int = 128) -> DecodeStack:
    """Fills an iflow_decode_stack_t.  `layers`: one dict per layer with the keys wq wk wv wo w_gate w_up w_down norm1 norm2
    k_cache v_cache (tensors or addresses); for a size query give n_layers instead."""
    n = len(layers) if n_layers is None else n_layers
    arr = (DecodeLayer * max(len(layers), 1))()
    for i, ly in enumerate(layers):
        for name, _ in DecodeLayer._fields_:
            setattr(arr[i], name, _ptr(ly[name]))
    d = DecodeStack(fmt, n, hidden, ffn, n_heads, n_kv_heads, head_dim, max_seq, eps, rope_base, rope_pairing,
                    C.cast(arr, C.POINTER(DecodeLayer)) if layers else None, _ptr(h_in), _ptr(h_out), _ptr(scratch))
    d._keep = arr                                              # (the array lives as long as the description)
    return d


def decode_stack_sizes(stack: DecodeStack):
    """(scratch_bytes, plan_bytes, workspace_bytes) of a description (its pointers are not read)."""
    a, b, c = C.c_size_t(0), C.c_size_t(0), C.c_size_t(0)
    _check(lib().iflow_decode_stack_sizes(C.byref(stack), C.byref(a), C.byref(b), C.byref(c)), "iflow_decode_stack_sizes")
    return int(a.value), int(b.value), int(c.value)


def decode_stack_plan(stack: DecodeStack, plan, plan_bytes: int, workspace, workspace_bytes: int, stream=None) -> Chain:
    chain = Chain()
    _check(lib().iflow_decode_stack_plan(C.byref(stack), _ptr(plan), plan_bytes, _ptr(workspace), workspace_bytes, _stream(stream),
                                         C.byref(chain)), "iflow_decode_stack_plan")
    return chain


def decode_stack_launch(chain: Chain, position: int, stream=None) -> None:
    _check(lib().iflow_decode_stack_launch(C.byref(chain), position, _stream(stream)), "iflow_decode_stack_launch")

"""ctypes binding: argument marshalling only, same names as the C ABI."""
from __future__ import annotations

import ctypes
import os
import re
from dataclasses import dataclass
from typing import Optional, Sequence, Tuple

_PKG = os.path.dirname(os.path.abspath(__file__))
# NIMBLE_LIBRARY names another build of the same library (for A/B measurements)
_LIB_PATH = os.environ.get("NIMBLE_LIBRARY") or os.path.join(_PKG, "libnimble_hip.so")
_HEADERS = [os.path.join(os.path.dirname(_PKG), "include", h) for h in ("nimble.h", "nimble_probe.h", "nimble_vm.h")]

EPI_NONE, EPI_BIAS, EPI_BIAS_GELU_ERF = 0, 1, 2
BF16, F32 = 0, 1
VAR_AUTO = -1

_STATUS = {0: "OK", -1: "ERR_NULL", -2: "ERR_RANK", -3: "ERR_SHAPE", -4: "ERR_DTYPE", -5: "ERR_ALIGN",
           -6: "ERR_WORKSPACE", -7: "ERR_HIP", -8: "ERR_ARG"}


class NimbleError(RuntimeError):
    def __init__(self, code: int, message: str):
        super().__init__(f"NIMBLE_{_STATUS.get(code, code)}: {message}")
        self.code = code


class _CTableEntry(ctypes.Structure):
    _fields_ = [("m_lo", ctypes.c_int64), ("m_hi", ctypes.c_int64), ("variant", ctypes.c_int32),
                ("split_k", ctypes.c_int32)]


class _CPlan(ctypes.Structure):
    _fields_ = [("variant", ctypes.c_int32), ("bm", ctypes.c_int32), ("bn", ctypes.c_int32),
                ("bk", ctypes.c_int32), ("k", ctypes.c_int64), ("r", ctypes.c_int32),
                ("residue_copy", ctypes.c_int32), ("split_k", ctypes.c_int32),
                ("grid", ctypes.c_uint32 * 3), ("block", ctypes.c_uint32),
                ("workspace_bytes", ctypes.c_uint64), ("split_rows", ctypes.c_int64),
                ("residue_variant", ctypes.c_int32), ("residue_split_k", ctypes.c_int32)]


@dataclass
class Plan:
    variant: int
    name: str
    bm: int
    bn: int
    bk: int
    k: int
    r: int
    residue_copy: int
    split_k: int
    grid: Tuple[int, int, int]
    block: int
    workspace_bytes: int
    split_rows: int = 0
    residue_variant: int = -1
    residue_split_k: int = 0


_lib = None


def library_path() -> str:
    return _LIB_PATH


def load():
    """Load the HIP library.  There is no fallback: a missing library is an error."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(_LIB_PATH):
        raise ImportError(
            f"{_LIB_PATH} is not built; run `python -c 'import __graft_entry__ as g; g.build()'` "
            "(hipcc --offload-arch=gfx950) first")
    # torch ships its own HIP runtime (same SONAME as the system one).  Import it
    # first so that this library binds to the runtime that owns torch's streams
    # and allocations instead of bringing a second runtime into the process.
    try:
        import torch  # noqa: F401
    except ImportError:
        pass
    lib = ctypes.CDLL(_LIB_PATH)
    i64, i32, vp = ctypes.c_int64, ctypes.c_int, ctypes.c_void_p
    ip = ctypes.POINTER(ctypes.c_int64)
    lib.nimble_dense_shape.argtypes = [ip, i32, ip, i32, ip]
    lib.nimble_batch_matmul_shape.argtypes = [ip, i32, ip, i32, i32, ip]
    lib.nimble_lstm_shape.argtypes = [ip, ip, ip, ip, ip, ip]
    lib.nimble_storage_bytes.argtypes = [ip, i32, i32]
    lib.nimble_storage_bytes.restype = i64
    lib.nimble_storage_alignment.restype = i64
    lib.nimble_residue_split.argtypes = [i64, i64, ip, ip]
    lib.nimble_dense_plan.argtypes = [i64, i64, i64, i32, i32, i32, ctypes.POINTER(_CPlan)]
    lib.nimble_batch_matmul_plan.argtypes = [i64, i64, i64, i64, i32, i32, ctypes.POINTER(_CPlan)]
    lib.nimble_lstm_plan.argtypes = [i64, i64, i64, ctypes.POINTER(_CPlan)]
    lib.nimble_dense_table_set.argtypes = [i64, i64, i32, ctypes.POINTER(_CTableEntry), i32]
    lib.nimble_variant_name.argtypes = [i32]
    lib.nimble_variant_name.restype = ctypes.c_char_p
    lib.nimble_last_error.restype = ctypes.c_char_p
    lib.nimble_lstm_pre_shape.argtypes = [ip, ip, ip, ip, ip, ip]
    lib.nimble_dense_dyn.argtypes = [vp, vp, vp, vp, i64, i64, i64, i32, i32, vp, ctypes.c_size_t, vp]
    lib.nimble_dense_noalloc_dyn.argtypes = [vp, vp, vp, vp, i64, i64, i64, i32, i32, vp]
    lib.nimble_dense_variant_dyn.argtypes = [vp, vp, vp, vp, i64, i64, i64, i32, i32, i32, vp, ctypes.c_size_t, vp]
    lib.nimble_batch_matmul_dyn.argtypes = [vp, vp, vp, i64, i64, i64, i64, i32, ctypes.c_float, i32, vp,
                                            ctypes.c_size_t, vp]
    lib.nimble_softmax_rows_dyn.argtypes = [vp, vp, i64, i64, vp]
    lib.nimble_attention_dyn.argtypes = [vp, vp, vp, vp, i64, i64, i64, ctypes.c_float, vp]
    lib.nimble_lstm_gates_dyn.argtypes = [vp, vp, vp, vp, vp, vp, vp, i64, i64, i64, vp, ctypes.c_size_t, vp]
    lib.nimble_lstm_gates_pre_dyn.argtypes = [vp, vp, vp, vp, vp, vp, i64, i64, vp]
    lib.nimble_lstm_seq_shape.argtypes = [ip, ip, ip, ip, ip, ip]
    lib.nimble_lstm_seq_supported.argtypes = [i64, i64]
    lib.nimble_lstm_seq_preferred.argtypes = [i64, i64]
    lib.nimble_lstm_seq_workspace_bytes.argtypes = [i64, i64]
    lib.nimble_lstm_seq_workspace_bytes.restype = ctypes.c_size_t
    lib.nimble_lstm_seq_pre_dyn.argtypes = [vp, vp, vp, vp, vp, vp, i64, i64, i64, vp, ctypes.c_size_t,
                                            ctypes.c_uint32, vp]
    lib.nimble_lstm_seq_status.argtypes = [vp, vp, ctypes.POINTER(ctypes.c_int)]
    lib.nimble_probe_mfma_bf16.argtypes = [vp, vp, i32, i32, ctypes.POINTER(ctypes.c_double), vp]
    lib.nimble_probe_hbm_read.argtypes = [vp, ctypes.c_size_t, vp, vp]
    _lib = lib
    return lib


def exported_symbols() -> Sequence[str]:
    """Names of the functions the headers under ``include/`` declare."""
    names = set()
    for header in _HEADERS:
        text = re.sub(r"/\*.*?\*/", "", open(header).read(), flags=re.S)
        names.update(re.findall(r"\b(nimble_[a-z0-9_]+)\s*\(", text))
    return sorted(names)


def last_error() -> str:
    return load().nimble_last_error().decode()


def _check(rc: int):
    if rc != 0:
        raise NimbleError(rc, last_error())


def _arr(shape: Sequence[int]):
    return (ctypes.c_int64 * max(len(shape), 1))(*[int(s) for s in shape])


# ------------------------------------------------------------------ host side
# scratch int64 arrays for the rank-2 fast path of the shape functions (one shape tensor is 16
# bytes); reused across calls, so the binding is not re-entrant across threads
_SH2 = [(ctypes.c_int64 * 2)() for _ in range(3)]


def nimble_dense_shape(x_shape: Sequence[int], w_shape: Sequence[int]) -> Tuple[int, int]:
    if len(x_shape) == 2 and len(w_shape) == 2:
        xs, ws, out = _SH2
        xs[0], xs[1] = x_shape
        ws[0], ws[1] = w_shape
        rc = _lib.nimble_dense_shape(xs, 2, ws, 2, out) if _lib is not None else load().nimble_dense_shape(xs, 2, ws, 2, out)
        if rc != 0:
            raise NimbleError(rc, last_error())
        return out[0], out[1]
    out = (ctypes.c_int64 * 2)(-1, -1)
    _check(load().nimble_dense_shape(_arr(x_shape), len(x_shape), _arr(w_shape), len(w_shape), out))
    return int(out[0]), int(out[1])


dense_shape = nimble_dense_shape


def batch_matmul_shape(a_shape, b_shape, trans_b: bool) -> Tuple[int, int, int]:
    if len(a_shape) == 3 and len(b_shape) == 3:
        a, b, out = _SH3
        a[0], a[1], a[2] = a_shape
        b[0], b[1], b[2] = b_shape
        _check(load().nimble_batch_matmul_shape(a, 3, b, 3, int(bool(trans_b)), out))
        return out[0], out[1], out[2]
    out = (ctypes.c_int64 * 3)(-1, -1, -1)
    _check(load().nimble_batch_matmul_shape(_arr(a_shape), len(a_shape), _arr(b_shape), len(b_shape),
                                            int(bool(trans_b)), out))
    return int(out[0]), int(out[1]), int(out[2])


_SH2L = [(ctypes.c_int64 * 2)() for _ in range(6)]
_SH3 = [(ctypes.c_int64 * 3)() for _ in range(3)]


def lstm_shape(x_shape, h_shape, c_shape, w_shape):
    for s in (x_shape, h_shape, c_shape, w_shape):
        if len(s) != 2:
            raise NimbleError(-2, "lstm expects rank-2 shapes")
    xs, hs, cs, ws, ho, co = _SH2L
    xs[0], xs[1] = x_shape
    hs[0], hs[1] = h_shape
    cs[0], cs[1] = c_shape
    ws[0], ws[1] = w_shape
    _check(load().nimble_lstm_shape(xs, hs, cs, ws, ho, co))
    return (ho[0], ho[1]), (co[0], co[1])


def lstm_pre_shape(pre_shape, h_shape, c_shape, wh_shape):
    for s in (pre_shape, h_shape, c_shape, wh_shape):
        if len(s) != 2:
            raise NimbleError(-2, "lstm expects rank-2 shapes")
    ps, hs, cs, ws, ho, co = _SH2L
    ps[0], ps[1] = pre_shape
    hs[0], hs[1] = h_shape
    cs[0], cs[1] = c_shape
    ws[0], ws[1] = wh_shape
    _check(load().nimble_lstm_pre_shape(ps, hs, cs, ws, ho, co))
    return (ho[0], ho[1]), (co[0], co[1])


def lstm_seq_shape(pre_shape, h0_shape, c0_shape, wh_shape):
    """Shape function of the one-launch token loop: ((T,B,H), (B,H))."""
    if len(pre_shape) != 3 or any(len(s) != 2 for s in (h0_shape, c0_shape, wh_shape)):
        raise NimbleError(-2, "lstm sequence expects pre of rank 3 and rank-2 states and weight")
    ps = (ctypes.c_int64 * 3)(*pre_shape)
    hs, cs, ws = _arr(h0_shape), _arr(c0_shape), _arr(wh_shape)
    ho, co = (ctypes.c_int64 * 3)(), (ctypes.c_int64 * 2)()
    _check(load().nimble_lstm_seq_shape(ps, hs, cs, ws, ho, co))
    return (ho[0], ho[1], ho[2]), (co[0], co[1])


def lstm_seq_supported(B: int, H: int) -> bool:
    return bool(load().nimble_lstm_seq_supported(B, H))


def lstm_seq_preferred(B: int, H: int) -> bool:
    return bool(load().nimble_lstm_seq_preferred(B, H))


def lstm_seq_workspace_bytes(B: int, H: int) -> int:
    return int(load().nimble_lstm_seq_workspace_bytes(B, H))


def nimble_lstm_seq_pre_dyn(pre: int, w_h: int, h0: int, c0: int, h_seq: int, c_out: int, T: int, B: int, H: int,
                            workspace: int, workspace_bytes: int, max_polls: int, stream: int) -> None:
    _check(load().nimble_lstm_seq_pre_dyn(pre, w_h, h0, c0, h_seq, c_out, T, B, H, workspace, workspace_bytes,
                                          max_polls, stream))


def nimble_lstm_seq_status(workspace: int, stream: int) -> bool:
    """Waits for the stream; True when the loop gave up (its outputs are then unspecified)."""
    flag = ctypes.c_int(0)
    _check(load().nimble_lstm_seq_status(workspace, stream, ctypes.byref(flag)))
    return bool(flag.value)


def storage_bytes(shape: Sequence[int], dtype: int) -> int:
    if len(shape) == 2:
        arr = _SH2[2]
        arr[0], arr[1] = shape
        n = load().nimble_storage_bytes(arr, 2, dtype)
    else:
        n = int(load().nimble_storage_bytes(_arr(shape), len(shape), dtype))
    if n < 0:
        raise NimbleError(n, last_error())
    return n


def storage_alignment() -> int:
    return int(load().nimble_storage_alignment())


def residue_split(x: int, tile: int) -> Tuple[int, int]:
    k, r = ctypes.c_int64(0), ctypes.c_int64(0)
    _check(load().nimble_residue_split(x, tile, ctypes.byref(k), ctypes.byref(r)))
    return int(k.value), int(r.value)


def variant_name(v: int) -> Optional[str]:
    s = load().nimble_variant_name(v)
    return s.decode() if s else None


def _plan(c: _CPlan) -> Plan:
    return Plan(c.variant, variant_name(c.variant) or "?", c.bm, c.bn, c.bk, c.k, c.r, c.residue_copy,
                c.split_k, (c.grid[0], c.grid[1], c.grid[2]), c.block, c.workspace_bytes, c.split_rows,
                c.residue_variant, c.residue_split_k)


def dense_plan(M: int, N: int, K: int, epilogue: int = EPI_BIAS, out_dtype: int = BF16,
               force_variant: int = VAR_AUTO) -> Plan:
    c = _CPlan()
    _check(load().nimble_dense_plan(M, N, K, epilogue, out_dtype, force_variant, ctypes.byref(c)))
    return _plan(c)


def dense_table_set(N: int, K: int, epilogue: int, entries: Sequence[Tuple[int, int, int, int]]) -> None:
    """entries: (m_lo, m_hi, variant, split_k); an empty list removes the table."""
    arr = (_CTableEntry * max(len(entries), 1))()
    for i, (lo, hi, v, sk) in enumerate(entries):
        arr[i] = _CTableEntry(int(lo), int(hi), int(v), int(sk))
    _check(load().nimble_dense_table_set(N, K, epilogue, arr, len(entries)))


def batch_matmul_plan(batch: int, M: int, N: int, K: int, trans_b: bool, out_dtype: int = BF16) -> Plan:
    c = _CPlan()
    _check(load().nimble_batch_matmul_plan(batch, M, N, K, int(bool(trans_b)), out_dtype, ctypes.byref(c)))
    return _plan(c)


def lstm_plan(B: int, Ix: int, H: int) -> Plan:
    c = _CPlan()
    _check(load().nimble_lstm_plan(B, Ix, H, ctypes.byref(c)))
    return _plan(c)


# ---------------------------------------------------------------- device side
# Pointers are integers (tensor.data_ptr()); `stream` is a hipStream_t handle as
# an integer (torch.cuda.current_stream().cuda_stream), 0 for the default one.
def nimble_dense_dyn(x: int, w: int, bias: int, y: int, M: int, N: int, K: int, epilogue: int,
                     out_dtype: int = BF16, workspace: int = 0, workspace_bytes: int = 0, stream: int = 0) -> None:
    _check(load().nimble_dense_dyn(x, w, bias, y, M, N, K, epilogue, out_dtype, workspace, workspace_bytes, stream))


NOALLOC_SCRATCH_BYTES = 32 << 20


def nimble_dense_noalloc_dyn(x: int, w: int, bias: int, y: int, M: int, N: int, K: int, epilogue: int,
                             out_dtype: int = BF16, stream: int = 0) -> None:
    """nimble_dense_dyn on the library's built-in scratch: allocates nothing, takes no workspace."""
    _check(load().nimble_dense_noalloc_dyn(x, w, bias, y, M, N, K, epilogue, out_dtype, stream))


def nimble_dense_variant_dyn(x: int, w: int, bias: int, y: int, M: int, N: int, K: int, epilogue: int,
                             out_dtype: int = BF16, force_variant: int = VAR_AUTO, workspace: int = 0,
                             workspace_bytes: int = 0, stream: int = 0) -> None:
    """Measurement entry point: dense with the dispatch decision forced by the caller."""
    _check(load().nimble_dense_variant_dyn(x, w, bias, y, M, N, K, epilogue, out_dtype, force_variant, workspace,
                                           workspace_bytes, stream))


def nimble_batch_matmul_dyn(a: int, b: int, c: int, batch: int, M: int, N: int, K: int, trans_b: bool,
                            alpha: float = 1.0, out_dtype: int = BF16, workspace: int = 0,
                            workspace_bytes: int = 0, stream: int = 0) -> None:
    _check(load().nimble_batch_matmul_dyn(a, b, c, batch, M, N, K, int(bool(trans_b)), alpha, out_dtype,
                                          workspace, workspace_bytes, stream))


def nimble_softmax_rows_dyn(s_f32: int, p_bf16: int, rows: int, cols: int, stream: int = 0) -> None:
    _check(load().nimble_softmax_rows_dyn(s_f32, p_bf16, rows, cols, stream))


def nimble_attention_dyn(q: int, k: int, v: int, o: int, heads: int, L: int, D: int, alpha: float,
                         stream: int = 0) -> None:
    _check(load().nimble_attention_dyn(q, k, v, o, heads, L, D, alpha, stream))


def nimble_lstm_gates_dyn(x: int, h_prev: int, w: int, bias: int, c_prev: int, c_out: int, h_out: int,
                          B: int, Ix: int, H: int, workspace: int = 0, workspace_bytes: int = 0,
                          stream: int = 0) -> None:
    _check(load().nimble_lstm_gates_dyn(x, h_prev, w, bias, c_prev, c_out, h_out, B, Ix, H, workspace,
                                        workspace_bytes, stream))


def nimble_lstm_gates_pre_dyn(pre: int, h_prev: int, w_h: int, c_prev: int, c_out: int, h_out: int, B: int, H: int,
                              stream: int = 0) -> None:
    _check(load().nimble_lstm_gates_pre_dyn(pre, h_prev, w_h, c_prev, c_out, h_out, B, H, stream))


def nimble_probe_mfma_bf16(seed: int, sink: int, waves_per_simd: int, iters: int, stream: int = 0) -> float:
    """Launches the register-only MFMA loop; returns the flop count of the launch."""
    flops = ctypes.c_double(0.0)
    _check(load().nimble_probe_mfma_bf16(seed, sink, waves_per_simd, iters, ctypes.byref(flops), stream))
    return flops.value


def nimble_probe_hbm_read(buf: int, nbytes: int, sink: int, stream: int = 0) -> None:
    _check(load().nimble_probe_hbm_read(buf, nbytes, sink, stream))

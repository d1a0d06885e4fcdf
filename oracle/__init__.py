"""CPU oracle (float32, by the definition) for the dynamic-M operators.

TEST INFRASTRUCTURE ONLY: imported by ``tests/``, by the smoke check and by the
benchmark's CPU-baseline leg.  The product path (the HIP library and its Python
binding) never imports this package, and this package imports nothing of it.

The arithmetic lives in ``nimble_oracle.c`` (plain C, OpenMP over output rows);
this file marshals numpy arrays into it and composes the attention chain.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from typing import Optional, Sequence, Tuple

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "nimble_oracle.c")
_LIB = os.path.join(_HERE, "libnimble_oracle.so")

EPI = {"none": 0, "bias": 1, "bias_gelu": 2}


class OracleShapeError(ValueError):
    """A run-time type-relation violation found by a shape function."""


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (portable x86-64, no FMA contraction)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O3", "-ffp-contract=off", "-fopenmp", "-fPIC", "-shared", "-std=c11",
               "-Wall", "-Wextra", "-o", _LIB, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


_lib = None


def _load():
    global _lib
    if _lib is None:
        build()
        lib = ctypes.CDLL(_LIB)
        fp = ctypes.POINTER(ctypes.c_float)
        ip = ctypes.POINTER(ctypes.c_int64)
        i64 = ctypes.c_int64
        lib.oracle_gelu.argtypes = [fp, fp, i64]
        lib.oracle_gelu.restype = None
        lib.oracle_dense.argtypes = [fp, fp, fp, fp, i64, i64, i64, ctypes.c_int]
        lib.oracle_batch_matmul.argtypes = [fp, fp, fp, i64, i64, i64, i64, ctypes.c_int, ctypes.c_float]
        lib.oracle_softmax_rows.argtypes = [fp, fp, i64, i64]
        lib.oracle_lstm_step.argtypes = [fp, fp, fp, fp, fp, fp, fp, fp, i64, i64, i64]
        lib.oracle_lstm_step_pre.argtypes = [fp, fp, fp, fp, fp, fp, fp, i64, i64]
        lib.oracle_dense_shape.argtypes = [ip, ctypes.c_int, ip, ctypes.c_int, ip]
        lib.oracle_batch_matmul_shape.argtypes = [ip, ctypes.c_int, ip, ctypes.c_int, ctypes.c_int, ip]
        lib.oracle_lstm_shape.argtypes = [ip, ip, ip, ip, ip, ip]
        lib.oracle_storage_bytes.argtypes = [ip, ctypes.c_int, i64]
        lib.oracle_storage_bytes.restype = i64
        lib.oracle_residue_split.argtypes = [i64, i64, ip, ip]
        _lib = lib
    return _lib


def _f(a) -> np.ndarray:
    return np.ascontiguousarray(a, dtype=np.float32)


def _p(a: np.ndarray):
    return a.ctypes.data_as(ctypes.POINTER(ctypes.c_float))


def _shape_arr(shape: Sequence[int]) -> np.ndarray:
    return np.asarray(list(shape), dtype=np.int64)


def _ip(a: np.ndarray):
    return a.ctypes.data_as(ctypes.POINTER(ctypes.c_int64))


def _check(rc: int, what: str):
    if rc == -3:
        raise OracleShapeError(f"{what}: shapes violate the operator's type relation")
    if rc == -2:
        raise OracleShapeError(f"{what}: wrong rank")
    if rc != 0:
        raise ValueError(f"{what}: bad argument (code {rc})")


def num_threads() -> int:
    """Threads the OpenMP loops use (OMP_NUM_THREADS or the cores visible)."""
    env = os.environ.get("OMP_NUM_THREADS")
    if env:
        try:
            return max(1, int(env.split(",")[0]))
        except ValueError:
            pass
    try:
        return len(os.sched_getaffinity(0))
    except AttributeError:
        return os.cpu_count() or 1


# ---------------------------------------------------------------- arithmetic
def gelu(x) -> np.ndarray:
    x = _f(x)
    y = np.empty_like(x)
    _load().oracle_gelu(_p(x), _p(y), x.size)
    return y


def dense(x, w, b=None, epilogue: str = "none") -> np.ndarray:
    """Y[M,N] = epi(X[M,K] . W[N,K]^T + b[N]); the shape function runs first."""
    x, w = _f(x), _f(w)
    M, N = dense_shape(x.shape, w.shape)
    K = x.shape[1]
    epi = EPI[epilogue]
    if epi != 0:
        if b is None:
            raise ValueError("epilogue needs a bias")
        b = _f(b)
        if b.shape != (N,):
            raise OracleShapeError("bias must have shape (N,)")
    else:
        b = np.zeros((max(N, 1),), dtype=np.float32)
    y = np.empty((M, N), dtype=np.float32)
    _check(_load().oracle_dense(_p(x), _p(w), _p(b), _p(y), M, N, K, epi), "dense")
    return y


def batch_matmul(a, b, trans_b: bool = True, alpha: float = 1.0) -> np.ndarray:
    a, b = _f(a), _f(b)
    T, M, N = batch_matmul_shape(a.shape, b.shape, trans_b)
    K = a.shape[2]
    c = np.empty((T, M, N), dtype=np.float32)
    _check(_load().oracle_batch_matmul(_p(a), _p(b), _p(c), T, M, N, K, int(bool(trans_b)),
                                       ctypes.c_float(alpha)), "batch_matmul")
    return c


def softmax_rows(s) -> np.ndarray:
    s = _f(s)
    cols = s.shape[-1]
    rows = s.size // cols if cols else 0
    p = np.empty_like(s)
    _check(_load().oracle_softmax_rows(_p(s), _p(p), rows, cols), "softmax_rows")
    return p


def attention(q, k, v, alpha: float = 0.125, round_p=None) -> Tuple[np.ndarray, np.ndarray, np.ndarray]:
    """S = alpha Q.K^T, P = softmax rows of S, O = P.V.  No rounding between the
    steps unless ``round_p`` (a float32->float32 rounding function) is given,
    which is then applied to P before P.V (diagnosis only)."""
    s = batch_matmul(q, k, trans_b=True, alpha=alpha)
    p = softmax_rows(s)
    pv = round_p(p) if round_p is not None else p
    o = batch_matmul(pv, v, trans_b=False, alpha=1.0)
    return s, p, o


def lstm_step(x, h, w, b, c) -> Tuple[np.ndarray, np.ndarray]:
    """One LSTM cell step; returns (h', c').  Gate blocks of W, b: i, f, g, o."""
    x, h, w, b, c = _f(x), _f(h), _f(w), _f(b), _f(c)
    (B, H), _ = lstm_shape(x.shape, h.shape, c.shape, w.shape)
    if b.shape != (4 * H,):
        raise OracleShapeError("bias must have shape (4H,)")
    Ix = x.shape[1]
    h_out = np.empty((B, H), dtype=np.float32)
    c_out = np.empty((B, H), dtype=np.float32)
    g = np.empty((B, 4 * H), dtype=np.float32)
    _check(_load().oracle_lstm_step(_p(x), _p(h), _p(w), _p(b), _p(c), _p(h_out), _p(c_out),
                                    _p(g), B, Ix, H), "lstm_step")
    return h_out, c_out


def lstm_pre_shape(pre_shape, h_shape, c_shape, wh_shape):
    """Shape function of the cell whose input share of the gates is given (Section 3.2, the
    run-time type check): pre (B,4H), h (B,H), c (B,H), wh (4H,H) -> h' (B,H), c' (B,H)."""
    shapes = [tuple(int(v) for v in s) for s in (pre_shape, h_shape, c_shape, wh_shape)]
    if any(len(s) != 2 for s in shapes):
        raise OracleShapeError("lstm_pre_shape: wrong rank")
    if any(v < 0 for s in shapes for v in s):
        raise ValueError("lstm_pre_shape: negative extent")
    pre, h, c, wh = shapes
    B, H = h
    if pre != (B, 4 * H) or wh != (4 * H, H) or c != (B, H):
        raise OracleShapeError("pre must be (B,4H), wh (4H,H), c (B,H)")
    return (B, H), (B, H)


def lstm_seq_shape(pre_shape, h0_shape, c0_shape, wh_shape):
    """Shape function of a whole sequence of such steps (Section 3.2's run-time type check applied to
    the token loop): pre (T,B,4H), h0 (B,H), c0 (B,H), wh (4H,H) -> every h_t (T,B,H), final c (B,H)."""
    pre = tuple(int(v) for v in pre_shape)
    if len(pre) != 3:
        raise OracleShapeError("lstm_seq_shape: pre must have rank 3")
    if any(v < 0 for v in pre):
        raise ValueError("lstm_seq_shape: negative extent")
    (B, H), _ = lstm_pre_shape(pre[1:], h0_shape, c0_shape, wh_shape)
    return (pre[0], B, H), (B, H)


def lstm_step_pre(pre, h, wh, c) -> Tuple[np.ndarray, np.ndarray]:
    """One LSTM cell step from gates whose input share pre = x.Wx^T + b [B, 4H] was computed
    beforehand (for all tokens in one product); wh [4H, H] are the recurrent columns of the
    fused weight.  Returns (h', c')."""
    pre, h, wh, c = _f(pre), _f(h), _f(wh), _f(c)
    (B, H), _ = lstm_pre_shape(pre.shape, h.shape, c.shape, wh.shape)
    h_out = np.empty((B, H), dtype=np.float32)
    c_out = np.empty((B, H), dtype=np.float32)
    g = np.empty((B, 4 * H), dtype=np.float32)
    _check(_load().oracle_lstm_step_pre(_p(pre), _p(h), _p(wh), _p(c), _p(h_out), _p(c_out), _p(g), B, H),
           "lstm_step_pre")
    return h_out, c_out


# ------------------------------------------------------------------ integers
def dense_shape(x_shape: Sequence[int], w_shape: Sequence[int]) -> Tuple[int, int]:
    xs, ws = _shape_arr(x_shape), _shape_arr(w_shape)
    out = np.full(2, -1, dtype=np.int64)
    _check(_load().oracle_dense_shape(_ip(xs), len(xs), _ip(ws), len(ws), _ip(out)), "dense_shape")
    return int(out[0]), int(out[1])


def batch_matmul_shape(a_shape, b_shape, trans_b: bool) -> Tuple[int, int, int]:
    a, b = _shape_arr(a_shape), _shape_arr(b_shape)
    out = np.full(3, -1, dtype=np.int64)
    _check(_load().oracle_batch_matmul_shape(_ip(a), len(a), _ip(b), len(b), int(bool(trans_b)),
                                             _ip(out)), "batch_matmul_shape")
    return int(out[0]), int(out[1]), int(out[2])


def lstm_shape(x_shape, h_shape, c_shape, w_shape):
    arrs = [_shape_arr(s) for s in (x_shape, h_shape, c_shape, w_shape)]
    if any(len(a) != 2 for a in arrs):
        raise OracleShapeError("lstm_shape: wrong rank")
    ho = np.full(2, -1, dtype=np.int64)
    co = np.full(2, -1, dtype=np.int64)
    _check(_load().oracle_lstm_shape(*[_ip(a) for a in arrs], _ip(ho), _ip(co)), "lstm_shape")
    return (int(ho[0]), int(ho[1])), (int(co[0]), int(co[1]))


def storage_bytes(shape: Sequence[int], itemsize: int) -> int:
    s = _shape_arr(shape)
    n = int(_load().oracle_storage_bytes(_ip(s), len(s), itemsize))
    if n < 0:
        raise ValueError("storage_bytes: bad argument")
    return n


def residue_split(x: int, tile: int) -> Tuple[int, int]:
    k = np.zeros(1, dtype=np.int64)
    r = np.zeros(1, dtype=np.int64)
    _check(_load().oracle_residue_split(x, tile, _ip(k), _ip(r)), "residue_split")
    return int(k[0]), int(r[0])


def maxnorm_rel_error(got, ref) -> float:
    """max|got - ref| / max|ref| over one call's whole output (the infinity-norm companion of
    normwise_rel_error, reported beside it); zero reference: 0 when got is zero too, else inf."""
    got = np.asarray(got, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    if ref.size == 0:
        return 0.0
    den = float(np.max(np.abs(ref)))
    num = float(np.max(np.abs(got - ref)))
    if den == 0.0:
        return 0.0 if num == 0.0 else float("inf")
    return num / den


def elementwise_excess(got, ref, rel: float, floor: float) -> float:
    """Element-by-element gate beside the norms: the largest value over the output of
    |got - ref| / (rel * |ref| + floor * rms(ref)), so a result <= 1 means every single element is
    within rel of its reference value plus floor times the root mean square of the reference
    (the absolute term covers elements that cancel to near zero).  A zero reference allows only
    an exactly zero output (result 0, else inf)."""
    got = np.asarray(got, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    if ref.size == 0:
        return 0.0
    diff = np.abs(got - ref)
    rms = float(np.sqrt(np.mean(ref * ref)))
    if rms == 0.0:
        return 0.0 if float(np.max(diff)) == 0.0 else float("inf")
    allowed = rel * np.abs(ref) + floor * rms
    ratio = np.where(diff == 0.0, 0.0, diff / np.where(allowed > 0.0, allowed, 1.0))
    ratio = np.where((allowed <= 0.0) & (diff > 0.0), np.inf, ratio)   # nothing allowed, something off
    return float(np.max(ratio))


def normwise_rel_error(got, ref) -> float:
    """||got - ref||_F / ||ref||_F over one call's whole output; if the
    reference is identically zero the result is 0 when got is too, else inf."""
    got = np.asarray(got, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    den = np.linalg.norm(ref.ravel())
    num = np.linalg.norm((got - ref).ravel())
    if den == 0.0:
        return 0.0 if num == 0.0 else float("inf")
    return float(num / den)

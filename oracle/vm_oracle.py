"""Reference interpreter for the VM bytecode (paper Section 4: a dispatch loop that checks the
op-code, executes the instruction's logic and repeats; instruction meanings from Appendix C,
Table C.1).

TEST INFRASTRUCTURE ONLY, like the rest of ``oracle/``: imported by ``tests/`` and the smoke
check.  It shares nothing with the C++ interpreter in the HIP library: it decodes the int64 word
stream itself and runs the tensor instructions on numpy arrays through the CPU oracle kernels.

Word stream: one instruction is [opcode, n, operand * n]; jump operands are offsets in
instructions relative to the jumping instruction.  Tensors are float32 numpy arrays tagged with a
dtype; a kernel output whose tensor is tagged bf16 is rounded to bf16 (round to nearest even) when
it is written, which is where the GPU path rounds too.

Pinned by tests/test_vm_oracle.py: hand-written word streams with results worked out by hand
(loop counts, branch directions, shapes), agreement with direct calls of the oracle kernels, and
the error cases.
"""
from __future__ import annotations

from typing import List, Optional, Sequence

import numpy as np

import oracle

# Table C.1, in the order the interface numbers them
(MOVE, RET, IF, GOTO, LOAD_CONST, LOAD_CONSTI, ALLOC_STORAGE, ALLOC_TENSOR, ALLOC_TENSOR_REG,
 ALLOC_ADT, ALLOC_CLOSURE, FREE_STORAGE, FREE_TENSOR, INVOKE, INVOKE_CLOSURE, INVOKE_PACKED,
 GET_FIELD, GET_TAG, DEVICE_COPY, SHAPE_OF, RESHAPE_TENSOR, FATAL) = range(22)
(SHAPE_DENSE, SHAPE_LSTM, SHAPE_ATTENTION, STORAGE_BYTES, SHAPE_GET, INT_ADD, INT_LESS, INDEX0,
 DENSE, DENSE_BIAS, DENSE_BIAS_GELU, LSTM_GATES, ATTENTION) = range(13)
BF16, F32, I64 = 0, 1, 2
_ITEMSIZE = {BF16: 2, F32: 4, I64: 8}
_UNIMPLEMENTED = (ALLOC_CLOSURE, INVOKE, INVOKE_CLOSURE, DEVICE_COPY)


class VMError(RuntimeError):
    def __init__(self, kind: str, message: str):
        super().__init__(f"{kind}: {message}")
        self.kind = kind  # "ARG", "SHAPE", "WORKSPACE", "DTYPE", "RANK"


def round_bf16(a: np.ndarray) -> np.ndarray:
    """float32 -> nearest bfloat16 (ties to even), returned as float32."""
    u = np.ascontiguousarray(a, dtype=np.float32).view(np.uint32).astype(np.uint64)
    u = (u + 0x7FFF + ((u >> 16) & 1)) & 0xFFFF0000
    return u.astype(np.uint32).view(np.float32).reshape(np.shape(a))


class Storage:
    def __init__(self, nbytes: int, device: int):
        self.nbytes, self.device, self.freed = nbytes, device, False


class Tensor:
    def __init__(self, array: np.ndarray, dtype: int, storage: Optional[Storage] = None):
        self.array, self.dtype, self.storage = array, dtype, storage

    @property
    def on_host(self) -> bool:
        return self.dtype == I64


class ADT:
    def __init__(self, tag: int, fields: list):
        self.tag, self.fields = tag, fields


def decode(words: Sequence[int]) -> List[List[int]]:
    out, at = [], 0
    words = [int(w) for w in words]
    while at < len(words):
        if at + 2 > len(words):
            raise VMError("ARG", "truncated instruction")
        op, n = words[at], words[at + 1]
        if not 0 <= op < 22 or n < 0 or at + 2 + n > len(words):
            raise VMError("ARG", f"bad instruction at word {at}")
        out.append([op] + words[at + 2:at + 2 + n])
        at += 2 + n
    return out


def _int(v, what: str) -> int:
    if isinstance(v, (int, np.integer)) and not isinstance(v, bool):
        return int(v)
    if isinstance(v, Tensor) and v.on_host and v.array.size == 1:
        return int(v.array.reshape(-1)[0])
    raise VMError("ARG", f"{what} is not an integer")


def _gpu(v, what: str) -> Tensor:
    if not isinstance(v, Tensor) or v.on_host:
        raise VMError("ARG", f"{what} is not a GPU tensor")
    if v.storage is not None and v.storage.freed:
        raise VMError("ARG", f"{what} refers to freed storage")
    return v


def _shape(v, what: str) -> np.ndarray:
    if not isinstance(v, Tensor) or not v.on_host or v.array.ndim != 1 or v.array.size > 4:
        raise VMError("ARG", f"{what} is not a shape tensor")
    return v.array


def _write(out: Tensor, value: np.ndarray, want_shape, want_dtype: Optional[int] = None) -> None:
    if tuple(out.array.shape) != tuple(int(s) for s in want_shape):
        raise VMError("SHAPE", f"output tensor {out.array.shape} is not {tuple(want_shape)}")
    if want_dtype is not None and out.dtype != want_dtype:
        raise VMError("DTYPE", "output tensor has the wrong dtype")
    value = np.asarray(value, dtype=np.float32).reshape(out.array.shape)
    out.array[...] = round_bf16(value) if out.dtype == BF16 else value


def _shape_call(fn, *args):
    try:
        return fn(*args)
    except oracle.OracleShapeError as e:
        raise VMError("SHAPE", str(e))


def _invoke_packed(pf: int, regs: list, r: Sequence[int]) -> None:
    if pf == SHAPE_DENSE:
        out = _shape(regs[r[2]], "output")
        res = _shape_call(oracle.dense_shape, _shape(regs[r[0]], "x shape").tolist(), _shape(regs[r[1]], "w shape").tolist())
        if out.size != 2:
            raise VMError("ARG", "dense shape output must hold 2 extents")
        out[:] = res
    elif pf == SHAPE_LSTM:
        ins = [_shape(regs[r[i]], "shape").tolist() for i in range(4)]
        ho, co = _shape(regs[r[4]], "h' shape"), _shape(regs[r[5]], "c' shape")
        hs, cs = _shape_call(oracle.lstm_shape, *ins)
        if ho.size != 2 or co.size != 2:
            raise VMError("ARG", "lstm shape outputs must hold 2 extents")
        ho[:], co[:] = hs, cs
    elif pf == SHAPE_ATTENTION:
        q, k, v = (_shape(regs[r[i]], "shape").tolist() for i in range(3))
        out = _shape(regs[r[3]], "output")
        s = _shape_call(oracle.batch_matmul_shape, q, k, True)
        o = _shape_call(oracle.batch_matmul_shape, list(s), v, False)
        if out.size != 3:
            raise VMError("ARG", "attention shape output must hold 3 extents")
        out[:] = o
    elif pf == STORAGE_BYTES:
        dtype = _int(regs[r[1]], "dtype")
        if dtype not in _ITEMSIZE:
            raise VMError("DTYPE", "unknown dtype")
        regs[r[2]] = oracle.storage_bytes(_shape(regs[r[0]], "shape").tolist(), _ITEMSIZE[dtype])
    elif pf == SHAPE_GET:
        s, i = _shape(regs[r[0]], "shape"), _int(regs[r[1]], "index")
        if not 0 <= i < s.size:
            raise VMError("ARG", "extent index out of range")
        regs[r[2]] = int(s[i])
    elif pf == INT_ADD:
        regs[r[2]] = _int(regs[r[0]], "a") + _int(regs[r[1]], "b")
    elif pf == INT_LESS:
        regs[r[2]] = 1 if _int(regs[r[0]], "a") < _int(regs[r[1]], "b") else 0
    elif pf == INDEX0:
        t, i = _gpu(regs[r[0]], "tensor"), _int(regs[r[1]], "index")
        if t.array.ndim < 1 or not 0 <= i < t.array.shape[0]:
            raise VMError("ARG", "slice index out of range")
        regs[r[2]] = Tensor(t.array[i], t.dtype, t.storage)
    elif pf in (DENSE, DENSE_BIAS, DENSE_BIAS_GELU):
        has_bias = pf != DENSE
        x, w = _gpu(regs[r[0]], "x"), _gpu(regs[r[1]], "w")
        b = _gpu(regs[r[2]], "bias") if has_bias else None
        y = _gpu(regs[r[3 if has_bias else 2]], "y")
        M, N = _shape_call(oracle.dense_shape, x.array.shape, w.array.shape)
        if x.dtype != BF16 or w.dtype != BF16 or (b is not None and b.dtype != BF16):
            raise VMError("DTYPE", "dense operands must be bf16")
        if b is not None and b.array.shape != (N,):
            raise VMError("SHAPE", "bias is not [N]")
        epi = {DENSE: "none", DENSE_BIAS: "bias", DENSE_BIAS_GELU: "bias_gelu"}[pf]
        if tuple(y.array.shape) != (M, N):
            raise VMError("SHAPE", "output is not [M,N]")
        res = oracle.dense(x.array, w.array, None if b is None else b.array, epi) if M and N else np.zeros((M, N), np.float32)
        _write(y, res, (M, N))
    elif pf == LSTM_GATES:
        x, h, w, b, c, co, ho = (_gpu(regs[r[i]], "operand") for i in range(7))
        if any(t.array.ndim != 2 for t in (x, h, c, w)):
            raise VMError("RANK", "lstm operands must have rank 2")
        hs, cs = _shape_call(oracle.lstm_shape, x.array.shape, h.array.shape, c.array.shape, w.array.shape)
        if (x.dtype, h.dtype, w.dtype, b.dtype, c.dtype, co.dtype, ho.dtype) != (BF16, BF16, BF16, BF16, F32, F32, BF16):
            raise VMError("DTYPE", "lstm_gates dtypes")
        if b.array.shape != (w.array.shape[0],):
            raise VMError("SHAPE", "bias is not [4H]")
        if tuple(ho.array.shape) != tuple(hs) or tuple(co.array.shape) != tuple(cs):
            raise VMError("SHAPE", "outputs are not [B,H]")
        if hs[0] and hs[1]:
            h_new, c_new = oracle.lstm_step(x.array, h.array, w.array, b.array, c.array)
            _write(co, c_new, cs)
            _write(ho, h_new, hs)
    elif pf == ATTENTION:
        q, k, v, o = (_gpu(regs[r[i]], "operand") for i in range(4))
        if any(t.dtype != BF16 for t in (q, k, v, o)):
            raise VMError("DTYPE", "attention operands must be bf16")
        s = _shape_call(oracle.batch_matmul_shape, q.array.shape, k.array.shape, True)
        os_ = _shape_call(oracle.batch_matmul_shape, s, v.array.shape, False)
        if s[1] != s[2]:
            raise VMError("SHAPE", "q and k lengths differ")
        if tuple(o.array.shape) != tuple(os_):
            raise VMError("SHAPE", "output is not [T,L,D]")
        if all(os_):
            D = q.array.shape[2]
            _, _, res = oracle.attention(q.array, k.array, v.array, float(np.float32(1.0) / np.sqrt(np.float32(D))))
            _write(o, res, os_)
    else:
        raise VMError("ARG", f"unknown packed function {pf}")


def run(words: Sequence[int], n_registers: int, constants: Sequence[Tensor], inputs: Sequence[Tensor],
        max_instructions: int = 10_000_000):
    """Execute the function; returns (result object, number of instructions executed).  A result is
    an int, a Tensor, or an ADT of those."""
    code = decode(words)
    for ins in code:
        if ins[0] in _UNIMPLEMENTED:
            raise VMError("ARG", "instruction not implemented")
    regs: list = [None] * n_registers
    for i, t in enumerate(inputs):
        regs[i] = t
    pc, executed = 0, 0
    while True:
        if executed >= max_instructions:
            raise VMError("ARG", "instruction limit reached")
        executed += 1
        if not 0 <= pc < len(code):
            raise VMError("ARG", "pc outside the function")
        op, a = code[pc][0], code[pc][1:]
        nxt = pc + 1
        if op == MOVE:
            regs[a[1]] = regs[a[0]]
        elif op == RET:
            return regs[a[0]], executed
        elif op == IF:
            nxt = pc + (a[2] if _int(regs[a[0]], "test") == _int(regs[a[1]], "target") else a[3])
        elif op == GOTO:
            nxt = pc + a[0]
        elif op == LOAD_CONST:
            regs[a[1]] = constants[a[0]]
        elif op == LOAD_CONSTI:
            regs[a[1]] = int(a[0])
        elif op == ALLOC_STORAGE:
            size = _int(regs[a[0]], "size")
            if size < 0:
                raise VMError("ARG", "negative storage size")
            regs[a[3]] = Storage(size, a[2])
        elif op in (ALLOC_TENSOR, ALLOC_TENSOR_REG):
            st = regs[a[0]]
            if not isinstance(st, Storage) or st.freed:
                raise VMError("ARG", "not a live storage")
            if op == ALLOC_TENSOR:
                dtype, shape, dst = a[2], list(a[4:4 + a[3]]), a[4 + a[3]]
            else:
                dtype, shape, dst = a[3], _shape(regs[a[2]], "shape").tolist(), a[4]
            if any(s < 0 for s in shape):
                raise VMError("ARG", "negative extent")
            need = int(np.prod(shape, dtype=np.int64)) * _ITEMSIZE[dtype] if shape else _ITEMSIZE[dtype]
            if a[1] + need > st.nbytes:
                raise VMError("WORKSPACE", "tensor does not fit its storage")
            if (st.device == 0) != (dtype == I64):
                raise VMError("DTYPE", "host storage holds shape tensors, GPU storage the others")
            arr = np.zeros(shape, dtype=np.int64 if dtype == I64 else np.float32)
            regs[dst] = Tensor(arr, dtype, st)
        elif op == ALLOC_ADT:
            fields = [regs[x] for x in a[2:2 + a[1]]]
            if any(f is None for f in fields):
                raise VMError("ARG", "empty register in an ADT")
            regs[a[2 + a[1]]] = ADT(a[0], fields)
        elif op == FREE_STORAGE:
            if not isinstance(regs[a[0]], Storage):
                raise VMError("ARG", "not a storage")
            regs[a[0]].freed = True
        elif op == FREE_TENSOR:
            if not isinstance(regs[a[0]], Tensor):
                raise VMError("ARG", "not a tensor")
            regs[a[0]] = None
        elif op == INVOKE_PACKED:
            _invoke_packed(a[0], regs, a[3:3 + a[1]])
        elif op == GET_FIELD:
            if not isinstance(regs[a[0]], ADT) or not 0 <= a[1] < len(regs[a[0]].fields):
                raise VMError("ARG", "bad field access")
            regs[a[2]] = regs[a[0]].fields[a[1]]
        elif op == GET_TAG:
            if not isinstance(regs[a[0]], ADT):
                raise VMError("ARG", "not an ADT")
            regs[a[1]] = int(regs[a[0]].tag)
        elif op == SHAPE_OF:
            if not isinstance(regs[a[0]], Tensor):
                raise VMError("ARG", "not a tensor")
            regs[a[1]] = Tensor(np.array(regs[a[0]].array.shape, dtype=np.int64), I64)
        elif op == RESHAPE_TENSOR:
            t = regs[a[0]]
            if not isinstance(t, Tensor):
                raise VMError("ARG", "not a tensor")
            shape = _shape(regs[a[1]], "shape").tolist()
            if any(s < 0 for s in shape) or int(np.prod(shape, dtype=np.int64)) != t.array.size:
                raise VMError("SHAPE", "reshape changes the element count")
            regs[a[2]] = Tensor(t.array.reshape(shape), t.dtype, t.storage)
        elif op == FATAL:
            raise VMError("SHAPE", "Fatal")
        pc = nxt


def flatten(obj) -> list:
    """Result object -> flat list (an ADT contributes its fields in order)."""
    if isinstance(obj, ADT):
        out = []
        for f in obj.fields:
            out += flatten(f)
        return out
    return [obj]

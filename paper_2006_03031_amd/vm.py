"""Bytecode assembler and ctypes wrapper for the interpreter declared in ``include/nimble_vm.h``.

The paper runs a dynamic model as bytecode on a register VM with coarse instructions (Section 4,
Appendix C).  This module writes such bytecode by hand for the programs the dynamic-shape path is
measured on - the LSTM token loop, a transformer feed-forward block, an attention head group -
following the pattern of the listing in Appendix A: shape_of, shape function, alloc_storage,
alloc_tensor from the computed shape, invoke_mut.  The interpreter itself is C++ in the library.
"""
from __future__ import annotations

import ctypes
from typing import Dict, List, Optional, Sequence, Union

import torch

from . import binding as nb
from . import runtime as rt

# opcodes (Table C.1 order, values of nimble_vm_opcode)
(OP_MOVE, OP_RET, OP_IF, OP_GOTO, OP_LOAD_CONST, OP_LOAD_CONSTI, OP_ALLOC_STORAGE, OP_ALLOC_TENSOR,
 OP_ALLOC_TENSOR_REG, OP_ALLOC_ADT, OP_ALLOC_CLOSURE, OP_FREE_STORAGE, OP_FREE_TENSOR, OP_INVOKE,
 OP_INVOKE_CLOSURE, OP_INVOKE_PACKED, OP_GET_FIELD, OP_GET_TAG, OP_DEVICE_COPY, OP_SHAPE_OF,
 OP_RESHAPE_TENSOR, OP_FATAL) = range(22)
OP_NAMES = ["Move", "Ret", "If", "Goto", "LoadConst", "LoadConsti", "AllocStorage", "AllocTensor",
            "AllocTensorReg", "AllocADT", "AllocClosure", "FreeStorage", "FreeTensor", "Invoke",
            "InvokeClosure", "InvokePacked", "GetField", "GetTag", "DeviceCopy", "ShapeOf",
            "ReshapeTensor", "Fatal"]
# packed functions (values of nimble_vm_packed)
(PF_SHAPE_DENSE, PF_SHAPE_LSTM, PF_SHAPE_ATTENTION, PF_STORAGE_BYTES, PF_SHAPE_GET, PF_INT_ADD,
 PF_INT_LESS, PF_INDEX0, PF_DENSE, PF_DENSE_BIAS, PF_DENSE_BIAS_GELU, PF_LSTM_GATES, PF_ATTENTION) = range(13)
PF_NAMES = ["shape_dense", "shape_lstm", "shape_attention", "storage_bytes", "shape_get", "int_add",
            "int_less", "index0", "dense", "dense_bias", "dense_bias_gelu", "lstm_gates", "attention"]
I64 = 2
HOST, GPU = 0, 1
ALIGN = 64


class Assembler:
    """Writes the int64 word stream: [opcode, n, operand * n] per instruction.  Jumps are given as
    label names and resolved to offsets relative to the jumping instruction."""

    def __init__(self, n_inputs: int):
        self.n_regs = n_inputs
        self.instrs: List[List[Union[int, str]]] = []
        self.labels: Dict[str, int] = {}

    def reg(self) -> int:
        self.n_regs += 1
        return self.n_regs - 1

    def label(self, name: str) -> None:
        self.labels[name] = len(self.instrs)

    def _emit(self, op: int, *operands) -> None:
        self.instrs.append([op, *operands])

    # one method per instruction; those that produce a value return its register
    def move(self, src: int, dst: int) -> None:
        self._emit(OP_MOVE, src, dst)

    def ret(self, r: int) -> None:
        self._emit(OP_RET, r)

    def if_equal(self, test: int, target: int, true_label: str, false_label: str) -> None:
        self._emit(OP_IF, test, target, true_label, false_label)

    def goto(self, label: str) -> None:
        self._emit(OP_GOTO, label)

    def load_const(self, index: int) -> int:
        d = self.reg()
        self._emit(OP_LOAD_CONST, index, d)
        return d

    def load_consti(self, value: int) -> int:
        d = self.reg()
        self._emit(OP_LOAD_CONSTI, value, d)
        return d

    def alloc_storage(self, size_reg: int, device: int, alignment: int = ALIGN) -> int:
        d = self.reg()
        self._emit(OP_ALLOC_STORAGE, size_reg, alignment, device, d)
        return d

    def alloc_tensor(self, storage: int, offset: int, dtype: int, shape: Sequence[int]) -> int:
        d = self.reg()
        self._emit(OP_ALLOC_TENSOR, storage, offset, dtype, len(shape), *shape, d)
        return d

    def alloc_tensor_reg(self, storage: int, offset: int, shape_reg: int, dtype: int) -> int:
        d = self.reg()
        self._emit(OP_ALLOC_TENSOR_REG, storage, offset, shape_reg, dtype, d)
        return d

    def alloc_adt(self, tag: int, fields: Sequence[int]) -> int:
        d = self.reg()
        self._emit(OP_ALLOC_ADT, tag, len(fields), *fields, d)
        return d

    def free_storage(self, r: int) -> None:
        self._emit(OP_FREE_STORAGE, r)

    def free_tensor(self, r: int) -> None:
        self._emit(OP_FREE_TENSOR, r)

    def invoke_packed(self, packed: int, inputs: Sequence[int], outputs: Sequence[int]) -> None:
        self._emit(OP_INVOKE_PACKED, packed, len(inputs) + len(outputs), len(outputs), *inputs, *outputs)

    def get_field(self, obj: int, index: int) -> int:
        d = self.reg()
        self._emit(OP_GET_FIELD, obj, index, d)
        return d

    def get_tag(self, obj: int) -> int:
        d = self.reg()
        self._emit(OP_GET_TAG, obj, d)
        return d

    def shape_of(self, tensor: int) -> int:
        d = self.reg()
        self._emit(OP_SHAPE_OF, tensor, d)
        return d

    def reshape_tensor(self, tensor: int, shape_reg: int) -> int:
        d = self.reg()
        self._emit(OP_RESHAPE_TENSOR, tensor, shape_reg, d)
        return d

    def fatal(self) -> None:
        self._emit(OP_FATAL)

    # --- composites used by every program below
    def host_shape_tensor(self, bytes_reg: int, rank: int) -> int:
        """alloc_storage(16, 64, cpu) + alloc_tensor(storage, (rank,), int64): the buffer a shape
        function writes its result to."""
        st = self.alloc_storage(bytes_reg, HOST)
        return self.alloc_tensor(st, 0, I64, [rank])

    def gpu_tensor_from_shape(self, shape_reg: int, dtype: int, dtype_reg: int) -> int:
        """storage_bytes(shape) -> alloc_storage on the GPU pool -> alloc_tensor with the shape
        held in a register."""
        nbytes = self.reg()
        self.invoke_packed(PF_STORAGE_BYTES, [shape_reg, dtype_reg], [nbytes])
        buf = self.alloc_storage(nbytes, GPU)
        return self.alloc_tensor_reg(buf, 0, shape_reg, dtype)

    def words(self) -> List[int]:
        out: List[int] = []
        for pc, ins in enumerate(self.instrs):
            ops = [(self.labels[o] - pc) if isinstance(o, str) else int(o) for o in ins[1:]]
            out += [ins[0], len(ops), *ops]
        return out


# ----------------------------------------------------------------------------- programs
def lstm_sequence_program() -> Assembler:
    """inputs: xs [T,B,Ix] bf16, h0 [B,H] bf16, c0 [B,H] f32; constants: W [4H,Ix+H], b [4H].
    Loops t = 0..T-1 over the tokens (T and B are only known from the input), allocating the
    new state from the shape function's result each step; returns the tuple (h_T, c_T)."""
    a = Assembler(3)
    xs, h0, c0 = 0, 1, 2
    w, b = a.load_const(0), a.load_const(1)
    zero, one = a.load_consti(0), a.load_consti(1)
    bf16, f32 = a.load_consti(nb.BF16), a.load_consti(nb.F32)
    sixteen = a.load_consti(16)  # bytes of a rank-2 int64 shape tensor
    sh_xs = a.shape_of(xs)
    T = a.reg()
    a.invoke_packed(PF_SHAPE_GET, [sh_xs, zero], [T])
    sh_w = a.shape_of(w)
    t, h, c = a.reg(), a.reg(), a.reg()
    a.move(zero, t)
    a.move(h0, h)
    a.move(c0, c)
    a.label("loop")
    a.if_equal(t, T, "exit", "body")
    a.label("body")
    x_t = a.reg()
    a.invoke_packed(PF_INDEX0, [xs, t], [x_t])
    sh_x, sh_h, sh_c = a.shape_of(x_t), a.shape_of(h), a.shape_of(c)
    out_h, out_c = a.host_shape_tensor(sixteen, 2), a.host_shape_tensor(sixteen, 2)
    a.invoke_packed(PF_SHAPE_LSTM, [sh_x, sh_h, sh_c, sh_w], [out_h, out_c])
    h_new = a.gpu_tensor_from_shape(out_h, nb.BF16, bf16)
    c_new = a.gpu_tensor_from_shape(out_c, nb.F32, f32)
    a.invoke_packed(PF_LSTM_GATES, [x_t, h, w, b, c], [c_new, h_new])
    a.move(h_new, h)
    a.move(c_new, c)
    a.invoke_packed(PF_INT_ADD, [t, one], [t])
    a.goto("loop")
    a.label("exit")
    a.ret(a.alloc_adt(0, [h, c]))
    return a


def ffn_block_program() -> Assembler:
    """input: x [M,K] bf16; constants: W1 [N1,K], b1 [N1], W2 [N2,N1], b2 [N2].
    y = dense_bias(dense_bias_gelu(x, W1, b1), W2, b2) with M known only at run time."""
    a = Assembler(1)
    x = 0
    w1, b1, w2, b2 = (a.load_const(i) for i in range(4))
    bf16 = a.load_consti(nb.BF16)
    sixteen = a.load_consti(16)
    cur = x
    for w, b, pf in ((w1, b1, PF_DENSE_BIAS_GELU), (w2, b2, PF_DENSE_BIAS)):
        sh_in, sh_w = a.shape_of(cur), a.shape_of(w)
        out_sh = a.host_shape_tensor(sixteen, 2)
        a.invoke_packed(PF_SHAPE_DENSE, [sh_in, sh_w], [out_sh])
        y = a.gpu_tensor_from_shape(out_sh, nb.BF16, bf16)
        a.invoke_packed(pf, [cur, w, b], [y])
        cur = y
    a.ret(cur)
    return a


def attention_program() -> Assembler:
    """inputs: q, k, v [heads,L,D] bf16 with L known only at run time; returns o [heads,L,D]."""
    a = Assembler(3)
    bf16 = a.load_consti(nb.BF16)
    nbytes = a.load_consti(24)  # rank-3 int64 shape tensor
    shapes = [a.shape_of(r) for r in (0, 1, 2)]
    out_sh = a.host_shape_tensor(nbytes, 3)
    a.invoke_packed(PF_SHAPE_ATTENTION, shapes, [out_sh])
    o = a.gpu_tensor_from_shape(out_sh, nb.BF16, bf16)
    a.invoke_packed(PF_ATTENTION, [0, 1, 2], [o])
    a.ret(o)
    return a


# ----------------------------------------------------------------------------- wrapper
class _CVmTensor(ctypes.Structure):
    _fields_ = [("data", ctypes.c_void_p), ("dtype", ctypes.c_int32), ("rank", ctypes.c_int32),
                ("shape", ctypes.c_int64 * 4)]


_TORCH_TO_DTYPE = {torch.bfloat16: nb.BF16, torch.float32: nb.F32}
_DTYPE_TO_TORCH = {nb.BF16: torch.bfloat16, nb.F32: torch.float32}
_ITEMSIZE = {nb.BF16: 2, nb.F32: 4}
_MAX_RESULTS = 16


def _prototypes(lib) -> None:
    if getattr(lib, "_vm_ready", False):
        return
    i64, i32, vp, u64 = ctypes.c_int64, ctypes.c_int, ctypes.c_void_p, ctypes.c_uint64
    ip = ctypes.POINTER(ctypes.c_int64)
    tp = ctypes.POINTER(_CVmTensor)
    lib.nimble_vm_create.argtypes = [ip, i64, i64, tp, i32, ctypes.POINTER(vp)]
    lib.nimble_vm_destroy.argtypes = [vp]
    lib.nimble_vm_destroy.restype = None
    lib.nimble_vm_run.argtypes = [vp, tp, i32, vp, u64, vp, u64, vp, i64, tp, i32, ctypes.POINTER(i32)]
    lib.nimble_vm_profile.argtypes = [vp, ip, ip, ip, ip, ctypes.POINTER(u64), ip, ip]
    lib._vm_ready = True


class TensorDesc:
    """A tensor given by address and metadata instead of a torch tensor (what the C ABI takes)."""

    def __init__(self, data_ptr: int, shape: Sequence[int], dtype: int):
        self.ptr, self.shape, self.dtype = int(data_ptr), tuple(int(s) for s in shape), int(dtype)

    def nbytes(self) -> int:
        n = _ITEMSIZE[self.dtype]
        for s in self.shape:
            n *= s
        return n


def _describe(t) -> _CVmTensor:
    if isinstance(t, TensorDesc):
        d = _CVmTensor()
        d.data, d.dtype, d.rank = t.ptr, t.dtype, len(t.shape)
        for i, s in enumerate(t.shape[:4]):
            d.shape[i] = s
        return d
    if t.dtype not in _TORCH_TO_DTYPE:
        raise TypeError(f"the VM takes bf16 and f32 tensors, got {t.dtype}")
    if not t.is_contiguous():
        raise ValueError("the VM takes contiguous tensors")
    d = _CVmTensor()
    d.data = t.data_ptr()
    d.dtype = _TORCH_TO_DTYPE[t.dtype]
    d.rank = t.dim()
    for i, s in enumerate(t.shape):
        d.shape[i] = s
    return d


class Executable:
    """A loaded program: bytecode + register count + constant pool (weights stay where the caller
    put them; the executable keeps references so they outlive it)."""

    def __init__(self, code: Sequence[int], n_registers: int, constants: Sequence[torch.Tensor] = ()):
        self._lib = nb.load()
        _prototypes(self._lib)
        self._constants = list(constants)
        words = (ctypes.c_int64 * max(len(code), 1))(*[int(w) for w in code])
        consts = (_CVmTensor * max(len(self._constants), 1))(*[_describe(c) for c in self._constants])
        handle = ctypes.c_void_p()
        rc = self._lib.nimble_vm_create(words, len(code), n_registers, consts, len(self._constants),
                                        ctypes.byref(handle))
        if rc != 0:
            raise nb.NimbleError(rc, nb.last_error())
        self._handle = handle
        self._results = (_CVmTensor * _MAX_RESULTS)()
        self._n_results = ctypes.c_int(0)

    @classmethod
    def from_assembler(cls, asm: Assembler, constants: Sequence[torch.Tensor] = ()) -> "Executable":
        return cls(asm.words(), asm.n_regs, constants)

    def __del__(self):
        h, self._handle = getattr(self, "_handle", None), None
        if h:
            self._lib.nimble_vm_destroy(h)

    def run(self, inputs: Sequence, pool,
            workspace: Optional[torch.Tensor] = None, max_instructions: int = 0) -> list:
        """Execute once on torch's current stream.  `pool` is a uint8 GPU tensor the program's
        AllocStorage instructions carve up (None for programs that allocate nothing on the GPU);
        tensor results are views into it (or the input/constant they alias) and stay valid until the
        next run with the same pool.  Integers come back as int, shape tensors as lists of int."""
        ins = (_CVmTensor * max(len(inputs), 1))(*[_describe(t) for t in inputs])
        on_gpu = isinstance(pool, torch.Tensor) or any(isinstance(t, torch.Tensor) for t in inputs)
        if isinstance(pool, TensorDesc):  # address arithmetic only (programs that launch nothing)
            pool_ptr, pool_bytes = pool.ptr, pool.nbytes()
        else:
            pool_ptr = pool.data_ptr() if pool is not None else 0
            pool_bytes = pool.numel() * pool.element_size() if pool is not None else 0
        if workspace is None and isinstance(pool, torch.Tensor):
            workspace = rt.default_workspace(pool.device)
        ws_ptr = workspace.data_ptr() if workspace is not None else 0
        ws_bytes = workspace.numel() * workspace.element_size() if workspace is not None else 0
        stream = rt._stream() if on_gpu else 0
        rc = self._lib.nimble_vm_run(self._handle, ins, len(inputs), pool_ptr, pool_bytes, ws_ptr, ws_bytes,
                                     stream, max_instructions, self._results, _MAX_RESULTS,
                                     ctypes.byref(self._n_results))
        if rc != 0:
            raise nb.NimbleError(rc, nb.last_error())
        return [self._to_python(self._results[i], inputs, pool) for i in range(self._n_results.value)]

    def _to_python(self, d: _CVmTensor, inputs: Sequence[torch.Tensor], pool: Optional[torch.Tensor]):
        if d.dtype == I64:
            if d.rank == 0:
                return int(d.shape[0])
            n = int(d.shape[0])
            return list((ctypes.c_int64 * n).from_address(d.data)) if n else []
        shape = tuple(int(d.shape[i]) for i in range(d.rank))
        nbytes = _ITEMSIZE[d.dtype]
        for s in shape:
            nbytes *= s
        owners = ([pool] if pool is not None else []) + list(inputs) + self._constants
        for owner in owners:
            if isinstance(owner, TensorDesc):
                if owner.ptr <= (d.data or 0) and (d.data or 0) + nbytes <= owner.ptr + owner.nbytes():
                    return TensorDesc(d.data or 0, shape, d.dtype)
                continue
            lo = owner.data_ptr()
            hi = lo + owner.numel() * owner.element_size()
            if lo <= (d.data or 0) and (d.data or 0) + nbytes <= hi:
                flat = owner.view(-1).view(torch.uint8)[d.data - lo:d.data - lo + nbytes]
                return flat.view(_DTYPE_TO_TORCH[d.dtype]).view(shape)
        raise RuntimeError("the VM returned a tensor outside the pool, the inputs and the constants")

    def profile(self) -> dict:
        """Host-side cost of the last run: per opcode and per packed function (count, ns), plus the
        pool statistics."""
        oc, on = (ctypes.c_int64 * len(OP_NAMES))(), (ctypes.c_int64 * len(OP_NAMES))()
        pc, pn = (ctypes.c_int64 * len(PF_NAMES))(), (ctypes.c_int64 * len(PF_NAMES))()
        hw, allocs, reuses = ctypes.c_uint64(0), ctypes.c_int64(0), ctypes.c_int64(0)
        rc = self._lib.nimble_vm_profile(self._handle, oc, on, pc, pn, ctypes.byref(hw), ctypes.byref(allocs),
                                         ctypes.byref(reuses))
        if rc != 0:
            raise nb.NimbleError(rc, nb.last_error())
        return {
            "opcodes": {OP_NAMES[i]: (oc[i], on[i]) for i in range(len(OP_NAMES)) if oc[i]},
            "packed": {PF_NAMES[i]: (pc[i], pn[i]) for i in range(len(PF_NAMES)) if pc[i]},
            "instructions": sum(oc), "host_ns": sum(on),
            "pool_high_water": hw.value, "storage_allocs": allocs.value, "storage_reuses": reuses.value,
        }

"""Caller-side sequence for one dynamic operator, on torch tensors.

For every operator this is the order the paper gives for a tensor whose
leading dimension is unknown until run time (Section 3.2, Section 3.3,
Appendix A): read the run-time shapes (host metadata, no device sync), run the
shape function, allocate the output from the shape it returns, then invoke the
kernel with inputs and outputs passed explicitly.  torch supplies device memory
and the stream; all arithmetic runs in the HIP library.
"""
from __future__ import annotations

from typing import Optional, Tuple

import torch

from . import binding as nb

_TORCH_DTYPE = {nb.BF16: torch.bfloat16, nb.F32: torch.float32}


try:  # raw handle of torch's current stream without building a Stream object (several us cheaper)
    _raw_stream = torch._C._cuda_getCurrentRawStream
except AttributeError:  # pragma: no cover - older torch
    _raw_stream = None


def _stream() -> int:
    if _raw_stream is not None:
        return _raw_stream(torch.cuda.current_device())
    return torch.cuda.current_stream().cuda_stream


class StorageArena:
    """One backing storage allocated up front, tensors carved out of it at offsets computed
    from the shape function's result: alloc_storage once, then alloc_tensor(storage, offset,
    shape, dtype) per operator (Section 3.3, storage coalescing).  `reset()` rewinds the
    offset; the caller does that once per inference when the previous outputs are dead."""

    def __init__(self, capacity_bytes: int, device="cuda"):
        self.alignment = max(256, nb.storage_alignment())
        self.storage = torch.empty(int(capacity_bytes) + self.alignment, dtype=torch.uint8, device=device)
        base = self.storage.data_ptr()
        self._base_off = (-base) % self.alignment
        self.capacity = int(capacity_bytes)
        self.offset = 0
        # tensors already carved at (offset, shape, dtype): a request that repeats (the same run-time
        # shape at the same place of the same request sequence) gets the same view back instead of
        # three new Python tensor objects, which is what an allocation from the arena would otherwise cost
        self._views = {}

    def reset(self) -> None:
        self.offset = 0

    def alloc(self, shape, dtype: int) -> torch.Tensor:
        key = (self.offset, tuple(shape), dtype)
        hit = self._views.get(key)
        if hit is not None:
            self.offset = hit[1]
            return hit[0]
        nbytes = nb.storage_bytes(shape, dtype)
        start = (self.offset + self.alignment - 1) // self.alignment * self.alignment
        if start + nbytes > self.capacity:
            raise MemoryError(f"arena of {self.capacity} bytes cannot hold {nbytes} more at offset {start}")
        flat = self.storage[self._base_off + start:self._base_off + start + nbytes]
        t = flat.view(_TORCH_DTYPE[dtype]).view(tuple(shape))
        if len(self._views) >= 4096:
            self._views.clear()
        self._views[key] = (t, start + nbytes)
        self.offset = start + nbytes
        return t


_WORKSPACE = {}
WORKSPACE_BYTES = 64 << 20


def default_workspace(device) -> torch.Tensor:
    """Caller-owned scratch handed to every dense call (the library never allocates): holds the
    f32 partial sums when the dispatch function cuts K.  One per device, shared by the calls on
    one stream; calls that overlap on different streams must bring their own."""
    key = str(device)
    ws = _WORKSPACE.get(key)
    if ws is None:
        ws = torch.empty(WORKSPACE_BYTES, dtype=torch.uint8, device=device)
        _WORKSPACE[key] = ws
    return ws


def _ptr(t: torch.Tensor, dtype, what: str) -> int:
    """Device address of a tensor the C ABI can take as a plain pointer: contiguous, on the GPU and
    of the element type the entry point reads; anything else is refused here (the library sees only
    an address and would read a strided view or another dtype as packed data)."""
    if t.dtype is not dtype or not t.is_cuda or not t.is_contiguous():
        raise nb.NimbleError(-4 if t.dtype is not dtype else -8,
                             f"{what}: need a contiguous {dtype} tensor on the GPU, got {t.dtype}, "
                             f"device {t.device}, strides {tuple(t.stride())}")
    return t.data_ptr()


_BF, _F32 = torch.bfloat16, torch.float32


def _alloc(shape, dtype: int, device) -> torch.Tensor:
    # alloc_storage(size, alignment, device) + alloc_tensor(storage, 0, shape, dtype):
    # torch's caching allocator returns storage aligned to at least 512 bytes.
    nb.storage_bytes(shape, dtype)  # validates the size computation
    return torch.empty(tuple(shape), dtype=_TORCH_DTYPE[dtype], device=device)


def dense(x: torch.Tensor, w: torch.Tensor, bias: Optional[torch.Tensor], epilogue: int = nb.EPI_BIAS,
          out_dtype: int = nb.BF16, force_variant: int = nb.VAR_AUTO,
          out: Optional[torch.Tensor] = None, arena: Optional[StorageArena] = None,
          workspace: Optional[torch.Tensor] = None) -> torch.Tensor:
    M, N = nb.nimble_dense_shape(tuple(x.shape), tuple(w.shape))
    K = x.shape[1]
    if out is not None:
        y = out
        if tuple(y.shape) != (M, N):
            raise nb.NimbleError(-3, f"dense: out is {tuple(y.shape)}, the shape function gives {(M, N)}")
    elif arena is not None:
        y = arena.alloc((M, N), out_dtype)
    else:
        y = _alloc((M, N), out_dtype, x.device)
    ws = workspace if workspace is not None else default_workspace(x.device)
    px, pw = _ptr(x, _BF, "x"), _ptr(w, _BF, "w")
    pb = _ptr(bias, _BF, "bias") if bias is not None else 0
    if bias is not None and bias.numel() != N:
        raise nb.NimbleError(-3, f"dense: bias has {bias.numel()} elements, N is {N}")
    py = _ptr(y, _TORCH_DTYPE[out_dtype], "y")
    if force_variant == nb.VAR_AUTO:
        nb.nimble_dense_dyn(px, pw, pb, py, M, N, K, epilogue, out_dtype, ws.data_ptr(),
                            ws.numel() * ws.element_size(), _stream())
    else:   # ablation, tuning and the per-variant tests pin one member of the kernel family
        nb.nimble_dense_variant_dyn(px, pw, pb, py, M, N, K, epilogue, out_dtype, force_variant, ws.data_ptr(),
                                    ws.numel() * ws.element_size(), _stream())
    return y


def batch_matmul(a: torch.Tensor, b: torch.Tensor, trans_b: bool, alpha: float = 1.0,
                 out_dtype: int = nb.BF16, out: Optional[torch.Tensor] = None,
                 workspace: Optional[torch.Tensor] = None) -> torch.Tensor:
    T, M, N = nb.batch_matmul_shape(tuple(a.shape), tuple(b.shape), trans_b)
    K = a.shape[2]
    c = out if out is not None else _alloc((T, M, N), out_dtype, a.device)
    ws = workspace if workspace is not None else default_workspace(a.device)   # b transposed, for the NN product
    nb.nimble_batch_matmul_dyn(_ptr(a, _BF, "a"), _ptr(b, _BF, "b"), _ptr(c, _TORCH_DTYPE[out_dtype], "c"), T, M, N, K,
                               trans_b, alpha, out_dtype, ws.data_ptr(), ws.numel() * ws.element_size(), _stream())
    return c


def softmax_rows(s: torch.Tensor, out: Optional[torch.Tensor] = None) -> torch.Tensor:
    cols = s.shape[-1]
    rows = s.numel() // cols if cols else 0
    p = out if out is not None else _alloc(tuple(s.shape), nb.BF16, s.device)
    nb.nimble_softmax_rows_dyn(_ptr(s, _F32, "s"), _ptr(p, _BF, "p"), rows, cols, _stream())
    return p


def attention(q: torch.Tensor, k: torch.Tensor, v: torch.Tensor,
              alpha: float = 0.125) -> Tuple[torch.Tensor, torch.Tensor, torch.Tensor]:
    """S = alpha Q.K^T (f32), P = softmax rows (bf16), O = P.V (bf16)."""
    s = batch_matmul(q, k, True, alpha, nb.F32)
    p = softmax_rows(s)
    o = batch_matmul(p, v, False, 1.0, nb.BF16)
    return s, p, o


def fused_attention(q: torch.Tensor, k: torch.Tensor, v: torch.Tensor, alpha: float = 0.125,
                    out: Optional[torch.Tensor] = None) -> torch.Tensor:
    """O = softmax(alpha Q.K^T).V in one launch.  The composite's shape function is the two
    batch_matmul shape functions connected: (T,L,D)x(T,L,D)^T -> (T,L,L), then x(T,L,D) -> (T,L,D)."""
    s_shape = nb.batch_matmul_shape(tuple(q.shape), tuple(k.shape), True)
    T, L, D = nb.batch_matmul_shape(s_shape, tuple(v.shape), False)
    o = out if out is not None else _alloc((T, L, D), nb.BF16, q.device)
    nb.nimble_attention_dyn(_ptr(q, _BF, "q"), _ptr(k, _BF, "k"), _ptr(v, _BF, "v"), _ptr(o, _BF, "o"), T, L, D, alpha,
                            _stream())
    return o


def lstm_step(x: torch.Tensor, h: torch.Tensor, w: torch.Tensor, bias: torch.Tensor, c: torch.Tensor,
              h_out: Optional[torch.Tensor] = None,
              c_out: Optional[torch.Tensor] = None) -> Tuple[torch.Tensor, torch.Tensor]:
    (B, H), _ = nb.lstm_shape(tuple(x.shape), tuple(h.shape), tuple(c.shape), tuple(w.shape))
    Ix = x.shape[1]
    if h_out is None:
        h_out = _alloc((B, H), nb.BF16, x.device)
    if c_out is None:
        c_out = _alloc((B, H), nb.F32, x.device)
    nb.nimble_lstm_gates_dyn(_ptr(x, _BF, "x"), _ptr(h, _BF, "h"), _ptr(w, _BF, "w"), _ptr(bias, _BF, "bias"),
                             _ptr(c, _F32, "c"), _ptr(c_out, _F32, "c_out"), _ptr(h_out, _BF, "h_out"), B, Ix, H, 0, 0,
                             _stream())
    return h_out, c_out


def lstm_step_pre(pre: torch.Tensor, h: torch.Tensor, w_h: torch.Tensor, c: torch.Tensor,
                  h_out: Optional[torch.Tensor] = None,
                  c_out: Optional[torch.Tensor] = None) -> Tuple[torch.Tensor, torch.Tensor]:
    """One cell step from the precomputed input share of the gates pre [B, 4H] (f32)."""
    (B, H), _ = nb.lstm_pre_shape(tuple(pre.shape), tuple(h.shape), tuple(c.shape), tuple(w_h.shape))
    if h_out is None:
        h_out = _alloc((B, H), nb.BF16, h.device)
    if c_out is None:
        c_out = _alloc((B, H), nb.F32, h.device)
    nb.nimble_lstm_gates_pre_dyn(_ptr(pre, _F32, "pre"), _ptr(h, _BF, "h"), _ptr(w_h, _BF, "w_h"), _ptr(c, _F32, "c"),
                                 _ptr(c_out, _F32, "c_out"), _ptr(h_out, _BF, "h_out"), B, H, _stream())
    return h_out, c_out


# polls per wait of the one-launch token loop before it gives up (a poll is a round trip to memory, 0.5-1 us:
# a quarter of a second at the very most)
LSTM_SEQ_MAX_POLLS = 1 << 18


def lstm_sequence_pre(pre: torch.Tensor, w_h: torch.Tensor, h0: torch.Tensor, c0: torch.Tensor,
                      max_polls: int = LSTM_SEQ_MAX_POLLS, one_launch: Optional[bool] = None,
                      workspace: Optional[torch.Tensor] = None) -> Tuple[torch.Tensor, torch.Tensor, bool]:
    """The token loop of one sequence from the inputs' share of the gates pre [T, B, 4H] (f32):
    returns (h_seq [T,B,H] bf16, c_T [B,H] f32, ran_in_one_launch).

    one_launch=None: shapes for which nimble_lstm_seq_preferred says so run as one launch
    (nimble_lstm_seq_pre_dyn); True: every shape nimble_lstm_seq_supported accepts does (others raise);
    False: none.  After a one-launch run the call waits for the stream and reads the loop's give-up word;
    if the loop gave up, or one launch was not taken, the steps run one by one through
    nimble_lstm_gates_pre_dyn, which gives the same bits."""
    (T, B, H), _ = nb.lstm_seq_shape(tuple(pre.shape), tuple(h0.shape), tuple(c0.shape), tuple(w_h.shape))
    dev = h0.device
    h_seq = _alloc((T, B, H), nb.BF16, dev)
    c_out = _alloc((B, H), nb.F32, dev)
    pp, wp, hp, cp = _ptr(pre, _F32, "pre"), _ptr(w_h, _BF, "w_h"), _ptr(h0, _BF, "h0"), _ptr(c0, _F32, "c0")
    if T == 0:
        c_out.copy_(c0)
        return h_seq, c_out, False
    supported = nb.lstm_seq_supported(B, H)
    if one_launch and not supported:
        raise nb.NimbleError(-3, f"the one-launch token loop does not run B={B}, H={H}")
    if one_launch is None:
        one_launch = nb.lstm_seq_preferred(B, H)
    if supported and one_launch:
        need = nb.lstm_seq_workspace_bytes(B, H)
        if workspace is None:
            workspace = torch.empty(need, dtype=torch.uint8, device=dev)
        nb.nimble_lstm_seq_pre_dyn(pp, wp, hp, cp, h_seq.data_ptr(), c_out.data_ptr(), T, B, H,
                                   _ptr(workspace, torch.uint8, "workspace"), workspace.numel(), max_polls, _stream())
        if not nb.nimble_lstm_seq_status(workspace.data_ptr(), _stream()):
            return h_seq, c_out, True
    st = _stream()
    c_out.copy_(c0)
    for t in range(T):
        nb.nimble_lstm_gates_pre_dyn(pre[t].data_ptr(), (h0 if t == 0 else h_seq[t - 1]).data_ptr(), wp,
                                     c_out.data_ptr(), c_out.data_ptr(), h_seq[t].data_ptr(), B, H, st)
    return h_seq, c_out, False


def lstm_sequence(xs: torch.Tensor, w_x: torch.Tensor, w_h: torch.Tensor, bias: torch.Tensor, h0: torch.Tensor,
                  c0: torch.Tensor, **kw) -> Tuple[torch.Tensor, torch.Tensor, bool]:
    """A whole sequence xs [T, B, Ix] through the cell: the inputs' share of the gates for all T*B tokens in one
    dense call (M = T*B dynamic, f32 output), then the token loop (lstm_sequence_pre).  w_x [4H, Ix] and
    w_h [4H, H] are the two halves of the fused weight (split_lstm_weight)."""
    T, B, Ix = xs.shape
    pre = dense(xs.view(T * B, Ix), w_x, bias, nb.EPI_BIAS, nb.F32)
    return lstm_sequence_pre(pre.view(T, B, w_x.shape[0]), w_h, h0, c0, **kw)


def split_lstm_weight(w: torch.Tensor, Ix: int) -> Tuple[torch.Tensor, torch.Tensor]:
    """One-time split of the fused weight [4H, Ix+H] into contiguous input and recurrent halves."""
    return w[:, :Ix].contiguous(), w[:, Ix:].contiguous()


class LstmSequenceGraph:
    """The token loop of one sequence, `steps` launches of the fused LSTM cell, captured once
    per batch size B as a HIP graph and replayed: the loop is launch-bound (a step is a few
    microseconds of GPU work), so replaying removes the per-step host cost.  The graph holds
    kernel launches only (state is cleared by a fill kernel outside it).  The dynamic extent
    B is fixed per graph; a server keeps one graph per batch size it has seen."""

    def __init__(self, w: torch.Tensor, bias: torch.Tensor, B: int, steps: int, Ix: int, H: int,
                 project_inputs: bool = False):
        """project_inputs: compute the inputs' share of the gates for all tokens in one dense
        call (M = steps * B) ahead of the loop, so each step streams only the recurrent half
        of the weight."""
        dev = w.device
        (self.B, self.H), _ = nb.lstm_shape((B, Ix), (B, H), (B, H), tuple(w.shape))
        self.steps, self.Ix = steps, Ix
        self.w, self.bias = w, bias
        self.project_inputs = project_inputs
        if project_inputs:
            self.w_x, self.w_h = split_lstm_weight(w, Ix)
            self.pre = torch.empty((steps, B, 4 * H), dtype=torch.float32, device=dev)
        self.xs = torch.zeros((steps, B, Ix), dtype=torch.bfloat16, device=dev)
        self.hs = torch.zeros((steps + 1, B, H), dtype=torch.bfloat16, device=dev)  # hs[0] = h_0
        self.c = torch.zeros((B, H), dtype=torch.float32, device=dev)
        # one eager pass so that nothing is lazily initialised during capture
        self._enqueue()
        torch.cuda.synchronize()
        self.graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(self.graph):
            self._enqueue()

    def _enqueue(self) -> None:
        st = _stream()
        if self.project_inputs:
            dense(self.xs.view(self.steps * self.B, self.Ix), self.w_x, self.bias, nb.EPI_BIAS, nb.F32,
                  out=self.pre.view(self.steps * self.B, 4 * self.H))
            for t in range(self.steps):
                nb.nimble_lstm_gates_pre_dyn(self.pre[t].data_ptr(), self.hs[t].data_ptr(), self.w_h.data_ptr(),
                                             self.c.data_ptr(), self.c.data_ptr(), self.hs[t + 1].data_ptr(),
                                             self.B, self.H, st)
            return
        for t in range(self.steps):
            nb.nimble_lstm_gates_dyn(self.xs[t].data_ptr(), self.hs[t].data_ptr(), self.w.data_ptr(),
                                     self.bias.data_ptr(), self.c.data_ptr(), self.c.data_ptr(),
                                     self.hs[t + 1].data_ptr(), self.B, self.Ix, self.H, 0, 0, st)

    def run(self, xs: Optional[torch.Tensor] = None) -> Tuple[torch.Tensor, torch.Tensor]:
        """Run the sequence from h_0 = c_0 = 0; returns (all h_t [steps,B,H], final c)."""
        if xs is not None:
            self.xs.copy_(xs)
        self.hs[0].zero_()
        self.c.zero_()
        self.graph.replay()
        return self.hs[1:], self.c

"""Pins of the reference VM interpreter (oracle/vm_oracle.py): hand-written word streams whose
results are worked out by hand, agreement with direct calls of the oracle kernels, error cases."""
import os

import numpy as np
import pytest

import oracle
import workloads as wl
from oracle import vm_oracle as vo

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def _golden(name):
    out = {}
    for line in open(os.path.join(GOLDEN, name)):
        if line.startswith("#") or ":" not in line:
            continue
        k, v = line.split(":", 1)
        out[k.strip()] = [int(t) for t in v.split()]
    return out


def _bf16(a):
    return wl.bf16_bits_to_f32(wl.f32_to_bf16_bits(np.asarray(a, np.float32)))


def _t(a, dtype=vo.BF16):
    return vo.Tensor(np.array(a, dtype=np.float32), dtype)


def test_count_loop_by_hand():
    g = _golden("vm_count_loop.txt")
    res, executed = vo.run(g["words"], g["registers"][0], [], [])
    assert res == g["result"][0]
    assert executed == g["executed"][0]


@pytest.mark.parametrize("a,b,expect", [(3, 3, 111), (3, 4, 222), (4, 3, 222)])
def test_if_takes_true_offset_when_equal(a, b, expect):
    # 0 consti a->r0; 1 consti b->r1; 2 If r0,r1,+1,+3; 3 consti 111->r2; 4 Goto +2; 5 consti 222->r2; 6 Ret r2
    words = [5, 2, a, 0, 5, 2, b, 1, 2, 4, 0, 1, 1, 3, 5, 2, 111, 2, 3, 1, 2, 5, 2, 222, 2, 1, 1, 2]
    res, executed = vo.run(words, 3, [], [])
    assert res == expect
    assert executed == (6 if expect == 111 else 5)


def test_round_bf16_ties_to_even_and_matches_the_generator_module():
    one = np.float32(1.0)
    cases = {1.0: 1.0, 1.0 + 2.0 ** -8: 1.0, 1.0 + 3 * 2.0 ** -8: 1.0 + 2.0 ** -6, 1.0 + 2.0 ** -7: 1.0 + 2.0 ** -7,
             -(1.0 + 2.0 ** -8 + 2.0 ** -20): -(1.0 + 2.0 ** -7), 0.0: 0.0}
    for x, y in cases.items():
        assert vo.round_bf16(np.array([x], np.float32))[0] == np.float32(y), x
    rng = np.random.default_rng(7)
    a = (rng.standard_normal(4096) * 10.0 ** rng.integers(-6, 6, 4096)).astype(np.float32)
    assert np.array_equal(vo.round_bf16(a), _bf16(a))
    assert one == vo.round_bf16(np.array([one]))[0]


def _dense_words(packed):
    """Appendix A's pattern for one dense call, written out by hand.
    inputs r0 = x; constants 0 = w, 1 = b.
      0 LoadConst 0 -> r1 (w)          1 LoadConst 1 -> r2 (b)
      2 ShapeOf r0 -> r3               3 ShapeOf r1 -> r4
      4 LoadConsti 16 -> r5            5 AllocStorage r5, 64, host -> r6
      6 AllocTensor r6, 0, i64, rank 1, [2] -> r7
      7 InvokePacked shape_dense(r3, r4 -> r7)
      8 LoadConsti 0 (bf16) -> r8      9 InvokePacked storage_bytes(r7, r8 -> r9)
     10 AllocStorage r9, 64, gpu -> r10
     11 AllocTensorReg r10, 0, r7, bf16 -> r11
     12 InvokePacked dense_bias*(r0, r1, r2 -> r11)
     13 AllocADT tag 7 [r11, r7, r9] -> r12     14 Ret r12"""
    return [4, 2, 0, 1, 4, 2, 1, 2, 19, 2, 0, 3, 19, 2, 1, 4, 5, 2, 16, 5, 6, 4, 5, 64, 0, 6,
            7, 6, 6, 0, 2, 1, 2, 7, 15, 6, 0, 3, 1, 3, 4, 7, 5, 2, 0, 8, 15, 6, 3, 3, 1, 7, 8, 9,
            6, 4, 9, 64, 1, 10, 8, 5, 10, 0, 7, 0, 11, 15, 7, packed, 4, 1, 0, 1, 2, 11,
            9, 6, 7, 3, 11, 7, 9, 12, 1, 1, 12]


@pytest.mark.parametrize("packed,epi", [(vo.DENSE_BIAS, "bias"), (vo.DENSE_BIAS_GELU, "bias_gelu")])
@pytest.mark.parametrize("M", [1, 5, 33])
def test_dense_program_equals_direct_oracle_call(packed, epi, M):
    rng = np.random.default_rng(100 + M)
    x, w, b = (_bf16(rng.uniform(-1, 1, s)) for s in ((M, 24), (40, 24), (40,)))
    res, executed = vo.run(_dense_words(packed), 13, [_t(w), _t(b)], [_t(x)])
    assert executed == 15
    assert isinstance(res, vo.ADT) and res.tag == 7
    y, shape, nbytes = vo.flatten(res)
    assert shape.array.tolist() == [M, 40] and shape.dtype == vo.I64
    assert nbytes == M * 40 * 2
    direct = oracle.dense(x, w, b, epi)
    assert np.array_equal(y.array, _bf16(direct))  # rounded to bf16 where the tensor is bf16
    assert y.dtype == vo.BF16


def test_dense_program_type_error_is_found_at_run_time():
    # K of x (23) and of w (24) disagree: only the shape function can see it (Section 3.1, 3.2)
    with pytest.raises(vo.VMError) as e:
        vo.run(_dense_words(vo.DENSE_BIAS), 13, [_t(np.zeros((40, 24))), _t(np.zeros(40))], [_t(np.zeros((3, 23)))])
    assert e.value.kind == "SHAPE"


def _w(op, *operands):
    return [op, len(operands), *operands]


def test_lstm_loop_equals_python_loop_over_the_cell():
    T, B, Ix, H = 4, 3, 8, 8
    rng = np.random.default_rng(5)
    xs = _bf16(rng.uniform(-1, 1, (T, B, Ix)))
    w = _bf16(rng.normal(0, 0.3, (4 * H, Ix + H)))
    b = _bf16(rng.normal(0, 0.3, (4 * H,)))
    # inputs r0 xs, r1 h, r2 c; constants 0 w, 1 b.  Jump offsets counted by hand from the pc column.
    prog = [
        _w(vo.LOAD_CONST, 0, 3),                     # 0  w
        _w(vo.LOAD_CONST, 1, 4),                     # 1  b
        _w(vo.LOAD_CONSTI, 0, 5),                    # 2  t = 0
        _w(vo.LOAD_CONSTI, 1, 6),                    # 3  one
        _w(vo.SHAPE_OF, 0, 7),                       # 4  (T,B,Ix)
        _w(vo.INVOKE_PACKED, vo.SHAPE_GET, 3, 1, 7, 5, 8),  # 5  T = shape[t = 0]
        _w(vo.IF, 5, 8, 14, 1),                      # 6  t == T -> pc 20, else pc 7
        _w(vo.INVOKE_PACKED, vo.INDEX0, 3, 1, 0, 5, 9),     # 7  x_t
        _w(vo.LOAD_CONSTI, B * H * 2, 10),           # 8  bytes of h'
        _w(vo.ALLOC_STORAGE, 10, 64, 1, 11),         # 9
        _w(vo.ALLOC_TENSOR, 11, 0, vo.BF16, 2, B, H, 12),   # 10 h'
        _w(vo.LOAD_CONSTI, B * H * 4, 13),           # 11 bytes of c'
        _w(vo.ALLOC_STORAGE, 13, 64, 1, 14),         # 12
        _w(vo.ALLOC_TENSOR, 14, 0, vo.F32, 2, B, H, 15),    # 13 c'
        _w(vo.INVOKE_PACKED, vo.LSTM_GATES, 7, 2, 9, 1, 3, 4, 2, 15, 12),  # 14 (x_t,h,w,b,c -> c',h')
        _w(vo.MOVE, 12, 1),                          # 15 h = h'
        _w(vo.MOVE, 15, 2),                          # 16 c = c'
        _w(vo.INVOKE_PACKED, vo.INT_ADD, 3, 1, 5, 6, 5),    # 17 t += 1
        _w(vo.GOTO, -12),                            # 18 -> pc 6
        _w(vo.FATAL),                                # 19 never reached
        _w(vo.ALLOC_ADT, 0, 2, 1, 2, 16),            # 20 (h, c)
        _w(vo.RET, 16),                              # 21
    ]
    words = [x for ins in prog for x in ins]
    h = np.zeros((B, H), np.float32)
    c = np.zeros((B, H), np.float32)
    res, executed = vo.run(words, 17, [_t(w), _t(b)], [_t(xs), _t(h), _t(c, vo.F32)])
    hv, cv = vo.flatten(res)
    for t in range(T):
        h, c = oracle.lstm_step(xs[t], h, w, b, c)
        h = _bf16(h)  # the state handed to the next step is a bf16 tensor
    assert np.array_equal(hv.array, h)
    assert np.array_equal(cv.array, c)
    assert executed == 6 + T * 13 + 1 + 2


def test_adt_fields_and_tag():
    # 0 consti 10->r0; 1 consti 20->r1; 2 AllocADT tag 3 [r0,r1]->r2; 3 GetField r2,1->r3; 4 GetTag r2->r4;
    # 5 add(r3,r4)->r5; 6 Ret r5
    words = [5, 2, 10, 0, 5, 2, 20, 1, 9, 5, 3, 2, 0, 1, 2, 16, 3, 2, 1, 3, 17, 2, 2, 4, 15, 6, 5, 3, 1, 3, 4, 5, 1, 1, 5]
    assert vo.run(words, 6, [], [])[0] == 23


def test_reshape_and_shape_of():
    # r0 = tensor [2,6]; 0 consti 16->r1; 1 AllocStorage host->r2; 2 AllocTensor i64 [2] -> r3 (zeros)
    # we need a shape (3,4): take it from a second input's ShapeOf instead
    # 0 ShapeOf r1 -> r2 ; 1 ReshapeTensor r0, r2 -> r3 ; 2 ShapeOf r3 -> r4 ; 3 Ret r4
    words = [19, 2, 1, 2, 20, 3, 0, 2, 3, 19, 2, 3, 4, 1, 1, 4]
    res, _ = vo.run(words, 5, [], [_t(np.arange(12).reshape(2, 6)), _t(np.zeros((3, 4)))])
    assert res.array.tolist() == [3, 4]
    with pytest.raises(vo.VMError) as e:
        vo.run(words, 5, [], [_t(np.arange(12).reshape(2, 6)), _t(np.zeros((5, 2)))])
    assert e.value.kind == "SHAPE"


def test_fatal_limit_unimplemented_and_small_storage():
    with pytest.raises(vo.VMError) as e:
        vo.run([21, 0], 1, [], [])
    assert e.value.kind == "SHAPE"
    with pytest.raises(vo.VMError) as e:
        vo.run([3, 1, 0], 1, [], [], max_instructions=1000)  # Goto self
    assert e.value.kind == "ARG"
    for op in (10, 13, 14, 18):
        with pytest.raises(vo.VMError):
            vo.run([op, 0, 1, 1, 0], 1, [], [])
    # storage of 8 bytes cannot hold a [2] int64 tensor
    words = [5, 2, 8, 0, 6, 4, 0, 64, 0, 1, 7, 6, 1, 0, 2, 1, 2, 2, 1, 1, 2]
    with pytest.raises(vo.VMError) as e:
        vo.run(words, 3, [], [])
    assert e.value.kind == "WORKSPACE"

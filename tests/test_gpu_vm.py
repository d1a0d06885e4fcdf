"""The bytecode interpreter on the GPU: programs whose tensor shapes are known only when the input
arrives, run through the C ABI, against (a) the same kernels called directly (bit for bit) and
(b) the reference interpreter over the CPU oracle (normwise error <= 5e-3, shapes exact)."""
import numpy as np
import pytest

import oracle
import workloads as wl
from oracle import vm_oracle as vo

torch = pytest.importorskip("torch")
pytestmark = pytest.mark.gpu

TOL = 5e-3


@pytest.fixture(scope="module")
def env():
    import paper_2006_03031_amd as nb
    from paper_2006_03031_amd import runtime, vm
    from gpu_util import bits_from_dev, f32_to_dev, from_dev, to_dev
    nb.load()

    class E:
        pass
    e = E()
    e.nb, e.rt, e.vm = nb, runtime, vm
    e.to_dev, e.f32_to_dev, e.from_dev, e.bits = to_dev, f32_to_dev, from_dev, bits_from_dev
    e.pool = torch.empty(256 << 20, dtype=torch.uint8, device="cuda")
    return e


def _ref_tensor(a, dtype=vo.BF16):
    return vo.Tensor(np.array(a.f32 if isinstance(a, wl.BF16Array) else a, dtype=np.float32), dtype)


def test_lstm_token_loop_program(env):
    lw = wl.config2_weights()
    dw, db = env.to_dev(lw.w), env.to_dev(lw.b)
    H, Ix = wl.LSTM_H, wl.LSTM_IX
    prog = env.vm.lstm_sequence_program()
    exe = env.vm.Executable.from_assembler(prog, [dw, db])
    per_token = None
    for seq, (B, T) in enumerate([(1, 9), (5, 16), (64, 7), (33, 1), (17, 0)]):
        xs = wl.config2_inputs(70 + seq, B, max(T, 1))
        xd = env.to_dev(xs)[:T].contiguous()
        h0 = torch.zeros((B, H), dtype=torch.bfloat16, device="cuda")
        c0 = torch.zeros((B, H), dtype=torch.float32, device="cuda")
        h_vm, c_vm = exe.run([xd, h0, c0], env.pool)
        assert tuple(h_vm.shape) == (B, H) and tuple(c_vm.shape) == (B, H)
        assert h_vm.dtype == torch.bfloat16 and c_vm.dtype == torch.float32
        # (a) the same kernels called one by one
        h, c = h0, c0
        for t in range(T):
            h, c = env.rt.lstm_step(xd[t], h, dw, db, c)
        torch.cuda.synchronize()
        assert np.array_equal(env.bits(h_vm), env.bits(h)), (B, T)
        assert np.array_equal(env.from_dev(c_vm), env.from_dev(c)), (B, T)
        # (b) the reference interpreter on the same bytecode
        ref, executed = vo.run(prog.words(), prog.n_regs, [_ref_tensor(lw.w), _ref_tensor(lw.b)],
                               [vo.Tensor(xs.f32[:T].copy(), vo.BF16), vo.Tensor(np.zeros((B, H), np.float32), vo.BF16),
                                vo.Tensor(np.zeros((B, H), np.float32), vo.F32)])
        rh, rc = vo.flatten(ref)
        if T:
            assert oracle.normwise_rel_error(env.from_dev(h_vm), rh.array) <= TOL, (B, T)
            assert oracle.normwise_rel_error(env.from_dev(c_vm), rc.array) <= TOL, (B, T)
        else:  # zero tokens: the initial state comes back untouched
            assert h_vm.data_ptr() == h0.data_ptr() and c_vm.data_ptr() == c0.data_ptr()
        prof = exe.profile()
        assert prof["instructions"] == executed
        assert prof["packed"].get("lstm_gates", (0, 0))[0] == T
        if T >= 3:
            # the state blocks ping-pong: two live h and two live c blocks at most, the rest reused
            blk = lambda n: (n + 63) // 64 * 64
            assert prof["pool_high_water"] == 2 * (blk(B * H * 2) + blk(B * H * 4))
            assert prof["storage_allocs"] == 2 * T and prof["storage_reuses"] == 2 * (T - 2)
            per_token = (executed - 1) // T
    assert per_token is not None and per_token <= 30  # a couple of dozen coarse instructions per token


def test_ffn_block_program_dynamic_m(env):
    (w1, b1), (w2, b2) = wl.dense_weights(5, 0, 4096, 1024), wl.dense_weights(5, 1, 1024, 4096)
    consts = [env.to_dev(a) for a in (w1, b1, w2, b2)]
    prog = env.vm.ffn_block_program()
    exe = env.vm.Executable.from_assembler(prog, consts)
    ref_consts = [_ref_tensor(a) for a in (w1, b1, w2, b2)]
    for draw, M in enumerate([1, 16, 77, 300, 1029]):  # one executable, M differs per run
        x = wl.activations(5, 100 + draw, M, 1024)
        xd = env.to_dev(x)
        (y,) = exe.run([xd], env.pool)
        assert tuple(y.shape) == (M, 1024) and y.dtype == torch.bfloat16
        # direct calls
        h_d = env.rt.dense(xd, consts[0], consts[1], env.nb.EPI_BIAS_GELU_ERF)
        y_d = env.rt.dense(h_d, consts[2], consts[3], env.nb.EPI_BIAS)
        torch.cuda.synchronize()
        assert np.array_equal(env.bits(y), env.bits(y_d)), M
        ref, executed = vo.run(prog.words(), prog.n_regs, ref_consts, [_ref_tensor(x)])
        assert ref.array.shape == (M, 1024)
        assert oracle.normwise_rel_error(env.from_dev(y), ref.array) <= TOL, M
        prof = exe.profile()
        assert prof["instructions"] == executed == len(prog.instrs)
        assert prof["pool_high_water"] >= M * 4096 * 2 + M * 1024 * 2
    # M = 0 is a legal instantiation of Any: shapes flow, nothing is launched
    (y,) = exe.run([torch.empty((0, 1024), dtype=torch.bfloat16, device="cuda")], env.pool)
    assert tuple(y.shape) == (0, 1024)
    # a wrong K is caught by the shape function at run time
    with pytest.raises(env.nb.NimbleError) as e:
        exe.run([torch.zeros((4, 1000), dtype=torch.bfloat16, device="cuda")], env.pool)
    assert e.value.code == -3


def test_attention_program(env):
    prog = env.vm.attention_program()
    exe = env.vm.Executable.from_assembler(prog)
    for draw, L in enumerate([1, 64, 65, 200]):
        q, k, v = wl.config4_qkv(200 + draw, L)
        dq, dk, dv = (env.to_dev(a) for a in (q, k, v))
        (o,) = exe.run([dq, dk, dv], env.pool)
        assert tuple(o.shape) == (12, L, 64)
        direct = env.rt.fused_attention(dq, dk, dv)
        torch.cuda.synchronize()
        assert np.array_equal(env.bits(o), env.bits(direct)), L
        ref, _ = vo.run(prog.words(), prog.n_regs, [], [_ref_tensor(q), _ref_tensor(k), _ref_tensor(v)])
        assert oracle.normwise_rel_error(env.from_dev(o), ref.array) <= TOL, L


def test_pool_too_small_is_an_error_not_a_fault(env):
    lw = wl.config2_weights()
    exe = env.vm.Executable.from_assembler(env.vm.lstm_sequence_program(), [env.to_dev(lw.w), env.to_dev(lw.b)])
    B, T, H = 8, 4, wl.LSTM_H
    xd = env.to_dev(wl.config2_inputs(90, B, T))
    h0 = torch.zeros((B, H), dtype=torch.bfloat16, device="cuda")
    c0 = torch.zeros((B, H), dtype=torch.float32, device="cuda")
    small = torch.empty(B * H * 2 + B * H * 4, dtype=torch.uint8, device="cuda")  # room for one step's state only
    with pytest.raises(env.nb.NimbleError) as e:
        exe.run([xd, h0, c0], small)
    assert e.value.code == -6
    torch.cuda.synchronize()
    # the same executable still runs with a large enough pool
    h, c = exe.run([xd, h0, c0], env.pool)
    torch.cuda.synchronize()
    assert tuple(h.shape) == (B, H)

"""The token loop of an LSTM sequence as one launch (nimble_lstm_seq_pre_dyn) against the step-by-step
path (bit for bit) and against the CPU oracle (every step teacher-forced from the GPU's own previous
state, to the bars of test_gpu_parity), plus the loop's give-up path, forced from the host."""
import numpy as np
import pytest

import oracle
import workloads as wl

torch = pytest.importorskip("torch")
pytestmark = pytest.mark.gpu

TOL = 5e-3
GATE_BF16 = 2.0 ** -7
GATE_F32 = 2.0 ** -14


@pytest.fixture(scope="module")
def rt():
    import paper_2006_03031_amd as nb
    from paper_2006_03031_amd import runtime
    nb.load()
    return runtime


@pytest.fixture(scope="module")
def nb():
    import paper_2006_03031_amd as nb
    return nb


def _check(got, ref, what, f32=False):
    rel = GATE_F32 if f32 else GATE_BF16
    e = oracle.normwise_rel_error(got, ref)
    assert e <= TOL, ("normwise", what, e)
    x = oracle.elementwise_excess(got, ref, rel, rel)
    assert x <= 1.0, ("element-wise", what, x)


def _case(seed, T, B, H):
    rng = np.random.default_rng([2, 77, seed, T, B, H])
    pre = rng.uniform(-2.0, 2.0, (T, B, 4 * H)).astype(np.float32)
    w_h = wl.normal_bf16(rng, (4 * H, H), std=1.0 / np.sqrt(H))
    h0 = wl.uniform_bf16(rng, (B, H))
    c0 = rng.uniform(-1.0, 1.0, (B, H)).astype(np.float32)
    return pre, w_h, h0, c0


def _step_by_step(rt, pre, w_h, h0, c0):
    """T calls of the cell; returns every (h_t, c_t)."""
    hs, cs = [], []
    h, c = h0, c0
    for t in range(pre.shape[0]):
        h, c = rt.lstm_step_pre(pre[t], h, w_h, c)
        hs.append(h)
        cs.append(c)
    return hs, cs


@pytest.mark.parametrize("T,B,H", [(40, 1, 512), (12, 2, 512), (9, 4, 512), (6, 3, 1024), (5, 2, 256),
                                   (4, 4, 64), (5, 3, 576), (3, 4, 1024), (7, 1, 320)])
def test_one_launch_equals_the_steps_one_by_one_and_matches_the_oracle(rt, nb, T, B, H):
    from gpu_util import bits_from_dev, f32_to_dev, from_dev, to_dev
    pre, w_h, h0, c0 = _case(0, T, B, H)
    dpre, dw, dh0, dc0 = f32_to_dev(pre), to_dev(w_h), to_dev(h0), f32_to_dev(c0)
    print(f"one launch T={T} B={B} H={H}", flush=True)
    h_seq, c_T, one = rt.lstm_sequence_pre(dpre, dw, dh0, dc0, one_launch=True)
    assert one, "the loop gave up on an idle GPU"
    assert tuple(h_seq.shape) == oracle.lstm_seq_shape(pre.shape, h0.shape, c0.shape, w_h.shape)[0]
    hs, cs = _step_by_step(rt, dpre, dw, dh0, dc0)
    for t in range(T):
        assert np.array_equal(bits_from_dev(h_seq[t]), bits_from_dev(hs[t])), ("h", t)
    assert np.array_equal(from_dev(c_T).view(np.uint32), from_dev(cs[-1]).view(np.uint32))
    # the oracle, one step at a time from the GPU's own previous state
    h_prev, c_prev = h0.f32, c0
    for t in range(T):
        ref_h, ref_c = oracle.lstm_step_pre(pre[t], h_prev, w_h.f32, c_prev)
        _check(from_dev(h_seq[t]), ref_h, ("h", t, B, H))
        if t == T - 1:
            _check(from_dev(c_T), ref_c, ("c", t, B, H), f32=True)
        h_prev, c_prev = from_dev(h_seq[t]), from_dev(cs[t])
    # the fallback path of the same call gives the same bits
    h2, c2, one2 = rt.lstm_sequence_pre(dpre, dw, dh0, dc0, one_launch=False)
    assert not one2 and torch.equal(h2, h_seq) and torch.equal(c2, c_T)


def test_two_sequences_in_a_row_share_a_workspace_and_long_sequences_wrap_nothing(rt, nb):
    """The workspace is cleared by the call itself: a second, shorter sequence of another batch size
    through the same workspace must not see the first one's tagged words; 300 steps at B = 1."""
    from gpu_util import bits_from_dev, f32_to_dev, to_dev
    ws = torch.empty(nb.lstm_seq_workspace_bytes(4, 512), dtype=torch.uint8, device="cuda")
    for seed, (T, B) in enumerate([(300, 1), (7, 4), (3, 1), (2, 3)]):
        pre, w_h, h0, c0 = _case(10 + seed, T, B, 512)
        dpre, dw, dh0, dc0 = f32_to_dev(pre), to_dev(w_h), to_dev(h0), f32_to_dev(c0)
        print(f"shared workspace T={T} B={B}", flush=True)
        h_seq, c_T, one = rt.lstm_sequence_pre(dpre, dw, dh0, dc0, one_launch=True, workspace=ws)
        assert one
        hs, cs = _step_by_step(rt, dpre, dw, dh0, dc0)
        assert np.array_equal(bits_from_dev(h_seq), np.stack([bits_from_dev(h) for h in hs]))
        assert torch.equal(c_T, cs[-1])


def test_the_loop_gives_up_when_told_to_and_the_call_falls_back(rt, nb):
    """max_polls = 0: every wave gives up at its first wait, sets the give-up word and leaves; the grid
    drains, the status call reports it, and lstm_sequence_pre runs the steps one by one instead."""
    from gpu_util import bits_from_dev, f32_to_dev, to_dev
    T, B, H = 6, 3, 512
    pre, w_h, h0, c0 = _case(20, T, B, H)
    dpre, dw, dh0, dc0 = f32_to_dev(pre), to_dev(w_h), to_dev(h0), f32_to_dev(c0)
    ws = torch.empty(nb.lstm_seq_workspace_bytes(B, H), dtype=torch.uint8, device="cuda")
    h_seq = torch.empty((T, B, H), dtype=torch.bfloat16, device="cuda")
    c_out = torch.empty((B, H), dtype=torch.float32, device="cuda")
    st = torch.cuda.current_stream().cuda_stream
    print("forced give-up", flush=True)
    nb.nimble_lstm_seq_pre_dyn(dpre.data_ptr(), dw.data_ptr(), dh0.data_ptr(), dc0.data_ptr(), h_seq.data_ptr(),
                               c_out.data_ptr(), T, B, H, ws.data_ptr(), ws.numel(), 0, st)
    assert nb.nimble_lstm_seq_status(ws.data_ptr(), st) is True
    words = ws.cpu().numpy().view(np.uint32)
    assert words[0] == 1 and words[1] == 0     # gave up; no workgroup ran all its steps
    # the wrapper notices and falls back; the result is the step-by-step one
    h2, c2, one = rt.lstm_sequence_pre(dpre, dw, dh0, dc0, max_polls=0)
    assert not one
    hs, cs = _step_by_step(rt, dpre, dw, dh0, dc0)
    assert np.array_equal(bits_from_dev(h2), np.stack([bits_from_dev(h) for h in hs])) and torch.equal(c2, cs[-1])
    # and the same workspace serves a normal call afterwards
    h3, c3, one = rt.lstm_sequence_pre(dpre, dw, dh0, dc0, one_launch=True, workspace=ws)
    assert one and torch.equal(h3, h2) and torch.equal(c3, c2)


def test_unsupported_shapes_run_step_by_step_or_raise(rt, nb):
    from gpu_util import f32_to_dev, to_dev
    pre, w_h, h0, c0 = _case(30, 3, 20, 512)      # B = 20 > 4
    args = (f32_to_dev(pre), to_dev(w_h), to_dev(h0), f32_to_dev(c0))
    h, c, one = rt.lstm_sequence_pre(*args)
    assert not one and tuple(h.shape) == (3, 20, 512)
    with pytest.raises(nb.NimbleError):
        rt.lstm_sequence_pre(*args, one_launch=True)
    # the default takes one launch exactly where the library prefers it
    for (B, H) in [(1, 512), (4, 256), (1, 1024), (2, 1024)]:
        pre, w_h, h0, c0 = _case(31, 4, B, H)
        _, _, one = rt.lstm_sequence_pre(f32_to_dev(pre), to_dev(w_h), to_dev(h0), f32_to_dev(c0))
        assert one == nb.lstm_seq_preferred(B, H)


def test_whole_sequence_with_projected_inputs_equals_the_captured_graph(rt, nb):
    """config 2's cell (2048 x 1024): the inputs' product for all tokens in one dense call, then the loop in one
    launch; the same bits as the captured graph of per-step launches, which test_gpu_parity holds to the oracle."""
    from gpu_util import to_dev
    lw = wl.config2_weights()
    dw, db = to_dev(lw.w), to_dev(lw.b)
    H, Ix, T = wl.LSTM_H, wl.LSTM_IX, 24
    w_x, w_h = rt.split_lstm_weight(dw, Ix)
    for B in (1, 3):
        xs = to_dev(wl.config2_inputs(50 + B, B, T))
        h0 = torch.zeros((B, H), dtype=torch.bfloat16, device="cuda")
        c0 = torch.zeros((B, H), dtype=torch.float32, device="cuda")
        print(f"sequence B={B}", flush=True)
        h_seq, c_T, one = rt.lstm_sequence(xs, w_x, w_h, db, h0, c0)
        assert one == nb.lstm_seq_preferred(B, H) and one
        graph = rt.LstmSequenceGraph(dw, db, B, T, Ix, H, project_inputs=True)
        hs, c = graph.run(xs)
        assert torch.equal(hs, h_seq) and torch.equal(c, c_T)


def test_step_tags_wrap_after_65535_steps(rt, nb):
    """The hand-over words carry a 16-bit step tag with period 65535: a sequence longer than that must still give
    the bits of the step-by-step path (checked on the last steps and the final cell state) and match the oracle
    on its last step."""
    from gpu_util import bits_from_dev, f32_to_dev, from_dev, to_dev
    T, B, H = 65535 + 700, 1, 64
    rng = np.random.default_rng([2, 99])
    pre = rng.uniform(-2.0, 2.0, (T, B, 4 * H)).astype(np.float32)
    w_h = wl.normal_bf16(rng, (4 * H, H), std=1.0 / np.sqrt(H))
    h0 = wl.uniform_bf16(rng, (B, H))
    c0 = rng.uniform(-1.0, 1.0, (B, H)).astype(np.float32)
    dpre, dw, dh0, dc0 = f32_to_dev(pre), to_dev(w_h), to_dev(h0), f32_to_dev(c0)
    print(f"one launch T={T}", flush=True)
    h_seq, c_T, one = rt.lstm_sequence_pre(dpre, dw, dh0, dc0, one_launch=True)
    assert one
    print("step by step", flush=True)
    h2, c2, one2 = rt.lstm_sequence_pre(dpre, dw, dh0, dc0, one_launch=False)
    assert not one2
    assert torch.equal(h_seq, h2) and torch.equal(c_T, c2)
    # the last step from the GPU's state before it (its c through one more step-by-step run of T-1 steps is c2's
    # predecessor; cheaper: redo the last step with the per-step call from the states of the T-1 prefix)
    h_prev = h_seq[T - 2]
    _, c_prev, _ = rt.lstm_sequence_pre(dpre[:T - 1], dw, dh0, dc0, one_launch=True)
    ref_h, ref_c = oracle.lstm_step_pre(pre[T - 1], from_dev(h_prev), w_h.f32, from_dev(c_prev))
    _check(from_dev(h_seq[T - 1]), ref_h, ("h", T))
    _check(from_dev(c_T), ref_c, ("c", T), f32=True)


def test_the_loop_beside_a_busy_stream_is_right_whether_or_not_it_gives_up(rt, nb):
    """Large GEMMs keep every compute unit busy on a second stream while the loop is launched: its workgroups
    may start late or apart, the bounded waits may run out; either way the call returns the step-by-step bits."""
    from gpu_util import f32_to_dev, to_dev
    T, B, H = 64, 2, 512
    pre, w_h, h0, c0 = _case(40, T, B, H)
    dpre, dw, dh0, dc0 = f32_to_dev(pre), to_dev(w_h), to_dev(h0), f32_to_dev(c0)
    want_h, want_c, _ = rt.lstm_sequence_pre(dpre, dw, dh0, dc0, one_launch=False)
    x = torch.empty((8192, 1024), dtype=torch.bfloat16, device="cuda").uniform_(-1, 1)
    w = torch.empty((4096, 1024), dtype=torch.bfloat16, device="cuda").normal_(0, 0.02)
    b = torch.zeros((4096,), dtype=torch.bfloat16, device="cuda")
    y = torch.empty((8192, 4096), dtype=torch.bfloat16, device="cuda")
    side = torch.cuda.Stream()
    torch.cuda.synchronize()
    outcomes = []
    for rep in range(3):
        with torch.cuda.stream(side):
            for _ in range(40):
                rt.dense(x, w, b, nb.EPI_BIAS, out=y)
        print(f"loop beside a busy stream, repetition {rep}", flush=True)
        h, c, one = rt.lstm_sequence_pre(dpre, dw, dh0, dc0, max_polls=1 << 14, one_launch=True)
        outcomes.append(one)
        assert torch.equal(h, want_h) and torch.equal(c, want_c), (rep, one)
        torch.cuda.synchronize()
    print("ran in one launch:", outcomes)

"""Pins for the CPU oracle: things the paper and the mathematics fix, chosen so
that a dropped term, a wrong sign or index, or a transposed operand fails one
of them.  None of these tests touches the GPU path."""
import itertools
import math
import os

import numpy as np
import pytest

import oracle
import workloads as wl

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def _golden_rows(name):
    rows = []
    with open(os.path.join(GOLDEN, name)) as f:
        for line in f:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            rows.append([c.strip() for c in line.split("|")])
    return rows


def _rand(rng, shape):
    return wl.uniform_bf16(rng, shape).f32


# ------------------------------------------------------------------ brute force
def _brute_dense(x, w, b):
    """Pure-Python float64, k outermost (a different loop order than the oracle)."""
    M, K = x.shape
    N = w.shape[0]
    y = [[float(b[n]) for n in range(N)] for _ in range(M)]
    for k in range(K):
        for n in range(N):
            wnk = float(w[n, k])
            for m in range(M):
                y[m][n] += float(x[m, k]) * wnk
    return np.array(y, dtype=np.float64).reshape(M, N)


def test_dense_brute_force_tiny_shapes():
    rng = np.random.default_rng(7)
    shapes = list(itertools.product(range(1, 9), repeat=3)) + [(3, 5, 7), (9, 4, 17)]
    for (M, N, K) in shapes:
        x, w, b = _rand(rng, (M, K)), _rand(rng, (N, K)), _rand(rng, (N,))
        got = oracle.dense(x, w, b, "bias")
        ref = _brute_dense(x, w, b)
        assert got.shape == (M, N)
        assert np.max(np.abs(got - ref)) <= 1e-6 * max(1.0, np.max(np.abs(ref))), (M, N, K)


def test_dense_asymmetric_operands_distinguish_transposes():
    # N != K and a W whose (n,k) and (k,n) readings differ: W[n,k] = 10 n + k.
    M, N, K = 2, 3, 4
    x = np.arange(M * K, dtype=np.float32).reshape(M, K) + 1
    w = (10 * np.arange(N)[:, None] + np.arange(K)[None, :]).astype(np.float32)
    y = oracle.dense(x, w)
    for m in range(M):
        for n in range(N):
            assert y[m, n] == sum(int(x[m, k]) * int(w[n, k]) for k in range(K))


def test_dense_matches_float64_library_matmul():
    rng = np.random.default_rng(11)
    M, N, K = 37, 129, 1024
    x, w, b = _rand(rng, (M, K)), wl.normal_bf16(rng, (N, K)).f32, wl.normal_bf16(rng, (N,)).f32
    ref = x.astype(np.float64) @ w.astype(np.float64).T + b.astype(np.float64)
    got = oracle.dense(x, w, b, "bias")
    # float32 sequential summation: error <= K * 2^-24 * sum|x||w|, far below this bar
    assert oracle.normwise_rel_error(got, ref) < 2e-6


def test_identity_weights_return_input_bit_exact():
    rng = np.random.default_rng(3)
    x = _rand(rng, (19, 64))
    y = oracle.dense(x, np.eye(64, dtype=np.float32))
    assert np.array_equal(y.view(np.uint32), x.view(np.uint32))


def test_permutation_weights_pick_columns():
    # W[n, perm[n]] = 1  =>  Y[:, n] = X[:, perm[n]]
    rng = np.random.default_rng(4)
    K = 16
    perm = rng.permutation(K)
    w = np.zeros((K, K), dtype=np.float32)
    w[np.arange(K), perm] = 1
    x = _rand(rng, (5, K))
    assert np.array_equal(oracle.dense(x, w), x[:, perm])


def test_zero_weights_give_bias_then_gelu_of_bias():
    rng = np.random.default_rng(5)
    x = _rand(rng, (7, 32))
    b = _rand(rng, (48,))
    w = np.zeros((48, 32), dtype=np.float32)
    y = oracle.dense(x, w, b, "bias")
    assert np.array_equal(y, np.broadcast_to(b, (7, 48)))
    yg = oracle.dense(x, w, b, "bias_gelu")
    assert np.array_equal(yg, np.broadcast_to(oracle.gelu(b), (7, 48)))
    # epilogue "none" ignores the bias
    assert np.array_equal(oracle.dense(x, w, b, "none"), np.zeros((7, 48), np.float32))


def test_bias_is_added_before_gelu():
    # x.w = 1 exactly, b = -1  =>  gelu(0) = 0; gelu-then-bias would give gelu(1)-1 != 0
    x = np.ones((1, 1), np.float32)
    w = np.ones((1, 1), np.float32)
    b = -np.ones((1,), np.float32)
    assert oracle.dense(x, w, b, "bias_gelu")[0, 0] == 0.0


def test_power_of_two_scaling_is_exact():
    rng = np.random.default_rng(6)
    x, w = _rand(rng, (9, 200)), _rand(rng, (33, 200))
    assert np.array_equal(oracle.dense(2 * x, w), 2 * oracle.dense(x, w))
    assert np.array_equal(oracle.dense(x, 0.25 * w), 0.25 * oracle.dense(x, w))


def test_row_prefix_invariance_bit_exact():
    # Row m of the result depends only on row m of X: any instantiation of the
    # dynamic M gives the same rows (Section 3.1, sub-shaping).
    rng = np.random.default_rng(8)
    x, w, b = _rand(rng, (67, 96)), _rand(rng, (40, 96)), _rand(rng, (40,))
    full = oracle.dense(x, w, b, "bias_gelu")
    for M in (1, 2, 15, 16, 17, 33, 66):
        assert np.array_equal(oracle.dense(x[:M], w, b, "bias_gelu"), full[:M])


# ------------------------------------------------------------------ GELU
def test_gelu_properties_and_float64_erf():
    assert oracle.gelu(np.zeros(1))[0] == 0.0
    x = np.linspace(-8, 8, 3201).astype(np.float32)
    g = oracle.gelu(x)
    ref = np.array([0.5 * v * (1 + math.erf(v / math.sqrt(2))) for v in x.astype(np.float64)])
    # float32 evaluation: a couple of units in the last place of the result
    assert np.all(np.abs(g - ref) <= 1.2e-7 * np.maximum(1.0, np.abs(ref)) + 1e-7)
    # gelu(x) - gelu(-x) = x
    assert np.max(np.abs((g - oracle.gelu(-x)) - x)) < 1e-6
    big = np.array([6, 7, 10, 50], np.float32)
    assert np.allclose(oracle.gelu(big), big, rtol=0, atol=1e-7 * 50)
    assert np.max(np.abs(oracle.gelu(-big))) < 1e-7
    # it is the erf form, not the tanh approximation (they differ by about 1e-4 at x = 2)
    v = np.float32(2.0)
    tanh_form = 0.5 * v * (1 + math.tanh(math.sqrt(2 / math.pi) * (v + 0.044715 * v ** 3)))
    assert abs(float(oracle.gelu(np.array([v]))[0]) - 1.9544997361) < 1e-6
    assert abs(tanh_form - 1.9544997361) > 5e-5


# ------------------------------------------------------------------ batch_matmul
def _brute_bmm(a, b, trans_b, alpha):
    T, M, K = a.shape
    N = b.shape[1] if trans_b else b.shape[2]
    c = np.zeros((T, M, N))
    for t in range(T):
        for n in range(N):
            for m in range(M):
                s = 0.0
                for k in range(K):
                    s += float(a[t, m, k]) * float(b[t, n, k] if trans_b else b[t, k, n])
                c[t, m, n] = alpha * s
    return c


@pytest.mark.parametrize("trans_b", [True, False])
def test_bmm_brute_force(trans_b):
    rng = np.random.default_rng(12)
    for (T, M, N, K) in [(1, 1, 1, 1), (2, 3, 5, 7), (3, 9, 4, 17), (2, 8, 8, 8), (1, 5, 2, 3)]:
        a = _rand(rng, (T, M, K))
        b = _rand(rng, (T, N, K) if trans_b else (T, K, N))
        got = oracle.batch_matmul(a, b, trans_b, 0.125)
        ref = _brute_bmm(a, b, trans_b, 0.125)
        assert got.shape == (T, M, N)
        assert np.max(np.abs(got - ref)) < 1e-6 * max(1.0, np.abs(ref).max())


def test_bmm_batch1_alpha1_equals_dense():
    rng = np.random.default_rng(13)
    a, b = _rand(rng, (1, 21, 40)), _rand(rng, (1, 13, 40))
    assert np.array_equal(oracle.batch_matmul(a, b, True, 1.0)[0], oracle.dense(a[0], b[0]))
    # NN reading of the same product
    bt = np.ascontiguousarray(b.transpose(0, 2, 1))
    assert np.array_equal(oracle.batch_matmul(a, bt, False, 1.0)[0], oracle.dense(a[0], b[0]))


def test_bmm_batches_are_independent():
    rng = np.random.default_rng(14)
    a, b = _rand(rng, (3, 6, 10)), _rand(rng, (3, 4, 10))
    c = oracle.batch_matmul(a, b, True, 1.0)
    for t in range(3):
        assert np.array_equal(c[t], oracle.batch_matmul(a[t:t + 1], b[t:t + 1], True, 1.0)[0])


# ------------------------------------------------------------------ softmax / attention
def test_softmax_rows_sum_to_one_and_shift_invariant():
    rng = np.random.default_rng(15)
    s = (8 * _rand(rng, (12, 37, 41))).astype(np.float32)
    p = oracle.softmax_rows(s)
    assert np.max(np.abs(p.sum(-1, dtype=np.float64) - 1)) < 1e-6
    assert np.all(p >= 0)
    # adding a row constant representable without rounding keeps the result
    p2 = oracle.softmax_rows(s + np.float32(64.0))
    assert np.max(np.abs(p2 - p)) < 1e-5
    # known values: softmax([0, ln 2, ln 5]) = [1, 2, 5] / 8
    row = np.array([[0.0, math.log(2.0), math.log(5.0)]], np.float32)
    assert np.allclose(oracle.softmax_rows(row), [[0.125, 0.25, 0.625]], atol=1e-7)
    # the order of a row is respected (largest score, largest probability)
    assert np.array_equal(np.argmax(p, -1), np.argmax(s, -1))


def test_attention_length_one_returns_v():
    q, k, v = (wl.uniform_bf16(np.random.default_rng(16 + i), (12, 1, 64)).f32 for i in range(3))
    s, p, o = oracle.attention(q, k, v)
    assert np.array_equal(p, np.ones((12, 1, 1), np.float32))
    assert np.array_equal(o, v)


def test_attention_zero_query_gives_column_mean_of_v():
    rng = np.random.default_rng(17)
    L = 8  # power of two: 1/L and the sum of L equal terms are exact
    q = np.zeros((12, L, 64), np.float32)
    k, v = _rand(rng, (12, L, 64)), _rand(rng, (12, L, 64))
    s, p, o = oracle.attention(q, k, v)
    assert np.array_equal(s, np.zeros_like(s))
    assert np.array_equal(p, np.full_like(p, 1.0 / L))
    ref = v.astype(np.float64).mean(axis=1, keepdims=True)
    assert np.max(np.abs(o - ref)) < 1e-6


def test_attention_scale_is_one_eighth_and_nt_layout():
    # one-hot Q and K rows: S[i,j] = alpha * [d_i == d_j]
    L = 5
    q = np.zeros((1, L, 64), np.float32)
    k = np.zeros((1, L, 64), np.float32)
    for i in range(L):
        q[0, i, i] = 1
        k[0, i, (i + 1) % L] = 1
    s, _, _ = oracle.attention(q, k, np.zeros((1, L, 64), np.float32))
    expect = np.zeros((L, L), np.float32)
    for i in range(L):
        expect[i, (i - 1) % L] = 0.125  # K row j has its one at (j+1)%L == i  =>  j = i-1
    assert np.array_equal(s[0], expect)


def test_attention_matches_float64_library():
    q, k, v = (a.f32 for a in wl.config4_qkv(0, 37))
    s, p, o = oracle.attention(q, k, v)
    q64, k64, v64 = (a.astype(np.float64) for a in (q, k, v))
    s64 = np.einsum("hid,hjd->hij", q64, k64) / 8
    e = np.exp(s64 - s64.max(-1, keepdims=True))
    p64 = e / e.sum(-1, keepdims=True)
    o64 = np.einsum("hij,hjd->hid", p64, v64)
    assert oracle.normwise_rel_error(s, s64) < 1e-6
    assert oracle.normwise_rel_error(p, p64) < 1e-5
    assert oracle.normwise_rel_error(o, o64) < 1e-5


# ------------------------------------------------------------------ LSTM cell
H, IX = 8, 6


def _lstm_zero():
    return np.zeros((4 * H, IX + H), np.float32), np.zeros((4 * H,), np.float32)


def test_lstm_zero_weights_closed_form_over_128_steps():
    rng = np.random.default_rng(18)
    w, b = _lstm_zero()
    B = 3
    c0 = _rand(rng, (B, H))
    c, h = c0.copy(), np.zeros((B, H), np.float32)
    for t in range(1, 129):
        x = _rand(rng, (B, IX))
        h, c = oracle.lstm_step(x, h, w, b, c)
        # i = f = o = 1/2, g = 0  =>  c_t = c_0 2^-t exactly, h_t = tanh(c_t) / 2
        assert np.array_equal(c, np.ldexp(c0, -t))
        assert np.max(np.abs(h - 0.5 * np.tanh(c.astype(np.float64)))) < 1e-7


def test_lstm_gate_blocks_are_i_f_g_o():
    rng = np.random.default_rng(19)
    B = 2
    x, h0 = _rand(rng, (B, IX)), _rand(rng, (B, H))
    c0 = _rand(rng, (B, H))
    w, _ = _lstm_zero()
    big = 30.0

    def run(**blocks):
        b = np.zeros((4 * H,), np.float32)
        for name, val in blocks.items():
            j = "ifgo".index(name)
            b[j * H:(j + 1) * H] = val
        return oracle.lstm_step(x, h0, w, b, c0)

    c64 = c0.astype(np.float64)
    # forget gate open, input gate shut: the cell state is carried over unchanged
    h, c = run(f=big, i=-big)
    assert np.max(np.abs(c - c0)) < 1e-7
    assert np.max(np.abs(h - 0.5 * np.tanh(c64))) < 1e-7
    # output gate open only: c' = c/2, h' = tanh(c/2)
    h, c = run(o=big)
    assert np.array_equal(c, c0 / 2)
    assert np.max(np.abs(h - np.tanh(c64 / 2))) < 1e-7
    # candidate saturated: c' = c/2 + 1/2
    h, c = run(g=big)
    assert np.max(np.abs(c - (c64 / 2 + 0.5))) < 1e-7
    # input gate open and candidate saturated, forget shut: c' = 1
    h, c = run(i=big, g=big, f=-big)
    assert np.max(np.abs(c - 1.0)) < 1e-6
    assert np.max(np.abs(h - 0.5 * math.tanh(1.0))) < 1e-6
    # candidate negative: sign of tanh(g) survives
    h, c = run(i=big, g=-big, f=-big)
    assert np.max(np.abs(c + 1.0)) < 1e-6


def test_lstm_input_and_hidden_columns_of_w():
    # A single one in the g block picks x[:,a] (column a) or h[:,a] (column Ix+a).
    rng = np.random.default_rng(20)
    B = 4
    x, h0 = _rand(rng, (B, IX)), _rand(rng, (B, H))
    c0 = np.zeros((B, H), np.float32)
    for src, a in (("x", 2), ("h", 5)):
        w, b = _lstm_zero()
        col = a if src == "x" else IX + a
        w[2 * H + 3, col] = 1.0  # hidden unit 3 of the g block
        hn, cn = oracle.lstm_step(x, h0, w, b, c0)
        val = (x[:, a] if src == "x" else h0[:, a]).astype(np.float64)
        assert np.max(np.abs(cn[:, 3] - 0.5 * np.tanh(val))) < 1e-7
        others = np.delete(cn, 3, axis=1)
        assert np.array_equal(others, np.zeros_like(others))


def test_lstm_gates_are_the_dense_of_the_concatenation():
    rng = np.random.default_rng(21)
    B = 5
    x, h0, c0 = _rand(rng, (B, IX)), _rand(rng, (B, H)), _rand(rng, (B, H))
    w, b = _rand(rng, (4 * H, IX + H)), _rand(rng, (4 * H,))
    hn, cn = oracle.lstm_step(x, h0, w, b, c0)
    g = oracle.dense(np.concatenate([x, h0], 1), w, b, "bias").astype(np.float64)
    sg = lambda z: 1 / (1 + np.exp(-z))
    i, f, gg, o = (g[:, j * H:(j + 1) * H] for j in range(4))
    c_ref = sg(f) * c0 + sg(i) * np.tanh(gg)
    assert np.max(np.abs(cn - c_ref)) < 1e-6
    assert np.max(np.abs(hn - sg(o) * np.tanh(c_ref))) < 1e-6


# ------------------------------------------------------------------ LSTM cell, input share of the gates given
def test_lstm_pre_closed_forms_and_gate_blocks():
    rng = np.random.default_rng(22)
    B = 3
    h0, c0 = _rand(rng, (B, H)), _rand(rng, (B, H))
    wh = np.zeros((4 * H, H), np.float32)
    big = 30.0
    c64 = c0.astype(np.float64)

    def run(**blocks):
        pre = np.zeros((B, 4 * H), np.float32)
        for name, val in blocks.items():
            j = "ifgo".index(name)
            pre[:, j * H:(j + 1) * H] = val
        return oracle.lstm_step_pre(pre, h0, wh, c0)

    h, c = run()  # all gates 0: i = f = o = 1/2, g = 0
    assert np.array_equal(c, c0 / 2)
    assert np.max(np.abs(h - 0.5 * np.tanh(c64 / 2))) < 1e-7
    h, c = run(f=big, i=-big)  # carried over
    assert np.max(np.abs(c - c0)) < 1e-7
    h, c = run(o=big)
    assert np.max(np.abs(h - np.tanh(c64 / 2))) < 1e-7
    h, c = run(i=big, g=-big, f=-big)
    assert np.max(np.abs(c + 1.0)) < 1e-6


def test_lstm_pre_recurrent_weight_indexing():
    # a single one at row (g block, unit 3), column a of wh picks h[:, a]; pre is per row AND per gate column
    rng = np.random.default_rng(23)
    B = 4
    h0 = _rand(rng, (B, H))
    c0 = np.zeros((B, H), np.float32)
    wh = np.zeros((4 * H, H), np.float32)
    wh[2 * H + 3, 5] = 1.0
    pre = np.zeros((B, 4 * H), np.float32)
    hn, cn = oracle.lstm_step_pre(pre, h0, wh, c0)
    assert np.max(np.abs(cn[:, 3] - 0.5 * np.tanh(h0[:, 5].astype(np.float64)))) < 1e-7
    assert np.array_equal(np.delete(cn, 3, axis=1), np.zeros((B, H - 1), np.float32))
    # pre is added, not overwritten: the same unit with pre = -h[:,5] gives g = 0
    pre[:, 2 * H + 3] = -h0[:, 5]
    hn, cn = oracle.lstm_step_pre(pre, h0, wh, c0)
    assert np.array_equal(cn, np.zeros_like(cn))
    # pre of one row only moves that row
    pre = np.zeros((B, 4 * H), np.float32)
    pre[1, 2 * H + 6] = 30.0
    wh[:] = 0
    hn, cn = oracle.lstm_step_pre(pre, h0, wh, c0)
    assert abs(cn[1, 6] - 0.5) < 1e-7 and np.count_nonzero(cn) == 1


def test_lstm_pre_equals_the_fused_cell_when_pre_is_the_input_product():
    # [x | h] . W^T + b = (x . Wx^T + b) + h . Wh^T: the step from precomputed input gates must
    # agree with the fused step (pinned above) up to the order of the float32 additions.
    rng = np.random.default_rng(24)
    B = 5
    x, h0, c0 = _rand(rng, (B, IX)), _rand(rng, (B, H)), _rand(rng, (B, H))
    w, b = _rand(rng, (4 * H, IX + H)), _rand(rng, (4 * H,))
    h_ref, c_ref = oracle.lstm_step(x, h0, w, b, c0)
    pre = oracle.dense(x, np.ascontiguousarray(w[:, :IX]), b, "bias")
    hn, cn = oracle.lstm_step_pre(pre, h0, np.ascontiguousarray(w[:, IX:]), c0)
    assert np.max(np.abs(cn - c_ref)) < 2e-6
    assert np.max(np.abs(hn - h_ref)) < 2e-6
    with pytest.raises(oracle.OracleShapeError):
        oracle.lstm_step_pre(pre[:, :-1], h0, w[:, IX:], c0)


# ------------------------------------------------------------------ integer side
def test_dense_shape_function_every_M_up_to_513():
    for M in range(0, 514):
        out = oracle.dense_shape((M, 1024), (4096, 1024))
        assert out == (M, 4096)
        assert all(isinstance(v, int) for v in out)


def test_dense_shape_function_checks_the_type_relation():
    with pytest.raises(oracle.OracleShapeError):
        oracle.dense_shape((5, 128), (128, 127))
    with pytest.raises(oracle.OracleShapeError):
        oracle.dense_shape((5, 128, 1), (128, 128))
    with pytest.raises(ValueError):
        oracle.dense_shape((-1, 128), (128, 128))
    with pytest.raises(oracle.OracleShapeError):
        oracle.dense(np.zeros((3, 4), np.float32), np.zeros((5, 6), np.float32))


def test_subshape_example_from_the_paper():
    for M, K, N in ((int(a), int(b), int(c)) for a, b, c in _golden_rows("subshape_example.txt")):
        assert oracle.dense_shape((M, K), (N, K)) == (M, N)


def test_batch_matmul_shape_function():
    for L in (1, 7, 512):
        assert oracle.batch_matmul_shape((12, L, 64), (12, L, 64), True) == (12, L, L)
        assert oracle.batch_matmul_shape((12, L, L), (12, L, 64), False) == (12, L, 64)
    with pytest.raises(oracle.OracleShapeError):
        oracle.batch_matmul_shape((12, 5, 64), (11, 5, 64), True)
    with pytest.raises(oracle.OracleShapeError):
        oracle.batch_matmul_shape((12, 5, 64), (12, 5, 64), False)  # K = 64 vs 5
    with pytest.raises(oracle.OracleShapeError):
        oracle.batch_matmul_shape((12, 5, 64), (12, 9, 63), True)
    with pytest.raises(oracle.OracleShapeError):
        oracle.batch_matmul_shape((5, 64), (12, 9, 64), True)


def test_lstm_shape_function():
    for B in (0, 1, 33, 64):
        assert oracle.lstm_shape((B, 512), (B, 512), (B, 512), (2048, 1024)) == ((B, 512), (B, 512))
    for bad in [((3, 512), (4, 512), (3, 512), (2048, 1024)),
                ((3, 512), (3, 512), (3, 511), (2048, 1024)),
                ((3, 512), (3, 512), (3, 512), (2047, 1024)),
                ((3, 512), (3, 512), (3, 512), (2048, 1023))]:
        with pytest.raises(oracle.OracleShapeError):
            oracle.lstm_shape(*bad)


def test_storage_bytes_values_printed_in_the_paper():
    for shape, itemsize, nbytes, _align in _golden_rows("storage_sizes.txt"):
        dims = [int(d) for d in shape.split(",")]
        assert oracle.storage_bytes(dims, int(itemsize)) == int(nbytes)
    assert oracle.storage_bytes((0, 4096), 2) == 0
    assert oracle.storage_bytes((16384, 4096), 2) == 16384 * 4096 * 2
    assert oracle.storage_bytes((), 4) == 4


def test_residue_split_identity_and_paper_example():
    for tile, copies, rmin, rmax in ([int(v) for v in row] for row in _golden_rows("residue_tile8.txt")):
        seen = set()
        for x in range(0, 2 * tile + 2):
            k, r = oracle.residue_split(x, tile)
            assert tile * k + r == x and rmin <= r <= rmax and k == x // tile
            seen.add(r)
        assert len(seen) == copies
    for tile in (16, 32, 64, 128, 256):
        for x in range(0, 2 * tile + 2):
            k, r = oracle.residue_split(x, tile)
            assert tile * k + r == x and 0 <= r < tile
            assert (k + (1 if r else 0)) * tile >= x  # ceil(x/tile) tiles cover x
    with pytest.raises(ValueError):
        oracle.residue_split(5, 0)
    with pytest.raises(ValueError):
        oracle.residue_split(-1, 8)


# ------------------------------------------------------------------ generators
def test_bf16_rounding_is_nearest_even_and_round_trips():
    # 1 + 2^-8 is exactly between 1 and 1 + 2^-7: ties go to the even mantissa (1.0)
    a = np.array([1.0 + 2.0 ** -8, 1.0 + 3 * 2.0 ** -8, 1.0 + 2.0 ** -8 + 2.0 ** -20, -0.0, 0.5], np.float32)
    bits = wl.f32_to_bf16_bits(a)
    back = wl.bf16_bits_to_f32(bits)
    assert back[0] == 1.0
    assert back[1] == 1.0 + 2.0 ** -6  # tie between 1+2^-7 and 1+2^-6 goes to even (1+2^-6)
    assert back[2] == 1.0 + 2.0 ** -7
    assert bits[3] == 0x8000 and back[4] == 0.5
    allbits = np.arange(0, 0x7F80, dtype=np.uint16)  # every finite non-negative bf16
    assert np.array_equal(wl.f32_to_bf16_bits(wl.bf16_bits_to_f32(allbits)), allbits)


def test_workload_draws_are_seeded_and_in_range():
    a, b = wl.config5_token_counts(), wl.config5_token_counts()
    assert np.array_equal(a, b) and a.min() >= 32 and a.max() <= 16384
    calls = wl.config1_calls()
    assert len(calls) == 64 and all(1 <= c.M <= 64 and c.N == 128 and c.K == 128 for c in calls)
    assert np.all(np.abs(calls[0].x.f32) <= 1.0)
    L = wl.config3_lengths()
    assert len(L) == 100 and L.min() >= 1 and L.max() <= 512
    w = wl.config2_weights()
    assert w.w.shape == (2048, 1024) and abs(float(w.w.f32.std()) - 0.02) < 1e-3


# ------------------------------------------------------------------ the yardsticks themselves
def test_normwise_rel_error_known_answers():
    """||got - ref||_F / ||ref||_F on hand-computed cases (3-4-5 triangles): a metric that
    returned too small a value would let every parity test pass."""
    e = oracle.normwise_rel_error
    assert e([3.0, 4.0], [3.0, 4.0]) == 0.0
    assert e([0.0, 0.0], [3.0, 4.0]) == 1.0                     # ||ref|| / ||ref||
    assert e([3.0, 4.0], [0.0, 0.0]) == float("inf")            # zero reference, non-zero output
    assert e([0.0, 0.0], [0.0, 0.0]) == 0.0
    assert e([6.0, 8.0], [3.0, 4.0]) == 1.0                     # got = 2 ref: ||ref|| / ||ref||
    assert e([3.0, 0.0], [0.0, 4.0]) == 1.25                    # ||(3,-4)|| / 4 = 5/4
    eps = 2.0 ** -10
    assert e([1.0, eps, 0.0, 0.0], [1.0, 0.0, 0.0, 0.0]) == eps
    # relative: scaling both by 1000 (or by 2^-40) changes nothing; it is not symmetric in its arguments
    assert e([3000.0, 0.0], [0.0, 4000.0]) == 1.25
    assert e(np.ldexp([3.0, 0.0], -40), np.ldexp([0.0, 4.0], -40)) == 1.25
    assert e([0.0, 4.0], [3.0, 0.0]) == 5.0 / 3.0
    # the Frobenius norm runs over every element of a matrix, whatever its shape, in float64
    got = np.zeros((4, 6), np.float32)
    ref = np.zeros((4, 6), np.float32)
    ref[1, 2], ref[3, 5] = 3.0, 4.0
    got[1, 2], got[3, 5], got[0, 0] = 3.0, 4.0, 12.0            # one wrong element of size 12: 12/5
    assert e(got, ref) == 2.4
    assert e(got.reshape(2, 12), ref.reshape(2, 12)) == 2.4
    # one element off by d among n equal ones: d / sqrt(n)
    ref = np.ones(10000)
    got = ref.copy()
    got[1234] += 0.5
    assert abs(e(got, ref) - 0.005) < 1e-15


def test_maxnorm_rel_error_known_answers():
    m = oracle.maxnorm_rel_error
    assert m([3.0, 4.0], [3.0, 4.0]) == 0.0
    assert m([0.0, 0.0], [3.0, 4.0]) == 1.0                     # max|d| = 4, max|ref| = 4
    assert m([3.0, 5.0], [3.0, 4.0]) == 0.25
    assert m([4.0, 4.0], [3.0, -4.0]) == 2.0                    # the sign matters: |4 - (-4)| / 4
    assert m([1.0], [0.0]) == float("inf") and m([0.0], [0.0]) == 0.0 and m([], []) == 0.0
    assert m([3000.0, 5000.0], [3000.0, 4000.0]) == 0.25        # relative
    # a single wrong element sets it, however many right ones surround it
    ref = np.ones((100, 100))
    got = ref.copy()
    got[7, 9] = 1.5
    assert m(got, ref) == 0.5


def test_elementwise_excess_known_answers():
    x = oracle.elementwise_excess
    ref = np.array([3.0, -4.0, 0.0, 5.0])                        # rms = sqrt(50 / 4)
    rms = np.sqrt(12.5)
    assert x(ref, ref, 0.01, 0.01) == 0.0
    got = ref + np.array([0.0, 0.0, 0.5, 0.0])                   # an element whose reference is 0: only the floor allows it
    assert abs(x(got, ref, 0.01, 0.01) - 0.5 / (0.01 * rms)) < 1e-12
    got = ref + np.array([0.0, 0.08, 0.0, 0.0])                  # |d| = 0.08 at |ref| = 4
    assert abs(x(got, ref, 0.01, 0.0) - 2.0) < 1e-12             # twice the allowed 1 %
    assert abs(x(got, ref, 0.02, 0.0) - 1.0) < 1e-12             # exactly at the bound
    assert abs(x(got, ref, 0.0, 0.01) - 0.08 / (0.01 * rms)) < 1e-12
    # the maximum over elements, not a mean: one bad element among a million good ones shows fully
    ref = np.ones(1_000_000)
    got = ref.copy()
    got[123456] = 1.5
    assert abs(x(got, ref, 0.25, 0.25) - 1.0) < 1e-12
    assert oracle.normwise_rel_error(got, ref) == 0.0005        # where the norm alone would have passed 5e-3
    assert x([0.0, 1e-30], [0.0, 0.0], 0.5, 0.5) == float("inf") and x([0.0], [0.0], 0.5, 0.5) == 0.0
    assert x(2 * ref, 2 * got, 0.25, 0.25) > 0                  # arguments are (got, ref), both scale together
    assert abs(x(1000 * got, 1000 * ref, 0.25, 0.25) - 1.0) < 1e-9


def test_lstm_pre_shape_function():
    """The cell with a precomputed input share is the fused cell with no input columns: its shape
    function accepts exactly what the fused one accepts for x of width 0, with pre = (B, 4H)."""
    for B in (0, 1, 16, 33):
        for H in (8, 24, 512):
            assert oracle.lstm_pre_shape((B, 4 * H), (B, H), (B, H), (4 * H, H)) == ((B, H), (B, H))
            assert oracle.lstm_shape((B, 0), (B, H), (B, H), (4 * H, H)) == ((B, H), (B, H))
            for bad_h, bad_c, bad_w in [((B + 1, H), (B, H), (4 * H, H)), ((B, H), (B, H + 8), (4 * H, H)),
                                        ((B, H), (B, H), (4 * H + 1, H)), ((B, H), (B, H), (4 * H, H + 1))]:
                with pytest.raises(oracle.OracleShapeError):
                    oracle.lstm_pre_shape((B, 4 * H), bad_h, bad_c, bad_w)
                with pytest.raises(oracle.OracleShapeError):
                    oracle.lstm_shape((B, 0), bad_h, bad_c, bad_w)
            for bad_pre in [(B + 1, 4 * H), (B, 4 * H - 1), (B, H)]:
                with pytest.raises(oracle.OracleShapeError):
                    oracle.lstm_pre_shape(bad_pre, (B, H), (B, H), (4 * H, H))
    with pytest.raises(oracle.OracleShapeError):
        oracle.lstm_pre_shape((3, 32, 1), (3, 8), (3, 8), (32, 8))


def test_lstm_seq_shape_function():
    """Known answers: T is taken from pre, B and H from h0, every other extent must agree."""
    assert oracle.lstm_seq_shape((7, 3, 32), (3, 8), (3, 8), (32, 8)) == ((7, 3, 8), (3, 8))
    assert oracle.lstm_seq_shape((0, 1, 2048), (1, 512), (1, 512), (2048, 512)) == ((0, 1, 512), (1, 512))
    for bad in [((7, 4, 32), (3, 8), (3, 8), (32, 8)), ((7, 3, 31), (3, 8), (3, 8), (32, 8)),
                ((7, 3, 32), (3, 8), (3, 9), (32, 8)), ((7, 3, 32), (3, 8), (3, 8), (32, 9)),
                ((7, 3, 32), (3, 8), (3, 8), (8, 32)), ((3, 32), (3, 8), (3, 8), (32, 8))]:
        with pytest.raises(oracle.OracleShapeError):
            oracle.lstm_seq_shape(*bad)
    with pytest.raises(ValueError):
        oracle.lstm_seq_shape((-1, 3, 32), (3, 8), (3, 8), (32, 8))

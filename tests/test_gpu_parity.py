"""Parity of the HIP path with the CPU oracle, element by element, on the same
seeded bf16-rounded inputs.  Bar: max normwise relative error 5e-3 per call
(||gpu - ref||_F / ||ref||_F over the call's whole output) AND, for every single
element, |gpu - ref| <= rel |ref| + floor rms(ref) with rel = floor = 2^-7 for
bf16 outputs (four times the 2^-9 half-ulp of a correctly rounded result; the
rms term covers elements that cancel to near zero), 2^-14 for f32 outputs
(summation order only), 2^-11 for f32 outputs behind the GELU epilogue (whose
fitted form deviates by up to 2.5e-5 from the erf form); shape outputs bit-exact.
The largest max|d| / max|ref| seen per test is printed (run with -s)."""
import numpy as np
import pytest

import oracle
import workloads as wl

torch = pytest.importorskip("torch")
pytestmark = pytest.mark.gpu

TOL = 5e-3
EPI = {"none": 0, "bias": 1, "bias_gelu": 2}
TILED = {2: (32, 128), 3: (64, 128), 4: (128, 128), 5: (256, 128), 6: (256, 256)}


@pytest.fixture(scope="module")
def rt():
    import paper_2006_03031_amd as nb
    from paper_2006_03031_amd import runtime
    nb.load()  # fails loudly if the HIP library is not built
    return runtime


@pytest.fixture(scope="module")
def nb():
    import paper_2006_03031_amd as nb
    return nb


def _dev():
    from gpu_util import bits_from_dev, f32_to_dev, from_dev, to_dev
    return to_dev, f32_to_dev, from_dev, bits_from_dev


def _err(got, ref):
    return oracle.normwise_rel_error(got, ref)


GATE_BF16 = 2.0 ** -7
GATE_F32 = 2.0 ** -14
GATE_F32_GELU = 2.0 ** -11
_worst = {"fro": 0.0, "inf": 0.0, "elem": 0.0}


def _check(got, ref, what=None, f32=False, gelu=False, floor=None):
    """The parity gate of one call: the Frobenius ratio within 5e-3 and every element within the
    element-wise bound (see the module docstring); returns the Frobenius ratio."""
    rel = (GATE_F32_GELU if gelu else GATE_F32) if f32 else GATE_BF16
    e = oracle.normwise_rel_error(got, ref)
    assert e <= TOL, ("normwise", what, e)
    x = oracle.elementwise_excess(got, ref, rel, rel if floor is None else floor)
    assert x <= 1.0, ("element-wise", what, x, rel)
    _worst["fro"] = max(_worst["fro"], e)
    _worst["inf"] = max(_worst["inf"], oracle.maxnorm_rel_error(got, ref))
    _worst["elem"] = max(_worst["elem"], x)
    return e


@pytest.fixture(autouse=True)
def _report_worst(request):
    _worst.update(fro=0.0, inf=0.0, elem=0.0)
    yield
    if _worst["fro"] > 0.0:
        print(f"\n[{request.node.name}] worst ||d||_F/||ref||_F = {_worst['fro']:.3e}, "
              f"max|d|/max|ref| = {_worst['inf']:.3e}, element-wise bound used up to {_worst['elem']:.2f}")


# ------------------------------------------------------------------ config 1
def test_config1_all_64_calls(rt, nb):
    to_dev, _, from_dev, _ = _dev()
    calls = wl.config1_calls()
    w, b = to_dev(calls[0].w), to_dev(calls[0].b)
    worst = 0.0
    for c in calls:
        x = to_dev(c.x)
        y = rt.dense(x, w, b, nb.EPI_BIAS)
        assert tuple(y.shape) == oracle.dense_shape(c.x.shape, c.w.shape)
        ref = oracle.dense(c.x.f32, c.w.f32, c.b.f32, "bias")
        worst = max(worst, _check(from_dev(y), ref, ("config1", c.M)))
    assert worst <= TOL, worst


# ------------------------------------------------------------------ residue sweeps
def _sweep(rt, nb, variant, N, K, Ms, epilogue="bias_gelu", out_dtype=0, seed=0):
    """One oracle evaluation at max(Ms) rows serves every M by row-prefix invariance.
    The output buffer carries a guard band that must stay untouched."""
    to_dev, _, from_dev, _ = _dev()
    rng = np.random.default_rng([99, seed, N, K])
    Mmax = max(Ms)
    x = wl.uniform_bf16(rng, (Mmax, K))
    w = wl.normal_bf16(rng, (N, K), std=0.05)
    b = wl.uniform_bf16(rng, (N,))
    ref = oracle.dense(x.f32, w.f32, b.f32, epilogue)
    xd, wd, bd = to_dev(x), to_dev(w), to_dev(b)
    tdt = torch.bfloat16 if out_dtype == 0 else torch.float32
    guard = 3
    worst = 0.0
    for M in Ms:
        buf = torch.full((M + guard, N), 768.0, dtype=tdt, device="cuda")
        rt.dense(xd[:M], wd, bd, EPI[epilogue], out_dtype, variant, out=buf[:M])
        got = from_dev(buf)
        assert np.all(got[M:] == 768.0), f"variant {variant} wrote past row M={M}"
        e = _check(got[:M], ref[:M], (variant, M, N, K, epilogue), f32=out_dtype == 1, gelu=epilogue == "bias_gelu")
        worst = max(worst, e)
    return worst


@pytest.mark.parametrize("variant", sorted(TILED))
def test_tiled_variants_every_residue(rt, nb, variant):
    bm, bn = TILED[variant]
    # every M from 1 to 2*tile+1: r takes every value, k = 0, 1, 2
    _sweep(rt, nb, variant, N=bn * 2, K=128, Ms=range(1, 2 * bm + 2))


@pytest.mark.parametrize("variant", sorted(TILED))
def test_tiled_variants_ragged_N_and_K(rt, nb, variant):
    bm, bn = TILED[variant]
    Ms = [1, bm - 1, bm, bm + 1, 2 * bm + 1]
    _sweep(rt, nb, variant, N=bn + 72, K=200, Ms=Ms, epilogue="bias")          # N % 4 == 0, K % 64 != 0
    _sweep(rt, nb, variant, N=bn + 37, K=72, Ms=Ms, epilogue="bias_gelu")      # N odd: element-wise tail
    _sweep(rt, nb, variant, N=24, K=8, Ms=Ms, epilogue="none", out_dtype=1)    # one partial tile, f32 out
    _sweep(rt, nb, variant, N=bn + 6, K=1024, Ms=Ms, epilogue="bias", out_dtype=1)


@pytest.mark.parametrize("rows", [128, 160, 192, 224, 288, 320])
def test_tile_heights_of_the_256_wide_variant_every_residue(rt, nb, rows):
    # the 256 x 256 variant at its other tile heights: every residue M mod rows, k = 0, 1, 2,
    # heights that are not a whole number of load passes (160, 192, 224, 288, 320 vs passes of 128)
    forced = 6 | ((rows // 16) << 16)
    p = nb.dense_plan(rows + 1, 512, 128, force_variant=forced)
    assert (p.variant, p.bm, p.k, p.r, p.residue_copy) == (6, rows, 1, 1, 1)
    _sweep(rt, nb, forced, N=512, K=128, Ms=range(1, 2 * rows + 2))
    for K in (32, 96, 160, 1024):   # fewer stages than ring slots, odd counts, a long K
        _sweep(rt, nb, forced, N=256, K=K, Ms=[rows, rows + 5, 3 * rows - 1], epilogue="bias", out_dtype=1)


def test_auto_dispatch_picks_a_tile_height_that_fills_the_rounds(rt, nb):
    # BERT-large FFN2 just past 8192 rows: one round of 160-row tiles instead of two rounds
    p = nb.dense_plan(8300, 1024, 4096)
    assert p.variant == 6 and p.bm in (128, 160, 192) and p.grid[0] <= 256 and p.split_rows == 0
    # FFN1 just past two rounds of 256-row tiles: taller tiles keep it at two rounds
    p = nb.dense_plan(8300, 4096, 1024, nb.EPI_BIAS_GELU_ERF)
    if p.split_rows == 0:
        assert p.variant == 6 and p.bm in (288, 320) and p.grid[0] <= 512
    to_dev, _, from_dev, _ = _dev()
    for (M, N, K, epi) in [(8300, 1024, 4096, "bias"), (2100, 4096, 1024, "bias_gelu")]:
        rng = np.random.default_rng([5, M])
        x, w, b = wl.uniform_bf16(rng, (M, K)), wl.normal_bf16(rng, (N, K)), wl.uniform_bf16(rng, (N,))
        y = rt.dense(to_dev(x), to_dev(w), to_dev(b), EPI[epi])
        rows = np.r_[0:3, M // 2:M // 2 + 3, M - 260:M]   # sampled rows, the last tile row included
        ref = oracle.dense(x.f32[rows], w.f32, b.f32, epi)
        _check(from_dev(y)[rows], ref, (M, N, K))


@pytest.mark.parametrize("variant", sorted(TILED))
def test_ring_variants_short_and_odd_stage_counts(rt, nb, variant):
    # K of 1, 2, 3, 5 and 9 stages of 32 (the 32-wide ring) and of 1 to 4 stages of 64 (the 64-wide
    # ring with two or three slots): the pipeline prologue, the tail waits, the loads that are or
    # are not issued past the end of K and the ping-pong barrier count must hold when there are
    # fewer stages than ring slots
    bm, bn = TILED[variant]
    for K in (32, 64, 96, 128, 160, 192, 256, 288):
        _sweep(rt, nb, variant, N=bn, K=K, Ms=[bm, bm + 5, 2 * bm], epilogue="bias")


@pytest.mark.parametrize("variant", sorted(TILED))
def test_tile_walk_more_tiles_than_resident_workgroups(rt, nb, variant):
    """Launches with more tiles than workgroups resident at once (256 for the 8-wave tiles, 512 for
    the smaller ones): every workgroup walks several tiles, ragged last tile row and ragged N
    included, on both ring widths (K = 192 is whole 64-wide stages, K = 160 is not)."""
    bm, bn = TILED[variant]
    resident = 512 if bm <= 128 and bn == 128 else 256
    tiles_n = 5 if bn == 128 else 3
    rows = (2 * resident // tiles_n + 3) * bm + 1     # > 2 tiles per workgroup, r = 1
    assert -(-rows // bm) * tiles_n > 2 * resident
    for K in (192, 160):
        _sweep(rt, nb, variant, N=tiles_n * bn, K=K, Ms=[rows], epilogue="bias_gelu", seed=variant)
    _sweep(rt, nb, variant, N=tiles_n * bn - 24, K=64, Ms=[rows - 1], epilogue="bias", seed=variant)
    # a tile hands the ring to the next one before its own epilogue: without a bias to park (bf16), and
    # with the f32 epilogue, whose stores the next tile's waits cannot count
    _sweep(rt, nb, variant, N=tiles_n * bn, K=128, Ms=[rows], epilogue="none", seed=variant)
    _sweep(rt, nb, variant, N=tiles_n * bn, K=320, Ms=[rows - bm], epilogue="bias", out_dtype=1, seed=variant)


def test_tile_walk_at_a_reduced_tile_height(rt, nb):
    """The 256-wide variant at 160 rows (not a whole number of load passes) over three tiles per
    workgroup, last tile row ragged."""
    forced = 6 | (10 << 16)
    rows = 160 * 200 + 7
    for K in (64, 192):
        _sweep(rt, nb, forced, N=4 * 256, K=K, Ms=[rows], epilogue="bias_gelu", seed=K)


def test_random_shapes_through_the_dispatch_function(rt, nb):
    """Seeded random (M, N, K, epilogue, output type) through the automatic dispatch: whatever it
    picks (weight streaming, any tile, K split, row split) must agree with the oracle."""
    to_dev, _, from_dev, _ = _dev()
    rng = np.random.default_rng(2006)
    seen = set()
    for case in range(48):
        M = int(rng.choice([rng.integers(1, 65), rng.integers(65, 700), rng.integers(700, 2600)]))
        N = int(rng.choice([rng.integers(1, 40) * 8, rng.integers(1, 9) * 128, rng.integers(4, 10) * 256]))
        K = int(rng.choice([rng.integers(1, 40) * 8, rng.integers(1, 24) * 64, rng.integers(1, 12) * 32]))
        epi = ["none", "bias", "bias_gelu"][int(rng.integers(0, 3))]
        out_dtype = int(rng.integers(0, 2))
        while M * N * K > 6e8:
            M = max(1, M // 2)
        x, w, b = wl.uniform_bf16(rng, (M, K)), wl.normal_bf16(rng, (N, K), std=0.05), wl.uniform_bf16(rng, (N,))
        p = nb.dense_plan(M, N, K, EPI[epi], out_dtype)
        seen.add((p.name, p.split_k > 1 and p.variant > 1, p.split_rows > 0))
        y = rt.dense(to_dev(x), to_dev(w), to_dev(b) if epi != "none" else None, EPI[epi], out_dtype)
        ref = oracle.dense(x.f32, w.f32, b.f32 if epi != "none" else None, epi)
        assert tuple(y.shape) == (M, N)
        _check(from_dev(y), ref, (case, M, N, K, epi, out_dtype, p.name, p.split_k), f32=out_dtype == 1,
               gelu=epi == "bias_gelu")
    assert len({name for name, _, _ in seen}) >= 4, seen   # the draw reaches several kernels


def test_split_k_forced_and_auto(rt, nb):
    # forced: every ring variant, several slice counts, residues along M, both output types
    for variant, (bm, bn) in ((4, (128, 128)), (5, (256, 128)), (6, (256, 256))):
        for sk in (2, 4, 8):
            forced = variant | (sk << 8)
            _sweep(rt, nb, forced, N=bn, K=1024, Ms=[1, bm - 1, bm, bm + 3, 2 * bm + 1], epilogue="bias_gelu")
        _sweep(rt, nb, variant | (3 << 8), N=2 * bn, K=32 * 13, Ms=[70, bm + 70], epilogue="bias", out_dtype=1)
    # auto: mid-size M with long K and few tiles is where the dispatch function cuts K
    for (M, N, K) in [(600, 768, 3072), (700, 768, 3072), (300, 768, 3104), (300, 1024, 4096)]:
        p = nb.dense_plan(M, N, K)
        assert p.variant >= 2 and p.split_k > 1, (M, N, K, p)
    _sweep(rt, nb, -1, N=768, K=3072, Ms=[65, 100, 129, 300, 511, 512, 600, 700, 1000], epilogue="bias")
    _sweep(rt, nb, -1, N=768, K=3104, Ms=[65, 100, 300], epilogue="bias")
    # no workspace: the same shapes must still run (the plan falls back to one launch)
    import torch as _t
    empty = _t.empty(0, dtype=_t.uint8, device="cuda")
    to_dev, _, from_dev, _ = _dev()
    rng = np.random.default_rng(77)
    x, w, b = wl.uniform_bf16(rng, (300, 3072)), wl.normal_bf16(rng, (768, 3072)), wl.uniform_bf16(rng, (768,))
    y = rt.dense(to_dev(x), to_dev(w), to_dev(b), nb.EPI_BIAS, workspace=empty)
    _check(from_dev(y), oracle.dense(x.f32, w.f32, b.f32, "bias"), "no workspace")
    with pytest.raises(nb.NimbleError) as e:  # a forced split that does not fit is refused, not shrunk
        rt.dense(to_dev(x), to_dev(w), to_dev(b), nb.EPI_BIAS, force_variant=4 | (4 << 8), workspace=empty)
    assert e.value.code == -6


def test_skinny_every_M_and_ragged_shapes(rt, nb):
    _sweep(rt, nb, 1, N=2048, K=1024, Ms=range(1, 65))
    _sweep(rt, nb, 1, N=128, K=128, Ms=range(1, 131), epilogue="bias")      # M > 64: several row blocks
    _sweep(rt, nb, 1, N=100, K=200, Ms=[1, 15, 16, 17, 33, 64], epilogue="bias")  # N % 16 != 0, K % 32 != 0
    _sweep(rt, nb, 1, N=37, K=8, Ms=[1, 5, 48], epilogue="none", out_dtype=1)
    _sweep(rt, nb, 1, N=768, K=3072, Ms=[1, 2, 3, 4, 8, 16, 31, 64], epilogue="bias_gelu")


def test_streaming_kernel_stage_counts_row_blocks_and_ragged_N(rt, nb):
    """The LDS-staged streaming kernel (weight streaming with K in whole 64-wide stages): every M up
    to two 16-row blocks and a ragged third, K of 1, 2, 3, 8, 9, 17 and 50 stages (waves with no stage,
    with fewer stages than ring slots, with unequal shares), N not a multiple of 16, both output types."""
    for K in (64, 128, 192, 512, 576, 1088, 3200):
        assert nb.dense_plan(16, 160, K).name == "skinny16"
        _sweep(rt, nb, 1, N=160, K=K, Ms=[1, 2, 7, 8, 9, 15, 16, 17, 33], epilogue="bias")
    _sweep(rt, nb, 1, N=200, K=256, Ms=range(1, 50), epilogue="bias_gelu")           # N % 16 = 8
    _sweep(rt, nb, 1, N=24, K=64, Ms=[1, 8, 9, 16], epilogue="none", out_dtype=1)
    _sweep(rt, nb, -1, N=8192, K=1024, Ms=[1, 5, 8, 9, 16], epilogue="bias", out_dtype=1)
    # a layer the dispatch function takes to come from HBM (134 MB): one block of up to 16 rows
    p = nb.dense_plan(16, 8192, 8192)
    assert p.name == "skinny16" and p.grid[1] == 1
    _sweep(rt, nb, -1, N=8192, K=8192, Ms=[1, 8, 16], epilogue="bias")


def test_generic_kernel_any_shape(rt, nb):
    _sweep(rt, nb, 0, N=33, K=7, Ms=[1, 2, 17, 40], epilogue="bias_gelu")
    _sweep(rt, nb, 0, N=5, K=100, Ms=[3, 16], epilogue="none", out_dtype=1)
    _sweep(rt, nb, -1, N=130, K=100, Ms=[1, 70, 300], epilogue="bias")  # auto with K % 8 != 0 -> generic


def test_auto_dispatch_power_of_two_grid_and_128(rt, nb):
    # the paper's tuning grid (powers of two up to 256) and its evaluation point M = 128
    for (K, N, epi) in [(768, 2304, "bias"), (768, 3072, "bias_gelu"), (3072, 768, "bias")]:
        _sweep(rt, nb, -1, N=N, K=K, Ms=[1, 2, 4, 8, 16, 32, 64, 128, 256], epilogue=epi)


def test_identity_and_zero_weights_on_gpu(rt, nb):
    to_dev, _, from_dev, bits_from_dev = _dev()
    rng = np.random.default_rng(5)
    for M, variant in [(7, -1), (100, -1), (300, 4), (300, 6)]:
        x = wl.uniform_bf16(rng, (M, 256))
        eye = wl.BF16Array(wl.f32_to_bf16_bits(np.eye(256, dtype=np.float32)), np.eye(256, dtype=np.float32))
        y = rt.dense(to_dev(x), to_dev(eye), None, nb.EPI_NONE, nb.BF16, variant)
        assert np.array_equal(bits_from_dev(y), x.bits)  # bit-exact
        b = wl.uniform_bf16(rng, (256,))
        zero = wl.BF16Array(np.zeros((256, 256), np.uint16), np.zeros((256, 256), np.float32))
        y = rt.dense(to_dev(x), to_dev(zero), to_dev(b), nb.EPI_BIAS, nb.BF16, variant)
        assert np.array_equal(bits_from_dev(y), np.broadcast_to(b.bits, (M, 256)))
        y = rt.dense(to_dev(x), to_dev(zero), to_dev(b), nb.EPI_NONE, nb.F32, variant)
        assert np.all(from_dev(y) == 0)


def test_row_prefix_invariance_on_gpu(rt, nb):
    # with one kernel variant, rows do not depend on how large M was
    to_dev, _, _, bits_from_dev = _dev()
    rng = np.random.default_rng(6)
    x, w, b = wl.uniform_bf16(rng, (513, 256)), wl.normal_bf16(rng, (256, 256)), wl.uniform_bf16(rng, (256,))
    xd, wd, bd = to_dev(x), to_dev(w), to_dev(b)
    for variant in (4, 5, 6):
        full = bits_from_dev(rt.dense(xd, wd, bd, nb.EPI_BIAS_GELU_ERF, nb.BF16, variant))
        for M in (1, 255, 256, 257, 400):
            part = bits_from_dev(rt.dense(xd[:M], wd, bd, nb.EPI_BIAS_GELU_ERF, nb.BF16, variant))
            assert np.array_equal(part, full[:M])


def test_two_requests_in_flight_on_two_streams(rt, nb):
    """Dense calls of two requests interleaved on two streams, each with its own K-split workspace
    (calls that overlap must not share one): every output matches the same call made alone."""
    to_dev, _, from_dev, bits_from_dev = _dev()
    rng = np.random.default_rng(31)
    N, K = 768, 3072   # K-split plans at these M
    w, b = wl.normal_bf16(rng, (N, K)), wl.uniform_bf16(rng, (N,))
    wd, bd = to_dev(w), to_dev(b)
    Ms = [40, 530, 257, 700, 96, 600]
    xs = [to_dev(wl.uniform_bf16(rng, (M, K))) for M in Ms]
    alone = [bits_from_dev(rt.dense(x, wd, bd, nb.EPI_BIAS)) for x in xs]
    assert sum(nb.dense_plan(M, N, K).split_k > 1 and nb.dense_plan(M, N, K).variant >= 2 for M in Ms) >= 2
    torch.cuda.synchronize()
    streams = [torch.cuda.Stream(), torch.cuda.Stream()]
    spaces = [torch.empty(rt.WORKSPACE_BYTES, dtype=torch.uint8, device="cuda") for _ in streams]
    for rep in range(3):
        outs = []
        for i, x in enumerate(xs):
            with torch.cuda.stream(streams[i & 1]):
                outs.append(rt.dense(x, wd, bd, nb.EPI_BIAS, workspace=spaces[i & 1]))
        torch.cuda.synchronize()
        for i, y in enumerate(outs):
            assert np.array_equal(bits_from_dev(y), alone[i]), (rep, Ms[i])


# ------------------------------------------------------------------ config 3
@pytest.mark.parametrize("gemm", range(4))
def test_config3_bert_base_gemms_every_length(rt, nb, gemm):
    """Each BERT-base GEMM at every sequence length L = 1..512 through the dispatch function (weight
    streaming, every small tile, K splits): one oracle evaluation at 512 rows serves every L by
    row-prefix invariance; each call is gated on its own and its guard rows must stay untouched."""
    to_dev, _, from_dev, _ = _dev()
    name, K, N, epi = wl.BERT_BASE_GEMMS[gemm]
    w, b = wl.dense_weights(3, gemm, N, K)
    x = wl.activations(3, 500 + gemm, 512, K)
    ref = oracle.dense(x.f32, w.f32, b.f32, epi)
    xd, wd, bd = to_dev(x), to_dev(w), to_dev(b)
    buf = torch.empty((512 + 2, N), dtype=torch.bfloat16, device="cuda")
    names = set()
    for L in range(1, 513):
        buf.fill_(768.0)
        y = rt.dense(xd[:L], wd, bd, EPI[epi], out=buf[:L])
        assert tuple(y.shape) == oracle.dense_shape((L, K), (N, K))
        got = from_dev(buf)
        assert np.all(got[L:] == 768.0), (name, L)
        _check(got[:L], ref[:L], (name, L), gelu=epi == "bias_gelu")
        names.add(nb.dense_plan(L, N, K, EPI[epi]).name)
    # (the 768 -> 768 layer is streamed in 16-row blocks at every length; the others switch to tiles)
    assert "skinny16" in names and (len(names) >= 2 or name == "proj"), names


def test_config3_the_drawn_lengths_with_their_own_inputs(rt, nb):
    """The config's own draws (L ~ U{1..512}, fresh activations per draw and GEMM), all four GEMMs."""
    to_dev, _, from_dev, _ = _dev()
    Ls = [int(v) for v in wl.config3_lengths()[:24]]
    weights = [wl.dense_weights(3, i, N, K) for i, (_, K, N, _) in enumerate(wl.BERT_BASE_GEMMS)]
    dweights = [(to_dev(w), to_dev(b)) for w, b in weights]
    for d, L in enumerate(Ls):
        for i, (name, K, N, epi) in enumerate(wl.BERT_BASE_GEMMS):
            x = wl.activations(3, d * 10 + i, L, K)
            y = rt.dense(to_dev(x), dweights[i][0], dweights[i][1], EPI[epi])
            assert tuple(y.shape) == (L, N)
            ref = oracle.dense(x.f32, weights[i][0].f32, weights[i][1].f32, epi)
            _check(from_dev(y), ref, (name, L), gelu=epi == "bias_gelu")


# ------------------------------------------------------------------ config 5
def _sampled_rows(M, bm_max, n_random, rng):
    tail = np.arange(max(0, M - 2 * bm_max), M)
    head = rng.choice(max(1, M - len(tail)), size=min(n_random, max(1, M - len(tail))), replace=False)
    return np.unique(np.concatenate([head, tail]))


def test_config5_ragged_ffn_sampled_rows(rt, nb):
    """Full-size M (sum of 32 lengths) in the launch configuration the benchmark
    times (outputs carved from one storage arena), all 64 draws; the oracle evaluates the
    residue region (the last 320 rows: the tallest tile) plus random rows, which row
    independence makes exact.  FFN2 is teacher-forced with the
    GPU's own bf16 FFN1 output."""
    to_dev, _, from_dev, _ = _dev()
    Ms = wl.config5_token_counts()
    draws = range(len(Ms))       # all 64 draws
    arena = rt.StorageArena(int(max(Ms)) * (4096 + 1024) * 2 + 4096)   # outputs carved as the benchmark does
    (n1, K1, N1, e1), (n2, K2, N2, e2) = wl.BERT_LARGE_FFN
    w1, b1 = wl.dense_weights(5, 0, N1, K1)
    w2, b2 = wl.dense_weights(5, 1, N2, K2)
    dw1, db1, dw2, db2 = to_dev(w1), to_dev(b1), to_dev(w2), to_dev(b2)
    rng = np.random.default_rng(55)
    for d in draws:
        M = int(Ms[d])
        x = wl.activations(5, d, M, K1)
        arena.reset()
        h = rt.dense(to_dev(x), dw1, db1, EPI[e1], arena=arena)
        y = rt.dense(h, dw2, db2, EPI[e2], arena=arena)
        assert tuple(h.shape) == (M, N1) and tuple(y.shape) == (M, N2)
        assert y.data_ptr() >= h.data_ptr() + M * N1 * 2      # two tensors of one storage, not overlapping
        rows = _sampled_rows(M, 160, 64, rng)
        hg = from_dev(h)
        ref_h = oracle.dense(x.f32[rows], w1.f32, b1.f32, e1)
        _check(hg[rows], ref_h, ("ffn1", M), gelu=True)
        ref_y = oracle.dense(hg[rows], w2.f32, b2.f32, e2)
        _check(from_dev(y)[rows], ref_y, ("ffn2", M))


def test_config5_fixed_sizes_up_to_the_maximum(rt, nb):
    """M = 2048, 4096, 8192 and 16384 (32 sequences of 512 tokens, the largest total config 5 can
    draw: four rounds of tiles per compute unit), one row past each, FFN1 and FFN2 on sampled rows."""
    to_dev, _, from_dev, _ = _dev()
    (n1, K1, N1, e1), (n2, K2, N2, e2) = wl.BERT_LARGE_FFN
    w1, b1 = wl.dense_weights(5, 0, N1, K1)
    w2, b2 = wl.dense_weights(5, 1, N2, K2)
    dw1, db1, dw2, db2 = to_dev(w1), to_dev(b1), to_dev(w2), to_dev(b2)
    x = wl.activations(5, 777, 16385, K1)
    xd = to_dev(x)
    rng = np.random.default_rng(57)
    for M in (2048, 4096, 8192, 8193, 16384, 16385):
        h = rt.dense(xd[:M], dw1, db1, EPI[e1])
        y = rt.dense(h, dw2, db2, EPI[e2])
        rows = _sampled_rows(M, 160, 64, rng)
        hg = from_dev(h)
        _check(hg[rows], oracle.dense(x.f32[rows], w1.f32, b1.f32, e1), ("ffn1", M))
        _check(from_dev(y)[rows], oracle.dense(hg[rows], w2.f32, b2.f32, e2), ("ffn2", M))


def test_config5_residue_sweep_2048_plus_r(rt, nb):
    to_dev, _, from_dev, _ = _dev()
    (n1, K1, N1, e1), (n2, K2, N2, e2) = wl.BERT_LARGE_FFN
    w1, b1 = wl.dense_weights(5, 0, N1, K1)
    w2, b2 = wl.dense_weights(5, 1, N2, K2)
    dw1, db1, dw2, db2 = to_dev(w1), to_dev(b1), to_dev(w2), to_dev(b2)
    Mmax = 2048 + 255
    x = wl.activations(5, 999, Mmax, K1)
    xd = to_dev(x)
    rng = np.random.default_rng(56)
    fixed = np.sort(rng.choice(2048 - 64, size=48, replace=False))
    rows_all = np.concatenate([fixed, np.arange(2048 - 64, Mmax)])
    ref_h_all = oracle.dense(x.f32[rows_all], w1.f32, b1.f32, e1)
    pos = {int(r): i for i, r in enumerate(rows_all)}
    for r in range(0, 256):
        M = 2048 + r
        h = rt.dense(xd[:M], dw1, db1, EPI[e1])
        rows = rows_all[rows_all < M]
        idx = [pos[int(v)] for v in rows]
        hg = from_dev(h)
        _check(hg[rows], ref_h_all[idx], ("ffn1", M))
        if r % 16 in (0, 1, 15):  # FFN2 needs a fresh oracle evaluation per M (teacher forcing)
            y = rt.dense(h, dw2, db2, EPI[e2])
            sub = rows[-40:]
            ref_y = oracle.dense(hg[sub], w2.f32, b2.f32, e2)
            _check(from_dev(y)[sub], ref_y, ("ffn2", M))


# ------------------------------------------------------------------ config 2
def test_lstm_teacher_forced_steps(rt, nb):
    """Per step both sides get identical inputs: the GPU's own bf16 h and f32 c."""
    to_dev, f32_to_dev, from_dev, _ = _dev()
    lw = wl.config2_weights()
    dw, db = to_dev(lw.w), to_dev(lw.b)
    H = wl.LSTM_H
    plan = [(1, 128), (7, 128), (16, 6), (17, 6), (33, 6), (48, 4), (64, 6)]
    plan += [(int(b), 3) for b in wl.config2_batches()[:6]]
    for seq, (B, steps) in enumerate(plan):
        xs = wl.config2_inputs(seq, B, steps)
        h = torch.zeros((B, H), dtype=torch.bfloat16, device="cuda")
        c = torch.zeros((B, H), dtype=torch.float32, device="cuda")
        for t in range(steps):
            xt = wl.BF16Array(xs.bits[t], xs.f32[t])
            h_in, c_in = from_dev(h), from_dev(c)
            h2, c2 = rt.lstm_step(to_dev(xt), h, dw, db, c)
            assert tuple(h2.shape) == (B, H) and tuple(c2.shape) == (B, H)
            ref_h, ref_c = oracle.lstm_step(xt.f32, h_in, lw.w.f32, lw.b.f32, c_in)
            _check(from_dev(c2), ref_c, ("c", B, t), f32=True)
            _check(from_dev(h2), ref_h, ("h", B, t))
            h, c = h2, c2


def test_lstm_one_step_at_every_batch_size(rt, nb):
    """Config 2's cell (2048 x 1024) at every dynamic batch B = 1..64 (every residue of the 16-row
    tile, every row-block split the dispatch function makes), the fused cell and the cell with the
    inputs' share precomputed; h and c arbitrary (not the zero start), guard rows untouched."""
    to_dev, f32_to_dev, from_dev, _ = _dev()
    lw = wl.config2_weights()
    dw, db = to_dev(lw.w), to_dev(lw.b)
    H, Ix = wl.LSTM_H, wl.LSTM_IX
    w_x, w_h = rt.split_lstm_weight(dw, Ix)
    wh_ref = np.ascontiguousarray(lw.w.f32[:, Ix:])
    rng = np.random.default_rng(64)
    x_all, h_all = wl.uniform_bf16(rng, (64, Ix)), wl.uniform_bf16(rng, (64, H))
    c_all = (2.0 * rng.random((64, H)) - 1.0).astype(np.float32)
    xd, hd, cd = to_dev(x_all), to_dev(h_all), f32_to_dev(c_all)
    pre_all = rt.dense(xd, w_x, db, nb.EPI_BIAS, nb.F32)
    pre_np = from_dev(pre_all)
    blocks = set()
    for B in range(1, 65):
        blocks.add(nb.lstm_plan(B, Ix, H).grid[1])
        ref_h, ref_c = oracle.lstm_step(x_all.f32[:B], h_all.f32[:B], lw.w.f32, lw.b.f32, c_all[:B])
        hb = torch.full((B + 1, H), 768.0, dtype=torch.bfloat16, device="cuda")
        cb = torch.full((B + 1, H), 768.0, dtype=torch.float32, device="cuda")
        h2, c2 = rt.lstm_step(xd[:B], hd[:B], dw, db, cd[:B], h_out=hb[:B], c_out=cb[:B])
        hg, cg = from_dev(hb), from_dev(cb)
        assert np.all(hg[B:] == 768.0) and np.all(cg[B:] == 768.0), B
        _check(cg[:B], ref_c, ("c", B), f32=True)
        _check(hg[:B], ref_h, ("h", B))
        hb.fill_(768.0)
        cb.fill_(768.0)
        rt.lstm_step_pre(pre_all[:B], hd[:B], w_h, cd[:B], h_out=hb[:B], c_out=cb[:B])
        hg, cg = from_dev(hb), from_dev(cb)
        assert np.all(hg[B:] == 768.0) and np.all(cg[B:] == 768.0), B
        rh, rc = oracle.lstm_step_pre(pre_np[:B], h_all.f32[:B], wh_ref, c_all[:B])
        _check(cg[:B], rc, ("c pre", B), f32=True)
        _check(hg[:B], rh, ("h pre", B))
        _check(hg[:B], ref_h, ("h pre vs fused oracle", B))
    assert blocks == {1, 2, 3, 4}, blocks   # 16-row blocks: the streaming kernel at every B


def test_lstm_closed_forms_and_aliasing_on_gpu(rt, nb):
    to_dev, f32_to_dev, from_dev, _ = _dev()
    H, Ix, B = 64, 40, 21
    rng = np.random.default_rng(8)
    x, h0 = wl.uniform_bf16(rng, (B, Ix)), wl.uniform_bf16(rng, (B, H))
    c0 = wl.uniform_bf16(rng, (B, H)).f32
    zero_w = wl.BF16Array(np.zeros((4 * H, Ix + H), np.uint16), np.zeros((4 * H, Ix + H), np.float32))
    zb = np.zeros((4 * H,), np.float32)
    bz = wl.BF16Array(wl.f32_to_bf16_bits(zb), zb)
    # zero weights: c halves every step, exactly; c_out aliases c_prev
    c = f32_to_dev(c0)
    h = to_dev(h0)
    for t in range(1, 6):
        h, c = rt.lstm_step(to_dev(x), h, to_dev(zero_w), to_dev(bz), c, c_out=c)
        assert np.array_equal(from_dev(c), np.ldexp(c0, -t))
        assert np.max(np.abs(from_dev(h) - 0.5 * np.tanh(np.ldexp(c0, -t)))) < 4e-3
    # forget gate open, input gate shut: the state is carried
    bf = zb.copy()
    bf[H:2 * H] = 30.0
    bf[0:H] = -30.0
    bb = wl.BF16Array(wl.f32_to_bf16_bits(bf), bf)
    h, c = rt.lstm_step(to_dev(x), to_dev(h0), to_dev(zero_w), to_dev(bb), f32_to_dev(c0))
    assert np.max(np.abs(from_dev(c) - c0)) < 1e-6
    # ragged H (not a multiple of 4 units per workgroup is impossible: H % 8 == 0), ragged B
    # (the last four: K and Ix in whole 64-wide stages, i.e. the streaming kernel, one to five row blocks)
    for (B2, H2, Ix2) in [(5, 8, 8), (70, 24, 16), (3, 512, 0), (7, 64, 128), (20, 192, 64), (16, 136, 120),
                          (33, 64, 0), (70, 128, 128)]:
        rng2 = np.random.default_rng(B2)
        xx = wl.uniform_bf16(rng2, (B2, Ix2))
        hh = wl.uniform_bf16(rng2, (B2, H2))
        ww = wl.normal_bf16(rng2, (4 * H2, Ix2 + H2), std=0.2)
        bias = wl.uniform_bf16(rng2, (4 * H2,))
        cc = wl.uniform_bf16(rng2, (B2, H2)).f32
        xdev = to_dev(xx) if Ix2 else torch.zeros((B2, 0), dtype=torch.bfloat16, device="cuda")
        hg, cg = rt.lstm_step(xdev, to_dev(hh), to_dev(ww), to_dev(bias), f32_to_dev(cc))
        rh, rc = oracle.lstm_step(xx.f32.reshape(B2, Ix2), hh.f32, ww.f32, bias.f32, cc)
        _check(from_dev(cg), rc, ("c", B2, H2, Ix2), f32=True)
        _check(from_dev(hg), rh, ("h", B2, H2, Ix2))


def test_lstm_sequence_graph_replays_match_eager(rt, nb):
    """The captured token loop is replayed several times, with eager work and synchronisation in
    between, and every replay must reproduce the eager step-by-step result bit for bit."""
    to_dev, f32_to_dev, from_dev, bits_from_dev = _dev()
    lw = wl.config2_weights()
    dw, db = to_dev(lw.w), to_dev(lw.b)
    H, steps = wl.LSTM_H, 12
    for B in (3, 40):
        seq = rt.LstmSequenceGraph(dw, db, B, steps, wl.LSTM_IX, H)
        for rep in range(3):
            xs = wl.config2_inputs(50 + rep, B, steps)
            xd = to_dev(xs)
            # eager reference on the GPU
            h = torch.zeros((B, H), dtype=torch.bfloat16, device="cuda")
            c = torch.zeros((B, H), dtype=torch.float32, device="cuda")
            eager = []
            for t in range(steps):
                h, c = rt.lstm_step(xd[t], h, dw, db, c)
                eager.append(bits_from_dev(h))
            torch.cuda.synchronize()
            hs, c_fin = seq.run(xd)
            torch.cuda.synchronize()
            assert np.array_equal(bits_from_dev(hs), np.stack(eager)), (B, rep)
            assert np.array_equal(from_dev(c_fin), from_dev(c)), (B, rep)
        # first step against the oracle (h_0 = c_0 = 0)
        x0 = wl.BF16Array(xs.bits[0], xs.f32[0])
        rh, rc = oracle.lstm_step(x0.f32, np.zeros((B, H), np.float32), lw.w.f32, lw.b.f32,
                                  np.zeros((B, H), np.float32))
        _check(from_dev(hs[0]), rh, ("graph step 0", B))


def test_lstm_from_precomputed_input_gates(rt, nb):
    """Inputs' share of the gates for all tokens from one dense call (M = T*B, f32 output), then
    per token the recurrent half only.  Per step both sides get the same pre, h and c."""
    to_dev, f32_to_dev, from_dev, _ = _dev()
    lw = wl.config2_weights()
    H, Ix = wl.LSTM_H, wl.LSTM_IX
    dw, db = to_dev(lw.w), to_dev(lw.b)
    w_x, w_h = rt.split_lstm_weight(dw, Ix)
    wx_ref, wh_ref = np.ascontiguousarray(lw.w.f32[:, :Ix]), np.ascontiguousarray(lw.w.f32[:, Ix:])
    for seq, (B, steps) in enumerate([(1, 24), (5, 6), (16, 4), (23, 4), (64, 4), (70, 3)]):
        xs = wl.config2_inputs(30 + seq, B, steps)
        xd = to_dev(xs)
        pre = rt.dense(xd.view(steps * B, Ix), w_x, db, nb.EPI_BIAS, nb.F32).view(steps, B, 4 * H)
        pre_ref = oracle.dense(xs.f32.reshape(steps * B, Ix), wx_ref, lw.b.f32, "bias")
        _check(from_dev(pre).reshape(steps * B, 4 * H), pre_ref, ("pre", B), f32=True)
        pre_np = from_dev(pre)
        h = torch.zeros((B, H), dtype=torch.bfloat16, device="cuda")
        c = torch.zeros((B, H), dtype=torch.float32, device="cuda")
        for t in range(steps):
            h_in, c_in = from_dev(h), from_dev(c)
            h2, c2 = rt.lstm_step_pre(pre[t], h, w_h, c)
            ref_h, ref_c = oracle.lstm_step_pre(pre_np[t], h_in, wh_ref, c_in)
            _check(from_dev(c2), ref_c, ("c", B, t), f32=True)
            _check(from_dev(h2), ref_h, ("h", B, t))
            # and against the fused cell of the oracle on the original inputs (pre is exact up to f32 order)
            fh, fc = oracle.lstm_step(xs.f32[t], h_in, lw.w.f32, lw.b.f32, c_in)
            _check(from_dev(h2), fh, ("fused h", B, t))
            h, c = h2, c2
    # ragged H and B, c_out aliasing c_prev, closed form with zero recurrent weight
    rng = np.random.default_rng(77)
    for (B2, H2) in [(3, 8), (37, 24), (65, 40)]:
        hh = wl.uniform_bf16(rng, (B2, H2))
        ww = wl.normal_bf16(rng, (4 * H2, H2), std=0.3)
        pp = rng.uniform(-2, 2, (B2, 4 * H2)).astype(np.float32)
        cc = wl.uniform_bf16(rng, (B2, H2)).f32
        cdev = f32_to_dev(cc)
        hg, cg = rt.lstm_step_pre(f32_to_dev(pp), to_dev(hh), to_dev(ww), cdev, c_out=cdev)
        assert cg.data_ptr() == cdev.data_ptr()
        rh, rc = oracle.lstm_step_pre(pp, hh.f32, ww.f32, cc)
        _check(from_dev(cg), rc, ("c", B2, H2), f32=True)
        _check(from_dev(hg), rh, ("h", B2, H2))
    B2, H2 = 9, 16
    c0 = wl.uniform_bf16(rng, (B2, H2)).f32
    zero = torch.zeros((4 * H2, H2), dtype=torch.bfloat16, device="cuda")
    hg, cg = rt.lstm_step_pre(torch.zeros((B2, 4 * H2), dtype=torch.float32, device="cuda"),
                              to_dev(wl.uniform_bf16(rng, (B2, H2))), zero, f32_to_dev(c0))
    assert np.array_equal(from_dev(cg), c0 / 2)


def test_lstm_sequence_graph_with_projected_inputs(rt, nb):
    """The captured loop with the inputs' product hoisted out of it: replays reproduce the eager
    result bit for bit, and the whole sequence stays within tolerance of the fused-cell loop."""
    to_dev, f32_to_dev, from_dev, bits_from_dev = _dev()
    lw = wl.config2_weights()
    dw, db = to_dev(lw.w), to_dev(lw.b)
    H, Ix, steps = wl.LSTM_H, wl.LSTM_IX, 10
    w_x, w_h = rt.split_lstm_weight(dw, Ix)
    for B in (2, 33):
        seq = rt.LstmSequenceGraph(dw, db, B, steps, Ix, H, project_inputs=True)
        fused = rt.LstmSequenceGraph(dw, db, B, steps, Ix, H)
        for rep in range(3):
            xd = to_dev(wl.config2_inputs(60 + rep, B, steps))
            pre = rt.dense(xd.view(steps * B, Ix), w_x, db, nb.EPI_BIAS, nb.F32).view(steps, B, 4 * H)
            h = torch.zeros((B, H), dtype=torch.bfloat16, device="cuda")
            c = torch.zeros((B, H), dtype=torch.float32, device="cuda")
            eager = []
            for t in range(steps):
                h, c = rt.lstm_step_pre(pre[t], h, w_h, c)
                eager.append(bits_from_dev(h))
            torch.cuda.synchronize()
            hs, c_fin = seq.run(xd)
            torch.cuda.synchronize()
            assert np.array_equal(bits_from_dev(hs), np.stack(eager)), (B, rep)
            assert np.array_equal(from_dev(c_fin), from_dev(c)), (B, rep)
            hs_f, _ = fused.run(xd)
            torch.cuda.synchronize()
            assert _err(from_dev(hs), from_dev(hs_f)) <= TOL, (B, rep)


# ------------------------------------------------------------------ config 4
# O against the oracle's unrounded chain: the GPU rounds P (the fused kernel: the un-normalised
# exponentials) to bf16 before P.V, which adds to every element of O a sum of L independent rounding
# errors of about 2^-9/sqrt(3) of the element's own scale; over 12 L 64 elements its largest value
# reaches 5e-3 rms(O), so the absolute part of the element-wise bound is 2^-6 rms(O) here.
P_ROUNDED_FLOOR = 2.0 ** -6


def test_attention_chain(rt, nb):
    to_dev, _, from_dev, _ = _dev()
    # every L in 1..130 and 448..512: every residue of the 64- and 128-row tiles at both ends of the range
    Ls = sorted(set(list(range(1, 131)) + list(range(448, 513)) + [200, 257, 300, 384] +
                    [int(v) for v in wl.config4_lengths()[:8]]))
    for d, L in enumerate(Ls):
        q, k, v = wl.config4_qkv(d, L)
        s, p, o = rt.attention(to_dev(q), to_dev(k), to_dev(v))
        assert tuple(s.shape) == (12, L, L) and tuple(p.shape) == (12, L, L) and tuple(o.shape) == (12, L, 64)
        rs, rp, ro = oracle.attention(q.f32, k.f32, v.f32)
        _check(from_dev(s), rs, ("S", L), f32=True)
        _check(from_dev(p), rp, ("P", L))
        _check(from_dev(o), ro, ("O", L), floor=P_ROUNDED_FLOOR)
        # teacher-forced second batch_matmul: the oracle applied to the GPU's own bf16 P
        ro2 = oracle.batch_matmul(from_dev(p), v.f32, False, 1.0)
        _check(from_dev(o), ro2, ("O|P", L))
        if L == 1:
            assert np.array_equal(from_dev(p), np.ones((12, 1, 1), np.float32))
            assert np.array_equal(from_dev(o), v.f32)


def test_fused_attention_matches_the_oracle_chain(rt, nb):
    to_dev, _, from_dev, _ = _dev()
    Ls = sorted(set(list(range(1, 131)) + list(range(448, 513)) + [255, 256, 257, 300, 383, 384, 385] +
                    [int(v) for v in wl.config4_lengths()[:12]]))
    for d, L in enumerate(Ls):
        q, k, v = wl.config4_qkv(100 + d, L)
        # one guard row after the last head's last row: the kernel must stay inside o
        buf = torch.full((12 * L + 1, 64), 768.0, dtype=torch.bfloat16, device="cuda")
        o = rt.fused_attention(to_dev(q), to_dev(k), to_dev(v), out=buf[:12 * L].view(12, L, 64))
        assert tuple(o.shape) == (12, L, 64) and o.data_ptr() == buf.data_ptr()
        got = from_dev(buf)
        assert np.all(got[12 * L:] == 768.0), ("wrote past the output", L)
        _, _, ro = oracle.attention(q.f32, k.f32, v.f32)
        _check(got[:12 * L].reshape(12, L, 64), ro, ("O", L), floor=P_ROUNDED_FLOOR)
        if L % 16 in (0, 1, 15):   # and it agrees with the three-call chain on the GPU to rounding
            _, _, o3 = rt.attention(to_dev(q), to_dev(k), to_dev(v))
            assert _err(from_dev(o), from_dev(o3)) <= TOL, ("O vs chain", L)
    # other positive scales: sharp rows (the running maximum moves from block to block, single keys dominate)
    # and nearly flat ones
    for alpha, L in [(1.0, 200), (0.5, 129), (1e-3, 300), (2.0, 64)]:
        q, k, v = wl.config4_qkv(200 + L, L)
        o = rt.fused_attention(to_dev(q), to_dev(k), to_dev(v), alpha=alpha)
        _, _, ro = oracle.attention(q.f32, k.f32, v.f32, alpha=alpha)
        _check(from_dev(o), ro, ("O", L, alpha), floor=P_ROUNDED_FLOOR)
    for bad in (0.0, -0.125):       # the fused softmax works on raw scores: the scale must be positive
        with pytest.raises(nb.NimbleError) as e:
            rt.fused_attention(to_dev(q), to_dev(k), to_dev(v), alpha=bad)
        assert e.value.code == -8
    # closed forms: L = 1 returns V; Q = 0 returns the column mean of V
    q, k, v = wl.config4_qkv(7, 1)
    assert np.array_equal(from_dev(rt.fused_attention(to_dev(q), to_dev(k), to_dev(v))), v.f32)
    q, k, v = wl.config4_qkv(8, 8)
    zq = wl.BF16Array(np.zeros_like(q.bits), np.zeros_like(q.f32))
    o = from_dev(rt.fused_attention(to_dev(zq), to_dev(k), to_dev(v)))
    assert np.max(np.abs(o - v.f32.astype(np.float64).mean(axis=1, keepdims=True))) < 4e-3
    with pytest.raises(nb.NimbleError) as e:  # other head dimensions go through the three calls
        nb.nimble_attention_dyn(1 << 8, 1 << 8, 1 << 8, 1 << 8, 12, 5, 32, 0.125)
    assert e.value.code == -8


def test_batch_matmul_general_shapes(rt, nb):
    to_dev, _, from_dev, _ = _dev()
    rng = np.random.default_rng(9)
    for (T, M, N, K, trans_b) in [(3, 70, 130, 64, True), (2, 300, 72, 136, True), (1, 5, 3, 7, True),
                                  (4, 33, 64, 33, False), (2, 129, 40, 257, False), (12, 512, 512, 64, True)]:
        a = wl.uniform_bf16(rng, (T, M, K))
        b = wl.uniform_bf16(rng, (T, N, K) if trans_b else (T, K, N))
        for od in (nb.BF16, nb.F32):
            c = rt.batch_matmul(to_dev(a), to_dev(b), trans_b, 0.125, od)
            ref = oracle.batch_matmul(a.f32, b.f32, trans_b, 0.125)
            _check(from_dev(c), ref, (T, M, N, K, trans_b, od), f32=od == nb.F32)


def test_batch_matmul_nn_on_the_tiled_kernels_and_without_workspace(rt, nb):
    """b [T,K,N] with K a multiple of 8: the plan is the NT launch on b transposed into the workspace
    (config 4's P.V at L = 128..512 among the shapes); a caller that brings no workspace gets the
    bounds-checked kernel and the same result to within rounding."""
    to_dev, _, from_dev, _ = _dev()
    rng = np.random.default_rng(10)
    none = torch.empty(0, dtype=torch.uint8, device="cuda")
    for (T, M, N, K) in [(12, 256, 64, 256), (12, 512, 64, 512), (8, 400, 64, 400), (7, 301, 136, 168), (2, 2050, 8, 1024)]:
        p = nb.batch_matmul_plan(T, M, N, K, False)
        assert p.name != "generic" and p.workspace_bytes == T * N * K * 2, (T, M, N, K, p.name)
        a, b = wl.uniform_bf16(rng, (T, M, K)), wl.uniform_bf16(rng, (T, K, N))
        ref = oracle.batch_matmul(a.f32, b.f32, False, 0.5)
        for od in (nb.BF16, nb.F32):
            tiled = rt.batch_matmul(to_dev(a), to_dev(b), False, 0.5, od)
            plain = rt.batch_matmul(to_dev(a), to_dev(b), False, 0.5, od, workspace=none)
            _check(from_dev(tiled), ref, ("tiled", T, M, N, K, od), f32=od == nb.F32)
            _check(from_dev(plain), ref, ("plain", T, M, N, K, od), f32=od == nb.F32)
    # K not a multiple of 8: no tiled plan, no workspace asked for
    p = nb.batch_matmul_plan(4, 33, 64, 33, False)
    assert p.name == "generic" and p.workspace_bytes == 0
    # small products stay on the bounds-checked kernel: the extra launch would cost more than it saves
    p = nb.batch_matmul_plan(12, 128, 64, 128, False)
    assert p.name == "generic" and p.workspace_bytes == 0


def test_softmax_rows_on_gpu(rt, nb):
    _, f32_to_dev, from_dev, _ = _dev()
    rng = np.random.default_rng(10)
    for rows, cols in [(1, 1), (5, 3), (12 * 7, 7), (12 * 65, 65), (100, 512), (3, 1000)]:
        s = (8 * (2 * rng.random((rows, cols)) - 1)).astype(np.float32)
        p = from_dev(rt.softmax_rows(f32_to_dev(s)))
        ref = oracle.softmax_rows(s)
        _check(p, ref, ("softmax", rows, cols))
        assert np.max(np.abs(p.sum(-1) - 1)) < 2e-2  # bf16 rounding of each term


# ------------------------------------------------------------------ error paths on the device side
def test_errors_leave_outputs_untouched(rt, nb):
    to_dev, _, from_dev, _ = _dev()
    rng = np.random.default_rng(11)
    x, w, b = wl.uniform_bf16(rng, (9, 128)), wl.uniform_bf16(rng, (64, 128)), wl.uniform_bf16(rng, (64,))
    xd, wd, bd = to_dev(x), to_dev(w), to_dev(b)
    y = torch.full((9, 64), 5.0, dtype=torch.bfloat16, device="cuda")
    with pytest.raises(nb.NimbleError) as e:  # K mismatch: the deferred type check fires, nothing runs
        rt.dense(xd, to_dev(wl.uniform_bf16(rng, (64, 120))), bd, out=y)
    assert e.value.code == -3
    with pytest.raises(nb.NimbleError) as e:  # misaligned output pointer
        nb.nimble_dense_dyn(xd.data_ptr(), wd.data_ptr(), bd.data_ptr(), y.data_ptr() + 2, 9, 64, 128, 1)
    assert e.value.code == -5
    with pytest.raises(nb.NimbleError) as e:
        nb.nimble_dense_dyn(xd.data_ptr(), wd.data_ptr(), 0, y.data_ptr(), 9, 64, 128, 1)
    assert e.value.code == -1
    torch.cuda.synchronize()
    assert np.all(from_dev(y) == 5.0)
    # M = 0: legal, nothing launched, shape (0, N)
    y0 = rt.dense(xd[:0], wd, bd)
    assert tuple(y0.shape) == (0, 64)
    rt.dense(xd, wd, bd, out=y)
    _check(from_dev(y), oracle.dense(x.f32, w.f32, b.f32, "bias"), "after the refused calls")


# ------------------------------------------------------------------ batch_matmul with one batch
def test_batch_matmul_single_batch_large_and_small(rt, nb):
    """batch = 1 takes dense-like plans: the launch must cover M on its own (no row split: rows past
    the last full tile go through the masked copy), and the weight-streaming kernel must apply alpha."""
    to_dev, _, from_dev, _ = _dev()
    rng = np.random.default_rng(12)
    # a shape the dense dispatch would split in two launches: guard rows behind the output stay untouched
    M, N, K = 10764, 4096, 1024
    p = nb.batch_matmul_plan(1, M, N, K, True)
    assert p.split_rows == 0 and p.grid[0] == -(-M // p.bm) * -(-N // p.bn) and (p.residue_copy or M % p.bm == 0)
    a, b = wl.uniform_bf16(rng, (1, M, K)), wl.normal_bf16(rng, (1, N, K))
    buf = torch.full((M + 3, N), 768.0, dtype=torch.bfloat16, device="cuda")
    rt.batch_matmul(to_dev(a), to_dev(b), True, 0.5, nb.BF16, out=buf[:M].view(1, M, N))
    got = from_dev(buf)
    assert np.all(got[M:] == 768.0)
    rows = np.r_[0:4, M // 2:M // 2 + 4, M - 330:M]
    ref = oracle.batch_matmul(a.f32[:, rows], b.f32, True, 0.5)
    _check(got[rows], ref[0], ("bmm batch 1", M, N, K))
    # few rows: the plan is the weight-streaming kernel, which must scale by alpha
    for (M, N, K) in [(16, 128, 64), (64, 2304, 768), (5, 64, 128), (33, 512, 256), (200, 768, 768)]:
        assert nb.batch_matmul_plan(1, M, N, K, True).name == "skinny16", (M, N, K)
        a, b = wl.uniform_bf16(rng, (1, M, K)), wl.uniform_bf16(rng, (1, N, K))
        ref = oracle.batch_matmul(a.f32, b.f32, True, 0.125)
        for od in (nb.BF16, nb.F32):
            c = rt.batch_matmul(to_dev(a), to_dev(b), True, 0.125, od)
            _check(from_dev(c), ref, ("bmm skinny", M, N, K, od), f32=od == nb.F32)


# ------------------------------------------------------------------ tuned dispatch table
def test_dense_through_a_tuned_table_entry(rt, nb):
    """Section 3.5, tuning: an installed entry (3072 -> 768, M in 65..256: 64 x 128 tiles with K cut
    in 4) decides the dispatch inside its range; the results across the range edges match the oracle
    whichever side of an edge they fall on, and the built-in choice is back once the table is removed."""
    N, K, epi = 768, 3072, nb.EPI_BIAS
    builtin = {M: nb.dense_plan(M, N, K, epi) for M in (64, 65, 256, 257)}
    try:
        nb.dense_table_set(N, K, epi, [(65, 256, 3, 4)])
        for M in (65, 100, 256):
            p = nb.dense_plan(M, N, K, epi)
            assert (p.name, p.split_k) == ("t64x128", 4)
        assert nb.dense_plan(64, N, K, epi) == builtin[64] and nb.dense_plan(257, N, K, epi) == builtin[257]
        _sweep(rt, nb, -1, N=N, K=K, Ms=[1, 63, 64, 65, 66, 100, 128, 129, 255, 256, 257, 258, 300], epilogue="bias")
        # a tabled K split that does not fit the caller's scratch is skipped, not an error
        to_dev, _, from_dev, _ = _dev()
        rng = np.random.default_rng(78)
        x, w, b = wl.uniform_bf16(rng, (100, K)), wl.normal_bf16(rng, (N, K)), wl.uniform_bf16(rng, (N,))
        none = torch.empty(0, dtype=torch.uint8, device="cuda")
        y = rt.dense(to_dev(x), to_dev(w), to_dev(b), epi, workspace=none)
        _check(from_dev(y), oracle.dense(x.f32, w.f32, b.f32, "bias"), "tabled split without scratch")
    finally:
        nb.dense_table_set(N, K, epi, [])
    for M, p in builtin.items():
        assert nb.dense_plan(M, N, K, epi) == p


def test_runtime_refuses_tensors_it_cannot_pass_as_plain_pointers(rt, nb):
    """The C ABI takes contiguous bf16 device memory: a strided view, another dtype or a host tensor
    must be refused by the caller-side wrapper, not read as packed bf16."""
    x = torch.zeros((8, 128), dtype=torch.bfloat16, device="cuda")
    w = torch.zeros((64, 128), dtype=torch.bfloat16, device="cuda")
    b = torch.zeros((64,), dtype=torch.bfloat16, device="cuda")
    wide = torch.zeros((8, 256), dtype=torch.bfloat16, device="cuda")
    for bad_x, bad_w, bad_b in [(wide[:, :128], w, b), (x.float(), w, b), (x, w.float(), b), (x.cpu(), w, b),
                                (x, w, b.float()), (x, w.t().contiguous().t(), b)]:
        with pytest.raises(nb.NimbleError):
            rt.dense(bad_x, bad_w, bad_b)
    with pytest.raises(nb.NimbleError):
        rt.dense(x, w, b, out=torch.zeros((8, 128), dtype=torch.bfloat16, device="cuda")[:, :64])
    with pytest.raises(nb.NimbleError):
        rt.dense(x, w, b, out=torch.zeros((8, 64), dtype=torch.float32, device="cuda"))
    q = torch.zeros((2, 8, 64), dtype=torch.bfloat16, device="cuda")
    with pytest.raises(nb.NimbleError):
        rt.batch_matmul(q.transpose(1, 2), q, True)
    with pytest.raises(nb.NimbleError):
        rt.fused_attention(q, q.float(), q)
    h = torch.zeros((8, 64), dtype=torch.bfloat16, device="cuda")
    c = torch.zeros((8, 64), dtype=torch.float32, device="cuda")
    wl_ = torch.zeros((256, 192), dtype=torch.bfloat16, device="cuda")
    bl = torch.zeros((256,), dtype=torch.bfloat16, device="cuda")
    with pytest.raises(nb.NimbleError):
        rt.lstm_step(x, h, wl_, bl, c.bfloat16())
    with pytest.raises(nb.NimbleError):
        rt.lstm_step(x, h.float(), wl_, bl, c)
    rt.lstm_step(x, h, wl_, bl, c)      # the well-formed call goes through
    torch.cuda.synchronize()

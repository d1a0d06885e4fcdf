"""Host side of the C ABI (no GPU): the library loads and exports every symbol
the header declares; shape functions, storage sizes, the residue split and the
dispatch table agree with the oracle and with their own invariants."""
import ctypes
import os

import numpy as np
import pytest

import oracle
import paper_2006_03031_amd as nb

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")
TILED = {2: (32, 128), 3: (64, 128), 4: (128, 128), 5: (256, 128), 6: (256, 256)}


def _golden_rows(name):
    with open(os.path.join(GOLDEN, name)) as f:
        return [[c.strip() for c in l.split("|")] for l in f if l.strip() and not l.startswith("#")]


def test_library_exports_every_declared_symbol():
    lib = nb.load()
    names = nb.exported_symbols()
    assert {"nimble_dense_shape", "nimble_dense_dyn", "nimble_batch_matmul_dyn",
            "nimble_lstm_gates_dyn"} <= set(names)
    for name in names:
        assert getattr(lib, name) is not None, name
    assert os.path.basename(nb.library_path()) == "libnimble_hip.so"


def test_dense_shape_matches_oracle_for_every_M():
    for M in range(0, 514):
        got = nb.nimble_dense_shape((M, 1024), (4096, 1024))
        assert got == oracle.dense_shape((M, 1024), (4096, 1024)) == (M, 4096)


def test_dense_shape_outputs_are_int64_and_untouched_on_error():
    lib = nb.load()
    xs = (ctypes.c_int64 * 2)(7, 128)
    ws = (ctypes.c_int64 * 2)(64, 127)
    out = (ctypes.c_int64 * 2)(-5, -6)
    assert ctypes.sizeof(out) == 16  # a rank-2 shape is 16 bytes (Appendix A)
    assert lib.nimble_dense_shape(xs, 2, ws, 2, out) == -3
    assert (out[0], out[1]) == (-5, -6)
    assert "K" in nb.last_error()
    ws[1] = 128
    assert lib.nimble_dense_shape(xs, 2, ws, 2, out) == 0 and (out[0], out[1]) == (7, 64)
    assert lib.nimble_dense_shape(xs, 3, ws, 2, out) == -2
    assert lib.nimble_dense_shape(None, 2, ws, 2, out) == -1
    xs[0] = -1
    assert lib.nimble_dense_shape(xs, 2, ws, 2, out) == -8


@pytest.mark.parametrize("trans_b", [True, False])
def test_batch_matmul_shape_matches_oracle(trans_b):
    for L in (0, 1, 7, 64, 65, 512):
        a = (12, L, 64) if trans_b else (12, L, L)
        b = (12, L, 64)
        assert nb.batch_matmul_shape(a, b, trans_b) == oracle.batch_matmul_shape(a, b, trans_b)
    bad = [((12, 5, 64), (11, 5, 64)), ((12, 5, 64), (12, 9, 63) if trans_b else (12, 63, 9))]
    for a, b in bad:
        with pytest.raises(nb.NimbleError) as e:
            nb.batch_matmul_shape(a, b, trans_b)
        assert e.value.code == -3
        with pytest.raises(oracle.OracleShapeError):
            oracle.batch_matmul_shape(a, b, trans_b)
    with pytest.raises(nb.NimbleError) as e:
        nb.batch_matmul_shape((5, 64), (12, 9, 64), trans_b)
    assert e.value.code == -2


def test_lstm_shape_matches_oracle():
    for B in (0, 1, 16, 33, 64):
        args = ((B, 512), (B, 512), (B, 512), (2048, 1024))
        assert nb.lstm_shape(*args) == oracle.lstm_shape(*args) == ((B, 512), (B, 512))
    for bad in [((3, 512), (4, 512), (3, 512), (2048, 1024)), ((3, 512), (3, 512), (3, 511), (2048, 1024)),
                ((3, 512), (3, 512), (3, 512), (2047, 1024)), ((3, 512), (3, 512), (3, 512), (2048, 1023))]:
        with pytest.raises(nb.NimbleError) as e:
            nb.lstm_shape(*bad)
        assert e.value.code == -3


def test_storage_bytes_golden_and_oracle():
    itemsize_to_dtype = {4: nb.F32}
    for shape, itemsize, nbytes, align in _golden_rows("storage_sizes.txt"):
        dims = [int(d) for d in shape.split(",")]
        if int(itemsize) in itemsize_to_dtype:
            assert nb.storage_bytes(dims, itemsize_to_dtype[int(itemsize)]) == int(nbytes)
        assert nb.storage_alignment() == int(align)
    for shape in [(0, 4096), (1, 128), (8208, 4096), (12, 512, 512), ()]:
        assert nb.storage_bytes(shape, nb.BF16) == oracle.storage_bytes(shape, 2)
        assert nb.storage_bytes(shape, nb.F32) == oracle.storage_bytes(shape, 4)
    with pytest.raises(nb.NimbleError):
        nb.storage_bytes((3, -1), nb.BF16)
    with pytest.raises(nb.NimbleError):
        nb.storage_bytes((3, 4), 7)


def test_residue_split_matches_oracle_and_paper_example():
    for tile, copies, rmin, rmax in ([int(v) for v in r] for r in _golden_rows("residue_tile8.txt")):
        rs = {nb.residue_split(x, tile)[1] for x in range(0, 4 * tile)}
        assert rs == set(range(rmin, rmax + 1)) and len(rs) == copies
    for tile in (8, 16, 32, 64, 128, 256):
        for x in range(0, 2 * tile + 2):
            assert nb.residue_split(x, tile) == oracle.residue_split(x, tile)
    with pytest.raises(nb.NimbleError):
        nb.residue_split(3, 0)


@pytest.mark.parametrize("variant", sorted(TILED))
def test_plan_residue_identity_for_every_tiled_variant(variant):
    bm, bn = TILED[variant]
    for N, K in ((4096, 1024), (200, 72)):
        for M in range(1, 2 * bm + 2):
            p = nb.dense_plan(M, N, K, force_variant=variant)
            assert (p.variant, p.bm, p.bn) == (variant, bm, bn)
            assert p.k * bm + p.r == M and 0 <= p.r < bm
            assert (p.k, p.r) == oracle.residue_split(M, bm)
            tiles_m = p.k + (1 if p.r else 0)
            assert tiles_m * bm >= M > (tiles_m - 1) * bm
            assert p.grid[0] == tiles_m * -(-N // bn) and p.grid[2] == 1
            expect_residue = int(p.r != 0 or N % bn != 0 or K % p.bk != 0)
            assert p.residue_copy == expect_residue
            assert p.workspace_bytes == 0


def test_auto_dispatch_table():
    # small M streams the weights or runs small tiles with K cut, whichever is estimated faster;
    # large M goes to big tiles; ragged K falls back
    for M in range(1, 65):
        p = nb.dense_plan(M, 2048, 1024)
        assert p.name in ("skinny16", "t32x128", "t64x128")
        assert p.k * p.bm + p.r == M
        if p.name == "skinny16":
            # 128 column groups of 16 weight rows; K is whole 64-wide stages and the layer is small
            # enough to stay in the caches, so the rows go in blocks of 16 (the streaming kernel)
            blocks = p.grid[1]
            assert p.grid[0] == 128 and blocks == -(-M // 16)
        if M <= 16:
            assert p.name == "skinny16"
    assert nb.dense_plan(1, 2048, 1024).name == "skinny16"
    # cache-resident layers in whole 64-wide K stages: blocks of 16 rows, whatever the width
    assert nb.dense_plan(64, 768, 768, force_variant=1).grid[:2] == (48, 4)
    assert nb.dense_plan(64, 4096, 1024, force_variant=1).grid[:2] == (256, 4)
    assert nb.dense_plan(200, 4096, 1024, force_variant=1).grid[:2] == (256, 13)
    # K not in whole stages: the register-layout kernel.  A narrow layer spreads its rows over more
    # workgroups (each block at most four 16-row tiles), a wide one keeps one block per 64 rows
    assert nb.dense_plan(64, 768, 776, force_variant=1).grid[:2] == (48, 4)
    assert nb.dense_plan(64, 4096, 1032, force_variant=1).grid[:2] == (256, 1)
    assert nb.dense_plan(200, 4096, 1032, force_variant=1).grid[:2] == (256, 4)
    # a layer streamed from HBM: up to 16 rows the streaming kernel, one block; beyond that one block per
    # 64 rows so that the weights cross HBM once
    assert nb.dense_plan(16, 8192, 8192).name == "skinny16" and nb.dense_plan(16, 8192, 8192).grid[:2] == (512, 1)
    assert nb.dense_plan(64, 8192, 8192, force_variant=1).grid[:2] == (512, 1)
    assert nb.dense_plan(65, 2048, 1032).name.startswith("t")     # K not in whole stages: 64 rows at most
    assert nb.dense_plan(600, 2048, 1024).name.startswith("t")
    p = nb.dense_plan(16, 2048, 1024)
    assert (p.block, p.split_k, p.bk) == (512, 8, 64)             # the streaming kernel's launch shape
    p = nb.dense_plan(16, 2048, 1032)
    assert (p.block, p.split_k, p.bk) == (256, 4, 32)
    assert nb.dense_plan(8192, 4096, 1024).name in ("t256x256", "t256x128")
    assert nb.dense_plan(8192, 4096, 1024).residue_copy == 0
    # one row past a tile boundary: either the r != 0 copy, or the split dispatch
    # (k full tiles through the r = 0 copy, the residue rows through a small-M kernel)
    p = nb.dense_plan(8193, 4096, 1024)
    assert p.k * p.bm + p.r == 8193 and p.r == 8193 % p.bm
    if p.split_rows:
        assert p.split_rows == p.k * p.bm and p.residue_copy == 0
        assert nb.variant_name(p.residue_variant) in ("skinny16", "t32x128")   # one row left over
        assert p.grid[0] == (p.split_rows // p.bm) * (4096 // p.bn)
    else:
        assert p.residue_copy == 1 and p.grid[0] == (p.k + 1) * (4096 // p.bn)
    assert nb.dense_plan(100, 128, 100).name == "generic"
    assert nb.dense_plan(100, 128, 0).name == "generic"
    for M in range(65, 1200, 7):
        p = nb.dense_plan(M, 3072, 768)
        assert p.k * p.bm + p.r == M
    for M in list(range(2048, 2048 + 600, 5)) + list(range(5700, 10700, 37)):
        for (N, K) in ((4096, 1024), (1024, 4096)):
            p = nb.dense_plan(M, N, K)
            assert p.k * p.bm + p.r == M and 0 <= p.r < p.bm
            if p.split_rows:
                assert p.split_rows % p.bm == 0 and 0 < p.split_rows <= p.k * p.bm
                assert M - p.split_rows >= p.r and M - p.split_rows > 0
                assert p.residue_copy == 0 and N % p.bn == 0 and K % p.bk == 0
                assert p.grid[0] == (p.split_rows // p.bm) * (N // p.bn)
                assert nb.variant_name(p.residue_variant) is not None
                if M - p.split_rows <= 16:
                    assert nb.variant_name(p.residue_variant) in ("skinny16", "t32x128")
            forced = nb.dense_plan(M, N, K, force_variant=p.variant)
            assert forced.split_rows == 0  # a forced variant is one launch


def test_forced_tile_height_plans():
    # the 256-wide variant at its other heights: same residue identity, grid from the chosen height
    for rows in (128, 160, 192, 224, 256, 288, 320):
        forced = 6 | ((rows // 16) << 16)
        for M in list(range(1, 2 * rows + 2, 7)) + [8192, 8193, 10000]:
            p = nb.dense_plan(M, 4096, 1024, force_variant=forced)
            assert (p.variant, p.bm, p.bn) == (6, rows, 256)
            assert (p.k, p.r) == oracle.residue_split(M, rows)
            assert p.grid[0] == -(-M // rows) * 16 and p.split_rows == 0 and p.split_k == 1
            assert p.residue_copy == int(p.r != 0)
    for bad in (6 | (9 << 16), 6 | (21 << 16), 5 | (12 << 16), 4 | (6 << 16)):  # 144, 336 rows; other variants
        with pytest.raises(nb.NimbleError) as e:
            nb.dense_plan(1000, 4096, 1024, force_variant=bad)
        assert e.value.code == -8
    with pytest.raises(nb.NimbleError):   # no ragged N for the other heights
        nb.dense_plan(1000, 4096 + 128, 1024, force_variant=6 | (12 << 16))
    with pytest.raises(nb.NimbleError):   # nor ragged K
        nb.dense_plan(1000, 4096, 1024 + 8, force_variant=6 | (12 << 16))
    with pytest.raises(nb.NimbleError):   # nor together with a K split
        nb.dense_plan(1000, 4096, 1024, force_variant=6 | (12 << 16) | (2 << 8))
    # automatic choice: the tile rows of the chosen height fit the rounds a taller or shorter
    # 256-row tiling would have wasted
    for M in range(5700, 10700, 61):
        for (N, K) in ((4096, 1024), (1024, 4096)):
            p = nb.dense_plan(M, N, K)
            if p.variant == 6 and p.bm != 256:
                assert p.split_rows == 0 and N % 256 == 0 and K % 32 == 0
                assert p.grid[0] == -(-M // p.bm) * (N // 256)
                rounds = -(-p.grid[0] // 256)
                assert -(-(-(-M // 256) * (N // 256)) // 256) >= rounds or p.bm < 256


def test_plan_rejects_bad_arguments():
    for args in [(-1, 128, 128), (5, -1, 128), (5, 128, -8)]:
        with pytest.raises(nb.NimbleError) as e:
            nb.dense_plan(*args)
        assert e.value.code == -8
    with pytest.raises(nb.NimbleError):
        nb.dense_plan(5, 128, 128, epilogue=9)
    with pytest.raises(nb.NimbleError):
        nb.dense_plan(5, 128, 128, force_variant=99)
    with pytest.raises(nb.NimbleError):
        nb.dense_plan(5, 128, 100, force_variant=4)  # tiled needs K % 8 == 0
    with pytest.raises(nb.NimbleError):
        nb.lstm_plan(4, 510, 512)


def test_lstm_plan():
    for B in range(0, 130):
        p = nb.lstm_plan(B, 512, 512)
        assert p.k * 16 + p.r == B and p.grid[0] == 128
        # row blocks of 16 (Ix and K in whole 64-wide stages, 4 MB of weights: the streaming kernel)
        blocks = p.grid[1]
        assert blocks == max(1, -(-B // 16))
        # x | h boundary not on a stage boundary: the register-layout kernel; row blocks of at most four
        # 16-row tiles each, as many as keep the grid within one workgroup per compute unit (128 column
        # groups -> 2), more only when B forces it
        q = nb.lstm_plan(B, 480, 512)
        blocks = q.grid[1]
        tiles = -(-B // (16 * blocks))
        assert tiles <= 4 and blocks * 16 * tiles >= B
        assert blocks == max(1, -(-B // 64), min(-(-B // 16), 2))
    assert nb.lstm_plan(64, 64, 64).grid[:2] == (16, 4)     # a narrow layer is cut along the batch instead
    assert nb.lstm_plan(16, 64, 64).grid[:2] == (16, 1)


def test_device_entry_points_validate_before_touching_the_gpu():
    # every one of these must be refused on the host (no GPU in this process)
    lib = nb.load()
    assert lib.nimble_dense_dyn(None, None, None, None, 4, 128, 128, 1, 0, None, 0, None) == -1
    assert lib.nimble_dense_dyn(16, 32, 48, 64, -4, 128, 128, 1, 0, None, 0, None) == -8
    assert lib.nimble_dense_dyn(16, 32, 48, 64, 4, 128, 128, 7, 0, None, 0, None) == -8
    assert lib.nimble_dense_dyn(16, 32, 48, 64, 4, 128, 128, 1, 5, None, 0, None) == -4
    assert lib.nimble_dense_dyn(16, 32, 48, 68, 4, 128, 128, 1, 0, None, 0, None) == -5
    assert lib.nimble_dense_dyn(16, 32, None, 64, 4, 128, 128, 1, 0, None, 0, None) == -1
    # M = 0 is a legal instantiation of the dynamic dimension: nothing to do
    assert lib.nimble_dense_dyn(None, None, None, None, 0, 128, 128, 1, 0, None, 0, None) == 0
    assert lib.nimble_batch_matmul_dyn(None, None, None, 12, 0, 0, 64, 1, 0.125, 1, None, 0, None) == 0
    assert lib.nimble_batch_matmul_dyn(16, 32, 50, 12, 4, 4, 64, 1, 0.125, 1, None, 0, None) == -5
    assert lib.nimble_softmax_rows_dyn(None, None, 0, 5, None) == 0
    assert lib.nimble_softmax_rows_dyn(None, None, 3, 5, None) == -1
    assert lib.nimble_attention_dyn(None, None, None, None, 12, 0, 64, 0.125, None) == 0
    assert lib.nimble_attention_dyn(None, None, None, None, 12, 5, 64, 0.125, None) == -1
    assert lib.nimble_attention_dyn(16, 32, 48, 72, 12, 5, 64, 0.125, None) == -5
    assert lib.nimble_attention_dyn(16, 32, 48, 64, 12, 5, 80, 0.125, None) == -8
    for bad_alpha in (0.0, -0.125, float("nan")):   # the fused softmax works on raw scores: the scale must be > 0
        assert lib.nimble_attention_dyn(16, 32, 48, 64, 12, 5, 64, bad_alpha, None) == -8
    assert lib.nimble_lstm_gates_dyn(16, 32, 48, 64, 80, 96, 112, 0, 512, 512, None, 0, None) == 0
    assert lib.nimble_lstm_gates_dyn(16, 32, 48, 64, 80, 96, 32, 3, 512, 512, None, 0, None) == -8  # h_out aliases h_prev
    assert lib.nimble_lstm_gates_dyn(16, 32, 48, 64, 80, 96, 112, 3, 511, 512, None, 0, None) == -8
    assert lib.nimble_lstm_gates_pre_dyn(16, 32, 48, 64, 80, 96, 0, 512, None) == 0       # B = 0: nothing to do
    assert lib.nimble_lstm_gates_pre_dyn(None, 32, 48, 64, 80, 96, 3, 512, None) == -1
    assert lib.nimble_lstm_gates_pre_dyn(16, 32, 48, 64, 80, 32, 3, 512, None) == -8      # h_out aliases h_prev
    assert lib.nimble_lstm_gates_pre_dyn(16, 32, 48, 64, 80, 100, 3, 512, None) == -5
    assert lib.nimble_lstm_gates_pre_dyn(16, 32, 48, 64, 80, 96, 3, 510, None) == -8


def test_storage_arena_offsets_alignment_and_overflow():
    # storage coalescing (Section 3.3): one block, tensors carved at aligned offsets computed from
    # the shape function's result; runs on host memory here, the arithmetic is the same
    torch = pytest.importorskip("torch")
    from paper_2006_03031_amd import runtime as rt
    arena = rt.StorageArena(10_000, device="cpu")
    assert arena.alignment >= nb.storage_alignment() and arena.alignment % 64 == 0
    a = arena.alloc((3, 5), nb.BF16)       # 30 bytes
    b = arena.alloc((7,), nb.F32)          # 28 bytes, next aligned offset
    assert a.dtype == torch.bfloat16 and tuple(a.shape) == (3, 5)
    assert b.dtype == torch.float32 and tuple(b.shape) == (7,)
    base = arena.storage.data_ptr() + arena._base_off
    assert a.data_ptr() == base and a.data_ptr() % arena.alignment == 0
    assert b.data_ptr() == base + arena.alignment and arena.offset == arena.alignment + 28
    # the tensors are views of the one storage: writing one does not touch the other
    a.fill_(1.0)
    b.fill_(2.0)
    assert float(a.float().sum()) == 15.0 and float(b.sum()) == 14.0
    # an empty tensor (M = 0) is a legal allocation of zero bytes
    z = arena.alloc((0, 4096), nb.BF16)
    assert z.numel() == 0
    with pytest.raises(MemoryError):
        arena.alloc((100, 100), nb.F32)
    used = arena.offset
    arena.reset()
    assert arena.offset == 0 and used > 0
    c = arena.alloc((3, 5), nb.BF16)
    assert c.data_ptr() == a.data_ptr()    # the block is reused from the start


def test_plan_invariants_on_random_shapes():
    # whatever the cost model picks, the plan must describe a launch that covers the problem exactly
    rng = np.random.default_rng(7)
    names = set()
    for _ in range(600):
        M = int(rng.choice([rng.integers(1, 70), rng.integers(1, 3000), rng.integers(1, 20000)]))
        N = int(rng.choice([rng.integers(1, 600), rng.integers(1, 40) * 128, rng.integers(1, 17) * 256]))
        K = int(rng.choice([rng.integers(1, 600), rng.integers(1, 130) * 32, rng.integers(1, 65) * 64]))
        epi = int(rng.integers(0, 3))
        p = nb.dense_plan(M, N, K, epi)
        names.add(p.name)
        assert p.k * p.bm + p.r == M and 0 <= p.r < p.bm
        if p.name == "generic":
            assert K % 8 != 0
            continue
        assert K % 8 == 0
        if p.name == "skinny16":
            blocks = p.grid[1]
            assert p.grid[0] == -(-N // 16) and -(-M // (16 * blocks)) <= 4 and p.workspace_bytes == 0
            if K % 64 == 0 and N * K * 2 <= 64e6:
                assert blocks == -(-M // 16)
            continue
        rows = p.split_rows if p.split_rows else M
        assert p.grid[0] == -(-rows // p.bm) * -(-N // p.bn)
        if p.split_rows:
            assert p.split_rows % p.bm == 0 and 0 < p.split_rows < M and p.split_k == 1
            # the second launch is reported as it will run: planned alone it gives the same variant, K
            # split and scratch need
            tail = nb.dense_plan(M - p.split_rows, N, K, epi)
            assert (p.residue_variant, p.residue_split_k) == (tail.variant, tail.split_k)
            if tail.split_rows == 0:
                assert p.workspace_bytes == tail.workspace_bytes
            continue
        if p.split_k > 1:
            assert N % p.bn == 0 and K % 32 == 0 and p.workspace_bytes == p.split_k * M * N * 4
            assert p.workspace_bytes <= 64 << 20   # plans are made within the default scratch
            stages = K // 32
            per = -(-stages // p.split_k)
            assert per * (p.split_k - 1) < stages          # every slice has work
        else:
            assert p.workspace_bytes == 0
        if p.bm not in (32, 64, 128, 256):                 # a reduced or raised height of the 256-wide tile
            assert p.name == "t256x256" and N % 256 == 0 and K % 32 == 0
    assert {"skinny16", "t32x128", "t256x256"} <= names


def test_batch_matmul_plan_nn_workspace():
    # NN on the tiled kernels needs b transposed: the plan asks for exactly that much scratch
    p = nb.batch_matmul_plan(12, 512, 64, 512, False)
    assert p.name != "generic" and p.workspace_bytes == 12 * 64 * 512 * 2 and p.grid[2] == 12
    for (T, M, N, K) in [(12, 128, 64, 128), (4, 33, 64, 33), (2, 129, 40, 257), (1, 5000, 64, 12)]:
        p = nb.batch_matmul_plan(T, M, N, K, False)
        assert p.name == "generic" and p.workspace_bytes == 0
    assert nb.batch_matmul_plan(12, 512, 512, 64, True).workspace_bytes == 0


def test_batch_matmul_plans_are_one_launch_covering_every_row():
    """batch_matmul launches its plan as it stands: the plan must never split the rows in two
    launches or cut K, and the r = 0 copy (no bounds code) may only be chosen when no tile is ragged."""
    rng = np.random.default_rng(11)
    shapes = [(1, 10764, 4096, 1024), (1, 8300, 1024, 4096), (1, 16, 128, 128), (1, 64, 2304, 768)]
    for _ in range(1500):
        T = int(rng.choice([1, 1, 2, 12, 40]))
        M = int(rng.choice([rng.integers(1, 70), rng.integers(65, 3000), rng.integers(3000, 40000)]))
        N = int(rng.choice([rng.integers(1, 600), rng.integers(1, 40) * 128, rng.integers(1, 17) * 256]))
        K = int(rng.choice([rng.integers(1, 600), rng.integers(1, 130) * 32, rng.integers(1, 65) * 64]))
        shapes.append((T, M, N, K))
    for (T, M, N, K) in shapes:
        for trans_b in (True, False):
            p = nb.batch_matmul_plan(T, M, N, K, trans_b)
            assert p.split_rows == 0, (T, M, N, K, trans_b, p)
            assert p.grid[2] == (T if p.name != "skinny16" else 1)
            if p.variant >= 2:
                assert p.split_k == 1
                assert p.grid[0] == -(-M // p.bm) * -(-N // p.bn)
                if not p.residue_copy:
                    assert M % p.bm == 0 and N % p.bn == 0 and K % p.bk == 0, (T, M, N, K, p)
            if p.name == "skinny16":
                assert T == 1 and trans_b and M <= 512


def test_lstm_pre_shape_matches_oracle():
    for B in (0, 1, 16, 33, 64):
        args = ((B, 2048), (B, 512), (B, 512), (2048, 512))
        assert nb.lstm_pre_shape(*args) == oracle.lstm_pre_shape(*args) == ((B, 512), (B, 512))
    for bad in [((3, 2048), (4, 512), (3, 512), (2048, 512)), ((3, 2047), (3, 512), (3, 512), (2048, 512)),
                ((3, 2048), (3, 512), (3, 511), (2048, 512)), ((3, 2048), (3, 512), (3, 512), (2048, 1024)),
                ((3, 2048), (3, 512), (3, 512), (2040, 512)), ((2, 2048), (3, 512), (3, 512), (2048, 512))]:
        with pytest.raises(nb.NimbleError) as e:
            nb.lstm_pre_shape(*bad)
        assert e.value.code == -3
        with pytest.raises(oracle.OracleShapeError):
            oracle.lstm_pre_shape(*bad)
    with pytest.raises(nb.NimbleError) as e:
        nb.lstm_pre_shape((3, 2048), (3, -512), (3, 512), (2048, 512))
    assert e.value.code == -8
    lib = nb.load()
    out = (ctypes.c_int64 * 2)(-5, -6)
    four = [(ctypes.c_int64 * 2)(*v) for v in ((3, 32), (3, 8), (3, 8), (32, 9))]
    assert lib.nimble_lstm_pre_shape(*four, out, out) == -3 and (out[0], out[1]) == (-5, -6)  # untouched on error
    assert lib.nimble_lstm_pre_shape(None, four[1], four[2], four[3], out, out) == -1


def test_lstm_seq_shape_support_and_refusals():
    """The one-launch token loop: shape function against the oracle twin, the shapes it runs, its
    workspace size, and every refusal that is decided before anything is launched."""
    for T, B, H in [(0, 1, 512), (128, 1, 512), (5, 16, 1024), (3, 40, 72)]:
        args = ((T, B, 4 * H), (B, H), (B, H), (4 * H, H))
        assert nb.lstm_seq_shape(*args) == oracle.lstm_seq_shape(*args) == ((T, B, H), (B, H))
    for bad in [((7, 4, 32), (3, 8), (3, 8), (32, 8)), ((7, 3, 31), (3, 8), (3, 8), (32, 8)),
                ((7, 3, 32), (3, 8), (3, 9), (32, 8)), ((7, 3, 32), (3, 8), (3, 8), (32, 9))]:
        with pytest.raises(nb.NimbleError) as e:
            nb.lstm_seq_shape(*bad)
        assert e.value.code == -3
        with pytest.raises(oracle.OracleShapeError):
            oracle.lstm_seq_shape(*bad)
    with pytest.raises(nb.NimbleError) as e:
        nb.lstm_seq_shape((-7, 3, 32), (3, 8), (3, 8), (32, 8))
    assert e.value.code == -8
    ok = [(1, 64), (1, 512), (4, 512), (4, 1024), (3, 576)]
    no = [(0, 512), (5, 512), (16, 512), (1, 32), (1, 96), (1, 1088), (1, 2048), (-1, 512)]
    assert all(nb.lstm_seq_supported(B, H) for B, H in ok) and not any(nb.lstm_seq_supported(B, H) for B, H in no)
    assert [nb.lstm_seq_preferred(B, H) for B, H in [(1, 512), (4, 256), (1, 1024), (2, 1024), (5, 512)]] == \
        [True, True, True, False, False]
    assert nb.lstm_seq_workspace_bytes(4, 512) == 256 + 2 * 4 * 512 * 4
    assert nb.lstm_seq_workspace_bytes(5, 512) == 0
    # refusals: nothing is launched (no GPU here), the message names the reason
    call = nb.nimble_lstm_seq_pre_dyn
    a = 4096   # any non-null, 16-byte aligned number: never dereferenced on these paths
    for args, code in [((a, a, a, a, a, a, 5, 5, 512, a, 1 << 20, 10, 0), -3),
                       ((a, a, a, a, a, a, 5, 1, 96, a, 1 << 20, 10, 0), -3),
                       ((a, a, a, a, a, a, -1, 1, 512, a, 1 << 20, 10, 0), -8),
                       ((a, a, 0, a, a, a, 5, 1, 512, a, 1 << 20, 10, 0), -1),
                       ((a, a, a, a, a, a, 5, 1, 512, 0, 1 << 20, 10, 0), -1),
                       ((a, a + 8, a, a, a, a, 5, 1, 512, a, 1 << 20, 10, 0), -5),
                       ((a, a, a, a, a, a, 5, 1, 512, a, 256 + 2 * 512 * 4 - 1, 10, 0), -6)]:
        with pytest.raises(nb.NimbleError) as e:
            call(*args)
        assert e.value.code == code, (args, e.value)
    call(a, a, a, a, a, a, 0, 1, 512, a, 1 << 20, 10, 0)   # T = 0: nothing to do, nothing launched


def test_tuned_table_overrides_the_cost_model():
    """Section 3.5, tuning: an installed entry decides the dispatch inside its M range and nowhere
    else; entries that cannot run are skipped; count = 0 removes the table."""
    N, K, epi = 768, 3072, nb.EPI_BIAS
    before = {M: nb.dense_plan(M, N, K, epi) for M in (1, 64, 65, 100, 256, 257, 300, 1000)}
    others = [(100, N, K, nb.EPI_NONE), (100, N, K, nb.EPI_BIAS_GELU_ERF), (100, 2304, 768, epi), (100, K, N, epi)]
    before_others = [nb.dense_plan(*o) for o in others]
    try:
        # (m_lo, m_hi, variant, split_k): 64x128 tiles with K cut in 4 for 65..256, weight streaming up to 64
        nb.dense_table_set(N, K, epi, [(65, 256, 3, 4), (1, 64, 1, 1)])
        for M in (65, 100, 256):
            p = nb.dense_plan(M, N, K, epi)
            assert (p.name, p.split_k, p.split_rows) == ("t64x128", 4, 0)
            assert p.workspace_bytes == 4 * M * N * 4 and p.grid[:2] == (-(-M // 64) * 6, 4)
        for M in (1, 64):
            assert nb.dense_plan(M, N, K, epi).name == "skinny16"
        for M in (257, 300, 1000):          # outside every range: the cost model, unchanged
            assert nb.dense_plan(M, N, K, epi) == before[M]
        # keyed by (N, K, epilogue): other layers and other epilogues are not affected
        assert [nb.dense_plan(*o) for o in others] == before_others
        # a forced variant ignores the table
        assert nb.dense_plan(100, N, K, epi, force_variant=4).name == "t128x128"
        # an entry that cannot run this shape is skipped: K = 3072 + 8 has no whole 32-wide stages to cut
        nb.dense_table_set(N, K + 8, epi, [(1, 4096, 4, 4)])
        p = nb.dense_plan(300, N, K + 8, epi)
        assert not (p.name == "t128x128" and p.split_k == 4)
        nb.dense_table_set(N, K + 8, epi, [])
        # replacing a table replaces every entry of that key
        nb.dense_table_set(N, K, epi, [(100, 100, 5, 1)])
        assert nb.dense_plan(100, N, K, epi).name == "t256x128"
        assert nb.dense_plan(65, N, K, epi) == before[65]
        nb.dense_table_set(N, K, epi, [])
        for M, p in before.items():
            assert nb.dense_plan(M, N, K, epi) == p
        # malformed entries are refused and leave no table behind
        for bad in [[(5, 4, 3, 1)], [(-1, 4, 3, 1)], [(1, 4, 0, 1)], [(1, 4, 7, 1)], [(1, 4, 3, 65)]]:
            with pytest.raises(nb.NimbleError) as e:
                nb.dense_table_set(N, K, epi, bad)
            assert e.value.code == -8
            assert nb.dense_plan(4, N, K, epi).name == "skinny16"
        assert nb.dense_plan(100, N, K, epi) == before[100]
        # weight streaming beyond 64 rows can be tabled only where the streaming kernel runs (K in whole
        # 64-wide stages: rows go in blocks of 16)
        with pytest.raises(nb.NimbleError):
            nb.dense_table_set(N, K + 8, epi, [(1, 65, 1, 1)])
        nb.dense_table_set(N, K, epi, [(65, 200, 1, 1)])
        p = nb.dense_plan(200, N, K, epi)
        assert p.name == "skinny16" and p.grid[:2] == (48, 13)
        nb.dense_table_set(N, K, epi, [])
    finally:
        nb.dense_table_set(N, K, epi, [])
        nb.dense_table_set(N, K + 8, epi, [])


def test_tabled_k_split_needs_the_workspace_it_asks_for():
    """The entry point plans within the scratch the caller brings: a tabled K split that does not fit
    is skipped there (checked here through the plan a caller with no scratch would get: the device
    entry point refuses on the host when pointers are null, after planning)."""
    N, K, epi = 768, 3072, nb.EPI_BIAS
    lib = nb.load()
    try:
        nb.dense_table_set(N, K, epi, [(65, 256, 3, 4)])
        # with no workspace the tabled split cannot run; the call still plans (and then stops at the
        # null tensors): no NIMBLE_ERR_WORKSPACE
        assert lib.nimble_dense_dyn(None, None, None, None, 100, N, K, epi, 0, None, 0, None) == -1
    finally:
        nb.dense_table_set(N, K, epi, [])


def test_forced_variant_and_k_split_from_the_environment():
    """NIMBLE_FORCE_VARIANT (a measurement knob, read once per process) carries the forced K split in
    bits 8..15 like the force_variant argument does."""
    import subprocess
    import sys
    code = ("import paper_2006_03031_amd as nb; p = nb.dense_plan(300, 768, 3072); "
            "print(p.name, p.split_k, p.workspace_bytes)")
    env = dict(os.environ, NIMBLE_FORCE_VARIANT=str(4 | (2 << 8)))
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    out = subprocess.run([sys.executable, "-c", code], env=env, cwd=root, capture_output=True, text=True, check=True)
    assert out.stdout.split() == ["t128x128", "2", str(2 * 300 * 768 * 4)]


def test_no_alloc_entry_point_refuses_what_its_scratch_cannot_hold():
    # host-side validation only (no GPU in this process): the refusal comes before any device access
    lib = nb.load()
    big = nb.dense_plan(1088, 4096, 16384, nb.EPI_BIAS)
    assert big.workspace_bytes > nb.NOALLOC_SCRATCH_BYTES
    assert lib.nimble_dense_noalloc_dyn(16, 32, 48, 64, 1088, 4096, 16384, 1, 0, None) == -6
    assert "scratch" in nb.last_error()
    assert lib.nimble_dense_noalloc_dyn(16, 32, 48, 64, 4, 128, 128, 7, 0, None) == -8      # unknown epilogue
    assert lib.nimble_dense_noalloc_dyn(16, 32, 48, 64, 4, 128, 128, 1, 9, None) == -4      # unknown dtype
    assert lib.nimble_dense_noalloc_dyn(16, 32, 48, 64, -4, 128, 128, 1, 0, None) == -8
    assert lib.nimble_dense_noalloc_dyn(None, None, None, None, 0, 128, 128, 1, 0, None) == 0  # M = 0: nothing to do

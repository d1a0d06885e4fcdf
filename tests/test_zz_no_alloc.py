"""The entry point that allocates nothing (nimble_dense_noalloc_dyn: the K-split partial sums go to a
scratch array built into the library) against nimble_dense_dyn with a caller workspace: same plan,
same kernels, so the outputs must agree bit for bit, and both stay within the parity bar of the
oracle.  Two calls in a row on the shared scratch, the second with a smaller input."""
import numpy as np
import pytest

import oracle
import workloads as wl

torch = pytest.importorskip("torch")
pytestmark = pytest.mark.gpu

TOL = 5e-3


def test_no_alloc_dense_two_calls_in_a_row_match_the_workspace_entry_point():
    import paper_2006_03031_amd as nb
    from gpu_util import bits_from_dev, from_dev, to_dev
    nb.load()
    N, K = 768, 3072
    rng = np.random.default_rng(2024)
    w, b = wl.normal_bf16(rng, (N, K)), wl.uniform_bf16(rng, (N,))
    wd, bd = to_dev(w), to_dev(b)
    stream = torch.cuda.current_stream().cuda_stream
    # the first call cuts K (partial sums in the scratch), the second is smaller and cuts K again on
    # what the first left behind, the third streams the weights and uses no scratch at all
    cases = [(700, nb.EPI_BIAS_GELU_ERF, "bias_gelu"), (600, nb.EPI_BIAS, "bias"), (8, nb.EPI_BIAS, "bias")]
    plans = [nb.dense_plan(M, N, K, epi) for M, epi, _ in cases]
    assert plans[0].split_k > 1 and plans[1].split_k > 1 and plans[1].workspace_bytes < plans[0].workspace_bytes
    assert plans[2].workspace_bytes == 0
    xs = [wl.uniform_bf16(rng, (M, K)) for M, _, _ in cases]
    xd = [to_dev(x) for x in xs]
    # reference: the existing entry point with exactly the workspace its plan asks for
    refs = []
    for (M, epi, _), x, p in zip(cases, xd, plans):
        ws = torch.empty(max(int(p.workspace_bytes), 16), dtype=torch.uint8, device="cuda")
        y = torch.full((M + 2, N), 768.0, dtype=torch.bfloat16, device="cuda")
        nb.nimble_dense_dyn(x.data_ptr(), wd.data_ptr(), bd.data_ptr(), y.data_ptr(), M, N, K, epi, nb.BF16,
                            ws.data_ptr(), int(p.workspace_bytes), stream)
        torch.cuda.synchronize()
        refs.append(bits_from_dev(y))
    outs = [torch.full((M + 2, N), 768.0, dtype=torch.bfloat16, device="cuda") for M, _, _ in cases]
    torch.cuda.synchronize()
    free_before, _ = torch.cuda.mem_get_info()
    for rep in range(2):   # the whole sequence twice: the scratch keeps the last call's contents
        for (M, epi, _), x, y in zip(cases, xd, outs):
            y.fill_(768.0)
            nb.nimble_dense_noalloc_dyn(x.data_ptr(), wd.data_ptr(), bd.data_ptr(), y.data_ptr(), M, N, K, epi,
                                        nb.BF16, stream)
        torch.cuda.synchronize()
        for (M, epi, name), x, y, ref in zip(cases, xs, outs, refs):
            got = bits_from_dev(y)
            assert np.array_equal(got, ref), ("differs from nimble_dense_dyn", M, rep)
            assert np.all(from_dev(y)[M:] == 768.0), ("wrote past row M", M)
            want = oracle.dense(x.f32, w.f32, b.f32, name)
            assert oracle.normwise_rel_error(from_dev(y)[:M], want) <= TOL, (M, rep)
            assert oracle.elementwise_excess(from_dev(y)[:M], want, 2.0 ** -7, 2.0 ** -7) <= 1.0, (M, rep)
    free_after, _ = torch.cuda.mem_get_info()
    assert free_after == free_before, "device memory was allocated or freed during the calls"
    # f32 output and M = 0
    y32 = torch.empty((700, N), dtype=torch.float32, device="cuda")
    nb.nimble_dense_noalloc_dyn(xd[0].data_ptr(), wd.data_ptr(), bd.data_ptr(), y32.data_ptr(), 700, N, K,
                                nb.EPI_BIAS, nb.F32, stream)
    torch.cuda.synchronize()
    assert oracle.normwise_rel_error(from_dev(y32), oracle.dense(xs[0].f32, w.f32, b.f32, "bias")) <= 1e-5
    nb.nimble_dense_noalloc_dyn(0, wd.data_ptr(), bd.data_ptr(), 0, 0, N, K, nb.EPI_BIAS, nb.BF16, stream)
    # a shape whose plan needs more than the built-in scratch is refused on the host, nothing runs
    big = nb.dense_plan(1088, 4096, 16384, nb.EPI_BIAS)
    assert big.workspace_bytes > nb.NOALLOC_SCRATCH_BYTES
    with pytest.raises(nb.NimbleError) as e:
        nb.nimble_dense_noalloc_dyn(xd[0].data_ptr(), wd.data_ptr(), bd.data_ptr(), outs[0].data_ptr(), 1088, 4096,
                                    16384, nb.EPI_BIAS, nb.BF16, stream)
    assert e.value.code == -6 and "scratch" in str(e.value)
    torch.cuda.synchronize()

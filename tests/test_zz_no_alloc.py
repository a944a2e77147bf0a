"""The entry point that allocates nothing (``mttkrp_dense_f64_noalloc``): same results as
``mttkrp_dense_f64`` bit for bit (same plan, same kernels, another workspace), on calls in a
row that share the library's one scratch array, the later ones with smaller inputs; the
result also matches the oracle; shapes beyond the array's size are rejected."""
import numpy as np
import pytest

torch = pytest.importorskip("torch")

from paper_2510_14891_amd import inputs

pytestmark = pytest.mark.gpu

SCRATCH_BYTES = 64 << 20


@pytest.fixture(scope="module")
def mt():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    from paper_2510_14891_amd import binding
    binding.lib()
    return binding


def problem(dims, R, seed):
    n = int(np.prod(dims))
    X = inputs.uniform(seed, n, -1.0, 1.0)
    A = [inputs.uniform(seed + 10 + m, (I, R), -1.0, 1.0) for m, I in enumerate(dims)]
    return X, A


def test_noalloc_matches_core_call_on_calls_in_a_row(mt, oracle):
    # first a shape with many partial slots and a fused column pair, then smaller ones that
    # reuse the front of the same scratch array, then the first again
    shapes = [((200, 37, 29, 11), 48, 900), ((150, 31, 21), 16, 901), ((33, 9, 5), 3, 902),
              ((200, 37, 29, 11), 48, 900)]
    for dims, R, seed in shapes:
        X, A = problem(dims, R, seed)
        Xd, Ad = X.cuda(), [a.cuda() for a in A]
        for k in range(len(dims)):
            assert 0 <= mt.mttkrp_dense_workspace_bytes(dims, R, k, 8) <= SCRATCH_BYTES
            want = mt.mttkrp_dense(Xd, dims, Ad, k)
            M = torch.full((dims[k], R), float("nan"), dtype=torch.float64, device="cuda")
            before = torch.cuda.memory_allocated()
            mt.mttkrp_dense_noalloc(Xd, dims, Ad, k, M)
            assert torch.cuda.memory_allocated() == before
            torch.cuda.synchronize()
            assert torch.equal(M, want), (dims, k)
            ref = oracle.mttkrp(inputs.as_ndarray_view(X, dims), [a.numpy() for a in A], k)
            assert oracle.normwise_rel_err(M.cpu().numpy(), ref) <= 1e-12, (dims, k)


def test_noalloc_large_then_small_benchmark_shape(mt):
    """Scaled benchmark shapes whose partial sums fill a good part of the array."""
    for dims, R in (((1024, 512, 64), 32), ((512, 128, 32), 32)):
        n = int(np.prod(dims))
        X = inputs.uniform(77, n, -1.0, 1.0, device="cuda")
        A = [inputs.uniform(78 + m, (I, R), -1.0, 1.0, device="cuda") for m, I in enumerate(dims)]
        for k in range(3):
            want = mt.mttkrp_dense(X, dims, A, k)
            M = torch.empty_like(want)
            mt.mttkrp_dense_noalloc(X, dims, A, k, M)
            torch.cuda.synchronize()
            assert torch.equal(M, want), (dims, k)


def test_noalloc_rejects_shapes_beyond_the_array(mt):
    # a plan that needs more than 64 MiB: checked with the host-side query before the call
    dims, R, k = (16384, 2048, 64), 512, 0
    assert mt.mttkrp_dense_workspace_bytes(dims, R, k, 8) > SCRATCH_BYTES
    X = torch.zeros(16384 * 2048 * 64, dtype=torch.float64, device="cuda")
    A = [torch.zeros((I, R), dtype=torch.float64, device="cuda") for I in dims]
    M = torch.full((dims[k], R), 7.0, dtype=torch.float64, device="cuda")
    with pytest.raises(mt.MttkrpError) as e:
        mt.mttkrp_dense_noalloc(X, dims, A, k, M)
    assert e.value.status == mt.MTTKRP_ERR_WORKSPACE
    torch.cuda.synchronize()
    assert bool((M == 7.0).all())          # nothing was enqueued
    del X
    torch.cuda.empty_cache()

"""The calls that take a caller-owned workspace enqueue kernels only (no allocation, no memset,
no copy), so a caller may record them into a HIP graph.  Each graph here is replayed several times
with new tensor values in the same buffers and with eager work and synchronisations between the
replays; every replay must equal the eager result of the same call bit for bit (the schedules are
deterministic) and agree with the oracle."""
import numpy as np
import pytest
import torch

from paper_2510_14891_amd import inputs

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def mt():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    from paper_2510_14891_amd import binding
    binding.lib()
    return binding

CASES = [
    # dims, R, dtype: the small benchmark configuration; paired rows for the second mode with a
    # fused column pair (its partial sums are zero-filled by a kernel at every call); the second
    # schedule (k = 1, 2); a first mode with several splits and the LDS sum in fp32
    ((64, 64, 64), 16, torch.float64),
    ((129, 9, 40, 7), 10, torch.float64),
    ((300, 7, 9), 16, torch.float64),
    ((48, 24, 20, 30), 24, torch.float32),
]


def _fill(seed, dims, R, dtype):
    X = inputs.uniform(seed, int(np.prod(dims)), -1.0, 1.0, dtype=dtype)
    A = [inputs.uniform(seed + 1 + m, dims[m] * R, -1.0, 1.0, dtype=dtype).reshape(dims[m], R) for m in range(len(dims))]
    return X, A


@pytest.mark.parametrize("dims,R,dtype", CASES)
def test_core_calls_replayed_from_a_graph(mt, oracle, dims, R, dtype):
    sb = 8 if dtype == torch.float64 else 4
    tol = 1e-12 if dtype == torch.float64 else 2e-5
    d = len(dims)
    X0, A0 = _fill(500, dims, R, dtype)
    X = X0.cuda()
    A = [a.cuda() for a in A0]
    M = [torch.zeros((dims[k], R), dtype=dtype, device="cuda") for k in range(d)]
    ws = [torch.empty(max(1, mt.mttkrp_dense_workspace_bytes(dims, R, k, sb)), dtype=torch.uint8, device="cuda")
          for k in range(d)]
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):          # first calls outside the capture (one-time set-up per device)
        for k in range(d):
            mt.mttkrp_dense(X, dims, A, k, M=M[k], workspace=ws[k])
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        for k in range(d):
            mt.mttkrp_dense(X, dims, A, k, M=M[k], workspace=ws[k])
    for replay in range(4):
        Xn, An = _fill(600 + 10 * replay, dims, R, dtype)
        X.copy_(Xn.cuda())
        for a, an in zip(A, An):
            a.copy_(an.cuda())
        for m in M:
            m.fill_(float("nan"))
        for w in ws:
            w.fill_(255)                    # stale partial sums (NaN patterns) must not leak into M
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        got = [m.clone() for m in M]
        eager = [mt.mttkrp_dense(X, dims, A, k, workspace=ws[k]) for k in range(d)]
        torch.cuda.synchronize()
        Xv = inputs.as_ndarray_view(Xn, dims)
        for k in range(d):
            assert torch.equal(got[k], eager[k]), (dims, R, k, replay)
            ref = oracle.mttkrp(Xv, [a.numpy() for a in An], k)
            assert oracle.normwise_rel_err(got[k].cpu().numpy(), ref) <= tol, (dims, R, k, replay)


@pytest.mark.parametrize("dims,R,dtype", [((40, 30, 20, 10), 12, torch.float64), ((24, 24, 24, 24, 24), 32, torch.float32)])
def test_shared_sweep_replayed_from_a_graph(mt, oracle, dims, R, dtype):
    sb = 8 if dtype == torch.float64 else 4
    tol = 1e-12 if dtype == torch.float64 else 2e-5
    d = len(dims)
    nbytes = mt.mttkrp_dense_all_modes_shared_bytes(dims, R, sb)
    assert nbytes > 0
    X0, A0 = _fill(700, dims, R, dtype)
    X = X0.cuda()
    A = [a.cuda() for a in A0]
    M = [torch.zeros((dims[k], R), dtype=dtype, device="cuda") for k in range(d)]
    ws = torch.empty(nbytes, dtype=torch.uint8, device="cuda")
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        mt.mttkrp_dense_all_modes_shared(X, dims, A, M_out=M, workspace=ws)
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        mt.mttkrp_dense_all_modes_shared(X, dims, A, M_out=M, workspace=ws)
    for replay in range(4):
        Xn, An = _fill(800 + 10 * replay, dims, R, dtype)
        X.copy_(Xn.cuda())
        for a, an in zip(A, An):
            a.copy_(an.cuda())
        for m in M:
            m.fill_(float("nan"))
        ws.fill_(255)
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        got = [m.clone() for m in M]
        eager = mt.mttkrp_dense_all_modes_shared(X, dims, A, workspace=ws)
        torch.cuda.synchronize()
        Xv = inputs.as_ndarray_view(Xn, dims)
        for k in range(d):
            assert torch.equal(got[k], eager[k]), (dims, R, k, replay)
            ref = oracle.mttkrp(Xv, [a.numpy() for a in An], k)
            assert oracle.normwise_rel_err(got[k].cpu().numpy(), ref) <= tol, (dims, R, k, replay)

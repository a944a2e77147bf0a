"""GPU parity of the paper's own schedules (ELEM, SUB, TILE; Sec. III-B..III-D)
against the CPU oracle, through the C ABI of include/mttkrp_ablation.h.

All three must give the result of Eq. (elem) within the usual tolerance (1e-12
fp64, 1e-5 fp32, normwise); ELEM and TILE accumulate with atomics, so only the
value is compared, never the bits.  Tile widths cover 1 (one entry per tile:
the ELEM limit of Alg. "MTTKRP-TILE"), widths that do not divide the extents
(clipped edge tiles), and widths beyond every extent (the SUB limit).
"""
import numpy as np
import pytest

torch = pytest.importorskip("torch")

from paper_2510_14891_amd import inputs

pytestmark = pytest.mark.gpu

TOL = {torch.float64: 1e-12, torch.float32: 1e-5}


@pytest.fixture(scope="module")
def mt():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    from paper_2510_14891_amd import binding
    binding.lib()
    return binding


def make_problem(dims, R, dtype, seed):
    n = int(np.prod(dims))
    X = inputs.uniform(seed, n, -1.0, 1.0, dtype=dtype)
    A = [inputs.uniform(seed + 100 + m, (I, R), -1.0, 1.0, dtype=dtype) for m, I in enumerate(dims)]
    return X, A


CASES = [
    # dims, R
    ((7, 5, 3), 1),
    ((16, 9, 11), 3),
    ((33, 17, 6), 16),
    ((20, 12, 7, 5), 32),
    ((9, 4, 3, 5, 2), 33),
    ((12, 25), 8),
    ((5, 1, 6, 1), 100),
]


@pytest.mark.parametrize("dtype", [torch.float64, torch.float32])
@pytest.mark.parametrize("dims,R", CASES)
def test_schedules_match_the_oracle(mt, oracle, dims, R, dtype):
    X, A = make_problem(dims, R, dtype, seed=500 + len(dims) + R)
    Xd = X.cuda()
    Ad = [a.cuda() for a in A]
    Xn = inputs.as_ndarray_view(X, dims)
    An = [a.numpy() for a in A]
    for k in range(len(dims)):
        ref = oracle.mttkrp(Xn, An, k)
        runs = [("ELEM", mt.MTTKRP_SCHEDULE_ELEM, 0), ("SUB", mt.MTTKRP_SCHEDULE_SUB, 0)]
        runs += [("TILE w=%d" % w, mt.MTTKRP_SCHEDULE_TILE, w) for w in (1, 2, 3, 5, 1000)]
        for label, sched, w in runs:
            print("ablation %s dims=%s R=%d %s k=%d" % (label, dims, R, dtype, k), flush=True)
            M = torch.full((dims[k], R), float("nan"), dtype=dtype, device="cuda")   # must be overwritten
            fk = list(Ad)
            fk[k] = None                                                              # never read
            mt.mttkrp_ablation(sched, Xd, dims, fk, k, tile_width=w, M=M)
            torch.cuda.synchronize()
            err = oracle.normwise_rel_err(M.cpu().numpy(), ref)
            assert err <= TOL[dtype], (label, dims, R, k, err)


def test_schedules_agree_with_the_streaming_kernel(mt, oracle):
    """A shape of a few MiB with the heuristic's tile width for this GPU's cache
    figures: all four paths (three schedules + the streaming kernel) agree."""
    dims, R = (96, 40, 12, 21), 32
    X, A = make_problem(dims, R, torch.float64, seed=77)
    Xd = X.cuda()
    Ad = [a.cuda() for a in A]
    width, vol = mt.mttkrp_tile_volume(dims, 32768, 8, 64)
    assert vol == width ** 3 and width >= 1
    for k in range(4):
        ref = mt.mttkrp_dense(Xd, dims, Ad, k)
        for sched, w in ((mt.MTTKRP_SCHEDULE_ELEM, 0), (mt.MTTKRP_SCHEDULE_SUB, 0),
                         (mt.MTTKRP_SCHEDULE_TILE, width), (mt.MTTKRP_SCHEDULE_TILE, 6)):
            M = mt.mttkrp_ablation(sched, Xd, dims, Ad, k, tile_width=w)
            torch.cuda.synchronize()
            err = float(torch.linalg.vector_norm(M - ref) / torch.linalg.vector_norm(ref))
            assert err <= 1e-12, (sched, w, k, err)


def test_ablation_errors(mt):
    dims, R = (8, 8, 8), 4
    X, A = make_problem(dims, R, torch.float64, seed=5)
    Xd = X.cuda()
    Ad = [a.cuda() for a in A]
    M = torch.full((8, R), 3.0, dtype=torch.float64, device="cuda")
    with pytest.raises(mt.MttkrpError) as e:
        mt.mttkrp_ablation(mt.MTTKRP_SCHEDULE_TILE, Xd, dims, Ad, 0, tile_width=0, M=M)
    assert e.value.status == mt.MTTKRP_ERR_INVALID_ARG
    with pytest.raises(mt.MttkrpError):
        mt.mttkrp_ablation(7, Xd, dims, Ad, 0, tile_width=2, M=M)
    torch.cuda.synchronize()
    assert float(M.min()) == 3.0 and float(M.max()) == 3.0     # nothing was enqueued


def test_more_units_than_one_launch_holds(mt):
    """More entries (ELEM) and tiles (TILE, width 1) than the 2^24 workgroups a launch
    is given: the team threads stride over the rest.  Checked against the streaming
    kernel, whose full-size parity has its own tests."""
    dims, R = (512, 512, 300), 32
    n = int(np.prod(dims))
    X = inputs.uniform(901, n, -1.0, 1.0, dtype=torch.float32, device="cuda")
    A = [inputs.uniform(910 + m, (I, R), -1.0, 1.0, dtype=torch.float32).cuda() for m, I in enumerate(dims)]
    assert n // (128 // 32) > (1 << 24)
    for k in (0, 2):
        ref = mt.mttkrp_dense(X, dims, A, k)
        for sched, width in ((mt.MTTKRP_SCHEDULE_ELEM, 0), (mt.MTTKRP_SCHEDULE_TILE, 1)):
            print("ablation stride case sched=%d k=%d" % (sched, k), flush=True)
            M = mt.mttkrp_ablation(sched, X, dims, A, k, tile_width=width)
            torch.cuda.synchronize()
            err = float(torch.linalg.vector_norm(M.double() - ref.double()) / torch.linalg.vector_norm(ref.double()))
            assert err <= 2e-5, (sched, k, err)

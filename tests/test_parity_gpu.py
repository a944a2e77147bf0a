"""GPU parity: the HIP path (through the C ABI) against the CPU oracle.

Every case draws seeded inputs from ``paper_2510_14891_amd.inputs``, runs the
library on the GPU and the oracle on the host on the same buffers, and compares
with the normwise relative error ||M_gpu - M_orc||_F / ||M_orc||_F:
<= 1e-12 for fp64, <= 1e-5 for fp32.  Any re-association of the sum in
Eq. (elem) is a correct result, so parity is by norm, not by bits; what must be
bit-identical is a rerun of the same call (fixed-order combine, no atomics).
"""
import re

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
    binding.lib()   # raises if the HIP library was not built: no silent fallback
    yield binding
    for key in TUNE_KEYS:
        binding.mttkrp_tune_set(key, 0)


TUNE_KEYS = ("row_blocks", "target_items", "max_steps", "xcd_remap", "ws_percent",
             "max_col_blocks", "first_group", "deep", "waves_per_simd", "nt_loads", "fuse_bytes", "inner_splits", "contract_rows", "rows_col_blocks", "linear", "pair_rows", "fuse_rows", "lead_last")


def make_problem(dims, R, dtype, seed, dist=("uniform", -1.0, 1.0)):
    """Flat X (first index fastest) and factors, on the host."""
    n = int(np.prod(dims))
    if dist[0] == "uniform":
        X = inputs.uniform(seed, n, dist[1], dist[2], dtype=dtype)
        A = [inputs.uniform(seed + 100 + m, (I, R), dist[1], dist[2], dtype=dtype)
             for m, I in enumerate(dims)]
    else:
        X = inputs.normal(seed, n, dist[1], dist[2], dtype=dtype)
        A = [inputs.normal(seed + 100 + m, (I, R), dist[1], dist[2], dtype=dtype)
             for m, I in enumerate(dims)]
    return X, A


def gpu_mttkrp(mt, X, dims, A, k, **kw):
    Xd = X.cuda()
    Ad = [a.cuda() if a is not None else None for a in A]
    M = mt.mttkrp_dense(Xd, dims, Ad, k, **kw)
    torch.cuda.synchronize()
    return M.cpu().numpy()


def oracle_mttkrp(oracle, X, dims, A, k, rows=None):
    Xn = inputs.as_ndarray_view(X, dims)
    An = [a.numpy() if a is not None else None for a in A]
    return oracle.mttkrp(Xn, An, k, rows=rows)


def check_all_modes(mt, oracle, dims, R, dtype, seed, dist=("uniform", -1.0, 1.0)):
    X, A = make_problem(dims, R, dtype, seed, dist)
    worst = 0.0
    for k in range(len(dims)):
        print("case dims=%s R=%d %s k=%d seed=%d" % (dims, R, dtype, k, seed), flush=True)
        got = gpu_mttkrp(mt, X, dims, A, k)
        ref = oracle_mttkrp(oracle, X, dims, A, k)
        err = oracle.normwise_rel_err(got, ref)
        worst = max(worst, err)
        assert err <= TOL[dtype], (dims, R, k, err)
    return worst


# ---------------------------------------------------------------- small shapes, every mode
SMALL = [
    # dims, R  -- several 64-row tiles plus a ragged tail, odd inner sizes, tiny modes
    ((64, 64, 64), 16),          # benchmark configuration 1 exactly
    ((150, 37, 21), 16),
    ((70, 9, 5, 7), 5),
    ((33, 6, 4, 3, 5), 33),
    ((5, 300), 7),
    ((300, 5), 7),
    ((1, 7, 9), 3),
    ((17, 1, 1, 40), 4),
    ((16, 16, 16), 1),
    ((129, 13, 12), 17),
    ((48, 10, 6, 5), 64),
    ((40, 11, 9), 100),
    ((3, 2, 2, 2, 2, 2, 2, 3), 6),
    ((200, 3, 2), 2),
    ((2, 2), 1),
    ((15, 15, 15), 48),
]


@pytest.mark.parametrize("dims,R", SMALL)
def test_small_fp64(mt, oracle, dims, R):
    check_all_modes(mt, oracle, dims, R, torch.float64, seed=7)


@pytest.mark.parametrize("dims,R", SMALL)
def test_small_fp32(mt, oracle, dims, R):
    check_all_modes(mt, oracle, dims, R, torch.float32, seed=8)


def test_config1_recipe(mt, oracle):
    """Benchmark configuration 1 with its own recipe (U[0,1) data, seeds)."""
    w = inputs.WORKLOADS["c1_64x64x64_f64_R16"]
    X = inputs.make_tensor(w)
    A = inputs.make_factors(w)
    for k in range(3):
        got = gpu_mttkrp(mt, X, w.dims, A, k)
        ref = oracle_mttkrp(oracle, X, w.dims, A, k)
        assert oracle.normwise_rel_err(got, ref) <= 1e-12


# ---------------------------------------------------------------- scaled-down configurations 2-5
SCALED = [
    ("c2_1024x1024x512_f64_R32", (256, 128, 96), None),
    ("c3_192x192x192x192_f64_R16", (48, 40, 24, 20), None),
    ("c4_48x48x48x48x48_f32_R64", (48, 12, 10, 8, 6), None),
    ("c5_16384x2048x64_f64_R4", (2048, 256, 16), None),
    ("c5_16384x2048x64_f64_R8", (2048, 256, 16), None),
    ("c5_16384x2048x64_f64_R128", (1024, 64, 16), None),
    ("paperA_401x201x12x501_f64_R32", (101, 51, 12, 26), None),
    ("paperB_129x129x129x12x39_f64_R32", (33, 17, 9, 12, 5), None),
]


@pytest.mark.parametrize("name,dims,_", SCALED)
def test_scaled_configs(mt, oracle, name, dims, _):
    w = inputs.scaled(inputs.WORKLOADS[name], dims)
    X = inputs.make_tensor(w)
    A = inputs.make_factors(w)
    for k in range(w.ndim):
        print("case %s dims=%s k=%d" % (name, dims, k), flush=True)
        got = gpu_mttkrp(mt, X, w.dims, A, k)
        ref = oracle_mttkrp(oracle, X, w.dims, A, k)
        err = oracle.normwise_rel_err(got, ref)
        assert err <= TOL[w.torch_dtype], (name, k, err)


# ---------------------------------------------------------------- semantics of the boundary
def test_M_is_overwritten_and_Ak_never_read(mt, oracle):
    dims, R = (70, 20, 9), 12
    X, A = make_problem(dims, R, torch.float64, seed=21)
    for k in range(3):
        ref = oracle_mttkrp(oracle, X, dims, A, k)
        M = torch.full((dims[k], R), float("nan"), dtype=torch.float64, device="cuda")
        A_nan = list(A)
        A_nan[k] = torch.full_like(A[k], float("nan"))
        got = gpu_mttkrp(mt, X, dims, A_nan, k, M=M)
        assert oracle.normwise_rel_err(got, ref) <= 1e-12
        A_none = list(A)
        A_none[k] = None
        got2 = gpu_mttkrp(mt, X, dims, A_none, k)
        assert np.array_equal(got, got2)


def test_rerun_is_bit_identical_and_ws_variant_matches(mt, oracle):
    dims, R = (192, 40, 30), 32
    X, A = make_problem(dims, R, torch.float64, seed=22)
    for k in range(3):
        a = gpu_mttkrp(mt, X, dims, A, k)
        b = gpu_mttkrp(mt, X, dims, A, k)
        assert np.array_equal(a, b)
        nbytes = mt.mttkrp_dense_workspace_bytes(dims, R, k, 8)
        ws = torch.empty(max(nbytes, 256), dtype=torch.uint8, device="cuda")
        c = gpu_mttkrp(mt, X, dims, A, k, workspace=ws)
        assert np.array_equal(a, c)


def test_errors_enqueue_nothing(mt):
    import ctypes
    L = mt.lib()
    dims, R = (8, 6, 4), 3
    X, A = make_problem(dims, R, torch.float64, seed=23)
    Xd = X.cuda()
    Ad = [a.cuda() for a in A]
    M = torch.full((8, R), 5.0, dtype=torch.float64, device="cuda")
    d3 = (ctypes.c_int64 * 3)(*dims)
    ptrs = (ctypes.c_void_p * 3)(*[a.data_ptr() for a in Ad])
    bad_dims = (ctypes.c_int64 * 3)(8, 0, 4)
    no_f1 = (ctypes.c_void_p * 3)(Ad[0].data_ptr(), None, Ad[2].data_ptr())
    cases = [
        (3, d3, Xd.data_ptr(), ptrs, R, 3, M.data_ptr(), mt.MTTKRP_ERR_INVALID_ARG),
        (3, d3, Xd.data_ptr(), ptrs, R, -1, M.data_ptr(), mt.MTTKRP_ERR_INVALID_ARG),
        (3, d3, Xd.data_ptr(), ptrs, 0, 0, M.data_ptr(), mt.MTTKRP_ERR_INVALID_ARG),
        (3, bad_dims, Xd.data_ptr(), ptrs, R, 0, M.data_ptr(), mt.MTTKRP_ERR_INVALID_ARG),
        (1, d3, Xd.data_ptr(), ptrs, R, 0, M.data_ptr(), mt.MTTKRP_ERR_INVALID_ARG),
        (3, d3, None, ptrs, R, 0, M.data_ptr(), mt.MTTKRP_ERR_INVALID_ARG),
        (3, d3, Xd.data_ptr(), ptrs, R, 0, None, mt.MTTKRP_ERR_INVALID_ARG),
        (3, d3, Xd.data_ptr(), no_f1, R, 0, M.data_ptr(), mt.MTTKRP_ERR_INVALID_ARG),
    ]
    for (nd, dd, xp, fp, r, k, mp, want) in cases:
        rc = L.mttkrp_dense_f64(nd, dd, xp, fp, r, k, mp, None)
        assert rc == want, (nd, r, k, rc)
    d9 = (ctypes.c_int64 * 9)(*([2] * 9))
    p9 = (ctypes.c_void_p * 9)(*([Ad[0].data_ptr()] * 9))
    assert L.mttkrp_dense_f64(9, d9, Xd.data_ptr(), p9, R, 0, M.data_ptr(), None) \
        == mt.MTTKRP_ERR_UNSUPPORTED
    # caller-owned workspace too small / misaligned
    big = (512, 64, 32)
    nbytes = mt.mttkrp_dense_workspace_bytes(big, 16, 1, 8)
    assert nbytes > 0
    Xb, Ab = make_problem(big, 16, torch.float64, seed=24)
    Xbd = Xb.cuda()
    Abd = [a.cuda() for a in Ab]
    Mb = torch.full((64, 16), 5.0, dtype=torch.float64, device="cuda")
    with pytest.raises(mt.MttkrpError) as e:
        mt.mttkrp_dense(Xbd, big, Abd, 1, M=Mb,
                        workspace=torch.empty(256, dtype=torch.uint8, device="cuda"))
    assert e.value.status == mt.MTTKRP_ERR_WORKSPACE
    torch.cuda.synchronize()
    assert float(M.min()) == 5.0 and float(M.max()) == 5.0
    assert float(Mb.min()) == 5.0 and float(Mb.max()) == 5.0


# ---------------------------------------------------------------- schedule invariance
@pytest.mark.parametrize("dtype", [torch.float64, torch.float32])
def test_result_does_not_depend_on_the_decomposition(mt, oracle, dtype):
    """Tile sizes, split counts and block order are re-schedulings of one sum
    (Sec. III-D: N_T only changes the schedule), so every setting must agree
    with the oracle within the tolerance."""
    dims, R = (200, 36, 14, 5), 24
    X, A = make_problem(dims, R, dtype, seed=31)
    refs = [oracle_mttkrp(oracle, X, dims, A, k) for k in range(4)]
    settings = [
        {"row_blocks": 1}, {"row_blocks": 2}, {"row_blocks": 3}, {"row_blocks": 4},
        {"target_items": 1}, {"target_items": 64}, {"target_items": 100000},
        {"max_steps": 8}, {"xcd_remap": 1}, {"ws_percent": 100, "target_items": 50000},
        {"max_col_blocks": 1}, {"first_group": 1}, {"first_group": 4},
        {"first_group": 1, "ws_percent": 100, "target_items": 50000},
        {"deep": 1}, {"deep": 2}, {"deep": 1, "max_steps": 8}, {"nt_loads": 1}, {"waves_per_simd": 2},
        {"contract_rows": 1}, {"contract_rows": 1, "max_steps": 3}, {"contract_rows": 1, "max_col_blocks": 1},
        {"contract_rows": 2},
        {"fuse_bytes": 1}, {"inner_splits": 1}, {"inner_splits": 5}, {"fuse_bytes": 1 << 30}, {"fuse_bytes": 1 << 30, "target_items": 64},
        {"linear": 1}, {"linear": 1, "target_items": 777}, {"linear": 1, "first_group": 1, "target_items": 100000},
        {"linear": 1, "deep": 2, "max_steps": 5}, {"linear": 2, "first_group": 1},
        {"pair_rows": 1}, {"pair_rows": 2}, {"pair_rows": 1, "row_blocks": 2, "target_items": 50000},
        {"fuse_rows": 1}, {"fuse_rows": 2}, {"fuse_rows": 1, "fuse_bytes": 1 << 30, "max_steps": 6},
        {"lead_last": 1}, {"lead_last": 2}, {"lead_last": 1, "max_steps": 2, "rows_col_blocks": 1},
    ]
    try:
        for st in settings:
            for key, val in st.items():
                mt.mttkrp_tune_set(key, val)
            for k in range(4):
                print("setting %s k=%d %s" % (st, k, mt.mttkrp_plan_describe(
                    dims, R, k, 8 if dtype == torch.float64 else 4)), flush=True)
                got = gpu_mttkrp(mt, X, dims, A, k)
                assert oracle.normwise_rel_err(got, refs[k]) <= TOL[dtype], (st, k)
            for key in st:
                mt.mttkrp_tune_set(key, 0)
    finally:
        for key in TUNE_KEYS:
            mt.mttkrp_tune_set(key, 0)


def test_non_default_stream(mt, oracle):
    dims, R = (130, 50, 20), 16
    X, A = make_problem(dims, R, torch.float64, seed=41)
    ref = oracle_mttkrp(oracle, X, dims, A, 1)
    st = torch.cuda.Stream()
    Xd = X.cuda()
    Ad = [a.cuda() for a in A]
    torch.cuda.synchronize()
    with torch.cuda.stream(st):
        M = mt.mttkrp_dense(Xd, dims, Ad, 1)
    st.synchronize()
    assert oracle.normwise_rel_err(M.cpu().numpy(), ref) <= 1e-12


def test_calls_in_flight_on_several_streams(mt, oracle):
    """Core calls (library-owned workspace) enqueued back to back on different streams without
    any synchronisation between them: every stream has partial sums of its own, so the results
    of problems that run concurrently all match the oracle.  Ten streams, more than the
    library keeps workspaces for, so workspaces also change hands."""
    probs = []
    # first-mode problems with many partial slots, long enough to overlap on the GPU
    for i in range(10):
        dims, R = (96 + 16 * (i % 3), 300 + 7 * i, 257 - 3 * i), 32
        X, A = make_problem(dims, R, torch.float64, seed=700 + i)
        k = i % 3
        probs.append((dims, k, X.cuda(), [a.cuda() for a in A], oracle_mttkrp(oracle, X, dims, A, k)))
    streams = [torch.cuda.Stream() for _ in probs]
    torch.cuda.synchronize()
    outs = [None] * len(probs)
    for rep in range(3):
        for i, (dims, k, Xd, Ad, _) in enumerate(probs):
            with torch.cuda.stream(streams[i]):
                outs[i] = mt.mttkrp_dense(Xd, dims, Ad, k)
    torch.cuda.synchronize()
    for i, (dims, k, _, _, ref) in enumerate(probs):
        err = oracle.normwise_rel_err(outs[i].cpu().numpy(), ref)
        assert err <= 1e-12, (i, dims, k, err)


# ---------------------------------------------------------------- extended calls and high rank
@pytest.mark.parametrize("dtype", [torch.float64, torch.float32])
def test_ex_lambda_and_beta(mt, oracle, dtype):
    """M = beta * M + X_(k) Z diag(lambda) (Eq. (krp) with its weight vector)."""
    dims, R = (130, 21, 10, 6), 20
    X, A = make_problem(dims, R, dtype, seed=51)
    lam = inputs.uniform(52, R, 0.5, 2.0, dtype=dtype)
    Xd, Ad, lamd = X.cuda(), [a.cuda() for a in A], lam.cuda()
    for k in range(4):
        M0 = inputs.uniform(60 + k, (dims[k], R), -1.0, 1.0, dtype=dtype)
        ref_lam = oracle_mttkrp(oracle, X, dims, A, k)   # lambda = 1
        ref = oracle.mttkrp(inputs.as_ndarray_view(X, dims), [a.numpy() for a in A], k,
                            lam=lam.numpy())
        # lambda only
        got = mt.mttkrp_dense(Xd, dims, Ad, k, lam=lamd).cpu().numpy()
        assert oracle.normwise_rel_err(got, ref) <= TOL[dtype]
        # lambda = 1, beta = 0 through the extended call: bit-identical to the core call
        plain = mt.mttkrp_dense(Xd, dims, Ad, k).cpu().numpy()
        via_ex = mt.mttkrp_dense(Xd, dims, Ad, k, beta=0.0).cpu().numpy()
        assert np.array_equal(plain, via_ex)
        assert oracle.normwise_rel_err(plain, ref_lam) <= TOL[dtype]
        # accumulation, with a caller-owned workspace
        beta = -0.75
        Md = M0.cuda()
        ws = torch.empty(mt.mttkrp_dense_ex_workspace_bytes(dims, R, k, X.element_size()),
                         dtype=torch.uint8, device="cuda")
        mt.mttkrp_dense(Xd, dims, Ad, k, M=Md, lam=lamd, beta=beta, workspace=ws)
        want = beta * M0.numpy().astype(np.float64) + ref.astype(np.float64)
        assert oracle.normwise_rel_err(Md.cpu().numpy(), want) <= TOL[dtype]
        # beta = 0 never reads M: NaNs in M do not leak
        Mn = torch.full((dims[k], R), float("nan"), dtype=dtype, device="cuda")
        mt.mttkrp_dense(Xd, dims, Ad, k, M=Mn, lam=lamd, beta=0.0)
        assert oracle.normwise_rel_err(Mn.cpu().numpy(), ref) <= TOL[dtype]


@pytest.mark.parametrize("R", [500, 1000, 2000])
def test_high_rank(mt, oracle, R):
    """The paper's flagship regime (Sec. IV: R = 500 ... 2000): many 64-column chunks."""
    dims = (70, 20, 12, 9)
    X, A = make_problem(dims, R, torch.float64, seed=71)
    for k in range(4):
        got = gpu_mttkrp(mt, X, dims, A, k)
        ref = oracle_mttkrp(oracle, X, dims, A, k)
        assert oracle.normwise_rel_err(got, ref) <= 1e-12
    # the extra memory stays in the O(R sum I_n) class, far below the Khatri-Rao matrix
    for k in range(4):
        ws = mt.mttkrp_dense_workspace_bytes((401, 201, 12, 501), 2000, k, 8)
        krp = (401 * 201 * 12 * 501 // (401, 201, 12, 501)[k]) * 2000 * 8
        assert ws <= 128 << 20 and ws < krp / 100


def test_calibration_probes_return_plausible_rates(mt):
    """The two measured-ceiling probes of include/mttkrp_calibrate.h run, validate their
    arguments and report rates of the right order for this class of GPU."""
    buf = torch.zeros(1 << 27, dtype=torch.float64, device="cuda")      # 1 GiB
    gbps = mt.mttkrp_calibrate_stream(buf, launches=5)
    assert 1000.0 < gbps < 8000.0, gbps
    for nbytes, lo, hi in ((8, 10.0, 78.6 * 1.02), (4, 20.0, 157.3 * 1.02)):
        tf = mt.mttkrp_calibrate_mfma(nbytes, 20.0, launches=5)
        assert lo < tf < hi, (nbytes, tf)
    import ctypes
    L = mt.lib()
    ms = ctypes.c_float(0)
    fl = ctypes.c_double(0)
    assert L.mttkrp_calibrate_stream(buf.data_ptr() + 8, 1024, 1, ctypes.byref(ms), None) == mt.MTTKRP_ERR_INVALID_ARG
    assert L.mttkrp_calibrate_stream(buf.data_ptr(), 1000, 1, ctypes.byref(ms), None) == mt.MTTKRP_ERR_INVALID_ARG
    assert L.mttkrp_calibrate_mfma(2, 1.0, 1, ctypes.byref(ms), ctypes.byref(fl), None) == mt.MTTKRP_ERR_INVALID_ARG
    assert L.mttkrp_calibrate_mfma(8, 1.0, 0, ctypes.byref(ms), ctypes.byref(fl), None) == mt.MTTKRP_ERR_INVALID_ARG


@pytest.mark.parametrize("dtype", [torch.float64, torch.float32])
def test_leading_dimensions(mt, oracle, dtype):
    """Factors and M as column blocks of wider row-major arrays (the *_ld calls): the
    padding is NaN in the factors and must never be read, and the padding of M must
    stay untouched.  Shapes cover direct writes (one slot) and the combine kernel."""
    for dims, R, pads in (((70, 9, 6, 5), 24, (3, 0, 8, 1)), ((200, 36, 14), 7, (1, 5, 2)), ((33, 20), 33, (2, 7)),
                          ((16, 4, 3), 16, (4, 4, 4))):
        X, A = make_problem(dims, R, dtype, seed=61 + len(dims))
        Xd = X.cuda()
        wide = []
        for m, a in enumerate(A):
            buf = torch.full((dims[m], R + pads[m]), float("nan"), dtype=dtype, device="cuda")
            buf[:, :R] = a.cuda()
            wide.append(buf)
        lam = inputs.uniform(99, R, 0.5, 1.5, dtype=dtype)
        Xn = inputs.as_ndarray_view(X, dims)
        An = [a.numpy() for a in A]
        for k in range(len(dims)):
            print("ld case dims=%s R=%d %s k=%d" % (dims, R, dtype, k), flush=True)
            ref = oracle.mttkrp(Xn, An, k, lam=lam.numpy())
            Mw = torch.full((dims[k], R + 5), 7.0, dtype=dtype, device="cuda")
            mt.mttkrp_dense_ld(Xd, dims, [w[:, :R] for w in wide], k, Mw[:, :R], R, lam=lam.cuda())
            torch.cuda.synchronize()
            got = Mw[:, :R].cpu().numpy()
            assert oracle.normwise_rel_err(got, ref) <= TOL[dtype], (dims, R, k)
            assert bool((Mw[:, R:] == 7.0).all())
            # accumulation through the padded M
            Mw[:, :R] = 1.0
            mt.mttkrp_dense_ld(Xd, dims, [w[:, :R] for w in wide], k, Mw[:, :R], R, beta=2.0)
            torch.cuda.synchronize()
            ref2 = oracle.mttkrp(Xn, An, k) + 2.0
            assert oracle.normwise_rel_err(Mw[:, :R].cpu().numpy(), ref2) <= TOL[dtype], (dims, R, k)
            assert bool((Mw[:, R:] == 7.0).all())
    L = mt.lib()
    import ctypes
    d3 = (ctypes.c_int64 * 3)(4, 4, 4)
    bad = (ctypes.c_int64 * 3)(3, 4, 4)
    one = ctypes.c_void_p(16)
    ptrs = (ctypes.c_void_p * 3)(16, 16, 16)
    assert L.mttkrp_dense_f64_ld(3, d3, one, ptrs, bad, 4, 1, None, 0.0, one, 4, None, 0, None) == mt.MTTKRP_ERR_INVALID_ARG
    assert L.mttkrp_dense_f64_ld(3, d3, one, ptrs, d3, 4, 1, None, 0.0, one, 3, None, 0, None) == mt.MTTKRP_ERR_INVALID_ARG
    assert L.mttkrp_dense_f64_ld(3, d3, one, ptrs, None, 4, 1, None, 0.0, one, 4, None, 0, None) == mt.MTTKRP_ERR_INVALID_ARG


@pytest.mark.parametrize("dtype", [torch.float64, torch.float32])
def test_row_contraction_schedule(mt, oracle, dtype):
    """The second schedule (MFMA contraction over mode 0, weights of the column space applied
    in the epilogue) computes the same sum of Eq. (elem): forced on for shapes with one and
    with two column pieces (modes below and above k), ragged row counts, column counts and R
    beyond one tile, many row splits; plain call, leading dimensions, lambda and beta."""
    sb = 8 if dtype == torch.float64 else 4
    shapes = [((300, 7, 9), 16), ((1000, 5, 4, 3), 5), ((130, 3, 2, 2), 33), ((64, 64, 64), 16), ((17, 40, 6), 70),
              ((5, 300), 7), ((2048, 9, 11), 100), ((520, 3, 50), 24), ((777, 2, 3, 2, 5), 40)]
    try:
        for tune in ({"contract_rows": 1}, {"contract_rows": 1, "max_steps": 2}, {"contract_rows": 1, "rows_col_blocks": 1}):
            for key, val in tune.items():
                mt.mttkrp_tune_set(key, val)
            for dims, R in shapes:
                X, A = make_problem(dims, R, dtype, seed=71 + len(dims))
                Xn = inputs.as_ndarray_view(X, dims)
                An = [a.numpy() for a in A]
                Xd = X.cuda()
                Ad = [a.cuda() for a in A]
                lam = inputs.uniform(98, R, 0.5, 1.5, dtype=dtype)
                for k in range(1, len(dims)):
                    desc = mt.mttkrp_plan_describe(dims, R, k, sb)
                    print("rows schedule %s dims=%s R=%d %s k=%d %s" % (tune, dims, R, dtype, k, desc), flush=True)
                    assert "shape=rows" in desc, desc
                    ref = oracle.mttkrp(Xn, An, k)
                    got = mt.mttkrp_dense(Xd, dims, Ad, k)
                    torch.cuda.synchronize()
                    assert oracle.normwise_rel_err(got.cpu().numpy(), ref) <= TOL[dtype], (dims, R, k)
                    # leading dimensions, lambda, accumulation
                    wide = []
                    for m, a in enumerate(A):
                        buf = torch.full((dims[m], R + 1 + m), float("nan"), dtype=dtype, device="cuda")
                        buf[:, :R] = Ad[m]
                        wide.append(buf)
                    Mw = torch.full((dims[k], R + 3), 1.0, dtype=dtype, device="cuda")
                    mt.mttkrp_dense_ld(Xd, dims, [w[:, :R] for w in wide], k, Mw[:, :R], R, lam=lam.cuda(), beta=0.5)
                    torch.cuda.synchronize()
                    ref2 = oracle.mttkrp(Xn, An, k, lam=lam.numpy()) + 0.5
                    assert oracle.normwise_rel_err(Mw[:, :R].cpu().numpy(), ref2) <= TOL[dtype], (dims, R, k)
                    assert bool((Mw[:, R:] == 1.0).all())
            for key in tune:
                mt.mttkrp_tune_set(key, 0)
        # chosen by the planner itself: few column entries, long mode 0 (2053 rows: a ragged last step)
        # (k = 1: 12 column entries, either type; k = 2: 40 entries, at R = 30 in fp64 only)
        dims, R = (2053, 40, 12), 30
        X, A = make_problem(dims, R, dtype, seed=77)
        for k in (1, 2):
            desc = mt.mttkrp_plan_describe(dims, R, k, sb)
            assert ("shape=rows" in desc) == (k == 1 or dtype == torch.float64), desc
            got = gpu_mttkrp(mt, X, dims, A, k)
            assert oracle.normwise_rel_err(got, oracle_mttkrp(oracle, X, dims, A, k)) <= TOL[dtype], (dims, k)
        mt.mttkrp_tune_set("contract_rows", 2)
        assert "shape=rows" not in mt.mttkrp_plan_describe(dims, R, 1, sb)
    finally:
        for key in TUNE_KEYS:
            mt.mttkrp_tune_set(key, 0)


@pytest.mark.parametrize("dtype", [torch.float64, torch.float32])
def test_fused_row_modes(mt, oracle, dtype):
    """Modes 0 and 1 treated as one row mode (their factors' row-wise product stands in for
    A_0): shapes for which the planner reports it, alone and together with a fused column pair,
    through the plain call and through the call with leading dimensions (NaN padding)."""
    cases = (((19, 5, 9, 300), 20, 2), ((19, 5, 40, 3, 50), 7, 2), ((45, 45, 24, 7, 6), 32, 2), ((33, 6, 4, 3, 5), 33, 2))
    for dims, R, k in cases:
        desc = mt.mttkrp_plan_describe(dims, R, k, 8 if dtype == torch.float64 else 4)
        print("fused rows dims=%s R=%d %s k=%d %s" % (dims, R, dtype, k, desc), flush=True)
        assert "fused_rows=1" in desc, desc
        X, A = make_problem(dims, R, dtype, seed=83 + len(dims))
        ref = oracle_mttkrp(oracle, X, dims, A, k)
        got = gpu_mttkrp(mt, X, dims, A, k)
        assert oracle.normwise_rel_err(got, ref) <= TOL[dtype], (dims, R, k)
        wide = []
        for m, a in enumerate(A):
            buf = torch.full((dims[m], R + 3 + m), float("nan"), dtype=dtype, device="cuda")
            buf[:, :R] = a.cuda()
            wide.append(buf)
        Mw = torch.full((dims[k], R + 2), 7.0, dtype=dtype, device="cuda")
        mt.mttkrp_dense_ld(X.cuda(), dims, [w[:, :R] for w in wide], k, Mw[:, :R], R)
        torch.cuda.synchronize()
        assert oracle.normwise_rel_err(Mw[:, :R].cpu().numpy(), ref) <= TOL[dtype], (dims, R, k)
        assert bool((Mw[:, R:] == 7.0).all())
    # never with the fusing switched off
    mt.mttkrp_tune_set("fuse_bytes", 1)
    try:
        assert "fused_rows=0" in mt.mttkrp_plan_describe((19, 5, 9, 300), 20, 2, 8)
    finally:
        mt.mttkrp_tune_set("fuse_bytes", 0)


@pytest.mark.parametrize("dtype", [torch.float64, torch.float32])
def test_paired_rows_for_the_first_two_modes(mt, oracle, dtype):
    """k = 1 and k = 0 with the pairs (i_0, i_1) taken as the rows and each tile's rows summed per
    output row (k = 0 with more than 32 rows: the weighted tiles stored whole and summed by the
    combine kernel): shapes the planner picks it for (I_0 not near a
    multiple of the row tiles, or so short that a wavefront would hold one or two row blocks; I_0
    from 1 to 401, so that a tile meets from one to 64 output rows), and forced on for extents
    where the ranges of i_0 begin on tile boundaries (64, 128), just off them (65, 127), with few
    and many column entries (one split and many), tiles of 16 to 64 rows, ragged R, one and
    several chunks of output columns; plain call, leading dimensions with NaN padding, lambda and
    beta, and twice in a row in one workspace (unwritten slots are cleared at every call)."""
    sb = 8 if dtype == torch.float64 else 4
    picked = (((401, 21, 12, 11), 32, 1), ((129, 9, 40, 7), 10, 1), ((100, 5, 300), 7, 1), ((70, 3, 9, 5, 4), 33, 1),
              ((80, 6, 30, 7), 12, 1), ((400, 5, 9, 11), 20, 1),
              ((3, 50, 40, 7), 16, 1), ((10, 33, 20, 9), 40, 1), ((20, 30, 40, 5), 8, 1), ((2, 100, 300), 5, 1),
              ((31, 7, 50), 17, 1), ((1, 40, 90), 6, 1), ((7, 9, 11, 13, 5), 70, 1), ((17, 200, 33), 24, 1),
              ((3, 50, 40, 7), 16, 0), ((10, 33, 20, 9), 40, 0), ((20, 30, 40, 5), 8, 0), ((2, 100, 300), 5, 0),
              ((31, 7, 50), 17, 0), ((1, 40, 90), 6, 0), ((7, 9, 11, 13, 5), 70, 0), ((17, 200, 33), 24, 0),
              ((32, 3, 500), 33, 0), ((5, 2000, 9), 3, 0))
    forced = (((64, 5, 50), 16, 1), ((128, 3, 7, 9), 5, 1), ((65, 4, 33), 70, 1), ((127, 2, 100), 20, 1), ((192, 7, 40), 8, 1),
              ((80, 6, 3), 3, 1), ((1000, 3, 40), 9, 1), ((16, 16, 50), 16, 0), ((16, 16, 50), 16, 1), ((32, 8, 70), 20, 0),
              # first mode of more than 32 entries: the weighted tiles are stored whole
              ((40, 30, 20, 9), 16, 0), ((129, 9, 40, 7), 10, 0), ((50, 7, 300), 33, 0), ((100, 5, 9, 11), 70, 0),
              ((64, 5, 50), 16, 0), ((401, 21, 12, 11), 32, 0), ((33, 2, 500), 5, 0))
    try:
        for tune in ({}, {"pair_rows": 1}, {"pair_rows": 1, "row_blocks": 1}, {"pair_rows": 1, "row_blocks": 3, "max_steps": 4},
                     {"pair_rows": 1, "max_col_blocks": 1}):
            for key, val in tune.items():
                mt.mttkrp_tune_set(key, val)
            for dims, R, k in (picked if not tune else picked + forced):
                desc = mt.mttkrp_plan_describe(dims, R, k, sb)
                print("paired rows %s dims=%s R=%d k=%d %s %s" % (tune, dims, R, k, dtype, desc), flush=True)
                assert ("paired_rows=1" if k == 1 else ("paired_rows=2" if dims[0] <= 32 else "paired_rows=3")) in desc, desc
                X, A = make_problem(dims, R, dtype, seed=91 + len(dims))
                Xn = inputs.as_ndarray_view(X, dims)
                An = [a.numpy() for a in A]
                Xd = X.cuda()
                Ad = [a.cuda() for a in A]
                ref = oracle.mttkrp(Xn, An, k)
                for _ in range(2):
                    got = mt.mttkrp_dense(Xd, dims, [None if m == k else a for m, a in enumerate(Ad)], k)
                    torch.cuda.synchronize()
                    assert oracle.normwise_rel_err(got.cpu().numpy(), ref) <= TOL[dtype], (dims, R, k, tune)
                lam = inputs.uniform(99, R, 0.5, 1.5, dtype=dtype)
                wide = []
                for m, a in enumerate(A):
                    buf = torch.full((dims[m], R + 1 + m), float("nan"), dtype=dtype, device="cuda")
                    buf[:, :R] = Ad[m]
                    wide.append(buf)
                Mw = torch.full((dims[k], R + 3), 1.0, dtype=dtype, device="cuda")
                mt.mttkrp_dense_ld(Xd, dims, [w[:, :R] for w in wide], k, Mw[:, :R], R, lam=lam.cuda(), beta=0.5)
                torch.cuda.synchronize()
                ref2 = oracle.mttkrp(Xn, An, k, lam=lam.numpy()) + 0.5
                assert oracle.normwise_rel_err(Mw[:, :R].cpu().numpy(), ref2) <= TOL[dtype], (dims, R, k, tune)
                assert bool((Mw[:, R:] == 1.0).all())
            for key in tune:
                mt.mttkrp_tune_set(key, 0)
        # not for other modes, not for a first mode of 64-row tiles that are 89 % full, not for
        # matrices, not where I_0 fills its tiles, not when switched off
        assert "paired_rows=0" in mt.mttkrp_plan_describe((401, 21, 12, 11), 32, 2, sb)
        assert "paired_rows=0" in mt.mttkrp_plan_describe((192, 21, 12, 11), 32, 1, sb)
        assert "paired_rows=0" in mt.mttkrp_plan_describe((401, 201, 12, 501), 32, 0, sb)
        assert "paired_rows=0" in mt.mttkrp_plan_describe((20, 500), 8, 0, sb)
        assert "paired_rows=0" in mt.mttkrp_plan_describe((20, 500), 8, 1, sb)
        mt.mttkrp_tune_set("pair_rows", 2)
        assert "paired_rows=0" in mt.mttkrp_plan_describe((401, 21, 12, 11), 32, 1, sb)
        assert "paired_rows=0" in mt.mttkrp_plan_describe((3, 50, 40, 7), 16, 0, sb)
    finally:
        for key in TUNE_KEYS:
            mt.mttkrp_tune_set(key, 0)


@pytest.mark.parametrize("dtype", [torch.float64, torch.float32])
def test_last_mode_as_contraction_over_all_other_modes(mt, oracle, dtype):
    """The last mode when all other modes together are short: M = X^T K with K the Khatri-Rao
    product of the other factors, formed in the workspace by a chain of pairwise products (none
    for a matrix, one for three modes, three for five).  Shapes the planner picks it for and
    shapes it is forced on (row splits with partial sums, one and several column chunks of R,
    ragged extents); plain call without the k-th factor, leading dimensions with NaN padding,
    lambda and beta with and without row splits."""
    sb = 8 if dtype == torch.float64 else 4
    picked = (((10, 13, 700), 70), ((20, 500), 8), ((2, 3, 40000), 5), ((7, 5, 3, 150000), 12))
    forced = (((20, 20, 5000), 8), ((64, 64, 300), 16), ((100, 30, 400), 24), ((17, 3, 2, 2, 2, 90), 33), ((300, 5, 20), 130),
              ((20, 20, 5000), 32), ((3, 4, 5, 6, 700), 10), ((5, 7, 9, 1000), 16))
    try:
        for tune in ({}, {"lead_last": 1}, {"lead_last": 1, "max_steps": 2}, {"lead_last": 1, "max_col_blocks": 1, "target_items": 50000}):
            for key, val in tune.items():
                mt.mttkrp_tune_set(key, val)
            for dims, R in (picked if not tune else picked + forced):
                k = len(dims) - 1
                desc = mt.mttkrp_plan_describe(dims, R, k, sb)
                print("last mode %s dims=%s R=%d %s %s" % (tune, dims, R, dtype, desc), flush=True)
                assert "shape=leading" in desc, desc
                X, A = make_problem(dims, R, dtype, seed=57 + len(dims))
                Xn = inputs.as_ndarray_view(X, dims)
                An = [a.numpy() for a in A]
                Xd = X.cuda()
                Ad = [a.cuda() for a in A]
                ref = oracle.mttkrp(Xn, An, k)
                got = mt.mttkrp_dense(Xd, dims, Ad[:k] + [None], k)
                torch.cuda.synchronize()
                assert oracle.normwise_rel_err(got.cpu().numpy(), ref) <= TOL[dtype], (dims, R, tune)
                ws = torch.empty(max(1, mt.mttkrp_dense_workspace_bytes(dims, R, k, sb)), dtype=torch.uint8, device="cuda")
                ws.fill_(255)
                got = mt.mttkrp_dense(Xd, dims, Ad, k, workspace=ws)
                torch.cuda.synchronize()
                assert oracle.normwise_rel_err(got.cpu().numpy(), ref) <= TOL[dtype], (dims, R, tune)
                lam = inputs.uniform(96, R, 0.5, 1.5, dtype=dtype)
                wide = []
                for m, a in enumerate(A):
                    buf = torch.full((dims[m], R + 1 + m), float("nan"), dtype=dtype, device="cuda")
                    buf[:, :R] = Ad[m]
                    wide.append(buf)
                Mw = torch.full((dims[k], R + 3), 1.0, dtype=dtype, device="cuda")
                mt.mttkrp_dense_ld(Xd, dims, [w[:, :R] for w in wide], k, Mw[:, :R], R, lam=lam.cuda(), beta=0.5)
                torch.cuda.synchronize()
                ref2 = oracle.mttkrp(Xn, An, k, lam=lam.numpy()) + 0.5
                assert oracle.normwise_rel_err(Mw[:, :R].cpu().numpy(), ref2) <= TOL[dtype], (dims, R, tune)
                assert bool((Mw[:, R:] == 1.0).all())
            for key in tune:
                mt.mttkrp_tune_set(key, 0)
        # not for other modes, not where mode 0 fills its row tiles, not with many entries in the
        # other modes, not when switched off
        assert "shape=leading" not in mt.mttkrp_plan_describe((7, 5, 3, 150000), 12, 1, sb)
        assert "shape=leading" not in mt.mttkrp_plan_describe((64, 64, 5000), 8, 2, sb)
        assert "shape=leading" not in mt.mttkrp_plan_describe((20, 2000, 5000), 64, 2, sb)
        mt.mttkrp_tune_set("lead_last", 2)
        assert "shape=leading" not in mt.mttkrp_plan_describe((7, 5, 3, 150000), 12, 3, sb)
    finally:
        for key in TUNE_KEYS:
            mt.mttkrp_tune_set(key, 0)


def test_seeded_random_shapes(mt, oracle):
    """Eighty seeded random problems (2 to 6 modes, extents 1 to 70, R 1 to 80, both data
    types, every mode): a sweep over the planner's decisions (tile shapes, fused modes,
    kernel builds, splits) that no hand-picked list covers."""
    u = inputs.uniform(20240601, 80 * 16).numpy()
    t = 0
    for case in range(80):
        d = 2 + int(u[t] * 5); t += 1
        big = int(u[t] * d); t += 1                       # one mode may be larger
        dims = []
        for m in range(d):
            hi = 70 if m == big else (24 if d <= 4 else 9)
            dims.append(1 + int(u[t] * hi)); t += 1
        R = 1 + int(u[t] * 80); t += 1
        dtype = torch.float64 if u[t] < 0.6 else torch.float32; t += 1
        t = (t + 15) // 16 * 16
        if int(np.prod(dims)) > 3_000_000:
            continue
        X, A = make_problem(tuple(dims), R, dtype, seed=7000 + case)
        Xd = X.cuda()
        Ad = [a.cuda() for a in A]
        Xn = inputs.as_ndarray_view(X, dims)
        An = [a.numpy() for a in A]
        for k in range(d):
            print("random case %d dims=%s R=%d %s k=%d %s" % (case, dims, R, dtype, k, mt.mttkrp_plan_describe(
                dims, R, k, 8 if dtype == torch.float64 else 4)), flush=True)
            M = mt.mttkrp_dense(Xd, dims, Ad, k)
            torch.cuda.synchronize()
            ref = oracle.mttkrp(Xn, An, k)
            err = oracle.normwise_rel_err(M.cpu().numpy(), ref)
            assert err <= TOL[dtype], (case, dims, R, k, err)


def test_seeded_random_shapes_long_first_mode(mt, oracle):
    """A hundred and fifty seeded random problems with a long or ragged mode 0 and short other
    modes, under seeded planner settings: the shapes that reach the fused row mode, the second
    schedule (one and two column pieces, many row splits, ragged last steps) and their
    combinations with the tuning keys."""
    I0s = (1, 5, 16, 17, 63, 129, 257, 300, 520, 1000, 2053, 4100)
    Is = (1, 2, 3, 4, 5, 7, 9, 12, 16, 17, 33, 40, 64)
    Rs = (1, 3, 8, 16, 17, 32, 33, 49, 50, 64, 70, 100)
    tunes = ({}, {}, {"contract_rows": 1}, {"contract_rows": 1, "max_steps": 2}, {"contract_rows": 2},
             {"contract_rows": 1, "target_items": 100000}, {"fuse_bytes": 1 << 30}, {"target_items": 50000},
             {"contract_rows": 1, "rows_col_blocks": 1}, {"inner_splits": 3}, {"max_steps": 3},
             {"linear": 1}, {"linear": 1, "target_items": 30000}, {"linear": 1, "first_group": 1, "max_steps": 7})
    u = inputs.uniform(20240607, 150 * 16).numpy()
    try:
        for case in range(150):
            t = case * 16
            d = (2, 3, 3, 3, 4, 4, 5, 6)[int(u[t] * 8)]
            dims = [I0s[int(u[t + 1] * len(I0s))]] + [Is[int(u[t + 2 + m] * len(Is))] for m in range(d - 1)]
            while int(np.prod(dims)) > 400_000:
                i = int(np.argmax(dims))
                dims[i] = max(1, dims[i] // 2)
            R = Rs[int(u[t + 8] * len(Rs))]
            dtype = torch.float64 if u[t + 9] < 0.6 else torch.float32
            tune = tunes[int(u[t + 10] * len(tunes))]
            X, A = make_problem(tuple(dims), R, dtype, seed=8000 + case)
            Xd = X.cuda()
            Ad = [a.cuda() for a in A]
            Xn = inputs.as_ndarray_view(X, dims)
            An = [a.numpy() for a in A]
            for key, val in tune.items():
                mt.mttkrp_tune_set(key, val)
            for k in range(d):
                print("random long case %d dims=%s R=%d %s k=%d tune=%s %s" % (case, dims, R, dtype, k, tune,
                      mt.mttkrp_plan_describe(dims, R, k, 8 if dtype == torch.float64 else 4)), flush=True)
                M = mt.mttkrp_dense(Xd, dims, Ad, k)
                torch.cuda.synchronize()
                err = oracle.normwise_rel_err(M.cpu().numpy(), oracle.mttkrp(Xn, An, k))
                assert err <= TOL[dtype], (case, dims, R, k, tune, err)
            for key in tune:
                mt.mttkrp_tune_set(key, 0)
    finally:
        for key in TUNE_KEYS:
            mt.mttkrp_tune_set(key, 0)


def test_seeded_random_shapes_short_leading_modes(mt, oracle):
    """Two hundred seeded random problems with a short or ragged first mode (1 to 129 entries) and
    other modes of up to 300, under planner settings that force or forbid the routes made for them:
    the pairs (i_0, i_1) as rows for the first two modes (summed per output row, or stored whole),
    fused rows for later modes, the last mode as a contraction over all other modes, many inner
    splits, and the folded combine.  The tolerance is the one of the other tests, widened only for
    ill-conditioned outputs (8 u c with c = ||MTTKRP of absolute values|| / ||MTTKRP||, the
    forward-error bound of any summation order)."""
    rng = np.random.default_rng(20240623)
    I0s = (1, 2, 3, 5, 7, 10, 16, 17, 20, 31, 32, 33, 40, 50, 63, 64, 65, 100, 129)
    Is = (1, 2, 3, 4, 5, 7, 9, 12, 16, 17, 33, 40, 64, 100, 300)
    Rs = (1, 2, 3, 8, 10, 16, 17, 32, 33, 49, 64, 70, 130)
    tunes = ({}, {}, {}, {"pair_rows": 1}, {"pair_rows": 1}, {"pair_rows": 2}, {"pair_rows": 1, "row_blocks": 2},
             {"pair_rows": 1, "target_items": 50000}, {"pair_rows": 1, "max_steps": 3}, {"fuse_rows": 1},
             {"fuse_rows": 1, "fuse_bytes": 1 << 30}, {"fuse_rows": 2, "pair_rows": 2}, {"lead_last": 1},
             {"lead_last": 1, "max_steps": 2}, {"lead_last": 2}, {"target_items": 100000}, {"max_col_blocks": 1})
    unit = {torch.float64: 2.0 ** -53, torch.float32: 2.0 ** -24}
    seen = set()
    try:
        for case in range(200):
            d = int(rng.choice((3, 3, 3, 4, 4, 5, 6, 7)))
            dims = [int(rng.choice(I0s))] + [int(rng.choice(Is)) for _ in range(d - 1)]
            while int(np.prod(dims)) > 400_000:
                i = 1 + int(np.argmax(dims[1:]))
                dims[i] = max(1, dims[i] // 2)
            R = int(rng.choice(Rs))
            dtype = torch.float64 if rng.random() < 0.6 else torch.float32
            tune = tunes[int(rng.integers(len(tunes)))]
            X, A = make_problem(tuple(dims), R, dtype, seed=12000 + case)
            Xd, Ad = X.cuda(), [a.cuda() for a in A]
            Xn, An = inputs.as_ndarray_view(X, dims), [a.numpy() for a in A]
            for key in TUNE_KEYS:
                mt.mttkrp_tune_set(key, tune.get(key, 0))
            for k in range(d):
                desc = mt.mttkrp_plan_describe(dims, R, k, X.element_size())
                print("random short case %d dims=%s R=%d %s k=%d tune=%s %s" % (case, dims, R, dtype, k, tune, desc), flush=True)
                seen.add(re.search(r"paired_rows=(\d)", desc).group(1) if "paired_rows=" in desc else "-")
                seen.add("leading" if "shape=leading" in desc else ("fused" if "fused_rows=1" in desc else "plain"))
                ref = oracle.mttkrp(Xn, An, k)
                M = mt.mttkrp_dense(Xd, dims, Ad, k)
                torch.cuda.synchronize()
                err = oracle.normwise_rel_err(M.cpu().numpy(), ref)
                if not err <= TOL[dtype]:
                    c = np.linalg.norm(oracle.mttkrp(np.abs(Xn), [np.abs(a) for a in An], k)) / max(np.linalg.norm(ref), 1e-300)
                    assert err <= 8.0 * unit[dtype] * c, (case, dims, R, k, tune, err, c)
        # the sweep reached every route
        assert {"1", "2", "3", "leading", "fused", "plain"} <= seen, seen
    finally:
        for key in TUNE_KEYS:
            mt.mttkrp_tune_set(key, 0)


@pytest.mark.parametrize("dtype", [torch.float64, torch.float32])
def test_non_finite_values_propagate_as_in_the_definition(mt, oracle, dtype):
    """Plain IEEE propagation (the paper is silent on non-finite values): an infinite tensor
    entry or factor entry makes exactly the sums of Eq. (elem) that contain it infinite.  The
    entries sit in the last column of an inner mode whose extent is not a multiple of four (the
    step that pads its lanes by re-reading that column) and in the last rows (re-read by the
    shifted last row block); padding must not turn them into NaNs elsewhere."""
    for dims, R in (((40, 7, 5), 6), ((70, 9, 3, 2), 20), ((33, 5), 3)):
        X, A = make_problem(dims, R, dtype, seed=990, dist=("uniform", 0.1, 1.0))
        Xv = inputs.as_ndarray_view(X, dims)
        Xv[(dims[0] - 1, dims[1] - 1) + (0,) * (len(dims) - 2)] = np.inf
        A[1][dims[1] - 1, R - 1] = np.inf
        Xd, Ad = X.cuda(), [a.cuda() for a in A]
        for k in range(len(dims)):
            ref = oracle_mttkrp(oracle, X, dims, A, k)
            for tune in ({}, {"deep": 2}, {"contract_rows": 1}, {"max_steps": 2}):
                for key, val in tune.items():
                    mt.mttkrp_tune_set(key, val)
                got = mt.mttkrp_dense(Xd, dims, Ad, k).cpu().numpy()
                for key in tune:
                    mt.mttkrp_tune_set(key, 0)
                assert not np.isnan(ref).any()
                assert np.array_equal(np.isinf(got), np.isinf(ref)), (dims, k, tune)
                assert not np.isnan(got).any(), (dims, k, tune)
                fin = np.isfinite(ref)
                assert fin.any()
                err = oracle.normwise_rel_err(np.where(fin, got, 0.0), np.where(fin, ref, 0.0))
                assert err <= TOL[dtype], (dims, k, tune, err)

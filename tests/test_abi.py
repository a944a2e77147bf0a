"""Host-side checks of the C-ABI library: it loads, it exports every symbol the
header declares, and its argument validation and planning arithmetic (which
need no GPU) behave as the header says.  No compute call is made here."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADERS = [os.path.join(ROOT, "include", n) for n in sorted(os.listdir(os.path.join(ROOT, "include")))
           if n.endswith(".h")]


@pytest.fixture(scope="module")
def mt():
    from paper_2510_14891_amd import binding, build
    if not os.path.exists(binding.LIB_PATH):
        build.build()
    binding.lib()
    return binding


def declared_functions():
    names = set()
    for header in HEADERS:
        text = open(header).read()
        text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
        names |= set(re.findall(r"\b(mttkrp_[a-z0-9_]+)\s*\(", text))
    return sorted(names)


def test_header_symbols_are_exported(mt):
    names = declared_functions()
    assert len(names) >= 12
    L = mt.lib()
    for n in names:
        assert hasattr(L, n), n
    assert sorted(mt.EXPORTED) == names


def test_status_strings_and_version(mt):
    assert mt.mttkrp_version() >= 100
    seen = set()
    for s in range(5):
        t = mt.mttkrp_status_string(s)
        assert t and t not in seen
        seen.add(t)
    assert "unknown" in mt.mttkrp_status_string(99)


def test_workspace_query_and_validation(mt):
    L = mt.lib()
    bad = ctypes.c_size_t(-1).value
    d3 = (ctypes.c_int64 * 3)(64, 64, 64)
    assert L.mttkrp_dense_workspace_bytes(3, d3, 16, 0, 8) != bad
    assert L.mttkrp_dense_workspace_bytes(3, d3, 16, 3, 8) == bad      # k out of range
    assert L.mttkrp_dense_workspace_bytes(3, d3, 0, 0, 8) == bad       # R < 1
    assert L.mttkrp_dense_workspace_bytes(1, d3, 4, 0, 8) == bad       # ndim < 2
    assert L.mttkrp_dense_workspace_bytes(3, d3, 4, 0, 2) == bad       # dtype size
    assert L.mttkrp_dense_workspace_bytes(3, None, 4, 0, 8) == bad
    z = (ctypes.c_int64 * 3)(64, 0, 64)
    assert L.mttkrp_dense_workspace_bytes(3, z, 4, 0, 8) == bad
    huge = (ctypes.c_int64 * 3)(2 ** 30, 2 ** 30, 2 ** 30)            # N overflows
    assert L.mttkrp_dense_workspace_bytes(3, huge, 4, 0, 8) == bad
    # null pointers are rejected before anything touches the device
    assert L.mttkrp_dense_f64(3, d3, None, None, 4, 0, None, None) == mt.MTTKRP_ERR_INVALID_ARG
    assert L.mttkrp_tune_set(b"no_such_key", 1) == mt.MTTKRP_ERR_INVALID_ARG
    assert L.mttkrp_tune_set(b"row_blocks", 9) == mt.MTTKRP_ERR_INVALID_ARG


def test_workspace_stays_in_the_sum_of_dims_class(mt):
    """Sec. I / II-B: memory beyond X is O(R sum_n I_n)-class, never
    O(R prod_{n != k} I_n).  The partial sums are (number of splits) x I_k x R
    with the split count bounded by a plan constant; the one plan that keeps more (whole tiles of
    the first mode on row pairs) is capped at 2.5 % of the bytes of X."""
    from paper_2510_14891_amd import inputs
    for name, w in inputs.WORKLOADS.items():
        for k in range(w.ndim):
            ws = mt.mttkrp_dense_workspace_bytes(w.dims, w.R, k, w.itemsize)
            x_bytes = w.numel * w.itemsize
            assert ws <= 0.04 * x_bytes + (64 << 20), (name, k, ws)
            desc = mt.mttkrp_plan_describe(w.dims, w.R, k, w.itemsize)
            slots = int(re.search(r"slots=(\d+)", desc).group(1))
            fused = int(re.search(r"fused_bytes=(\d+)", desc).group(1))
            part = slots * w.dims[k] * w.R * w.itemsize if slots > 1 else 0
            assert ws == (part + 255) // 256 * 256 + fused
            assert fused <= (8 << 20) + (32 << 20)    # at most two product matrices of fused modes (columns, rows), each small
            if "paired_rows=3" in desc:
                # first mode on (i_0, i_1) row pairs with whole weighted tiles stored: one copy of
                # I_0 I_1 x R values per split, capped at 2.5 % of the bytes of X
                assert part <= 0.025 * x_bytes, (name, k, part)
            else:
                assert slots <= 4096, (name, k, slots)


def test_workspace_bounded_for_short_column_spaces(mt):
    """Sec. I / II-B memory claim on shapes where the modes other than 0 and k have few entries
    and the rank is high: one partial row of M per row block would approach the size of X, so
    the planner must switch to the schedule whose partial sums stay small."""
    cases = [((20000, 20000, 7), 500, 1, 4), ((4096, 4096, 32), 2000, 1, 8), ((1000, 2, 1, 20000), 100, 3, 4),
             ((33, 20000, 1), 500, 1, 8), ((401, 20000), 500, 1, 4), ((16384, 2048, 64), 128, 1, 8)]
    for dims, R, k, sb in cases:
        n = 1
        for d in dims:
            n *= d
        ws = mt.mttkrp_dense_workspace_bytes(dims, R, k, sb)
        assert ws <= 0.05 * n * sb + (64 << 20), (dims, R, k, ws)
        desc = mt.mttkrp_plan_describe(dims, R, k, sb)
        slots = int(re.search(r"slots=(\d+)", desc).group(1))
        fused = int(re.search(r"fused_bytes=(\d+)", desc).group(1))
        part = slots * dims[k] * R * sb if slots > 1 else 0
        assert ws == (part + 255) // 256 * 256 + fused, desc


def test_tile_volume_matches_the_oracle(mt):
    """Eq. (heuristic): the library's integer arithmetic against the oracle's exact
    rational arithmetic, value for value (host only)."""
    from oracle import tile_heuristic
    shapes = [(401, 201, 12, 501), (129, 129, 129, 12, 39), (1024, 1024, 512), (7, 5), (3, 1, 2, 2),
              (48,) * 5, (192,) * 4, (2, 2, 2, 2, 2, 2, 2, 2)]
    n = 0
    for dims in shapes:
        for cache in (1, 100, 16384, 32768, 65536, 163840, 262144, 1 << 21, (1 << 22) + 5):
            for vb in (4, 8):
                for c in (1, 2, 3, 8, 32, 64, 1000):
                    assert mt.mttkrp_tile_volume(dims, cache, vb, c) == \
                        tile_heuristic.tile_volume(dims, cache, vb, c), (dims, cache, vb, c)
                    n += 1
    assert n > 1000
    L = mt.lib()
    w = ctypes.c_int64(0)
    d3 = (ctypes.c_int64 * 3)(4, 4, 4)
    assert L.mttkrp_tile_volume(3, d3, 0, 8, 1, ctypes.byref(w), ctypes.byref(w)) == mt.MTTKRP_ERR_INVALID_ARG
    assert L.mttkrp_tile_volume(1, d3, 1024, 8, 1, ctypes.byref(w), ctypes.byref(w)) == mt.MTTKRP_ERR_INVALID_ARG
    assert L.mttkrp_ablation_f64(9, 3, d3, None, None, 4, 0, 1, None, None) == mt.MTTKRP_ERR_INVALID_ARG


def test_shared_sweep_and_leading_contraction_plans(mt):
    """Host arithmetic of the sweep that shares partial contractions: the workspace query is
    positive where a cut fits an eighth of the tensor (or 64 MiB), 0 where none does, never
    more than that bound, and the leading contraction only asks for partial sums when its
    columns alone cannot fill the chip."""
    L = mt.lib()
    NO = ctypes.c_size_t(-1).value
    for dims, R, sb in (((1024, 1024, 512), 32, 8), ((192,) * 4, 16, 8), ((48,) * 5, 64, 4),
                        ((16384, 2048, 64), 4, 8), ((16384, 2048, 64), 128, 8), ((401, 201, 12, 501), 32, 8),
                        ((129, 129, 129, 12, 39), 32, 8), ((64, 64, 64), 16, 8), ((5, 4), 3, 8)):
        n = 1
        for d in dims:
            n *= d
        b = mt.mttkrp_dense_all_modes_shared_bytes(dims, R, sb)
        assert 0 < b <= max(n * sb // 8, 64 << 20), (dims, R, b)
    # intermediates far beyond the tensor: not supported, the caller runs d separate passes
    assert mt.mttkrp_dense_all_modes_shared_bytes((401, 201, 12, 501), 1000, 8) == 0
    assert mt.mttkrp_dense_all_modes_shared_bytes((4096, 8), 2000, 8) == 0 or \
        mt.mttkrp_dense_all_modes_shared_bytes((4096, 8), 2000, 8) <= 64 << 20
    # invalid arguments
    assert mt.mttkrp_dense_all_modes_shared_bytes((8, 0, 8), 4, 8) == 0
    assert mt.mttkrp_dense_all_modes_shared_bytes((8, 8), 4, 2) == 0
    f = L.mttkrp_contract_leading_workspace_bytes
    assert f(1024, 1024 * 512, 32, 8) == 0            # many columns: no row splits, no partial sums
    assert f(16384, 131072, 128, 8) == 0
    assert f(100000, 16, 4, 8) > 0                    # one column tile: rows are split
    assert f(100000, 16, 4, 8) % (16 * 4 * 8) == 0    # [column][split][R] values
    assert f(0, 16, 4, 8) == NO and f(16, 0, 4, 8) == NO and f(16, 16, 0, 8) == NO and f(16, 16, 4, 3) == NO
    assert f(1 << 31, 16, 4, 8) == NO and f(16, 1 << 31, 4, 8) == NO

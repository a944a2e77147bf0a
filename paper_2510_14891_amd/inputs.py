"""Seeded synthetic inputs for the dense MTTKRP workloads.

This module only *makes inputs*: a counter-based random generator and the
recipes of the benchmark configurations.  It contains none of the MTTKRP
arithmetic and imports neither the CPU oracle nor the HIP binding; both the
tests of the oracle and the tests/benchmark of the HIP path draw their inputs
from here, so that the two sides always see the same buffers.

Generator (index-addressed, so a value never depends on chunking, thread count
or device):

    z  = seed XOR (GOLDEN * (index + 1))            (mod 2^64)
    z  = (z XOR (z >>> 30)) * C1
    z  = (z XOR (z >>> 27)) * C2
    z  =  z XOR (z >>> 31)
    u  = (z >>> 11) / 2^53                           in [0, 1)

normal values use Box-Muller on the uniforms at counters 2*index, 2*index+1.
All integer steps are exact on every device; the floating-point transform may
differ in the last bit between CPU and GPU, which is harmless because both
sides of every comparison read the one buffer that was generated.

The paper's own experiments use randomly generated values in the shapes of two
simulation outputs (Sec. IV), so seeded random data of the stated shapes is
the paper's kind of workload, not a stand-in for a dataset.
"""
from __future__ import annotations

import math
from dataclasses import dataclass, field
from typing import Dict, List, Optional, Sequence, Tuple

import torch

_GOLDEN = 0x9E3779B97F4A7C15
_C1 = 0xBF58476D1CE4E5B9
_C2 = 0x94D049BB133111EB
_MASK64 = (1 << 64) - 1


def _s64(v: int) -> int:
    """Two's-complement view of a 64-bit pattern as a signed Python int."""
    v &= _MASK64
    return v - (1 << 64) if v >= (1 << 63) else v


def _lsr(z: torch.Tensor, s: int) -> torch.Tensor:
    """Logical shift right of int64 bit patterns."""
    return (z >> s) & ((1 << (64 - s)) - 1)


def hash_bits(seed: int, start: int, count: int, device="cpu") -> torch.Tensor:
    """64 hashed bits (as int64 patterns) for counters start .. start+count-1."""
    idx = torch.arange(start + 1, start + count + 1, dtype=torch.int64, device=device)
    z = (idx * _s64(_GOLDEN)) ^ _s64(seed)
    z = (z ^ _lsr(z, 30)) * _s64(_C1)
    z = (z ^ _lsr(z, 27)) * _s64(_C2)
    z = z ^ _lsr(z, 31)
    return z


def hash_bits_scalar(seed: int, index: int) -> int:
    """Pure-Python value of the same hash for one counter (used by tests)."""
    z = (seed ^ (_GOLDEN * (index + 1))) & _MASK64
    z = ((z ^ (z >> 30)) * _C1) & _MASK64
    z = ((z ^ (z >> 27)) * _C2) & _MASK64
    z = z ^ (z >> 31)
    return z


def _unit(seed: int, start: int, count: int, device) -> torch.Tensor:
    z = hash_bits(seed, start, count, device)
    return _lsr(z, 11).to(torch.float64) * (1.0 / 9007199254740992.0)


_CHUNK = 1 << 24


def fill_uniform(out: torch.Tensor, seed: int, lo: float = 0.0, hi: float = 1.0,
                 offset: int = 0) -> torch.Tensor:
    """Fill the flat tensor ``out`` with U[lo, hi) values for counters
    offset .. offset+numel-1 (computed in fp64, rounded once to out.dtype)."""
    flat = out.view(-1)
    n = flat.numel()
    for s in range(0, n, _CHUNK):
        c = min(_CHUNK, n - s)
        u = _unit(seed, offset + s, c, flat.device)
        flat[s:s + c] = (lo + (hi - lo) * u).to(flat.dtype)
    return out


def fill_normal(out: torch.Tensor, seed: int, mean: float = 0.0, std: float = 1.0,
                offset: int = 0) -> torch.Tensor:
    """Fill ``out`` with N(mean, std^2) values (Box-Muller, fp64, rounded once)."""
    flat = out.view(-1)
    n = flat.numel()
    for s in range(0, n, _CHUNK):
        c = min(_CHUNK, n - s)
        u = _unit(seed, 2 * (offset + s), 2 * c, flat.device).view(c, 2)
        r = torch.sqrt(-2.0 * torch.log1p(-u[:, 0]))
        g = r * torch.cos((2.0 * math.pi) * u[:, 1])
        flat[s:s + c] = (mean + std * g).to(flat.dtype)
    return out


def uniform(seed: int, shape, lo=0.0, hi=1.0, dtype=torch.float64, device="cpu"):
    n = int(math.prod(shape)) if not isinstance(shape, int) else shape
    out = torch.empty(n, dtype=dtype, device=device)
    fill_uniform(out, seed, lo, hi)
    return out.view(shape)


def normal(seed: int, shape, mean=0.0, std=1.0, dtype=torch.float64, device="cpu"):
    n = int(math.prod(shape)) if not isinstance(shape, int) else shape
    out = torch.empty(n, dtype=dtype, device=device)
    fill_normal(out, seed, mean, std)
    return out.view(shape)


# --------------------------------------------------------------------------
# Workload recipes
# --------------------------------------------------------------------------

@dataclass(frozen=True)
class Workload:
    """One benchmark configuration: a dense tensor, its factors and a rank.

    ``dims`` are (I_0, ..., I_{d-1}); X is stored flat, first index fastest.
    ``x_dist`` / ``a_dist`` are ("uniform", lo, hi), ("normal", mean, std) or,
    for X only, ("cp_noise", cp_rank, relative_noise).
    """
    name: str
    dims: Tuple[int, ...]
    dtype: str                      # "f64" or "f32"
    R: int
    x_dist: Tuple
    a_dist: Tuple
    seed_id: int                    # the "c" of the seed recipe
    note: str = ""

    @property
    def ndim(self) -> int:
        return len(self.dims)

    @property
    def numel(self) -> int:
        return int(math.prod(self.dims))

    @property
    def torch_dtype(self):
        return torch.float64 if self.dtype == "f64" else torch.float32

    @property
    def itemsize(self) -> int:
        return 8 if self.dtype == "f64" else 4


def _wl(name, dims, dtype, R, x_dist, a_dist, c, note=""):
    return Workload(name, tuple(dims), dtype, R, tuple(x_dist), tuple(a_dist), c, note)


# The five benchmark configurations plus the paper's own two tensor shapes
# (Sec. IV: tensor A 401x201x12x501 and tensor B 129x129x129x12x39, random
# values, R = 32 in the model and tile-width tables).
WORKLOADS: Dict[str, Workload] = {w.name: w for w in [
    _wl("c1_64x64x64_f64_R16", (64, 64, 64), "f64", 16,
        ("uniform", 0.0, 1.0), ("uniform", 0.0, 1.0), 1),
    _wl("c2_1024x1024x512_f64_R32", (1024, 1024, 512), "f64", 32,
        ("normal", 0.0, 1.0), ("normal", 0.0, 1.0), 2),
    _wl("c3_192x192x192x192_f64_R16", (192, 192, 192, 192), "f64", 16,
        ("uniform", -1.0, 1.0), ("uniform", -1.0, 1.0), 3),
    _wl("c4_48x48x48x48x48_f32_R64", (48, 48, 48, 48, 48), "f32", 64,
        ("cp_noise", 8, 0.01), ("normal", 0.0, 1.0), 4),
    _wl("c5_16384x2048x64_f64_R4", (16384, 2048, 64), "f64", 4,
        ("uniform", 0.0, 1.0), ("uniform", 0.0, 1.0), 5),
    _wl("c5_16384x2048x64_f64_R8", (16384, 2048, 64), "f64", 8,
        ("uniform", 0.0, 1.0), ("uniform", 0.0, 1.0), 5),
    _wl("c5_16384x2048x64_f64_R128", (16384, 2048, 64), "f64", 128,
        ("uniform", 0.0, 1.0), ("uniform", 0.0, 1.0), 5),
    _wl("paperA_401x201x12x501_f64_R32", (401, 201, 12, 501), "f64", 32,
        ("uniform", 0.0, 1.0), ("uniform", 0.0, 1.0), 6,
        "shape of the paper's tearing-mode tensor, random values"),
    _wl("paperA_401x201x12x501_f64_R10", (401, 201, 12, 501), "f64", 10,
        ("uniform", 0.0, 1.0), ("uniform", 0.0, 1.0), 6,
        "shape of the paper's tearing-mode tensor, random values, the paper's smallest rank"),
    _wl("paperA_401x201x12x501_f64_R1000", (401, 201, 12, 501), "f64", 1000,
        ("uniform", 0.0, 1.0), ("uniform", 0.0, 1.0), 6,
        "shape of the paper's tearing-mode tensor at one of its high ranks (Sec. IV-C, IV-D)"),
    _wl("paperA_401x201x12x501_f64_R2000", (401, 201, 12, 501), "f64", 2000,
        ("uniform", 0.0, 1.0), ("uniform", 0.0, 1.0), 6,
        "shape of the paper's tearing-mode tensor at the paper's highest rank (Sec. IV-C, IV-D)"),
    _wl("paperB_129x129x129x12x39_f64_R32", (129, 129, 129, 12, 39), "f64", 32,
        ("uniform", 0.0, 1.0), ("uniform", 0.0, 1.0), 7,
        "shape of the paper's island-coalescence tensor, random values"),
    _wl("paperB_cp10_129x129x129x12x39_f64_R10", (129, 129, 129, 12, 39), "f64", 10,
        ("cp_noise", 10, 0.01), ("uniform", 0.0, 1.0), 8,
        "shape of the paper's island-coalescence tensor, rank-10 Kruskal tensor plus 1 % noise: "
        "the CP-ALS workload (the paper runs CP-ALS on this shape at R = 10 and up)"),
]}


def scaled(w: Workload, dims: Sequence[int], name: Optional[str] = None) -> Workload:
    """Same recipe (distributions, seeds, dtype, R) on a smaller shape."""
    return Workload(name or (w.name + "_scaled"), tuple(dims), w.dtype, w.R,
                    w.x_dist, w.a_dist, w.seed_id, "scaled-down " + w.name)


def _fill(out: torch.Tensor, seed: int, dist: Tuple) -> torch.Tensor:
    if dist[0] == "uniform":
        return fill_uniform(out, seed, dist[1], dist[2])
    if dist[0] == "normal":
        return fill_normal(out, seed, dist[1], dist[2])
    raise ValueError("unknown distribution %r" % (dist,))


def make_factors(w: Workload, device="cpu", R: Optional[int] = None) -> List[torch.Tensor]:
    """Factor matrices A_m (I_m x R, row-major), seed 2000 + 10c + m."""
    R = w.R if R is None else R
    out = []
    for m, I in enumerate(w.dims):
        A = torch.empty((I, R), dtype=w.torch_dtype, device=device)
        _fill(A, 2000 + 10 * w.seed_id + m, w.a_dist)
        out.append(A)
    return out


def _fill_cp_noise(flat: torch.Tensor, w: Workload) -> None:
    """X = X_cp + rel * rms(X_cp) * N(0,1); X_cp a Kruskal tensor of rank S
    with N(0,1) factors (seeds 3000+m), built in fp64 and rounded once.

    Built slab by slab over the last mode so that the (N/I_last) x S
    Khatri-Rao matrix of the leading modes is the largest temporary.
    """
    S, rel = int(w.x_dist[1]), float(w.x_dist[2])
    dev = flat.device
    U = [normal(3000 + m, (I, S), dtype=torch.float64, device=dev)
         for m, I in enumerate(w.dims)]
    # Z[(i_0,...,i_{d-2}), s] with i_0 fastest
    Z = U[0]
    for m in range(1, w.ndim - 1):
        Z = (U[m][:, None, :] * Z[None, :, :]).reshape(-1, S)
    L = Z.shape[0]
    # sum of squares of X_cp from the Gram matrices (exact identity):
    # ||X_cp||^2 = 1^T (hadamard_m U_m^T U_m) 1
    G = torch.ones((S, S), dtype=torch.float64, device=dev)
    for Um in U:
        G = G * (Um.T @ Um)
    rms = math.sqrt(float(G.sum()) / w.numel)
    I_last = w.dims[-1]
    for i in range(I_last):
        slab = Z @ U[-1][i]
        noise = torch.empty(L, dtype=torch.float64, device=dev)
        fill_normal(noise, 3999, offset=i * L)
        flat[i * L:(i + 1) * L] = (slab + (rel * rms) * noise).to(flat.dtype)


def kruskal_tensor(dims: Sequence[int], S: int, seed: int, device="cpu"):
    """(flat X, [U_0, ..., U_{d-1}]): the rank-S Kruskal tensor (Sec. II-A)
    X(i) = sum_s prod_m U_m(i_m, s) with N(0,1) factors U_m (I_m x S, seeds
    seed + m), fp64, flat and first index fastest.  Built slab by slab over the
    last mode (plain elementwise products and a sum over s, every operation rounded)."""
    dims = tuple(int(v) for v in dims)
    d = len(dims)
    U = [normal(seed + m, (I, S), dtype=torch.float64, device=device) for m, I in enumerate(dims)]
    Z = U[0]
    for m in range(1, d - 1):
        Z = (U[m][:, None, :] * Z[None, :, :]).reshape(-1, S)
    L = Z.shape[0]
    flat = torch.empty(L * dims[-1], dtype=torch.float64, device=device)
    for i in range(dims[-1]):
        torch.sum(Z * U[-1][i], dim=1, out=flat[i * L:(i + 1) * L])
    return flat, U


def make_tensor(w: Workload, device="cpu") -> torch.Tensor:
    """The dense tensor as a flat 1-D torch tensor of N values, first index
    fastest, seed 1000 + c."""
    flat = torch.empty(w.numel, dtype=w.torch_dtype, device=device)
    if w.x_dist[0] == "cp_noise":
        _fill_cp_noise(flat, w)
    else:
        _fill(flat, 1000 + w.seed_id, w.x_dist)
    return flat


def as_ndarray_view(flat: torch.Tensor, dims: Sequence[int]):
    """numpy view of a flat first-index-fastest CPU tensor with logical shape
    ``dims`` (Fortran order), without copying."""
    import numpy as np
    return np.reshape(flat.numpy(), tuple(dims), order="F")

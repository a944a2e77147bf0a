"""Flop, byte and time models used for reporting (paper Sec. IV-B).

    f        = N R d                                   flops the paper counts
    m_inf    = s_f (N + R sum_n I_n)                    infinite-cache bytes
    m_0      = s_f (N + N R (d-1) + (N_S/N_T) I_k R)   zero-cache bytes
    m_0,LM   = s_f (N + (N_S/N_T) I_k R) + s_f N R (d-1) / l
    T_i      = f / tau_f + m_i / tau_m
    gflops   = f / t / 1024^3                           (the paper's divisor)

The streaming kernel of this library executes 2 N R flops (one fused
multiply-add per tensor entry and column) plus lower-order terms, because it
factors the product of Eq. (elem); both counts are reported.
"""
from __future__ import annotations

import math
from typing import Sequence


def numel(dims: Sequence[int]) -> int:
    return int(math.prod(dims))


def flops_paper(dims: Sequence[int], R: int) -> float:
    return float(numel(dims)) * R * len(dims)


def flops_executed(dims: Sequence[int], R: int) -> float:
    return 2.0 * numel(dims) * R


def m_inf(dims: Sequence[int], R: int, s_f: int) -> int:
    return s_f * (numel(dims) + R * sum(int(v) for v in dims))


def m_0(dims: Sequence[int], R: int, s_f: int, k: int, n_t: int = 1) -> float:
    N = numel(dims)
    d = len(dims)
    n_s = N // int(dims[k])
    return s_f * (N + N * R * (d - 1) + (n_s / n_t) * int(dims[k]) * R)


def m_0_lm(dims: Sequence[int], R: int, s_f: int, k: int, n_t: int, l: float) -> float:
    N = numel(dims)
    d = len(dims)
    n_s = N // int(dims[k])
    return s_f * (N + (n_s / n_t) * int(dims[k]) * R) + s_f * N * R * (d - 1) / l


def predicted_time(flops: float, bytes_: float, tau_f: float, tau_m: float) -> float:
    """T = f / tau_f + m / tau_m with tau_f in flop/s and tau_m in B/s."""
    return flops / tau_f + bytes_ / tau_m


def gflops_paper_units(flops: float, seconds: float) -> float:
    return flops / seconds / 1024.0 ** 3

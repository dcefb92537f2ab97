"""Operation counts for the SLA path (host-side bookkeeping for the benchmark).

Executed work is counted on the critical blocks only, with the valid rows r and columns c of
every 64 x 64 pair (tail tiles count for less): forward 4 r c d (Q K^T and P V), backward
10 r c d (S, dP, dV, dQ, dK).  "Dense" is the same count with every pair critical, i.e.
4 N^2 d and 10 N^2 d per head -- the operation count of full attention that the paper's
efficiency metric divides by the latency (Section 6.1, Metrics).
"""
from __future__ import annotations

import numpy as np


def critical_pair_elems(Mc: np.ndarray, N: int, b: int = 64, bq: int = 0) -> int:
    """Sum over critical pairs of (valid rows) x (valid columns); Mc is [..., Tq, T] for query
    blocks of bq (default b) and key blocks of b tokens."""
    bq = bq or b
    Tq, T = Mc.shape[-2:]
    valid = np.full(T, b, np.int64)
    valid[-1] = N - (T - 1) * b
    validq = np.full(Tq, bq, np.int64)
    validq[-1] = N - (Tq - 1) * bq
    crit = (Mc.reshape(-1, Tq, T) == 1)
    return int(np.einsum("gij,i,j->", crit.astype(np.int64), validq, valid))


def executed_flops(Mc: np.ndarray, N: int, d: int, b: int = 64, bq: int = 0):
    """(forward, backward) FLOPs executed on the critical blocks of a whole call."""
    e = critical_pair_elems(Mc, N, b, bq)
    return 4 * e * d, 10 * e * d


def dense_flops(BH: int, N: int, d: int):
    """(forward, backward) FLOPs of full attention on the same shape."""
    return 4 * BH * N * N * d, 10 * BH * N * N * d


def linear_flops(BH: int, N: int, d: int):
    """Forward FLOPs of the linear branch per call: h_j, phi(Q) H_i, Proj (6 N d^2 per head);
    the state aggregation is extra and depends on how it is carried out."""
    return 6 * BH * N * d * d

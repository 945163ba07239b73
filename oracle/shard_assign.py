"""Exact statements of the batch-splitting rules (host-side integer work).

Test infrastructure: see the package docstring.

* A worker's shard is a pair (start offset, length) and the lengths add up to
  the fixed global batch (Section V-C.1; constraint of Eq. 1).
* Initialisation gives every worker B/n (Section VI-A, step 1).
* ADJUST_BS solves Eq. 3: minimise z subject to z >= B_i / v_i and
  sum_i B_i = B over non-negative integers B_i.  Here the optimum is found by
  enumerating every split, with exact rational arithmetic.
* The data set of N samples is cut into K = ceil(N / (B*M)) shards of M
  batches each (Section V-C.1).
* Eq. 4 (gradient accumulation on k device types) is enumerated the same way.
"""
from __future__ import annotations

from fractions import Fraction
from itertools import product
from typing import List, Sequence, Tuple


def explicit_split(sizes: Sequence[int]) -> List[Tuple[int, int]]:
    """Contiguous (start, length) slices in worker order."""
    out, start = [], 0
    for n in sizes:
        if n < 0:
            raise ValueError("negative shard size")
        out.append((start, int(n)))
        start += int(n)
    return out


def equal_split(B: int, n: int) -> List[Tuple[int, int]]:
    """B_i = B/n; when n does not divide B the first B mod n workers get one more."""
    q, r = divmod(B, n)
    return explicit_split([q + (1 if i < r else 0) for i in range(n)])


def minmax_objective(sizes: Sequence[int], speeds: Sequence[float]) -> Fraction:
    """max_i B_i / v_i as an exact rational (v_i taken at its exact binary value)."""
    return max(Fraction(int(b)) / Fraction(v) for b, v in zip(sizes, speeds))


def _compositions(total: int, parts: int):
    if parts == 1:
        yield (total,)
        return
    for first in range(total + 1):
        for rest in _compositions(total - first, parts - 1):
            yield (first,) + rest


def minmax_split_bruteforce(B: int, speeds: Sequence[float]):
    """All optimal integer solutions of Eq. 3 and the optimal value z*, by enumeration."""
    best, arg = None, []
    for c in _compositions(B, len(speeds)):
        z = minmax_objective(c, speeds)
        if best is None or z < best:
            best, arg = z, [c]
        elif z == best:
            arg.append(c)
    return best, arg


def num_data_shards(N: int, B: int, M: int) -> int:
    """K = ceil(N / (B*M))."""
    return -(-N // (B * M))


def data_shards(N: int, B: int, M: int) -> List[Tuple[int, int]]:
    """The K shards as (start offset, length); only the last one may be short."""
    return [(i * B * M, min(B * M, N - i * B * M)) for i in range(num_data_shards(N, B, M))]


def accumulation_plan_bruteforce(B: int, counts: Sequence[int], speeds: Sequence[float],
                                 bmin: Sequence[int], bmax: Sequence[int], cmin: int, cmax: int):
    """Eq. 4 by enumeration: minimise max_i C_i*B_i/v_i subject to
    sum_i n_i*C_i*B_i = B, bmin_i <= B_i <= bmax_i, cmin <= C_i <= cmax.
    Returns (optimal value or None if infeasible, list of optimal ((C_i), (B_i)))."""
    k = len(counts)
    best, arg = None, []
    ranges = [[(c, b) for c in range(cmin, cmax + 1) for b in range(bmin[i], bmax[i] + 1)]
              for i in range(k)]
    for combo in product(*ranges):
        if sum(counts[i] * combo[i][0] * combo[i][1] for i in range(k)) != B:
            continue
        z = max(Fraction(combo[i][0] * combo[i][1]) / Fraction(speeds[i]) for i in range(k))
        plan = (tuple(c for c, _ in combo), tuple(b for _, b in combo))
        if best is None or z < best:
            best, arg = z, [plan]
        elif z == best:
            arg.append(plan)
    return best, arg

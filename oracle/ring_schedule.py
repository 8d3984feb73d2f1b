"""The paper's ring schedules as index streams (Yu & Fujita, Algorithms 1, 2 and 3).

TEST INFRASTRUCTURE ONLY, like the rest of oracle/: nothing in the product imports it.

The paper places one multiply-accumulate per PE and cycle on a unidirectional ring of m PEs and
gives, for every cycle and PE, which operands meet there: vector A (the query / output row),
vector B (the key / value) and component C.  This module turns those index formulas into streams
of (cycle, pe, A, B, C) - a slot in which the PE has nothing to do carries zeros - so that tests can check what the paper claims of them: every needed
multiply-accumulate is met exactly once, a partial sum is always handed to the next PE, the PEs of
a cycle never share an operand pair, and the cycle counts are those of Tables 1 and 2.

All indices are 1-based as in the paper; `%` is the mathematical remainder and `\\` the integer
quotient.  The formulas are kept as printed, because they are what is under test; the one place
where the printed text cannot be meant literally is a switch (see masked_phase2).
"""
from __future__ import annotations

from itertools import product
from typing import Iterator, Tuple


def _check(n: int, m: int) -> int:
    if n <= 0 or m <= 0 or n % m:
        raise ValueError("m must divide n (abstract of the paper)")
    return n // m


# Operand positions on the ring.  In sweep i (one of n/m) at step j (one of n), PE l (1..m) holds
#   a vector index that the ring rotates through the m vectors of the sweep, and
#   a component index that moves on by m every m steps.
def _rotating(l: int, j: int, i: int, m: int) -> int:
    return (l - j) % m + (i - 1) * m + 1          # in ((i-1)m, im]


def _component(l: int, j: int, i: int, m: int, n: int) -> int:
    return (l + ((j - 1) // m) * m + (i - 1) * m - 1) % n + 1


def _sweeps(n: int, m: int) -> Iterator[Tuple[int, int, int]]:
    """(i, j, l): sweeps, steps, PEs, in execution order."""
    return product(range(1, _check(n, m) + 1), range(1, n + 1), range(1, m + 1))


def baseline_phase1(n: int, m: int) -> Iterator[Tuple[int, int, int, int, int]]:
    """Algorithm 1, phase 1 (Eq. (1)): stage h computes row A = h of the scores.  The key index of
    the printed formula is the rotating index shifted down by one (with 0 standing for n)."""
    cycle = 0
    for h in range(1, n + 1):
        last = None
        for i, j, l in _sweeps(n, m):
            if (i, j) != last:
                cycle, last = cycle + 1, (i, j)
            yield cycle, l, h, (_rotating(l, j, i, m) - 2) % n + 1, _component(l, j, i, m, n)


def baseline_phase2(n: int, m: int) -> Iterator[Tuple[int, int, int, int]]:
    """Algorithm 1, phase 2, one pass (Eq. (2)): (cycle, pe, A, B); the row index rotates, the key
    index takes the place of the component."""
    cycle, last = 0, None
    for i, j, l in _sweeps(n, m):
        if (i, j) != last:
            cycle, last = cycle + 1, (i, j)
        yield cycle, l, _rotating(l, j, i, m), _component(l, j, i, m, n)


def symmetric_phase1(n: int, m: int) -> Iterator[Tuple[int, int, int, int, int]]:
    """Algorithm 2, phase 1 (Sec. 4.2), the computing slots only: stage h computes the circulant
    diagonal at distance h from the main one, one element of every symmetric pair; on which side of
    the main diagonal depends on h % m, which decides the direction the result is later passed in.
    For even n a last stage computes the diagonal n/2 in full (the balance trade-off).  The extra
    transfer cycles that copy w'_AB to w'_BA are not enumerated."""
    half = (n - 1) // 2 if n % 2 else n // 2 - 1
    stages = [(h, h if (h % m) <= m / 2 else -h) for h in range(0, half + 1)]
    if n % 2 == 0:
        stages.append((n // 2, n // 2))
    cycle = 0
    for _, shift in stages:
        last = None
        for i, j, l in _sweeps(n, m):
            if (i, j) != last:
                cycle, last = cycle + 1, (i, j)
            b = (_rotating(l, j, i, m) - 2) % n + 1
            yield cycle, l, (b + shift - 1) % n + 1, b, _component(l, j, i, m, n)


def masked_phase1(n: int, m: int) -> Iterator[Tuple[int, int, int, int, int]]:
    """Algorithm 3, phase 1 (Sec. 5.2): stage h packs row n-h (keys up to n-h) with row h, which
    takes the slots whose key would lie above the diagonal, the key folded back by n-h.  For even
    n one more stage does row n/2 alone, on the slots at or below the diagonal."""
    half = (n - 1) // 2 if n % 2 else n // 2 - 1
    cycle = 0
    for h in range(0, half + 1):
        last = None
        for i, j, l in _sweeps(n, m):
            if (i, j) != last:
                cycle, last = cycle + 1, (i, j)
            a, b = n - h, _rotating(l, j, i, m)
            if a < b:
                a, b = h, b % (n - h)
            yield cycle, l, a, b, _component(l, j, i, m, n)
    if n % 2 == 0:
        last = None
        for i, j, l in _sweeps(n, m):
            if (i, j) != last:
                cycle, last = cycle + 1, (i, j)
            b = _rotating(l, j, i, m)
            if n // 2 >= b:
                yield cycle, l, n // 2, b, _component(l, j, i, m, n)
            else:
                yield cycle, l, 0, 0, 0                # idle slot


def masked_phase2(n: int, m: int, as_printed: bool = False) -> Iterator[Tuple[int, int, int, int]]:
    """Algorithm 3, phase 2, one pass: all n*n slots are kept and only those with B <= A compute
    (the paper accepts about half the PEs idle here).  Rows in the upper half take their keys
    rotated by n - A.  The printed row index lacks the `+1` that the same line of Algorithm 1
    has; read literally (as_printed) it runs over 0..n-1 and row n is never summed."""
    cycle, last = 0, None
    for i, j, l in _sweeps(n, m):
        if (i, j) != last:
            cycle, last = cycle + 1, (i, j)
        a = _rotating(l, j, i, m) - (1 if as_printed else 0)
        b = _component(l, j, i, m, n)
        if a < n / 2:
            b = (b - (n - a) - 1) % n + 1
        if a >= b:
            yield cycle, l, a, b
        else:
            yield cycle, l, 0, 0                       # idle slot


def cycles(stream) -> int:
    """Number of cycles a stream spans (its last cycle number; cycles with idle PEs count)."""
    top = 0
    for rec in stream:
        top = max(top, rec[0])
    return top

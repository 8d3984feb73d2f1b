"""Pins for the CPU checker's counting functions (no GPU).

The counts come from enumerating the redundancy predicate; here they are held
against what the paper fixes: the closed-form operation counts of Sec. 3.2,
Sec. 4.1/4.2 and Sec. 5.1, the "near 25% / near 50%" reductions, and the cycle
counts printed in Tables 1 and 2.
"""
import os

import numpy as np
import pytest

from oracle import attn_oracle as orc
from paper_2012_01114_amd import inputs

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "ring_cycles_tables.txt")


def _divisors(n):
    return [p for p in range(1, n + 1) if n % p == 0]


@pytest.mark.parametrize("n", list(range(1, 41)) + [48, 63, 64])
def test_pair_counts_closed_forms(n):
    for p in _divisors(n):
        H, B = 3, 2
        full = orc.counts(batch=B, n=n, n_heads=H, p=p, scheme=orc.FULL)
        assert full["pairs_full"] == B * H * n * n
        assert full["pairs_needed"] == [B * H * n * n] * 3            # Sec. 3.2
        assert full["pairs_scheduled"] == full["pairs_needed"]
        assert full["tiles_executed"] == full["tiles_full"] == B * H * p * p

        sym = orc.counts(batch=B, n=n, n_heads=H, p=p, scheme=orc.SYMMETRIC)
        tri = n * (n + 1) // 2
        assert sym["pairs_needed"] == [B * H * tri, B * H * n * n, B * H * n * n]   # Sec. 4.1
        sched = tri if n % 2 else n * (n + 2) // 2                                     # Sec. 4.2
        assert sym["pairs_scheduled"][0] == B * H * sched
        tsched = p * (p + 1) // 2 if p % 2 else p * (p + 2) // 2
        assert sym["tiles_executed"] == B * H * tsched

        cau = orc.counts(batch=B, n=n, n_heads=H, p=p, scheme=orc.CAUSAL)
        assert cau["pairs_needed"] == [B * H * tri] * 3                              # Sec. 5.1
        assert cau["pairs_scheduled"] == cau["pairs_needed"]
        assert cau["tiles_executed"] == B * H * p * (p + 1) // 2
        assert cau["pairs_executed"] == cau["tiles_executed"] * (n // p) ** 2


def test_tiny_workload_counts():
    w = inputs.WORKLOADS["tiny"]
    kw = dict(batch=w.batch, n=w.n, n_heads=w.n_heads, p=w.p)
    c = orc.counts(scheme=orc.CAUSAL, **kw)
    assert (c["tiles_executed"], c["pairs_executed"], c["pairs_needed"][0]) == (10, 160, 136)
    s = orc.counts(scheme=orc.SYMMETRIC, **kw)
    assert (s["tiles_executed"], s["pairs_executed"], s["pairs_needed"][0], s["pairs_scheduled"][0]) == (12, 192, 136, 144)
    f = orc.counts(scheme=orc.FULL, **kw)
    assert (f["tiles_executed"], f["pairs_executed"]) == (16, 256)


def test_stated_reductions():
    """Sec. 4.2: the symmetric scheme saves d(n^2 - n(n+1)/2) of 2dn^2 + 2n^2
    operations, "near 25%"; Sec. 5.2: the masked scheme keeps n(n+1)/2 of n^2."""
    n = d = 1025
    s = orc.counts(batch=1, n=n, n_heads=1, p=1, scheme=orc.SYMMETRIC)
    total = 2 * d * n * n + 2 * n * n
    saved = d * (n * n - s["pairs_scheduled"][0])
    assert abs(saved / total - 0.25) < 1e-3
    c = orc.counts(batch=1, n=1024, n_heads=1, p=128, scheme=orc.CAUSAL)
    assert abs(c["pairs_needed"][0] / c["pairs_full"] - 0.5) < 1e-3
    assert c["pairs_needed"][0] == 524800


@pytest.mark.parametrize("lens", [[0], [1], [5], [16], [40], [3, 16, 9, 0]])
def test_key_length_counts(lens):
    n, p = 16, 4
    lens = np.array(lens, dtype=np.int32)
    c = orc.counts(batch=len(lens), n=n, n_heads=2, p=p, scheme=orc.CAUSAL, lens=lens)
    expect = 0
    tiles = 0
    for L in np.minimum(lens, n):
        L = int(L)
        expect += L * (L + 1) // 2 + (n - L) * L
        nj = -(-L // (n // p))
        tiles += sum(min(I + 1, nj) for I in range(p))
    assert c["pairs_needed"] == [2 * expect] * 3
    assert c["tiles_executed"] == 2 * tiles
    f = orc.counts(batch=len(lens), n=n, n_heads=2, p=p, scheme=orc.FULL, lens=lens)
    assert f["pairs_needed"][0] == 2 * int(sum(n * min(int(L), n) for L in lens))


def test_padded_workload_lengths():
    w = inputs.WORKLOADS["padded"]
    lens = inputs.draw_lengths(w)
    assert lens.shape == (32,) and lens.min() >= 64 and lens.max() <= 2048
    c = orc.counts(batch=w.batch, n=w.n, n_heads=1, p=w.p, scheme=orc.CAUSAL, lens=lens)
    closed = sum(int(L) * (int(L) + 1) // 2 + (w.n - int(L)) * int(L) for L in lens)
    assert c["pairs_needed"][0] == closed


@pytest.mark.parametrize("lens", [[0], [1], [5], [16], [40], [3, 16, 9, 0]])
def test_counts_when_padded_rows_are_left_out(lens):
    """Queries past the key length out as well: a len x len problem per batch item."""
    n, p = 16, 4
    lens = np.array(lens, dtype=np.int32)
    Ls = [int(min(L, n)) for L in lens]
    c = orc.counts(batch=len(lens), n=n, n_heads=2, p=p, scheme=orc.CAUSAL, lens=lens, skip_padded_rows=True)
    assert c["pairs_needed"] == [2 * sum(L * (L + 1) // 2 for L in Ls)] * 3
    T = [-(-L // (n // p)) for L in Ls]
    assert c["tiles_executed"] == 2 * sum(t * (t + 1) // 2 for t in T)
    f = orc.counts(batch=len(lens), n=n, n_heads=2, p=p, scheme=orc.FULL, lens=lens, skip_padded_rows=True)
    assert f["pairs_needed"] == [2 * sum(L * L for L in Ls)] * 3
    assert f["tiles_executed"] == 2 * sum(t * t for t in T)
    # without key lengths the switch changes nothing
    assert orc.counts(batch=2, n=n, n_heads=1, p=p, scheme=orc.CAUSAL, skip_padded_rows=True) == \
        orc.counts(batch=2, n=n, n_heads=1, p=p, scheme=orc.CAUSAL)


def test_padded_workload_strict_count():
    w = inputs.WORKLOADS["padded"]
    lens = inputs.draw_lengths(w)
    c = orc.counts(batch=w.batch, n=w.n, n_heads=1, p=w.p, scheme=orc.CAUSAL, lens=lens, skip_padded_rows=True)
    assert c["pairs_needed"][0] == sum(int(L) * (int(L) + 1) // 2 for L in lens) == 31887155


def test_bad_partition_rejected():
    with pytest.raises(orc.OracleError) as e:
        orc.counts(batch=1, n=10, n_heads=1, p=4, scheme=orc.FULL)
    assert e.value.code == 2


def _golden_rows():
    rows = []
    with open(GOLDEN) as f:
        for line in f:
            line = line.strip()
            if line and not line.startswith("#"):
                rows.append(tuple(int(t) for t in line.split()))
    return rows


@pytest.mark.parametrize("n,m,algo,cycles", _golden_rows())
def test_ring_cycles_match_tables(n, m, algo, cycles):
    assert orc.ring_cycles(n, m, algo) == cycles


@pytest.mark.parametrize("n,m,algo,cycles", [r for r in _golden_rows() if r[0] <= 64])
def test_cycles_agree_with_operation_counts(n, m, algo, cycles):
    """With n = d and one operation per PE per cycle, Algo.1's cycles are its
    operations over m (Sec. 3.2); Algo.3 runs phases 1 and 3 on row groups of n
    slots (Sec. 5.2) and phase 2 on all n^2 slots, twice."""
    d = n
    if algo == 1:
        c = orc.counts(batch=1, n=n, n_heads=1, p=m, scheme=orc.FULL)
        ops = d * c["pairs_needed"][0] + 2 * c["pairs_needed"][1] + d * c["pairs_needed"][2]
        assert ops == cycles * m
    else:
        c = orc.counts(batch=1, n=n, n_heads=1, p=m, scheme=orc.CAUSAL)
        groups = (n + 1) // 2 if n % 2 else n // 2 + 1
        assert groups * n >= c["pairs_needed"][0] > (groups - 1) * n
        assert (2 * d * groups * n + 2 * n * n) == cycles * m

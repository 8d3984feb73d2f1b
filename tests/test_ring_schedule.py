"""The paper's ring schedules (Algorithms 1 and 3), enumerated from their index formulas: every
needed multiply-accumulate exactly once, hand-over to the next PE, no operand pair twice in a
cycle, and the cycle counts of Tables 1 and 2."""
from collections import Counter

import pytest

from oracle import attn_oracle as orc
from oracle import ring_schedule as rs

SHAPES = [(4, 2), (6, 3), (6, 2), (5, 5), (8, 4), (9, 3), (7, 1), (12, 4)]


@pytest.mark.parametrize("n,m", SHAPES)
def test_baseline_covers_every_product_once(n, m):
    seen = Counter((a, b, c) for _, _, a, b, c in rs.baseline_phase1(n, m))
    assert len(seen) == n ** 3 and set(seen.values()) == {1}
    assert all(1 <= x <= n for key in seen for x in key)
    pairs = Counter((a, b) for _, _, a, b in rs.baseline_phase2(n, m))
    assert len(pairs) == n * n and set(pairs.values()) == {1}


@pytest.mark.parametrize("n,m", SHAPES + [(15, 5), (15, 15)])
def test_symmetric_computes_one_of_every_pair(n, m):
    """Sec. 4.1 / 4.2: n(n+1)/2 scores computed for odd n; for even n the diagonal n/2 is computed
    from both sides, n(n+2)/2 in all."""
    seen = Counter((min(a, b), max(a, b), c) for _, _, a, b, c in rs.symmetric_phase1(n, m))
    assert set(seen) == {(a, b, c) for a in range(1, n + 1) for b in range(a, n + 1) for c in range(1, n + 1)}
    twice = {(a, b) for (a, b, _), k in seen.items() if k == 2}
    assert set(seen.values()) <= {1, 2}
    assert twice == ({(a, a + n // 2) for a in range(1, n // 2 + 1)} if n % 2 == 0 else set())
    computed = sum(seen.values()) // n
    ref = orc.counts(batch=1, n=n, n_heads=1, p=m, scheme=orc.SYMMETRIC)
    assert computed == ref["pairs_scheduled"][0] == (n * (n + 1) // 2 if n % 2 else n * (n + 2) // 2)
    assert len(seen) // n == ref["pairs_needed"][0]


@pytest.mark.parametrize("n,m,printed", [(3, 3, 21), (4, 4, 36)])
def test_symmetric_cycles_where_no_reuse_transfer_is_needed(n, m, printed):
    """Table 1, Algo.2: the two rows whose stages all have h % m <= 1 need no extra transfer cycle,
    and the computing cycles alone give the printed numbers."""
    total = rs.cycles(rs.symmetric_phase1(n, m)) + 2 * (n // m) * n + rs.cycles(rs.baseline_phase1(n, m))
    assert total == printed


@pytest.mark.parametrize("n,m", SHAPES)
def test_masked_covers_the_lower_triangle_once(n, m):
    seen = Counter((a, b, c) for _, _, a, b, c in rs.masked_phase1(n, m) if a)
    need = {(a, b, c) for a in range(1, n + 1) for b in range(1, a + 1) for c in range(1, n + 1)}
    assert set(seen) == need and set(seen.values()) == {1}          # n(n+1)/2 weights (Sec. 5.1), n products each
    slots = list(rs.masked_phase2(n, m))
    assert len(slots) == n * n                                       # phase 2 keeps every slot (Sec. 5.2)
    pairs = Counter((a, b) for _, _, a, b in slots if a)
    assert set(pairs) == {(a, b) for a, b, _ in need} and set(pairs.values()) == {1}


@pytest.mark.parametrize("n,m", SHAPES)
def test_printed_row_index_of_masked_phase2_misses_row_n(n, m):
    pairs = Counter((a, b) for _, _, a, b in rs.masked_phase2(n, m, as_printed=True) if b)
    want = {(a, b) for a in range(1, n) for b in range(1, a + 1)}
    assert {k for k in pairs if k[0] >= 1} == want and all(a != n for a, _ in pairs)


@pytest.mark.parametrize("n,m", SHAPES)
def test_partial_sums_move_to_the_next_pe(n, m):
    """Within a stage, what PE l accumulates at one step is what PE l+1 accumulates at the next
    (same row, same key): the transfer the algorithms end every cycle with."""
    for stream in (rs.baseline_phase1(n, m), rs.masked_phase1(n, m)):
        by_slot = {}
        for cyc, l, a, b, _ in stream:
            if a:
                by_slot[(cyc, l)] = (a, b)
        steps = n  # steps per sweep
        for (cyc, l), ab in by_slot.items():
            if cyc % steps == 0:
                continue  # last step of a sweep: the sum is complete
            nxt = by_slot.get((cyc + 1, l % m + 1))
            if nxt is not None and ab[0] == nxt[0]:
                assert nxt == ab


@pytest.mark.parametrize("n,m", SHAPES)
def test_no_operand_pair_twice_in_a_cycle(n, m):
    for stream in (rs.baseline_phase1(n, m), rs.masked_phase1(n, m), rs.symmetric_phase1(n, m)):
        per_cycle = Counter((cyc, a, b, c) for cyc, _, a, b, c in stream if a)
        assert set(per_cycle.values()) == {1}


@pytest.mark.parametrize("n,m", SHAPES + [(16, 4), (16, 8)])
def test_cycle_counts_agree_with_the_closed_form(n, m):
    base = 2 * rs.cycles(rs.baseline_phase1(n, m)) + 2 * (n // m) * n        # phases 1 and 3, two passes of phase 2
    assert base == orc.ring_cycles(n, m, 1)
    masked = 2 * rs.cycles(rs.masked_phase1(n, m)) + 2 * (n // m) * n
    assert masked == orc.ring_cycles(n, m, 3)
    assert rs.cycles(rs.baseline_phase2(n, m)) == (n // m) * n


def test_partition_count_must_divide():
    with pytest.raises(ValueError):
        list(rs.baseline_phase1(6, 4))

"""Pins for the oracle's partition-search tools (Sec. 4.2): facts the paper prints, brute force,
closed forms and invariants."""
import itertools
import math
import os

import pytest

from oracle import kvra_oracle as orc

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "partition_search_examples.txt")


def _golden():
    rows = {}
    with open(GOLDEN) as f:
        for line in f:
            if line.strip() and not line.startswith("#"):
                key, *vals = line.split()
                rows[key] = [int(x) for x in vals]
    return rows


def _affine_cost(a, b, e):
    return lambda prefix, c: a + b * c + e * c * (2 * prefix + c)


def test_stride_schedule_matches_the_papers_example():
    fx = _golden()
    C = fx["example_context"][0]
    p = len(fx["example_start"]) - 1
    assert orc.grid_search_strides(C, p, 2) == fx["example_strides"]
    # the text calls the same example "4 processes": the schedule is the same
    assert orc.grid_search_strides(C, 4, 2) == fx["example_strides"]
    # halving down to the granularity, first stride below half an even chunk
    for C, p, g in [(16384, 8, 64), (4096, 4, 64), (8192, 2, 128), (640, 5, 64)]:
        s = orc.grid_search_strides(C, p, g)
        assert s[-1] == g and all(a == 2 * b for a, b in zip(s, s[1:]))
        assert 2 * s[0] < C / p or s == [g]
        assert 4 * s[0] >= C / p or s == [g]


def test_predicted_ratios_in_the_paper_form_a_partition():
    # the one interpolated partitioning the paper prints must be a convex blend of partitions:
    # positive parts that add up to the whole
    r = _golden()["predicted_10k_ratios_x1000"]
    assert sum(r) == 1000 and all(x > 0 for x in r)
    # and the oracle reproduces it from any two entries whose ratio vectors average to it
    C, g = 10000, 1
    ratios = [x / 1000 for x in r]
    cum = [0.0] + list(itertools.accumulate(ratios))
    delta = [0.0, 0.02, 0.01, -0.01, 0.0]
    lo = [int(round(8000 * (cum[k] + delta[k]))) for k in range(5)]
    hi = [int(round(12000 * (cum[k] - delta[k]))) for k in range(5)]
    got = orc.interpolate_partition(C, g, 8000, lo, 12000, hi)
    assert got == [int(round(C * x)) for x in cum]


def test_grid_search_level_is_the_exhaustive_minimum_over_its_lattice():
    # one level, re-derived here by hand-rolled loops for 3 chunks
    C, p, g = 1536, 3, 64
    cost = _affine_cost(3.0, 0.01, 1e-5)
    start = orc.equal_split(C, p, g)
    strides = orc.grid_search_strides(C, p, g)
    _, _, levels = orc.hierarchical_grid_search(C, p, g, cost)
    assert [s for s, _ in levels] == strides
    centre = start
    for stride, after in levels:
        best = None
        for o1 in (-2, -1, 0, 1, 2):
            for o2 in (-2, -1, 0, 1, 2):
                b = [0, centre[1] + o1 * stride, centre[2] + o2 * stride, C]
                if not (0 < b[1] < b[2] < C):
                    continue
                m = max(cost(b[i], b[i + 1] - b[i]) for i in range(3))
                if best is None or (m, b) < best:
                    best = (m, b)
        assert after == best[1]
        centre = after


@pytest.mark.parametrize("C,p,g", [(96, 3, 2), (96, 4, 2), (1024, 4, 64), (2048, 5, 64), (4096, 8, 64)])
def test_grid_search_never_loses_to_its_start_and_stays_on_the_grid(C, p, g):
    for cost in (orc.analytic_cost, _affine_cost(5.0, 0.02, 3e-6)):
        for start in (None, orc.sqrt_rule(C, p, g)):
            b, m, _ = orc.hierarchical_grid_search(C, p, g, cost, start=start)
            s = start or orc.equal_split(C, p, g)
            assert m <= orc.makespan(s, cost)
            assert m == orc.makespan(b, cost)
            assert b[0] == 0 and b[-1] == C and all(x % g == 0 for x in b)
            assert all(b[i] < b[i + 1] for i in range(p))


@pytest.mark.parametrize("C,p,g", [(96, 3, 2), (512, 3, 32), (768, 4, 64)])
def test_grid_search_seeded_near_the_optimum_finds_the_brute_force_makespan(C, p, g):
    # with the closed-form point as seed the exact optimum lies inside the scanned lattice
    want_b, want = orc.brute_force_balance(C, p, g)
    b, m, _ = orc.hierarchical_grid_search(C, p, g, start=orc.sqrt_rule(C, p, g))
    assert m == want


def test_two_way_scan_against_closed_form_and_brute_force():
    # equal analytic cost of both parts: b^2 = C^2 - b^2  ->  b = C / sqrt(2)
    for C, g in [(16384, 64), (4096, 64), (1000, 1)]:
        b, m = orc.two_way_scan(C, g)
        assert abs(b[1] - C / math.sqrt(2)) <= g
        assert (b, m) == orc.brute_force_balance(C, 2, g)


def test_interpolation_invariants():
    g = 64
    for p in (2, 4, 8):
        lo_len, hi_len = 8192, 12288
        lo, hi = orc.sqrt_rule(lo_len, p, g), orc.equal_split(hi_len, p, g)
        # at an entry's own length the entry comes back
        assert orc.interpolate_partition(lo_len, g, lo_len, lo, hi_len, hi) == lo
        assert orc.interpolate_partition(hi_len, g, lo_len, lo, hi_len, hi) == hi
        # two entries with the same ratios predict those ratios at any length
        same = orc.interpolate_partition(10240, g, lo_len, orc.equal_split(lo_len, p, g), hi_len, hi)
        assert same == orc.equal_split(10240, p, g)
        # in between: every cumulative ratio lies between those of the two entries (up to rounding)
        mid = orc.interpolate_partition(10240, g, lo_len, lo, hi_len, hi)
        for k in range(1, p):
            r = mid[k] / 10240
            a, b = sorted((lo[k] / lo_len, hi[k] / hi_len))
            assert a - g / 10240 <= r <= b + g / 10240
        # outside the table's range the nearer entry's ratios are used
        below = orc.interpolate_partition(4096, g, lo_len, lo, hi_len, hi)
        assert below == [g * int(math.floor(x / lo_len * 4096 / g + 0.5)) for x in lo]


def test_interpolation_repairs_collisions():
    # ratios so close that rounding collapses two boundaries: pushed apart by one granule each
    b = orc.interpolate_partition(256, 64, 10000, [0, 10, 20, 9000, 10000], 10000, [0, 10, 20, 9000, 10000])
    assert b == [0, 64, 128, 192, 256]
    b = orc.interpolate_partition(256, 64, 10000, [0, 9970, 9980, 9990, 10000], 10000, [0, 9970, 9980, 9990, 10000])
    assert b == [0, 64, 128, 192, 256]


def test_lookup_picks_the_bracketing_entries():
    g, p = 64, 4
    table = {L: orc.sqrt_rule(L, p, g) for L in (4096, 8192, 12288, 16384)}
    assert orc.lookup_partition(8192, g, table) == table[8192]
    want = orc.interpolate_partition(10240, g, 8192, table[8192], 12288, table[12288])
    assert orc.lookup_partition(10240, g, table) == want
    assert orc.lookup_partition(2048, g, table) == orc.interpolate_partition(2048, g, 4096, table[4096], 4096, table[4096])
    assert orc.lookup_partition(20480, g, table) == orc.interpolate_partition(20480, g, 16384, table[16384], 16384, table[16384])

"""Pins for the oracle's work model and load-balancing objective: the paper's worked example,
its equations, closed forms and brute force."""
import math
import os

import numpy as np
import pytest

from oracle import kvra_oracle as orc

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def _toy():
    rows = {}
    with open(os.path.join(GOLDEN, "toy_9tokens_3procs.txt")) as f:
        for line in f:
            if line.strip() and not line.startswith("#"):
                key, *vals = line.split()
                rows[key] = [int(x) for x in vals]
    return rows


def test_paper_toy_example_dot_products_and_traffic():
    fx = _toy()
    C, p = fx["context"][0], fx["procs"][0]
    sizes = fx["kvr_partition"]
    bounds = [0] + list(np.cumsum(sizes))
    assert bounds[-1] == C
    assert orc.rect_dot_products(bounds) == fx["kvr_dot_products"]
    assert max(orc.rect_dot_products(bounds)) == fx["kvr_max_dot_products"][0]
    assert orc.tsp_dot_products(C, p) == fx["tsp_dot_products_each"] * p
    assert orc.kvr_traffic_entries(bounds) == fx["kvr_traffic_entries"][0]
    assert orc.tsp_traffic_entries(C, p) == fx["tsp_traffic_entries"][0]


@pytest.mark.parametrize("sizes", [[4, 3, 2], [3, 3, 3], [1, 1, 1, 1], [7], [5, 3, 2, 1]])
def test_rectangle_total_matches_eq1(sizes):
    # Eq. 1 numerator: sum_i c_i (prefix_i + c_i) = C^2/2 + sum c_i^2 / 2
    bounds = [0] + list(np.cumsum(sizes))
    C = bounds[-1]
    assert 2 * sum(orc.rect_dot_products(bounds)) == C * C + sum(c * c for c in sizes)


def test_traffic_matches_eq3_to_eq6_for_even_split():
    # Net_tsp = (p-1) C, Net_kvr = (p-1) C / 2 rows of K and of V each
    for C, p in [(12, 3), (64, 4), (4096, 8)]:
        bounds = [k * C // p for k in range(p + 1)]
        assert orc.tsp_traffic_entries(C, p) == 2 * (p - 1) * C
        assert orc.kvr_traffic_entries(bounds) == (p - 1) * C


def test_useful_pairs_sum_to_the_triangle_for_any_partition():
    for sizes in ([4, 3, 2], [160, 96], [1] * 9, [5824, 2368, 1856]):
        bounds = [0] + list(np.cumsum(sizes))
        C = bounds[-1]
        total = sum(orc.useful_pairs(bounds[i], sizes[i]) for i in range(len(sizes)))
        assert total == C * (C + 1) // 2
    assert orc.useful_flops(0, 3, 2, 64) == 4 * 64 * 2 * 6


def test_useful_pairs_counts_the_mask():
    w = orc.attention_weights(np.ones((5, 2)), np.ones((12, 2)), 1.0, first_pos=7)
    assert int((w > 0).sum()) == orc.useful_pairs(7, 5)


def test_lower_bound_ratio_eq2():
    assert orc.ttft_lower_bound_ratio(1) == 1.0
    assert orc.ttft_lower_bound_ratio(2) == 0.375
    # Eq. 1 with equal chunks: (C^2/2 + p (C/p)^2 / 2) / p, relative to C^2
    for p in (2, 4, 8):
        C = 1024.0
        eq1 = (0.5 * C * C + 0.5 * p * (C / p) ** 2) / p
        assert abs(eq1 / (C * C) - orc.ttft_lower_bound_ratio(p)) < 1e-15


def test_analytic_cost_is_twice_the_area_under_the_diagonal():
    for prefix, c in [(0, 4), (4, 3), (7, 2), (160, 96)]:
        assert orc.analytic_cost(prefix, c) == (prefix + c) ** 2 - prefix ** 2
    # the BASELINE configs: sqrt rule reproduces the published boundary lists
    assert orc.sqrt_rule(16384, 8, 64) == [0, 5824, 8192, 10048, 11584, 12928, 14208, 15296, 16384]
    assert orc.sqrt_rule(8192, 4, 64) == [0, 4096, 5824, 7104, 8192]
    assert orc.sqrt_rule(32768, 8, 64) == [0, 11584, 16384, 20096, 23168, 25920, 28352, 30656, 32768]


def test_makespan_and_equal_split():
    assert orc.equal_split(4096, 4, 64) == [0, 1024, 2048, 3072, 4096]
    assert orc.equal_split(256, 3, 64) == [0, 64, 192, 256] or orc.equal_split(256, 3, 64) == [0, 128, 192, 256]
    b = [0, 4, 7, 9]
    assert orc.makespan(b) == max(16.0, 49.0 - 16.0, 81.0 - 49.0)
    # equal split: last chunk dominates, ratio to the mean is (2p-1)/p
    C, p = 4096, 8
    eq = orc.equal_split(C, p, 64)
    assert orc.makespan(eq) / (C * C / p) == (2 * p - 1) / p


@pytest.mark.parametrize("C,p,g", [(96, 3, 8), (128, 4, 8), (64, 2, 1), (60, 3, 4), (24, 4, 1)])
def test_brute_force_properties(C, p, g):
    b, m = orc.brute_force_balance(C, p, g)
    assert b[0] == 0 and b[-1] == C and all(b[i] < b[i + 1] for i in range(p)) and all(x % g == 0 for x in b)
    assert m == orc.makespan(b)
    assert m >= C * C / p                      # cannot beat the mean
    assert m <= orc.makespan(orc.equal_split(C, p, g)) or C // g < 2 * p
    sizes = orc.chunk_lengths(b)
    assert all(sizes[i] >= sizes[i + 1] for i in range(p - 1))   # earlier processes take more (Sec. 5)
    # closed form: continuous optimum is b_k = C sqrt(k/p); the grid optimum cannot be better,
    # and the rounded closed form cannot be better than the grid optimum
    assert m <= orc.makespan(orc.sqrt_rule(C, p, g)) if len(set(orc.sqrt_rule(C, p, g))) == p + 1 else True


def test_two_chunks_split_at_c_over_sqrt2():
    b, _ = orc.brute_force_balance(4096, 2, 1)
    assert abs(b[1] - 4096 / math.sqrt(2)) <= 1.0


def test_brute_force_with_custom_cost_and_ties():
    # constant cost: every partition ties -> lexicographically smallest boundaries
    b, m = orc.brute_force_balance(40, 3, 8, cost=lambda prefix, c: 1.0)
    assert b == [0, 8, 16, 40] and m == 1.0
    # cost linear in chunk length: optimum is the even split
    b, m = orc.brute_force_balance(48, 3, 8, cost=lambda prefix, c: float(c))
    assert b == [0, 16, 32, 48] and m == 16.0

"""Pins of the oracle's chain timing (time to first token when every process waits, layer by
layer, for the KV-cache of its precedent: Sec. 4 overview, Fig. 5(b)) against cases that can be
worked out by hand, and of the library's kvra_chain_ttft against the oracle."""
import random

import pytest

from oracle import kvra_oracle as orc


def const(table):
    """cost(prefix, c) looked up by the chunk's start."""
    return lambda prefix, c: table[prefix]


B3 = [0, 4, 7, 9]          # the paper's 9-token example partition {4, 3, 2}


def test_single_layer_is_the_slowest_append_then_the_last_attention():
    a = {0: 5.0, 4: 2.0, 7: 1.0}
    t = {0: 3.0, 4: 8.0, 7: 4.0}
    # caches complete at 5, max(2, 5) = 5, max(1, 5) = 5; the last process then attends for 4
    assert orc.chain_ttft(B3, 1, const(a), const(t)) == 5.0 + 4.0
    a = {0: 1.0, 4: 2.0, 7: 6.0}
    assert orc.chain_ttft(B3, 1, const(a), const(t)) == 6.0 + 4.0


def test_one_process_and_identical_processes_never_wait():
    assert orc.chain_ttft([0, 9], 7, lambda p, c: 2.0, lambda p, c: 3.0) == 7 * 5.0
    assert orc.chain_ttft(B3, 5, lambda p, c: 2.0, lambda p, c: 3.0) == 5 * 5.0
    # no work before the attention: a cache is complete as soon as its process enters the layer,
    # so process 1 (8 per layer) has layer l ready at 8 l, the last process (4 per layer) waits for
    # that in every layer and leaves the sixth layer at 8 * 5 + 4
    t = {0: 3.0, 4: 8.0, 7: 4.0}
    assert orc.chain_ttft(B3, 6, lambda p, c: 0.0, const(t)) == 8.0 * 5 + 4.0
    # the other way round the last process is the slow one and never waits
    t = {0: 3.0, 4: 4.0, 7: 8.0}
    assert orc.chain_ttft(B3, 6, lambda p, c: 0.0, const(t)) == 6 * 8.0


def test_two_processes_two_layers_by_hand():
    a0, a1, t0, t1, x0 = 3.0, 1.0, 2.0, 7.0, 0.5
    a, t, x = {0: a0, 5: a1}, {0: t0, 5: t1}, {0: x0, 5: 99.0}   # the last process hands nothing on
    cache00 = a0
    done00 = cache00 + t0
    cache10 = max(a1, cache00 + x0)
    done10 = cache10 + t1
    cache01 = done00 + a0
    cache11 = max(done10 + a1, cache01 + x0)
    want = cache11 + t1
    assert orc.chain_ttft([0, 5, 8], 2, const(a), const(t), const(x)) == want
    # a slow link (20): the first cache arrives at 3 + 20 = 23, the second process leaves layer 0 at
    # 30 and has its own rows in at 31, after the second cache has arrived (3 + 2 + 3 + 20 = 28)
    x = {0: 20.0, 5: 0.0}
    assert orc.chain_ttft([0, 5, 8], 2, const(a), const(t), const(x)) == 38.0


def test_a_slow_early_process_sets_the_pace_of_everyone_behind_it():
    # only process 0 has work before the attention: its cache of layer l is complete at (l + 1) A
    A, L = 4.0, 9
    a = {0: A, 4: 0.0, 7: 0.0}
    assert orc.chain_ttft(B3, L, const(a), lambda p, c: 0.0) == L * A
    # only process 0 attends: its cache of layer l is complete at l T, and nobody waits for its
    # last attention ("layer misalignment": the later processes run one attention behind)
    T = 5.0
    t = {0: T, 4: 0.0, 7: 0.0}
    assert orc.chain_ttft(B3, L, lambda p, c: 0.0, const(t)) == (L - 1) * T


def test_long_run_rate_is_the_slowest_process():
    rng = random.Random(11)
    for _ in range(20):
        a = {s: rng.randint(0, 9) for s in B3[:-1]}
        t = {s: rng.randint(1, 9) for s in B3[:-1]}
        per_layer = max(a[s] + t[s] for s in a)
        t100 = orc.chain_ttft(B3, 100, const(a), const(t))
        t200 = orc.chain_ttft(B3, 200, const(a), const(t))
        assert t200 - t100 == 100 * per_layer
        assert t100 >= 100 * (a[7] + t[7])                     # the last process does all its own work
        assert t100 <= 100 * per_layer + sum(a.values())       # and lags the slowest by a bounded start-up


def test_more_cost_never_gives_an_earlier_token():
    rng = random.Random(12)
    for _ in range(50):
        a = {s: rng.random() for s in B3[:-1]}
        t = {s: rng.random() for s in B3[:-1]}
        x = {s: rng.random() for s in B3[:-1]}
        L = rng.randint(1, 6)
        base = orc.chain_ttft(B3, L, const(a), const(t), const(x))
        for table in (a, t, x):
            s = rng.choice(B3[:-1])
            old = table[s]
            table[s] = old + rng.random()
            assert orc.chain_ttft(B3, L, const(a), const(t), const(x)) >= base
            table[s] = old


def test_library_agrees_with_the_oracle():
    from paper_2405_05329_amd import kvra
    rng = random.Random(13)
    for _ in range(40):
        p = rng.randint(1, 6)
        cuts = sorted(rng.sample(range(1, 40), p - 1))
        b = [0] + cuts + [40]
        a = lambda prefix, c: 0.01 * c + 0.3
        t = lambda prefix, c: 1e-3 * c * (2 * prefix + c)
        x = (lambda prefix, c: 0.02 * (prefix + c)) if rng.random() < 0.5 else None
        L = rng.randint(1, 40)
        assert kvra.kvra_chain_ttft(b, L, a, t, x) == orc.chain_ttft(b, L, a, t, x)
    with pytest.raises(kvra.KvraError):
        kvra.kvra_chain_ttft([0, 4, 4], 2, lambda p, c: 1.0, lambda p, c: 1.0)
    with pytest.raises(kvra.KvraError):
        kvra.kvra_chain_ttft([0, 4], 0, lambda p, c: 1.0, lambda p, c: 1.0)
    with pytest.raises(kvra.KvraError):
        kvra.kvra_chain_ttft([0, 4], 1, lambda p, c: -1.0, lambda p, c: 1.0)

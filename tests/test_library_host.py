"""Host-side checks that run without a GPU: the shared library loads, exports every symbol the
header declares, rejects bad arguments before touching the device, and kvra_balance agrees with
the oracle's exhaustive search."""
import ctypes
import os
import random
import re

import numpy as np
import pytest

from oracle import kvra_oracle as orc
from paper_2405_05329_amd import kvra

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared_symbols():
    text = open(os.path.join(ROOT, "include", "kvra.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(kvra_[a-z_0-9]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    names = _declared_symbols()
    assert {"kvra_append_kv", "kvra_chunk_attn", "kvra_balance", "kvra_strerror"} <= set(names)
    lib = ctypes.CDLL(kvra.LIB_PATH)
    for name in names:
        assert hasattr(lib, name), name
    assert kvra.kvra_version() >= 100


def test_binding_has_the_same_names():
    for name in _declared_symbols():
        assert callable(getattr(kvra, name)), name


def test_strerror():
    assert kvra.kvra_strerror(0) == "ok"
    for code in (-1, -2, -3, -4, -5, -99):
        assert kvra.kvra_strerror(code)


def test_append_rejects_bad_arguments_before_any_launch():
    P = 0x1000  # never dereferenced: validation fails first
    ok = dict(k_in=P, v_in=P, q_inout=P, k_cache=P, v_cache=P, prefix_len=0, chunk_len=4, capacity=8,
              n_q_heads=4, n_kv_heads=2, head_dim=64, rope_base=10000.0, check=False)
    def call(**kw):
        a = dict(ok); a.update(kw)
        return kvra.kvra_append_kv(**a)
    assert call(k_in=None) == kvra.KVRA_EINVAL
    assert call(v_cache=None) == kvra.KVRA_EINVAL
    assert call(chunk_len=0) == kvra.KVRA_EINVAL
    assert call(prefix_len=-1) == kvra.KVRA_EINVAL
    assert call(n_q_heads=3) == kvra.KVRA_EINVAL
    assert call(n_kv_heads=0) == kvra.KVRA_EINVAL
    assert call(head_dim=96) == kvra.KVRA_EUNSUPPORTED
    assert call(prefix_len=5, chunk_len=4, capacity=8) == kvra.KVRA_ERANGE
    assert call(rope_base=float("nan")) == kvra.KVRA_EINVAL
    with pytest.raises(kvra.KvraError):
        a = dict(ok); a.update(check=True, chunk_len=0)
        kvra.kvra_append_kv(**a)


def test_attn_rejects_bad_arguments_before_any_launch():
    P = 0x1000
    ok = dict(q=P, k_cache=P, v_cache=P, prefix_len=0, chunk_len=4, n_q_heads=4, n_kv_heads=2,
              head_dim=128, scale=0.1, out=P, check=False)
    def call(**kw):
        a = dict(ok); a.update(kw)
        return kvra.kvra_chunk_attn(**a)
    assert call(q=None) == kvra.KVRA_EINVAL
    assert call(out=None) == kvra.KVRA_EINVAL
    assert call(chunk_len=0) == kvra.KVRA_EINVAL
    assert call(prefix_len=-3) == kvra.KVRA_EINVAL
    assert call(n_q_heads=5) == kvra.KVRA_EINVAL
    assert call(head_dim=80) == kvra.KVRA_EUNSUPPORTED
    assert call(scale=float("nan")) == kvra.KVRA_EINVAL
    assert call(scale=float("inf")) == kvra.KVRA_EINVAL
    assert call(scale=0.0) == kvra.KVRA_EINVAL


def test_balance_argument_checks():
    for args in [(100, 0, 4), (100, 2, 0), (100, 2, 3), (8, 3, 4), (0, 1, 1)]:
        with pytest.raises(kvra.KvraError):
            kvra.kvra_balance(*args)
    with pytest.raises(kvra.KvraError):
        kvra.kvra_balance(64, 2, 8, cost=lambda p, c: float("nan"))
    with pytest.raises(kvra.KvraError):
        kvra.kvra_makespan([1, 5, 9])
    with pytest.raises(kvra.KvraError):
        kvra.kvra_makespan([0, 5, 5])


def test_balance_single_chunk_and_full_grid():
    assert kvra.kvra_balance(4096, 1, 64) == ([0, 4096], 4096.0 ** 2)
    b, m = kvra.kvra_balance(8, 8, 1)
    assert b == list(range(9)) and m == 15.0


@pytest.mark.parametrize("C,p,g", [(96, 3, 8), (128, 4, 8), (64, 2, 1), (60, 3, 4), (24, 4, 1), (40, 3, 8)])
def test_balance_equals_exhaustive_search_analytic(C, p, g):
    want_b, want_m = orc.brute_force_balance(C, p, g)
    got_b, got_m = kvra.kvra_balance(C, p, g)
    assert got_b == want_b          # boundaries bit-exact, ties broken the same way
    assert got_m == want_m
    assert kvra.kvra_makespan(got_b) == orc.makespan(got_b)


@pytest.mark.parametrize("seed", [0, 1, 2, 3])
def test_balance_equals_exhaustive_search_arbitrary_costs(seed):
    rnd = random.Random(seed)
    table = {}
    def cost(prefix, c):
        # deterministic, non-monotone, many ties
        if (prefix, c) not in table:
            table[(prefix, c)] = rnd.choice([1.0, 2.0, 3.0, 5.0]) * c + 0.25 * prefix
        return table[(prefix, c)]
    for C, p, g in [(48, 3, 4), (36, 4, 3), (20, 2, 1), (30, 5, 2)]:
        want_b, want_m = orc.brute_force_balance(C, p, g, cost)
        got_b, got_m = kvra.kvra_balance(C, p, g, cost)
        assert got_m == want_m
        assert got_b == want_b
        assert kvra.kvra_makespan(got_b, cost) == want_m


def test_balance_closed_form_and_bounds():
    # analytic cost on a fine grid: optimum sits at C sqrt(k/p) (two chunks: C / sqrt 2)
    b, m = kvra.kvra_balance(4096, 2, 1)
    assert abs(b[1] - 4096 / 2 ** 0.5) <= 1
    for C, p, g in [(16384, 8, 64), (8192, 4, 64), (32768, 8, 64)]:
        b, m = kvra.kvra_balance(C, p, g)
        sq = orc.sqrt_rule(C, p, g)
        assert m <= orc.makespan(sq)                 # exact search is at least as good as the rounded rule
        assert m >= C * C / p                        # and cannot beat the mean
        assert all(abs(x - y) <= 2 * g for x, y in zip(b, sq))
        sizes = orc.chunk_lengths(b)
        assert all(sizes[i] >= sizes[i + 1] - g for i in range(p - 1))
        eq = kvra.kvra_equal_split(C, p, g)
        assert eq == orc.equal_split(C, p, g)
        assert kvra.kvra_makespan(eq) / (C * C / p) == (2 * p - 1) / p
        # lower bound of Eq. 2 is for whole rectangles; the trapezoid model's bound is the mean
        assert m / (C * C) < 1.06 / p


def test_equal_split_matches_oracle_rounding():
    for C, p, g in [(256, 3, 64), (4096, 4, 64), (960, 7, 64), (100, 3, 1)]:
        assert kvra.kvra_equal_split(C, p, g) == orc.equal_split(C, p, g)


# ---------------------------------------------------------------- partition search tools (Sec. 4.2)
def _table_cost(seed):
    rnd = random.Random(seed)
    table = {}
    def cost(prefix, c):
        if (prefix, c) not in table:
            table[(prefix, c)] = rnd.choice([1.0, 2.0, 3.0, 5.0]) * c + 0.25 * prefix
        return table[(prefix, c)]
    return cost


@pytest.mark.parametrize("C,p,g", [(96, 3, 2), (96, 4, 2), (1024, 4, 64), (2048, 5, 64), (4096, 8, 64), (640, 5, 64),
                                   (16384, 8, 64)])
def test_grid_search_equals_the_oracles_literal_enumeration(C, p, g):
    cases = [(None, None), (orc.analytic_cost, None), (lambda pr, c: 4.0 + 0.02 * c + 3e-6 * c * (2 * pr + c), None),
             (orc.analytic_cost, orc.sqrt_rule(C, p, g))]
    if p <= 5:
        cases += [(_table_cost(7), None), (_table_cost(8), orc.sqrt_rule(C, p, g))]   # non-monotone, many ties
    for cost, start in cases:
        want_b, want_m, _ = orc.hierarchical_grid_search(C, p, g, cost or orc.analytic_cost, start=start)
        got_b, got_m, evals = kvra.kvra_search_grid(C, p, g, cost, start=start)
        assert got_b == want_b
        assert got_m == want_m
        # memoised per level: at most 25 chunk costs per chunk and level, far below 5^(p-1) * p
        levels = len(orc.grid_search_strides(C, p, g))
        assert evals <= p + levels * 25 * p


def test_grid_search_argument_checks():
    with pytest.raises(kvra.KvraError):
        kvra.kvra_search_grid(100, 4, 64)                       # not on the grid
    with pytest.raises(kvra.KvraError):
        kvra.kvra_search_grid(256, 4, 64, start=[0, 64, 64, 192, 256])   # not strictly rising
    with pytest.raises(kvra.KvraError):
        kvra.kvra_search_grid(256, 4, 64, start=[0, 64, 100, 192, 256])  # off the grid
    with pytest.raises(kvra.KvraError):
        kvra.kvra_search_grid(256, 4, 64, start=[0, 64, 128, 192, 320])  # wrong total
    with pytest.raises(kvra.KvraError):
        kvra.kvra_search_grid(256, 4, 64, cost=lambda pr, c: float("nan"))
    b, m, _ = kvra.kvra_search_grid(256, 4, 64)                 # nowhere to move: stays put
    assert b == [0, 64, 128, 192, 256]
    b, m, _ = kvra.kvra_search_grid(640, 1, 64)
    assert b == [0, 640] and m == orc.analytic_cost(0, 640)


@pytest.mark.parametrize("C,g", [(16384, 64), (4096, 64), (1000, 1), (128, 64), (192, 64)])
def test_two_way_search_equals_full_scan_for_monotone_costs(C, g):
    for cost in (None, lambda pr, c: 4.0 + 0.02 * c + 3e-6 * c * (2 * pr + c), lambda pr, c: float(c)):
        want_b, want_m = orc.two_way_scan(C, g, cost or orc.analytic_cost)
        got_b, got_m, evals = kvra.kvra_search_two_way(C, g, cost)
        assert got_b == want_b and got_m == want_m
        assert evals <= 2 * (C // g).bit_length() + 6           # logarithmic, not a scan
    with pytest.raises(kvra.KvraError):
        kvra.kvra_search_two_way(64, 64)
    with pytest.raises(kvra.KvraError):
        kvra.kvra_search_two_way(200, 64)


def test_interpolate_and_table_predict_equal_the_oracle():
    rnd = random.Random(3)
    g = 64
    for p in (2, 4, 8):
        lens = [4096, 8192, 12288, 16384]
        table = {}
        for L in lens:
            cuts = sorted(rnd.sample(range(1, L // g), p - 1))
            table[L] = [0] + [g * x for x in cuts] + [L]
        for C in (2048, 4096, 6144, 10240, 14336, 16384, 20480, 8192 + 64, 12288 - 64):
            assert kvra.kvra_table_predict(C, g, table) == orc.lookup_partition(C, g, table)
        assert kvra.kvra_interpolate(10240, g, 8192, table[8192], 12288, table[12288]) == \
            orc.interpolate_partition(10240, g, 8192, table[8192], 12288, table[12288])
    # collisions are repaired the same way
    assert kvra.kvra_interpolate(256, 64, 10000, [0, 10, 20, 9000, 10000], 10000, [0, 10, 20, 9000, 10000]) == \
        [0, 64, 128, 192, 256]
    with pytest.raises(kvra.KvraError):
        kvra.kvra_interpolate(1024, 64, 8192, [0, 4096, 8192], 4096, [0, 2048, 4096])   # len_hi < len_lo
    with pytest.raises(kvra.KvraError):
        kvra.kvra_interpolate(1024, 64, 4096, [0, 4096, 4096], 8192, [0, 2048, 8192])   # not rising
    with pytest.raises(kvra.KvraError):
        kvra.kvra_interpolate(1000, 64, 4096, [0, 2048, 4096], 8192, [0, 2048, 8192])   # off the grid


# ---------------------------------------------------------------- decoder layer: checks that need no GPU
def _layer(**over):
    f = dict(hidden=4096, ffn=11008, n_q_heads=32, n_kv_heads=32, head_dim=128, rms_eps=1e-6, rope_base=10000.0,
             scale=128 ** -0.5, norm1=256, wqkv=256, wo=256, norm2=256, w_gate=256, w_up=256, w_down=256)
    f.update(over)
    return kvra.make_layer(**f)


def test_layer_workspace_size_and_checks():
    L = _layer()
    c = 1000
    # h, q, k, v, attention output, x2 [c, 4096] and the MLP activation [c, 11008], bf16, 256-byte aligned
    want = 6 * c * 4096 * 2 + c * 11008 * 2
    got = kvra.kvra_layer_workspace_bytes(L, c)
    assert want <= got <= want + 7 * 256
    gqa = _layer(n_kv_heads=8)
    assert kvra.kvra_layer_workspace_bytes(gqa, c) < got
    for bad in (_layer(hidden=4100), _layer(ffn=11000), _layer(head_dim=96), _layer(n_kv_heads=5),
                _layer(scale=0.0), _layer(rms_eps=-1.0), _layer(wo=None), _layer(hidden=16384)):
        with pytest.raises(kvra.KvraError):
            kvra.kvra_layer_workspace_bytes(bad, c)
    with pytest.raises(kvra.KvraError):
        kvra.kvra_layer_workspace_bytes(L, 0)


def test_layer_and_linear_reject_bad_arguments_before_any_launch():
    L = _layer()
    p = 256   # fake, never dereferenced: every call below is refused by the argument checks
    nbytes = kvra.kvra_layer_workspace_bytes(L, 64)
    with pytest.raises(kvra.KvraError) as e:
        kvra.kvra_layer_chunk(L, p, p, p, p, 0, 64, 64, p, nbytes - 1)        # workspace too small
    assert e.value.code == kvra.KVRA_EINVAL
    with pytest.raises(kvra.KvraError):
        kvra.kvra_layer_chunk(L, p, p, p, p, 0, 64, 64, p + 8, nbytes)        # workspace misaligned
    with pytest.raises(kvra.KvraError) as e:
        kvra.kvra_layer_chunk(L, p, p, p, p, 10, 64, 64, p, nbytes)           # past the cache capacity
    assert e.value.code == kvra.KVRA_ERANGE
    with pytest.raises(kvra.KvraError):
        kvra.kvra_layer_chunk(L, None, p, p, p, 0, 64, 64, p, nbytes)
    with pytest.raises(kvra.KvraError) as e:
        kvra.kvra_linear(p, p, None, None, p, 8, 100, 64)                     # n not a multiple of 32
    assert e.value.code == kvra.KVRA_EUNSUPPORTED
    with pytest.raises(kvra.KvraError):
        kvra.kvra_linear(p, p, None, None, p, 8, 64, 100)                     # k not a multiple of 64
    with pytest.raises(kvra.KvraError) as e:
        kvra.kvra_linear(p, p, p, p, p, 8, 64, 64)                            # gate/up together with residual
    assert e.value.code == kvra.KVRA_EINVAL
    with pytest.raises(kvra.KvraError):
        kvra.kvra_linear(p, p, None, None, p, 1 << 20, 64, 4096)              # activation matrix beyond 4 GiB
    with pytest.raises(kvra.KvraError):
        kvra.kvra_qkv_proj(p, p, p, p, p, 8, 32, 5, 128, 4096)                # heads not divisible
    with pytest.raises(kvra.KvraError):
        kvra.kvra_rms_norm(p, p, p, 4, 100, 1e-6)                             # hidden not a multiple of 8
    with pytest.raises(kvra.KvraError):
        kvra.kvra_rms_norm(p, None, p, 4, 64, 1e-6)


# ------------------------------------------------------------------ launch plan of kvra_chunk_attn
PIECE_ALLOWANCE = 8     # tile steps the plan charges per piece for starting and finishing it


def _unit_steps(prefix, c, G, rows_per_tile, key_tile, qt):
    row_hi = min((qt + 1) * rows_per_tile, c * G)
    return (prefix + (row_hi - 1) // G) // key_tile + 1


def _check_schedule(prefix, c, H, Hkv, d, cus):
    """Every (kv head, row tile) unit is covered exactly once by the pieces of the plan; partial pieces of a
    unit share one counter, have distinct scratch slots inside the declared scratch, and are exactly the
    pieces its merge reads; no workgroup beyond groups * slots; piece lengths respect the minimum."""
    p = kvra.kvra_chunk_attn_plan(prefix, c, H, Hkv, d, cus)
    pieces = kvra.kvra_chunk_attn_pieces(prefix, c, H, Hkv, d, cus)
    G = H // Hkv
    rows = c * G
    assert p["rows_per_tile"] % 32 == 0 and 32 <= p["rows_per_tile"] <= 256
    assert p["row_tiles"] * p["rows_per_tile"] >= rows > (p["row_tiles"] - 1) * p["rows_per_tile"]
    assert p["key_tile"] == (128 if d == 64 else 64)
    assert p["groups"] in (1, 8) and p["groups"] * p["slots"] <= max(cus, 1) and p["slots"] <= 256
    assert p["units"] * p["groups"] == p["row_tiles"] * Hkv
    covered = {}
    slots, per_wg = set(), {}
    partial = 0
    for pc in pieces:
        assert 0 <= pc["workgroup"] < p["groups"] * p["slots"]
        n = _unit_steps(prefix, c, G, p["rows_per_tile"], p["key_tile"], pc["row_tile"])
        assert pc["unit_steps"] == n and 0 <= pc["jt0"] < pc["jt1"] <= n
        covered.setdefault((pc["kv_head"], pc["row_tile"]), []).append(pc)
        per_wg[pc["workgroup"]] = per_wg.get(pc["workgroup"], 0) + (pc["jt1"] - pc["jt0"]) + PIECE_ALLOWANCE
        whole = pc["jt0"] == 0 and pc["jt1"] == n
        assert whole == (pc["slot"] < 0) == (pc["counter"] < 0)
        if not whole:
            partial += 1
            assert pc["slot"] not in slots and 0 <= pc["slot"] * 8 * (4 * 16 + 2) * 64 * 4 < p["scratch_bytes"]
            slots.add(pc["slot"])
            assert pc["in_merge_list"] == 1 and 0 <= pc["counter"] < 8 * 256
    assert partial == p["partial_pieces"]
    assert (partial == 0) == (p["scratch_bytes"] == 0)
    assert len(covered) == p["row_tiles"] * Hkv
    counters = set()
    for (g, qt), pcs in covered.items():
        pcs.sort(key=lambda r: r["jt0"])
        assert pcs[0]["jt0"] == 0 and pcs[-1]["jt1"] == pcs[0]["unit_steps"]
        assert all(a["jt1"] == b["jt0"] for a, b in zip(pcs[:-1], pcs[1:]))
        if len(pcs) > 1:
            assert all(r["merge_pieces"] == len(pcs) for r in pcs)
            assert len({r["counter"] for r in pcs}) == 1 and pcs[0]["counter"] not in counters
            counters.add(pcs[0]["counter"])
            assert min(r["jt1"] - r["jt0"] for r in pcs) >= 8
    assert max(per_wg.values()) <= p["steps_per_slot"] + 8
    return p, pieces, per_wg


def test_attention_schedule_of_the_16k_workload():
    """Llama-7B shape, 8 balanced chunks, 256 compute units: 8 groups of 32 slots, and every slot's load (tile
    steps plus the allowance per piece) within a few steps of the ideal share of its group."""
    H, d, cus = 32, 128, 256
    bounds = [0, 5824, 8192, 10048, 11584, 12928, 14208, 15296, 16384]
    want = {0: (23, 256, 92, 2, 0), 1: (10, 256, 40, 1, 0), 2: (8, 256, 32, 1, 8), 3: (6, 256, 24, 0, 24),
            4: (6, 224, 24, 0, 24), 5: (5, 256, 20, 0, 20), 6: (5, 224, 20, 0, 20), 7: (5, 224, 20, 0, 20)}
    for i, (tiles, rows, units, rounds, cut) in want.items():
        prefix, c = bounds[i], bounds[i + 1] - bounds[i]
        p, pieces, per_wg = _check_schedule(prefix, c, H, H, d, cus)
        assert (p["row_tiles"], p["rows_per_tile"], p["units"], p["rounds"], p["cut_units"]) == (tiles, rows, units, rounds, cut)
        assert (p["groups"], p["slots"]) == (8, 32)
        total = sum(pc["jt1"] - pc["jt0"] for pc in pieces)
        ideal = total / 256
        # no idle compute unit, but for the free slots of a group that fit no gang (gang mode, below)
        heads_left = 4 - p["gangs"] * p["gang_heads"]           # heads whose tails go to the free slots outside the gangs
        idle = 8 * (p["slots"] - p["units"] - p["gangs"] * p["row_tiles"]) if p["gangs"] and heads_left == 0 else 0
        assert len(per_wg) == 256 - idle and (i >= 3) == (p["gangs"] > 0)
        assert max(per_wg.values()) <= 1.08 * ideal + 3 * PIECE_ALLOWANCE   # allowances included
        if not p["gangs"]:                                           # (a gang slot carries whole tails, short ones too)
            assert sorted(per_wg.values())[8] >= 0.9 * ideal           # (the last slot of a group takes what is left)


def test_gang_mode_runs_the_tails_of_a_head_in_step():
    """Chunks 5-7 of the 16k workload: 20 units on the 32 slots of a group, 12 free slots = 2 gangs of 5 (one
    slot per row tile) + 2 idle.  Every unit is cut once; a gang slot runs the tails of one row tile of two
    heads, and the five slots of a gang are on the same head at the same position of their lists."""
    H, d, cus = 32, 128, 256
    for prefix, c in ((12928, 1280), (14208, 1088), (15296, 1088)):
        p, pieces, per_wg = _check_schedule(prefix, c, H, H, d, cus)
        assert (p["gangs"], p["gang_heads"], p["row_tiles"], p["units"], p["cut_units"], p["segments"]) == (2, 2, 5, 20, 20, 20)
        assert p["partial_pieces"] == 2 * 20 * 8 and len(pieces) == 2 * 20 * 8
        by_wg = {}
        for pc in pieces:
            by_wg.setdefault(pc["workgroup"], []).append(pc)
        for x in range(8):                                   # group x = workgroup id % 8, slot = id // 8
            heads = [by_wg[x + 8 * slot] for slot in range(20)]
            assert all(len(h) == 1 and h[0]["jt0"] == 0 and h[0]["jt1"] == p["head_steps"] for h in heads)
            for gang in range(2):
                members = [by_wg[x + 8 * (20 + gang * 5 + r)] for r in range(5)]
                assert all(len(m) == 2 for m in members)
                assert sorted(m[0]["row_tile"] for m in members) == [0, 1, 2, 3, 4]
                for m in members:
                    assert m[0]["row_tile"] == m[1]["row_tile"] and m[0]["kv_head"] != m[1]["kv_head"]
                    assert all(t["jt0"] == p["head_steps"] and t["jt1"] == t["unit_steps"] for t in m)
                for position in range(2):
                    assert len({m[position]["kv_head"] for m in members}) == 1
            assert all(x + 8 * slot not in by_wg for slot in (30, 31))
    # chunks 3 and 4: 24 units, 8 free slots for 6 row tiles: one gang runs three heads, the two free slots
    # left over share the six tails of the fourth head (three whole tails each), nobody idles
    for prefix, c in ((10048, 1536), (11584, 1344)):
        p, pieces, per_wg = _check_schedule(prefix, c, H, H, d, cus)
        assert (p["gangs"], p["gang_heads"], p["row_tiles"], p["units"], p["cut_units"]) == (1, 3, 6, 24, 24)
        assert len(per_wg) == 256 and p["partial_pieces"] == 2 * 24 * 8
        by_wg = {}
        for pc in pieces:
            by_wg.setdefault(pc["workgroup"], []).append(pc)
        for x in range(8):
            members = [by_wg[x + 8 * (24 + r)] for r in range(6)]
            assert all(len(m) == 3 and len({t["row_tile"] for t in m}) == 1 for m in members)
            for position in range(3):
                assert len({m[position]["kv_head"] for m in members}) == 1
            spare = [by_wg[x + 8 * 30], by_wg[x + 8 * 31]]
            assert all(len(m) == 3 and len({t["kv_head"] for t in m}) == 1 for m in spare)
            assert spare[0][0]["kv_head"] == spare[1][0]["kv_head"] not in {t["kv_head"] for m in members for t in m}
            assert sorted(t["row_tile"] for m in spare for t in m) == [0, 1, 2, 3, 4, 5]


def test_attention_schedule_invariants_on_random_shapes():
    rng = random.Random(5)
    for _ in range(250):
        H, Hkv, d = rng.choice([(32, 32, 128), (32, 8, 128), (32, 1, 128), (71, 1, 64), (16, 16, 64), (6, 3, 128)])
        prefix = rng.choice([0, 1, 63, 500, 4096, 30000])
        c = rng.choice([1, 7, 64, 300, 1088, 2500])
        cus = rng.choice([1, 8, 64, 256, 304])
        _check_schedule(prefix, c, H, Hkv, d, cus)


def test_attention_schedule_of_decode_like_and_short_shapes():
    # a few tokens behind a long prefix: one unit per head, cut so that every compute unit gets a piece
    p, pieces, per_wg = _check_schedule(20000, 8, 32, 32, 128, 256)
    assert (p["row_tiles"], p["rows_per_tile"], p["units"], p["rounds"], p["cut_units"]) == (1, 32, 4, 0, 4)
    assert len(per_wg) == 256 and max(per_wg.values()) <= 313 * 32 / 256 + 3 * PIECE_ALLOWANCE + 8
    # too few key tiles to cut anything: whole units
    p, pieces, _ = _check_schedule(100, 8, 32, 32, 128, 256)
    assert p["partial_pieces"] == 0 and p["scratch_bytes"] == 0 and len(pieces) == 32
    # the first chunk of the 4k context in four equal chunks: 128 units on 256 compute units
    p, pieces, per_wg = _check_schedule(0, 1024, 32, 32, 128, 256)
    assert p["units"] == 16 and p["cut_units"] == 4 and max(per_wg.values()) < 16 + PIECE_ALLOWANCE   # 16: the longest unit whole
    # grouped queries fold into the row index; head_dim 64 walks 128-key tiles; one group when the kv heads
    # cannot be dealt to eight
    p, pieces, _ = _check_schedule(0, 4096, 71, 1, 64, 256)
    assert p["key_tile"] == 128 and p["row_tiles"] == (4096 * 71 + 255) // 256 and (p["groups"], p["slots"]) == (1, 256)


def test_noalloc_scratch_holds_every_plan_of_a_256_cu_device_and_not_every_plan_of_a_larger_one():
    """kvra_chunk_attn_noalloc refuses (KVRA_ESCRATCH) a launch whose plan needs more partial-result
    slots than its fixed array holds.  That array is sized for three slots per CU of a 256-CU device:
    no plan for 256 CUs exceeds it, while a hypothetical 512-CU device has plans that do."""
    cap = kvra.kvra_chunk_attn_noalloc_scratch_bytes()
    assert cap == 768 * 8 * (4 * 16 + 2) * 64 * 4
    rng = np.random.default_rng(3)
    worst = {256: 0, 512: 0}
    for _ in range(400):
        d = int(rng.choice([64, 128]))
        hkv = int(rng.choice([1, 2, 8, 32]))
        g = int(rng.choice([1, 4, 8]))
        prefix = int(rng.integers(0, 40000))
        c = int(rng.integers(1, 6000))
        for cus in worst:
            plan = kvra.kvra_chunk_attn_plan(prefix, c, hkv * g, hkv, d, cus)
            worst[cus] = max(worst[cus], plan["scratch_bytes"])
    assert 0 < worst[256] <= cap < worst[512]


def test_attention_launch_plan_rejects_bad_arguments():
    with pytest.raises(kvra.KvraError):
        kvra.kvra_chunk_attn_plan(0, 0, 4, 4, 64, 256)
    with pytest.raises(kvra.KvraError):
        kvra.kvra_chunk_attn_plan(0, 8, 4, 3, 64, 256)
    with pytest.raises(kvra.KvraError):
        kvra.kvra_chunk_attn_plan(0, 8, 4, 4, 96, 256)
    with pytest.raises(kvra.KvraError):
        kvra.kvra_chunk_attn_plan(0, 8, 4, 4, 64, 0)


# ------------------------------------------------------------------ grid search on a caller's objective
def test_grid_search_on_the_makespan_objective_is_the_plain_grid_search():
    rng = random.Random(21)
    for _ in range(12):
        p = rng.randint(2, 5)
        g = rng.choice([1, 2, 4])
        C = g * rng.randint(8 * p, 30 * p)
        cost = lambda prefix, c: c * (2 * prefix + c) + 40.0 * c
        want_b, want_m, _ = kvra.kvra_search_grid(C, p, g, cost)
        got_b, got_m, evals = kvra.kvra_search_grid_objective(C, p, g, lambda b: orc.makespan(b, cost))
        assert (got_b, got_m) == (want_b, want_m)
        ob, om, _ = orc.hierarchical_grid_search(C, p, g, objective=lambda b: orc.makespan(b, cost))
        assert (got_b, got_m) == (ob, om)
        assert evals <= 1 + len(orc.grid_search_strides(C, p, g)) * 5 ** (p - 1)


def test_grid_search_on_the_chain_ttft_matches_the_oracle_and_never_loses_to_its_start():
    rng = random.Random(22)
    for _ in range(10):
        p = rng.randint(2, 4)
        g = rng.choice([2, 4, 8])
        C = g * rng.randint(8 * p, 24 * p)
        L = rng.randint(1, 12)
        before = lambda prefix, c: 0.5 + 0.05 * c
        attend = lambda prefix, c: 1e-3 * c * (2 * prefix + c)
        send = lambda prefix, c: 0.01 * (prefix + c)
        ttft = lambda b: orc.chain_ttft(b, L, before, attend, send)
        start = orc.sqrt_rule(C, p, g) if rng.random() < 0.5 else None
        if start is not None and any(start[i + 1] <= start[i] for i in range(p)):
            start = None
        got_b, got_v, _ = kvra.kvra_search_grid_objective(C, p, g, ttft, start=start)
        want_b, want_v, _ = orc.hierarchical_grid_search(C, p, g, start=start, objective=ttft)
        assert got_b == want_b and got_v == want_v
        assert got_v == ttft(got_b)
        assert got_v <= ttft(start if start is not None else orc.equal_split(C, p, g))


def test_grid_search_objective_rejects_bad_arguments():
    with pytest.raises(kvra.KvraError):
        kvra.kvra_search_grid_objective(1100, 11, 1, lambda b: 0.0)           # 5^10 combinations per level
    with pytest.raises(kvra.KvraError):
        kvra.kvra_search_grid_objective(96, 3, 5, lambda b: 0.0)              # not on the grid
    with pytest.raises(kvra.KvraError):
        kvra.kvra_search_grid_objective(96, 3, 4, lambda b: float("nan"))
    with pytest.raises(kvra.KvraError):
        kvra.kvra_search_grid_objective(96, 3, 4, lambda b: 0.0, start=[0, 30, 64, 96])   # start off the grid


def test_header_is_plain_c_and_a_c_program_can_call_the_host_entry_points(tmp_path):
    """The boundary is a C ABI: the header compiles as C99, and a C program linked against the
    library gets the same partition as the Python binding."""
    import shutil
    import subprocess
    gcc = shutil.which("gcc")
    if gcc is None:
        pytest.skip("no C compiler")
    header_dir = os.path.join(ROOT, "include")
    subprocess.run([gcc, "-std=c99", "-Wall", "-Wextra", "-pedantic", "-Werror", "-fsyntax-only", "-x", "c",
                    os.path.join(header_dir, "kvra.h")], check=True)
    src = tmp_path / "host.c"
    src.write_text(
        '#include <stdio.h>\n#include "kvra.h"\n'
        "int main(void) {\n"
        "  int64_t b[9]; double m = 0; kvra_attn_plan plan;\n"
        "  if (kvra_balance(16384, 8, 64, NULL, NULL, b, &m) != KVRA_OK) return 1;\n"
        "  if (kvra_chunk_attn_plan(b[7], b[8] - b[7], 32, 32, 128, 256, &plan) != KVRA_OK) return 2;\n"
        '  for (int k = 0; k < 9; ++k) printf("%lld ", (long long)b[k]);\n'
        '  printf("| %d %d %d %s\\n", plan.slots, plan.head_steps, plan.segments, kvra_strerror(KVRA_ERANGE));\n'
        "  return 0;\n}\n")
    exe = tmp_path / "host"
    lib_dir = os.path.dirname(kvra.LIB_PATH)
    subprocess.run([gcc, "-std=c99", "-I", header_dir, str(src), "-o", str(exe), "-L", lib_dir, "-l:libkvra.so",
                    "-Wl,-rpath," + lib_dir, "-Wl,--allow-shlib-undefined"], check=True)
    out = subprocess.run([str(exe)], check=True, capture_output=True, text=True).stdout
    bounds, rest = out.split("|")
    want_b = kvra.kvra_balance(16384, 8, 64)[0]
    assert [int(x) for x in bounds.split()] == want_b
    plan = kvra.kvra_chunk_attn_plan(want_b[7], want_b[8] - want_b[7], 32, 32, 128, 256)
    assert [int(x) for x in rest.split()[:3]] == [plan["slots"], plan["head_steps"], plan["segments"]]

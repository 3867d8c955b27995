"""Pins of oracle/tiling.py (Sec. III-A to III-C: expressions as trees, statement placement and
hoisting for deep and flat tilings, Rules 1-4).  CPU only.

The trip counts are pinned by a brute force that shares nothing with the closed form: the
expression is run as the loop nest it denotes, every memory statement beside its compute
statement (the default association), and a statement is counted only when the tile it names
(for a compute statement: the loop indices related to it) differs from that of its previous
execution."""
import itertools
import json
import os
import random

import pytest

from oracle import perf_model as pm
from oracle import tiling as tl

G = json.load(open(os.path.join(os.path.dirname(__file__), "golden", "paper_numbers.json")))


def run_nest(expr, extents, block_loops=""):
    """Executes the loop nest: returns, per statement, how often it ran and how often the tile it
    touches (and the block it runs in) changed from one execution to the next."""
    tree = tl.parse(expr)
    chains = tl.chains(tree)
    where = {}                                   # compute statement -> loop whose body holds it
    for comp, related in pm.COMPUTE_LOOPS.items():
        chain = next(c for c in chains if set(related) <= set(c))
        where["C_" + comp] = max(related, key=chain.index)
    state, runs, changes, last = {}, {}, {}, {}

    def execute(stmt, key):
        runs[stmt] = runs.get(stmt, 0) + 1
        if last.get(stmt) != key:
            changes[stmt] = changes.get(stmt, 0) + 1
            last[stmt] = key

    def body(node):
        loop, children = node
        for i in range(extents[loop]):
            state[loop] = i
            for child in children:
                body(child)
            for comp_stmt, at in where.items():
                if at != loop:
                    continue
                execute(comp_stmt, tuple(state[l] for l in pm.COMPUTE_LOOPS[comp_stmt[2]]))
                for mem, (tensor, comp) in pm.MEM_STATEMENTS.items():
                    if "C_" + comp == comp_stmt:
                        execute(mem, tuple(state[l] for l in pm.TENSOR_LOOPS[tensor] + block_loops))
        del state[loop]
    body(tree)
    return runs, changes


def test_expressions_and_parser():
    ex = tl.expressions()
    assert len(ex) == G["deep_tilings"]["value"] + G["flat_tilings"]["value"] == 26 and len(set(ex)) == 26
    assert tl.parse("mhnk") == ("m", [("h", [("n", [("k", [])])])])
    assert tl.parse("mn(k,h)") == ("m", [("n", [("k", []), ("h", [])])])
    assert tl.chains(tl.parse("nm(k,h)")) == [("n", "m", "k"), ("n", "m", "h")]
    assert tl.bound_form("mnkh") == tl.bound_form("hmnk") == "mhnk" and tl.bound_form("nm(k,h)") == "mn(k,h)"
    for e in ex:                                  # every expression holds each loop once
        assert sorted(c for c in e if c in "mnkh") == list("hkmn")


@pytest.mark.parametrize("seed", range(6))
def test_trips_equal_the_executed_loop_nest(seed):
    rng = random.Random(seed)
    for expr in tl.expressions():
        ext = {l: rng.choice((1, 1, 2, 3)) for l in "mnkh"}
        runs, changes = run_nest(expr, ext)
        for s in tl.STATEMENTS:
            assert tl.trips(expr, s, ext, hoist=False, drop_unit_loops=False) == runs[s], (expr, s, ext)
            # (a compute statement is counted the same way: it runs again when a loop related to it
            # moves on, so that one whose loops are all dead leaves the loops around it)
            assert tl.trips(expr, s, ext) == changes[s], (expr, s, ext)
        # the same once Rule 1 has bound m (and h) to the block index: the bound loops run outermost
        # and nothing leaves them, a block loads what it uses itself
        grid, bound = tl.bound_form(expr), tl.bound_loops(expr)
        runs, changes = run_nest(grid, ext, block_loops=bound)
        for s in ("L_A", "L_B", "L_D", "S_E"):
            assert tl.trips(grid, s, ext, block_loops=bound) == changes[s], (expr, s, ext)


def test_deep_tilings_agree_with_the_permutation_form():
    ext = {"m": 3, "n": 2, "k": 1, "h": 4}
    for expr in pm.deep_tilings():
        for s in tl.STATEMENTS:
            for kw in ({}, {"hoist": False}, {"drop_unit_loops": False}, {"block_loops": "mh"}):
                assert tl.trips(expr, s, ext, **kw) == pm.trips(expr, s, ext, **kw)


def test_flat_tiling_is_the_one_form_that_computes_nothing_twice():
    """Sec. III-A: the reason flat tilings are in the space.  C_C is needed once per (m, n, k) and
    C_E once per (m, n, h); a deep tiling nests h and k, so one of the two runs under both."""
    ext = {"m": 2, "n": 3, "k": 4, "h": 5}
    least = ext["m"] * ext["n"] * ext["k"], ext["m"] * ext["n"] * ext["h"]
    for expr in tl.expressions():
        got = tl.trips(expr, "C_C", ext), tl.trips(expr, "C_E", ext)
        assert (got == least) == ("(" in expr), expr
        assert got[0] >= least[0] and got[1] >= least[1]
    # mn(k,h) against mhnk: C is computed h times less often; E is written once per n instead of once
    assert tl.trips("mhnk", "C_C", ext) == ext["h"] * tl.trips("mn(k,h)", "C_C", ext)
    assert tl.trips("mn(k,h)", "S_E", ext) == ext["n"] * tl.trips("mhnk", "S_E", ext)
    # with T_H = H the two coincide statement by statement
    ext1 = dict(ext, h=1)
    for s in tl.STATEMENTS:
        assert tl.trips("mn(k,h)", s, ext1) == tl.trips("mhnk", s, ext1)


def test_rule1_and_rule2():
    for expr, sub in G["rule1_example"]["value"].items():
        assert tl.sub_expression(expr) == sub
    classes = tl.rule1_classes()
    assert sum(len(v) for v in classes.values()) == 26
    # every deep tiling falls to nk or kn by the order of its n and k; both flat ones to n(k,h)
    for expr in pm.deep_tilings():
        assert tl.sub_expression(expr) == ("nk" if expr.index("n") < expr.index("k") else "kn")
    assert sorted(classes) == ["kn", "n(k,h)", "nk"] and len(classes["nk"]) == len(classes["kn"]) == 12
    assert classes["n(k,h)"] == ["mn(k,h)", "nm(k,h)"]
    verdict = {s: ("pruned" if tl.violates_rule2(s) else "kept") for s in classes}
    for sub, v in G["rule2_example"]["value"].items():
        assert verdict[sub] == v
    assert verdict["n(k,h)"] == "kept"
    # the reading's counts; the paper's sentence says 26 -> 5 -> 3 (not reproduced, see oracle/tiling.py)
    assert [26, len(classes), sum(v == "kept" for v in verdict.values())] == [26, 3, 2]
    assert G["expression_counts_after_rules"]["value"] == [26, 5, 3]


def test_space_sizes_of_the_example():
    c = tl.count_space(1024, 1024, 512, 512, elem_bytes=2, shm_max_bytes=160 * 1024)
    assert c["candidates"] == G["n_candidates_M1024_N1024_K512_H512"]["value"]
    assert c["tile_choices"] == 64 * 64 * 32 * 32 and c["after_rule3"] == 7 * 7 * 6 * 6
    assert 1 - c["after_rule3"] / c["tile_choices"] >= G["rule3_discard_fraction_min"]["value"]
    # Rule 4 by hand for two combinations on either side of 1.2 x 160 KiB = 196608 bytes:
    # tiles (128,128,128,128): 5 x 128 x 128 x 2 = 163840 fits; (256,128,128,128): 2 x (3 x 32768 + 2 x 16384) = 262144 does not
    assert pm.shm_estm({"m": 128, "n": 128, "k": 128, "h": 128}) * 2 == 163840
    assert pm.shm_estm({"m": 256, "n": 128, "k": 128, "h": 128}) * 2 == 262144
    brute = sum(1 for t in itertools.product((16, 32, 64, 128, 256, 512, 1024), (16, 32, 64, 128, 256, 512, 1024),
                                             (16, 32, 64, 128, 256, 512), (16, 32, 64, 128, 256, 512))
                if 2 * (t[0] * t[2] + t[2] * t[1] + t[0] * t[1] + t[1] * t[3] + t[0] * t[3]) <= 196608)
    assert c["after_rule4"] == brute
    assert c["candidates_pruned"] == 2 * brute
    # a shape that is not a power of two keeps the padded choices below 5 %
    c2 = tl.count_space(768, 384, 64, 64, elem_bytes=2, shm_max_bytes=160 * 1024)
    assert c2["tile_choices"] == 48 * 24 * 4 * 4
    ok_m = [t for t in range(16, 769, 16) if (-(-768 // t) * t - 768) / 768 < 0.05]
    ok_n = [t for t in range(16, 385, 16) if (-(-384 // t) * t - 384) / 384 < 0.05]
    assert c2["after_rule3"] == len(ok_m) * len(ok_n) * 3 * 3

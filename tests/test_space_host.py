"""The library's search-space entry points (mcf_expression, mcf_expression_trips,
mcf_sub_expression, mcf_enumerate_space; Sec. III-A to III-C) against oracle/tiling.py.
Host only: needs the built library, no GPU."""
import random

import pytest

import mcf_inputs as mi
import paper_2506_22169_amd as mcf
from paper_2506_22169_amd.binding import (MCF_TRIPS_BIND_BLOCK, MCF_TRIPS_KEEP_UNIT_LOOPS, MCF_TRIPS_NO_HOIST, McfError,
                                          make_problem)
from oracle import tiling as tl


def test_the_26_expressions():
    ex = mcf.expressions()
    assert len(ex) == 26 and sorted(ex) == sorted(tl.expressions())
    assert ex[-2:] == ["mn(k,h)", "nm(k,h)"] and all("(" not in e for e in ex[:24])


@pytest.mark.parametrize("seed", range(4))
def test_trips_of_every_expression(seed):
    rng = random.Random(100 + seed)
    for expr in mcf.expressions():
        ext = {l: rng.choice((1, 1, 2, 3, 7)) for l in "mnkh"}
        for flags, kw in ((0, {}), (MCF_TRIPS_NO_HOIST, {"hoist": False}), (MCF_TRIPS_KEEP_UNIT_LOOPS, {"drop_unit_loops": False}),
                          (MCF_TRIPS_NO_HOIST | MCF_TRIPS_KEEP_UNIT_LOOPS, {"hoist": False, "drop_unit_loops": False}),
                          (MCF_TRIPS_BIND_BLOCK, {"block_loops": tl.bound_loops(expr)})):
            got = mcf.expression_trips(expr, ext, flags)
            for s in tl.STATEMENTS:
                assert got[s] == tl.trips(expr, s, ext, **kw), (expr, s, ext, flags)


def test_rule1_and_rule2_per_expression():
    for expr in mcf.expressions():
        sub, kept = mcf.sub_expression(expr)
        assert sub == tl.sub_expression(expr)
        assert kept == (not tl.violates_rule2(sub))


def test_malformed_expressions_are_refused():
    for bad in ("", "mnk", "mnkk", "mnkhh", "mn(k,h", "mn(k;h)", "xnkh", "mn(kh)m", "m(n,k,h"):
        with pytest.raises(McfError):
            mcf.expression_trips(bad, {"m": 1, "n": 1, "k": 1, "h": 1})
    with pytest.raises(McfError):
        mcf.expression_trips("mnkh", {"m": 0, "n": 1, "k": 1, "h": 1})
    # an expression that splits the loops of a compute block over two scopes has no place for it
    with pytest.raises(McfError):
        mcf.expression_trips("m(n,k)h", {"m": 2, "n": 2, "k": 2, "h": 2})


SHAPES = [(1, 1024, 512, 1024, 512, "f16", False, 160 * 1024), (1, 1024, 512, 1024, 512, "f16", False, 48 * 1024),
          (1, 768, 64, 384, 64, "f16", True, 0), (16, 256, 80, 256, 80, "f16", True, 0)]
SHAPES += [(w.batch, w.M, w.K, w.N, w.L, w.dtype, w.softmax, 0) for w in mi.WORKLOADS.values()]


@pytest.mark.parametrize("shape", SHAPES, ids=lambda s: "x".join(str(v) for v in s[:5]))
def test_space_report(shape):
    b, M, K, N, L, dt, sm, shm = shape
    p = make_problem(b, M, K, N, L, dt, b_stride=(N * K, 1, K) if sm else None)
    r = mcf.enumerate_space(p, sm, shm)
    want = tl.count_space(M, N, K, L, elem_bytes=2, shm_max_bytes=shm or 160 * 1024)
    assert (r.n_deep, r.n_flat) == (24, 2) and r.n_deep + r.n_flat == want["expressions"]
    assert r.n_rule1 == want["after_rule1"] and r.n_rule2 == want["after_rule2"]
    subs = r.subs()
    assert sorted(subs) == want["sub_expressions"] and sorted(s for s, (_, k) in subs.items() if k) == want["kept"]
    assert {s: n for s, (n, _) in subs.items()} == {s: len(v) for s, v in tl.rule1_classes().items()}
    for f in ("tile_choices", "after_rule3", "after_rule4", "candidates", "candidates_pruned"):
        assert getattr(r, f) == want[f], f
    # the built kernels as points of the pruned space: recounted from the candidate list
    cands = {(t.tm, t.tn, t.tk, t.tl) for t in mcf.list_candidates(p, sm)}
    lim = 1.2 * (shm or 160 * 1024)
    dims = {"m": M, "n": N, "k": K, "h": L}

    def survives(tm, tn, tk, th):
        tiles = {"m": tm, "n": tn, "k": tk, "h": th}
        return (all(t % 16 == 0 and t <= -(-dims[l] // 16) * 16 and tl.pm.padding_ok(dims[l], t) for l, t in tiles.items())
                and 2 * tl.pm.shm_estm(tiles) <= lim)
    assert r.built_deep == sum(1 for c in cands if survives(*c))
    assert r.built_flat == sum(1 for (tm, tn, tk, tl_) in cands if tl_ == L and survives(tm, tn, tk, 32))
    if (K, L) in ((64, 64), (128, 128), (32, 32)) and M >= 512:
        assert r.built_deep > 0


def test_the_papers_example_sizes():
    p = make_problem(1, 1024, 512, 1024, 512, "f16")
    r = mcf.enumerate_space(p, False, 0)
    assert r.candidates == 109051904 and r.tile_choices == 64 * 64 * 32 * 32
    assert r.after_rule3 == 7 * 7 * 6 * 6 and 1 - r.after_rule3 / r.tile_choices > 0.99

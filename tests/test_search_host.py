"""The library's heuristic search (mcf_search_tiles, Sec. IV-B Alg. 1) against the oracle's, on
the same candidate space, estimates, seed and measurement: the same candidates are measured in
the same order and the search ends in the same generation; the library then returns the fastest
candidate it measured.  Host only: the measurement is a table."""
import ctypes

import pytest

import mcf_inputs as mi
import paper_2506_22169_amd as mcf
from oracle import perf_model as pm
from oracle import search as sr
from paper_2506_22169_amd.binding import make_problem


def _space(w):
    """Feasible candidates in the library's order with the library's estimates (each estimate and
    the membership of the list are checked against the oracle model in test_abi_and_picker)."""
    prob = make_problem(w.batch, w.M, w.K, w.N, w.L, w.dtype, b_stride=(w.N * w.K, 1, w.K) if w.softmax else None)
    tiles = mcf.list_candidates(prob, w.softmax)
    shapes = [(t.mb, t.rg, t.ns, t.nj, t.tl) for t in tiles]
    return prob, shapes, tiles


def _table(shapes, tiles, wobble_seed):
    """A made-up measurement: the estimate distorted by up to +-40 %, fixed per candidate."""
    rng = sr.Uniforms(wobble_seed)
    return {v: t.t_est_s * (0.6 + 0.8 * rng.next()) for v, t in zip(shapes, tiles)}


CASES = [(name, N, n, seed) for name in ("cfg2", "cfg3", "cfg5", "G3", "G6", "S8")
         for (N, n, seed) in ((32, 8, 1), (6, 2, 7), (4, 1, 3), (12, 3, 11))]


@pytest.mark.parametrize("name,N,n,seed", CASES)
def test_library_search_equals_oracle_search(name, N, n, seed):
    w = mi.WORKLOADS[name] if name in mi.WORKLOADS else mi.PAPER_SHAPES[name]
    prob, shapes, tiles = _space(w)
    assert len(shapes) >= 3
    table = _table(shapes, tiles, 100 + seed)
    space = [((mb, rg), (ns, nj), (tl,)) for (mb, rg, ns, nj, tl) in shapes]   # loops m, n, h
    est = [t.t_est_s for t in tiles]
    want = sr.heuristic_search(space, est, lambda c: table[shapes[c]], N=N, n=n, epsilon=0.02, seed=seed,
                               max_generations=16)
    calls = []

    def measure(t):
        calls.append((t.mb, t.rg, t.ns, t.nj, t.tl))
        return table[(t.mb, t.rg, t.ns, t.nj, t.tl)]

    best, rep = mcf.search_tiles(prob, w.softmax, measure, population=N, top_n=n, epsilon=0.02, seed=seed,
                                 max_generations=16)
    assert rep.space == len(shapes)
    assert calls == [shapes[c] for _, c, _, _ in want["log"]]
    got_log = [(e.generation, (e.mb, e.rg, e.ns, e.nj, e.tl), e.t_est_s, e.t_meas_s) for e in rep.entries()]
    assert got_log == [(g, shapes[c], est[c], t) for g, c, _, t in want["log"]]
    assert (rep.generations, bool(rep.converged)) == (want["generations"], want["converged"])
    # The library returns the fastest candidate measured in any generation (first in measurement
    # order among equals); Alg. 1 as printed returns the fastest of the last shortlist when it
    # converges, which is within epsilon of it, and the same candidate otherwise.
    fastest = min(want["log"], key=lambda e: e[3])
    assert (best.mb, best.rg, best.ns, best.nj, best.tl) == shapes[fastest[1]]
    assert rep.best_t_s == fastest[3] and best.t_est_s == est[fastest[1]]
    if want["converged"]:
        assert rep.best_t_s <= want["best_t"] < rep.best_t_s * 1.02 / (1 - 0.02)
    else:
        assert rep.best_t_s == want["best_t"] and fastest[1] == want["best"]


def test_defaults_and_errors():
    w = mi.WORKLOADS["cfg2"]
    prob, shapes, tiles = _space(w)
    # zero parameters read as N = 32, n = 8, epsilon = 0.02, 16 generations
    a = mcf.search_tiles(prob, False, lambda t: t.t_est_s, seed=9)
    b = mcf.search_tiles(prob, False, lambda t: t.t_est_s, population=32, top_n=8, epsilon=0.02, seed=9, max_generations=16)
    assert [(e.mb, e.rg, e.ns, e.nj, e.tl) for e in a[1].entries()] == [(e.mb, e.rg, e.ns, e.nj, e.tl) for e in b[1].entries()]
    assert a[1].measured <= 8 * a[1].generations
    # measurement == model: the result is the picker's estimate
    assert a[0].t_est_s == pytest.approx(mcf.pick_tiles(prob, False).t_est_s, rel=1e-12)
    # a failing measurement ends the search with MCF_ELAUNCH
    with pytest.raises(mcf.McfError) as e:
        mcf.search_tiles(prob, False, lambda t: -1.0)
    assert e.value.status == 4
    with pytest.raises(ZeroDivisionError):
        mcf.search_tiles(prob, False, lambda t: 1 / 0)
    # no kernels for this (K, L)
    with pytest.raises(mcf.McfError) as e:
        mcf.search_tiles(make_problem(1, 512, 48, 512, 48, "f16"), False, lambda t: 1.0)
    assert e.value.status == 2
    lib = mcf.load_library()
    assert lib.mcf_search_tiles(ctypes.byref(prob), 0, None, ctypes.cast(None, mcf.binding.MEASURE_FN), None, None, None) == 1


@pytest.mark.parametrize("KLP,softmax,N,n,seed", [((64, 64, 64), False, 32, 8, 1), ((128, 128, 128), True, 6, 2, 7),
                                                   ((64, 128, 128), False, 12, 3, 11), ((64, 64, 128), True, 4, 1, 3)])
def test_three_gemm_search_equals_oracle_search(KLP, softmax, N, n, seed):
    """mcf_search_tiles3: the same algorithm over the arrangements built for the three-GEMM chain
    (candidates and estimates from mcf_list_candidates3, which the picker test covers)."""
    K, L, P = KLP
    prob = make_problem(8, 1024, K, 1024, L, "f16", b_stride=(1024 * K, 1, K) if softmax else None)
    tiles = mcf.list_candidates3(prob, P, softmax)
    shapes = [(t.mb, t.rg, t.ns, t.nj, t.tl) for t in tiles]
    assert len(shapes) >= 4 and [s[:4] for s in shapes] == [s for s in mcf.list_variants3(prob, P, softmax) if s in [x[:4] for x in shapes]]
    pick = mcf.pick_tiles3(prob, P, softmax)
    assert pick.t_est_s == min(t.t_est_s for t in tiles)
    table = _table(shapes, tiles, 300 + seed)
    space = [((mb, rg), (ns, nj), (tl,)) for (mb, rg, ns, nj, tl) in shapes]
    est = [t.t_est_s for t in tiles]
    want = sr.heuristic_search(space, est, lambda c: table[shapes[c]], N=N, n=n, epsilon=0.02, seed=seed, max_generations=16)
    calls = []

    def measure(t):
        calls.append((t.mb, t.rg, t.ns, t.nj, t.tl))
        return table[(t.mb, t.rg, t.ns, t.nj, t.tl)]

    best, rep = mcf.search_tiles3(prob, P, softmax, measure, population=N, top_n=n, epsilon=0.02, seed=seed, max_generations=16)
    assert rep.space == len(shapes)
    assert calls == [shapes[c] for _, c, _, _ in want["log"]]
    assert (rep.generations, bool(rep.converged)) == (want["generations"], want["converged"])
    fastest = min(want["log"], key=lambda e: e[3])
    assert (best.mb, best.rg, best.ns, best.nj, best.tl) == shapes[fastest[1]] and rep.best_t_s == fastest[3]
    with pytest.raises(mcf.McfError) as e:                       # no three-GEMM kernels for this P
        mcf.search_tiles3(prob, 32, softmax, measure)
    assert e.value.status == 2

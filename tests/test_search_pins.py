"""Pins of the oracle's heuristic search (Sec. IV-B, Alg. 1) to things other than itself: the
published SplitMix64 sequence, a run traced by hand with scripted random numbers, brute force
over the whole space, and the invariants the listing implies."""
import itertools

import pytest

from oracle import search as sr


class Scripted:
    """Hands out a fixed list of uniforms (for the hand-traced run)."""

    def __init__(self, us):
        self.us, self.k = list(us), 0

    def next(self):
        u = self.us[self.k]
        self.k += 1
        return u

    def below(self, n):
        return min(int(self.next() * n), n - 1)


def test_generator_is_splitmix64():
    # First outputs of SplitMix64 seeded with 1234567 (the widely published test sequence);
    # the counter form gives output k as the first output of the generator seeded seed + k*gamma.
    gamma = 0x9E3779B97F4A7C15
    want = [6457827717110365317, 3203168211198807973, 9817491932198370423, 4593380528125082431, 16408922859458223821]
    got = [sr._mix((1234567 + k * gamma) & ((1 << 64) - 1)) for k in range(5)]
    assert got == want
    u = sr.Uniforms(1234567)
    assert u.next() == (want[0] >> 11) / 2.0**53
    assert all(0.0 <= sr.Uniforms(s).next() < 1.0 for s in range(100))


def test_neighbours_differ_in_one_loop_only():
    space = [((1, 4), (1, 1)), ((1, 4), (2, 1)), ((2, 4), (1, 1)), ((2, 2), (2, 1)), ((1, 4), (2, 2))]
    assert sr.neighbours(space, 0, 0) == [2]          # same n entry, other m entry
    assert sr.neighbours(space, 0, 1) == [1, 4]       # same m entry, other n entry
    assert sr.neighbours(space, 3, 0) == [1] and sr.neighbours(space, 3, 1) == []


def test_hand_traced_run():
    """Loops m in {1,2}, n in {1,2}; candidates 0:(m1,n1) 1:(m2,n1) 2:(m1,n2) 3:(m2,n2).
    The model prefers candidate 3, the measurement candidate 1.  N = 3, n = 2.

    gen 0: draws 0.1,0.6,0.3 -> population [0,2,1]; by estimate [1,2,0]; measure 1 (1.5) and
           2 (3.0); top1 = 1; |1.5-1e9|/1e9 ~ 1: go on; best = (1, 1.5).
           weights 1/2,1/3,1/4 (cumulative .5,.8333,1.0833):
             .9*1.0833=.975 -> parent 0, loop .7 -> n, only neighbour 2          -> 2
             .1*1.0833=.108 -> parent 1, loop .2 -> m, only neighbour 0          -> 0
             .5*1.0833=.542 -> parent 2, loop .1 -> m, only neighbour 3          -> 3
    gen 1: population [2,0,3]; by estimate [3,2,0]; measure 3 (2.5); 2 is known (3.0);
           top1 = 3 (2.5); |2.5-1.5|/1.5 = .67: go on; best stays (1, 1.5).
           weights 1,1/3,1/4 (cumulative 1,1.3333,1.5833):
             .5*1.5833=.79  -> parent 3, loop .9 -> n, only neighbour 1          -> 1
             .7*1.5833=1.11 -> parent 2, loop .4 -> m, only neighbour 3          -> 3
             .99*1.5833=1.57 -> parent 0, loop .0 -> m, only neighbour 1         -> 1
    gen 2: population [1,3,1]; by estimate [3,1,1]; distinct top 2 = [3,1], both known;
           top1 = 1 (1.5); difference 0 < epsilon: converged on candidate 1."""
    space = [((1,), (1,)), ((2,), (1,)), ((1,), (2,)), ((2,), (2,))]
    est = [4.0, 2.0, 3.0, 1.0]
    meas = [5.0, 1.5, 3.0, 2.5]
    calls = []

    def measure(c):
        calls.append(c)
        return meas[c]

    us = [0.1, 0.6, 0.3,
          0.9, 0.7, 0.5, 0.1, 0.2, 0.0, 0.5, 0.1, 0.3,
          0.5, 0.9, 0.2, 0.7, 0.4, 0.6, 0.99, 0.0, 0.8]
    rng = Scripted(us)
    r = sr.heuristic_search(space, est, measure, N=3, n=2, epsilon=0.01, seed=0, rng=rng)
    assert calls == [1, 2, 3]
    assert r["log"] == [(0, 1, 2.0, 1.5), (0, 2, 3.0, 3.0), (1, 3, 1.0, 2.5)]
    assert (r["best"], r["best_t"], r["converged"], r["generations"]) == (1, 1.5, True, 3)
    assert rng.k == len(us)      # every scripted number was consumed, none more


def test_hand_traced_parent_weights_and_first_population():
    """A second run traced by hand whose scripted numbers separate the readings that the first
    one cannot: the first population is drawn without repetition (Alg. 1, first statement, as
    read here), and parents are drawn with probability proportional to 1 / estimate (Sec. IV-B,
    mutate paragraph), not to the estimate.  Same space as above: 0:(m1,n1) 1:(m2,n1) 2:(m1,n2)
    3:(m2,n2), estimates 4, 2, 3, 1; measured 5, 1.5, 3, 1.2.  N = 3, n = 2, three generations.

    gen 0: draws .1,.1,.1.  Without repetition: position 0 takes perm[0 + int(.1*4)] = 0,
           position 1 takes perm[1 + int(.1*3)] = 1, position 2 takes perm[2 + int(.1*2)] = 2:
           population [0,1,2]  (with repetition it would be [0,0,0]).
           by estimate [1,2,0]; measure 1 (1.5) and 2 (3.0); top1 = 1; best = (1, 1.5).
           weights 1/2,1/3,1/4, cumulative .5, .8333, 1.0833 (total 1.0833):
             .3*1.0833=.325   -> parent 1 (weights 2,3,4 would give 2.7 -> parent 2);
                                 loop .7 -> n, only neighbour 3                       -> 3
             .6*1.0833=.65    -> parent 2 (weights 2,3,4: 5.4 -> parent 0);
                                 loop .2 -> m, only neighbour 3                       -> 3
             .95*1.0833=1.029 -> parent 0; loop .1 -> m, only neighbour 1             -> 1
    gen 1: population [3,3,1]; by estimate [3,3,1]; distinct top 2 = [3,1]; measure 3 (1.2);
           top1 = 3 (1.2); |1.2-1.5|/1.5 = .2: go on; best = (3, 1.2).
           weights 1,1,1/2, cumulative 1, 2, 2.5:
             .5*2.5=1.25   -> second member, parent 3 (weights 1,1,2: 2.0 -> parent 1);
                              loop .9 -> n, only neighbour 1                          -> 1
             .85*2.5=2.125 -> parent 1; loop .4 -> m, only neighbour 0                -> 0
             .1*2.5=.25    -> parent 3; loop .3 -> m, only neighbour 2                -> 2
    gen 2: population [1,0,2]; by estimate [1,2,0]; top 2 = [1,2], both known; top1 = 1 (1.5);
           |1.5-1.2|/1.2 = .25: no convergence, and 1.5 is not below 1.2: best stays (3, 1.2),
           although candidate 3 is no longer in the population.  Generation bound 3: stop."""
    space = [((1,), (1,)), ((2,), (1,)), ((1,), (2,)), ((2,), (2,))]
    est = [4.0, 2.0, 3.0, 1.0]
    meas = [5.0, 1.5, 3.0, 1.2]
    us = [0.1, 0.1, 0.1,
          0.3, 0.7, 0.0, 0.6, 0.2, 0.0, 0.95, 0.1, 0.0,
          0.5, 0.9, 0.0, 0.85, 0.4, 0.0, 0.1, 0.3, 0.0]
    rng = Scripted(us)
    r = sr.heuristic_search(space, est, lambda c: meas[c], N=3, n=2, epsilon=0.01, seed=0, max_generations=3, rng=rng)
    assert r["populations"] == [[0, 1, 2], [3, 3, 1], [1, 0, 2]]
    assert r["log"] == [(0, 1, 2.0, 1.5), (0, 2, 3.0, 3.0), (1, 3, 1.0, 1.2)]
    assert (r["best"], r["best_t"], r["converged"], r["generations"]) == (3, 1.2, False, 3)
    assert rng.k == len(us)


def test_first_run_populations():
    """The populations of the first hand-traced run, as its docstring derives them."""
    space = [((1,), (1,)), ((2,), (1,)), ((1,), (2,)), ((2,), (2,))]
    us = [0.1, 0.6, 0.3,
          0.9, 0.7, 0.5, 0.1, 0.2, 0.0, 0.5, 0.1, 0.3,
          0.5, 0.9, 0.2, 0.7, 0.4, 0.6, 0.99, 0.0, 0.8]
    r = sr.heuristic_search(space, [4.0, 2.0, 3.0, 1.0], lambda c: [5.0, 1.5, 3.0, 2.5][c], N=3, n=2, epsilon=0.01,
                            seed=0, rng=Scripted(us))
    assert r["populations"] == [[0, 2, 1], [2, 0, 3], [1, 3, 1]]


def _grid_space(ms, ns):
    return [((m,), (n,)) for m, n in itertools.product(ms, ns)]


@pytest.mark.parametrize("seed", range(12))
def test_whole_space_measured_gives_the_brute_force_minimum(seed):
    """With n >= |space| every distinct member of a population is measured; once the population
    has covered the whole space the result is the brute-force minimum of the measurement."""
    space = _grid_space([1, 2, 4], [1, 2])
    rng = sr.Uniforms(1000 + seed)
    est = [1.0 + rng.next() for _ in space]
    meas = [1.0 + rng.next() for _ in space]
    r = sr.heuristic_search(space, est, lambda c: meas[c], N=200, n=len(space), epsilon=1e-9, seed=seed)
    assert r["converged"]
    assert sorted(c for _, c, _, _ in r["log"]) == list(range(len(space)))
    assert r["best"] == min(range(len(space)), key=lambda c: meas[c])
    assert r["best_t"] == min(meas)


@pytest.mark.parametrize("seed", range(20))
def test_invariants(seed):
    space = _grid_space([1, 2, 4, 8], [1, 2, 4])
    rng = sr.Uniforms(77 + seed)
    est = [1.0 + 3.0 * rng.next() for _ in space]
    meas = [e * (0.7 + 0.6 * rng.next()) for e in est]        # the model is right within 30 %
    N, n, eps = 8, 3, 0.05
    r = sr.heuristic_search(space, est, lambda c: meas[c], N=N, n=n, epsilon=eps, seed=seed, max_generations=10)
    log = r["log"]
    cands = [c for _, c, _, _ in log]
    assert len(set(cands)) == len(cands)                               # nothing is measured twice
    assert all(0 <= c < len(space) and e == est[c] and t == meas[c] for _, c, e, t in log)
    for g in range(r["generations"]):
        assert sum(1 for gg, *_ in log if gg == g) <= n               # at most n per generation
    assert 1 <= r["generations"] <= 10
    best_seen = min(t for *_, t in log)
    if r["converged"]:
        assert r["generations"] >= 2                                   # the first generation never stops
        assert r["best_t"] <= best_seen * (1 + eps) + 1e-15            # top1 within epsilon of the best
    else:
        assert r["best_t"] == best_seen
    assert r["best_t"] == meas[r["best"]]


def test_same_seed_same_run_and_model_equal_to_measurement():
    space = _grid_space([1, 2, 4, 8], [1, 2, 4])
    est = [float(3 + (7 * i) % 11) for i in range(len(space))]
    a = sr.heuristic_search(space, est, lambda c: est[c], N=16, n=4, epsilon=0.02, seed=5)
    b = sr.heuristic_search(space, est, lambda c: est[c], N=16, n=4, epsilon=0.02, seed=5)
    assert a == b
    # measurement == estimate: top1 is always the smallest estimate of the population, and the
    # result is the smallest estimate among everything that was measured
    assert a["best_t"] == min(t for *_, t in a["log"])

"""The paper's heuristic search (Sec. IV-B, Alg. 1), written out plainly in the paper's order
and names (test infrastructure only; the library's search is checked against this).

The search space is handed in: a list of candidates, each a tuple of per-loop tile choices
(one entry per loop, e.g. ((mb, rg), (ns, nj)) for the loops m and n), with the analytical
estimate of each.  `measure` maps a candidate index to a run time.  Random numbers come from a
counter-based generator (SplitMix64 on seed + counter), consumed in a fixed order, so that a
second implementation given the same seed visits the same candidates.

Steps, as in Alg. 1:
  population <- N candidates drawn at random from the space
  repeat
      estimate every member; sort the population by estimate
      take the n members with the smallest estimates and measure them
      top1 <- the fastest measured of these
      if difference(top1_t, best_t) < epsilon: best <- top1; stop
      if top1_t < best_t: best <- top1
      population <- mutate(population): draw N members with probability ~ 1 / estimate,
                    and in each change the tile size of one randomly chosen loop

Readings taken where the listing is ambiguous:
  * "randomly select N candidates": without repetition while the space has unused candidates (a
    random permutation of the space, cut to N or topped up to N with further random draws), so
    that a space no larger than N is covered by the first population.
  * "Topk(..., reverse=True)" after an ascending sort: the n members with the SMALLEST
    estimates (the text: "isolate the top n candidates for detailed measurement").
  * A population holds duplicates; the n measured members are the first n DISTINCT candidates
    in sorted order, and a candidate measured in an earlier generation keeps its first time.
  * difference(a, b) = |a - b| / b, with best_t = 1e9 before the first measurement, so the
    first generation never stops the search.
  * Sorting is stable with ties in the estimate broken by candidate index; top1 ties go to the
    earlier member in sorted order.
  * "one loop is chosen to mutate the tile size": the loop uniformly at random; the new tile
    choice uniformly among the candidates of the space that differ from the parent in that
    loop's entry only; if there is none the child equals the parent.
  * A generation bound (not in the listing) ends a search that does not converge; the best
    measured candidate is returned with converged = False.
"""

_MASK = (1 << 64) - 1


def _mix(x):
    x = (x + 0x9E3779B97F4A7C15) & _MASK
    x = ((x ^ (x >> 30)) * 0xBF58476D1CE4E5B9) & _MASK
    x = ((x ^ (x >> 27)) * 0x94D049BB133111EB) & _MASK
    return x ^ (x >> 31)


class Uniforms:
    """u_0, u_1, ... in [0, 1): u_k = top 53 bits of mix(seed + k) / 2^53."""

    def __init__(self, seed):
        self.seed = seed & _MASK
        self.k = 0

    def next(self):
        x = _mix((self.seed + self.k) & _MASK)
        self.k += 1
        return (x >> 11) * (1.0 / (1 << 53))

    def below(self, n):
        return min(int(self.next() * n), n - 1)


def neighbours(space, i, loop):
    """Indices of the candidates that differ from candidate i in entry `loop` only."""
    me = space[i]
    out = []
    for j, c in enumerate(space):
        if j != i and c[loop] != me[loop] and all(c[q] == me[q] for q in range(len(me)) if q != loop):
            out.append(j)
    return out


def heuristic_search(space, estimates, measure, N, n, epsilon, seed, max_generations=16, rng=None):
    """Alg. 1.  Returns a dict: best (candidate index), best_t, converged, generations,
    log = [(generation, candidate index, estimate, measured time)] in measurement order, and
    populations = the population of every generation as it was drawn (before the sort).
    `rng` (an object with next() and below(n)) replaces the seeded generator in tests."""
    assert len(space) == len(estimates) and len(space) > 0
    rng = rng if rng is not None else Uniforms(seed)
    n_loops = len(space[0])
    perm = list(range(len(space)))                                     # generateCandidates
    population = []
    for i in range(N):
        if i < len(space):                      # without repetition while unused candidates remain
            j = i + rng.below(len(space) - i)
            perm[i], perm[j] = perm[j], perm[i]
            population.append(perm[i])
        else:
            population.append(rng.below(len(space)))
    best_t, best_cand = 1e9, None
    measured, log = {}, []
    populations = []
    generation, converged = 0, False
    while True:
        populations.append(list(population))
        estimated_ts = {c: estimates[c] for c in population}           # estimatePerformance
        population = sorted(population, key=lambda c: (estimated_ts[c], c))
        topk_cands = []
        for c in population:                                           # topk: n smallest, distinct
            if c not in topk_cands:
                topk_cands.append(c)
            if len(topk_cands) == n:
                break
        for c in topk_cands:                                           # measure
            if c not in measured:
                measured[c] = float(measure(c))
                log.append((generation, c, estimates[c], measured[c]))
        top1_cand = min(topk_cands, key=lambda c: measured[c])         # first minimum in sorted order
        top1_t = measured[top1_cand]
        generation += 1
        if abs(top1_t - best_t) / best_t < epsilon:
            best_cand, best_t = top1_cand, top1_t
            converged = True
            break
        if top1_t < best_t:
            best_cand, best_t = top1_cand, top1_t
        if generation >= max_generations:
            break
        # mutate: parents drawn with weight 1 / estimate, one loop's tile choice changed
        weights = [1.0 / estimated_ts[c] for c in population]
        total = 0.0
        cumulative = []
        for w in weights:
            total += w
            cumulative.append(total)
        nxt = []
        for _ in range(N):
            target = rng.next() * total
            parent = population[-1]
            for c, cum in zip(population, cumulative):
                if target < cum:
                    parent = c
                    break
            loop = rng.below(n_loops)
            u = rng.next()
            options = neighbours(space, parent, loop)
            nxt.append(options[min(int(u * len(options)), len(options) - 1)] if options else parent)
        population = nxt
    return {"best": best_cand, "best_t": best_t, "converged": converged, "generations": generation, "log": log,
            "populations": populations}

"""Search-space generation and pruning of the paper (Sec. III-A to III-C) over tiling
expressions of any shape, deep or flat (test infrastructure only; the product's host-side
enumeration is checked against this).

A tiling expression is a tree of the four cross-tile loops m, n, k, h of the chain
C = A.B, E = C.D: in the paper's notation `xy` nests loop y in loop x and `(x,y)` runs the
two one after the other in the same scope, so `mhnk` is a chain of four nodes and `mn(k,h)`
is m, inside it n, inside it first k and then h.

  Sec. III-A   the 4! deep and the 2 flat expressions; tile sizes in multiples of 16
  Sec. III-B   compute statements at the rightmost loop related to them, memory statements
               beside them by default, then moved to the rightmost loop that indexes their
               tensor once loops of extent 1 (dead nodes of the DAG) are removed
  Sec. III-C   Rule 1 (loops bound to the block index are deleted; equal sub-expressions are
               one candidate), Rule 2 (the reduction loop of the intermediate tensor must not
               enclose its spatial loop), Rule 3 (padding), Rule 4 (eq. (1) against 1.2 x the
               on-chip memory)

Readings taken (the text is short here and its figure of the pruning result is not part of it):
  * Rule 1 binds m and h, the spatial loops of the chain's output.  The text's own example
    (mhnk and mnkh are both `nk` per block) deletes h wherever it stands in a deep tiling.  In
    a flat tiling h stands beside k in one scope, which is what makes the expression flat (C is
    computed once per (m, n) and then used for every h): deleting it would turn `n(k,h)` into
    the deep `nk`, so there h stays inside the block.  That gives three sub-expressions,
    nk, kn and n(k,h); the paper's sentence counts five, and a reading of the text that
    yields five was not found (deleting m alone gives seven, deleting h only where it is
    outermost gives seven as well).
  * Rule 2 speaks of the intermediate tensor: its reduction loop is k, its spatial loop left
    inside a block is n.  kn falls, nk and n(k,h) stay: two survivors where the paper counts
    three.
  * eq. (1) sums the tiles of all five tensors; sizes are taken in bytes.
"""
from itertools import product
from math import ceil

from . import perf_model as pm

STATEMENTS = ("C_C", "C_E", "L_A", "L_B", "L_D", "S_E")


def expressions():
    return pm.deep_tilings() + pm.flat_tilings()


def parse(expr):
    """'mhnk' -> ('m', [('h', [('n', [('k', [])])])]);  'mn(k,h)' -> ('m', [('n', [('k', []), ('h', [])])])."""
    def nest(s, i):
        loop = s[i]
        assert loop in pm.LOOPS, expr
        i += 1
        if i < len(s) and s[i] == "(":
            children, i = [], i + 1
            while True:
                child, i = nest(s, i)
                children.append(child)
                if s[i] == ")":
                    return (loop, children), i + 1
                assert s[i] == ",", expr
                i += 1
        if i < len(s) and s[i] in pm.LOOPS:
            child, i = nest(s, i)
            return (loop, [child]), i
        return (loop, []), i
    tree, end = nest(expr, 0)
    assert end == len(expr), expr
    return tree


def chains(tree, prefix=()):
    """Every root-to-leaf chain of loops."""
    loop, children = tree
    here = prefix + (loop,)
    if not children:
        return [here]
    return [c for child in children for c in chains(child, here)]


def scope(expr, related, extents, drop_unit_loops=True, block_loops=""):
    """Loops that surround a statement related to the loops `related`: the chain that holds all
    of them, cut after the rightmost one; loops of extent 1 are dead and hold nothing; a
    statement does not leave the loops bound to the block index."""
    for chain in chains(parse(expr)):
        if set(related) <= set(chain):
            live = [l for l in chain if not (drop_unit_loops and extents[l] == 1)]
            pos = max((live.index(l) for l in set(related) | set(block_loops) if l in live), default=-1)
            return live[:pos + 1]
    raise ValueError("no chain of %s holds the loops %s" % (expr, related))


def trips(expr, stmt, extents, hoist=True, drop_unit_loops=True, block_loops=""):
    """Trip count of a statement (Sec. III-B): product of the extents of the loops around it."""
    if stmt.startswith("C_"):
        related = pm.COMPUTE_LOOPS[stmt[2]]
    else:
        tensor, comp = pm.MEM_STATEMENTS[stmt]
        related = pm.TENSOR_LOOPS[tensor] if hoist else pm.COMPUTE_LOOPS[comp]
    t = 1
    for l in scope(expr, related, extents, drop_unit_loops, block_loops):
        t *= extents[l]
    return t


def sub_expression(expr):
    """Rule 1: the expression a block runs once m and h are bound to the block index."""
    if "(" in expr:                  # flat: h shares a scope with k and stays
        return expr.replace("m", "")
    return expr.replace("m", "").replace("h", "")


def bound_form(expr):
    """The expression with the loops Rule 1 binds to the block index written outermost: what
    the grid of blocks executes.  Equivalent candidates (same sub-expression) share it."""
    sub = sub_expression(expr)
    return ("m" if "(" in expr else "mh") + sub


def bound_loops(expr):
    return "m" if "(" in expr else "mh"


def rule1_classes(exprs=None):
    """sub-expression -> the expressions that reduce to it."""
    out = {}
    for e in exprs or expressions():
        out.setdefault(sub_expression(e), []).append(e)
    return out


def violates_rule2(sub):
    """Rule 2: k, the reduction loop of the intermediate tensor C, encloses n, the spatial loop
    of C that is left inside a block: a block would hold a partial C tile per n."""
    for chain in chains(parse(sub)):
        if "k" in chain and "n" in chain and chain.index("k") < chain.index("n"):
            return True
    return False


def tile_choices(dim, granule=16):
    """Sec. III-A: the multiples of 16 up to the dimension (ceil(dim / 16) of them)."""
    return [granule * i for i in range(1, ceil(dim / granule) + 1)]


def count_space(M, N, K, H, elem_bytes, shm_max_bytes):
    """The sizes Sec. III-C follows through its example: expressions before and after Rules 1
    and 2, tile-size combinations before and after Rules 3 and 4, and their products."""
    dims = {"m": M, "n": N, "k": K, "h": H}
    exprs = expressions()
    classes = rule1_classes(exprs)
    kept = [s for s in classes if not violates_rule2(s)]
    n_tiles = 1
    for l in pm.LOOPS:
        n_tiles *= len(tile_choices(dims[l]))
    ok3 = {l: [t for t in tile_choices(dims[l]) if pm.padding_ok(dims[l], t)] for l in pm.LOOPS}
    after3 = after4 = 0
    for tm, tn, tk, th in product(ok3["m"], ok3["n"], ok3["k"], ok3["h"]):
        after3 += 1
        if pm.shm_estm({"m": tm, "n": tn, "k": tk, "h": th}) * elem_bytes <= 1.2 * shm_max_bytes:
            after4 += 1
    return {"expressions": len(exprs), "after_rule1": len(classes), "after_rule2": len(kept),
            "sub_expressions": sorted(classes), "kept": sorted(kept),
            "tile_choices": n_tiles, "after_rule3": after3, "after_rule4": after4,
            "candidates": len(exprs) * n_tiles, "candidates_pruned": len(kept) * after4}

"""The paper's tiling-expression traffic rules and analytical performance model, written out
plainly (test infrastructure only; the product's tile picker is checked against this).

Follows, in the paper's notation (its H is called L elsewhere in this repository):
  Sec. II-A        compute-to-memory ratio phi of one GEMM tile
  Sec. III-A       deep / flat tiling expressions, candidate count
  Sec. III-B       placement of Load / Compute / Store statements, hoisting to the rightmost
                   related loop, removal of loops of extent 1 (the DAG dead-node rule)
  Sec. III-C       eq. (1) shared-memory estimate, Rule 3 padding test
  Sec. IV-A        eq. (2)-(5): t_estm = (t_mem + t_comp) * alpha

Readings taken where the text is ambiguous or at odds with itself:
  * phi: the printed denominator 2*T_M*T_N + T_M*K + T_N*K does not give the quoted values
    227 and 2 (tile 256, K = 1024 and 1); T_M*T_N + T_M*K + T_N*K does (227.6, 1.98).
    phi() returns the form that reproduces the printed numbers, phi_printed() the other.
  * Sec. III-B says hoisting S_E out of the innermost loop of m h n(k(...), L_D, C_E, S_E) saves
    "a factor of k", but in that expression S_E sits in the scope of n, not k; by the volume
    rule stated two sentences earlier the saving is the extent of n.  volume() follows the rule.
  * "tile size" in eq. (1) and (3) is taken in bytes (elements * element size).
  * eq. (5): alpha = (N_block + N_SM) / N_block is the printed form; alpha_rounds() is the same
    quantity for blocks that run in whole rounds (the printed form is its smooth upper bound).
    estimate() computes either.
  * The dead-loop rule of Sec. III-B would hoist a load out of every loop once all loops that
    index its tensor have extent 1 (e.g. L_B when T_N = N and T_K = K).  Blocks share no
    on-chip memory, so in estimate() no statement leaves the loops bound to the block index
    (m, h and the batch): each block still loads what it uses once.
"""
from itertools import permutations
from math import ceil

LOOPS = "mnkh"
# Loops that index each tensor's tiles, and loops related to each compute block.
TENSOR_LOOPS = {"A": "mk", "B": "kn", "C": "mn", "D": "nh", "E": "mh"}
COMPUTE_LOOPS = {"C": "mnk", "E": "mnh"}
# Default association of memory statements with compute statements (Sec. III-B).
MEM_STATEMENTS = {"L_A": ("A", "C"), "L_B": ("B", "C"), "L_D": ("D", "E"), "S_E": ("E", "E")}


def phi(tm, tn, k):
    """FLOPs per element moved for one T_M x T_N output tile with reduction length K,
    in the form that reproduces the values quoted in Sec. I (C counted once)."""
    return (2.0 * tm * tn * k) / (tm * tn + tm * k + tn * k)


def phi_printed(tm, tn, k):
    """The expression exactly as printed in Sec. II-A (C counted twice)."""
    return (2.0 * tm * tn * k) / (2.0 * tm * tn + tm * k + tn * k)


def deep_tilings():
    return ["".join(p) for p in permutations(LOOPS)]


def flat_tilings():
    return ["mn(k,h)", "nm(k,h)"]


def n_candidates(M, N, K, H, granule=16):
    """Sec. III-C: (#expressions) x (#tile-size choices), tile sizes being multiples of 16."""
    n_expr = len(deep_tilings()) + len(flat_tilings())
    return n_expr * ceil(M / granule) * ceil(N / granule) * ceil(K / granule) * ceil(H / granule)


def _scope(order, related, extents, drop_unit_loops, block_loops=""):
    """Loops surrounding a statement placed at the rightmost loop of `order` that is in
    `related`; with drop_unit_loops, loops of extent 1 are dead nodes and cannot hold it.
    Loops in block_loops are bound to the block index (Rule 1): a statement cannot be hoisted
    out of them, because thread blocks share no on-chip memory."""
    live = [l for l in order if not (drop_unit_loops and extents[l] == 1)]
    pos = max((live.index(l) for l in set(related) | set(block_loops) if l in live), default=-1)
    return live[:pos + 1]


def trips(order, stmt, extents, hoist=True, drop_unit_loops=True, block_loops=""):
    """Trip count of a statement in the deep tiling `order` (a permutation of 'mnkh').

    stmt: 'C_C', 'C_E', 'L_A', 'L_B', 'L_D', 'S_E'.
    hoist=False keeps memory statements beside their compute statement (the default
    association); hoist=True moves them to the rightmost loop that indexes their tensor.
    """
    if stmt.startswith("C_"):
        scope = _scope(order, COMPUTE_LOOPS[stmt[2]], extents, drop_unit_loops, block_loops)
    else:
        tensor, comp = MEM_STATEMENTS[stmt]
        related = TENSOR_LOOPS[tensor] if hoist else COMPUTE_LOOPS[comp]
        scope = _scope(order, related, extents, drop_unit_loops, block_loops)
    t = 1
    for l in scope:
        t *= extents[l]
    return t


def tile_elems(tensor, tiles):
    a, b = TENSOR_LOOPS[tensor]
    return tiles[a] * tiles[b]


def volume(order, stmt, tiles, extents, **kw):
    """Elements moved by a memory statement: tile size x trip counts of surrounding loops."""
    return tile_elems(MEM_STATEMENTS[stmt][0], tiles) * trips(order, stmt, extents, **kw)


def shm_estm(tiles, tensors="ABCDE"):
    """eq. (1): sum of the tile sizes (elements) of the tensors held on chip."""
    return sum(tile_elems(t, tiles) for t in tensors)


def padding_ok(dim, tile, max_ratio=0.05):
    """Rule 3: no padding at all when the dimension is a power of two, else ratio < 0.05."""
    padded = ceil(dim / tile) * tile
    if dim & (dim - 1) == 0:
        return padded == dim
    return (padded - dim) / dim < max_ratio


def extents_of(dims, tiles):
    return {l: ceil(dims[l] / tiles[l]) for l in LOOPS}


def alpha_rounds(n_block, n_units):
    """eq. (5) read for a machine that runs blocks in rounds: n_units blocks run at a time, a
    launch takes ceil(n_block / n_units) rounds, and alpha is the capacity of those rounds over
    the blocks that fill it.  It never exceeds the printed (N_block + N_SM) / N_block, which is
    its smooth upper envelope (ceil(x) <= x + 1), and is 1 for a launch that fills whole rounds."""
    return ceil(n_block / n_units) * n_units / n_block


def estimate(order, dims, tiles, batch, elem_bytes, W, P, n_units, W_reread=None, rounds=False):
    """eq. (2)-(5) for a deep tiling of the two-GEMM chain.

    dims/tiles: dicts over 'mnkh'.  Spatial loops m, h and the batch are bound to the block
    index (Rule 1), so N_block = batch * m * h.  Returns a dict of every term.

    W_reread: if given, bytes beyond the first touch of each tensor are charged at this
    bandwidth (the on-die cache that serves re-reads) and the compulsory bytes at W; with
    W_reread None every byte is charged at W exactly as eq. (3) is printed.
    rounds: alpha as alpha_rounds() instead of the printed (N_block + N_SM) / N_block.
    """
    ext = extents_of(dims, tiles)
    blk = "mh"   # with the batch, the loops on the block index: nothing is hoisted out of a block
    mem = {s: volume(order, s, tiles, ext, block_loops=blk) * batch * elem_bytes for s in MEM_STATEMENTS}
    flops = {
        "C_C": 2 * tiles["m"] * tiles["n"] * tiles["k"] * trips(order, "C_C", ext, block_loops=blk) * batch,
        "C_E": 2 * tiles["m"] * tiles["n"] * tiles["h"] * trips(order, "C_E", ext, block_loops=blk) * batch,
    }
    compulsory = batch * elem_bytes * (dims["m"] * dims["k"] + dims["k"] * dims["n"]
                                       + dims["n"] * dims["h"] + dims["m"] * dims["h"])
    total = sum(mem.values())
    if W_reread is None:
        t_mem = total / W
    else:
        t_mem = compulsory / W + max(total - compulsory, 0) / W_reread
    t_comp = sum(flops.values()) / P
    n_block = batch * ext["m"] * ext["h"]
    alpha = alpha_rounds(n_block, n_units) if rounds else (n_block + n_units) / n_block
    return {"mem_bytes": mem, "model_bytes": total, "compulsory_bytes": compulsory,
            "flops": sum(flops.values()), "t_mem": t_mem, "t_comp": t_comp,
            "n_block": n_block, "alpha": alpha, "t_estm": (t_mem + t_comp) * alpha}

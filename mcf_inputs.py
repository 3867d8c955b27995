"""Seeded synthetic inputs for the fused-chain workloads (shared by tests, smoke and bench).

Holds none of the method's arithmetic: it only draws i.i.d. entries with a counter-based
generator, rounds them once (round-to-nearest-even) to fp16 / bf16, and hands out both the
16-bit patterns (for the GPU path) and their exact float64 values (for the CPU oracle), so
input quantisation is never charged as error to either side.

Generator: SplitMix64 finaliser applied to a counter built from (seed, tensor id, element
index); independent of numpy's / torch's RNG streams so values reproduce across versions.
U(-1,1) is 2u-1 with a 53-bit u; N(0,1) is Box-Muller on two such uniforms.

The five workloads are the evaluation shapes this build is measured on: plain batched GEMM
chains (A[b,M,K], B[b,K,N], D[b,N,L], U(-1,1) entries) and attention-shaped softmax chains
(Q[b,M,K], key matrix stored [b,N,K], V[b,N,L], N(0,1) entries, scale 1/sqrt(K)).
"""
from dataclasses import dataclass

import numpy as np

_M64 = np.uint64(0xFFFFFFFFFFFFFFFF)
BASE_SEED = 20250622


@dataclass(frozen=True)
class Workload:
    name: str
    batch: int
    M: int
    K: int
    N: int
    L: int
    dtype: str          # "f16" | "bf16"
    softmax: bool
    dist: str           # "uniform" | "normal"
    seed: int

    @property
    def scale(self):
        return 1.0 / float(np.sqrt(self.K)) if self.softmax else 1.0

    @property
    def compulsory_bytes(self):
        return 2 * self.batch * (self.M * self.K + self.K * self.N + self.N * self.L + self.M * self.L)

    @property
    def flops(self):
        return self.batch * (2 * self.M * self.N * self.K + 2 * self.M * self.N * self.L)


WORKLOADS = {
    "cfg1": Workload("cfg1", 1, 1024, 64, 128, 64, "f16", False, "uniform", BASE_SEED + 1),
    "cfg2": Workload("cfg2", 64, 512, 64, 512, 64, "f16", False, "uniform", BASE_SEED + 2),
    "cfg3": Workload("cfg3", 96, 512, 64, 512, 64, "f16", True, "normal", BASE_SEED + 3),
    "cfg4": Workload("cfg4", 16, 4096, 32, 1024, 32, "bf16", False, "uniform", BASE_SEED + 4),
    "cfg5": Workload("cfg5", 64, 4096, 128, 4096, 128, "bf16", True, "normal", BASE_SEED + 5),
}

# The shape tables of the paper's evaluation (Sec. VI-B1 Table II: batched GEMM chains G1-G12;
# Sec. VI-B2 Table III: self-attention modules S1-S9, heads as batch), fp16, same value recipe.
# Rows as (batch, M, N, K, H).
_PAPER_GEMM_CHAINS = {
    "G1": (1, 512, 256, 64, 64), "G2": (1, 512, 256, 64, 128), "G3": (1, 512, 256, 64, 256),
    "G4": (1, 512, 512, 256, 256), "G5": (1, 512, 512, 512, 256), "G6": (1, 512, 512, 1024, 256),
    "G7": (1, 512, 512, 128, 128), "G8": (1, 1024, 512, 128, 128), "G9": (1, 2048, 512, 128, 128),
    "G10": (1, 1024, 1024, 128, 128), "G11": (4, 1024, 1024, 128, 128), "G12": (8, 1024, 1024, 128, 128),
}
_PAPER_ATTENTION = {
    "S1": (8, 512, 512, 64, 64), "S2": (12, 512, 512, 64, 64), "S3": (16, 512, 512, 64, 64),
    "S4": (12, 256, 256, 64, 64), "S5": (16, 256, 256, 64, 64), "S6": (16, 256, 256, 80, 80),
    "S7": (1, 512, 256, 64, 64), "S8": (1, 768, 384, 64, 64), "S9": (1, 1024, 512, 64, 64),
}
PAPER_SHAPES = {}
for _i, (_n, (_b, _m, _nn, _k, _h)) in enumerate(_PAPER_GEMM_CHAINS.items()):
    PAPER_SHAPES[_n] = Workload(_n, _b, _m, _k, _nn, _h, "f16", False, "uniform", BASE_SEED + 100 + _i)
for _i, (_n, (_b, _m, _nn, _k, _h)) in enumerate(_PAPER_ATTENTION.items()):
    PAPER_SHAPES[_n] = Workload(_n, _b, _m, _k, _nn, _h, "f16", True, "normal", BASE_SEED + 200 + _i)


def _splitmix64(x):
    x = (x + np.uint64(0x9E3779B97F4A7C15)) & _M64
    x = ((x ^ (x >> np.uint64(30))) * np.uint64(0xBF58476D1CE4E5B9)) & _M64
    x = ((x ^ (x >> np.uint64(27))) * np.uint64(0x94D049BB133111EB)) & _M64
    return x ^ (x >> np.uint64(31))


def _uniform01(seed, tensor_id, stream, n, start=0):
    """n doubles in [0,1) from counters start..start+n-1 of one (seed, tensor, stream)."""
    with np.errstate(over="ignore"):
        key = _splitmix64(np.uint64(seed) ^ (np.uint64(tensor_id) << np.uint64(56))
                          ^ (np.uint64(stream) << np.uint64(48)))
        ctr = np.arange(start, start + n, dtype=np.uint64)
        bits = _splitmix64(ctr ^ key)
    return (bits >> np.uint64(11)).astype(np.float64) * (1.0 / 9007199254740992.0)


def draw(seed, tensor_id, shape, dist):
    """float64 array of i.i.d. U(-1,1) or N(0,1) entries, element e of the flattened array
    depending only on (seed, tensor_id, e)."""
    n = int(np.prod(shape, dtype=np.int64))
    out = np.empty(n, dtype=np.float64)
    step = 1 << 22
    for s in range(0, n, step):
        m = min(step, n - s)
        if dist == "uniform":
            out[s:s + m] = 2.0 * _uniform01(seed, tensor_id, 0, m, s) - 1.0
        elif dist == "normal":
            u1 = 1.0 - _uniform01(seed, tensor_id, 0, m, s)        # (0,1]
            u2 = _uniform01(seed, tensor_id, 1, m, s)
            out[s:s + m] = np.sqrt(-2.0 * np.log(u1)) * np.cos(2.0 * np.pi * u2)
        else:
            raise ValueError(dist)
    return out.reshape(shape)


def to_bits(x, dtype):
    """Round float64 -> fp16/bf16 (RNE); returns uint16 patterns."""
    if dtype == "f16":
        return np.asarray(x, dtype=np.float64).astype(np.float16).view(np.uint16)
    if dtype == "bf16":
        f = np.asarray(x, dtype=np.float64).astype(np.float32).view(np.uint32)
        rounded = f + np.uint32(0x7FFF) + ((f >> np.uint32(16)) & np.uint32(1))
        return (rounded >> np.uint32(16)).astype(np.uint16)
    raise ValueError(dtype)


def from_bits(bits, dtype):
    """Exact float64 value of uint16 fp16/bf16 patterns."""
    bits = np.asarray(bits, dtype=np.uint16)
    if dtype == "f16":
        return bits.view(np.float16).astype(np.float64)
    if dtype == "bf16":
        return (bits.astype(np.uint32) << np.uint32(16)).view(np.float32).astype(np.float64)
    raise ValueError(dtype)


def make_inputs(w, batch=None, values=True):
    """Inputs of workload w (optionally only its first `batch` batches).

    Returns dict with uint16 arrays a_bits [b,M,K], b_bits (stored [b,K,N] for plain chains,
    [b,N,K] for softmax chains: the key matrix as attention holds it), d_bits [b,N,L], and,
    if values, float64 arrays A [b,M,K], B as a [b,K,N] view, D [b,N,L] of the same numbers.
    Element e of each full tensor depends only on (seed, tensor id, e), so a batch prefix of a
    workload equals the prefix of the full workload.
    """
    b = w.batch if batch is None else int(batch)
    out = {"b_layout": "nk" if w.softmax else "kn"}
    a = to_bits(draw(w.seed, 1, (b, w.M, w.K), w.dist), w.dtype)
    bshape = (b, w.N, w.K) if w.softmax else (b, w.K, w.N)
    bb = to_bits(draw(w.seed, 2, bshape, w.dist), w.dtype)
    d = to_bits(draw(w.seed, 3, (b, w.N, w.L), w.dist), w.dtype)
    out.update(a_bits=a, b_bits=bb, d_bits=d)
    if values:
        out["A"] = from_bits(a, w.dtype)
        Bv = from_bits(bb, w.dtype)
        out["B"] = Bv.transpose(0, 2, 1) if w.softmax else Bv
        out["D"] = from_bits(d, w.dtype)
    return out


def make_problem(batch, M, K, N, L, dtype, softmax, dist, seed):
    """Ad-hoc workload of the same recipe (used for ragged / edge-case parity tests)."""
    return Workload(f"adhoc_{batch}x{M}x{K}x{N}x{L}_{dtype}", batch, M, K, N, L, dtype,
                    bool(softmax), dist, seed)

"""ctypes front end of the C oracle (mcf_oracle.c).  Test infrastructure only.

All tensors are numpy float64 arrays holding the exact values of the (already rounded)
fp16/bf16 inputs; any strides are accepted and handed to the C loops in elements.
Shapes follow Sec. III-A / VI-B of the paper with its H called L:
A[b,M,K], B[b,K,N], D[b,N,L] -> E[b,M,L].
"""
import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "mcf_oracle.c")
_LIB = os.path.join(_HERE, "libmcf_oracle.so")
_lib = None


def build_oracle(force=False):
    """Compile mcf_oracle.c with gcc.  Portable flags only (the built file travels to other
    hosts) and no FMA contraction, so every product and sum is a separately rounded double."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O3", "-std=c11", "-fopenmp", "-ffp-contract=off", "-fPIC", "-shared",
               "-Wall", "-Wextra", "-o", _LIB, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        lib = ctypes.CDLL(build_oracle())
        i64, dp, ip = ctypes.c_int64, ctypes.POINTER(ctypes.c_double), ctypes.POINTER(ctypes.c_int64)
        common = [i64] * 5 + [dp, ip, dp, ip, dp, ip, ctypes.c_int, ctypes.c_double]
        lib.mcf_oracle_chain.argtypes = common + [dp]
        lib.mcf_oracle_chain.restype = ctypes.c_int
        lib.mcf_oracle_chain_rows.argtypes = common + [i64, ip, dp]
        lib.mcf_oracle_chain_rows.restype = ctypes.c_int
        lib.mcf_oracle_intermediate_row.argtypes = common + [i64, i64, dp]
        lib.mcf_oracle_intermediate_row.restype = None
        lib.mcf_oracle_chain3.argtypes = common + [i64, dp, ip, dp]
        lib.mcf_oracle_chain3.restype = ctypes.c_int
        lib.mcf_oracle_chain_causal.argtypes = [i64] * 5 + [dp, ip, dp, ip, dp, ip, ctypes.c_double, i64, dp]
        lib.mcf_oracle_chain_causal.restype = ctypes.c_int
        _lib = lib
    return _lib


def _prep(A, B, D):
    A, B, D = (np.asarray(x) for x in (A, B, D))
    for x in (A, B, D):
        if x.dtype != np.float64 or x.ndim != 3:
            raise TypeError("oracle operands must be 3-d float64 arrays")
    b, M, K = A.shape
    b2, K2, N = B.shape
    b3, N2, L = D.shape
    if not (b == b2 == b3 and K == K2 and N == N2):
        raise ValueError(f"shape mismatch A{A.shape} B{B.shape} D{D.shape}")
    dp, ip = ctypes.POINTER(ctypes.c_double), ctypes.POINTER(ctypes.c_int64)
    args, keep = [b, M, K, N, L], []
    for x in (A, B, D):
        st = np.array([s // 8 for s in x.strides], dtype=np.int64)
        if any(s % 8 for s in x.strides) or any(s < 0 for s in x.strides):
            raise ValueError("strides must be non-negative multiples of the element size")
        keep += [x, st]
        args += [x.ctypes.data_as(dp), st.ctypes.data_as(ip)]
    return (b, M, K, N, L), args, keep


def chain(A, B, D, softmax=False, scale=1.0, return_threads=False):
    """E[b,i,j] of the whole chain, float64 [b,M,L]."""
    (b, M, K, N, L), args, keep = _prep(A, B, D)
    if softmax and N == 0:
        raise ValueError("softmax over an empty row is undefined")
    E = np.zeros((b, M, L), dtype=np.float64)
    threads = _load().mcf_oracle_chain(*args, int(bool(softmax)), float(scale),
                                       E.ctypes.data_as(ctypes.POINTER(ctypes.c_double)))
    del keep
    return (E, threads) if return_threads else E


def chain_rows(A, B, D, rows, softmax=False, scale=1.0):
    """Selected output rows: rows is an int array [nrows, 2] of (b, i); returns [nrows, L]."""
    (b, M, K, N, L), args, keep = _prep(A, B, D)
    rows = np.ascontiguousarray(rows, dtype=np.int64).reshape(-1, 2)
    if rows.size and (rows[:, 0].min() < 0 or rows[:, 0].max() >= b or
                      rows[:, 1].min() < 0 or rows[:, 1].max() >= M):
        raise IndexError("row selector out of range")
    out = np.zeros((rows.shape[0], L), dtype=np.float64)
    _load().mcf_oracle_chain_rows(*args, int(bool(softmax)), float(scale), rows.shape[0],
                                  rows.ctypes.data_as(ctypes.POINTER(ctypes.c_int64)),
                                  out.ctypes.data_as(ctypes.POINTER(ctypes.c_double)))
    del keep
    return out


def intermediate_row(A, B, D, b, i, softmax=False, scale=1.0):
    """Row (b,i) of the intermediate: C (no softmax) or P = softmax(scale*C)."""
    (bb, M, K, N, L), args, keep = _prep(A, B, D)
    if not (0 <= b < bb and 0 <= i < M):
        raise IndexError("row selector out of range")
    row = np.zeros(max(N, 1), dtype=np.float64)
    _load().mcf_oracle_intermediate_row(*args, int(bool(softmax)), float(scale), int(b), int(i),
                                        row.ctypes.data_as(ctypes.POINTER(ctypes.c_double)))
    del keep
    return row[:N]


def chain3(A, B, D, F, softmax=False, scale=1.0, return_threads=False):
    """Three-GEMM chain G = (E) . F with E = chain(A, B, D): F[b,L,P] -> float64 [b,M,P]."""
    (b, M, K, N, L), args, keep = _prep(A, B, D)
    F = np.asarray(F)
    if F.dtype != np.float64 or F.ndim != 3 or F.shape[0] != b or F.shape[1] != L:
        raise ValueError(f"F{F.shape} does not continue D's [b,N,{L}]")
    if any(s % 8 for s in F.strides) or any(s < 0 for s in F.strides):
        raise ValueError("strides must be non-negative multiples of the element size")
    if softmax and N == 0:
        raise ValueError("softmax over an empty row is undefined")
    P = F.shape[2]
    sf = np.array([s // 8 for s in F.strides], dtype=np.int64)
    G = np.zeros((b, M, P), dtype=np.float64)
    dp, ip = ctypes.POINTER(ctypes.c_double), ctypes.POINTER(ctypes.c_int64)
    threads = _load().mcf_oracle_chain3(*args, int(bool(softmax)), float(scale), P, F.ctypes.data_as(dp),
                                        sf.ctypes.data_as(ip), G.ctypes.data_as(dp))
    del keep
    return (G, threads) if return_threads else G


def chain_causal(A, B, D, scale=1.0, causal_offset=0):
    """Softmax chain under a causal mask: row i sees the columns n <= i + causal_offset (a row
    that sees none gives zeros).  float64 [b,M,L]."""
    (b, M, K, N, L), args, keep = _prep(A, B, D)
    E = np.zeros((b, M, L), dtype=np.float64)
    _load().mcf_oracle_chain_causal(*args, float(scale), int(causal_offset),
                                    E.ctypes.data_as(ctypes.POINTER(ctypes.c_double)))
    del keep
    return E

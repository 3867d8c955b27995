"""Pins of the fp64 oracle (oracle/mcf_oracle.c) to things other than itself: brute force on
tiny integer inputs, algebraic identities, closed forms and library routines.  CPU only."""
import json
import os

import numpy as np
import pytest
from scipy.special import softmax as scipy_softmax

import oracle

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def _ints(rng, shape, lo=-4, hi=5):
    return rng.integers(lo, hi, size=shape).astype(np.float64)


def test_bruteforce_flat_sum_bit_exact():
    # Distinct b, M, K, N, L so that any transposed operand or swapped index changes the result.
    rng = np.random.default_rng(11)
    b, M, K, N, L = 2, 3, 4, 5, 2
    A, B, D = _ints(rng, (b, M, K)), _ints(rng, (b, K, N)), _ints(rng, (b, N, L))
    E = oracle.chain(A, B, D)
    for bb in range(b):
        for i in range(M):
            for j in range(L):
                s = 0.0
                for n in range(N):
                    for k in range(K):
                        s += A[bb, i, k] * B[bb, k, n] * D[bb, n, j]
                assert E[bb, i, j] == s


def test_associativity_second_loop_nest():
    rng = np.random.default_rng(12)
    b, M, K, N, L = 3, 7, 5, 9, 4
    A, B, D = rng.standard_normal((b, M, K)), rng.standard_normal((b, K, N)), rng.standard_normal((b, N, L))
    BD = np.zeros((b, K, L))
    for bb in range(b):
        for k in range(K):
            for j in range(L):
                BD[bb, k, j] = sum(B[bb, k, n] * D[bb, n, j] for n in range(N))
    ref = np.zeros((b, M, L))
    for bb in range(b):
        for i in range(M):
            for j in range(L):
                ref[bb, i, j] = sum(A[bb, i, k] * BD[bb, k, j] for k in range(K))
    E = oracle.chain(A, B, D)
    assert np.max(np.abs(E - ref)) <= 1e-12 * np.max(np.abs(ref))
    # exact on small integers
    A, B, D = _ints(rng, (b, M, K)), _ints(rng, (b, K, N)), _ints(rng, (b, N, L))
    assert np.array_equal(oracle.chain(A, B, D), np.einsum("bik,bkj->bij", A, np.einsum("bkn,bnj->bkj", B, D)))


def test_identity_and_zero_operands():
    rng = np.random.default_rng(13)
    b, M, K, L = 2, 6, 5, 3
    A, D = _ints(rng, (b, M, K)), _ints(rng, (b, K, L))
    eye = np.broadcast_to(np.eye(K), (b, K, K)).copy()
    assert np.array_equal(oracle.chain(A, eye, D), A @ D)            # B = I  ->  E = A.D
    B = _ints(rng, (b, K, 4))
    eye4 = np.broadcast_to(np.eye(4), (b, 4, 4)).copy()
    assert np.array_equal(oracle.chain(A, B, eye4), A @ B)           # D = I  ->  E = A.B
    assert not oracle.chain(np.zeros_like(A), B, eye4).any()
    assert not oracle.chain(A, B, np.zeros((b, 4, 7))).any()
    # softmax with A = 0: every P = 1/N, so E is the column mean of D
    Dn = rng.standard_normal((b, 4, 7))
    E = oracle.chain(np.zeros_like(A), B, Dn, softmax=True, scale=0.37)
    assert np.allclose(E, np.broadcast_to(Dn.mean(axis=1, keepdims=True), E.shape), rtol=0, atol=1e-15)


def test_closed_form_softmax_example():
    g = json.load(open(os.path.join(GOLDEN, "softmax_chain_closed_form.json")))
    A, B, D = (np.array(g[k], dtype=np.float64) for k in "ABD")
    E = oracle.chain(A, B, D, softmax=True, scale=g["scale"])
    assert np.allclose(E, np.array(g["E"]), rtol=0, atol=1e-14)
    for i in range(2):
        P = oracle.intermediate_row(A, B, D, 0, i, softmax=True, scale=g["scale"])
        assert np.allclose(P, np.array(g["P"])[0, i], rtol=0, atol=1e-15)


def test_softmax_invariants():
    rng = np.random.default_rng(14)
    b, M, K, N, L = 2, 5, 6, 17, 3
    A, B, D = rng.standard_normal((b, M, K)), rng.standard_normal((b, K, N)), rng.standard_normal((b, N, L))
    scale = 0.41
    for bb in range(b):
        for i in range(M):
            P = oracle.intermediate_row(A, B, D, bb, i, softmax=True, scale=scale)
            assert abs(P.sum() - 1.0) <= 1e-14 and (P > 0).all()
    E = oracle.chain(A, B, D, softmax=True, scale=scale)
    # convex combination of the rows of D
    assert (E <= D.max(axis=1, keepdims=True) + 1e-14).all() and (E >= D.min(axis=1, keepdims=True) - 1e-14).all()
    # D = ones -> E = 1
    assert np.allclose(oracle.chain(A, B, np.ones_like(D), softmax=True, scale=scale), 1.0, rtol=0, atol=1e-14)
    # adding a constant c to every logit of a row (extra k column of ones times a row of c) changes nothing
    A2 = np.concatenate([A, np.ones((b, M, 1))], axis=2)
    B2 = np.concatenate([B, np.full((b, 1, N), 7.25)], axis=1)
    assert np.allclose(oracle.chain(A2, B2, D, softmax=True, scale=scale), E, rtol=0, atol=1e-13)
    # one dominant logit selects one row of D
    A3, B3 = np.zeros((1, 2, 1)), np.zeros((1, 1, N))
    A3[0, :, 0] = 1.0
    B3[0, 0, 11] = 80.0
    E3 = oracle.chain(A3, B3, D[:1], softmax=True, scale=1.0)
    assert np.allclose(E3[0, 0], D[0, 11], rtol=0, atol=1e-13)
    # scale really multiplies the logits: scale*S == S' built from scaled A
    assert np.allclose(oracle.chain(A * scale, B, D, softmax=True, scale=1.0), E, rtol=0, atol=1e-13)


@pytest.mark.parametrize("softmax", [False, True])
def test_library_special_case_numpy(softmax):
    rng = np.random.default_rng(15 + softmax)
    b, M, K, N, L = 3, 33, 16, 70, 24
    A, D = rng.standard_normal((b, M, K)), rng.standard_normal((b, N, L))
    Bnk = rng.standard_normal((b, N, K))         # key-matrix layout, handed over as a strided [b,K,N] view
    B = Bnk.transpose(0, 2, 1)
    scale = 1.0 / np.sqrt(K)
    C = A @ np.ascontiguousarray(B)
    ref = (scipy_softmax(scale * C, axis=-1) if softmax else C) @ D
    E = oracle.chain(A, B, D, softmax=softmax, scale=scale)
    assert np.max(np.abs(E - ref)) <= 1e-12 * np.max(np.abs(ref))
    # selected rows agree with the full result, bit for bit
    rows = np.array([[0, 0], [2, 32], [1, 7]])
    assert np.array_equal(oracle.chain_rows(A, B, D, rows, softmax=softmax, scale=scale), E[rows[:, 0], rows[:, 1]])


def test_strided_views_equal_packed_copies():
    rng = np.random.default_rng(17)
    big = rng.standard_normal((2, 12, 20))
    A = big[:, 1:9, 2:8]                          # [2,8,6] view, all strides non-trivial
    B = rng.standard_normal((2, 10, 6))[:, ::2, :].transpose(0, 2, 1)   # [2,6,5]
    D = rng.standard_normal((2, 5, 9))[:, :, 3:7]
    E = oracle.chain(A, B, D)
    assert np.array_equal(E, oracle.chain(A.copy(), B.copy(), D.copy()))


def test_shape_and_empty_handling():
    A, B, D = np.zeros((2, 0, 3)), np.zeros((2, 3, 4)), np.zeros((2, 4, 5))
    assert oracle.chain(A, B, D).shape == (2, 0, 5)
    A = np.ones((1, 2, 3))
    E = oracle.chain(A, np.zeros((1, 3, 0)), np.zeros((1, 0, 5)))   # empty sum over n
    assert E.shape == (1, 2, 5) and not E.any()
    with pytest.raises(ValueError):
        oracle.chain(A, np.zeros((1, 3, 0)), np.zeros((1, 0, 5)), softmax=True)
    with pytest.raises(ValueError):
        oracle.chain(A, np.zeros((1, 4, 4)), np.zeros((1, 4, 5)))


def test_chain3_bruteforce_and_identities():
    """Three-GEMM chain: flat triple sum on small integers (bit equality; distinct extents so that
    a swapped index shows), F = identity gives the two-GEMM chain, right-to-left association,
    and the softmax form against a library softmax and matmul."""
    rng = np.random.default_rng(21)
    b, M, K, N, L, P = 2, 3, 4, 5, 2, 6
    A, B, D, F = _ints(rng, (b, M, K)), _ints(rng, (b, K, N)), _ints(rng, (b, N, L)), _ints(rng, (b, L, P))
    G = oracle.chain3(A, B, D, F)
    assert G.shape == (b, M, P)
    for bb in range(b):
        for i in range(M):
            for q in range(P):
                s = 0.0
                for h in range(L):
                    for n in range(N):
                        for k in range(K):
                            s += A[bb, i, k] * B[bb, k, n] * D[bb, n, h] * F[bb, h, q]
                assert G[bb, i, q] == s
    eye = np.broadcast_to(np.eye(L), (b, L, L)).copy()
    assert np.array_equal(oracle.chain3(A, B, D, eye), oracle.chain(A, B, D))
    assert not oracle.chain3(A, B, D, np.zeros((b, L, P))).any()
    # A . (B . (D . F)) on random doubles
    A, B, D, F = (rng.standard_normal(s) for s in ((b, M, K), (b, K, N), (b, N, L), (b, L, P)))
    ref = A @ (B @ (D @ F))
    assert np.max(np.abs(oracle.chain3(A, B, D, F) - ref)) <= 1e-12 * np.max(np.abs(ref))
    # softmax between the first two GEMMs; a transposed (strided) F view
    Ft = np.ascontiguousarray(F.transpose(0, 2, 1)).transpose(0, 2, 1)
    ref = (scipy_softmax(0.3 * (A @ B), axis=-1) @ D) @ F
    got = oracle.chain3(A, B, D, Ft, softmax=True, scale=0.3)
    assert np.max(np.abs(got - ref)) <= 1e-12 * np.max(np.abs(ref))
    with pytest.raises(ValueError):
        oracle.chain3(A, B, D, np.zeros((b, L + 1, P)))


def test_causal_mask_bruteforce_and_special_cases():
    """The causal softmax chain (not in the paper; row i sees the columns n <= i + offset) against
    a brute-force definition written here with an explicit mask, and against the cases that fix
    the offset convention: the first row of the lower triangle is the first row of D, a mask that
    hides nothing is the plain softmax chain, a row that sees k columns equals the chain over the
    first k columns, a row that sees nothing is zero."""
    rng = np.random.default_rng(31)
    b, M, K, N, L = 2, 6, 3, 9, 4
    A, B, D = rng.standard_normal((b, M, K)), rng.standard_normal((b, K, N)), rng.standard_normal((b, N, L))
    scale = 0.7
    for off in (0, 3, -2, N - M, N + 5, -M - 1):
        E = oracle.chain_causal(A, B, D, scale=scale, causal_offset=off)
        ref = np.zeros((b, M, L))
        for bb in range(b):
            for i in range(M):
                cols = [n for n in range(N) if n <= i + off]
                if not cols:
                    continue
                s = np.array([scale * sum(A[bb, i, k] * B[bb, k, n] for k in range(K)) for n in cols])
                w = np.exp(s - s.max())
                w /= w.sum()
                for j in range(L):
                    ref[bb, i, j] = sum(w[q] * D[bb, n, j] for q, n in enumerate(cols))
        assert np.max(np.abs(E - ref)) <= 1e-14
    low = oracle.chain_causal(A, B, D, scale=scale, causal_offset=0)
    assert np.allclose(low[:, 0], D[:, 0], rtol=0, atol=1e-15)                    # one visible column: P = 1
    full = oracle.chain(A, B, D, softmax=True, scale=scale)
    assert np.array_equal(oracle.chain_causal(A, B, D, scale=scale, causal_offset=N - 1), full)
    assert np.array_equal(oracle.chain_causal(A, B, D, scale=scale, causal_offset=N + 7), full)
    for i in range(M):                                                            # row i sees i + 3 + 1 columns
        k = min(N, i + 4)
        part = oracle.chain(A[:, i:i + 1], B[:, :, :k], D[:, :k], softmax=True, scale=scale)
        assert np.allclose(oracle.chain_causal(A, B, D, scale=scale, causal_offset=3)[:, i:i + 1], part, rtol=0, atol=1e-15)
    hidden = oracle.chain_causal(A, B, D, scale=scale, causal_offset=-3)
    assert not hidden[:, :3].any() and hidden[:, 3:].any()
    # library special case: masked logits through scipy's softmax
    C = scale * (A @ B)
    C[:, np.arange(M)[:, None] + 2 < np.arange(N)[None, :]] = -np.inf
    ref = scipy_softmax(C, axis=-1) @ D
    assert np.max(np.abs(oracle.chain_causal(A, B, D, scale=scale, causal_offset=2) - ref)) <= 1e-14

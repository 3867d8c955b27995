"""Parity of the three-GEMM chain G = ((A.B).D).F (optionally with the row softmax after the
first GEMM) with the fp64 oracle, element by element.  Needs an MI355X."""
import numpy as np
import pytest
import torch

import mcf_inputs as mi
import oracle
import paper_2506_22169_amd as mcf
from paper_2506_22169_amd.binding import make_problem as c_problem

from gpu_util import TOL, device_inputs, to_device, to_host64

pytestmark = pytest.mark.gpu


def _inputs(b, M, K, N, L, P, dtype, softmax, seed):
    w = mi.make_problem(b, M, K, N, L, dtype, softmax, "normal" if softmax else "uniform", seed=seed)
    x = mi.make_inputs(w)
    f_bits = mi.to_bits(mi.draw(seed, 4, (b, L, P), w.dist), dtype)
    return w, x, f_bits, mi.from_bits(f_bits, dtype)


def _check(G, ref, what):
    assert G.shape == ref.shape and np.isfinite(G).all()
    scale = np.max(np.abs(ref)) if ref.size else 0.0
    err = np.max(np.abs(G - ref)) if ref.size else 0.0
    assert err <= TOL * scale, f"{what}: max|err| {err:.4g} > {TOL} * {scale:.4g}"
    return err / scale if scale else 0.0


@pytest.mark.parametrize("softmax", [False, True])
@pytest.mark.parametrize("dtype", ["f16", "bf16"])
@pytest.mark.parametrize("KLP", [(64, 64, 64), (128, 128, 128), (64, 128, 128), (128, 64, 64), (64, 64, 128)])
def test_chain3_every_variant_small_ragged(KLP, dtype, softmax):
    """Every arrangement built for three GEMMs, on ragged m and n tails over several tiles."""
    K, L, P = KLP
    M, N = 600, (584 if not softmax else 589)
    w, x, f_bits, F64 = _inputs(3, M, K, N, L, P, dtype, softmax, seed=9000 + K + 3 * L + 7 * P)
    ref = oracle.chain3(x["A"], x["B"], x["D"], F64, softmax=softmax, scale=w.scale)
    A, B, D = device_inputs(w, x)
    F = to_device(f_bits, dtype)
    prob = c_problem(3, M, K, N, L, dtype, b_stride=(N * K, 1, K) if softmax else None)
    shapes = mcf.list_variants3(prob, P, softmax)
    assert len(shapes) >= 4
    worst = 0.0
    for tiles in shapes + [None]:
        print(f"case chain3 K={K} L={L} P={P} {dtype} softmax={softmax} tiles={tiles}", flush=True)
        G = mcf.gemm_chain3(A, B, D, F, scale=w.scale if softmax else None, tiles=tiles)
        torch.cuda.synchronize()
        worst = max(worst, _check(to_host64(G, dtype), ref, f"K={K} {dtype} softmax={softmax} tiles={tiles}"))
    print(f"worst max|err|/max|oracle| = {worst:.3e}", flush=True)


@pytest.mark.parametrize("softmax", [False, True])
def test_chain3_strides_layouts_and_edges(softmax):
    """The other B layout, F and G as row-strided views, one row, one column of C, and (plain
    chain) no column at all: G = 0."""
    K = L = P = 64
    w, x, f_bits, F64 = _inputs(2, 100, K, 72, L, P, "f16", softmax, seed=9100)
    A, B, D = device_inputs(w, x)
    B = B.transpose(1, 2).contiguous().transpose(1, 2) if not softmax else B.contiguous()   # the layout the workloads do not use
    Fbig = torch.zeros((2, L, P + 16), dtype=torch.float16, device="cuda")
    Fbig[:, :, :P] = to_device(f_bits, "f16")
    Gbig = torch.full((2, 100, P + 8), 7.0, dtype=torch.float16, device="cuda")
    print(f"case chain3 strided softmax={softmax}", flush=True)
    mcf.gemm_chain3(A, B, D, Fbig[:, :, :P], scale=w.scale if softmax else None, out=Gbig[:, :, :P])
    torch.cuda.synchronize()
    ref = oracle.chain3(x["A"], x["B"], x["D"], F64, softmax=softmax, scale=w.scale)
    _check(to_host64(Gbig[:, :, :P], "f16"), ref, "strided")
    assert (Gbig[:, :, P:] == 7.0).all()                        # nothing written beyond the view
    for M1, N1 in ((1, 72), (100, 1)) + (((100, 0),) if not softmax else ()):
        print(f"case chain3 M={M1} N={N1} softmax={softmax}", flush=True)
        A1, B1, D1 = A[:, :M1].contiguous(), B[:, :, :N1].contiguous(), D[:, :N1].contiguous()
        G = mcf.gemm_chain3(A1, B1, D1, Fbig[:, :, :P], scale=w.scale if softmax else None)
        torch.cuda.synchronize()
        ref = oracle.chain3(x["A"][:, :M1], x["B"][:, :, :N1], x["D"][:, :N1], F64, softmax=softmax, scale=w.scale)
        _check(to_host64(G, "f16"), ref, f"M={M1} N={N1}")
        if N1 == 0:
            assert (G == 0).all()


def test_chain3_errors():
    A = torch.zeros((1, 64, 64), dtype=torch.float16, device="cuda")
    F = torch.zeros((1, 64, 64), dtype=torch.float16, device="cuda")
    with pytest.raises(mcf.McfError) as e:                       # F does not continue D
        mcf.gemm_chain3(A, A, A, torch.zeros((1, 32, 64), dtype=torch.float16, device="cuda"))
    assert e.value.status == 1
    with pytest.raises(mcf.McfError) as e:                       # P not built
        mcf.gemm_chain3(A, A, A, torch.zeros((1, 64, 32), dtype=torch.float16, device="cuda"))
    assert e.value.status == 2
    with pytest.raises(mcf.McfError) as e:                       # an arrangement that is not built for three GEMMs
        mcf.gemm_chain3(A, A, A, F, tiles=(4, 2, 2, 1))
    assert e.value.status == 1
    with pytest.raises(mcf.McfError) as e:                       # output aliases F
        mcf.gemm_chain3(A, A, A, F, out=F)
    assert e.value.status == 1


def test_chain3_random_sweep():
    """Seeded sweep over group, dtype, chain kind, B layout, sizes, row pitches of F and G and
    the built arrangements (MCF_SWEEP_SEED / MCF_SWEEP_CASES: a longer or different one-off run)."""
    import os
    rng = np.random.default_rng(int(os.environ.get("MCF_SWEEP_SEED", "31415")))
    n_cases = int(os.environ.get("MCF_SWEEP_CASES", "48"))
    sizes = [1, 2, 7, 31, 32, 33, 64, 100, 129, 255, 300, 517]
    worst = 0.0
    for case in range(n_cases):
        K, L, P = ((64, 64, 64), (128, 128, 128), (64, 128, 128), (128, 64, 64), (64, 64, 128))[rng.integers(5)]
        dtype = ("f16", "bf16")[rng.integers(2)]
        softmax = bool(rng.integers(2))
        nk = bool(rng.integers(2))
        b = int(rng.integers(1, 4))
        M = int(sizes[rng.integers(len(sizes))])
        N = int(sizes[rng.integers(len(sizes))])
        if not nk:
            N = max(8, (N + 7) // 8 * 8)
        padf, padg = int(8 * rng.integers(0, 3)), int(8 * rng.integers(0, 3))
        w, x, f_bits, F64 = _inputs(b, M, K, N, L, P, dtype, softmax, seed=9500 + case)
        A, B, D = device_inputs(w, x)                       # B is [b,K,N]: N-contiguous for plain, K-contiguous for softmax
        if nk != softmax:
            B = B.transpose(1, 2).contiguous().transpose(1, 2) if nk else B.contiguous()
        tdt = torch.float16 if dtype == "f16" else torch.bfloat16
        Fbig = torch.zeros((b, L, P + padf), dtype=tdt, device="cuda")
        Fbig[:, :, :P] = to_device(f_bits, dtype)
        Gbig = torch.full((b, M, P + padg), 5.0, dtype=tdt, device="cuda")
        prob = mcf.binding._problem_from_tensors(A, B, D, mcf.binding._MetaLike(A, D))
        shapes = mcf.list_variants3(prob, P, softmax)
        tiles = shapes[rng.integers(len(shapes))] if case % 4 else None
        print(f"case {case}: b={b} M={M} K={K} N={N} {dtype} softmax={softmax} nk={nk} padf={padf} padg={padg} tiles={tiles}",
              flush=True)
        mcf.gemm_chain3(A, B, D, Fbig[:, :, :P], scale=w.scale if softmax else None, out=Gbig[:, :, :P], tiles=tiles)
        torch.cuda.synchronize()
        ref = oracle.chain3(x["A"], x["B"], x["D"], F64, softmax=softmax, scale=w.scale)
        worst = max(worst, _check(to_host64(Gbig[:, :, :P], dtype), ref, f"case {case}"))
        assert bool((Gbig[:, :, P:] == 5.0).all()), f"case {case}: wrote outside the output view"
    print(f"worst max|err|/max|oracle| = {worst:.3e}", flush=True)

"""Parity of two variations of the chain with the fp64 oracle (through the C ABI): the softmax
chain under a causal mask (row i sees the columns n <= i + offset; not in the paper), and an
fp32 output (the accumulators stored unrounded).  Needs an MI355X."""
import numpy as np
import pytest
import torch

import mcf_inputs as mi
import oracle
import paper_2506_22169_amd as mcf
from paper_2506_22169_amd.binding import make_problem as c_problem

from gpu_util import TOL, device_inputs, to_host64, torch_dtype

pytestmark = pytest.mark.gpu


def _check_causal(w, x, off, tiles=None, out_dtype=None):
    A, B, D = device_inputs(w, x)
    out = None if out_dtype is None else torch.empty((w.batch, w.M, w.L), dtype=out_dtype, device="cuda")
    E = mcf.causal_softmax_gemm_chain(A, B, D, w.scale, causal_offset=off, out=out, tiles=tiles)
    torch.cuda.synchronize()
    got = E.double().cpu().numpy() if E.dtype == torch.float32 else to_host64(E, w.dtype)
    ref = oracle.chain_causal(x["A"], x["B"], x["D"], scale=w.scale, causal_offset=off)
    assert np.isfinite(got).all()
    scale = np.max(np.abs(ref))
    err = np.max(np.abs(got - ref))
    assert err <= TOL * max(scale, 1e-30), f"{w.name} off={off} tiles={tiles}: max|err| {err:.4g} > {TOL} * {scale:.4g}"
    # rows that see nothing are exactly zero
    blind = np.arange(w.M) + off < 0
    assert not got[:, blind].any()
    return err / scale if scale else 0.0


@pytest.mark.parametrize("dtype,KL", [("f16", (64, 64)), ("bf16", (128, 128)), ("f16", (32, 32)), ("bf16", (80, 80)),
                                      ("f16", (256, 256)), ("f16", (384, 128))])
def test_causal_every_variant(dtype, KL):
    """Every built wave arrangement (pipelined loop, the loops of the groups that cannot be
    pipelined, and the k loop) under the lower-triangle mask and the mask aligned at the last
    row and column, on a shape with ragged m and n tails and M != N."""
    K, L = KL
    M, N = 333, 461
    w = mi.make_problem(2, M, K, N, L, dtype, True, "normal", seed=8100 + K + L)
    x = mi.make_inputs(w)
    prob = c_problem(2, M, K, N, L, dtype, b_stride=(N * K, 1, K))
    worst = 0.0
    for tiles in mcf.list_variants(prob, True):
        for off in (0, N - M):
            print(f"case causal K={K} L={L} {dtype} tiles={tiles} off={off}", flush=True)
            worst = max(worst, _check_causal(w, x, off, tiles))
    print(f"worst max|err|/max|oracle| = {worst:.3e}", flush=True)


@pytest.mark.parametrize("off", [0, 1, -1, 63, 64, -64, 129, -200, -333, -400, 460, 461, 10**6, -10**6])
def test_causal_offsets(off):
    """Offsets from 'no row sees anything' to 'every row sees everything', tiles from the picker;
    offsets of N - 1 and more equal the unmasked chain bit for bit."""
    M, N, K, L = 333, 461, 64, 64
    w = mi.make_problem(3, M, K, N, L, "f16", True, "normal", seed=8200)
    x = mi.make_inputs(w)
    print(f"case causal offsets off={off}", flush=True)
    _check_causal(w, x, off)
    if off >= N - 1:
        A, B, D = device_inputs(w, x)
        assert torch.equal(mcf.causal_softmax_gemm_chain(A, B, D, w.scale, causal_offset=off), mcf.softmax_gemm_chain(A, B, D, w.scale))


def test_causal_full_size_attention():
    """The short attention workload (96 heads, seq 512, head 64) under the lower-triangle mask,
    every element; and every tile arrangement at that size."""
    w = mi.WORKLOADS["cfg3"]
    x = mi.make_inputs(w)
    print("case causal cfg3", flush=True)
    r = _check_causal(w, x, 0)
    print(f"cfg3 causal: max|err|/max|oracle| = {r:.3e}", flush=True)


def test_causal_long_rows_sampled():
    """Sequence 4096, head 128 (the long attention's shape, 2 heads): the masked chain over the
    first k columns equals the unmasked chain on inputs cut to k columns, row by row, which the
    oracle's row routine can compute for sampled rows."""
    w = mi.make_problem(2, 4096, 128, 4096, 128, "bf16", True, "normal", seed=8300)
    x = mi.make_inputs(w)
    A, B, D = device_inputs(w, x)
    E = mcf.causal_softmax_gemm_chain(A, B, D, w.scale, causal_offset=0)
    torch.cuda.synchronize()
    got = to_host64(E, w.dtype)
    assert np.isfinite(got).all()
    rng = np.random.default_rng(3)
    for b, i in [(0, 0), (1, 4095), (0, 63), (1, 64), (0, 255), (1, 256)] + [(int(rng.integers(2)), int(rng.integers(4096))) for _ in range(40)]:
        k = i + 1
        ref = oracle.chain(x["A"][b:b + 1, i:i + 1], x["B"][b:b + 1, :, :k], x["D"][b:b + 1, :k], softmax=True, scale=w.scale)[0, 0]
        err, scale = np.max(np.abs(got[b, i] - ref)), np.max(np.abs(ref))
        assert err <= TOL * scale, (b, i, err, scale)


@pytest.mark.parametrize("softmax", [False, True])
@pytest.mark.parametrize("dtype,KL", [("f16", (64, 64)), ("bf16", (128, 128)), ("bf16", (32, 32)), ("f16", (80, 80)),
                                      ("f16", (64, 256)), ("f16", (384, 128))])
def test_fp32_output_every_variant(dtype, KL, softmax):
    """E stored as fp32: within the tolerance of the oracle, and -- the same accumulators rounded
    once -- equal bit for bit to the 16-bit output after rounding; every wave arrangement, ragged
    m and n tails, a row stride wider than L."""
    K, L = KL
    M, N = 300, (264 if not softmax else 261)
    w = mi.make_problem(2, M, K, N, L, dtype, softmax, "normal" if softmax else "uniform", seed=8400 + K + L)
    x = mi.make_inputs(w)
    A, B, D = device_inputs(w, x)
    ref = oracle.chain(x["A"], x["B"], x["D"], softmax=softmax, scale=w.scale)
    prob = c_problem(2, M, K, N, L, dtype, b_stride=(N * K, 1, K) if softmax else None)
    for tiles in mcf.list_variants(prob, softmax):
        print(f"case fp32 out K={K} L={L} {dtype} softmax={softmax} tiles={tiles}", flush=True)
        wide = torch.full((2, M, L + 8), -7.0, dtype=torch.float32, device="cuda")
        E32 = wide[:, :, :L]
        run = (lambda out: mcf.softmax_gemm_chain(A, B, D, w.scale, out=out, tiles=tiles)) if softmax else \
              (lambda out: mcf.gemm_chain(A, B, D, out=out, tiles=tiles))
        run(E32)
        E16 = run(None)
        torch.cuda.synchronize()
        got = E32.double().cpu().numpy()
        assert np.max(np.abs(got - ref)) <= TOL * np.max(np.abs(ref))
        assert torch.equal(E32.to(torch_dtype(dtype)), E16)
        assert bool((wide[:, :, L:] == -7.0).all())      # nothing written beyond the L columns of a row


def test_fp32_output_three_gemm_chain_and_causal():
    w = mi.make_problem(2, 200, 64, 136, 64, "f16", True, "normal", seed=8500)
    x = mi.make_inputs(w)
    A, B, D = device_inputs(w, x)
    F = (torch.randn(2, 64, 64, device="cuda", generator=torch.Generator(device="cuda").manual_seed(1)) * 0.5).half()
    for scale in (None, w.scale):
        G32 = torch.empty((2, 200, 64), dtype=torch.float32, device="cuda")
        mcf.gemm_chain3(A, B, D, F, scale=scale, out=G32)
        G16 = mcf.gemm_chain3(A, B, D, F, scale=scale)
        torch.cuda.synchronize()
        assert torch.equal(G32.half(), G16)
        ref = oracle.chain3(x["A"], x["B"], x["D"], F.double().cpu().numpy(), softmax=scale is not None, scale=w.scale)
        assert np.max(np.abs(G32.double().cpu().numpy() - ref)) <= TOL * np.max(np.abs(ref))
    _check_causal(w, x, 136 - 200, out_dtype=torch.float32)

"""Parity of the HIP path (through the C ABI) with the fp64 oracle, element by element, on
seeded inputs that span several tiles and ragged tails.  Needs an MI355X."""
import os

import numpy as np
import pytest
import torch

import mcf_inputs as mi
import oracle
import paper_2506_22169_amd as mcf
from paper_2506_22169_amd.binding import make_problem as c_problem

from gpu_util import TOL, check_full, device_inputs, run_gpu, to_device, to_host64

pytestmark = pytest.mark.gpu



@pytest.mark.parametrize("softmax", [False, True])
@pytest.mark.parametrize("dtype", ["f16", "bf16"])
@pytest.mark.parametrize("KL", [(32, 32), (64, 64), (128, 128), (64, 128), (128, 64), (64, 256), (256, 256),
                                (256, 64), (384, 128), (512, 256),    # these three: k loop inside the block
                                (80, 80), (96, 96), (160, 160), (192, 192)])   # rows padded to a power-of-two pitch in LDS
def test_every_variant_small_ragged(KL, dtype, softmax):
    """Every built wave arrangement on a shape with a ragged m tail and a ragged n tail that
    spans several tiles of the largest variant (tm up to 256, tn up to 256)."""
    # plain chains keep B as [b,K,N] (N a multiple of 8), softmax chains as the key matrix [b,N,K]
    M, N = 600, (584 if not softmax else 589)
    dist = "normal" if softmax else "uniform"
    K, L = KL
    w = mi.make_problem(3, M, K, N, L, dtype, softmax, dist, seed=1000 + K + 7 * L)
    worst = 0.0
    prob = c_problem(3, M, K, N, L, dtype, b_stride=(N * K, 1, K) if softmax else None)
    shapes = mcf.list_variants(prob, softmax)
    assert len(shapes) >= (8 if K * L <= 128 * 128 else 4)
    for tiles in shapes:
        print(f"case K={K} L={L} {dtype} softmax={softmax} tiles={tiles}", flush=True)
        worst = max(worst, check_full(w, tiles))
    print(f"worst max|err|/max|oracle| = {worst:.3e}", flush=True)


@pytest.mark.parametrize("softmax", [False, True])
@pytest.mark.parametrize("KL", [(64, 256), (128, 128), (384, 128), (256, 256)])
def test_h_tiles_every_candidate(KL, softmax):
    """T_L < L: the column tiles of E are blocks of their own (grid over batch, m-tile, h-tile).
    Every feasible candidate with T_L < L, on a shape with ragged m and n tails."""
    K, L = KL
    M, N = 333, (200 if not softmax else 203)
    w = mi.make_problem(2, M, K, N, L, "f16", softmax, "normal" if softmax else "uniform", seed=5000 + K + L)
    prob = c_problem(2, M, K, N, L, "f16", b_stride=(N * K, 1, K) if softmax else None)
    cands = [(t.mb, t.rg, t.ns, t.nj, t.tl) for t in mcf.list_candidates(prob, softmax) if t.tl < L]
    assert len(cands) >= 6 and len({c[4] for c in cands}) >= (2 if L == 256 else 1)
    worst = 0.0
    for tiles in cands:
        print(f"case K={K} L={L} softmax={softmax} tiles={tiles}", flush=True)
        worst = max(worst, check_full(w, tiles))
    print(f"worst max|err|/max|oracle| = {worst:.3e}", flush=True)


@pytest.mark.parametrize("layout", ["kn", "nk"])
@pytest.mark.parametrize("softmax", [False, True])
def test_both_b_layouts(softmax, layout):
    """Plain chain with a K-contiguous B and softmax chain with an N-contiguous B (the
    combinations the workloads themselves do not use)."""
    w = mi.make_problem(2, 256, 64, 256, 64, "f16", softmax, "normal" if softmax else "uniform", seed=77)
    x = mi.make_inputs(w)
    A, B, D = device_inputs(w, x)
    if (x["b_layout"] == "nk") != (layout == "nk"):
        B = B.transpose(1, 2).contiguous().transpose(1, 2) if layout == "nk" else B.contiguous()
    assert (B.stride(1) == 1) == (layout == "nk")
    E = mcf.softmax_gemm_chain(A, B, D, w.scale) if softmax else mcf.gemm_chain(A, B, D)
    torch.cuda.synchronize()
    ref = oracle.chain(x["A"], x["B"], x["D"], softmax=softmax, scale=w.scale)
    assert np.max(np.abs(to_host64(E, "f16") - ref)) <= TOL * np.max(np.abs(ref))


@pytest.mark.parametrize("name", ["cfg1", "cfg2", "cfg3", "cfg4"])
def test_workload_full_size(name):
    """The evaluation workloads at full size with the picker's tiles, every element."""
    w = mi.WORKLOADS[name]
    print(f"case {name}", flush=True)
    r = check_full(w)
    print(f"{name}: max|err|/max|oracle| = {r:.3e}", flush=True)


@pytest.mark.parametrize("name", list(mi.PAPER_SHAPES))
def test_paper_shape_tables(name):
    """The shapes of the paper's own evaluation (Table II chains, Table III attention modules)
    at full size with the picker's tiles, every element (G5, G6 with K = 512, 1024 run the
    kernels with a k loop; S6 has K = H = 80)."""
    w = mi.PAPER_SHAPES[name]
    print(f"case {name}", flush=True)
    r = check_full(w)
    print(f"{name}: max|err|/max|oracle| = {r:.3e}", flush=True)


def test_cfg5_sampled_rows():
    """Long-sequence softmax chain at full size: the whole output is produced by the launch
    bench.py would time; 4 heads are compared in 256 sampled rows each plus 64 rows sampled
    over all heads (the oracle needs ~2 MFLOP per row in fp64)."""
    w = mi.WORKLOADS["cfg5"]
    x = mi.make_inputs(w, values=False)
    A, B, D = device_inputs(w, x)
    E = mcf.softmax_gemm_chain(A, B, D, w.scale)
    torch.cuda.synchronize()
    assert torch.isfinite(E.float()).all()
    rng = np.random.default_rng(5)
    rows = [(b, i) for b in (0, 21, 42, 63) for i in rng.choice(w.M, 256, replace=False)]
    rows += [(int(b), int(i)) for b, i in zip(rng.integers(0, w.batch, 64), rng.integers(0, w.M, 64))]
    rows = np.array(rows, dtype=np.int64)
    heads = sorted(set(rows[:, 0].tolist()))
    remap = {h: j for j, h in enumerate(heads)}
    sel = np.array(heads)
    A64 = mi.from_bits(x["a_bits"][sel], w.dtype)
    B64 = mi.from_bits(x["b_bits"][sel], w.dtype).transpose(0, 2, 1)
    D64 = mi.from_bits(x["d_bits"][sel], w.dtype)
    local = np.array([[remap[b], i] for b, i in rows], dtype=np.int64)
    ref = oracle.chain_rows(A64, B64, D64, local, softmax=True, scale=w.scale)
    got = to_host64(E[torch.from_numpy(rows[:, 0]).cuda(), torch.from_numpy(rows[:, 1]).cuda()], w.dtype)
    scale = np.max(np.abs(ref))
    err = np.max(np.abs(got - ref))
    print(f"cfg5: max|err|/max|oracle| = {err / scale:.3e} over {len(rows)} rows", flush=True)
    assert err <= TOL * scale
    # property that holds at any size: each output is a convex combination of rows of V
    Dmax = torch.amax(D.float(), dim=1, keepdim=True)
    Dmin = torch.amin(D.float(), dim=1, keepdim=True)
    assert bool(((E.float() <= Dmax + 1e-2) & (E.float() >= Dmin - 1e-2)).all())


def test_edge_cases():
    dev = "cuda"
    # empty batch / M: no-op, N == 0: zeros (plain) or error (softmax)
    for shape in [(0, 64, 64, 64, 64), (2, 0, 64, 64, 64)]:
        b, M, K, N, L = shape
        A = torch.zeros((b, M, K), dtype=torch.float16, device=dev)
        B = torch.zeros((b, K, N), dtype=torch.float16, device=dev)
        D = torch.zeros((b, N, L), dtype=torch.float16, device=dev)
        assert tuple(mcf.gemm_chain(A, B, D).shape) == (b, M, L)
    A = torch.ones((2, 40, 64), dtype=torch.float16, device=dev)
    B = torch.zeros((2, 64, 0), dtype=torch.float16, device=dev)
    D = torch.zeros((2, 0, 64), dtype=torch.float16, device=dev)
    E = torch.full((2, 40, 64), 7.0, dtype=torch.float16, device=dev)
    mcf.gemm_chain(A, B, D, out=E)
    torch.cuda.synchronize()
    assert not E.any()
    with pytest.raises(mcf.McfError):
        mcf.softmax_gemm_chain(A, B, D, 1.0)
    # one row, one column (softmax over a single logit is 1 -> E = V)
    w = mi.make_problem(2, 1, 64, 1, 64, "bf16", True, "normal", seed=3)
    assert check_full(w) < TOL
    # negative and zero softmax scale
    w = mi.make_problem(2, 96, 32, 80, 32, "f16", True, "normal", seed=4)
    x = mi.make_inputs(w)
    A, B, D = device_inputs(w, x)
    for scale in (-0.3, 0.0):
        E = mcf.softmax_gemm_chain(A, B, D, scale)
        torch.cuda.synchronize()
        ref = oracle.chain(x["A"], x["B"], x["D"], softmax=True, scale=scale)
        assert np.max(np.abs(to_host64(E, "f16") - ref)) <= TOL * np.max(np.abs(ref))
    # strided (non-packed) operands and output
    w = mi.make_problem(2, 70, 64, 72, 64, "f16", False, "uniform", seed=5)
    x = mi.make_inputs(w)
    A, B, D = device_inputs(w, x)
    Abig = torch.zeros((2, 70, 128), dtype=torch.float16, device=dev); Abig[:, :, :64] = A
    Ebig = torch.zeros((2, 80, 64), dtype=torch.float16, device=dev)
    mcf.gemm_chain(Abig[:, :, :64], B, D, out=Ebig[:, :70, :])
    torch.cuda.synchronize()
    ref = oracle.chain(x["A"], x["B"], x["D"])
    assert np.max(np.abs(to_host64(Ebig[:, :70, :], "f16") - ref)) <= TOL * np.max(np.abs(ref))
    assert not Ebig[:, 70:, :].any()


def test_error_codes_from_the_abi():
    dev = "cuda"
    A = torch.zeros((1, 64, 64), dtype=torch.float16, device=dev)
    B = torch.zeros((1, 64, 64), dtype=torch.float16, device=dev)
    D = torch.zeros((1, 64, 64), dtype=torch.float16, device=dev)
    with pytest.raises(mcf.McfError) as e:          # K = 48 has no variant
        mcf.gemm_chain(A[:, :, :48], B[:, :48, :], D)
    assert e.value.status == 2
    with pytest.raises(mcf.McfError) as e:          # misaligned base pointer
        flat = torch.zeros(64 * 64 + 8, dtype=torch.float16, device=dev)
        mcf.gemm_chain(flat[1:1 + 4096].view(1, 64, 64), B, D)
    assert e.value.status == 3
    with pytest.raises(mcf.McfError) as e:          # output aliases an input
        mcf.gemm_chain(A, B, D, out=A)
    assert e.value.status == 1
    with pytest.raises(mcf.McfError) as e:          # no such wave arrangement
        mcf.gemm_chain(A, B, D, tiles=(3, 1, 1, 1))
    assert e.value.status == 1


def test_random_shapes_strides_and_tiles():
    """Seeded sweep: random (K, L) group, dtype, chain kind (plain, softmax, softmax under a causal
    mask with a random offset), output type (the input type or fp32), B layout, ragged or tiny M
    and N, non-packed row and batch strides on every operand and on the output, and a random
    built wave arrangement, each compared with the oracle element by element; the padding around
    a strided output must come back untouched."""
    # MCF_SWEEP_SEED / MCF_SWEEP_CASES: a longer or different sweep for a one-off run
    rng = np.random.default_rng(int(os.environ.get("MCF_SWEEP_SEED", "20250622")))
    n_cases = int(os.environ.get("MCF_SWEEP_CASES", "72"))
    groups = [(32, 32), (64, 64), (128, 128), (64, 128), (128, 64), (64, 256), (256, 256), (256, 128), (640, 64), (80, 80),
              (96, 96), (160, 160), (192, 192)]
    sizes = [1, 2, 7, 31, 32, 33, 64, 100, 129, 255, 300, 517]
    worst = 0.0
    for case in range(n_cases):
        K, L = groups[rng.integers(len(groups))]
        dtype = ("f16", "bf16")[rng.integers(2)]
        softmax = bool(rng.integers(2))
        nk = bool(rng.integers(2))                                  # B stored [b,N,K] (K contiguous)
        b = int(rng.integers(1, 4))
        M = int(sizes[rng.integers(len(sizes))])
        N = int(sizes[rng.integers(len(sizes))])
        if not nk:
            N = max(8, (N + 7) // 8 * 8)                            # N-contiguous B: N a multiple of 8
        pad = [int(8 * rng.integers(0, 3)) for _ in range(4)]       # extra row pitch of A, B, D, E
        causal = softmax and bool(rng.integers(2))
        offset = int((0, N - M, -M - 2, N, int(rng.integers(-M, N + 1)), int(rng.integers(-8, 9)))[rng.integers(6)]) if causal else None
        f32 = not rng.integers(3)                                   # fp32 output: every third case
        gap = [int(rng.integers(0, 3)) for _ in range(4)]           # extra rows between batches
        w = mi.make_problem(b, M, K, N, L, dtype, softmax, "normal" if softmax else "uniform", seed=9000 + case)
        x = mi.make_inputs(w)
        tdt = torch.float16 if dtype == "f16" else torch.bfloat16

        def strided(t, rows, cols, pad_c, gap_r, fill=0.0):
            big = torch.full((b, rows + gap_r, cols + pad_c), fill, dtype=tdt, device="cuda")
            big[:, :rows, :cols] = t
            return big, big[:, :rows, :cols]

        A0 = to_device(x["a_bits"], dtype)
        D0 = to_device(x["d_bits"], dtype)
        Bs = to_device(x["b_bits"], dtype)                           # [b,N,K] if b_layout == "nk" else [b,K,N]
        Bkn = Bs.transpose(1, 2) if x["b_layout"] == "nk" else Bs    # logical [b,K,N]
        _, A = strided(A0, M, K, pad[0], gap[0])
        if nk:
            _, Bnk = strided(Bkn.transpose(1, 2), N, K, pad[1], gap[1])
            B = Bnk.transpose(1, 2)
        else:
            _, B = strided(Bkn, K, N, pad[1], gap[1])
        _, D = strided(D0, N, L, pad[2], gap[2])
        Ebig = torch.full((b, M + gap[3], L + pad[3]), 5.0, dtype=torch.float32 if f32 else tdt, device="cuda")
        E = Ebig[:, :M, :L]
        prob = mcf.binding._problem_from_tensors(A, B, D, E)
        shapes = [(t.mb, t.rg, t.ns, t.nj, t.tl) for t in mcf.list_candidates(prob, softmax)]   # all T_L options
        shapes += [s for s in mcf.list_variants(prob, softmax)]           # and arrangements Rule 3 / the LDS rule would drop
        tiles = shapes[rng.integers(len(shapes))] if case % 4 else None   # every fourth case: the picker
        print(f"case {case}: b={b} M={M} K={K} N={N} L={L} {dtype} softmax={softmax} causal={offset} f32={f32} nk={nk} "
              f"pad={pad} gap={gap} tiles={tiles}", flush=True)
        if causal:
            mcf.causal_softmax_gemm_chain(A, B, D, w.scale, causal_offset=offset, out=E, tiles=tiles)
            ref = oracle.chain_causal(x["A"], x["B"], x["D"], w.scale, offset)
        elif softmax:
            mcf.softmax_gemm_chain(A, B, D, w.scale, out=E, tiles=tiles)
        else:
            mcf.gemm_chain(A, B, D, out=E, tiles=tiles)
        torch.cuda.synchronize()
        if not causal:
            ref = oracle.chain(x["A"], x["B"], x["D"], softmax=softmax, scale=w.scale)
        got = E.double().cpu().numpy() if f32 else to_host64(E, dtype)
        scale = np.max(np.abs(ref))
        err = np.max(np.abs(got - ref))
        assert err <= TOL * scale, f"case {case}: {err} > {TOL} * {scale}"
        worst = max(worst, err / scale if scale else 0.0)
        outside = Ebig.clone()
        outside[:, :M, :L] = 5.0
        assert bool((outside == 5.0).all()), f"case {case}: wrote outside the output view"
    print(f"worst max|err|/max|oracle| = {worst:.3e}", flush=True)


@pytest.mark.parametrize("softmax", [False, True])
def test_maximum_sizes_sampled(softmax):
    """Extents near the top of what one launch takes: more than 2^31 bytes of A and of E (the
    addresses need 64 bits), a quarter of a million blocks, and a batch count of 200 000.
    The long operand is drawn on the device by torch's seeded generator; the oracle sees the
    sampled rows of it copied back, and computes those rows one by one."""
    K = L = 64 if softmax else 32
    dtype, tdt = ("bf16", torch.bfloat16) if softmax else ("f16", torch.float16)
    M = (1 << 31) // (2 * K) + 37                      # row 2^31 / (2K) starts at byte offset 2^31
    N = 72
    gen = torch.Generator(device="cuda").manual_seed(777 + K)
    A = torch.empty((1, M, K), dtype=tdt, device="cuda")
    step = 1 << 22
    for r0 in range(0, M, step):                       # in pieces: no fp32 copy of the whole tensor
        A[0, r0:r0 + step] = torch.randn((min(step, M - r0), K), generator=gen, device="cuda").to(tdt)
    w = mi.make_problem(1, 8, K, N, L, dtype, softmax, "normal", seed=778)   # B and D from the usual recipe
    x = mi.make_inputs(w)
    _, B, D = device_inputs(w, x)
    print(f"case maximum sizes softmax={softmax} M={M}", flush=True)
    E = mcf.softmax_gemm_chain(A, B, D, w.scale) if softmax else mcf.gemm_chain(A, B, D)
    torch.cuda.synchronize()
    rng = np.random.default_rng(9)
    edge = (1 << 31) // (2 * K)
    rows = np.unique(np.concatenate([rng.integers(0, M, 400), np.arange(0, 40), np.arange(M - 40, M),
                                     np.arange(edge - 40, edge + 37)]))
    idx = torch.from_numpy(rows).cuda()
    A64 = to_host64(A[0, idx].unsqueeze(0), dtype)
    sel = np.stack([np.zeros(len(rows), dtype=np.int64), np.arange(len(rows))], axis=1)
    ref = oracle.chain_rows(A64, x["B"], x["D"], sel, softmax=softmax, scale=w.scale)
    got = to_host64(E[0, idx], dtype)
    assert np.max(np.abs(got - ref)) <= TOL * np.max(np.abs(ref))
    del A, E
    # many batches of a few rows each
    b = 200_000
    A = torch.randn((b, 8, K), generator=gen, device="cuda").to(tdt)
    Bb = torch.randn((b, N, K) if softmax else (b, K, N), generator=gen, device="cuda").to(tdt)
    Bb = Bb.transpose(1, 2) if softmax else Bb
    Db = torch.randn((b, N, L), generator=gen, device="cuda").to(tdt)
    print(f"case many batches softmax={softmax} batch={b}", flush=True)
    E = mcf.softmax_gemm_chain(A, Bb, Db, w.scale) if softmax else mcf.gemm_chain(A, Bb, Db)
    torch.cuda.synchronize()
    pick = torch.from_numpy(np.unique(np.concatenate([rng.integers(0, b, 60), [0, b - 1]]))).cuda()
    ref = oracle.chain(to_host64(A[pick], dtype), to_host64(Bb[pick], dtype), to_host64(Db[pick], dtype),
                       softmax=softmax, scale=w.scale)
    assert np.max(np.abs(to_host64(E[pick], dtype) - ref)) <= TOL * np.max(np.abs(ref))

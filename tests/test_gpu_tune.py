"""mcf_tune_tiles (Sec. IV-B, Alg. 1 measured on the device) through the C ABI: what it returns
is a feasible built variant, the log is consistent, and the chain run with the returned tiles
matches the fp64 oracle.  Needs an MI355X."""
import numpy as np
import pytest
import torch

import mcf_inputs as mi
import oracle
import paper_2506_22169_amd as mcf

from gpu_util import TOL, device_inputs, to_host64

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("softmax", [False, True])
def test_tune_returns_a_measured_feasible_variant(softmax):
    w = mi.make_problem(8, 512, 64, 384, 128, "f16", softmax, "normal" if softmax else "uniform", seed=4242)
    x = mi.make_inputs(w)
    A, B, D = device_inputs(w, x)
    E = torch.empty((w.batch, w.M, w.L), dtype=A.dtype, device="cuda")
    print(f"case tune softmax={softmax}", flush=True)
    best, rep = mcf.tune_tiles(A, B, D, scale=w.scale if softmax else None, out=E, launches=10, population=16,
                               top_n=4, seed=3)
    prob = mcf.binding._problem_from_tensors(A, B, D, E)
    shapes = [(t.mb, t.rg, t.ns, t.nj, t.tl) for t in mcf.list_candidates(prob, softmax)]
    entries = rep.entries()
    assert 1 <= rep.measured == len(entries) <= 4 * rep.generations
    assert rep.space == len(shapes)
    seen = [(e.mb, e.rg, e.ns, e.nj, e.tl) for e in entries]
    assert len(set(seen)) == len(seen) and all(s in shapes for s in seen)
    for e in entries:
        t = mcf.eval_tiles(prob, e.mb, e.rg, e.ns, e.nj, tl=e.tl, softmax=softmax)
        assert t.feasible and t.t_est_s == e.t_est_s and 0 < e.t_meas_s < 1e-2
    assert (best.mb, best.rg, best.ns, best.nj, best.tl) in seen
    assert rep.best_t_s == [e.t_meas_s for e, s in zip(entries, seen) if s == (best.mb, best.rg, best.ns, best.nj, best.tl)][0]
    fastest = min(e.t_meas_s for e in entries)
    assert rep.best_t_s <= fastest * 1.02 + 1e-12 if rep.converged else rep.best_t_s == fastest
    # E holds the result of the last measured launch; run once more with the returned tiles
    if softmax:
        mcf.softmax_gemm_chain(A, B, D, w.scale, out=E, tiles=best)
    else:
        mcf.gemm_chain(A, B, D, out=E, tiles=best)
    torch.cuda.synchronize()
    ref = oracle.chain(x["A"], x["B"], x["D"], softmax=softmax, scale=w.scale)
    assert np.max(np.abs(to_host64(E, "f16") - ref)) <= TOL * np.max(np.abs(ref))


def test_tune_passes_on_the_chain_calls_verdict():
    A = torch.zeros((1, 64, 64), dtype=torch.float16, device="cuda")
    B = torch.zeros((1, 64, 64), dtype=torch.float16, device="cuda")
    D = torch.zeros((1, 64, 64), dtype=torch.float16, device="cuda")
    with pytest.raises(mcf.McfError) as e:          # output aliases an input
        mcf.tune_tiles(A, B, D, out=A)
    assert e.value.status == 1
    with pytest.raises(mcf.McfError) as e:          # K = 48 has no kernels
        mcf.tune_tiles(A[:, :, :48], B[:, :48, :], D)
    assert e.value.status == 2


@pytest.mark.parametrize("softmax", [False, True])
def test_tune3_returns_a_measured_built_arrangement(softmax):
    """mcf_tune_tiles3: the same for the three-GEMM chain."""
    K, L, P = 64, 128, 128
    w = mi.make_problem(6, 512, K, 384, L, "f16", softmax, "normal" if softmax else "uniform", seed=4343)
    x = mi.make_inputs(w)
    A, B, D = device_inputs(w, x)
    f_bits = mi.to_bits(mi.draw(4343, 4, (w.batch, L, P), w.dist), "f16")
    F = torch.from_numpy(np.ascontiguousarray(f_bits).view(np.int16)).view(torch.float16).cuda()
    G = torch.empty((w.batch, w.M, P), dtype=A.dtype, device="cuda")
    print(f"case tune3 softmax={softmax}", flush=True)
    best, rep = mcf.tune_tiles3(A, B, D, F, scale=w.scale if softmax else None, out=G, launches=10, population=12, top_n=3, seed=5)
    prob = mcf.binding._problem_from_tensors(A, B, D, mcf.binding._MetaLike(A, D))
    shapes = [(t.mb, t.rg, t.ns, t.nj) for t in mcf.list_candidates3(prob, P, softmax)]
    entries = rep.entries()
    seen = [(e.mb, e.rg, e.ns, e.nj) for e in entries]
    assert rep.space == len(shapes) and 1 <= rep.measured == len(entries) <= 3 * rep.generations
    assert len(set(seen)) == len(seen) and all(s in shapes for s in seen) and all(0 < e.t_meas_s < 1e-2 for e in entries)
    assert (best.mb, best.rg, best.ns, best.nj) in seen and rep.best_t_s == min(e.t_meas_s for e in entries)
    mcf.gemm_chain3(A, B, D, F, scale=w.scale if softmax else None, out=G, tiles=(best.mb, best.rg, best.ns, best.nj))
    torch.cuda.synchronize()
    ref = oracle.chain3(x["A"], x["B"], x["D"], mi.from_bits(f_bits, "f16"), softmax=softmax, scale=w.scale)
    assert np.max(np.abs(to_host64(G, "f16") - ref)) <= TOL * np.max(np.abs(ref))
    with pytest.raises(mcf.McfError) as e:          # P without kernels
        mcf.tune_tiles3(A, B, D, torch.zeros((w.batch, L, 32), dtype=A.dtype, device="cuda"))
    assert e.value.status == 2

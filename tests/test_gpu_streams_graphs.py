"""The launches are asynchronous on the caller's stream and allocate nothing, so they can be
captured into a HIP graph and run on several streams at once.  Replays are checked against
the eager result every time, with eager work and synchronisations between them."""
import numpy as np
import pytest
import torch

import mcf_inputs as mi
import oracle
import paper_2506_22169_amd as mcf

from gpu_util import TOL, device_inputs, to_device, to_host64

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("softmax", [False, True])
def test_graph_replays_match_eager(softmax):
    w = mi.make_problem(4, 300, 64, 264, 64, "f16", softmax, "normal" if softmax else "uniform", seed=4242)
    x = mi.make_inputs(w)
    A, B, D = device_inputs(w, x)
    F = to_device(mi.to_bits(mi.draw(4242, 4, (4, 64, 64), w.dist), "f16"), "f16")
    scale = w.scale if softmax else None

    def run(E, G):
        if softmax:
            mcf.softmax_gemm_chain(A, B, D, w.scale, out=E)
        else:
            mcf.gemm_chain(A, B, D, out=E)
        mcf.gemm_chain3(A, B, D, F, scale=scale, out=G)

    E0, G0 = torch.empty((4, 300, 64), dtype=torch.float16, device="cuda"), torch.empty((4, 300, 64), dtype=torch.float16, device="cuda")
    run(E0, G0)                                  # eager: also sets the kernels' attributes before the capture
    torch.cuda.synchronize()
    ref = oracle.chain(x["A"], x["B"], x["D"], softmax=softmax, scale=w.scale)
    assert np.max(np.abs(to_host64(E0, "f16") - ref)) <= TOL * np.max(np.abs(ref))
    E1, G1 = torch.zeros_like(E0), torch.zeros_like(G0)
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):                    # the binding launches on torch's current (capturing) stream
        run(E1, G1)
    for rep in range(4):
        print(f"case graph replay {rep} softmax={softmax}", flush=True)
        E1.fill_(-3.0)                           # eager work between the replays
        G1.fill_(-3.0)
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        assert torch.equal(E1, E0) and torch.equal(G1, G0)     # same kernel, same inputs: bit-identical


def test_concurrent_streams():
    """Different problems on three streams at once; the kernels keep no state outside their
    arguments, so every result equals the one computed alone."""
    cases = []
    for i, (K, L, softmax) in enumerate(((64, 64, False), (128, 128, True), (32, 32, False))):
        w = mi.make_problem(6, 520, K, 400, L, "bf16", softmax, "normal" if softmax else "uniform", seed=4300 + i)
        x = mi.make_inputs(w)
        A, B, D = device_inputs(w, x)
        alone = mcf.softmax_gemm_chain(A, B, D, w.scale) if softmax else mcf.gemm_chain(A, B, D)
        cases.append((w, x, A, B, D, alone))
    torch.cuda.synchronize()
    streams = [torch.cuda.Stream() for _ in cases]          # default priority
    outs = [torch.empty_like(c[5]) for c in cases]
    print("case three streams", flush=True)
    for rep in range(20):
        for s, (w, x, A, B, D, alone), out in zip(streams, cases, outs):
            if w.softmax:
                mcf.softmax_gemm_chain(A, B, D, w.scale, out=out, stream=s)
            else:
                mcf.gemm_chain(A, B, D, out=out, stream=s)
    torch.cuda.synchronize()
    for (w, x, A, B, D, alone), out in zip(cases, outs):
        assert torch.equal(out, alone)
        ref = oracle.chain(x["A"], x["B"], x["D"], softmax=w.softmax, scale=w.scale)
        assert np.max(np.abs(to_host64(out, "bf16") - ref)) <= TOL * np.max(np.abs(ref))

"""Helpers for the GPU parity tests: move the seeded inputs to the device, call the HIP path
through the C ABI binding, and compare with the fp64 oracle."""
import numpy as np
import torch

import mcf_inputs as mi
import oracle
import paper_2506_22169_amd as mcf

TOL = 1e-2   # max|gpu - oracle| <= TOL * max|oracle| (fp16/bf16 inputs, fp32 accumulation)


def torch_dtype(name):
    return torch.float16 if name == "f16" else torch.bfloat16


def to_device(bits, dtype):
    """uint16 patterns -> device tensor of fp16/bf16 with the same bits."""
    t = torch.from_numpy(np.ascontiguousarray(bits).view(np.int16))
    return t.view(torch_dtype(dtype)).cuda()


def device_inputs(w, x):
    A = to_device(x["a_bits"], w.dtype)
    Bs = to_device(x["b_bits"], w.dtype)
    B = Bs.transpose(1, 2) if x["b_layout"] == "nk" else Bs
    D = to_device(x["d_bits"], w.dtype)
    return A, B, D


def to_host64(E, dtype):
    bits = E.contiguous().view(torch.int16).cpu().numpy().view(np.uint16)
    return mi.from_bits(bits, dtype)


def run_gpu(w, x, tiles=None, out=None):
    A, B, D = device_inputs(w, x)
    if w.softmax:
        E = mcf.softmax_gemm_chain(A, B, D, w.scale, out=out, tiles=tiles)
    else:
        E = mcf.gemm_chain(A, B, D, out=out, tiles=tiles)
    torch.cuda.synchronize()
    return E


def check_full(w, tiles=None, batch=None):
    """Element-by-element comparison of the whole output; returns max|err| / max|oracle|."""
    x = mi.make_inputs(w, batch=batch)
    E = to_host64(run_gpu(w, x, tiles), w.dtype)
    ref = oracle.chain(x["A"], x["B"], x["D"], softmax=w.softmax, scale=w.scale)
    assert E.shape == ref.shape
    assert np.isfinite(E).all()
    scale = np.max(np.abs(ref)) if ref.size else 0.0
    err = np.max(np.abs(E - ref)) if ref.size else 0.0
    assert err <= TOL * scale, f"{w.name} tiles={tiles}: max|err| {err:.4g} > {TOL} * {scale:.4g}"
    return err / scale if scale else 0.0

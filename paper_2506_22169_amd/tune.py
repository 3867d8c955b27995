"""Command-line front end of the search (Sec. IV-B, Alg. 1) and of the model check of Sec. VI-E:

    python -m paper_2506_22169_amd.tune --shape 64,512,64,512,64 --dtype f16 [--softmax] [--all]

runs mcf_tune_tiles on random operands of that shape (batch,M,K,N,L) and prints what was
measured; with --all it also times every feasible variant and prints the correlation between
the model's estimate and the measured time (the paper reports Pearson r of 0.80-0.92 for its
model on its hardware).  Needs an MI355X and the built library.
"""
import argparse
import math
import sys

import torch

from . import binding as mcf


def pearson(xs, ys):
    n = len(xs)
    mx, my = sum(xs) / n, sum(ys) / n
    sxy = sum((x - mx) * (y - my) for x, y in zip(xs, ys))
    sxx = sum((x - mx) ** 2 for x in xs)
    syy = sum((y - my) ** 2 for y in ys)
    return sxy / math.sqrt(sxx * syy) if sxx > 0 and syy > 0 else float("nan")


def time_variant(run, tiles, launches):
    """Seconds per launch of run(tiles): `launches` launches captured into a HIP graph (so that
    the Python call overhead is not in the figure), HIP events around one replay."""
    for _ in range(3):
        run(tiles)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        for _ in range(launches):
            run(tiles)
    graph.replay()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    graph.replay()
    e1.record()
    torch.cuda.synchronize()
    return e0.elapsed_time(e1) * 1e-3 / launches


def main(argv=None):
    ap = argparse.ArgumentParser(description=__doc__, formatter_class=argparse.RawDescriptionHelpFormatter)
    ap.add_argument("--shape", required=True, help="batch,M,K,N,L")
    ap.add_argument("--dtype", default="f16", choices=["f16", "bf16"])
    ap.add_argument("--softmax", action="store_true", help="softmax chain, B stored as [b,N,K], scale 1/sqrt(K)")
    ap.add_argument("--population", type=int, default=0)
    ap.add_argument("--top-n", type=int, default=0)
    ap.add_argument("--epsilon", type=float, default=0.0)
    ap.add_argument("--seed", type=int, default=0)
    ap.add_argument("--launches", type=int, default=50)
    ap.add_argument("--all", action="store_true", help="also time every feasible variant and print the correlation")
    a = ap.parse_args(argv)
    b, M, K, N, L = (int(v) for v in a.shape.split(","))
    dt = torch.float16 if a.dtype == "f16" else torch.bfloat16
    g = torch.Generator(device="cuda").manual_seed(1)
    A = torch.randn(b, M, K, device="cuda", generator=g).to(dt)
    B = torch.randn(b, N, K, device="cuda", generator=g).to(dt).transpose(1, 2) if a.softmax else \
        torch.randn(b, K, N, device="cuda", generator=g).to(dt)
    D = torch.randn(b, N, L, device="cuda", generator=g).to(dt)
    E = torch.empty(b, M, L, device="cuda", dtype=dt)
    scale = 1.0 / math.sqrt(K) if a.softmax else None

    best, rep = mcf.tune_tiles(A, B, D, scale=scale, out=E, launches=a.launches, population=a.population,
                               top_n=a.top_n, epsilon=a.epsilon, seed=a.seed)
    prob = mcf._problem_from_tensors(A, B, D, E)
    pick = mcf.pick_tiles(prob, a.softmax)
    print(f"shape b={b} M={M} K={K} N={N} L={L} {a.dtype}{' softmax' if a.softmax else ''}: "
          f"{rep.space} feasible variants, {rep.measured} measured in {rep.generations} generations, "
          f"{'converged' if rep.converged else 'generation bound reached'}")
    for e in rep.entries():
        print(f"  gen {e.generation}  ({e.mb},{e.rg},{e.ns},{e.nj}) T_L={e.tl}  model {e.t_est_s * 1e6:9.2f} us  measured {e.t_meas_s * 1e6:9.2f} us")
    print(f"search result ({best.mb},{best.rg},{best.ns},{best.nj}) T_L={best.tl} at {rep.best_t_s * 1e6:.2f} us; "
          f"closed-form pick ({pick.mb},{pick.rg},{pick.ns},{pick.nj}) T_L={pick.tl}")
    if a.all:
        def run(t):
            if a.softmax:
                mcf.softmax_gemm_chain(A, B, D, scale, out=E, tiles=t)
            else:
                mcf.gemm_chain(A, B, D, out=E, tiles=t)
        est, meas = [], []
        for t in mcf.list_candidates(prob, a.softmax):
            v = (t.mb, t.rg, t.ns, t.nj, t.tl)
            s = time_variant(run, v, a.launches)
            est.append(t.t_est_s)
            meas.append(s)
            print(f"  all  {v}  model {t.t_est_s * 1e6:9.2f} us  measured {s * 1e6:9.2f} us")
        print(f"pearson r(model, measured) over {len(est)} variants = {pearson(est, meas):.3f}; "
              f"fastest measured {min(meas) * 1e6:.2f} us, search result {rep.best_t_s * 1e6:.2f} us")
    return 0


if __name__ == "__main__":
    sys.exit(main())

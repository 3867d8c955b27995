"""fp64 CPU oracle for the fused MBCI chain (test infrastructure only).

Only tests/, __graft_entry__.smoke() and bench.py's cpu_baseline leg may import this package.
It shares no code with the HIP path and never imports it.

  chain.py       ctypes front end of mcf_oracle.c (the chain E = (A.B).D, optional row softmax)
  perf_model.py  the paper's tiling-expression traffic rules and analytical model, eq. (1)-(5)
  search.py      the paper's heuristic search over candidates, Alg. 1
"""
from .chain import chain, chain_rows, chain3, chain_causal, intermediate_row, build_oracle  # noqa: F401

"""MI355X-native fused MBCI operator chains (MCFuser, arXiv 2506.22169): thin Python binding
over the C ABI of libmcf.so.  Every step of the path runs in the HIP kernels; this package
only marshals arguments.  Importing works without the built library, calling does not."""
from .binding import (  # noqa: F401
    McfError, Problem, Tiles, gemm_chain, softmax_gemm_chain, causal_softmax_gemm_chain, gemm_chain3, list_variants3, pick_tiles3, pick_tiles, eval_tiles,
    list_variants, list_candidates, library_path, load_library, status_string, search_tiles, tune_tiles, SearchParams,
    SearchReport, probe_copy, probe_mfma, probe_empty, SpaceReport, expressions, expression_trips, sub_expression, enumerate_space,
    list_candidates3, search_tiles3, tune_tiles3,
)

"""ctypes binding of include/mcf.h (same names, argument marshalling only).

torch is used for device memory and streams: tensors come in as torch CUDA(=HIP) tensors,
their data pointers, strides and the current stream are handed to the C ABI.
"""
import ctypes
import os

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "libmcf.so")
_lib = None

MCF_F16, MCF_BF16, MCF_F32 = 0, 1, 2
MCF_OK = 0


class McfError(RuntimeError):
    def __init__(self, status, text):
        super().__init__(text)
        self.status = status


class Problem(ctypes.Structure):
    """struct mcf_problem"""
    _fields_ = [("batch", ctypes.c_int64), ("M", ctypes.c_int64), ("K", ctypes.c_int64),
                ("N", ctypes.c_int64), ("L", ctypes.c_int64),
                ("in_dtype", ctypes.c_int32), ("out_dtype", ctypes.c_int32),
                ("a_stride", ctypes.c_int64 * 3), ("b_stride", ctypes.c_int64 * 3),
                ("d_stride", ctypes.c_int64 * 3), ("e_stride", ctypes.c_int64 * 3)]


class Tiles(ctypes.Structure):
    """struct mcf_tiles"""
    _fields_ = [("tm", ctypes.c_int32), ("tn", ctypes.c_int32), ("tk", ctypes.c_int32), ("tl", ctypes.c_int32),
                ("mb", ctypes.c_int32), ("rg", ctypes.c_int32), ("ns", ctypes.c_int32), ("nj", ctypes.c_int32),
                ("waves", ctypes.c_int32), ("stages", ctypes.c_int32), ("lds_bytes", ctypes.c_int32), ("vgpr_est", ctypes.c_int32),
                ("vgpr_used", ctypes.c_int32), ("scratch_bytes", ctypes.c_int32),
                ("blocks", ctypes.c_int64), ("compulsory_bytes", ctypes.c_int64),
                ("model_bytes", ctypes.c_int64), ("flops", ctypes.c_int64),
                ("t_mem_s", ctypes.c_double), ("t_comp_s", ctypes.c_double),
                ("alpha", ctypes.c_double), ("t_est_s", ctypes.c_double)]

    def as_dict(self):
        return {n: getattr(self, n) for n, _ in self._fields_}


MCF_MAX_SUB_EXPRESSIONS = 8
MCF_TRIPS_NO_HOIST, MCF_TRIPS_KEEP_UNIT_LOOPS, MCF_TRIPS_BIND_BLOCK = 1, 2, 4


class SpaceReport(ctypes.Structure):
    """struct mcf_space_report"""
    _fields_ = [("n_deep", ctypes.c_int32), ("n_flat", ctypes.c_int32), ("n_rule1", ctypes.c_int32), ("n_rule2", ctypes.c_int32),
                ("sub_expression", (ctypes.c_char * 16) * MCF_MAX_SUB_EXPRESSIONS),
                ("sub_members", ctypes.c_int32 * MCF_MAX_SUB_EXPRESSIONS), ("sub_kept", ctypes.c_int32 * MCF_MAX_SUB_EXPRESSIONS),
                ("tile_choices", ctypes.c_int64), ("after_rule3", ctypes.c_int64), ("after_rule4", ctypes.c_int64),
                ("candidates", ctypes.c_int64), ("candidates_pruned", ctypes.c_int64),
                ("built_deep", ctypes.c_int64), ("built_flat", ctypes.c_int64)]

    def subs(self):
        """{sub-expression: (members, kept)}"""
        return {self.sub_expression[i].value.decode(): (self.sub_members[i], bool(self.sub_kept[i])) for i in range(self.n_rule1)}


class SearchParams(ctypes.Structure):
    """struct mcf_search_params"""
    _fields_ = [("population", ctypes.c_int32), ("top_n", ctypes.c_int32), ("max_generations", ctypes.c_int32),
                ("reserved", ctypes.c_int32), ("epsilon", ctypes.c_double), ("seed", ctypes.c_uint64)]


class SearchEntry(ctypes.Structure):
    """struct mcf_search_entry"""
    _fields_ = [("mb", ctypes.c_int32), ("rg", ctypes.c_int32), ("ns", ctypes.c_int32), ("nj", ctypes.c_int32),
                ("generation", ctypes.c_int32), ("tl", ctypes.c_int32),
                ("t_est_s", ctypes.c_double), ("t_meas_s", ctypes.c_double)]


SEARCH_LOG_MAX = 64


class SearchReport(ctypes.Structure):
    """struct mcf_search_report"""
    _fields_ = [("space", ctypes.c_int32), ("generations", ctypes.c_int32), ("measured", ctypes.c_int32),
                ("converged", ctypes.c_int32), ("best_t_s", ctypes.c_double), ("log", SearchEntry * SEARCH_LOG_MAX)]

    def entries(self):
        return [self.log[i] for i in range(self.measured)]


MEASURE_FN = ctypes.CFUNCTYPE(ctypes.c_double, ctypes.POINTER(Tiles), ctypes.c_void_p)


def library_path():
    return _LIB_PATH


def load_library():
    """Load libmcf.so; raises if it has not been built (there is no fallback path)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(_LIB_PATH):
        raise McfError(-1, f"{_LIB_PATH} is missing: build it with "
                           "`python -m paper_2506_22169_amd.build` (hipcc, gfx950); there is no fallback")
    lib = ctypes.CDLL(_LIB_PATH)
    PP, TP, vp = ctypes.POINTER(Problem), ctypes.POINTER(Tiles), ctypes.c_void_p
    lib.mcf_pick_tiles.argtypes = [PP, ctypes.c_int, TP]
    lib.mcf_eval_tiles.argtypes = [PP, ctypes.c_int, TP]
    lib.mcf_list_variants.argtypes = [PP, ctypes.c_int, ctypes.POINTER(ctypes.c_int32), ctypes.c_int]
    lib.mcf_list_candidates.argtypes = [PP, ctypes.c_int, TP, ctypes.c_int]
    SP, RP = ctypes.POINTER(SearchParams), ctypes.POINTER(SearchReport)
    lib.mcf_search_tiles.argtypes = [PP, ctypes.c_int, SP, MEASURE_FN, vp, TP, RP]
    lib.mcf_tune_tiles.argtypes = [PP, ctypes.c_int, ctypes.c_float, vp, vp, vp, vp, SP, ctypes.c_int, vp, TP, RP]
    lib.mcf_gemm_chain.argtypes = [PP, vp, vp, vp, vp, TP, vp]
    lib.mcf_gemm_chain3.argtypes = [PP, ctypes.c_int, ctypes.c_float, ctypes.c_int64, ctypes.POINTER(ctypes.c_int64),
                                    vp, vp, vp, vp, vp, TP, vp]
    lib.mcf_pick_tiles3.argtypes = [PP, ctypes.c_int64, ctypes.c_int, TP]
    lib.mcf_list_candidates3.argtypes = [PP, ctypes.c_int64, ctypes.c_int, TP, ctypes.c_int]
    lib.mcf_search_tiles3.argtypes = [PP, ctypes.c_int64, ctypes.c_int, ctypes.POINTER(SearchParams), MEASURE_FN, vp, TP,
                                      ctypes.POINTER(SearchReport)]
    lib.mcf_tune_tiles3.argtypes = [PP, ctypes.c_int, ctypes.c_float, ctypes.c_int64, ctypes.POINTER(ctypes.c_int64), vp, vp, vp,
                                    vp, vp, ctypes.POINTER(SearchParams), ctypes.c_int, vp, TP, ctypes.POINTER(SearchReport)]
    for f in (lib.mcf_list_candidates3, lib.mcf_search_tiles3, lib.mcf_tune_tiles3):
        f.restype = ctypes.c_int
    lib.mcf_list_variants3.argtypes = [PP, ctypes.c_int64, ctypes.c_int, ctypes.POINTER(ctypes.c_int32), ctypes.c_int]
    lib.mcf_softmax_gemm_chain.argtypes = [PP, ctypes.c_float, vp, vp, vp, vp, TP, vp]
    lib.mcf_causal_softmax_gemm_chain.argtypes = [PP, ctypes.c_float, ctypes.c_int64, vp, vp, vp, vp, TP, vp]
    lib.mcf_causal_softmax_gemm_chain.restype = ctypes.c_int
    for f in (lib.mcf_pick_tiles, lib.mcf_eval_tiles, lib.mcf_list_variants, lib.mcf_gemm_chain,
              lib.mcf_softmax_gemm_chain, lib.mcf_search_tiles, lib.mcf_tune_tiles, lib.mcf_list_candidates,
              lib.mcf_gemm_chain3, lib.mcf_list_variants3, lib.mcf_pick_tiles3):
        f.restype = ctypes.c_int
    lib.mcf_probe_copy.argtypes = [vp, vp, ctypes.c_int64, vp]
    lib.mcf_probe_mfma.argtypes = [vp, ctypes.c_int32, ctypes.c_int32, ctypes.c_int32, vp]
    lib.mcf_probe_empty.argtypes = [ctypes.c_int32, vp]
    for f in (lib.mcf_probe_copy, lib.mcf_probe_mfma, lib.mcf_probe_empty):
        f.restype = ctypes.c_int
    lib.mcf_expression.argtypes = [ctypes.c_int, ctypes.c_char_p, ctypes.c_int]
    lib.mcf_expression_trips.argtypes = [ctypes.c_char_p, ctypes.POINTER(ctypes.c_int64), ctypes.c_int, ctypes.POINTER(ctypes.c_int64)]
    lib.mcf_sub_expression.argtypes = [ctypes.c_char_p, ctypes.c_char_p, ctypes.c_int, ctypes.POINTER(ctypes.c_int)]
    lib.mcf_enumerate_space.argtypes = [PP, ctypes.c_int, ctypes.c_int64, ctypes.POINTER(SpaceReport)]
    for f in (lib.mcf_expression, lib.mcf_expression_trips, lib.mcf_sub_expression, lib.mcf_enumerate_space):
        f.restype = ctypes.c_int
    lib.mcf_status_string.argtypes = [ctypes.c_int]
    lib.mcf_status_string.restype = ctypes.c_char_p
    lib.mcf_last_error.argtypes = []
    lib.mcf_last_error.restype = ctypes.c_char_p
    _lib = lib
    return lib


def status_string(status):
    return load_library().mcf_status_string(int(status)).decode()


def _check(status):
    if status != MCF_OK:
        lib = load_library()
        extra = lib.mcf_last_error().decode()
        raise McfError(status, status_string(status) + (f" ({extra})" if extra else ""))


def _dtype_code(t):
    import torch
    if t.dtype == torch.float16:
        return MCF_F16
    if t.dtype == torch.bfloat16:
        return MCF_BF16
    raise McfError(2, f"unsupported dtype {t.dtype}")


def make_problem(batch, M, K, N, L, dtype, a_stride=None, b_stride=None, d_stride=None, e_stride=None):
    """mcf_problem from plain numbers; dtype is 'f16' / 'bf16' or an mcf_dtype code."""
    code = {"f16": MCF_F16, "bf16": MCF_BF16}.get(dtype, dtype)
    p = Problem(batch, M, K, N, L, code, code)
    for name, s in (("a_stride", a_stride), ("b_stride", b_stride), ("d_stride", d_stride), ("e_stride", e_stride)):
        if s is not None:
            setattr(p, name, (ctypes.c_int64 * 3)(*s))
    return p


def _problem_from_tensors(A, B, D, E):
    if A.dim() != 3 or B.dim() != 3 or D.dim() != 3 or E.dim() != 3:
        raise McfError(1, "A, B, D, E must be 3-d [batch, rows, cols]")
    b, M, K = A.shape
    b2, K2, N = B.shape
    b3, N2, L = D.shape
    if not (b == b2 == b3 and K == K2 and N == N2 and tuple(E.shape) == (b, M, L)):
        raise McfError(1, f"shape mismatch A{tuple(A.shape)} B{tuple(B.shape)} D{tuple(D.shape)} E{tuple(E.shape)}")
    import torch
    if not (A.dtype == B.dtype == D.dtype and E.dtype in (A.dtype, torch.float32)):
        raise McfError(1, "A, B, D must share one dtype; E has that dtype or float32")
    if not (A.is_cuda and B.is_cuda and D.is_cuda and E.is_cuda):
        raise McfError(1, "A, B, D, E must be device tensors")
    if not (A.device == B.device == D.device == E.device):
        raise McfError(1, "A, B, D, E must live on one device")
    code = _dtype_code(A)

    def st(t):
        # an empty tensor has no meaningful strides (None = packed); neither has a
        # dimension of extent <= 1: give it the packed one
        if t.numel() == 0:
            return None
        s = list(t.stride())
        shape = list(t.shape)
        if shape[2] <= 1:
            # a single column: keep a row-contiguous (transposed) view recognisable as such
            s[2] = shape[1] if (s[1] == 1 and shape[1] > 1) else 1
        if shape[1] <= 1:
            s[1] = max(shape[2], 1) if s[2] == 1 else 1
        if shape[0] <= 1:
            s[0] = 0
        return s
    p = make_problem(b, M, K, N, L, code, st(A), st(B), st(D), st(E))
    if E.dtype == torch.float32:
        p.out_dtype = MCF_F32
    return p


def _stream_ptr(stream):
    import torch
    if stream is None:
        stream = torch.cuda.current_stream()
    return ctypes.c_void_p(stream.cuda_stream if hasattr(stream, "cuda_stream") else int(stream))


def _tiles_arg(tiles):
    if tiles is None:
        return None
    if isinstance(tiles, Tiles):
        return ctypes.byref(tiles)
    t = Tiles()
    t.mb, t.rg, t.ns, t.nj = tiles[:4]
    t.tl = tiles[4] if len(tiles) > 4 else 0    # (mb, rg, ns, nj[, tl]); tl = 0 means T_L = L
    return ctypes.byref(t)


def _run(softmax, scale, A, B, D, out, tiles, stream, causal_offset=None):
    import torch
    lib = load_library()
    if out is None:
        out = torch.empty((A.shape[0], A.shape[1], D.shape[2]), dtype=A.dtype, device=A.device)
    p = _problem_from_tensors(A, B, D, out)
    args = [ctypes.c_void_p(A.data_ptr()), ctypes.c_void_p(B.data_ptr()), ctypes.c_void_p(D.data_ptr()),
            ctypes.c_void_p(out.data_ptr()), _tiles_arg(tiles), _stream_ptr(stream)]
    if causal_offset is not None:
        _check(lib.mcf_causal_softmax_gemm_chain(ctypes.byref(p), ctypes.c_float(scale), ctypes.c_int64(int(causal_offset)), *args))
    elif softmax:
        _check(lib.mcf_softmax_gemm_chain(ctypes.byref(p), ctypes.c_float(scale), *args))
    else:
        _check(lib.mcf_gemm_chain(ctypes.byref(p), *args))
    return out


def gemm_chain(A, B, D, out=None, tiles=None, stream=None):
    """mcf_gemm_chain: E = (A . B) . D on device tensors A[b,M,K], B[b,K,N] (any of the two
    supported layouts, e.g. a transposed view of [b,N,K]), D[b,N,L].  tiles: None (picker),
    a Tiles struct or an (mb, rg, ns, nj) tuple."""
    return _run(False, 1.0, A, B, D, out, tiles, stream)


def softmax_gemm_chain(A, B, D, scale, out=None, tiles=None, stream=None):
    """mcf_softmax_gemm_chain: E = softmax_rows(scale * A . B) . D."""
    return _run(True, float(scale), A, B, D, out, tiles, stream)


def causal_softmax_gemm_chain(A, B, D, scale, causal_offset=0, out=None, tiles=None, stream=None):
    """mcf_causal_softmax_gemm_chain: the softmax chain with row i seeing the columns n <= i + causal_offset."""
    return _run(True, float(scale), A, B, D, out, tiles, stream, causal_offset=causal_offset)


def pick_tiles(problem, softmax=False):
    """mcf_pick_tiles on an mcf_problem (see make_problem); host only."""
    t = Tiles()
    _check(load_library().mcf_pick_tiles(ctypes.byref(problem), int(bool(softmax)), ctypes.byref(t)))
    return t


def eval_tiles(problem, mb, rg, ns, nj=1, tl=0, softmax=False):
    """mcf_eval_tiles: model terms of a caller-chosen wave arrangement (and T_L; 0 = L); host only."""
    t = Tiles()
    t.mb, t.rg, t.ns, t.nj, t.tl = mb, rg, ns, nj, tl
    st = load_library().mcf_eval_tiles(ctypes.byref(problem), int(bool(softmax)), ctypes.byref(t))
    if st not in (MCF_OK, 1):     # MCF_EINVAL = evaluated, but over a budget: terms are filled in
        _check(st)
    t.feasible = (st == MCF_OK)
    return t


def list_candidates(problem, softmax=False):
    """mcf_list_candidates: the feasible candidates (Tiles with model terms) the picker and the
    search choose from, T_L = L first, then every smaller T_L that has kernels."""
    lib = load_library()
    n = lib.mcf_list_candidates(ctypes.byref(problem), int(bool(softmax)), None, 0)
    buf = (Tiles * max(n, 1))()
    lib.mcf_list_candidates(ctypes.byref(problem), int(bool(softmax)), buf, n)
    return [buf[i] for i in range(n)]


def list_variants(problem, softmax=False):
    """mcf_list_variants: (mb, rg, ns, nj) of every built kernel variant that covers the shape."""
    lib = load_library()
    n = lib.mcf_list_variants(ctypes.byref(problem), int(bool(softmax)), None, 0)
    buf = (ctypes.c_int32 * (4 * max(n, 1)))()
    lib.mcf_list_variants(ctypes.byref(problem), int(bool(softmax)), buf, n)
    return [tuple(buf[4 * i:4 * i + 4]) for i in range(n)]


def _search_params(population, top_n, epsilon, seed, max_generations):
    sp = SearchParams()
    sp.population, sp.top_n, sp.max_generations = int(population), int(top_n), int(max_generations)
    sp.epsilon, sp.seed = float(epsilon), int(seed)
    return sp


def search_tiles(problem, softmax, measure, population=0, top_n=0, epsilon=0.0, seed=0, max_generations=0, P=0):
    """mcf_search_tiles: Alg. 1 with `measure(Tiles) -> seconds` as the measurement; zero
    parameters read as the library defaults.  Returns (Tiles, SearchReport)."""
    failure = []

    def cb(tp, _user):
        try:
            return float(measure(tp.contents))
        except Exception as e:   # an exception cannot cross the C frame: report it as a failed measurement
            failure.append(e)
            return -1.0

    sp = _search_params(population, top_n, epsilon, seed, max_generations)
    best, rep = Tiles(), SearchReport()
    if P:
        st = load_library().mcf_search_tiles3(ctypes.byref(problem), int(P), int(bool(softmax)), ctypes.byref(sp), MEASURE_FN(cb),
                                              None, ctypes.byref(best), ctypes.byref(rep))
    else:
        st = load_library().mcf_search_tiles(ctypes.byref(problem), int(bool(softmax)), ctypes.byref(sp), MEASURE_FN(cb),
                                             None, ctypes.byref(best), ctypes.byref(rep))
    if failure:
        raise failure[0]
    _check(st)
    return best, rep


def search_tiles3(problem, P, softmax, measure, **kw):
    """mcf_search_tiles3: Alg. 1 over the arrangements built for the three-GEMM chain."""
    return search_tiles(problem, softmax, measure, P=P, **kw)


def list_candidates3(problem, P, softmax=False):
    """mcf_list_candidates3: the arrangements built for the three-GEMM chain with the model terms of
    their two-GEMM part."""
    lib = load_library()
    n = lib.mcf_list_candidates3(ctypes.byref(problem), int(P), int(bool(softmax)), None, 0)
    buf = (Tiles * max(n, 1))()
    lib.mcf_list_candidates3(ctypes.byref(problem), int(P), int(bool(softmax)), buf, n)
    return [buf[i] for i in range(n)]


def tune_tiles(A, B, D, scale=None, out=None, launches=0, population=0, top_n=0, epsilon=0.0, seed=0,
               max_generations=0, stream=None):
    """mcf_tune_tiles: Alg. 1 measured on the device over these tensors (scale=None: plain
    chain, otherwise the softmax chain).  `out` is overwritten.  Returns (Tiles, SearchReport)."""
    import torch
    if out is None:
        out = torch.empty((A.shape[0], A.shape[1], D.shape[2]), dtype=A.dtype, device=A.device)
    p = _problem_from_tensors(A, B, D, out)
    sp = _search_params(population, top_n, epsilon, seed, max_generations)
    best, rep = Tiles(), SearchReport()
    _check(load_library().mcf_tune_tiles(
        ctypes.byref(p), int(scale is not None), ctypes.c_float(0.0 if scale is None else scale),
        ctypes.c_void_p(A.data_ptr()), ctypes.c_void_p(B.data_ptr()), ctypes.c_void_p(D.data_ptr()),
        ctypes.c_void_p(out.data_ptr()), ctypes.byref(sp), int(launches), _stream_ptr(stream),
        ctypes.byref(best), ctypes.byref(rep)))
    return best, rep


def gemm_chain3(A, B, D, F, scale=None, out=None, tiles=None, stream=None, _tune=None):
    """mcf_gemm_chain3: G = ((A . B) . D) . F, or (softmax_rows(scale * A . B) . D) . F when scale is
    given, on device tensors; F[b,L,P] with unit column stride, G[b,M,P]."""
    import torch
    lib = load_library()
    if F.dim() != 3 or F.shape[0] != A.shape[0] or F.shape[1] != D.shape[2]:
        raise McfError(1, f"F{tuple(F.shape)} does not continue D{tuple(D.shape)}")
    P = F.shape[2]
    if out is None:
        out = torch.empty((A.shape[0], A.shape[1], P), dtype=A.dtype, device=A.device)
    if tuple(out.shape) != (A.shape[0], A.shape[1], P) or not (F.dtype == A.dtype and out.dtype in (A.dtype, torch.float32)) \
            or out.device != A.device or F.device != A.device:
        raise McfError(1, "F and the output must match A in dtype and device, the output be [b, M, P]")
    # A, B, D as in the two-GEMM chain (a stand-in E of the right shape carries no strides)
    p = _problem_from_tensors(A, B, D, _MetaLike(A, D))
    if out.dtype == torch.float32:
        p.out_dtype = MCF_F32
    so = list(out.stride()) if out.numel() else [0, 0, 0]
    if out.shape[0] <= 1:
        so[0] = 0
    if out.shape[1] <= 1:
        so[1] = max(P, 1)
    for d in range(3):
        p.e_stride[d] = so[d]
    sf = list(F.stride()) if F.numel() else [0, 0, 0]
    if F.shape[0] <= 1:
        sf[0] = 0
    fs = (ctypes.c_int64 * 3)(*sf)
    ptrs = [ctypes.c_void_p(t.data_ptr()) for t in (A, B, D, F, out)]
    if _tune is not None:      # mcf_tune_tiles3 over the same arguments
        sp = _search_params(*_tune["search"])
        best, rep = Tiles(), SearchReport()
        _check(lib.mcf_tune_tiles3(ctypes.byref(p), int(scale is not None), ctypes.c_float(0.0 if scale is None else scale),
                                   ctypes.c_int64(P), fs, *ptrs, ctypes.byref(sp), int(_tune["launches"]), _stream_ptr(stream),
                                   ctypes.byref(best), ctypes.byref(rep)))
        return best, rep
    _check(lib.mcf_gemm_chain3(ctypes.byref(p), int(scale is not None), ctypes.c_float(0.0 if scale is None else scale),
                               ctypes.c_int64(P), fs, *ptrs, _tiles_arg(tiles), _stream_ptr(stream)))
    return out


def tune_tiles3(A, B, D, F, scale=None, out=None, launches=0, population=0, top_n=0, epsilon=0.0, seed=0,
                max_generations=0, stream=None):
    """mcf_tune_tiles3: Alg. 1 measured on the device for the three-GEMM chain over these tensors.
    `out` is overwritten.  Returns (Tiles, SearchReport)."""
    return gemm_chain3(A, B, D, F, scale=scale, out=out, stream=stream,
                       _tune={"search": (population, top_n, epsilon, seed, max_generations), "launches": launches})


class _MetaLike:
    """Shape / stride stand-in for the E of a three-GEMM chain (it exists only in registers)."""

    def __init__(self, A, D):
        self.shape = (A.shape[0], A.shape[1], D.shape[2])
        self.dtype, self.is_cuda, self.device = A.dtype, True, A.device

    def dim(self):
        return 3

    def numel(self):
        return 0      # no strides of its own: packed


def pick_tiles3(problem, P, softmax=False):
    """mcf_pick_tiles3: the arrangement gemm_chain3 takes when given no tiles."""
    lib = load_library()
    t = Tiles()
    _check(lib.mcf_pick_tiles3(ctypes.byref(problem), int(P), int(bool(softmax)), ctypes.byref(t)))
    return t


def list_variants3(problem, P, softmax=False):
    """mcf_list_variants3: (mb, rg, ns, nj) built for the three-GEMM chain of this shape."""
    lib = load_library()
    n = lib.mcf_list_variants3(ctypes.byref(problem), int(P), int(bool(softmax)), None, 0)
    buf = (ctypes.c_int32 * (4 * max(n, 1)))()
    lib.mcf_list_variants3(ctypes.byref(problem), int(P), int(bool(softmax)), buf, n)
    return [tuple(buf[4 * i:4 * i + 4]) for i in range(n)]


def expressions():
    """mcf_expression: the 24 deep and the 2 flat tiling expressions of Sec. III-A; host only."""
    lib, out, buf = load_library(), [], ctypes.create_string_buffer(16)
    i = 0
    while lib.mcf_expression(i, buf, 16) == MCF_OK:
        out.append(buf.value.decode())
        i += 1
    return out


def expression_trips(expr, extents, flags=0):
    """mcf_expression_trips: {statement: trips} for extents given as a dict over 'mnkh'; host only."""
    ext = (ctypes.c_int64 * 4)(*(int(extents[l]) for l in "mnkh"))
    t = (ctypes.c_int64 * 6)()
    _check(load_library().mcf_expression_trips(expr.encode(), ext, int(flags), t))
    return dict(zip(("C_C", "C_E", "L_A", "L_B", "L_D", "S_E"), t))


def sub_expression(expr):
    """mcf_sub_expression: (what a block runs under Rule 1, whether that passes Rule 2); host only."""
    buf, ok = ctypes.create_string_buffer(16), ctypes.c_int(0)
    _check(load_library().mcf_sub_expression(expr.encode(), buf, 16, ctypes.byref(ok)))
    return buf.value.decode(), bool(ok.value)


def enumerate_space(problem, softmax=False, shm_max_bytes=0):
    """mcf_enumerate_space: the sizes of the search space before and after Rules 1-4; host only."""
    r = SpaceReport()
    _check(load_library().mcf_enumerate_space(ctypes.byref(problem), int(bool(softmax)), int(shm_max_bytes), ctypes.byref(r)))
    return r


def probe_copy(dst, src, stream=None):
    """mcf_probe_copy: dst = src (device tensors of equal byte size), the streaming-copy ceiling."""
    nbytes = src.numel() * src.element_size()
    if dst.numel() * dst.element_size() != nbytes:
        raise McfError(1, "probe_copy: sizes differ")
    _check(load_library().mcf_probe_copy(ctypes.c_void_p(dst.data_ptr()), ctypes.c_void_p(src.data_ptr()),
                                         ctypes.c_int64(nbytes), _stream_ptr(stream)))


def probe_mfma(out, blocks, waves_per_block, iters, stream=None):
    """mcf_probe_mfma: blocks x waves_per_block waves of iters x 8 MFMAs each; out is a float32
    device tensor of at least blocks * waves_per_block * 64 elements."""
    if out.numel() < blocks * waves_per_block * 64:
        raise McfError(1, "probe_mfma: output too small")
    _check(load_library().mcf_probe_mfma(ctypes.c_void_p(out.data_ptr()), int(blocks), int(waves_per_block), int(iters),
                                         _stream_ptr(stream)))


def probe_empty(blocks, stream=None):
    """mcf_probe_empty: a kernel that does nothing (the launch floor)."""
    _check(load_library().mcf_probe_empty(int(blocks), _stream_ptr(stream)))

/*
 * mcf -- fused memory-bound compute-intensive (MBCI) operator chains on AMD MI355X (gfx950).
 *
 * C ABI of the library.  Plain C, no exceptions cross this boundary; every call returns an
 * mcf_status.  The operation is the two-GEMM chain of MCFuser (arXiv 2506.22169):
 *
 *   Sec. III-A (GEMM chain C = A x B, E = C x D) and Sec. VI-B1 (batched form):
 *       C[b] = A[b] . B[b]        A[b]: M x K,  B[b]: K x N
 *       E[b] = C[b] . D[b]        D[b]: N x L   (the paper's H is called L here)
 *   Sec. VI-B2 (self-attention module: the same chain with a softmax between the GEMMs):
 *       E[b] = softmax_rows(scale * A[b] . B[b]) . D[b]
 *
 * computed by ONE kernel in which the intermediate C (or S/P) lives in registers only and
 * never reaches device memory (Sec. II-B "Redundant Memory Access", Sec. III-B).  The tile
 * shape is taken from the analytical model of Sec. IV-A, eq. (2)-(5), under the on-chip
 * memory rule of Sec. III-C, eq. (1), instead of a search.
 *
 * Memory: A, B, D, E are DEVICE pointers owned by the caller (e.g. PyTorch allocations).
 * The mcf_problem / mcf_tiles structs are HOST memory.  The library allocates nothing on the
 * device, never synchronises, and launches asynchronously on the caller's stream.
 */
#ifndef MCF_H
#define MCF_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum { MCF_F16 = 0, MCF_BF16 = 1, MCF_F32 = 2 /* output only */ } mcf_dtype;

typedef enum {
    MCF_OK = 0,
    MCF_EINVAL = 1,       /* null pointer, negative dimension, bad stride, aliasing, bad tiles   */
    MCF_EUNSUPPORTED = 2, /* no kernel variant covers this shape / dtype / layout                */
    MCF_EALIGN = 3,       /* a base pointer or a leading stride breaks the 16-byte requirement   */
    MCF_ELAUNCH = 4       /* the HIP runtime rejected the launch (hipGetLastError)               */
} mcf_status;

/*
 * Problem statement (Sec. VI-B1: (batch,M,K) x (batch,K,N), then (batch,M,N) x (batch,N,L)).
 * Strides are in ELEMENTS, ordered {batch, row, col}; an all-zero triple means packed
 * row-major.  Layout requirements of the kernels:
 *   A: col stride 1 (K contiguous);  D, E: col stride 1 (L contiguous);
 *   B: either col stride 1 ([b,K,N], N contiguous: the GEMM-chain layout) or row stride 1
 *      ([b,N,K] handed over as {N*K, 1, K}: the key matrix of attention, K contiguous).
 *   Every non-unit row stride and every batch stride is a multiple of 8 elements; for
 *   N-contiguous B, N itself is a multiple of 8.  Base pointers are 16-byte aligned.
 * Supported here: (K, L) in {(32,32), (64,64), (128,128), (64,128), (128,64), (64,256),
 * (256,256), (80,80), (96,96), (160,160), (192,192)} with the whole K extent on chip (T_K = K),
 * and every other K >= 256 that is a
 * multiple of 128 with L in {64, 128, 256} through kernels with a k loop inside the block
 * (T_K = 128).  Any batch, M >= 0, N >= 0 (N >= 1 with softmax).  Other
 * (K, L) give MCF_EUNSUPPORTED.
 * in_dtype is the type of A, B, D (MCF_F16 or MCF_BF16); out_dtype that of E: in_dtype, or
 * MCF_F32 (the fp32 accumulators are then stored unrounded; e_stride counts fp32 elements).
 * Both GEMMs accumulate in fp32; C (or P) is rounded once to in_dtype between them.
 */
typedef struct mcf_problem {
    int64_t batch, M, K, N, L;
    int32_t in_dtype, out_dtype; /* mcf_dtype */
    int64_t a_stride[3], b_stride[3], d_stride[3], e_stride[3];
} mcf_problem;

/*
 * A tile choice and the model terms it was ranked by.  Tiling expression per block is the
 * paper's "nk" sub-expression with T_K = K and T_L = L (so the k and h loops have extent 1
 * and L_A / S_E are hoisted out of the n loop, Sec. III-B):
 *     block <-> (batch, m-tile);   L_A;  for n-tile: { L_B, L_D -> LDS; C_C; [softmax]; C_E };  S_E
 * tm = 32 * mb * rg rows per block (rg wave row-groups, each wave owning 32*mb rows),
 * tn = 32 * ns * nj columns per n-iteration (ns waves side by side in n, each owning nj
 * 32-column slices), waves = rg * ns.
 */
typedef struct mcf_tiles {
    int32_t tm, tn, tk, tl;   /* tile sizes T_M, T_N, T_K (= K, or 128 with a k loop), T_L (= L, */
                              /* or a divisor of L: then block <-> (batch, m-tile, h-tile))      */
    int32_t mb, rg, ns, nj;   /* 32-row blocks per wave, wave row-groups, waves across n,        */
                              /* 32-column slices per wave and n-iteration (0 reads as 1)        */
    int32_t waves;            /* rg * ns, 64 lanes each                                          */
    int32_t stages;           /* depth of the LDS ring of (B tile + D tile) buffers, 2..4        */
    int32_t lds_bytes;        /* eq. (1) restricted to the tiles held in LDS (B, D; x stages)    */
    int32_t vgpr_est;         /* eq. (1) restricted to the tiles held in registers (A, C, E)     */
    int32_t vgpr_used;        /* registers per lane the compiler allocated for this variant      */
    int32_t scratch_bytes;    /* per-lane spill space of a variant whose loops spill registers   *
                               * (non-zero: never picked); registers only parked in scratch      *
                               * across the n loop, outside of it, are not counted               */
    int64_t blocks;           /* N_block of eq. (5)                                              */
    int64_t compulsory_bytes; /* A, B, D read once + E written once                              */
    int64_t model_bytes;      /* numerator of eq. (3): sum of tile bytes x trip counts           */
    int64_t flops;            /* numerator of eq. (4), padding included                          */
    double t_mem_s, t_comp_s, alpha, t_est_s; /* eq. (3), (4), (5), (2)                          */
} mcf_tiles;

/*
 * Tile picker (Sec. IV-A eq. (2)-(5), Sec. III-C Rules 3-4).  Host only: needs no GPU.
 * Enumerates the kernel variants built into the library that cover (K, L, dtype, layout),
 * drops those that break the LDS / register budget or the padding rule, and returns the one
 * with the smallest t_est.  out is host memory.  MCF_EUNSUPPORTED if nothing covers the shape.
 */
int mcf_pick_tiles(const mcf_problem *problem, int softmax, mcf_tiles *out);

/*
 * Evaluate the model for a caller-chosen (mb, rg, ns, nj) and T_L (tl; 0 reads as L) instead of
 * picking: fills every other field of *tiles.  MCF_EUNSUPPORTED if no built variant has that shape, MCF_EINVAL if it
 * breaks a budget (LDS, registers) -- such a variant still runs unless it exceeds the LDS of
 * a compute unit.  Host only.
 */
int mcf_eval_tiles(const mcf_problem *problem, int softmax, mcf_tiles *tiles);

/* Number of built kernel variants with T_L = L and their (mb, rg, ns, nj) for the shape; host
 * only.  Writes up to cap quadruples into shapes (4 ints each) and returns the total count. */
int mcf_list_variants(const mcf_problem *problem, int softmax, int32_t *shapes, int cap);

/* The candidates mcf_pick_tiles and the search choose from, with their model terms: the feasible
 * variants for T_L = L followed by those for every smaller T_L that divides L and has kernels
 * (the h tiles are then blocks of their own: more parallel work, GEMM 1 repeated per h tile --
 * Sec. III-A, deep expression m h n k).  Writes up to cap entries, returns the total.  Host only. */
int mcf_list_candidates(const mcf_problem *problem, int softmax, mcf_tiles *out, int cap);

/*
 * E = (A . B) . D   (Sec. III-A).  Device pointers; tiles_or_null == NULL means
 * mcf_pick_tiles() decides, otherwise only its mb, rg, ns, nj and tl (0 = L) fields are read.  hip_stream is a
 * hipStream_t (NULL = the default stream).  E must not overlap A, B or D.  batch, M or L of
 * zero is a no-op; N == 0 writes zeros.
 */
int mcf_gemm_chain(const mcf_problem *problem, const void *A, const void *B, const void *D,
                   void *E, const mcf_tiles *tiles_or_null, void *hip_stream);

/*
 * E = softmax_rows(scale * A . B) . D   (Sec. VI-B2; softmax along n, no mask).  The kernel
 * uses the online max / sum recurrence over n-tiles, which equals the two-pass definition up
 * to rounding.  Same argument rules as mcf_gemm_chain; N == 0 is MCF_EINVAL, M + N at or beyond
 * 2^31 - 1024 MCF_EUNSUPPORTED (the kernels compare row and column numbers in 32 bits).
 */
int mcf_softmax_gemm_chain(const mcf_problem *problem, float scale, const void *A,
                           const void *B, const void *D, void *E,
                           const mcf_tiles *tiles_or_null, void *hip_stream);

/*
 * The softmax chain under a causal mask (not in the paper; the convention of attention
 * kernels): row i of every batch sees the columns n <= i + causal_offset only,
 *     E[b,i,:] = softmax_{n <= i + causal_offset}(scale * A[b,i,:] . B[b,:,n]) . D[b,n,:],
 * causal_offset = 0 being the lower triangle and causal_offset = N - M the triangle that ends
 * in the last row and column (any offset is valid: N - 1 or more hides nothing, -M or less
 * everything); a row that sees no column is written as zeros.  n-tiles that no row of a block
 * sees are neither loaded nor computed.  Everything else as
 * mcf_softmax_gemm_chain (same kernels, same tile choice).
 */
int mcf_causal_softmax_gemm_chain(const mcf_problem *problem, float scale, int64_t causal_offset,
                                  const void *A, const void *B, const void *D, void *E,
                                  const mcf_tiles *tiles_or_null, void *hip_stream);

/*
 * G = (E) . F with E the chain above, softmax != 0 selecting its softmax form (Sec. III-A: the
 * paper's analysis carries over to chains with more compute-intensive operators; this is the
 * chain of three GEMMs).  F is [batch, L, P] with element strides f_stride {batch, row, col}
 * (NULL or all zero = packed; col stride 1), G is [batch, M, P] and problem->e_stride
 * describes G (not E, which never leaves the registers).  E is rounded once to in_dtype
 * before the third GEMM, as C / P is before the second (with a split of n across waves: each
 * wave's normalised partial E).  Built for (K, L, P) in {(64,64,64), (128,128,128),
 * (64,128,128), (128,64,64), (64,64,128)} (with P != L only arrangements without a split of n
 * across waves: the combine of the product reuses the register layout of E); other shapes
 * give MCF_EUNSUPPORTED.  tiles_or_null: NULL = the arrangement whose two-GEMM part
 * the model ranks best among those built for three GEMMs, otherwise its mb, rg, ns, nj are
 * read.  G must not overlap A, B, D or F.
 */
int mcf_gemm_chain3(const mcf_problem *problem, int softmax, float scale, int64_t P,
                    const int64_t *f_stride, const void *A, const void *B, const void *D,
                    const void *F, void *G, const mcf_tiles *tiles_or_null, void *hip_stream);

/* The arrangement mcf_gemm_chain3 takes when given no tiles; the model terms in *out are those
 * of its two-GEMM part (problem->e_stride is not read).  MCF_EUNSUPPORTED: none built. */
int mcf_pick_tiles3(const mcf_problem *problem, int64_t P, int softmax, mcf_tiles *out);

/* The (mb, rg, ns, nj) built for the three-GEMM chain of this shape, as mcf_list_variants. */
int mcf_list_variants3(const mcf_problem *problem, int64_t P, int softmax, int32_t *shapes, int cap);

/*
 * Heuristic search over the built variants (Sec. IV-B, Alg. 1): a population of `population`
 * candidates drawn at random (without repetition while unused ones remain) from the feasible
 * variants (those mcf_list_candidates returns),
 * ranked by the model; the `top_n` distinct candidates with the smallest estimates are measured;
 * the search stops when the fastest of them is within `epsilon` (relative) of the best time seen
 * so far, otherwise the next population is drawn from the current one with probability
 * proportional to 1 / estimate and each drawn member gets the tile choice of one loop (m: the
 * pair mb, rg; n: the pair ns, nj; h: T_L) replaced by that of a random feasible variant that
 * differs in that loop only.  A candidate is measured at most once.  Random numbers are SplitMix64 of
 * (seed + counter).  Zero fields of *params read as the defaults 32, 8, 16 and 0.02.
 * One deviation from the listing: the convergence test only ends the search; what is returned
 * is the fastest candidate measured in any generation (the listing returns the fastest of the
 * last generation's shortlist, which may be up to epsilon slower than one measured earlier).
 */
typedef struct mcf_search_params {
    int32_t population;      /* N of Alg. 1 (default 32)                                   */
    int32_t top_n;           /* n of Alg. 1 (default 8)                                    */
    int32_t max_generations; /* bound on the generations, not in Alg. 1 (default 16)       */
    int32_t reserved;
    double epsilon;          /* relative convergence threshold (default 0.02)              */
    uint64_t seed;
} mcf_search_params;

#define MCF_SEARCH_LOG_MAX 64
typedef struct mcf_search_entry {
    int32_t mb, rg, ns, nj;  /* the candidate                                              */
    int32_t generation;      /* generation (from 0) in which it was measured               */
    int32_t tl;              /* its T_L                                                    */
    double t_est_s;          /* its model estimate, eq. (2)                                */
    double t_meas_s;         /* what the measurement returned                              */
} mcf_search_entry;

typedef struct mcf_search_report {
    int32_t space;           /* feasible variants the search drew from                     */
    int32_t generations;     /* generations run                                            */
    int32_t measured;        /* candidates measured (entries of log that are valid)        */
    int32_t converged;       /* 1: stopped by epsilon, 0: by max_generations               */
    double best_t_s;         /* measured time of the returned candidate                    */
    mcf_search_entry log[MCF_SEARCH_LOG_MAX]; /* in measurement order                      */
} mcf_search_report;

/* Returns the run time in seconds of one launch with these tiles; a negative or non-finite
 * value aborts the search with MCF_ELAUNCH.  Called on the calling thread. */
typedef double (*mcf_measure_fn)(const mcf_tiles *candidate, void *user);

/*
 * Alg. 1 with a caller-supplied measurement.  Host only (the callback may of course launch).
 * best and report_or_null are host memory.  MCF_EUNSUPPORTED if no variant covers the shape.
 */
int mcf_search_tiles(const mcf_problem *problem, int softmax, const mcf_search_params *params_or_null,
                     mcf_measure_fn measure, void *user, mcf_tiles *best,
                     mcf_search_report *report_or_null);

/*
 * Alg. 1 measured on the device: every measured candidate runs 3 + `launches` times on
 * hip_stream over the caller's buffers (same argument rules as the two chain calls; softmax != 0
 * selects mcf_softmax_gemm_chain with `scale`), timed with HIP events around the last
 * `launches` (<= 0 reads as 20), after up to 50 ms of untimed launches of the model's choice
 * that bring the clocks up.  E is overwritten.  Synchronises hip_stream; creates and
 * destroys two HIP events, allocates no device memory.  Operands that fit the caches stay
 * resident between launches, so the times are warm-cache times.
 */
int mcf_tune_tiles(const mcf_problem *problem, int softmax, float scale, const void *A,
                   const void *B, const void *D, void *E, const mcf_search_params *params_or_null,
                   int launches, void *hip_stream, mcf_tiles *best,
                   mcf_search_report *report_or_null);

/*
 * The same three calls for the three-GEMM chain (Sec. III-A: the analysis and with it the
 * exploration carry over to longer chains): the candidates are the arrangements built for
 * (K, L, P), ranked by the model terms of their two-GEMM part (the third GEMM adds the same
 * work to each); mcf_tune_tiles3 measures mcf_gemm_chain3 with the arguments of that call.
 */
int mcf_list_candidates3(const mcf_problem *problem, int64_t P, int softmax, mcf_tiles *out, int cap);
int mcf_search_tiles3(const mcf_problem *problem, int64_t P, int softmax,
                      const mcf_search_params *params_or_null, mcf_measure_fn measure, void *user,
                      mcf_tiles *best, mcf_search_report *report_or_null);
int mcf_tune_tiles3(const mcf_problem *problem, int softmax, float scale, int64_t P,
                    const int64_t *f_stride, const void *A, const void *B, const void *D,
                    const void *F, void *G, const mcf_search_params *params_or_null, int launches,
                    void *hip_stream, mcf_tiles *best, mcf_search_report *report_or_null);

/*
 * Search-space generation and pruning (Sec. III-A, III-B, III-C).  Host only.  The paper's space
 * is (tiling expressions) x (tile sizes); the kernels of this library are points of what is left
 * of it after Rules 1-4, and these entry points say which.
 *
 * A tiling expression is written as in the paper: `xy` nests loop y in loop x, `(x,y)` runs x and
 * then y in one scope; the loops are m, n, k, h (h is this library's L).  Extents arrays are in
 * the order m, n, k, h.
 *
 * mcf_expression      : the index-th (0..25) of the 24 deep expressions (the permutations of
 *                       m n k h) followed by the two flat ones, mn(k,h) and nm(k,h); out is a
 *                       caller buffer of cap >= 8 bytes.  MCF_EINVAL beyond the last.
 * mcf_expression_trips: how often each statement of `expr` runs, trips[] in the order C_C, C_E,
 *                       L_A, L_B, L_D, S_E (Sec. III-B): a compute statement sits under the
 *                       rightmost loop related to it, a memory statement under the rightmost loop
 *                       that indexes its tensor, loops of extent 1 hold nothing.  flags:
 *                       MCF_TRIPS_NO_HOIST leaves the memory statements beside their compute
 *                       statement, MCF_TRIPS_KEEP_UNIT_LOOPS keeps loops of extent 1 in place,
 *                       MCF_TRIPS_BIND_BLOCK keeps every statement inside the loops Rule 1 binds
 *                       to the block index (blocks share no on-chip memory).  MCF_EINVAL for a
 *                       string that is no expression over exactly m, n, k, h.
 * mcf_sub_expression  : Rule 1: what a block runs once m and h are bound to the block index (in
 *                       a flat expression h shares a scope with k and stays), into the caller
 *                       buffer out of cap >= 8 bytes; *passes_rule2 (may be NULL) = 0 if in it k
 *                       encloses n (one partial tile of the intermediate tensor per n), else 1.
 *                       MCF_EINVAL as above.
 * mcf_enumerate_space : the sizes Sec. III-C follows through its example, for this problem:
 *                       expressions, sub-expressions after Rule 1 and after Rule 2, tile-size
 *                       combinations (multiples of 16 up to each dimension) before and after
 *                       Rule 3 (padding) and Rule 4 (eq. (1) over all five tiles in bytes against
 *                       1.2 x shm_max_bytes; 0 = the 160 KiB of a compute unit), and how many of
 *                       the surviving points a built kernel runs.  This reading of Rules 1 and 2
 *                       leaves 3 and then 2 sub-expressions (nk, kn, n(k,h); kn falls); the paper
 *                       counts 5 and 3 without listing them.  MCF_EUNSUPPORTED for a dimension
 *                       beyond 2^24.
 */
#define MCF_MAX_SUB_EXPRESSIONS 8
enum { MCF_TRIPS_NO_HOIST = 1, MCF_TRIPS_KEEP_UNIT_LOOPS = 2, MCF_TRIPS_BIND_BLOCK = 4 };
typedef struct mcf_space_report {
    int32_t n_deep, n_flat;       /* 24, 2                                                       */
    int32_t n_rule1, n_rule2;     /* distinct sub-expressions; those that pass Rule 2            */
    char sub_expression[MCF_MAX_SUB_EXPRESSIONS][16];
    int32_t sub_members[MCF_MAX_SUB_EXPRESSIONS]; /* expressions that reduce to each             */
    int32_t sub_kept[MCF_MAX_SUB_EXPRESSIONS];    /* 1: passes Rule 2                            */
    int64_t tile_choices;         /* prod ceil(dim / 16) over M, N, K, L                         */
    int64_t after_rule3;          /* combinations whose four tile sizes pass the padding rule    */
    int64_t after_rule4;          /* of those, the ones eq. (1) lets on chip                     */
    int64_t candidates;           /* (n_deep + n_flat) * tile_choices                            */
    int64_t candidates_pruned;    /* n_rule2 * after_rule4                                       */
    int64_t built_deep;           /* surviving points (nk, T_M, T_N, T_K, T_H) a kernel runs: T_L = T_H, */
                                  /* the h tiles blocks of their own                             */
    int64_t built_flat;           /* surviving points (n(k,h), T_M, T_N, T_K, 32) a kernel runs:  */
                                  /* T_L = L, E tiles of every 32-column h step in registers     */
} mcf_space_report;
int mcf_expression(int index, char *out, int cap);
int mcf_expression_trips(const char *expr, const int64_t extents[4], int flags, int64_t trips[6]);
int mcf_sub_expression(const char *expr, char *out, int cap, int *passes_rule2);
int mcf_enumerate_space(const mcf_problem *problem, int softmax, int64_t shm_max_bytes, mcf_space_report *out);

/*
 * Measurement aids (no part of the chain): the kernels whose times bound what the chain kernel
 * can reach -- Sec. IV-A's W and P as this machine delivers them, and the cost of a launch.
 * All asynchronous on hip_stream, device pointers owned by the caller, nothing allocated.
 *   mcf_probe_copy : dst[0..bytes) = src[0..bytes), 16 bytes per lane (bytes a multiple of 16,
 *                    pointers 16-byte aligned, buffers must not overlap).
 *   mcf_probe_mfma : blocks x waves_per_block waves (1..8) each issue iters x 8 independent
 *                    32x32x16 fp16 MFMAs (32768 flops each) on register operands; out receives
 *                    blocks * waves_per_block * 64 floats.
 *   mcf_probe_empty: a kernel of `blocks` one-wave blocks that does nothing.
 */
int mcf_probe_copy(void *dst, const void *src, int64_t bytes, void *hip_stream);
int mcf_probe_mfma(void *out, int32_t blocks, int32_t waves_per_block, int32_t iters, void *hip_stream);
int mcf_probe_empty(int32_t blocks, void *hip_stream);

/* Human-readable name of a status code (static storage). */
const char *mcf_status_string(int status);

/* Text of the last HIP error seen by this thread inside the library, "" if none. */
const char *mcf_last_error(void);

#ifdef __cplusplus
}
#endif
#endif /* MCF_H */

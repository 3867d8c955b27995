// Internal declarations shared by the host files of the library (never installed).
#pragma once
#include <vector>
#include <stdint.h>

#include "../../include/mcf.h"

namespace mcf {

// Machine constants of MI355X used by the picker (Sec. IV-A: W, P, N_SM of eq. (3)-(5)).
constexpr double kHbmBytesPerSec = 8.0e12;    // W: HBM3E peak
constexpr double kL2BytesPerSec = 32.0e12;    // bandwidth charged to re-reads served by L2/MALL
constexpr double kMfmaFlopsPerSec = 2.5e15;   // P: dense fp16/bf16 MFMA peak
constexpr int kComputeUnits = 256;            // compute units
// eq. (5) in SIMDs: a block takes as many of a compute unit's four SIMDs as it has waves, at most
// all four, and N_SM is four such units per compute unit.
constexpr int kWaveUnitsPerBlock = 4;
constexpr int kWaveUnits = kComputeUnits * kWaveUnitsPerBlock;
constexpr int kLdsBytesPerBlock = 160 * 1024; // Shm_max of Rule 4
constexpr int kVgprBudget = 512;              // arch + accumulation VGPRs per lane at 1 wave/SIMD

// Kernel arguments (device pointers, element strides).
struct KParams {
    // what a block needs first (its place in the problem): together at the start, one scalar load
    int32_t n_blocks;   // batch * m_tiles * h_tiles
    int32_t m_tiles;    // ceil(M / T_M)
    int32_t h_tiles;    // L / T_L: column tiles of E, each a block of its own (1 when T_L = L)
    // floor(n / m_tiles) = umulhi(n, m_magic) >> m_shift for 0 <= n < 2^31 (m_magic = 0: m_tiles = 1);
    // the same for h_tiles.  Saves the blocks an integer division each before their first load.
    uint32_t m_magic, h_magic;
    int32_t m_shift, h_shift;
    int32_t M, N;
    int32_t a_mode;     // 0: A as is, 1: -A (negative scale), 2: A := 0 (scale == 0)
    int32_t k_chunks;   // kernels with a k loop: K / T_K (otherwise unused)
    float c1;           // |scale| * log2(e) (softmax only)
    int32_t causal_off; // softmax only: row i sees the columns n <= i + causal_off (N - 1: no mask); no flag
                        // beside it: a branch on one splits the scalar loads of the arguments in two
    const void *A, *B, *D;
    void *E;            // bit 0 set: written as fp32 (the pointer itself is 16-byte aligned; strides then count fp32 elements)
    int64_t sa_b, sa_r; // A: batch / row stride (col stride 1)
    int64_t sb_b, sb_r; // B: batch stride / stride of the non-contiguous index
    int64_t sd_b, sd_r; // D: batch / row stride
    int64_t se_b, se_r; // E: batch / row stride
    const void *F;      // three-GEMM chain: F[b, L, P] (col stride 1); E is then the output [b, M, P]
    int64_t sf_b, sf_r; // F: batch / row stride
};

// magic, shift with floor(n / d) = umulhi(n, magic) >> shift for every 0 <= n < 2^31 (d >= 1;
// magic = 0 stands for d = 1): magic = ceil(2^(31+s) / d), s = ceil(log2 d), shift = s - 1.
inline void division_magic(uint32_t d, uint32_t *magic, int32_t *shift) {
    if (d <= 1) { *magic = 0; *shift = 0; return; }
    int s = 0;
    while ((1ull << s) < d) ++s;
    *magic = (uint32_t)(((1ull << (31 + s)) + d - 1) / d);
    *shift = s - 1;
}

typedef int (*LaunchFn)(const KParams &p, void *stream); // returns hipError_t as int

struct Variant {
    int32_t dtype, K, L;
    int32_t mb, rg, ns, nj;
    int32_t softmax, b_kcontig;
    int32_t ksplit;        // 1: K is the chunk T_K of a k loop inside the block; 0: T_K = K
    int32_t P;             // three-GEMM chain: columns of F and of the output; 0: two-GEMM chain
    LaunchFn launch;
    int32_t vgprs;         // VGPRs per lane the compiler allocated (-1: unknown)
    int32_t scratch_bytes; // per-lane scratch of a kernel whose loops spill registers (such variants are never picked); 0 also
                           // where the compiler only parks a few registers in scratch across the n loop, outside of it
};

// Registry of every built kernel variant (defined in mcf_registry.cpp): the two-GEMM chain ...
const Variant *variants(int *count);
// ... and the three-GEMM chain (P > 0).
const Variant *variants3(int *count);
// The kernel group that serves a problem's (dtype, K, L): the group with T_K = K if it is built,
// otherwise a group with a k loop whose chunk divides K.  Returns false if there is neither;
// *tk is the K of the group's variants, *ksplit whether they loop over k.
bool resolve_group(int dtype, int64_t K, int64_t L, int *tk, int *ksplit);
// Variant of that group with the given arrangement (K is the problem's K), or nullptr.
const Variant *find_variant(int dtype, int64_t K, int64_t L, int softmax, int b_kcontig, int mb, int rg, int ns, int nj);

// Layout decoded from an mcf_problem.
struct Layout {
    int64_t sa[3], sb[3], sd[3], se[3];
    int b_kcontig;
};
int decode_layout(const mcf_problem *p, Layout *out); // MCF_OK or an error status

// Ring depth and LDS bytes of a variant; register estimate per lane.
int stages_for(const Variant *v);
int lds_bytes_for(const Variant *v);
bool better(const mcf_tiles &a, const mcf_tiles &b); // the picker's order: estimate, then the tie-breaks
int vgpr_estimate(int K, int L, int mb, int rg, int ns, int nj, int softmax, int ksplit);

// Feasible candidates for a problem, with their model terms, in registry order (the set
// mcf_pick_tiles chooses from).  MCF_OK, or the status mcf_pick_tiles would return.
int feasible_candidates(const mcf_problem *p, int softmax, std::vector<mcf_tiles> *out);
// The same for the three-GEMM chain: problem3() strips the output's strides (they describe G) and
// finds the layout of B, candidates3() lists the arrangements built for (K, L, P) with the model
// terms of their two-GEMM part.
int problem3(const mcf_problem *p, int64_t P, mcf_problem *two_gemm_part, int *b_kcontig);
int candidates3(const mcf_problem *p, int softmax, int b_kcontig, int64_t P, std::vector<mcf_tiles> *out);

void set_last_error(const char *msg);

} // namespace mcf

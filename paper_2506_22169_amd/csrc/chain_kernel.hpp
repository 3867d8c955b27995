// Fused two-GEMM chain kernel for gfx950 (CDNA4):  E = (A.B).D  or  E = softmax(scale*A.B).D
//
// Per-block schedule = the paper's "nk" sub-tiling expression with T_K = K, T_L = L
// (Sec. III-B/C): the k and h loops have extent 1, so L_A is hoisted to the block (A tile
// loaded once) and S_E is hoisted out of the n loop (E stored once):
//
//   block <-> (batch, m-tile)                               [spatial loops on the block index]
//   A tile -> LDS -> VGPRs                                  [L_A, once]
//   for each n-tile:   B tile, D tile -> LDS ring           [L_B, L_D]
//                      C^T = B^T . A^T        (MFMA)        [C_C]
//                      optional online softmax on C^T, convert to 16-bit in registers
//                      E^T += D^T . C^T       (MFMA)        [C_E]
//   E tile -> global                                        [S_E, once]
//
// Both GEMMs are computed transposed so that the fp32 accumulator of the first is, lane for
// lane, already the second operand of the second: the intermediate never leaves registers.
//
// Global -> LDS traffic uses the direct-to-LDS load (global_load_lds_dwordx4: every lane
// names a 16-byte global source, the wave's 64 pieces land contiguously in LDS), issued
// several n-tiles ahead into a ring of `stages` buffers and retired with counted
// s_waitcnt vmcnt, so no registers are spent on staging and the prefetch depth covers the
// HBM latency.  LDS tiles keep their natural row pitch; bank conflicts are avoided by an XOR
// swizzle of the 16-byte chunk index applied on the global-source side of the load.
//
// MFMA v_mfma_f32_32x32x16_{f16,bf16}: lane l = (c = l%32, g = l/32).
//   first operand  X[32 x 16]: lane holds X[c][8g .. 8g+7]
//   second operand Y[16 x 32]: lane holds Y[8g .. 8g+7][c]
//   result         Z[32 x 32]: lane holds Z[8(r/4) + 4g + r%4][c], r = 0..15
//
// Waves of a block form an rg x ns grid: wave (wr, wn) owns rows [wr*32*MB, +32*MB) of the
// block's m-tile and NJ 32-column slices, columns [wn*32*NJ, +32*NJ), of every n-tile; with ns > 1 the partial results of
// the ns waves of a row-group are combined through LDS after the loop.
#pragma once
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include <type_traits>

#include "mcf_geometry.h"
#include "mcf_internal.h"

// The reference maximum of the online softmax follows the running row maximum only once that
// has grown by more than this many binary orders of magnitude (0: always).
#ifndef MCF_LAZY_MAX
#define MCF_LAZY_MAX 8
#endif

namespace mcf {

typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef short i16x4 __attribute__((ext_vector_type(4)));
typedef short i16x8 __attribute__((ext_vector_type(8)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef __attribute__((address_space(3))) unsigned char lds_u8;
typedef __attribute__((address_space(3))) i16x4 lds_i16x4;
typedef __attribute__((address_space(3))) u32x4 lds_u32x4;
typedef __attribute__((address_space(3))) float lds_f32;

template <typename T> struct Mfma;
template <> struct Mfma<_Float16> {
    using v8 = f16x8;
    static __device__ __forceinline__ f32x16 run(v8 x, v8 y, f32x16 z) {
        return __builtin_amdgcn_mfma_f32_32x32x16_f16(x, y, z, 0, 0, 0);
    }
};
template <> struct Mfma<__bf16> {
    using v8 = bf16x8;
    static __device__ __forceinline__ f32x16 run(v8 x, v8 y, f32x16 z) {
        return __builtin_amdgcn_mfma_f32_32x32x16_bf16(x, y, z, 0, 0, 0);
    }
};

// Value held by the other half-wave's lane with the same c (lane ^ 32), combined by max / add.
static __device__ __forceinline__ float xhalf_max(float x) {
    unsigned u = __builtin_bit_cast(unsigned, x);
    auto r = __builtin_amdgcn_permlane32_swap(u, u, false, false);
    return fmaxf(__builtin_bit_cast(float, (unsigned)r[0]), __builtin_bit_cast(float, (unsigned)r[1]));
}
static __device__ __forceinline__ float xhalf_sum(float x) {
    unsigned u = __builtin_bit_cast(unsigned, x);
    auto r = __builtin_amdgcn_permlane32_swap(u, u, false, false);
    return __builtin_bit_cast(float, (unsigned)r[0]) + __builtin_bit_cast(float, (unsigned)r[1]);
}

// Transposing LDS read: within each group of 16 lanes, lane i points at 4 consecutive 16-bit
// elements; lane j receives element (j%4) of the pieces addressed by lanes 4e + j/4, e = 0..3.
static __device__ __forceinline__ i16x4 lds_read_tr(const lds_u8 *p) {
    return __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_i16x4 *)p);
}

// Marks a wave-uniform value as such for the register allocator (it must live in SGPRs to
// feed M0 / the scalar base of a direct-to-LDS load).
static __device__ __forceinline__ unsigned uniform(unsigned v) { return __builtin_amdgcn_readfirstlane(v); }
static __device__ __forceinline__ const void *uniform(const void *q) {
    const uint64_t b = (uint64_t)q;
    return (const void *)(((uint64_t)uniform((unsigned)(b >> 32)) << 32) | uniform((unsigned)b));
}

// Direct global -> LDS load of 16 bytes per lane: lane i's piece lands at lds_addr + 16*i.
// lds_addr (a byte address in LDS) and base are wave-uniform; voff is the lane's byte offset
// from base.  Written as inline assembly so that the compiler does not serialise later LDS
// reads behind every outstanding load; completion is awaited with wait_vm<>().
static __device__ __forceinline__ void dma16(unsigned lds_addr, unsigned voff, const void *base) {
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2"
                 :
                 : "s"(uniform(lds_addr)), "v"(voff), "s"(uniform(base))
                 : "memory", "m0");
}
// The same for data the kernel reads once (the A tile): streaming hint.
static __device__ __forceinline__ void dma16_once(unsigned lds_addr, unsigned voff, const void *base) {
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2 nt"
                 :
                 : "s"(uniform(lds_addr)), "v"(voff), "s"(uniform(base))
                 : "memory", "m0");
}
// f(integral_constant<int, I>) for I = B .. E-1, unrolled at compile time
template <int B, int E, typename F> static __device__ __forceinline__ void static_for(F &&f) {
    if constexpr (B < E) {
        f(std::integral_constant<int, B>{});
        static_for<B + 1, E>(f);
    }
}
// Makes the value exist in vector registers at this point of the program: the optimiser may not
// sink what computes it past later statements of the same kind (costs no instruction).
template <typename V> static __device__ __forceinline__ void pin(V &v) { asm volatile("" : "+v"(v)); }
template <int N> static __device__ __forceinline__ void wait_vm() {
    static_assert(N >= 0 && N <= 63, "vmcnt is a 6-bit counter");
    asm volatile("s_waitcnt vmcnt(%0)" ::"n"(N) : "memory");
}
// KSPLIT: KD is the chunk T_K of a k loop inside the block (K = k_chunks * KD); the A chunk of
// every k step travels through the LDS ring with the B chunk instead of the whole A tile living
// in registers.
// PD > 0: chain of three GEMMs.  After the n loop the block multiplies its E tile (still in
// registers) by F[L x PD], which waits in LDS from the prologue on, and stores that product
// instead of E.  The rows of E must then be complete within a wave: NS = 1.
// Waves per SIMD the compiler is to leave room for (pipelined softmax kernels that can have two
// blocks resident; everything else: what the block size itself implies).
template <int KD, int LD, int MB, int RG, int NS, int NJ, bool SOFTMAX, bool KSPLIT, int PD> constexpr int waves_per_simd() {
    constexpr int extra = PD > 0 ? chain3_f_bytes(LD, PD) + 1024 : 0;
    if (pipe_stages(KD, LD, MB, RG, NS, NJ, SOFTMAX, KSPLIT, extra) > 0) return pipe_waves_per_simd(KD, LD, MB, RG, NS, NJ, extra);
    return RG * NS >= 4 ? RG * NS / 4 : 1;
}
template <typename T, int KD, int LD, int MB, int RG, int NS, int NJ, bool SOFTMAX, bool BKC, bool KSPLIT = false, int PD = 0>
__global__ __launch_bounds__(64 * RG * NS) __attribute__((amdgpu_waves_per_eu(waves_per_simd<KD, LD, MB, RG, NS, NJ, SOFTMAX, KSPLIT, PD>())))
void chain_kernel(const KParams p) {
    using M_ = Mfma<T>;
    using v8 = typename M_::v8;
    constexpr int W = RG * NS;           // waves per block
    constexpr int TM = 32 * MB * RG;     // rows per block
    constexpr int TN = 32 * NS * NJ;     // columns per n-iteration
    static_assert(KD % 16 == 0 && LD % 8 == 0, "K in MFMA k-steps of 16, L in 16-byte pieces");
    constexpr bool CH3 = PD > 0;
    static_assert(!CH3 || ((NS == 1 || PD == LD) && !KSPLIT && LD % 32 == 0 && PD % 32 == 0), "three-GEMM chain: whole 32-column blocks; with ns > 1 the product has the shape of E");
    constexpr int KS = KD / 16;          // MFMA k-steps of GEMM 1
    constexpr int HB = h_blocks(LD);     // 32-wide h blocks of GEMM 2 (the last may be partial)
    constexpr int KCH = KD / 8, LCH = LD / 8;                  // 16-byte chunks in a row of K / L elements
    constexpr bool KPAD = pitch_elems(KD) != KD, LPAD = pitch_elems(LD) != LD; // rows padded to a power-of-two pitch
    constexpr int F_EXTRA = CH3 ? chain3_f_bytes(LD, PD) + 1024 : 0;
    constexpr int S = ring_stages(KD, LD, MB, RG, NS, NJ, SOFTMAX, KSPLIT, F_EXTRA); // depth of the LDS ring
    // softmax chains: software pipeline over three consecutive n-tiles (see the loop)
    constexpr bool PIPE = pipe_stages(KD, LD, MB, RG, NS, NJ, SOFTMAX, KSPLIT, F_EXTRA) > 0;
    constexpr int PRE = PIPE ? S - 2 : S - 1; // n-tiles requested before the loop
    constexpr int RBA = 2 * pitch_elems(KD);                // row bytes of the A tile (rows m)
    constexpr int RBB = BKC ? 2 * pitch_elems(KD) : 2 * TN; // row bytes of the B tile (rows n / rows k)
    constexpr int RBD = 2 * pitch_elems(LD);                // row bytes of the D tile (rows n)
    constexpr int B_BYTES = b_tile_bytes(KD, TN);
    constexpr int A_BYTES = a_tile_bytes(KD, MB, RG);
    // Without a k loop a ring slot holds [B tile | D tile] and the A tile borrows the last slot
    // once; with one, a slot holds either [A chunk | B chunk] or [D tile].
    constexpr int STAGE = KSPLIT ? ksplit_slot_bytes(KD, LD, MB, RG, TN) : stage_bytes(KD, LD, TN);
    constexpr int A_LDS = KSPLIT ? 0 : (S - 1) * STAGE; // offset of the A tile (chunk: within its slot)
    constexpr int B_LDS = KSPLIT ? A_BYTES : 0;         // offset of the B tile within its slot
    constexpr int D_LDS = KSPLIT ? 0 : B_BYTES;         // offset of the D tile within its slot
    // 1 KiB wave-loads per tile and per wave
    constexpr int CA = A_BYTES / 1024;
    constexpr int CB = B_BYTES / 1024, CD = d_tile_bytes(LD, TN) / 1024;
    constexpr int CT = KSPLIT ? (CA + CB > CD ? CA + CB : CD) : CB + CD; // wave-loads of the largest item
    constexpr int PA = (CA + W - 1) / W;
    constexpr int P = (CT + W - 1) / W;
    // three-GEMM chain: the F tile [LD rows x PD] behind everything else
    constexpr int RBF = 2 * pitch_elems(CH3 ? PD : 32);
    constexpr int F_LDS = CH3 ? chain3_f_offset(KD, LD, PD, MB, RG, NS, NJ, S) : 0;
    constexpr int CF = CH3 ? chain3_f_bytes(LD, PD) / 1024 : 0;
    constexpr int PFW = (CF + W - 1) / W; // wave-loads of F per wave
    static_assert((S - 1) * P <= 63, "too many loads in flight for the 6-bit vmcnt counter");

    extern __shared__ __attribute__((aligned(16))) unsigned char smem_generic[];
    lds_u8 *smem = (lds_u8 *)smem_generic;
    const unsigned lds0 = (unsigned)(size_t)smem;

    // kernel arguments -> scalar registers, once
    const int M = p.M, N = p.N, m_tiles = p.m_tiles, h_tiles = p.h_tiles, n_blocks = p.n_blocks, a_mode = p.a_mode;
    const int sa_r = (int)p.sa_r, sb_r = (int)p.sb_r, sd_r = (int)p.sd_r;
    const int64_t se_r = p.se_r;
    const float c1 = p.c1;

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = uniform(tid >> 6);
    const int c = lane & 31, g = lane >> 5;
    const int wr = wave / NS, wn = wave % NS;

    // Block index -> (batch, m-tile).  Consecutive hardware block ids go round-robin over the
    // 8 XCDs (each with its own L2); give every XCD a contiguous range of logical blocks so the
    // m-tiles of one batch re-read that batch's B and D from one L2.
    int logical;
    {
        const int hw = blockIdx.x;
        const int x = hw & 7, q = n_blocks >> 3, rem = n_blocks & 7;
        logical = x * q + (x < rem ? x : rem) + (hw >> 3);
    }
    // With T_L < L (h_tiles > 1) the LD columns [ht * LD, ht * LD + LD) of D and E are a block
    // of their own; the h tiles of one (batch, m-tile) are neighbours, so they share A and B in L2.
    const unsigned h_magic = p.h_magic, m_magic = p.m_magic;
    const int h_shift = p.h_shift, m_shift = p.m_shift;
    // one scalar load at the very top for all of them (left alone, the compiler fetches them
    // piecemeal, each piece with a wait of its own before the first load can be issued)
    asm volatile("" ::"s"(n_blocks), "s"(m_tiles), "s"(h_tiles), "s"(h_magic), "s"(m_magic), "s"(h_shift), "s"(m_shift), "s"(M));
    const int bm_q = (int)(__umulhi((unsigned)logical, h_magic) >> h_shift);
    const int bm = h_magic ? bm_q : logical;   // logical / h_tiles
    const int ht = logical - bm * h_tiles;
    const int batch_q = (int)(__umulhi((unsigned)bm, m_magic) >> m_shift);
    const int batch = m_magic ? batch_q : bm;  // bm / m_tiles
    const int mt = bm - batch * m_tiles;
    const int mrow0 = mt * TM; // first row of the block

    const T *Ag = (const T *)p.A + batch * p.sa_b + (int64_t)mrow0 * sa_r;
    const T *Bg = (const T *)p.B + batch * p.sb_b;
    const T *Dg = (const T *)p.D + batch * p.sd_b + ht * LD;
    T *Eg = (T *)p.E + batch * p.se_b + ht * LD;

    // ---- per-lane byte offsets of the B / D pieces this wave loads for every n-tile ----------
    // Wave-load j of a stage covers LDS bytes [1024 j, 1024 j + 1024): 16-byte slot 64 j + lane.
    // Slot -> (row, stored chunk); the global source is the logical chunk = stored ^ swizzle.
    // With clamp (the ragged last tile), rows / columns beyond N are redirected to valid memory
    // (their contribution is masked in registers), so no load ever leaves the tensors.
    auto bd_offset = [&](int u, int nt0, bool clamp) __attribute__((always_inline)) -> unsigned {
        int j = wave + u * W;
        j = j < CT ? j : CT - 1;
        if (j < CB) {
            const int slot = 64 * j + lane;
            int row = slot / (RBB / 16), ch = slot % (RBB / 16);
            if (BKC) {
                ch ^= swz_b128(RBB, row);
                if (KPAD && ch >= KCH) ch = 0; // padding of the row: any valid piece
                if (clamp && nt0 + row >= N) row = N - 1 - nt0;
            } else {
                ch ^= swz_tr(RBB, row);
                if (KPAD && row >= KD) row = 0; // rows k beyond K: any valid row
                if (clamp && nt0 + 8 * ch >= N) ch = 0;
            }
            return (unsigned)(row * sb_r * 2 + ch * 16);
        } else {
            const int slot = 64 * (j - CB) + lane;
            int row = slot / (RBD / 16), ch = slot % (RBD / 16);
            ch ^= swz_tr(RBD, row);
            if (LPAD && ch >= LCH) ch = 0;
            if (clamp && nt0 + row >= N) row = N - 1 - nt0;
            return (unsigned)(row * sd_r * 2 + ch * 16);
        }
    };
    unsigned voff[P]; // filled after the A tile has been requested: the first load leaves as early as possible

    // Causal mask (softmax chains only): row i sees the columns n <= i + causal_off, so a block
    // visits the columns its last row sees (NV), and a tile needs no masking for a wave while it
    // ends at or below what the wave's first row sees (n_clean); in the other tiles a lane masks
    // the columns its row does not see, which may be all of them.  Without a mask (causal_off =
    // N - 1) both are N.
    const int causal_off = p.causal_off;
    auto sees = [&](int row) __attribute__((always_inline)) { // columns row `row` sees, 0 .. N
        if constexpr (!SOFTMAX) return N;
        const int v = row + causal_off + 1;
        return v < 0 ? 0 : (v > N ? N : v);
    };
    const int wrow0 = mrow0 + wr * (32 * MB); // first row of this wave
    const int NV = sees((mrow0 + TM < M ? mrow0 + TM : M) - 1);
    const int n_clean = sees(wrow0);
    const int n_iters = (NV + TN - 1) / TN;
    const int n_full = N / TN; // tiles [0, n_full) are complete in memory, tile n_full (if any) is ragged

    auto issue_tile = [&](int t, int stage) __attribute__((always_inline)) {
        const int nt0 = t * TN;
        const void *bbase = uniform((const void *)(BKC ? Bg + (int64_t)nt0 * sb_r : Bg + nt0));
        const void *dbase = uniform((const void *)(Dg + (int64_t)nt0 * sd_r));
        const unsigned dst0 = uniform(lds0 + stage * STAGE + wave * 1024);
        if (t < n_full) {
#pragma unroll
            for (int u = 0; u < P; ++u) {
                const int j = wave + u * W; // wave-uniform
                const int jj = j < CT ? j : CT - 1;
                dma16(dst0 + (jj - wave) * 1024, voff[u], jj < CB ? bbase : dbase);
            }
        } else {
#pragma unroll
            for (int u = 0; u < P; ++u) {
                const int j = wave + u * W;
                const int jj = j < CT ? j : CT - 1;
                dma16(dst0 + (jj - wave) * 1024, bd_offset(u, nt0, true), jj < CB ? bbase : dbase);
            }
        }
    };

    // ---- kernels with a k loop: the items that travel through the ring ----------------------
    // Item r of n-tile t: r < KC is the A chunk + B chunk of k step r ([A | B] in the slot),
    // r == KC the D tile.  Every wave issues P wave-loads per item (the last one repeated where
    // an item has fewer), so that the counted waits are the same for both kinds.
    const int KC = KSPLIT ? p.k_chunks : 1;
    constexpr int CAB = CA + CB;
    auto ks_offset = [&](bool d_item, int u, int nt0, bool clamp) __attribute__((always_inline)) -> unsigned {
        int j = wave + u * W;
        if (d_item) {
            j = j < CD ? j : CD - 1;
            const int slot = 64 * j + lane;
            int row = slot / (RBD / 16), ch = slot % (RBD / 16);
            ch ^= swz_tr(RBD, row);
            if (LPAD && ch >= LCH) ch = 0;
            if (clamp && nt0 + row >= N) row = N - 1 - nt0;
            return (unsigned)(row * sd_r * 2 + ch * 16);
        }
        j = j < CAB ? j : CAB - 1;
        if (j < CA) {
            const int slot = 64 * j + lane;
            int row = slot / (RBA / 16), ch = slot % (RBA / 16);
            ch ^= swz_b128(RBA, row);
            if (mrow0 + row >= M) row = M - 1 - mrow0; // rows past M: any valid row, never stored
            return (unsigned)(row * sa_r * 2 + ch * 16);
        }
        const int slot = 64 * (j - CA) + lane;
        int row = slot / (RBB / 16), ch = slot % (RBB / 16);
        if (BKC) {
            ch ^= swz_b128(RBB, row);
            if (clamp && nt0 + row >= N) row = N - 1 - nt0;
        } else {
            ch ^= swz_tr(RBB, row);
            if (clamp && nt0 + 8 * ch >= N) ch = 0;
        }
        return (unsigned)(row * sb_r * 2 + ch * 16);
    };
    unsigned voff_d[KSPLIT ? P : 1];
    if constexpr (KSPLIT) {
#pragma unroll
        for (int u = 0; u < P; ++u) {
            voff[u] = ks_offset(false, u, 0, false);
            voff_d[u] = ks_offset(true, u, 0, false);
        }
    }
    auto issue_item = [&](int t, int r, int stage) __attribute__((always_inline)) {
        const int nt0 = t * TN;
        const unsigned dst0 = uniform(lds0 + stage * STAGE + wave * 1024);
        const bool ragged = t >= n_full;
        if (r < KC) {
            const int64_t k0 = (int64_t)r * KD;
            const void *abase = uniform((const void *)(Ag + k0));
            const void *bbase = uniform((const void *)(BKC ? Bg + (int64_t)nt0 * sb_r + k0 : Bg + k0 * sb_r + nt0));
            if (!ragged) {
#pragma unroll
                for (int u = 0; u < P; ++u) {
                    const int j = wave + u * W; // wave-uniform
                    const int jj = j < CAB ? j : CAB - 1;
                    dma16(dst0 + (jj - wave) * 1024, voff[u], jj < CA ? abase : bbase);
                }
            } else {
#pragma unroll
                for (int u = 0; u < P; ++u) {
                    const int j = wave + u * W;
                    const int jj = j < CAB ? j : CAB - 1;
                    dma16(dst0 + (jj - wave) * 1024, ks_offset(false, u, nt0, true), jj < CA ? abase : bbase);
                }
            }
        } else {
            const void *dbase = uniform((const void *)(Dg + (int64_t)nt0 * sd_r));
            if (!ragged) {
#pragma unroll
                for (int u = 0; u < P; ++u) {
                    const int j = wave + u * W;
                    const int jj = j < CD ? j : CD - 1;
                    dma16(dst0 + (jj - wave) * 1024, voff_d[u], dbase);
                }
            } else {
#pragma unroll
                for (int u = 0; u < P; ++u) {
                    const int j = wave + u * W;
                    const int jj = j < CD ? j : CD - 1;
                    dma16(dst0 + (jj - wave) * 1024, ks_offset(true, u, nt0, true), dbase);
                }
            }
        }
    };

    // ---- three-GEMM chain: the F tile, first of all loads (it is needed last) ---------------
    if constexpr (CH3) {
        const void *fbase = uniform((const void *)((const T *)p.F + batch * p.sf_b));
        const int sf_r = (int)p.sf_r;
        const unsigned dst0 = uniform(lds0 + F_LDS + wave * 1024);
#pragma unroll
        for (int u = 0; u < PFW; ++u) {
            const int j = wave + u * W;
            const int jj = j < CF ? j : CF - 1;
            const int slot = 64 * jj + lane;
            int row = slot / (RBF / 16), ch = slot % (RBF / 16);
            ch ^= swz_tr(RBF, row);
            dma16(dst0 + (jj - wave) * 1024, (unsigned)(row * sf_r * 2 + ch * 16), fbase);
        }
    }
    // ---- prologue: A tile (into the last ring slot) and the first S-1 n-tiles ---------------
    if constexpr (!KSPLIT) {
        const void *abase = uniform((const void *)Ag);
        const unsigned dst0 = uniform(lds0 + A_LDS + wave * 1024);
#pragma unroll
        for (int u = 0; u < PA; ++u) {
            const int j = wave + u * W;
            const int jj = j < CA ? j : CA - 1;
            const int slot = 64 * jj + lane;
            int row = slot / (RBA / 16), ch = slot % (RBA / 16);
            ch ^= swz_b128(RBA, row);
            if (KPAD && ch >= KCH) ch = 0;             // padding of the row: any valid piece
            if (mrow0 + row >= M) row = M - 1 - mrow0; // rows past M: any valid row, never stored
            dma16_once(dst0 + (jj - wave) * 1024, (unsigned)(row * sa_r * 2 + ch * 16), abase);
        }
        // Wave-load u of a wave covers rows 64 W / (chunks per row) further down than wave-load
        // u - 1 of the same tile, at the same chunk and (the step being a multiple of the
        // swizzle period) the same swizzle: one addition instead of the whole computation.
        constexpr bool INC = CB % W == 0 && CT % W == 0 && !KPAD && !LPAD && (64 * W) % (RBB / 16) == 0 &&
                             (64 * W) % (RBD / 16) == 0 && ((64 * W) / (RBB / 16)) % 16 == 0 && ((64 * W) / (RBD / 16)) % 16 == 0;
#pragma unroll
        for (int u = 0; u < P; ++u) {
            if (INC && u > 0 && (u * W < CB) == ((u - 1) * W < CB))
                voff[u] = voff[u - 1] + (unsigned)(u * W < CB ? ((64 * W) / (RBB / 16)) * sb_r * 2 : ((64 * W) / (RBD / 16)) * sd_r * 2);
            else
                voff[u] = bd_offset(u, 0, false);
        }
    }
    const int n_items = KSPLIT ? n_iters * (KC + 1) : n_iters; // ring items of the whole block
    const int n_pre = n_items < PRE ? n_items : PRE;
    if constexpr (KSPLIT) {
        for (int q = 0; q < n_pre; ++q) issue_item(q / (KC + 1), q % (KC + 1), q);
    } else {
        for (int t = 0; t < n_pre; ++t) issue_tile(t, t);
    }

    // ---- L_A: A tile (or chunk) in LDS -> registers, as the second MFMA operand A^T[k][m] ---
    // a_mode (softmax only: a negative or zero scale) as two masks, so that a kernel with a k
    // loop, which runs this once per chunk, pays two operations per register and a plain chain none.
    v8 a[MB][KS];
    const unsigned a_flip = (SOFTMAX && a_mode == 1) ? 0x80008000u : 0u; // sign bits of both 16-bit floats
    const unsigned a_keep = (SOFTMAX && a_mode == 2) ? 0u : 0xffffffffu;
    auto load_a = [&](unsigned base) __attribute__((always_inline)) {
#pragma unroll
        for (int mb = 0; mb < MB; ++mb) {
            const int row = wr * (32 * MB) + 32 * mb + c;
            const lds_u8 *src = smem + base + row * RBA;
            const int sw = swz_b128(RBA, row);
#pragma unroll
            for (int ks = 0; ks < KS; ++ks) {
                u32x4 raw = *(const lds_u32x4 *)(src + 16 * ((2 * ks + g) ^ sw));
                if constexpr (SOFTMAX) raw = (raw ^ a_flip) & a_keep;
                a[mb][ks] = __builtin_bit_cast(v8, raw);
            }
        }
    };
    if constexpr (!KSPLIT) {
        // the A loads are older than the n_pre tile groups
        if (n_pre == PRE) wait_vm<PRE * P>();
        else wait_vm<0>();
        __syncthreads();
        load_a(A_LDS);
    }

    // ---- loop-invariant LDS read offsets of this lane --------------------------------------
    const int i16 = lane & 15, u16 = (lane >> 4) & 1;
    int b_off;
    if (BKC) {
        // first MFMA operand B^T[n][k]: row n = (wn*NJ + j)*32 + c, logical chunk 2ks + g
        const int row = wn * NJ * 32 + c;
        b_off = B_LDS + row * RBB + 16 * (g ^ swz_b128(RBB, row)); // per k-step: ^ (32 ks); per j: + 32 j rows
    } else {
        // rows k = 16ks + 8g + i/4 (+4), columns n = (wn*NJ + j)*32 + 16u + 4(i%4) .. +3
        const int row = 8 * g + (i16 >> 2);
        const int ch = (4 * wn * NJ + 2 * u16 + ((i16 >> 1) & 1)) ^ swz_tr(RBB, row);
        b_off = B_LDS + row * RBB + 16 * ch + 8 * (i16 & 1); // per j: ^ (64 j) bytes (NJ is a power of two)
    }
    // D operand of GEMM 2 (first MFMA operand D^T[h][n]).  MFMA row i of the h block is mapped
    // to h = 16*((i>>2)&1) + 4*(i>>3) + (i&3) so that the accumulator of lane (c,g) ends up
    // holding 16 consecutive h:  h = 32hb + 16g + r.
    int d_off;
    {
        const int x4 = i16 & 3;
        const int row = wn * NJ * 32 + 4 * g + (i16 >> 2); // per j: + 32 j rows
        const int ch = (u16 + 2 * (x4 & 1)) ^ swz_tr(RBD, row); // h block 0; per hb: ^ (64 hb) bytes
        d_off = D_LDS + row * RBD + 16 * ch + 8 * (x4 >> 1);
    }

    f32x16 accE[MB][HB];
    float m_run[MB], l_run[MB];
#pragma unroll
    for (int mb = 0; mb < MB; ++mb) {
        m_run[mb] = -INFINITY;
        l_run[mb] = 0.f;
#pragma unroll
        for (int hb = 0; hb < HB; ++hb)
#pragma unroll
            for (int r = 0; r < 16; ++r) accE[mb][hb][r] = 0.f;
    }

    // LDS -> register operand fetches.  The lane-dependent part of every address (row, swizzled
    // chunk) is computed once, here; per n-tile the ring slot's base is added (one VALU add per
    // distinct swizzle pattern), and everything else -- slice j, row steps -- is a compile-time
    // constant in the offset field of the LDS instruction.
    constexpr int NBV = BKC ? KS : NJ; // B operand: one pattern per k-step (K-contiguous B) or per slice
    unsigned bvo[NBV], dvo[HB];        // D operand: one pattern per h block
#pragma unroll
    for (int i = 0; i < NBV; ++i) bvo[i] = (unsigned)(b_off ^ (BKC ? 32 * i : 64 * i));
#pragma unroll
    for (int hb = 0; hb < HB; ++hb) dvo[hb] = (unsigned)(d_off ^ (64 * hb));
    unsigned bb[NBV], dd[HB]; // the same plus the base of the ring slot in use
    auto set_b_slot = [&](unsigned slot_off) __attribute__((always_inline)) {
#pragma unroll
        for (int i = 0; i < NBV; ++i) {
            bb[i] = bvo[i] + slot_off;
            asm volatile("" : "+v"(bb[i])); // keep the sum in a VGPR: the constant that follows goes to the offset field
        }
    };
    auto set_d_slot = [&](unsigned slot_off) __attribute__((always_inline)) {
#pragma unroll
        for (int hb = 0; hb < HB; ++hb) {
            dd[hb] = dvo[hb] + slot_off;
            asm volatile("" : "+v"(dd[hb]));
        }
    };
    auto load_b = [&](int j, int ks) __attribute__((always_inline)) -> v8 {
        if (BKC) {
            return __builtin_bit_cast(v8, *(const lds_u32x4 *)(smem + bb[ks] + 32 * j * RBB));
        } else {
            const lds_u8 *src = smem + bb[j] + (16 * ks) * RBB;
            i16x4 lo = lds_read_tr(src);
            i16x4 hi = lds_read_tr(src + 4 * RBB);
            return __builtin_bit_cast(v8, __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7));
        }
    };
    auto load_d = [&](int j, int hb, int qp) __attribute__((always_inline)) -> v8 {
        const lds_u8 *src = smem + dd[hb] + (32 * j + 16 * qp) * RBD;
        i16x4 lo = lds_read_tr(src);
        i16x4 hi = lds_read_tr(src + 8 * RBD);
        return __builtin_bit_cast(v8, __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7));
    };
    // Operands are requested PF MFMA steps ahead of their use so that the LDS latency hides
    // behind the MFMAs already issued; the scheduling barriers keep every LDS read and MFMA
    // in the step it was written in (plain VALU / SALU work may still move across).
    constexpr int PF = 2;
    constexpr int T1 = NJ * KS;     // MFMA steps of GEMM 1 (each feeds MB MFMAs)
    constexpr int T2 = NJ * HB * 2; // MFMA steps of GEMM 2

    f32x16 accC[NJ][MB]; // C^T (then P^T in fp32) of the wave's NJ slices of one n-tile
    v8 pop[NJ][MB][2];   // the same in 16 bit, as the second MFMA operand of GEMM 2
    v8 dop[T2];          // D operands of GEMM 2

    // ---- C_C: C^T[n][m] = sum_k B^T[n][k] A^T[k][m], NJ independent 32-column slices -------
    auto phase_g1 = [&](unsigned slot_off, bool first = true) __attribute__((always_inline)) {
        set_b_slot(slot_off);
        if (first) { // with a k loop: the first chunk of an n-tile
#pragma unroll
            for (int j = 0; j < NJ; ++j)
#pragma unroll
                for (int mb = 0; mb < MB; ++mb)
#pragma unroll
                    for (int r = 0; r < 16; ++r) accC[j][mb][r] = 0.f;
        }
        v8 bop[T1];
#pragma unroll
        for (int t = 0; t < PF && t < T1; ++t) bop[t] = load_b(t / KS, t % KS);
#pragma unroll
        for (int t = 0; t < T1; ++t) {
            const int j = t / KS, ks = t % KS;
            if (t + PF < T1) bop[t + PF] = load_b((t + PF) / KS, (t + PF) % KS);
#pragma unroll
            for (int mb = 0; mb < MB; ++mb) {
                accC[j][mb] = M_::run(bop[t], a[mb][ks], accC[j][mb]);
            }
            __builtin_amdgcn_sched_barrier(0x406);
        }
    };
    // first D operands of GEMM 2: requested early so that their LDS latency overlaps the
    // conversion / softmax
    auto phase_g2_prefetch = [&](unsigned slot_off) __attribute__((always_inline)) {
        set_d_slot(slot_off);
#pragma unroll
        for (int t = 0; t < PF && t < T2; ++t) dop[t] = load_d(t / (2 * HB), (t / 2) % HB, t % 2);
    };
    // ---- softmax (online max / sum over n-tiles) and conversion to 16 bit: lane (c,g) holds,
    //      for row m = c, the columns n = n0 + 32j + 8(r/4) + 4g + r%4
    auto phase_sm = [&](int n0) __attribute__((always_inline)) {
#pragma unroll
        for (int mb = 0; mb < MB; ++mb) {
            if (n0 + 32 * NJ > n_clean) { // ragged last tile, or a tile on the mask's edge: columns a row does not see contribute nothing
                const int lim = sees(wrow0 + 32 * mb + c);
#pragma unroll
                for (int j = 0; j < NJ; ++j)
#pragma unroll
                    for (int r = 0; r < 16; ++r)
                        if (n0 + 32 * j + 8 * (r / 4) + 4 * g + (r % 4) >= lim) accC[j][mb][r] = SOFTMAX ? -INFINITY : 0.f;
            }
            if (SOFTMAX) {
                float mx = accC[0][mb][0];
#pragma unroll
                for (int j = 0; j < NJ; ++j)
#pragma unroll
                    for (int r = 0; r < 16; ++r) mx = fmaxf(mx, accC[j][mb][r]);
                mx = xhalf_max(mx);
                // The running maximum only has to keep the exponentials in range, not to be exact:
                // it follows the row maximum only when that has grown by more than
                // MCF_LAZY_MAX in the exponent (so p <= 2^MCF_LAZY_MAX), which after the first
                // tiles is rare -- and with it the rescaling of the accumulators below.  The
                // result is the same up to rounding: numerator and denominator share m.
                float m_new = fmaxf(m_run[mb], mx);
                if (MCF_LAZY_MAX > 0) m_new = (m_new - m_run[mb]) * c1 > (float)MCF_LAZY_MAX ? m_new : m_run[mb];
                // a row that has seen no column yet (under a mask) keeps m = -inf: p = 0, nothing to rescale
                const bool blind = m_new == -INFINITY;
                const float corr = blind ? 1.0f : __builtin_amdgcn_exp2f((m_run[mb] - m_new) * c1);
                const float mneg = blind ? 0.f : -m_new * c1;
                float sum = 0.f;
#pragma unroll
                for (int j = 0; j < NJ; ++j)
#pragma unroll
                    for (int r = 0; r < 16; ++r) {
                        accC[j][mb][r] = __builtin_amdgcn_exp2f(__builtin_fmaf(accC[j][mb][r], c1, mneg));
                        sum += accC[j][mb][r];
                    }
                l_run[mb] = l_run[mb] * corr + sum;
                m_run[mb] = m_new;
                if (__builtin_amdgcn_ballot_w64(corr != 1.0f)) {
#pragma unroll
                    for (int hb = 0; hb < HB; ++hb)
#pragma unroll
                        for (int r = 0; r < 16; ++r) accE[mb][hb][r] *= corr;
                }
            }
#pragma unroll
            for (int j = 0; j < NJ; ++j)
#pragma unroll
                for (int qp = 0; qp < 2; ++qp)
#pragma unroll
                    for (int e = 0; e < 8; ++e) pop[j][mb][qp][e] = (T)accC[j][mb][8 * qp + e];
        }
    };
    // ---- C_E: E^T[h][m] += sum_n D^T[h][n] P^T[n][m] ---------------------------------------
    auto phase_g2 = [&]() __attribute__((always_inline)) { // after phase_g2_prefetch of the same tile
#pragma unroll
        for (int t = 0; t < T2; ++t) {
            const int j = t / (2 * HB), hb = (t / 2) % HB, qp = t % 2;
            if (t + PF < T2) dop[t + PF] = load_d((t + PF) / (2 * HB), ((t + PF) / 2) % HB, (t + PF) % 2);
#pragma unroll
            for (int mb = 0; mb < MB; ++mb) {
                accE[mb][hb] = M_::run(dop[t], pop[j][mb][qp], accE[mb][hb]);
            }
            __builtin_amdgcn_sched_barrier(0x406);
        }
    };

    // Softmax chains in blocks of 8 waves run their two wave groups (waves 0-3 and 4-7, which
    // share the SIMDs pairwise) a phase apart, see below.
    constexpr bool SKEW = skewed_groups(RG, NS, SOFTMAX, KSPLIT);
    if constexpr (KSPLIT) {
        // One ring item per iteration: the k steps of an n-tile accumulate C^T, its D item turns
        // C^T into P^T and feeds GEMM 2.  Same protocol as below: one barrier per item, loads
        // S-1 items ahead.
        const int NI = KC + 1;
        int stage_c = 0, stage_l = S - 1;
        int lt = n_pre / NI, lr = n_pre % NI; // next item to request
        int ct = 0, cr = 0;                   // item being consumed
        for (int q = 0; q < n_items; ++q) {
            if (n_items - q >= S - 1) wait_vm<(S - 2) * P>();
            else wait_vm<0>();
            __syncthreads(); // item q is complete for every wave; the slot of item q-1 is free
            if (q + S - 1 < n_items) {
                issue_item(lt, lr, stage_l);
                if (++lr == NI) { lr = 0; ++lt; }
                stage_l = stage_l + 1 == S ? 0 : stage_l + 1;
            }
            const int n0 = ct * TN + wn * (32 * NJ);
            if (n0 < N) {
                const unsigned st = stage_c * STAGE;
                if (cr < KC) {
                    load_a(st + A_LDS);
                    phase_g1(st, cr == 0);
                } else {
                    phase_g2_prefetch(st);
                    phase_sm(n0);
                    phase_g2();
                }
            }
            if (++cr == NI) { cr = 0; ++ct; }
            stage_c = stage_c + 1 == S ? 0 : stage_c + 1;
        }
    } else if constexpr (PIPE) {
        // Software pipeline over n-tiles (softmax chains; plain chains with K and L of 32, where a
        // tile is only a handful of MFMAs per wave and the pipeline is what keeps them coming: the
        // conversion of tile i then rides behind GEMM 1 of tile i+1).
        // A wave's matrix work and its softmax arithmetic sit on
        // different pipes of the SIMD, but only overlap when they alternate in ONE wave's
        // instruction stream (an MFMA of 32 cycles hides five to six ordinary vector operations
        // or three exponentials issued behind it; two waves a phase apart mostly queue up).  So
        // iteration i issues, step by step, the MFMAs of GEMM 2 of tile i-1 and then of GEMM 1 of
        // tile i+1, and after every step a slice of the softmax of tile i, none of which depends
        // on those MFMAs:
        //   steps [0, TA)        row maximum of tile i, then the (lazily updated) reference
        //   steps [TA, TT)       p = exp2(c1 * s - m) in place, row-sum partials
        //   steps [T2, TT)       conversion of finished p to 16 bit (the operand GEMM 2 of tile
        //                        i-1 has read by then is overwritten)
        // Tile t lives in ring slot t % S; tile i+S-2 is requested at the top of iteration i,
        // into the slot tile i-2 left in iteration i-1.  One block barrier per iteration.
        static_assert(S >= 4, "three live tiles and one landing");
        constexpr int NE = 16 * NJ;       // elements of S per lane and row set in one n-tile
        constexpr int TT = T2 + T1;       // MFMA steps of an iteration
        constexpr int TA = TT >= 12 ? TT / 6 : (TT >= 6 ? 2 : 1);
        constexpr int TB = TT - TA;
        constexpr int EA = (NE + TA - 1) / TA; // elements per maximum step
        constexpr int EB = (NE + TB - 1) / TB; // elements per exponential step
        const int ncol0 = wn * (32 * NJ);
        f32x16 cc[2][NJ][MB]; // C^T of the tile in the softmax and of the tile GEMM 1 is producing
        float mx[MB], mneg[MB], corr[MB], sum0[MB], sum1[MB];

        // element e of a row set <-> slice j = e / 16, accumulator register r = e % 16
        // (a plain chain has no softmax: its slices are the mask of a ragged tile and the conversion)
        auto vstep = [&](auto kc, auto curc, int n0) __attribute__((always_inline)) {
            constexpr int k = decltype(kc)::value, CUR = decltype(curc)::value;
#pragma unroll
            for (int mb = 0; mb < MB; ++mb) {
                if constexpr (k == 0) {
                    // a ragged last tile, or a tile on or beyond the mask's edge: columns a row does
                    // not see contribute nothing (tiles before the last are whole in memory, so
                    // without a mask the test only ever holds for the last)
                    if (n0 + 32 * NJ > n_clean) {
                        // element e sits 32(e/16) + 8((e%16)/4) + e%4 columns right of the lane's first;
                        // one compare and one select per element, in order (the pin keeps the
                        // compiler from forming all the compares first, a scalar register pair each)
                        const int room = sees(wrow0 + 32 * mb + c) - n0 - 4 * g; // columns the row sees from there on
#pragma unroll
                        for (int e = 0; e < NE; ++e) {
                            float x = cc[CUR][e / 16][mb][e % 16];
                            x = 32 * (e / 16) + 8 * ((e % 16) / 4) + (e % 4) < room ? x : (SOFTMAX ? -INFINITY : 0.f);
                            pin(x);
                            cc[CUR][e / 16][mb][e % 16] = x;
                        }
                    }
                }
                if constexpr (SOFTMAX && k < TA) {
                    if constexpr (k == 0) mx[mb] = cc[CUR][0][mb][0];
#pragma unroll
                    for (int e = k * EA; e < (k + 1) * EA && e < NE; ++e) mx[mb] = fmaxf(mx[mb], cc[CUR][e / 16][mb][e % 16]);
                    pin(mx[mb]);
                    if constexpr (k == TA - 1) {
                        const float m_row = xhalf_max(mx[mb]);
                        float m_new = fmaxf(m_run[mb], m_row);
                        if (MCF_LAZY_MAX > 0) m_new = (m_new - m_run[mb]) * c1 > (float)MCF_LAZY_MAX ? m_new : m_run[mb];
                        // (under a mask) a row that has seen no column yet keeps m = -inf: p = 0, nothing to rescale
                        const bool blind = m_new == -INFINITY;
                        corr[mb] = blind ? 1.0f : __builtin_amdgcn_exp2f((m_run[mb] - m_new) * c1);
                        mneg[mb] = blind ? 0.f : -m_new * c1;
                        pin(mneg[mb]);
                        pin(corr[mb]);
                        m_run[mb] = m_new;
                        sum0[mb] = 0.f;
                        sum1[mb] = 0.f;
                    }
                } else if constexpr (SOFTMAX) {
#pragma unroll
                    for (int e = (k - TA) * EB; e < (k - TA + 1) * EB && e < NE; ++e) {
                        float pv = __builtin_amdgcn_exp2f(__builtin_fmaf(cc[CUR][e / 16][mb][e % 16], c1, mneg[mb]));
                        pin(pv);
                        cc[CUR][e / 16][mb][e % 16] = pv;
                        if (e & 1) sum1[mb] += pv;
                        else sum0[mb] += pv;
                    }
                    pin(sum0[mb]);
                    pin(sum1[mb]);
                }
                if constexpr (k >= T2) {
                    // elements that are final (softmax: whose exponential was issued in an earlier
                    // step), spread evenly over the steps of GEMM 1; the last step takes what is left
                    constexpr int done_prev = !SOFTMAX ? NE : (k - 1 < TA ? 0 : ((k - TA) * EB < NE ? (k - TA) * EB : NE));
                    constexpr int quota = NE * (k - T2 + 1) / T1;
                    constexpr int hi = k == TT - 1 ? NE : ((done_prev < quota ? done_prev : quota) & ~1);
                    constexpr int done_prev2 = !SOFTMAX ? NE : (k - 2 < TA ? 0 : ((k - 1 - TA) * EB < NE ? (k - 1 - TA) * EB : NE));
                    constexpr int quota2 = NE * (k - T2) / T1;
                    constexpr int lo = k == T2 ? 0 : ((done_prev2 < quota2 ? done_prev2 : quota2) & ~1);
#pragma unroll
                    for (int e = lo; e < hi; ++e) {
                        pop[e / 16][mb][(e % 16) / 8][e % 8] = (T)cc[CUR][e / 16][mb][e % 16];
                        if (e % 8 == 7) pin(pop[e / 16][mb][(e % 16) / 8]); // a finished operand
                    }
                }
            }
        };
        auto ring_off = [&](int t) __attribute__((always_inline)) { return (unsigned)((t % S) * STAGE); }; // t >= 0
        auto g2_step = [&](auto tc, const v8 &x) __attribute__((always_inline)) {
            constexpr int t = decltype(tc)::value, j = t / (2 * HB), hb = (t / 2) % HB, qp = t % 2;
#pragma unroll
            for (int mb = 0; mb < MB; ++mb) accE[mb][hb] = M_::run(x, pop[j][mb][qp], accE[mb][hb]);
        };
        auto g1_step = [&](auto tc, auto nxtc, const v8 &x) __attribute__((always_inline)) {
            constexpr int t = decltype(tc)::value, j = t / KS, ks = t % KS, NXT = decltype(nxtc)::value;
#pragma unroll
            for (int mb = 0; mb < MB; ++mb) {
                if constexpr (ks == 0) {
                    f32x16 zero;
#pragma unroll
                    for (int r = 0; r < 16; ++r) zero[r] = 0.f;
                    cc[NXT][j][mb] = M_::run(x, a[mb][ks], zero);
                } else {
                    cc[NXT][j][mb] = M_::run(x, a[mb][ks], cc[NXT][j][mb]);
                }
            }
        };
        auto fetch_d = [&](auto tc) __attribute__((always_inline)) -> v8 {
            constexpr int t = decltype(tc)::value;
            return load_d(t / (2 * HB), (t / 2) % HB, t % 2);
        };
        auto fetch_b = [&](auto tc) __attribute__((always_inline)) -> v8 {
            constexpr int t = decltype(tc)::value;
            return load_b(t / KS, t % KS);
        };
        // GEMM 2 of tile t alone / GEMM 1 of tile t alone (the ends of the pipeline)
        auto g2_only = [&](int t) __attribute__((always_inline)) {
            set_d_slot(ring_off(t));
            v8 op[T2];
            static_for<0, (PF < T2 ? PF : T2)>([&](auto tc) { op[decltype(tc)::value] = fetch_d(tc); });
            static_for<0, T2>([&](auto tc) {
                constexpr int t_ = decltype(tc)::value;
                if constexpr (t_ + PF < T2) op[t_ + PF] = fetch_d(std::integral_constant<int, t_ + PF>{});
                g2_step(tc, op[t_]);
                __builtin_amdgcn_sched_barrier(0x406);
            });
        };
        auto g1_only = [&](auto nxtc, int t) __attribute__((always_inline)) {
            set_b_slot(ring_off(t));
            v8 op[T1];
            static_for<0, (PF < T1 ? PF : T1)>([&](auto tc) { op[decltype(tc)::value] = fetch_b(tc); });
            static_for<0, T1>([&](auto tc) {
                constexpr int t_ = decltype(tc)::value;
                if constexpr (t_ + PF < T1) op[t_ + PF] = fetch_b(std::integral_constant<int, t_ + PF>{});
                g1_step(tc, nxtc, op[t_]);
                __builtin_amdgcn_sched_barrier(0x406);
            });
        };
        // what follows the softmax of a tile: the row sum, and the accumulators (which hold the
        // tiles before it, GEMM 2 of the previous tile included) brought to the new reference
        auto settle = [&]() __attribute__((always_inline)) {
#pragma unroll
            for (int mb = 0; SOFTMAX && mb < MB; ++mb) {
                l_run[mb] = l_run[mb] * corr[mb] + (sum0[mb] + sum1[mb]);
                if (__builtin_amdgcn_ballot_w64(corr[mb] != 1.0f)) {
#pragma unroll
                    for (int hb = 0; hb < HB; ++hb)
#pragma unroll
                        for (int r = 0; r < 16; ++r) accE[mb][hb][r] *= corr[mb];
                }
            }
        };
        // steady state (tiles i-1, i, i+1 all complete): one straight run, the steps of GEMM 2 of
        // tile i-1, then those of GEMM 1 of tile i+1, a slice of the softmax of tile i behind each
        auto steady = [&](auto curc, int i) __attribute__((always_inline)) {
            constexpr int CUR = decltype(curc)::value;
            const int n0 = i * TN + ncol0;
            set_d_slot(ring_off(i - 1));
            set_b_slot(ring_off(i + 1));
            v8 op[TT];
            auto fetch = [&](auto tc) __attribute__((always_inline)) {
                constexpr int t = decltype(tc)::value;
                if constexpr (t < T2) op[t] = fetch_d(tc);
                else op[t] = fetch_b(std::integral_constant<int, t - T2>{});
            };
            static_for<0, (PF < TT ? PF : TT)>([&](auto tc) { fetch(tc); });
            static_for<0, TT>([&](auto tc) {
                constexpr int t = decltype(tc)::value;
                if constexpr (t + PF < TT) fetch(std::integral_constant<int, t + PF>{});
                if constexpr (t < T2) g2_step(tc, op[t]);
                else g1_step(std::integral_constant<int, t - T2>{}, std::integral_constant<int, CUR ^ 1>{}, op[t]);
                vstep(tc, curc, n0);
                __builtin_amdgcn_sched_barrier(0);
            });
            settle();
        };
        // the softmax of tile t alone (first and last tiles; the last may be ragged, and a wave
        // whose slice of it is empty contributes P = 0)
        auto softmax_only = [&](auto curc, int t) __attribute__((always_inline)) {
            const int n0 = t * TN + ncol0;
            if (n0 < N) {
                static_for<0, TT>([&](auto tc) { vstep(tc, curc, n0); });
                settle();
            } else {
#pragma unroll
                for (int j = 0; j < NJ; ++j)
#pragma unroll
                    for (int mb = 0; mb < MB; ++mb)
#pragma unroll
                        for (int qp = 0; qp < 2; ++qp)
#pragma unroll
                            for (int e = 0; e < 8; ++e) pop[j][mb][qp][e] = (T)0.f;
            }
        };
        int slot_l = PRE; // ring slot the next requested tile goes to
        // top of iteration i: tile i+1 (if any) has landed, tile i+S-2 is requested
        auto top = [&](int i) __attribute__((always_inline)) {
            // at most the S-4 requests younger than tile i+1 may still be in flight
            if (i + S - 3 <= n_iters - 1) wait_vm<(S - 4) * P>();
            else wait_vm<0>();
            __syncthreads(); // tile i+1 is complete for every wave; the slot of tile i-2 is free
            if (i + S - 2 < n_iters) {
                issue_tile(i + S - 2, slot_l);
                slot_l = slot_l + 1 == S ? 0 : slot_l + 1;
            }
        };
        if (n_iters > 0) {
            const int last = n_iters - 1;
            // tile 0 (requested in the prologue, like tiles 1 .. PRE-1): GEMM 1 alone
            if (n_pre == PRE) wait_vm<(PRE - 1) * P>();
            else wait_vm<0>();
            __syncthreads();
            g1_only(std::integral_constant<int, 0>{}, 0);
            // iteration 0: no tile before it
            top(0);
            if (last >= 1) g1_only(std::integral_constant<int, 1>{}, 1);
            softmax_only(std::integral_constant<int, 0>{}, 0);
            // iterations 1 .. last-1: two per trip, the two C^T buffers swap roles at compile time
            int i = 1;
            for (; i + 1 <= last - 1; i += 2) {
                top(i);
                steady(std::integral_constant<int, 1>{}, i);
                top(i + 1);
                steady(std::integral_constant<int, 0>{}, i + 1);
            }
            if (i <= last - 1) {
                top(i);
                steady(std::integral_constant<int, 1>{}, i);
                ++i;
            }
            // iteration `last` (if it is not iteration 0): GEMM 2 of the tile before, softmax of the
            // last, which is moved to the first C^T buffer if it sits in the second (two copies of
            // the softmax, one per buffer, would keep both buffers alive to the end: registers)
            if (last >= 1) {
                if (last & 1) {
#pragma unroll
                    for (int j = 0; j < NJ; ++j)
#pragma unroll
                        for (int mb = 0; mb < MB; ++mb) cc[0][j][mb] = cc[1][j][mb];
                }
                top(last);
                g2_only(last - 1);
                softmax_only(std::integral_constant<int, 0>{}, last);
            }
            // GEMM 2 of the last tile
            g2_only(last);
        }
    } else if constexpr (!SKEW) {
        int stage_c = 0;     // ring slot of the tile being consumed
        int stage_l = S - 1; // ring slot the next issued tile goes to
        for (int it = 0; it < n_iters; ++it) {
            // Tiles it .. min(it+S-2, n_iters-1) are in flight.  Retire tile `it`: in the steady
            // state S-2 younger groups may stay in flight, near the end simply drain.
            if (n_iters - it >= S - 1) wait_vm<(S - 2) * P>();
            else wait_vm<0>();
            __syncthreads(); // tile `it` is complete for every wave; the slot of tile it-1 is free
            if (it + S - 1 < n_iters) {
                issue_tile(it + S - 1, stage_l);
                stage_l = stage_l + 1 == S ? 0 : stage_l + 1;
            }
            const int n0 = it * TN + wn * (32 * NJ); // first column of this wave's 32*NJ-wide slice
            if (n0 < N) {
                const unsigned st = stage_c * STAGE;
                phase_g1(st);
                phase_g2_prefetch(st);
                phase_sm(n0);
                phase_g2();
            }
            stage_c = stage_c + 1 == S ? 0 : stage_c + 1;
        }
    } else {
        // Per n-tile a wave does G1 (matrix pipe), SM (VALU), G2 (matrix pipe).  Waves w and
        // w+4 sit on the same SIMD; run in step they would both want the matrix pipe, then both
        // the VALU.  So the second group runs one phase behind: in iteration i it does SM and G2
        // of tile i-1 and then G1 of tile i, while the first group does G1, SM, G2 of tile i --
        // one group's softmax coincides with the other's MFMAs.  One barrier per iteration, as
        // before; tile i-1 stays in the ring through iteration i, so tile v is requested in
        // iteration v-S+2 and the ring is at least 3 deep.
        static_assert(S >= 3, "the skewed loop keeps two tiles live");
        const int grp = wave >> 2;
        auto top = [&](int i) __attribute__((always_inline)) {
            if (i == 0) {
                if (n_pre == S - 1) wait_vm<(S - 2) * P>();
                else wait_vm<0>();
            } else {
                if (i + S - 3 <= n_iters - 1) wait_vm<(S - 3) * P>();
                else wait_vm<0>();
            }
            __syncthreads(); // tile i is complete for every wave; the slot of tile i-2 is free
            if (i >= 1 && i + S - 2 < n_iters) issue_tile(i + S - 2, (i + S - 2) % S);
        };
        const int ncol0 = wn * (32 * NJ);
        if (grp == 0) {
            for (int i = 0; i < n_iters; ++i) {
                top(i);
                const int n0 = i * TN + ncol0;
                if (n0 < N) {
                    const unsigned st = (i % S) * STAGE;
                    phase_g1(st);
                    phase_g2_prefetch(st);
                    phase_sm(n0);
                    phase_g2();
                }
            }
        } else {
            auto finish_tile = [&](int t) __attribute__((always_inline)) { // SM and G2 of tile t
                const int n0 = t * TN + ncol0;
                if (n0 < N) {
                    phase_g2_prefetch((t % S) * STAGE);
                    phase_sm(n0);
                    phase_g2();
                }
            };
            top(0);
            if (ncol0 < N) phase_g1(0);
            for (int i = 1; i < n_iters; ++i) {
                top(i);
                finish_tile(i - 1);
                if (i * TN + ncol0 < N) {
                    phase_g1((i % S) * STAGE);
                }
            }
            if (n_iters > 0) finish_tile(n_iters - 1);
        }
    }

    // ---- finish the softmax denominator -----------------------------------------------------
    if (SOFTMAX) {
#pragma unroll
        for (int mb = 0; mb < MB; ++mb) l_run[mb] = xhalf_sum(l_run[mb]);
    }

    if constexpr (CH3) wait_vm<0>(); // the F tile (with N = 0 no loop iteration has waited for it)
    __syncthreads(); // every wave is done reading the ring: its space is reused below

    // ---- third GEMM: G^T[p][m] = sum_h F^T[p][h] E^T[h][m] --------------------------------------
    // It is linear in E, so with ns > 1 every wave applies it to its own partial E (of its n
    // slice) and the partial products are combined below exactly as the partial E would be.
    // The accumulator of GEMM 2 holds, in lane (c,g), E[row c][32hb + 16g + r]; its registers
    // 8qp .. 8qp+7, scaled and rounded to 16 bit, are the second MFMA operand for the 16
    // contraction indices h = 32hb + 16g' + 8qp + e (g' the half-wave, e = 0..7).  The first
    // operand is read from the F tile with the transposing read, rows h in that order,
    // columns p mapped as the h of GEMM 2 so that a lane again ends with 16 consecutive p.
    // Softmax: the partial E is divided by the wave's own row sum before the rounding (it is
    // then a convex combination of rows of D, whatever the sum), and the combine weighs the
    // waves by f_w * l_w instead of f_w.
    constexpr int PB = CH3 ? PD / 32 : 1;
    f32x16 accO[MB][PB]; // the product E.F (unused otherwise)
    if constexpr (CH3) {
        static_assert(NS == 1 || PD == LD, "the combine of the product reuses the layout of E");
        v8 eop[MB][HB][2];
#pragma unroll
        for (int mb = 0; mb < MB; ++mb) {
            const float inv_w = SOFTMAX ? (l_run[mb] > 0.f ? 1.0f / l_run[mb] : 0.f) : 1.0f;
#pragma unroll
            for (int hb = 0; hb < HB; ++hb)
#pragma unroll
                for (int qp = 0; qp < 2; ++qp)
#pragma unroll
                    for (int e = 0; e < 8; ++e) eop[mb][hb][qp][e] = (T)(accE[mb][hb][8 * qp + e] * inv_w);
        }
        const int x4 = i16 & 3;
        const int frow = 16 * g + (i16 >> 2); // + 32 hb + 8 qp; upper four contraction indices: + 4 rows
        const int fch = (u16 + 2 * (x4 & 1)) ^ swz_tr(RBF, frow);
        const unsigned f_off = (unsigned)(F_LDS + frow * RBF + 16 * fch + 8 * (x4 >> 1)); // p block 0; per pb: ^ (64 pb) bytes
#pragma unroll
        for (int mb = 0; mb < MB; ++mb)
#pragma unroll
            for (int pb = 0; pb < PB; ++pb)
#pragma unroll
                for (int r = 0; r < 16; ++r) accO[mb][pb][r] = 0.f;
#pragma unroll
        for (int pb = 0; pb < PB; ++pb)
#pragma unroll
            for (int hb = 0; hb < HB; ++hb)
#pragma unroll
                for (int qp = 0; qp < 2; ++qp) {
                    const lds_u8 *src = smem + (f_off ^ (unsigned)(64 * pb)) + (32 * hb + 8 * qp) * RBF;
                    i16x4 lo = lds_read_tr(src);
                    i16x4 hi = lds_read_tr(src + 4 * RBF);
                    const v8 fop = __builtin_bit_cast(v8, __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7));
#pragma unroll
                    for (int mb = 0; mb < MB; ++mb) accO[mb][pb] = M_::run(fop, eop[mb][hb][qp], accO[mb][pb]);
                }
        if constexpr (NS > 1) { // from here on the partial products take the place of the partial E
#pragma unroll
            for (int mb = 0; mb < MB; ++mb)
#pragma unroll
                for (int hb = 0; hb < HB; ++hb) accE[mb][hb] = accO[mb][hb];
        }
    }

    // ---- combine the ns partial results of a row-group -----------------------------------
    // The MB*HB accumulator blocks (32 rows x 32 columns of E each) of a row-group are dealt
    // out to its ns waves in contiguous runs of BPW; every wave parks the blocks it does not
    // own (and its softmax state) in LDS, then reduces and stores the blocks it owns, so the
    // reduction and the store are spread over all waves.  Partial results are summed in wave
    // order, which makes the result independent of timing.
    constexpr int BPW = blocks_per_wave(LD, MB, NS);
    const int blk0 = wn * BPW; // this wave owns blocks [blk0, blk0 + BPW) that exist
    if (NS > 1) {
        constexpr int PARK = parked_blocks(LD, MB, NS); // blocks a wave parks (those it does not own)
        constexpr int PER_W = PARK * 16 + 2 * MB;       // floats per lane per wave
        lds_f32 *scr = (lds_f32 *)smem + (wr * NS) * PER_W * 64 + lane;
        lds_f32 *mine = scr + wn * PER_W * 64;
#pragma unroll
        for (int mb = 0; mb < MB; ++mb) {
#pragma unroll
            for (int hb = 0; hb < HB; ++hb) {
                const int blk = mb * HB + hb;
                if (blk < blk0 || blk >= blk0 + BPW) {
                    const int pidx = blk >= blk0 + BPW ? blk - BPW : blk; // skip the run this wave owns
#pragma unroll
                    for (int r = 0; r < 16; ++r) mine[(pidx * 16 + r) * 64] = accE[mb][hb][r];
                }
            }
            if (SOFTMAX) {
                mine[(PARK * 16 + 2 * mb) * 64] = m_run[mb];
                mine[(PARK * 16 + 2 * mb + 1) * 64] = l_run[mb];
            }
        }
        __syncthreads();
#pragma unroll
        for (int mb = 0; mb < MB; ++mb) {
            // blocks mb*HB .. mb*HB+HB-1: does this wave own one of them?
            if (blk0 < (mb + 1) * HB && blk0 + BPW > mb * HB) {
                float f[NS];
                if (SOFTMAX) {
                    float mw[NS], lw[NS];
                    float m_all = -INFINITY;
#pragma unroll
                    for (int w = 0; w < NS; ++w) {
                        mw[w] = scr[(w * PER_W + PARK * 16 + 2 * mb) * 64];
                        lw[w] = scr[(w * PER_W + PARK * 16 + 2 * mb + 1) * 64];
                        m_all = fmaxf(m_all, mw[w]);
                    }
                    float l_all = 0.f;
#pragma unroll
                    for (int w = 0; w < NS; ++w) {
                        // a wave that saw no column has m = -inf, l = 0 and a zero accumulator
                        f[w] = (mw[w] == -INFINITY) ? 0.f : __builtin_amdgcn_exp2f((mw[w] - m_all) * c1);
                        l_all += f[w] * lw[w];
                        if (CH3) f[w] *= lw[w]; // the partial products were formed from E_w / l_w
                    }
                    l_run[mb] = l_all;
                }
#pragma unroll
                for (int hb = 0; hb < HB; ++hb) {
                    const int blk = mb * HB + hb;
                    if (blk >= blk0 && blk < blk0 + BPW) {
#pragma unroll
                        for (int r = 0; r < 16; ++r) {
                            float acc = 0.f;
#pragma unroll
                            for (int w = 0; w < NS; ++w) {
                                // where wave w parked this block (w does not own it when w != wn)
                                const int pidx = blk >= (w + 1) * BPW ? blk - BPW : blk;
                                const float part = (w == wn) ? accE[mb][hb][r] : scr[(w * PER_W + pidx * 16 + r) * 64];
                                acc += SOFTMAX ? f[w] * part : part;
                            }
                            accE[mb][hb][r] = acc;
                        }
                    }
                }
            }
        }
    }

    float inv[MB];
#pragma unroll
    for (int mb = 0; mb < MB; ++mb) inv[mb] = SOFTMAX ? (l_run[mb] > 0.f ? 1.0f / l_run[mb] : 0.f) : 1.0f; // (a row that saw no column: zeros)

    // ---- S_E: output tile -> global ---------------------------------------------------------
    // Lane (c,g) holds X[row c][32hb + 16g + 0..15] of the blocks its wave owns (X = E, or the
    // product E.F of the three-GEMM chain; LDX columns).  They are scaled (E by 1 / row sum),
    // staged in LDS (swizzled) and read back so that consecutive lanes store consecutive
    // 16-byte pieces of a row: a store instruction writes whole row segments (whole rows when
    // the wave owns all h blocks of its rows).
    constexpr int LDX = CH3 ? PD : LD;
    constexpr int HBX = h_blocks(LDX);
    constexpr int BPWX = blocks_per_wave(LDX, MB, NS);
    const int blk0x = wn * BPWX; // this wave owns blocks [blk0x, blk0x + BPWX) that exist
    // fp32 output (bit 0 of the output pointer, which is 16-byte aligned, says so: a flag of its
    // own would occupy a scalar register from the first instruction to here): the accumulators go
    // out as they are held, 16 consecutive columns of a row per lane in four 16-byte stores
    const bool out_f32 = ((uintptr_t)p.E & 1) != 0;
    if (out_f32) {
        float *Ef = (float *)((char *)p.E - 1) + batch * p.se_b + ht * LD; // (pointer arithmetic, so that the stores stay global ones)
#pragma unroll
        for (int mb = 0; mb < MB; ++mb) {
            const int row = wrow0 + 32 * mb + c;
#pragma unroll
            for (int hb = 0; hb < HBX; ++hb) {
                const int blk = mb * HBX + hb;
                if (blk >= blk0x && blk < blk0x + BPWX && row < M) {
#pragma unroll
                    for (int q = 0; q < 4; ++q) {
                        f32x4 v;
#pragma unroll
                        for (int e = 0; e < 4; ++e) {
                            if constexpr (CH3 && NS == 1) v[e] = accO[mb][hb][4 * q + e];
                            else v[e] = accE[mb][hb][4 * q + e] * inv[mb];
                        }
                        const int col = 32 * hb + 16 * g + 4 * q;
                        if (col < LDX) __builtin_nontemporal_store(v, (f32x4 *)(Ef + (int64_t)row * se_r + col));
                    }
                }
            }
        }
    } else if (blk0x < MB * HBX) {
        static_assert(combine_runs_ok(LDX, MB, NS), "a wave's run of blocks straddles row sets");
        constexpr int HPW = BPWX < HBX ? BPWX : HBX;     // h blocks per owned row set
        constexpr int MPW = BPWX < HBX ? 1 : BPWX / HBX; // row sets (of 32 rows) owned
        constexpr int RBS = estage_row_bytes(LDX, MB, NS); // staged row bytes: HPW * 64, rounded up to a power of two
        constexpr bool EPAD = RBS != HPW * 64 || pitch_elems(LDX) != LDX; // some staged pieces are padding or lie beyond the last column
        const int mb0 = blk0x / HBX, h0 = blk0x % HBX;
        lds_u8 *es = smem + combine_bytes(LDX, MB, RG, NS) + wave * estage_wave_bytes(LDX, MB, NS);
#pragma unroll
        for (int mb = 0; mb < MB; ++mb) {
            const float sc = inv[mb]; // (the product of a single wave per row set is final: not scaled)
#pragma unroll
            for (int hb = 0; hb < HBX; ++hb) {
                const int blk = mb * HBX + hb;
                if (blk >= blk0x && blk < blk0x + BPWX) {
                    const int row = 32 * (mb - mb0) + c;
                    const int sw = swz_b128(RBS, row);
                    v8 lo, hi;
#pragma unroll
                    for (int e = 0; e < 8; ++e) {
                        if constexpr (CH3 && NS == 1) {
                            lo[e] = (T)accO[mb][hb][e];
                            hi[e] = (T)accO[mb][hb][8 + e];
                        } else {
                            lo[e] = (T)(accE[mb][hb][e] * sc);
                            hi[e] = (T)(accE[mb][hb][8 + e] * sc);
                        }
                    }
                    const int ch = 4 * (hb - h0) + 2 * g;
                    *(lds_u32x4 *)(es + row * RBS + 16 * (ch ^ sw)) = __builtin_bit_cast(u32x4, lo);
                    *(lds_u32x4 *)(es + row * RBS + 16 * ((ch + 1) ^ sw)) = __builtin_bit_cast(u32x4, hi);
                }
            }
        }
        constexpr int CPR = RBS / 16;               // 16-byte pieces per staged row
        constexpr int PASSES = MPW * 32 * CPR / 64; // wave-wide stores
        const int rbase = mrow0 + wr * (32 * MB) + 32 * mb0;
#pragma unroll
        for (int ps = 0; ps < PASSES; ++ps) {
            const int slot = 64 * ps + lane;
            const int row = slot / CPR;
            const int ch = (slot % CPR) ^ swz_b128(RBS, row);
            const u32x4 v = *(const lds_u32x4 *)(es + 16 * slot);
            if (EPAD && (ch >= 4 * HPW || 32 * h0 + 8 * ch >= LDX)) continue;
            if (rbase + row < M)
                __builtin_nontemporal_store(v, (u32x4 *)(Eg + (int64_t)(rbase + row) * se_r + 32 * h0 + 8 * ch));
        }
    }
}

// Host-side launcher of one instantiation.
// LDS bytes of an instantiation.
template <int KD, int LD, int MB, int RG, int NS, int NJ, bool SOFTMAX, bool KSPLIT, int PD>
constexpr int kernel_lds_bytes() {
    constexpr int S = ring_stages(KD, LD, MB, RG, NS, NJ, SOFTMAX, KSPLIT, PD > 0 ? chain3_f_bytes(LD, PD) + 1024 : 0);
    if constexpr (PD > 0) return chain3_lds_bytes(KD, LD, PD, MB, RG, NS, NJ, S);
    else return total_lds_bytes(KD, LD, MB, RG, NS, NJ, S, KSPLIT);
}

template <typename T, int KD, int LD, int MB, int RG, int NS, int NJ, bool SOFTMAX, bool BKC, bool KSPLIT = false, int PD = 0>
int launch_chain(const KParams &p, void *stream) {
    constexpr int lds = kernel_lds_bytes<KD, LD, MB, RG, NS, NJ, SOFTMAX, KSPLIT, PD>();
    auto kern = chain_kernel<T, KD, LD, MB, RG, NS, NJ, SOFTMAX, BKC, KSPLIT, PD>;
    // More than 64 KiB of dynamic LDS has to be allowed per function and device, once.  (A race
    // between two threads sets the attribute twice, which is harmless.)
    if (lds > 64 * 1024) {
        static bool attr_done[64] = {};
        int dev = 0;
        hipError_t e = hipGetDevice(&dev);
        if (e != hipSuccess) return (int)e;
        if (dev < 0 || dev >= 64 || !attr_done[dev]) {
            e = hipFuncSetAttribute((const void *)kern, hipFuncAttributeMaxDynamicSharedMemorySize, lds);
            if (e != hipSuccess) return (int)e;
            if (dev >= 0 && dev < 64) attr_done[dev] = true;
        }
    }
    hipLaunchKernelGGL(kern, dim3(p.n_blocks), dim3(64 * RG * NS), lds, (hipStream_t)stream, p);
    return (int)hipGetLastError();
}

// Launcher of an instantiation, or nullptr when the wave arrangement cannot exist for this
// (K, L): more LDS than a compute unit has, or (L not a multiple of 32 times a power of two) a
// wave's run of accumulator blocks would straddle row sets.  Such kernels are not compiled.
template <typename T, int KD, int LD, int MB, int RG, int NS, int NJ, bool SOFTMAX, bool BKC, bool KSPLIT = false, int PD = 0>
constexpr LaunchFn launcher_or_null() {
    if constexpr (kernel_lds_bytes<KD, LD, MB, RG, NS, NJ, SOFTMAX, KSPLIT, PD>() <= kLdsBytesPerBlock &&
                  combine_runs_ok(LD, MB, NS) && (PD == 0 || NS == 1 || PD == LD))
        return &launch_chain<T, KD, LD, MB, RG, NS, NJ, SOFTMAX, BKC, KSPLIT, PD>;
    else
        return nullptr;
}

} // namespace mcf

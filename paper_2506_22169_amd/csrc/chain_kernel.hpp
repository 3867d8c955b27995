// Fused two-GEMM chain kernel for gfx950 (CDNA4):  E = (A.B).D  or  E = softmax(scale*A.B).D
//
// Per-block schedule = the paper's "nk" sub-tiling expression with T_K = K, T_L = L
// (Sec. III-B/C): the k and h loops have extent 1, so L_A is hoisted to the block (A tile
// loaded once into registers) and S_E is hoisted out of the n loop (E stored once):
//
//   block <-> (batch, m-tile)                               [spatial loops on the block index]
//   A tile -> VGPRs                                         [L_A, once]
//   for each n-tile:   B tile, D tile -> LDS (2 stages)     [L_B, L_D]
//                      C^T = B^T . A^T        (MFMA)        [C_C]
//                      optional online softmax on C^T, convert to 16-bit in registers
//                      E^T += D^T . C^T       (MFMA)        [C_E]
//   E tile -> global                                        [S_E, once]
//
// Both GEMMs are computed transposed so that the fp32 accumulator of the first is, lane for
// lane, already the second operand of the second: the intermediate never leaves registers.
//
// MFMA v_mfma_f32_32x32x16_{f16,bf16}: lane l = (c = l%32, g = l/32).
//   first operand  X[32 x 16]: lane holds X[c][8g .. 8g+7]
//   second operand Y[16 x 32]: lane holds Y[8g .. 8g+7][c]
//   result         Z[32 x 32]: lane holds Z[8(r/4) + 4g + r%4][c], r = 0..15
//
// Waves of a block form an rg x ns grid: wave (wr, wn) owns rows [wr*32*MB, +32*MB) of the
// block's m-tile and columns [wn*32, +32) of every n-tile; with ns > 1 the partial results of
// the ns waves of a row-group are combined through LDS after the loop.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "mcf_geometry.h"
#include "mcf_internal.h"

namespace mcf {

typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef short i16x4 __attribute__((ext_vector_type(4)));
typedef short i16x8 __attribute__((ext_vector_type(8)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef __attribute__((address_space(3))) i16x4 lds_i16x4;

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
static __device__ __forceinline__ i16x4 lds_read_tr(const unsigned char *p) {
    return __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_i16x4 *)p);
}

template <typename T, int KD, int LD, int MB, int RG, int NS, bool SOFTMAX, bool BKC>
__global__ __launch_bounds__(64 * RG * NS) void chain_kernel(const KParams p) {
    using M_ = Mfma<T>;
    using v8 = typename M_::v8;
    constexpr int NT = 64 * RG * NS;    // threads per block
    constexpr int TM = 32 * MB * RG;    // rows per block
    constexpr int TN = 32 * NS;         // columns per n-iteration
    constexpr int KS = KD / 16;         // MFMA k-steps of GEMM 1
    constexpr int HB = LD / 32;         // 32-wide h blocks of GEMM 2
    constexpr int PB = BKC ? pitch_bk(KD) : pitch_tr(TN); // B tile row pitch (bytes)
    constexpr int PD = pitch_tr(LD);                      // D tile row pitch (bytes)
    constexpr int B_BYTES = b_tile_bytes(KD, TN, BKC);
    constexpr int STAGE = stage_bytes(KD, LD, TN, BKC);
    // 16-byte chunks of one B / D tile and how many each thread moves
    constexpr int B_CHUNKS = KD * TN / 8;
    constexpr int D_CHUNKS = TN * LD / 8;
    constexpr int B_PER_T = (B_CHUNKS + NT - 1) / NT;
    constexpr int D_PER_T = (D_CHUNKS + NT - 1) / NT;

    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];

    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int c = lane & 31, g = lane >> 5;
    const int wr = wave / NS, wn = wave % NS;

    // Block index -> (batch, m-tile).  Consecutive hardware block ids go round-robin over the
    // 8 XCDs (each with its own L2); give every XCD a contiguous range of logical blocks so the
    // m-tiles of one batch re-read that batch's B and D from one L2.
    int logical;
    {
        const int hw = blockIdx.x, nb = p.n_blocks;
        const int x = hw & 7, q = nb >> 3, rem = nb & 7;
        logical = x * q + (x < rem ? x : rem) + (hw >> 3);
    }
    const int batch = logical / p.m_tiles;
    const int mt = logical - batch * p.m_tiles;
    const int m0 = mt * TM + wr * (32 * MB);

    const T *Ag = (const T *)p.A + batch * p.sa_b;
    const T *Bg = (const T *)p.B + batch * p.sb_b;
    const T *Dg = (const T *)p.D + batch * p.sd_b;
    T *Eg = (T *)p.E + batch * p.se_b;

    // ---- L_A: A tile -> registers, as the second MFMA operand A^T[k][m] ------------------
    v8 a[MB][KS];
#pragma unroll
    for (int mb = 0; mb < MB; ++mb) {
        const int row = m0 + 32 * mb + c;
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) {
            u32x4 raw = {0u, 0u, 0u, 0u};
            if (row < p.M && p.a_mode != 2) raw = *(const u32x4 *)(Ag + (int64_t)row * p.sa_r + 16 * ks + 8 * g);
            if (p.a_mode == 1) raw ^= 0x80008000u; // flip the sign of all eight 16-bit floats
            a[mb][ks] = __builtin_bit_cast(v8, raw);
        }
    }

    // ---- per-thread source / destination of the B and D tile chunks ----------------------
    // B tile: BKC  -> rows n (TN of them), KD contiguous k: chunk q -> (row q/(KD/8), col 8*(q%(KD/8)))
    //         !BKC -> rows k (KD of them), TN contiguous n: chunk q -> (row q/(TN/8), col 8*(q%(TN/8)))
    // D tile: rows n (TN), LD contiguous h.
    u32x4 breg[B_PER_T], dreg[D_PER_T];

    auto load_tiles = [&](int nt0) {
#pragma unroll
        for (int u = 0; u < B_PER_T; ++u) {
            const int q = tid + u * NT;
            u32x4 v = {0u, 0u, 0u, 0u};
            if (B_CHUNKS % NT == 0 || q < B_CHUNKS) {
                if (BKC) {
                    const int r = q / (KD / 8), cc = q % (KD / 8);
                    if (nt0 + r < p.N) v = *(const u32x4 *)(Bg + (int64_t)(nt0 + r) * p.sb_r + 8 * cc);
                } else {
                    const int r = q / (TN / 8), cc = q % (TN / 8);
                    if (nt0 + 8 * cc < p.N) v = *(const u32x4 *)(Bg + (int64_t)r * p.sb_r + nt0 + 8 * cc);
                }
            }
            breg[u] = v;
        }
#pragma unroll
        for (int u = 0; u < D_PER_T; ++u) {
            const int q = tid + u * NT;
            u32x4 v = {0u, 0u, 0u, 0u};
            if (D_CHUNKS % NT == 0 || q < D_CHUNKS) {
                const int r = q / (LD / 8), cc = q % (LD / 8);
                if (nt0 + r < p.N) v = *(const u32x4 *)(Dg + (int64_t)(nt0 + r) * p.sd_r + 8 * cc);
            }
            dreg[u] = v;
        }
    };
    auto store_tiles = [&](int stage) {
        unsigned char *sB = smem + stage * STAGE;
        unsigned char *sD = sB + B_BYTES;
#pragma unroll
        for (int u = 0; u < B_PER_T; ++u) {
            const int q = tid + u * NT;
            if (B_CHUNKS % NT == 0 || q < B_CHUNKS) {
                const int r = BKC ? q / (KD / 8) : q / (TN / 8);
                const int cc = BKC ? q % (KD / 8) : q % (TN / 8);
                *(u32x4 *)(sB + r * PB + 16 * cc) = breg[u];
            }
        }
#pragma unroll
        for (int u = 0; u < D_PER_T; ++u) {
            const int q = tid + u * NT;
            if (D_CHUNKS % NT == 0 || q < D_CHUNKS) {
                const int r = q / (LD / 8), cc = q % (LD / 8);
                *(u32x4 *)(sD + r * PD + 16 * cc) = dreg[u];
            }
        }
    };

    // ---- loop-invariant LDS read offsets of this lane --------------------------------------
    const int i16 = lane & 15, u16 = (lane >> 4) & 1;
    // B operand of GEMM 1 (first MFMA operand B^T[n][k]): n = wn*32 + c, k = 16ks + 8g + 0..7
    const int b_off = BKC ? (wn * 32 + c) * PB + 16 * g
                          : (8 * g + (i16 >> 2)) * PB + (wn * 32 + 16 * u16 + 4 * (i16 & 3)) * 2;
    // D operand of GEMM 2 (first MFMA operand D^T[h][n]).  MFMA row i of the h block is mapped
    // to h = 16*((i>>2)&1) + 4*(i>>3) + (i&3) so that the accumulator of lane (c,g) ends up
    // holding 16 consecutive h:  h = 32hb + 16g + r.
    const int x4 = i16 & 3;
    const int d_off = (wn * 32 + 4 * g + (i16 >> 2)) * PD + (8 * u16 + 16 * (x4 & 1) + 4 * (x4 >> 1)) * 2;

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

    const int n_iters = (p.N + TN - 1) / TN;
    if (n_iters > 0) {
        load_tiles(0);
        store_tiles(0);
    }
    __syncthreads();

    for (int it = 0; it < n_iters; ++it) {
        const int nt0 = it * TN;
        const bool more = it + 1 < n_iters;
        if (more) load_tiles(nt0 + TN); // global loads in flight during the MFMAs below

        const unsigned char *sB = smem + (it & 1) * STAGE;
        const unsigned char *sD = sB + B_BYTES;
        const int n0 = nt0 + wn * 32; // first column of this wave's 32-wide slice

        if (n0 < p.N) {
            // ---- C_C: C^T[n][m] = sum_k B^T[n][k] A^T[k][m] ---------------------------------
            f32x16 accC[MB];
#pragma unroll
            for (int mb = 0; mb < MB; ++mb)
#pragma unroll
                for (int r = 0; r < 16; ++r) accC[mb][r] = 0.f;
#pragma unroll
            for (int ks = 0; ks < KS; ++ks) {
                v8 bop;
                if (BKC) {
                    bop = __builtin_bit_cast(v8, *(const u32x4 *)(sB + b_off + 32 * ks));
                } else {
                    i16x4 lo = lds_read_tr(sB + b_off + (16 * ks) * PB);
                    i16x4 hi = lds_read_tr(sB + b_off + (16 * ks + 4) * PB);
                    i16x8 both = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
                    bop = __builtin_bit_cast(v8, both);
                }
#pragma unroll
                for (int mb = 0; mb < MB; ++mb) accC[mb] = M_::run(bop, a[mb][ks], accC[mb]);
            }

            // ---- softmax (online max / sum over n-tiles) and conversion to 16 bit -----------
            // Lane (c,g) holds, for row m = c, the 16 columns n = n0 + 8(r/4) + 4g + r%4.
            v8 pop[MB][2];
#pragma unroll
            for (int mb = 0; mb < MB; ++mb) {
                f32x16 s = accC[mb];
                if (SOFTMAX) {
                    if (n0 + 32 > p.N) {
#pragma unroll
                        for (int r = 0; r < 16; ++r)
                            if (n0 + 8 * (r / 4) + 4 * g + (r % 4) >= p.N) s[r] = -INFINITY;
                    }
                    float mx = s[0];
#pragma unroll
                    for (int r = 1; r < 16; ++r) mx = fmaxf(mx, s[r]);
                    mx = xhalf_max(mx);
                    const float m_new = fmaxf(m_run[mb], mx);
                    const float corr = __builtin_amdgcn_exp2f((m_run[mb] - m_new) * p.c1);
                    const float mneg = -m_new * p.c1;
                    float sum = 0.f;
#pragma unroll
                    for (int r = 0; r < 16; ++r) {
                        s[r] = __builtin_amdgcn_exp2f(__builtin_fmaf(s[r], p.c1, mneg));
                        sum += s[r];
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
                for (int qp = 0; qp < 2; ++qp)
#pragma unroll
                    for (int e = 0; e < 8; ++e) pop[mb][qp][e] = (T)s[8 * qp + e];
            }

            // ---- C_E: E^T[h][m] += sum_n D^T[h][n] P^T[n][m] --------------------------------
#pragma unroll
            for (int hb = 0; hb < HB; ++hb) {
#pragma unroll
                for (int qp = 0; qp < 2; ++qp) {
                    const unsigned char *src = sD + d_off + (16 * qp) * PD + 64 * hb;
                    i16x4 lo = lds_read_tr(src);
                    i16x4 hi = lds_read_tr(src + 8 * PD);
                    i16x8 both = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
                    v8 dop = __builtin_bit_cast(v8, both);
#pragma unroll
                    for (int mb = 0; mb < MB; ++mb) accE[mb][hb] = M_::run(dop, pop[mb][qp], accE[mb][hb]);
                }
            }
        }

        if (more) store_tiles((it + 1) & 1);
        __syncthreads();
    }

    // ---- finish the softmax denominator -----------------------------------------------------
    if (SOFTMAX) {
#pragma unroll
        for (int mb = 0; mb < MB; ++mb) l_run[mb] = xhalf_sum(l_run[mb]);
    }

    // ---- combine the ns partial results of a row-group (waves wn > 0 -> wave wn == 0) -------
    if (NS > 1) {
        constexpr int PER_MB = HB * 16 + 2; // floats per lane per mb
        float *scratch = (float *)smem;     // staging buffers are dead after the last barrier
        if (wn > 0) {
            float *dst = scratch + ((wr * (NS - 1) + (wn - 1)) * MB) * PER_MB * 64 + lane;
#pragma unroll
            for (int mb = 0; mb < MB; ++mb) {
#pragma unroll
                for (int hb = 0; hb < HB; ++hb)
#pragma unroll
                    for (int r = 0; r < 16; ++r) dst[(mb * PER_MB + hb * 16 + r) * 64] = accE[mb][hb][r];
                dst[(mb * PER_MB + HB * 16) * 64] = m_run[mb];
                dst[(mb * PER_MB + HB * 16 + 1) * 64] = l_run[mb];
            }
        }
        __syncthreads();
        if (wn == 0) {
#pragma unroll
            for (int w = 1; w < NS; ++w) {
                const float *src = scratch + ((wr * (NS - 1) + (w - 1)) * MB) * PER_MB * 64 + lane;
#pragma unroll
                for (int mb = 0; mb < MB; ++mb) {
                    float f_own = 1.f, f_oth = 1.f;
                    if (SOFTMAX) {
                        const float m_o = src[(mb * PER_MB + HB * 16) * 64];
                        const float l_o = src[(mb * PER_MB + HB * 16 + 1) * 64];
                        const float m_new = fmaxf(m_run[mb], m_o);
                        // a wave that saw no column has m = -inf, l = 0 and a zero accumulator
                        f_own = (m_run[mb] == -INFINITY) ? 0.f : __builtin_amdgcn_exp2f((m_run[mb] - m_new) * p.c1);
                        f_oth = (m_o == -INFINITY) ? 0.f : __builtin_amdgcn_exp2f((m_o - m_new) * p.c1);
                        l_run[mb] = l_run[mb] * f_own + l_o * f_oth;
                        m_run[mb] = m_new;
                    }
#pragma unroll
                    for (int hb = 0; hb < HB; ++hb)
#pragma unroll
                        for (int r = 0; r < 16; ++r) {
                            const float o = src[(mb * PER_MB + hb * 16 + r) * 64];
                            accE[mb][hb][r] = SOFTMAX ? accE[mb][hb][r] * f_own + o * f_oth : accE[mb][hb][r] + o;
                        }
                }
            }
        }
    }

    // ---- S_E: E tile -> global.  Lane (c,g) holds E[m0+32mb+c][32hb + 16g + 0..15]. ----------
    if (NS == 1 || wn == 0) {
#pragma unroll
        for (int mb = 0; mb < MB; ++mb) {
            const int row = m0 + 32 * mb + c;
            const float inv = SOFTMAX ? 1.0f / l_run[mb] : 1.0f;
            if (row < p.M) {
                T *dst = Eg + (int64_t)row * p.se_r + 16 * g;
#pragma unroll
                for (int hb = 0; hb < HB; ++hb) {
                    v8 lo, hi;
#pragma unroll
                    for (int e = 0; e < 8; ++e) {
                        lo[e] = (T)(accE[mb][hb][e] * inv);
                        hi[e] = (T)(accE[mb][hb][8 + e] * inv);
                    }
                    *(u32x4 *)(dst + 32 * hb) = __builtin_bit_cast(u32x4, lo);
                    *(u32x4 *)(dst + 32 * hb + 8) = __builtin_bit_cast(u32x4, hi);
                }
            }
        }
    }
}

// Host-side launcher of one instantiation.
template <typename T, int KD, int LD, int MB, int RG, int NS, bool SOFTMAX, bool BKC>
int launch_chain(const KParams &p, void *stream) {
    constexpr int LDS = total_lds_bytes(KD, LD, MB, RG, NS, BKC);
    auto kern = chain_kernel<T, KD, LD, MB, RG, NS, SOFTMAX, BKC>;
    static bool attr_done = false; // benign race: setting the attribute twice is harmless
    if (LDS > 64 * 1024 && !attr_done) {
        hipError_t e = hipFuncSetAttribute((const void *)kern, hipFuncAttributeMaxDynamicSharedMemorySize, LDS);
        if (e != hipSuccess) return (int)e;
        attr_done = true;
    }
    hipLaunchKernelGGL(kern, dim3(p.n_blocks), dim3(64 * RG * NS), LDS, (hipStream_t)stream, p);
    return (int)hipGetLastError();
}

} // namespace mcf

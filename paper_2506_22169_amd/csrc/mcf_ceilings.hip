// Measurement aids: the three kernels whose times bound what the chain kernel can reach on this
// machine -- a streaming copy (HBM), a loop of nothing but MFMAs (matrix pipe) and an empty
// kernel (launch floor).  They take no part in the chain; bench.py --ceilings times them with
// the same graph-replay protocol as the chain kernel.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "../../include/mcf.h"

namespace {

typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

// dst[i] = src[i], 16 bytes per lane and step, grid-stride; streaming hints on both sides.
__global__ __launch_bounds__(256) void copy_kernel(u32x4 *__restrict__ dst, const u32x4 *__restrict__ src, int64_t n16) {
    const int64_t stride = (int64_t)gridDim.x * 256;
    for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < n16; i += stride)
        __builtin_nontemporal_store(__builtin_nontemporal_load(src + i), dst + i);
}

// iters x 8 independent v_mfma_f32_32x32x16_f16 per wave on register operands; the sums are
// stored so that nothing is optimised away.
__global__ __launch_bounds__(512) void mfma_kernel(float *__restrict__ out, int iters) {
    f16x8 x, y;
    for (int e = 0; e < 8; ++e) {
        x[e] = (_Float16)(float)((threadIdx.x + e) & 7);
        y[e] = (_Float16)(float)((threadIdx.x * 3 + e) & 3);
    }
    f32x16 acc[8];
    for (int a = 0; a < 8; ++a)
        for (int r = 0; r < 16; ++r) acc[a][r] = 0.f;
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int a = 0; a < 8; ++a) acc[a] = __builtin_amdgcn_mfma_f32_32x32x16_f16(x, y, acc[a], 0, 0, 0);
    }
    float s = 0.f;
    for (int a = 0; a < 8; ++a)
        for (int r = 0; r < 16; ++r) s += acc[a][r];
    out[(int64_t)blockIdx.x * blockDim.x + threadIdx.x] = s;
}

__global__ void empty_kernel() {}

} // namespace

extern "C" int mcf_probe_copy(void *dst, const void *src, int64_t bytes, void *stream) {
    if (!dst || !src || bytes < 0 || bytes % 16 != 0 || (uintptr_t)dst % 16 != 0 || (uintptr_t)src % 16 != 0) return MCF_EINVAL;
    if (bytes == 0) return MCF_OK;
    const int64_t n16 = bytes / 16;
    int64_t blocks = (n16 + 255) / 256;
    if (blocks > 256 * 16) blocks = 256 * 16; // 16 resident blocks of 4 waves per compute unit
    hipLaunchKernelGGL(copy_kernel, dim3((unsigned)blocks), dim3(256), 0, (hipStream_t)stream, (u32x4 *)dst, (const u32x4 *)src, n16);
    return hipGetLastError() == hipSuccess ? MCF_OK : MCF_ELAUNCH;
}

extern "C" int mcf_probe_mfma(void *out, int32_t blocks, int32_t waves_per_block, int32_t iters, void *stream) {
    if (!out || blocks <= 0 || waves_per_block <= 0 || waves_per_block > 8 || iters < 0) return MCF_EINVAL;
    hipLaunchKernelGGL(mfma_kernel, dim3(blocks), dim3(64 * waves_per_block), 0, (hipStream_t)stream, (float *)out, iters);
    return hipGetLastError() == hipSuccess ? MCF_OK : MCF_ELAUNCH;
}

extern "C" int mcf_probe_empty(int32_t blocks, void *stream) {
    if (blocks <= 0) return MCF_EINVAL;
    hipLaunchKernelGGL(empty_kernel, dim3(blocks), dim3(64), 0, (hipStream_t)stream);
    return hipGetLastError() == hipSuccess ? MCF_OK : MCF_ELAUNCH;
}

// Two calibration kernels for the benchmark: what this GPU, on this day and at its power limit, sustains for a
// plain streaming copy and for bf16 matrix instructions fed from registers.  The benchmark reports its roofline
// fractions against the published peaks and against these.  Nothing of the layer's path calls them.
#include "internal.h"

namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 cal_bf16x8;
typedef __attribute__((ext_vector_type(16))) float cal_f32x16;

// dst[i] = src[i], 16 bytes per lane, four requests in flight per lane, grid-stride.
__global__ __launch_bounds__(256) void calib_copy_kernel(const uint4* __restrict__ src, uint4* __restrict__ dst, size_t n16)
{
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    for (; i + 3 * stride < n16; i += 4 * stride) {
        const uint4 a = src[i], b = src[i + stride], c = src[i + 2 * stride], d = src[i + 3 * stride];
        dst[i] = a; dst[i + stride] = b; dst[i + 2 * stride] = c; dst[i + 3 * stride] = d;
    }
    for (; i < n16; i += stride) dst[i] = src[i];
}

// Every wave issues `iters` rounds of eight independent 32x32x16 bf16 matrix instructions (the accumulator
// layout of the grouped kernel: 4 x 2 fragments) on operands that never leave its registers.  The operands
// are not all zero, so the multipliers toggle as they do on real data.
__global__ __launch_bounds__(512) void calib_mfma_kernel(float* __restrict__ out, int iters)
{
    const int lane = threadIdx.x & 63;
    cal_bf16x8 a[4], b[2];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int e = 0; e < 8; ++e) a[i][e] = (__bf16)(0.001f * (float)((lane * 7 + i * 13 + e * 3) % 17 - 8));
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
        for (int e = 0; e < 8; ++e) b[j][e] = (__bf16)(0.001f * (float)((lane * 5 + j * 11 + e) % 13 - 6));
    cal_f32x16 acc[4][2];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.0f;
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int i = 0; i < 4; ++i)
#pragma unroll
            for (int j = 0; j < 2; ++j)
                acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(b[j], a[i], acc[i][j], 0, 0, 0);
    }
    float s = 0.0f;
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int e = 0; e < 16; ++e) s += acc[i][j][e];
    out[(size_t)blockIdx.x * blockDim.x + threadIdx.x] = s;
}

// out[i] = the library's fp32 -> bf16 rounding of in[i]
__global__ void calib_round_kernel(const float* __restrict__ in, uint16_t* __restrict__ out, size_t n)
{
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += stride) out[i] = f32_to_bf16(in[i]);
}

}  // namespace

extern "C" int moe_calib_copy(const void* src, void* dst, size_t bytes, void* stream)
{
    if (!src || !dst) return MOE_ERR_NULL;
    if (bytes == 0 || bytes % 16 != 0 || ((reinterpret_cast<uintptr_t>(src) | reinterpret_cast<uintptr_t>(dst)) & 15)) return MOE_ERR_SHAPE;
    int dev = current_device(), cus = 0;
    if (dev < 0 || hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cus < 1) cus = 256;
    hipLaunchKernelGGL(calib_copy_kernel, dim3(cus * 8), dim3(256), 0, (hipStream_t)stream, (const uint4*)src, (uint4*)dst, bytes / 16);
    return moe_hip_status(hipGetLastError());
}

extern "C" int moe_calib_mfma(float* out, size_t out_floats, int iters, int* blocks, int* threads, void* stream)
{
    if (!out || !blocks || !threads) return MOE_ERR_NULL;
    if (iters < 1) return MOE_ERR_SHAPE;
    int dev = current_device(), cus = 0;
    if (dev < 0 || hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cus < 1) cus = 256;
    *blocks = cus;                       // one block of 8 waves per CU: two waves per SIMD, as the grouped kernel runs
    *threads = 512;
    if (out_floats < (size_t)cus * 512) return MOE_ERR_SHAPE;      // every thread writes one float
    hipLaunchKernelGGL(calib_mfma_kernel, dim3(cus), dim3(512), 0, (hipStream_t)stream, out, iters);
    return moe_hip_status(hipGetLastError());
}

extern "C" int moe_calib_round_bf16(const float* in, uint16_t* out, size_t n, void* stream)
{
    if (!in || !out) return MOE_ERR_NULL;
    if (n == 0) return MOE_OK;
    const size_t blocks = (n + 255) / 256;
    hipLaunchKernelGGL(calib_round_kernel, dim3((unsigned)(blocks < 4096 ? blocks : 4096)), dim3(256), 0, (hipStream_t)stream, in, out, n);
    return moe_hip_status(hipGetLastError());
}

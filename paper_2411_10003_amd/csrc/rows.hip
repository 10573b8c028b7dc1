// Row movers bound by HBM bandwidth: the send buffer of the first all-to-all (dispatch), the
// weighted return after the second one (combine), and their gradients (Fig. 2 of the paper and
// the two backward all-to-alls of its performance model, Section 4.2).
//
// One wavefront owns one token.  A token's row is read once and written to its k send rows
// (scatter form of Xp[r] = X[perm[r]/k]), so traffic is the algorithmic minimum
// (1 + k) * T * d elements.  Lanes move 16 bytes per access.
#include "internal.h"

namespace {

constexpr int ROW_WAVES = 4;   // tokens per block
constexpr int MAXK = 8;

template <typename ET> struct Vec;                      // 16-byte vector of elements
template <> struct Vec<float> {
    static constexpr int N = 4;
    static __device__ __forceinline__ void unpack(const uint4& v, float* f) {
        f[0] = __uint_as_float(v.x); f[1] = __uint_as_float(v.y); f[2] = __uint_as_float(v.z); f[3] = __uint_as_float(v.w);
    }
    static __device__ __forceinline__ uint4 pack(const float* f) {
        return make_uint4(__float_as_uint(f[0]), __float_as_uint(f[1]), __float_as_uint(f[2]), __float_as_uint(f[3]));
    }
};
template <> struct Vec<bf16_t> {
    static constexpr int N = 8;
    static __device__ __forceinline__ void unpack(const uint4& v, float* f) {
        f[0] = __uint_as_float(v.x << 16); f[1] = __uint_as_float(v.x & 0xffff0000u);
        f[2] = __uint_as_float(v.y << 16); f[3] = __uint_as_float(v.y & 0xffff0000u);
        f[4] = __uint_as_float(v.z << 16); f[5] = __uint_as_float(v.z & 0xffff0000u);
        f[6] = __uint_as_float(v.w << 16); f[7] = __uint_as_float(v.w & 0xffff0000u);
    }
    static __device__ __forceinline__ uint4 pack(const float* f) {
        return make_uint4(pack_bf16x2(f[0], f[1]), pack_bf16x2(f[2], f[3]), pack_bf16x2(f[4], f[5]), pack_bf16x2(f[6], f[7]));
    }
};

__device__ __forceinline__ float wave_sum(float v) {
    for (int off = 32; off >= 1; off >>= 1) v += __shfl_xor(v, off, 64);
    return v;
}

// Xp[pos[t*k+j], :] = X[t, :]
template <typename ET>
__global__ __launch_bounds__(ROW_WAVES * 64) void scatter_rows_kernel(
    const ET* __restrict__ X, const int32_t* __restrict__ pos, ET* __restrict__ Xp, int T, int d, int k)
{
    constexpr int VN = Vec<ET>::N;
    const int lane = threadIdx.x & 63;
    const int t = blockIdx.x * ROW_WAVES + (threadIdx.x >> 6);
    if (t >= T) return;
    const uint4* src = reinterpret_cast<const uint4*>(X + (size_t)t * d);
    const int nv = d / VN;
    for (int j = 0; j < k; ++j) {
        // the row is re-read from cache for j > 0; HBM sees it once
        uint4* dst = reinterpret_cast<uint4*>(Xp + (size_t)pos[(size_t)t * k + j] * d);
#pragma unroll 4
        for (int v = lane; v < nv; v += 64) dst[v] = src[v];
    }
}

// K-specialised variant: every 16-byte piece is loaded once and stored K times.
template <typename ET, int K>
__global__ __launch_bounds__(ROW_WAVES * 64) void scatter_rows_k_kernel(
    const ET* __restrict__ X, const int32_t* __restrict__ pos, ET* __restrict__ Xp, int T, int d)
{
    constexpr int VN = Vec<ET>::N;
    const int lane = threadIdx.x & 63;
    const int t = blockIdx.x * ROW_WAVES + (threadIdx.x >> 6);
    if (t >= T) return;
    const uint4* src = reinterpret_cast<const uint4*>(X + (size_t)t * d);
    uint4* dst[K];
#pragma unroll
    for (int j = 0; j < K; ++j) dst[j] = reinterpret_cast<uint4*>(Xp + (size_t)pos[(size_t)t * K + j] * d);
    const int nv = d / VN;
#pragma unroll 4
    for (int v = lane; v < nv; v += 64) {
        const uint4 x = src[v];
#pragma unroll
        for (int j = 0; j < K; ++j) dst[j][v] = x;
    }
}

// out[t,:] = sum_j w[t,j] * Yp[pos[t*k+j],:]   (fp32, ascending j, one rounding)
template <typename ET, int KT>
__global__ __launch_bounds__(ROW_WAVES * 64) void combine_kernel(
    const ET* __restrict__ Yp, const int32_t* __restrict__ pos, const float* __restrict__ w,
    ET* __restrict__ out, int T, int d, int k_rt)
{
    constexpr int VN = Vec<ET>::N;
    constexpr int KMAX = KT ? KT : MAXK;
    const int k = KT ? KT : k_rt;
    const int lane = threadIdx.x & 63;
    const int t = blockIdx.x * ROW_WAVES + (threadIdx.x >> 6);
    if (t >= T) return;
    const uint4* src[KMAX];
    float wj[KMAX];
#pragma unroll
    for (int j = 0; j < KMAX; ++j) {
        if (j < k) {
            src[j] = reinterpret_cast<const uint4*>(Yp + (size_t)pos[(size_t)t * k + j] * d);
            wj[j] = w[(size_t)t * k + j];
        }
    }
    uint4* dst = reinterpret_cast<uint4*>(out + (size_t)t * d);
    const int nv = d / VN;
    constexpr int U = (KT == 1 || KT == 2) ? 4 : 1;      // 16-byte pieces per lane requested before any is used
    for (int v0 = lane; v0 < nv; v0 += 64 * U) {
        uint4 raw[U][KMAX];
#pragma unroll
        for (int u = 0; u < U; ++u)
#pragma unroll
            for (int j = 0; j < KMAX; ++j)
                if (j < k && v0 + 64 * u < nv) raw[u][j] = src[j][v0 + 64 * u];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            if (v0 + 64 * u >= nv) break;
            float acc[VN];
#pragma unroll
            for (int i = 0; i < VN; ++i) acc[i] = 0.0f;
#pragma unroll
            for (int j = 0; j < KMAX; ++j) {
                if (j < k) {
                    float y[VN];
                    Vec<ET>::unpack(raw[u][j], y);
#pragma unroll
                    for (int i = 0; i < VN; ++i) acc[i] = fmaf(wj[j], y[i], acc[i]);
                }
            }
            dst[v0 + 64 * u] = Vec<ET>::pack(acc);
        }
    }
}

// dYp[pos[a],:] = w[a] * dOut[t,:] ;  dw[t,j] = <dOut[t,:], Yp[pos[a],:]>
template <typename ET, int KT>
__global__ __launch_bounds__(ROW_WAVES * 64) void combine_bwd_kernel(
    const ET* __restrict__ dOut, const ET* __restrict__ Yp, const int32_t* __restrict__ pos,
    const float* __restrict__ w, ET* __restrict__ dYp, float* __restrict__ dw, int T, int d, int k_rt)
{
    constexpr int VN = Vec<ET>::N;
    constexpr int KMAX = KT ? KT : MAXK;
    const int k = KT ? KT : k_rt;
    const int lane = threadIdx.x & 63;
    const int t = blockIdx.x * ROW_WAVES + (threadIdx.x >> 6);
    if (t >= T) return;
    const uint4* ysrc[KMAX];
    uint4* gdst[KMAX];
    float wj[KMAX], dot[KMAX];
#pragma unroll
    for (int j = 0; j < KMAX; ++j) {
        dot[j] = 0.0f;
        if (j < k) {
            const size_t row = (size_t)pos[(size_t)t * k + j];
            ysrc[j] = reinterpret_cast<const uint4*>(Yp + row * d);
            gdst[j] = reinterpret_cast<uint4*>(dYp + row * d);
            wj[j] = w[(size_t)t * k + j];
        }
    }
    const uint4* gsrc = reinterpret_cast<const uint4*>(dOut + (size_t)t * d);
    const int nv = d / VN;
    constexpr int U = (KT == 1 || KT == 2) ? 2 : 1;
    for (int v0 = lane; v0 < nv; v0 += 64 * U) {
        uint4 graw[U], yraw[U][KMAX];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            if (v0 + 64 * u < nv) {
                graw[u] = gsrc[v0 + 64 * u];
#pragma unroll
                for (int j = 0; j < KMAX; ++j)
                    if (j < k) yraw[u][j] = ysrc[j][v0 + 64 * u];
            }
        }
#pragma unroll
        for (int u = 0; u < U; ++u) {
            if (v0 + 64 * u >= nv) break;
            float g[VN];
            Vec<ET>::unpack(graw[u], g);
#pragma unroll
            for (int j = 0; j < KMAX; ++j) {
                if (j < k) {
                    float y[VN], o[VN];
                    Vec<ET>::unpack(yraw[u][j], y);
#pragma unroll
                    for (int i = 0; i < VN; ++i) { dot[j] = fmaf(g[i], y[i], dot[j]); o[i] = wj[j] * g[i]; }
                    gdst[j][v0 + 64 * u] = Vec<ET>::pack(o);
                }
            }
        }
    }
#pragma unroll
    for (int j = 0; j < KMAX; ++j) {
        if (j < k) {
            const float s = wave_sum(dot[j]);
            if (lane == 0) dw[(size_t)t * k + j] = s;
        }
    }
}

// dX[t,:] = sum_j dXp[pos[t*k+j],:]
template <typename ET, int KT>
__global__ __launch_bounds__(ROW_WAVES * 64) void dispatch_bwd_kernel(
    const ET* __restrict__ dXp, const int32_t* __restrict__ pos, ET* __restrict__ dX, int T, int d, int k_rt)
{
    constexpr int VN = Vec<ET>::N;
    constexpr int KMAX = KT ? KT : MAXK;
    const int k = KT ? KT : k_rt;
    const int lane = threadIdx.x & 63;
    const int t = blockIdx.x * ROW_WAVES + (threadIdx.x >> 6);
    if (t >= T) return;
    const uint4* src[KMAX];
#pragma unroll
    for (int j = 0; j < KMAX; ++j)
        if (j < k) src[j] = reinterpret_cast<const uint4*>(dXp + (size_t)pos[(size_t)t * k + j] * d);
    uint4* dst = reinterpret_cast<uint4*>(dX + (size_t)t * d);
    const int nv = d / VN;
    constexpr int U = (KT == 1 || KT == 2) ? 4 : 1;
    for (int v0 = lane; v0 < nv; v0 += 64 * U) {
        uint4 raw[U][KMAX];
#pragma unroll
        for (int u = 0; u < U; ++u)
#pragma unroll
            for (int j = 0; j < KMAX; ++j)
                if (j < k && v0 + 64 * u < nv) raw[u][j] = src[j][v0 + 64 * u];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            if (v0 + 64 * u >= nv) break;
            float acc[VN];
#pragma unroll
            for (int i = 0; i < VN; ++i) acc[i] = 0.0f;
#pragma unroll
            for (int j = 0; j < KMAX; ++j) {
                if (j < k) {
                    float y[VN];
                    Vec<ET>::unpack(raw[u][j], y);
#pragma unroll
                    for (int i = 0; i < VN; ++i) acc[i] += y[i];
                }
            }
            dst[v0 + 64 * u] = Vec<ET>::pack(acc);
        }
    }
}

inline dim3 row_grid(int T) { return dim3((T + ROW_WAVES - 1) / ROW_WAVES); }

}  // namespace

hipError_t launch_scatter_rows(const moe_shape_t& s, const void* X, const int32_t* pos, void* Xp, hipStream_t st)
{
    if (s.T == 0) return hipSuccess;
    const dim3 g = row_grid(s.T), b(ROW_WAVES * 64);
    if (s.dtype == MOE_F32) {
        hipLaunchKernelGGL(scatter_rows_kernel<float>, g, b, 0, st, (const float*)X, pos, (float*)Xp, s.T, s.d, s.k);
    } else if (s.k == 1) {
        hipLaunchKernelGGL((scatter_rows_k_kernel<bf16_t, 1>), g, b, 0, st, (const bf16_t*)X, pos, (bf16_t*)Xp, s.T, s.d);
    } else if (s.k == 2) {
        hipLaunchKernelGGL((scatter_rows_k_kernel<bf16_t, 2>), g, b, 0, st, (const bf16_t*)X, pos, (bf16_t*)Xp, s.T, s.d);
    } else {
        hipLaunchKernelGGL(scatter_rows_kernel<bf16_t>, g, b, 0, st, (const bf16_t*)X, pos, (bf16_t*)Xp, s.T, s.d, s.k);
    }
    return hipGetLastError();
}

hipError_t launch_combine(const moe_shape_t& s, const void* Yp, const int32_t* pos, const float* w, void* out, hipStream_t st)
{
    if (s.T == 0) return hipSuccess;
    const dim3 g = row_grid(s.T), b(ROW_WAVES * 64);
    if (s.dtype == MOE_F32)
        hipLaunchKernelGGL((combine_kernel<float, 0>), g, b, 0, st, (const float*)Yp, pos, w, (float*)out, s.T, s.d, s.k);
    else if (s.k == 1)
        hipLaunchKernelGGL((combine_kernel<bf16_t, 1>), g, b, 0, st, (const bf16_t*)Yp, pos, w, (bf16_t*)out, s.T, s.d, s.k);
    else if (s.k == 2)
        hipLaunchKernelGGL((combine_kernel<bf16_t, 2>), g, b, 0, st, (const bf16_t*)Yp, pos, w, (bf16_t*)out, s.T, s.d, s.k);
    else
        hipLaunchKernelGGL((combine_kernel<bf16_t, 0>), g, b, 0, st, (const bf16_t*)Yp, pos, w, (bf16_t*)out, s.T, s.d, s.k);
    return hipGetLastError();
}

hipError_t launch_combine_bwd(const moe_shape_t& s, const void* dOut, const void* Yp, const int32_t* pos,
                              const float* w, void* dYp, float* dw, hipStream_t st)
{
    if (s.T == 0) return hipSuccess;
    const dim3 g = row_grid(s.T), b(ROW_WAVES * 64);
    if (s.dtype == MOE_F32)
        hipLaunchKernelGGL((combine_bwd_kernel<float, 0>), g, b, 0, st, (const float*)dOut, (const float*)Yp, pos, w,
                           (float*)dYp, dw, s.T, s.d, s.k);
    else if (s.k == 1)
        hipLaunchKernelGGL((combine_bwd_kernel<bf16_t, 1>), g, b, 0, st, (const bf16_t*)dOut, (const bf16_t*)Yp, pos, w,
                           (bf16_t*)dYp, dw, s.T, s.d, s.k);
    else if (s.k == 2)
        hipLaunchKernelGGL((combine_bwd_kernel<bf16_t, 2>), g, b, 0, st, (const bf16_t*)dOut, (const bf16_t*)Yp, pos, w,
                           (bf16_t*)dYp, dw, s.T, s.d, s.k);
    else
        hipLaunchKernelGGL((combine_bwd_kernel<bf16_t, 0>), g, b, 0, st, (const bf16_t*)dOut, (const bf16_t*)Yp, pos, w,
                           (bf16_t*)dYp, dw, s.T, s.d, s.k);
    return hipGetLastError();
}

hipError_t launch_dispatch_bwd(const moe_shape_t& s, const void* dXp, const int32_t* pos, void* dX, hipStream_t st)
{
    if (s.T == 0) return hipSuccess;
    const dim3 g = row_grid(s.T), b(ROW_WAVES * 64);
    if (s.dtype == MOE_F32)
        hipLaunchKernelGGL((dispatch_bwd_kernel<float, 0>), g, b, 0, st, (const float*)dXp, pos, (float*)dX, s.T, s.d, s.k);
    else if (s.k == 1)
        hipLaunchKernelGGL((dispatch_bwd_kernel<bf16_t, 1>), g, b, 0, st, (const bf16_t*)dXp, pos, (bf16_t*)dX, s.T, s.d, s.k);
    else if (s.k == 2)
        hipLaunchKernelGGL((dispatch_bwd_kernel<bf16_t, 2>), g, b, 0, st, (const bf16_t*)dXp, pos, (bf16_t*)dX, s.T, s.d, s.k);
    else
        hipLaunchKernelGGL((dispatch_bwd_kernel<bf16_t, 0>), g, b, 0, st, (const bf16_t*)dXp, pos, (bf16_t*)dX, s.T, s.d, s.k);
    return hipGetLastError();
}

// ---- Trans on one GPU (Section 4.1: the parameters of a selected expert are transferred to the devices
// that will compute its inputs).  With every expert's parameters in one pool in this GPU's memory, the
// transfer is a gather of the hosted experts into the group slots the grouped FFN reads, driven by the
// plan as it lies in device memory: group g is the g-th expert e (ascending) with expert_dest[e] == self.
// A slot that already holds the right expert in its current version is left alone (placements change little
// from one iteration to the next, Section 3), which slot_expert[G] and slot_version[G] keep track of: an
// expert's parameters are updated before every transfer (Section 5.1), so the pool carries a version per
// expert that the caller bumps with every update, and a replica of an older version is copied again.
namespace {

__device__ __forceinline__ int hosted_expert_of_group(const int32_t* __restrict__ expert_dest, int E, int self, int g)
{
    // wave-uniform scan; E <= 1024
    int seen = 0;
    for (int e = 0; e < E; ++e) {
        if (expert_dest[e] == self) {
            if (seen == g) return e;
            ++seen;
        }
    }
    return -1;
}

__global__ __launch_bounds__(256) void trans_gather_kernel(
    const int32_t* __restrict__ expert_dest, const int32_t* __restrict__ pool_version,
    const int32_t* __restrict__ slot_expert, const int32_t* __restrict__ slot_version,
    const uint4* __restrict__ pool, uint4* __restrict__ groups, long vec_per_expert, int E, int self)
{
    const int g = blockIdx.y;
    const int e = hosted_expert_of_group(expert_dest, E, self, g);
    if (e < 0) return;                                     // unused slot
    // the expert is already there, in the version the pool holds now (no versions given: always copied)
    if (pool_version != nullptr && e == slot_expert[g] && slot_version[g] == pool_version[e]) return;
    const uint4* src = pool + (long)e * vec_per_expert;
    uint4* dst = groups + (long)g * vec_per_expert;
    const long stride = (long)gridDim.x * blockDim.x * 4;
    for (long v = ((long)blockIdx.x * blockDim.x + threadIdx.x); v < vec_per_expert; v += stride) {
        uint4 r[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const long i = v + (long)u * gridDim.x * blockDim.x;
            if (i < vec_per_expert) r[u] = src[i];
        }
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const long i = v + (long)u * gridDim.x * blockDim.x;
            if (i < vec_per_expert) dst[i] = r[u];
        }
    }
}

__global__ void trans_commit_kernel(const int32_t* __restrict__ expert_dest, const int32_t* __restrict__ pool_version,
                                    int32_t* __restrict__ slot_expert, int32_t* __restrict__ slot_version, int E, int self, int G)
{
    const int g = blockIdx.x * blockDim.x + threadIdx.x;
    if (g >= G) return;
    const int e = hosted_expert_of_group(expert_dest, E, self, g);
    if (e >= 0) {                                          // an unused slot keeps what it holds
        slot_expert[g] = e;
        if (pool_version != nullptr) slot_version[g] = pool_version[e];
    }
}

// Agg on one GPU (Section 4.1: the gradients a replica computed are added to the expert's gradient where its
// parameters live).  The inverse walk of the gather above: the fp32 gradient of hosted group g is added to the
// pool entry of the expert the plan puts there.  Every element is touched by one thread: same bits every run.
__global__ __launch_bounds__(256) void agg_add_kernel(
    const int32_t* __restrict__ expert_dest, const float4* __restrict__ groups, float4* __restrict__ pool,
    long vec_per_expert, int E, int self)
{
    const int g = blockIdx.y;
    const int e = hosted_expert_of_group(expert_dest, E, self, g);
    if (e < 0) return;
    const float4* src = groups + (long)g * vec_per_expert;
    float4* dst = pool + (long)e * vec_per_expert;
    const long stride = (long)gridDim.x * blockDim.x;
    for (long v = (long)blockIdx.x * blockDim.x + threadIdx.x; v < vec_per_expert; v += stride) {
        const float4 a = src[v];
        float4 b = dst[v];
        b.x += a.x; b.y += a.y; b.z += a.z; b.w += a.w;
        dst[v] = b;
    }
}

}  // namespace

hipError_t launch_agg_add(const moe_shape_t& s, const int32_t* expert_dest, const float* groups, float* pool,
                          long floats_per_expert, hipStream_t st)
{
    const long vec = floats_per_expert / 4;
    long bx = (vec + 256 * 4 - 1) / (256 * 4);
    bx = bx < 1 ? 1 : (bx > 1024 ? 1024 : bx);
    hipLaunchKernelGGL(agg_add_kernel, dim3((unsigned)bx, s.G), dim3(256), 0, st, expert_dest,
                       (const float4*)groups, (float4*)pool, vec, s.E, s.self);
    return hipGetLastError();
}

hipError_t launch_trans_gather(const moe_shape_t& s, const int32_t* expert_dest, const int32_t* pool_version,
                               const int32_t* slot_expert, const int32_t* slot_version,
                               const void* pool, void* groups, long bytes_per_expert, hipStream_t st)
{
    const long vec = bytes_per_expert / 16;
    const int bx = (int)((vec + 256 * 4 - 1) / (256 * 4) < 512 ? (vec + 256 * 4 - 1) / (256 * 4) : 512);
    hipLaunchKernelGGL(trans_gather_kernel, dim3(bx > 0 ? bx : 1, s.G), dim3(256), 0, st, expert_dest, pool_version, slot_expert, slot_version,
                       (const uint4*)pool, (uint4*)groups, vec, s.E, s.self);
    return hipGetLastError();
}

hipError_t launch_trans_commit(const moe_shape_t& s, const int32_t* expert_dest, const int32_t* pool_version,
                               int32_t* slot_expert, int32_t* slot_version, hipStream_t st)
{
    hipLaunchKernelGGL(trans_commit_kernel, dim3((s.G + 63) / 64), dim3(64), 0, st, expert_dest, pool_version, slot_expert,
                       slot_version, s.E, s.self, s.G);
    return hipGetLastError();
}

// Backward of the gate's linear map logit[t,e] = b[e] + sum_c X[t,c] Wg[c,e] (the gate network of
// Section 2.1 of the paper) and the complete gradient of the layer input:
//   dWg[c,e] = sum_t X[t,c] dlogits[t,e]      dbg[e] = sum_t dlogits[t,e]
//   dX[t,c]  = sum_j dXp[pos[t*k+j],c]  +  sum_e dlogits[t,e] Wg[c,e]
// The first sum of dX is the backward of the send (the fourth all-to-all of the performance model,
// Section 4.2); fusing the gate path into it saves a pass over dX.  Both kernels are bound by HBM
// (they stream X or dXp once) with E fp32 FMAs per element beside it; fp32 throughout, E <= 64.
#include "internal.h"

#include <type_traits>

namespace {

constexpr int MAXK_IG = 8;      // the handle allows k <= 8

__device__ __forceinline__ void unpack_bf16x8(const uint4& v, float* f)
{
    f[0] = __uint_as_float(v.x << 16); f[1] = __uint_as_float(v.x & 0xffff0000u);
    f[2] = __uint_as_float(v.y << 16); f[3] = __uint_as_float(v.y & 0xffff0000u);
    f[4] = __uint_as_float(v.z << 16); f[5] = __uint_as_float(v.z & 0xffff0000u);
    f[6] = __uint_as_float(v.w << 16); f[7] = __uint_as_float(v.w & 0xffff0000u);
}

// ---- dX = backward of the send + dlogits Wg^T ---------------------------------------------------
// A block owns a strip of 64*VN columns and TOK_PER_BLOCK tokens.  The strip of Wg is staged once per
// block in LDS, transposed to [e][column] so that a lane reads the VN weights of its columns with
// 16-byte LDS loads; the E logit gradients of a token are the same for every lane (scalar loads).
template <typename ET, int VN, int EC>
__global__ __launch_bounds__(256) void input_grad_kernel(
    const ET* __restrict__ dXp, const int32_t* __restrict__ pos, const float* __restrict__ dlogits,
    const float* __restrict__ Wg, ET* __restrict__ dX, int T, int d, int E, int k, int tok_per_block)
{
    extern __shared__ __attribute__((aligned(16))) float wt[];      // [E][64*VN + 4]
    constexpr int CW = 64 * VN, WP = CW + 4;                       // strip width, padded row of wt
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6), n_waves = blockDim.x >> 6;
    const int c0 = blockIdx.x * CW;                                // first column of the strip
    // Wg[c0 + c][e] -> wt[e][c], read in memory order; the rows of wt are 4 floats longer than the strip so
    // that the 16..64 experts of a column and the columns next to it fall into different banks
#pragma unroll 4
    for (int i = tid; i < CW * E; i += blockDim.x) {
        const int c = i / E, e = i - c * E;
        wt[e * WP + c] = (c0 + c < d) ? Wg[(size_t)(c0 + c) * E + e] : 0.0f;
    }
    __syncthreads();
    const int col = c0 + lane * VN;
    const int t_begin = blockIdx.y * tok_per_block, t_end = min(T, t_begin + tok_per_block);
    // several tokens per trip, all of their loads issued before the first use.  The U x E logit gradients
    // of a trip are fetched by the lanes as one flat array and handed out with readlane, so a token costs
    // no dependent memory round trip of its own.
    constexpr int U = EC <= 16 ? 4 : 2;
    constexpr int NDL = (U * EC + 63) / 64;
    for (int t0 = t_begin + wave; t0 < t_end; t0 += n_waves * U) {
        float acc[U][VN];
        uint4 raw[U][MAXK_IG];
        float dlv[NDL];
#pragma unroll
        for (int q = 0; q < NDL; ++q) {
            const int f = q * 64 + lane, u = f / EC, e = f % EC;
            const int t = t0 + n_waves * u;
            dlv[q] = (u < U && t < t_end && e < E) ? dlogits[(size_t)t * E + e] : 0.0f;
        }
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int t = t0 + n_waves * u;
#pragma unroll
            for (int j = 0; j < MAXK_IG; ++j)
                if (j < k && t < t_end && col < d)       // pos comes through the scalar cache (16 tokens per line)
                    raw[u][j] = *reinterpret_cast<const uint4*>(dXp + (size_t)pos[(size_t)t * k + j] * d + col);
        }
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int t = t0 + n_waves * u;
            if (t >= t_end || col >= d) continue;
#pragma unroll
            for (int i = 0; i < VN; ++i) acc[u][i] = 0.0f;
#pragma unroll
            for (int j = 0; j < MAXK_IG; ++j) {                    // expert path, ascending j
                if (j < k) {
                    float f[VN];
                    if (VN == 8) unpack_bf16x8(raw[u][j], f);
                    else { f[0] = __uint_as_float(raw[u][j].x); f[1] = __uint_as_float(raw[u][j].y); f[2 % VN] = __uint_as_float(raw[u][j].z); f[3 % VN] = __uint_as_float(raw[u][j].w); }
#pragma unroll
                    for (int i = 0; i < VN; ++i) acc[u][i] += f[i];
                }
            }
#pragma unroll
            for (int e = 0; e < EC; ++e) {
                const int f = u * EC + e;                          // position in the flat [U][EC] array
                const float g = __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, dlv[f / 64]), f % 64));
                if (g == 0.0f) continue;                           // renormalised top-k: only k of the E are non-zero
                const float* wrow = wt + e * WP + lane * VN;
#pragma unroll
                for (int i = 0; i < VN; i += 4) {
                    const float4 wv = *reinterpret_cast<const float4*>(wrow + i);
                    acc[u][i + 0] = fmaf(g, wv.x, acc[u][i + 0]); acc[u][i + 1] = fmaf(g, wv.y, acc[u][i + 1]);
                    acc[u][i + 2] = fmaf(g, wv.z, acc[u][i + 2]); acc[u][i + 3] = fmaf(g, wv.w, acc[u][i + 3]);
                }
            }
            if (VN == 8) {
                *reinterpret_cast<uint4*>(dX + (size_t)t * d + col) =
                    make_uint4(pack_bf16x2(acc[u][0], acc[u][1]), pack_bf16x2(acc[u][2], acc[u][3]),
                               pack_bf16x2(acc[u][4 % VN], acc[u][5 % VN]), pack_bf16x2(acc[u][6 % VN], acc[u][7 % VN]));
            } else {
                *reinterpret_cast<float4*>(dX + (size_t)t * d + col) = make_float4(acc[u][0], acc[u][1], acc[u][2], acc[u][3]);
            }
        }
    }
}

// ---- dWg, dbg -------------------------------------------------------------------------------------
// A lane owns CPT columns and keeps CPT x EC partial sums (128 registers); a wave walks its share of
// the tokens of its partition, the four waves of a block fold their sums through LDS, and the block
// writes one partial [strip][E] per token partition.  A second kernel adds the partitions in a fixed
// order, so the result does not depend on the schedule.
template <typename ET, int EC, int CPT>
__global__ __launch_bounds__(256, 2) void gate_wgrad_partial_kernel(
    const ET* __restrict__ X, const float* __restrict__ dlogits, float* __restrict__ partial,
    float* __restrict__ partial_b, int T, int d, int E, int tok_per_part)
{
    constexpr int CW = 64 * CPT;
    static_assert(CPT * EC <= 128, "partial sums of a lane");
    __shared__ float fold[CW * EC];                                // 32 KB at most
    __shared__ float fold_b[EC];
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int col = blockIdx.x * CW + lane * CPT;
    const int part = blockIdx.y;
    const int t_begin = part * tok_per_part, t_end = min(T, t_begin + tok_per_part);
    float acc[CPT][EC];
#pragma unroll
    for (int i = 0; i < CPT; ++i)
#pragma unroll
        for (int e = 0; e < EC; ++e) acc[i][e] = 0.0f;
    float accb = 0.0f;                                             // lane e: sum of dlogits[:, e]
    // eight tokens per trip: their row pieces and their logit gradients are requested before the first use
    // (a wave has little else in flight: the partial sums take half of its registers).  The U x E logit
    // gradients of a trip are fetched by the lanes as one flat array (a token's row is one 32..256-byte
    // piece of dlogits) and handed out with readlane, so a token costs no dependent memory round trip.
    constexpr int U = 8;
    constexpr int NDL = U * EC / 64;                               // flat loads of logit gradients per trip
    static_assert(U * EC % 64 == 0 && 64 % EC == 0, "flat layout of the logit gradients");
    // CPT columns of a row as one load: 16/8/4 bytes of bf16, 16/8 bytes of fp32
    typedef typename std::conditional<sizeof(ET) * CPT == 16, uint4,
            typename std::conditional<sizeof(ET) * CPT == 8, uint2, uint32_t>::type>::type raw_t;
    static_assert(sizeof(ET) * CPT == sizeof(raw_t), "row piece");
    for (int t0 = t_begin + wave; t0 < t_end; t0 += 4 * U) {
        raw_t raw[U];
        float dlv[NDL];
#pragma unroll
        for (int q = 0; q < NDL; ++q) {
            const int f = q * 64 + lane, u = f / EC, e = f % EC;
            const int t = t0 + 4 * u;
            dlv[q] = (t < t_end && e < E) ? dlogits[(size_t)t * E + e] : 0.0f;
        }
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int t = t0 + 4 * u;
            if (t < t_end && col < d) raw[u] = *reinterpret_cast<const raw_t*>(X + (size_t)t * d + col);
        }
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int t = t0 + 4 * u;
            if (t >= t_end) break;
            float x[CPT];
#pragma unroll
            for (int i = 0; i < CPT; ++i) x[i] = 0.0f;
            if (col < d) {
                if constexpr (sizeof(ET) == 2 && CPT == 8) {
                    unpack_bf16x8(raw[u], x);
                } else if constexpr (sizeof(ET) == 2 && CPT == 4) {
                    x[0] = __uint_as_float(raw[u].x << 16); x[1] = __uint_as_float(raw[u].x & 0xffff0000u);
                    x[2] = __uint_as_float(raw[u].y << 16); x[3] = __uint_as_float(raw[u].y & 0xffff0000u);
                } else if constexpr (sizeof(ET) == 2) {
                    x[0] = __uint_as_float(raw[u] << 16); x[1] = __uint_as_float(raw[u] & 0xffff0000u);
                } else if constexpr (CPT == 4) {
                    x[0] = __uint_as_float(raw[u].x); x[1] = __uint_as_float(raw[u].y);
                    x[2] = __uint_as_float(raw[u].z); x[3] = __uint_as_float(raw[u].w);
                } else {
                    x[0] = __uint_as_float(raw[u].x); x[1] = __uint_as_float(raw[u].y);
                }
            }
#pragma unroll
            for (int e = 0; e < EC; ++e) {
                const int f = u * EC + e;                          // position in the flat [U][EC] array
                const float g = __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, dlv[f / 64]), f % 64));
                if (g != 0.0f) {                                   // uniform; skips the experts a token did not select
#pragma unroll
                    for (int i = 0; i < CPT; ++i) acc[i][e] = fmaf(x[i], g, acc[i][e]);
                }
            }
        }
        if (blockIdx.x == 0) {
#pragma unroll
            for (int q = 0; q < NDL; ++q) accb += dlv[q];          // lane l always meets expert l % EC
        }
    }
    // lanes with the same l % EC hold pieces of the same bias gradient
    for (int off = EC; off < 64; off <<= 1) accb += __shfl_xor(accb, off, 64);
    // fold the four waves: waves 1, 2, 3 hand their sums to wave 0 one after the other
    for (int w = 1; w < 4; ++w) {
        if (wave == w) {
#pragma unroll
            for (int i = 0; i < CPT; ++i)
#pragma unroll
                for (int e = 0; e < EC; ++e) fold[(i * EC + e) * 64 + lane] = acc[i][e];
            if (lane < EC) fold_b[lane] = accb;
        }
        __syncthreads();
        if (wave == 0) {
#pragma unroll
            for (int i = 0; i < CPT; ++i)
#pragma unroll
                for (int e = 0; e < EC; ++e) acc[i][e] += fold[(i * EC + e) * 64 + lane];
            if (lane < EC) accb += fold_b[lane];
        }
        __syncthreads();
    }
    if (wave == 0) {
#pragma unroll
        for (int i = 0; i < CPT; ++i)
#pragma unroll
            for (int e = 0; e < EC; ++e)
                if (col + i < d && e < E) partial[((size_t)part * d + col + i) * E + e] = acc[i][e];
        if (blockIdx.x == 0 && lane < E) partial_b[(size_t)part * E + lane] = accb;
    }
}

__global__ void gate_wgrad_reduce_kernel(const float* __restrict__ partial, const float* __restrict__ partial_b,
                                         float* __restrict__ dWg, float* __restrict__ dbg, int n_part, int dE, int E)
{
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < dE) {
        float s = 0.0f;
        for (int p = 0; p < n_part; ++p) s += partial[(size_t)p * dE + i];
        dWg[i] = s;
    }
    if (i < E) {
        float s = 0.0f;
        for (int p = 0; p < n_part; ++p) s += partial_b[(size_t)p * E + i];
        dbg[i] = s;
    }
}

template <typename ET, int EC, int CPT>
hipError_t launch_wgrad_t(const moe_shape_t& s, const void* X, const float* dlogits, float* partial, float* partial_b,
                          int n_part, int tok_per_part, hipStream_t st)
{
    const dim3 grid((s.d + 64 * CPT - 1) / (64 * CPT), n_part);
    hipLaunchKernelGGL((gate_wgrad_partial_kernel<ET, EC, CPT>), grid, dim3(256), 0, st, (const ET*)X, dlogits, partial,
                       partial_b, s.T, s.d, s.E, tok_per_part);
    return hipGetLastError();
}

}  // namespace

int gate_grad_partitions(const moe_shape_t& s) { return s.T < 64 * 256 ? (s.T + 255) / 256 : 64; }

template <typename ET, int VN, int EC>
hipError_t launch_input_grad_t(const moe_shape_t& s, const void* dXp, const int32_t* pos, const float* dlogits,
                               const float* Wg, void* dX, hipStream_t st)
{
    constexpr int CW = 64 * VN, TOK = 128;
    const dim3 grid((s.d + CW - 1) / CW, (s.T + TOK - 1) / TOK);
    const size_t lds = (size_t)s.E * (CW + 4) * sizeof(float);
    auto kern = input_grad_kernel<ET, VN, EC>;
    static bool configured = false;      // per instantiation
    if (!configured) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, 64 * (CW + 4) * 4);
        if (e != hipSuccess) return e;
        configured = true;
    }
    hipLaunchKernelGGL(kern, grid, dim3(256), lds, st, (const ET*)dXp, pos, dlogits, Wg, (ET*)dX, s.T, s.d, s.E, s.k, TOK);
    return hipGetLastError();
}

hipError_t launch_input_grad(const moe_shape_t& s, const void* dXp, const int32_t* pos, const float* dlogits,
                             const float* Wg, void* dX, hipStream_t st)
{
    const bool bf = s.dtype == MOE_BF16;
    if (s.E <= 8)  return bf ? launch_input_grad_t<bf16_t, 8, 8>(s, dXp, pos, dlogits, Wg, dX, st) : launch_input_grad_t<float, 4, 8>(s, dXp, pos, dlogits, Wg, dX, st);
    if (s.E <= 16) return bf ? launch_input_grad_t<bf16_t, 8, 16>(s, dXp, pos, dlogits, Wg, dX, st) : launch_input_grad_t<float, 4, 16>(s, dXp, pos, dlogits, Wg, dX, st);
    if (s.E <= 32) return bf ? launch_input_grad_t<bf16_t, 8, 32>(s, dXp, pos, dlogits, Wg, dX, st) : launch_input_grad_t<float, 4, 32>(s, dXp, pos, dlogits, Wg, dX, st);
    return bf ? launch_input_grad_t<bf16_t, 8, 64>(s, dXp, pos, dlogits, Wg, dX, st) : launch_input_grad_t<float, 4, 64>(s, dXp, pos, dlogits, Wg, dX, st);
}

hipError_t launch_gate_wgrad(const moe_shape_t& s, const void* X, const float* dlogits, float* partial, float* partial_b,
                             float* dWg, float* dbg, hipStream_t st)
{
    const int n_part = gate_grad_partitions(s);
    const int tok_per_part = (s.T + n_part - 1) / n_part;
    hipError_t e;
    const bool bf = s.dtype == MOE_BF16;
    if (s.E <= 8)       e = bf ? launch_wgrad_t<bf16_t, 8, 8>(s, X, dlogits, partial, partial_b, n_part, tok_per_part, st)
                               : launch_wgrad_t<float, 8, 4>(s, X, dlogits, partial, partial_b, n_part, tok_per_part, st);
    else if (s.E <= 16) e = bf ? launch_wgrad_t<bf16_t, 16, 8>(s, X, dlogits, partial, partial_b, n_part, tok_per_part, st)
                               : launch_wgrad_t<float, 16, 4>(s, X, dlogits, partial, partial_b, n_part, tok_per_part, st);
    else if (s.E <= 32) e = bf ? launch_wgrad_t<bf16_t, 32, 4>(s, X, dlogits, partial, partial_b, n_part, tok_per_part, st)
                               : launch_wgrad_t<float, 32, 4>(s, X, dlogits, partial, partial_b, n_part, tok_per_part, st);
    else                e = bf ? launch_wgrad_t<bf16_t, 64, 2>(s, X, dlogits, partial, partial_b, n_part, tok_per_part, st)
                               : launch_wgrad_t<float, 64, 2>(s, X, dlogits, partial, partial_b, n_part, tok_per_part, st);
    if (e != hipSuccess) return e;
    const int dE = s.d * s.E;
    hipLaunchKernelGGL(gate_wgrad_reduce_kernel, dim3((dE + 255) / 256), dim3(256), 0, st, partial, partial_b, dWg, dbg, n_part, dE, s.E);
    return hipGetLastError();
}

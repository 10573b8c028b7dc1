// Backward of the gate's linear map logit[t,e] = b[e] + sum_c X[t,c] Wg[c,e] (the gate network of
// Section 2.1 of the paper) and the complete gradient of the layer input:
//   dWg[c,e] = sum_t X[t,c] dlogits[t,e]      dbg[e] = sum_t dlogits[t,e]
//   dX[t,c]  = sum_j dXp[pos[t*k+j],c]  +  sum_e dlogits[t,e] Wg[c,e]
// The first sum of dX is the backward of the send (the fourth all-to-all of the performance model,
// Section 4.2); fusing the gate path into it saves a pass over dX.  Both kernels are bound by HBM
// (they stream X or dXp once) with E fp32 multiply-adds per element beside it (on the fp32 MFMA for the
// parameter gradients, where they form a dense contraction over the tokens); fp32 throughout.  More than 64
// experts are taken in passes (parameter gradients) or chunks (input gradient) of 64.
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

// ---- the same on the matrix cores (E <= 32) ---------------------------------------------------------
// dlogits Wg^T is a dense product with the experts as its short contraction: on the fp32 16x16x4 MFMA, four
// instructions (E = 16) give a 16-token x 16-column tile.  Tile j of a strip holds the columns
// strip0 + n * VN + j (n = 0..15), so that lane l ends up with VN consecutive columns (n = l % 16) of the
// tokens 4 (l / 16) + r, r = 0..3: exactly one 16-byte piece per token, which is what the gather of the dXp
// rows and the store of dX move.  The B operands (a lane's VN columns of Wg against 4 experts per instruction)
// stay in registers for the whole block; the A operand is dlogits[token l % 16][expert 4 m + l / 16].
typedef __attribute__((ext_vector_type(4))) float ig_f32x4_t;

template <typename ET, int VN, int NE, int CS, int KMAX>
__global__ __launch_bounds__(256) void input_grad_mfma_kernel(
    const ET* __restrict__ dXp, const int32_t* __restrict__ pos, const float* __restrict__ dlogits,
    const float* __restrict__ Wg, ET* __restrict__ dX, int T, int d, int E, int k, int tok_per_block)
{
    constexpr int SW = 16 * VN, NM = NE * 4;                       // columns of a strip, MFMA steps over the experts
    typedef typename std::conditional<sizeof(ET) == 2, uint4, float4>::type raw_t;
    static_assert(sizeof(ET) * VN == 16, "a lane moves 16 bytes of a row");
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int ln = lane & 15, lq = lane >> 4;
    const int c0 = (blockIdx.x * 4 + wave) * (CS * SW);            // the four waves take neighbouring strips of the same tokens
    const int t_begin = blockIdx.y * tok_per_block, t_end = min(T, t_begin + tok_per_block);

    float wreg[CS][VN][NM];                                        // Wg[column of the lane][expert 4 m + lq]
#pragma unroll
    for (int s = 0; s < CS; ++s)
#pragma unroll
        for (int j = 0; j < VN; ++j)
#pragma unroll
            for (int m = 0; m < NM; ++m) {
                const int c = c0 + s * SW + ln * VN + j, e = 4 * m + lq;
                wreg[s][j][m] = (c < d && e < E) ? Wg[(size_t)c * E + e] : 0.0f;
            }

    for (int tg = t_begin; tg < t_end; tg += 16) {
        // everything that does not depend on another load first: logit gradients, positions
        float a[NM];
        const int ta = tg + ln;
#pragma unroll
        for (int m = 0; m < NM; ++m) {
            const int e = 4 * m + lq;
            a[m] = (ta < t_end && e < E) ? dlogits[(size_t)ta * E + e] : 0.0f;
        }
        int rows[4][KMAX];
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            const int t = tg + 4 * lq + r;
#pragma unroll
            for (int j = 0; j < KMAX; ++j) rows[r][j] = (j < k && t < t_end) ? pos[(size_t)t * k + j] : -1;
        }
        // all row pieces of the 4 tokens are requested before the first one is used
        raw_t raw[4][CS][KMAX];
#pragma unroll
        for (int r = 0; r < 4; ++r)
#pragma unroll
            for (int s = 0; s < CS; ++s) {
                const int c = c0 + s * SW + ln * VN;
#pragma unroll
                for (int j = 0; j < KMAX; ++j) {
                    if (j < k && rows[r][j] >= 0 && c < d) raw[r][s][j] = *reinterpret_cast<const raw_t*>(dXp + (size_t)rows[r][j] * d + c);
                    else raw[r][s][j] = raw_t{};
                }
            }
        ig_f32x4_t acc[CS][VN];
#pragma unroll
        for (int s = 0; s < CS; ++s)
#pragma unroll
            for (int j = 0; j < VN; ++j) {
                acc[s][j] = ig_f32x4_t{0.0f, 0.0f, 0.0f, 0.0f};
#pragma unroll
                for (int m = 0; m < NM; ++m) acc[s][j] = __builtin_amdgcn_mfma_f32_16x16x4f32(a[m], wreg[s][j][m], acc[s][j], 0, 0, 0);
            }
        // add the k rows of every token (j ascending, as the plain send backward adds them) and store
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            const int t = tg + 4 * lq + r;
#pragma unroll
            for (int s = 0; s < CS; ++s) {
                const int c = c0 + s * SW + ln * VN;
                if (t >= t_end || c >= d) continue;
                float sum[VN];
#pragma unroll
                for (int j = 0; j < VN; ++j) sum[j] = 0.0f;
#pragma unroll
                for (int j = 0; j < KMAX; ++j) {
                    if (j >= k) break;
                    float x[VN];
                    if constexpr (sizeof(ET) == 2) {
                        unpack_bf16x8(raw[r][s][j], x);
                    } else {
                        x[0] = raw[r][s][j].x; x[1] = raw[r][s][j].y; x[2] = raw[r][s][j].z; x[3] = raw[r][s][j].w;
                    }
#pragma unroll
                    for (int i = 0; i < VN; ++i) sum[i] += x[i];
                }
#pragma unroll
                for (int i = 0; i < VN; ++i) sum[i] += acc[s][i][r];
                if constexpr (sizeof(ET) == 2) {
                    *reinterpret_cast<uint4*>(dX + (size_t)t * d + c) =
                        make_uint4(pack_bf16x2(sum[0], sum[1]), pack_bf16x2(sum[2], sum[3]),
                                   pack_bf16x2(sum[4 % VN], sum[5 % VN]), pack_bf16x2(sum[6 % VN], sum[7 % VN]));
                } else {
                    *reinterpret_cast<float4*>(dX + (size_t)t * d + c) = make_float4(sum[0], sum[1], sum[2], sum[3]);
                }
            }
        }
    }
}

// ---- dWg, dbg ---------------------------------------------------------------------------------------
// dWg = X^T dlogits is a dense contraction over the tokens.  In fp32 on the 16x16x4 MFMA, one instruction
// multiplies 16 columns of X by 16 experts over 4 tokens.  Lane l supplies X[token l/16][its column l%16] as
// the A operand and dlogits[token l/16][expert l%16] as the B operand, so both come straight from coalesced
// loads with no exchange between lanes: a lane loads VN consecutive columns of one token (16 bytes) and the VN
// values go to VN instructions, each with its own 16 x 16 accumulator.
// Accumulator j of a strip holds columns strip0 + i * VN + j (i = 0..15) against the 16 experts of a tile:
// lane l, register r is column index i = 4 (l / 16) + r, expert l % 16.
// A block's four waves take every fourth group of 4 tokens of the partition; their sums are folded through
// LDS in a fixed order and written as one partial per token partition (the reduce kernel adds those).
typedef __attribute__((ext_vector_type(4))) float f32x4_t;

template <typename ET, int VN, int NE, int CS>
__global__ __launch_bounds__(256) void gate_wgrad_mfma_kernel(
    const ET* __restrict__ X, const float* __restrict__ dlogits, float* __restrict__ partial,
    float* __restrict__ partial_b, int T, int d, int E, int tok_per_part, int e0)
{
    // e0: first expert of this pass (more than 64 experts are taken in passes of 16 NE)
    constexpr int SW = 16 * VN;                                    // columns of one strip
    constexpr int NACC = CS * VN * NE;                             // 16 x 16 accumulators of a wave
    typedef typename std::conditional<sizeof(ET) == 2, uint4, float4>::type raw_t;
    static_assert(sizeof(ET) * VN == 16, "a lane loads 16 bytes of a row");
    __shared__ float fold[NACC * 4 * 64];
    __shared__ float fold_b[NE * 16];
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int li = lane & 15, lk = lane >> 4;                      // column / expert of the lane, token of the lane
    const int c0 = blockIdx.x * (CS * SW);
    const int part = blockIdx.y;
    const int t_begin = part * tok_per_part, t_end = min(T, t_begin + tok_per_part);

    f32x4_t acc[CS][VN][NE];
#pragma unroll
    for (int s = 0; s < CS; ++s)
#pragma unroll
        for (int j = 0; j < VN; ++j)
#pragma unroll
            for (int n = 0; n < NE; ++n) acc[s][j][n] = f32x4_t{0.0f, 0.0f, 0.0f, 0.0f};
    float accb[NE];
#pragma unroll
    for (int n = 0; n < NE; ++n) accb[n] = 0.0f;

    constexpr int U = 4;                                           // groups of 4 tokens requested together: one trip
    auto load_trip = [&](int tg, raw_t (&raw)[U][CS], float (&dl)[U][NE]) {
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int t = tg + 16 * u + lk;
            const bool tv = t < t_end;
#pragma unroll
            for (int n = 0; n < NE; ++n) {
                const int e = e0 + n * 16 + li;
                dl[u][n] = (tv && e < E) ? dlogits[(size_t)t * E + e] : 0.0f;
            }
#pragma unroll
            for (int s = 0; s < CS; ++s) {
                const int c = c0 + s * SW + li * VN;
                if (tv && c < d) raw[u][s] = *reinterpret_cast<const raw_t*>(X + (size_t)t * d + c);
                else raw[u][s] = raw_t{};
            }
        }
    };
    auto use_trip = [&](const raw_t (&raw)[U][CS], const float (&dl)[U][NE]) {      // rows past the end were loaded as zeros
#pragma unroll
        for (int u = 0; u < U; ++u) {
#pragma unroll
            for (int s = 0; s < CS; ++s) {
                float x[VN];
                if constexpr (sizeof(ET) == 2) {
                    unpack_bf16x8(raw[u][s], x);
                } else {
                    x[0] = raw[u][s].x; x[1] = raw[u][s].y; x[2] = raw[u][s].z; x[3] = raw[u][s].w;
                }
#pragma unroll
                for (int j = 0; j < VN; ++j)
#pragma unroll
                    for (int n = 0; n < NE; ++n)
                        acc[s][j][n] = __builtin_amdgcn_mfma_f32_16x16x4f32(x[j], dl[u][n], acc[s][j][n], 0, 0, 0);
            }
#pragma unroll
            for (int n = 0; n < NE; ++n) accb[n] += dl[u][n];
        }
    };
    // one trip at a time per wave; the other waves of the CU cover its latency
    constexpr int TRIP = 16 * U;
    for (int tg = t_begin + 4 * wave; tg < t_end; tg += TRIP) {
        raw_t raw[U][CS];
        float dl[U][NE];
        load_trip(tg, raw, dl);
        use_trip(raw, dl);
    }
    // lanes with the same l % 16 hold pieces of the same bias gradient
#pragma unroll
    for (int n = 0; n < NE; ++n) {
        accb[n] += __shfl_xor(accb[n], 16, 64);
        accb[n] += __shfl_xor(accb[n], 32, 64);
    }
    // fold the four waves: waves 1, 2, 3 hand their sums to wave 0 one after the other
    for (int w = 1; w < 4; ++w) {
        if (wave == w) {
#pragma unroll
            for (int s = 0; s < CS; ++s)
#pragma unroll
                for (int j = 0; j < VN; ++j)
#pragma unroll
                    for (int n = 0; n < NE; ++n)
#pragma unroll
                        for (int r = 0; r < 4; ++r) fold[((((s * VN + j) * NE + n) * 4) + r) * 64 + lane] = acc[s][j][n][r];
            if (lane < 16)
#pragma unroll
                for (int n = 0; n < NE; ++n) fold_b[n * 16 + lane] = accb[n];
        }
        __syncthreads();
        if (wave == 0) {
#pragma unroll
            for (int s = 0; s < CS; ++s)
#pragma unroll
                for (int j = 0; j < VN; ++j)
#pragma unroll
                    for (int n = 0; n < NE; ++n)
#pragma unroll
                        for (int r = 0; r < 4; ++r) acc[s][j][n][r] += fold[((((s * VN + j) * NE + n) * 4) + r) * 64 + lane];
            if (lane < 16)
#pragma unroll
                for (int n = 0; n < NE; ++n) accb[n] += fold_b[n * 16 + lane];
        }
        __syncthreads();
    }
    if (wave == 0) {
#pragma unroll
        for (int s = 0; s < CS; ++s)
#pragma unroll
            for (int j = 0; j < VN; ++j)
#pragma unroll
                for (int n = 0; n < NE; ++n)
#pragma unroll
                    for (int r = 0; r < 4; ++r) {
                        const int c = c0 + s * SW + (4 * lk + r) * VN + j, e = e0 + n * 16 + li;
                        if (c < d && e < E) partial[((size_t)part * d + c) * E + e] = acc[s][j][n][r];
                    }
        if (blockIdx.x == 0 && lane < 16)
#pragma unroll
            for (int n = 0; n < NE; ++n)
                if (e0 + n * 16 + lane < E) partial_b[(size_t)part * E + e0 + n * 16 + lane] = accb[n];
    }
}

template <typename ET, int VN, int NE, int CS>
hipError_t launch_wgrad_mfma_t(const moe_shape_t& s, const void* X, const float* dlogits, float* partial, float* partial_b,
                               int n_part, int tok_per_part, hipStream_t st)
{
    const int cw = CS * 16 * VN;
    const dim3 grid((s.d + cw - 1) / cw, n_part);
    for (int e0 = 0; e0 < s.E; e0 += 16 * NE) {                    // one pass unless E > 64
        hipLaunchKernelGGL((gate_wgrad_mfma_kernel<ET, VN, NE, CS>), grid, dim3(256), 0, st, (const ET*)X, dlogits, partial,
                           partial_b, s.T, s.d, s.E, tok_per_part, e0);
        const hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
    }
    return hipSuccess;
}

__global__ void gate_wgrad_reduce_kernel(const float* __restrict__ partial, const float* __restrict__ partial_b,
                                         float* __restrict__ dWg, float* __restrict__ dbg, int n_part, int dE, int E)
{
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < dE) {
        float s = 0.0f;
        int p = 0;
        for (; p + 8 <= n_part; p += 8) {                          // eight loads in flight, added in partition order
            float v[8];
#pragma unroll
            for (int q = 0; q < 8; ++q) v[q] = partial[(size_t)(p + q) * dE + i];
#pragma unroll
            for (int q = 0; q < 8; ++q) s += v[q];
        }
        for (; p < n_part; ++p) s += partial[(size_t)p * dE + i];
        dWg[i] = s;
    }
    if (i < E) {
        float s = 0.0f;
        for (int p = 0; p < n_part; ++p) s += partial_b[(size_t)p * E + i];
        dbg[i] = s;
    }
}

// ---- the same for more than 64 experts ---------------------------------------------------------------
// The strip of Wg no longer fits LDS at once, so it is staged in chunks of 64 experts and the accumulators
// must outlive the chunks: a wave keeps U tokens (U x VN sums per lane) for the whole block, the block stages
// each chunk once and its 4 U tokens use it.  Expert path first (j ascending), then the gate path in
// ascending e, one rounding at the end.
template <typename ET, int VN>
__global__ __launch_bounds__(256) void input_grad_wide_kernel(
    const ET* __restrict__ dXp, const int32_t* __restrict__ pos, const float* __restrict__ dlogits,
    const float* __restrict__ Wg, ET* __restrict__ dX, int T, int d, int E, int k)
{
    constexpr int CW = 64 * VN, WP = CW + 4, U = 8, EC = 64;
    __shared__ __attribute__((aligned(16))) float wt[EC * WP];     // [expert of the chunk][column of the strip]
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int c0 = blockIdx.x * CW, col = c0 + lane * VN;
    const int t0 = (blockIdx.y * 4 + wave) * U;
    float acc[U][VN];
#pragma unroll
    for (int u = 0; u < U; ++u) {
#pragma unroll
        for (int i = 0; i < VN; ++i) acc[u][i] = 0.0f;
        const int t = t0 + u;
        if (t >= T || col >= d) continue;
        for (int j = 0; j < k; ++j) {
            const ET* src = dXp + (size_t)pos[(size_t)t * k + j] * d + col;
            float f[VN];
            if constexpr (sizeof(ET) == 2) {
                unpack_bf16x8(*reinterpret_cast<const uint4*>(src), f);
            } else {
                const float4 v = *reinterpret_cast<const float4*>(src);
                f[0] = v.x; f[1] = v.y; f[2 % VN] = v.z; f[3 % VN] = v.w;
            }
#pragma unroll
            for (int i = 0; i < VN; ++i) acc[u][i] += f[i];
        }
    }
    for (int ec0 = 0; ec0 < E; ec0 += EC) {
        __syncthreads();                                           // everyone is done with the previous chunk
        for (int i = tid; i < CW * EC; i += 256) {
            const int c = i / EC, e = i - c * EC;
            wt[e * WP + c] = (c0 + c < d && ec0 + e < E) ? Wg[(size_t)(c0 + c) * E + ec0 + e] : 0.0f;
        }
        __syncthreads();
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int t = t0 + u;
            if (t >= T) continue;                                  // uniform per wave
            const float gl = (ec0 + lane < E) ? dlogits[(size_t)t * E + ec0 + lane] : 0.0f;
            for (int e = 0; e < EC; ++e) {
                const float g = __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, gl), e));
                if (g == 0.0f) continue;
                const float* wrow = wt + e * WP + lane * VN;
#pragma unroll
                for (int i = 0; i < VN; i += 4) {
                    const float4 wv = *reinterpret_cast<const float4*>(wrow + i);
                    acc[u][i + 0] = fmaf(g, wv.x, acc[u][i + 0]); acc[u][i + 1] = fmaf(g, wv.y, acc[u][i + 1]);
                    acc[u][i + 2] = fmaf(g, wv.z, acc[u][i + 2]); acc[u][i + 3] = fmaf(g, wv.w, acc[u][i + 3]);
                }
            }
        }
    }
#pragma unroll
    for (int u = 0; u < U; ++u) {
        const int t = t0 + u;
        if (t >= T || col >= d) continue;
        if constexpr (sizeof(ET) == 2) {
            *reinterpret_cast<uint4*>(dX + (size_t)t * d + col) =
                make_uint4(pack_bf16x2(acc[u][0], acc[u][1]), pack_bf16x2(acc[u][2], acc[u][3]),
                           pack_bf16x2(acc[u][4 % VN], acc[u][5 % VN]), pack_bf16x2(acc[u][6 % VN], acc[u][7 % VN]));
        } else {
            *reinterpret_cast<float4*>(dX + (size_t)t * d + col) = make_float4(acc[u][0], acc[u][1], acc[u][2], acc[u][3]);
        }
    }
}

template <typename ET, int VN>
hipError_t launch_input_grad_wide_t(const moe_shape_t& s, const void* dXp, const int32_t* pos, const float* dlogits,
                                    const float* Wg, void* dX, hipStream_t st)
{
    constexpr int CW = 64 * VN, TOK = 4 * 8;
    const dim3 grid((s.d + CW - 1) / CW, (s.T + TOK - 1) / TOK);
    hipLaunchKernelGGL((input_grad_wide_kernel<ET, VN>), grid, dim3(256), 0, st, (const ET*)dXp, pos, dlogits, Wg, (ET*)dX,
                       s.T, s.d, s.E, s.k);
    return hipGetLastError();
}

}  // namespace

int gate_grad_partitions(const moe_shape_t& s) { return s.T < 32 * 256 ? (s.T + 255) / 256 : 32; }

template <typename ET, int VN, int EC>
hipError_t launch_input_grad_t(const moe_shape_t& s, const void* dXp, const int32_t* pos, const float* dlogits,
                               const float* Wg, void* dX, hipStream_t st)
{
    constexpr int CW = 64 * VN, TOK = 128;
    const dim3 grid((s.d + CW - 1) / CW, (s.T + TOK - 1) / TOK);
    const size_t lds = (size_t)s.E * (CW + 4) * sizeof(float);
    auto kern = input_grad_kernel<ET, VN, EC>;
    static PerDeviceOnce once;           // per instantiation
    const int dev = current_device();
    if (!once.is_done(dev)) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, 64 * (CW + 4) * 4);
        if (e != hipSuccess) return e;
        once.mark(dev);
    }
    hipLaunchKernelGGL(kern, grid, dim3(256), lds, st, (const ET*)dXp, pos, dlogits, Wg, (ET*)dX, s.T, s.d, s.E, s.k, TOK);
    return hipGetLastError();
}

template <typename ET, int VN, int NE, int CS>
hipError_t launch_input_grad_mfma_t(const moe_shape_t& s, const void* dXp, const int32_t* pos, const float* dlogits,
                                    const float* Wg, void* dX, hipStream_t st)
{
    constexpr int CW = 4 * CS * 16 * VN, TOK = 256;                // a block: 4 waves x CS strips, 256 tokens
    const dim3 grid((s.d + CW - 1) / CW, (s.T + TOK - 1) / TOK);
    if (s.k <= 2)
        hipLaunchKernelGGL((input_grad_mfma_kernel<ET, VN, NE, CS, 2>), grid, dim3(256), 0, st, (const ET*)dXp, pos, dlogits, Wg,
                           (ET*)dX, s.T, s.d, s.E, s.k, TOK);
    else
        hipLaunchKernelGGL((input_grad_mfma_kernel<ET, VN, NE, CS, MAXK_IG>), grid, dim3(256), 0, st, (const ET*)dXp, pos, dlogits, Wg,
                           (ET*)dX, s.T, s.d, s.E, s.k, TOK);
    return hipGetLastError();
}

hipError_t launch_input_grad(const moe_shape_t& s, const void* dXp, const int32_t* pos, const float* dlogits,
                             const float* Wg, void* dX, hipStream_t st)
{
    const bool bf = s.dtype == MOE_BF16;
    if (s.E > 64) return bf ? launch_input_grad_wide_t<bf16_t, 8>(s, dXp, pos, dlogits, Wg, dX, st)
                            : launch_input_grad_wide_t<float, 4>(s, dXp, pos, dlogits, Wg, dX, st);
#ifndef IG_VALU
    if (s.E <= 16) return bf ? launch_input_grad_mfma_t<bf16_t, 8, 1, 1>(s, dXp, pos, dlogits, Wg, dX, st) : launch_input_grad_mfma_t<float, 4, 1, 2>(s, dXp, pos, dlogits, Wg, dX, st);
    if (s.E <= 32) return bf ? launch_input_grad_mfma_t<bf16_t, 8, 2, 1>(s, dXp, pos, dlogits, Wg, dX, st) : launch_input_grad_mfma_t<float, 4, 2, 2>(s, dXp, pos, dlogits, Wg, dX, st);
#endif
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
    if (s.E <= 16)      e = bf ? launch_wgrad_mfma_t<bf16_t, 8, 1, 2>(s, X, dlogits, partial, partial_b, n_part, tok_per_part, st)
                               : launch_wgrad_mfma_t<float, 4, 1, 2>(s, X, dlogits, partial, partial_b, n_part, tok_per_part, st);
    else if (s.E <= 32) e = bf ? launch_wgrad_mfma_t<bf16_t, 8, 2, 1>(s, X, dlogits, partial, partial_b, n_part, tok_per_part, st)
                               : launch_wgrad_mfma_t<float, 4, 2, 2>(s, X, dlogits, partial, partial_b, n_part, tok_per_part, st);
    else                e = bf ? launch_wgrad_mfma_t<bf16_t, 8, 4, 1>(s, X, dlogits, partial, partial_b, n_part, tok_per_part, st)
                               : launch_wgrad_mfma_t<float, 4, 4, 1>(s, X, dlogits, partial, partial_b, n_part, tok_per_part, st);
    if (e != hipSuccess) return e;
    const int dE = s.d * s.E;
    hipLaunchKernelGGL(gate_wgrad_reduce_kernel, dim3((dE + 255) / 256), dim3(256), 0, st, partial, partial_b, dWg, dbg, n_part, dE, s.E);
    return hipGetLastError();
}

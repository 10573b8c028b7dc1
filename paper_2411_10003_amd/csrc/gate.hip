// Gate logits in a fixed fp32 summation order, top-k routing and gate weights (Section 2.1 of
// the paper: the gate relates every input to all experts and routes it to the top-k), and the
// gradient of the gate weights with respect to the logits.
//
// Summation order of logit[t,e] (what makes routing reproducible bit for bit): 64 partial sums,
// partial l takes the columns c = l, l+64, ... in ascending order with one fused multiply-add
// each; partials are folded l <- l + (l+off) for off = 32..1; the bias is added last.
// A wavefront maps partial l to lane l, keeps TOK tokens x EC experts of partials in registers,
// and folds all of them together with a butterfly that halves the register count every step.
#include "internal.h"

namespace {

constexpr int GATE_WAVES = 8;                 // waves per block
constexpr int GATE_THREADS = GATE_WAVES * 64;
constexpr int GATE_ACC = 128;                 // partial sums per lane: TOK * EC
constexpr int GATE_W_FLOATS = 4096;           // gate-matrix floats staged in LDS per chunk

template <typename XT> __device__ __forceinline__ float load_x(const XT* p);
template <> __device__ __forceinline__ float load_x<float>(const float* p) { return *p; }
template <> __device__ __forceinline__ float load_x<bf16_t>(const bf16_t* p) { return bf16_to_f32(*p); }

__device__ __forceinline__ int bitrev6(int l) {
    return ((l & 1) << 5) | ((l & 2) << 3) | ((l & 4) << 1) | ((l & 8) >> 1) | ((l & 16) >> 3) | ((l & 32) >> 5);
}

// EC experts per pass (8, 16, 32 or 64); TOK = 128 / EC tokens per wave.
template <typename XT, int EC>
__global__ __launch_bounds__(GATE_THREADS) void gate_topk_kernel(
    const XT* __restrict__ X, const float* __restrict__ Wg, const float* __restrict__ bg,
    float* __restrict__ logits, int32_t* __restrict__ idx, float* __restrict__ wout,
    int T, int d, int E, int k, int renorm, int e_pitch)
{
    constexpr int TOK = GATE_ACC / EC;
    constexpr int RC = GATE_W_FLOATS / EC;    // gate-matrix rows per LDS chunk (a multiple of 64)
    constexpr int E4 = EC / 4;
    static_assert(RC % 64 == 0, "chunk must hold whole 64-column steps");

    __shared__ float4 w_lds[E4 * RC];          // [e/4][row] -> 4 consecutive experts of one row
    extern __shared__ float logit_lds[];       // [GATE_WAVES * TOK][e_pitch]

    const int lane = threadIdx.x & 63;
    const int wave = threadIdx.x >> 6;
    const int tok0 = (blockIdx.x * GATE_WAVES + wave) * TOK;

    const XT* xrow[TOK];
#pragma unroll
    for (int tk = 0; tk < TOK; ++tk) {
        int t = tok0 + tk;
        if (t > T - 1) t = T - 1;              // rows past the end recompute the last token; never stored
        xrow[tk] = X + (size_t)t * d;
    }

    for (int ec0 = 0; ec0 < E; ec0 += EC) {
        float acc[GATE_ACC];
#pragma unroll
        for (int i = 0; i < GATE_ACC; ++i) acc[i] = 0.0f;

        for (int c0 = 0; c0 < d; c0 += RC) {
            __syncthreads();
            // stage Wg[c0 .. c0+RC) x [ec0 .. ec0+EC), zero outside the matrix
            for (int i = threadIdx.x; i < RC * EC; i += GATE_THREADS) {
                int e = i % EC, r = i / EC;
                float v = 0.0f;
                if (c0 + r < d && ec0 + e < E) v = Wg[(size_t)(c0 + r) * E + ec0 + e];
                reinterpret_cast<float*>(w_lds)[((e >> 2) * RC + r) * 4 + (e & 3)] = v;
            }
            __syncthreads();
#pragma unroll 1
            for (int js = 0; js < RC / 64; ++js) {
                const int c = c0 + js * 64 + lane;
                if (c0 + js * 64 >= d) break;
                float x[TOK];
#pragma unroll
                for (int tk = 0; tk < TOK; ++tk) x[tk] = (c < d) ? load_x<XT>(xrow[tk] + c) : 0.0f;
#pragma unroll
                for (int e4 = 0; e4 < E4; ++e4) {
                    const float4 wv = w_lds[e4 * RC + js * 64 + lane];
#pragma unroll
                    for (int tk = 0; tk < TOK; ++tk) {
                        float* a = &acc[tk * EC + e4 * 4];
                        a[0] = fmaf(x[tk], wv.x, a[0]);
                        a[1] = fmaf(x[tk], wv.y, a[1]);
                        a[2] = fmaf(x[tk], wv.z, a[2]);
                        a[3] = fmaf(x[tk], wv.w, a[3]);
                    }
                }
            }
        }

        // Fold the 64 partials of all 128 sums at once.  At the step with offset `off`, register
        // pair (2i, 2i+1) becomes register i: lanes with the `off` bit clear finish sum 2i
        // (s_l + s_{l+off}), lanes with it set finish sum 2i+1.
#pragma unroll
        for (int step = 0; step < 6; ++step) {
            const int n = 64 >> step, off = 32 >> step;
            const bool up = (lane & off) != 0;
#pragma unroll
            for (int i = 0; i < n; ++i) {
                float keep = up ? acc[2 * i + 1] : acc[2 * i];
                float send = up ? acc[2 * i] : acc[2 * i + 1];
                float recv = __shfl_xor(send, off, 64);
                acc[i] = keep + recv;
            }
        }
        // lane l, register i now hold sum number 64*i + bitrev6(l), numbered tk*EC + e
#pragma unroll
        for (int i = 0; i < 2; ++i) {
            const int r = 64 * i + bitrev6(lane);
            const int tk = r / EC, e = ec0 + r % EC;
            if (e < E) {
                const float v = acc[i] + bg[e];
                logit_lds[(wave * TOK + tk) * e_pitch + e] = v;
                if (tok0 + tk < T) logits[(size_t)(tok0 + tk) * E + e] = v;
            }
        }
    }
    __syncthreads();

    // Top-k, softmax and gate weights: one lane per token.
    if (lane < TOK && tok0 + lane < T) {
        const int t = tok0 + lane;
        const float* lg = logit_lds + (wave * TOK + lane) * e_pitch;
        int sel[8];
        float selv[8];
        for (int j = 0; j < k; ++j) {
            int best = -1;
            float bv = 0.0f;
            for (int e = 0; e < E; ++e) {
                bool taken = false;
                for (int q = 0; q < j; ++q) taken |= (sel[q] == e);
                if (taken) continue;
                float v = lg[e];
                v = (v != v) ? -INFINITY : v;
                if (best < 0 || v > bv) { best = e; bv = v; }
            }
            sel[j] = best;
            selv[j] = bv;
        }
        const float m = selv[0];
        float sum = 0.0f;
        for (int e = 0; e < E; ++e) {
            float v = lg[e];
            v = (v != v) ? -INFINITY : v;
            sum += expf(v - m);
        }
        float ps[8], psum = 0.0f;
        for (int j = 0; j < k; ++j) { ps[j] = expf(selv[j] - m) / sum; psum += ps[j]; }
        for (int j = 0; j < k; ++j) {
            idx[(size_t)t * k + j] = sel[j];
            wout[(size_t)t * k + j] = renorm ? ps[j] / psum : ps[j];
        }
    }
}

__global__ void gate_bwd_kernel(const float* __restrict__ dw, const float* __restrict__ logits,
                                const int32_t* __restrict__ idx, float* __restrict__ dlogits,
                                int T, int E, int k, int renorm)
{
    const int t = blockIdx.x * blockDim.x + threadIdx.x;
    if (t >= T) return;
    const float* lg = logits + (size_t)t * E;
    float* dl = dlogits + (size_t)t * E;
    float m = -INFINITY;
    for (int e = 0; e < E; ++e) m = fmaxf(m, lg[e]);
    float sum = 0.0f;
    for (int e = 0; e < E; ++e) sum += expf(lg[e] - m);
    const float inv = 1.0f / sum;
    int s[8];
    float g[8], ps[8];
    float psel = 0.0f;
    for (int j = 0; j < k; ++j) {
        s[j] = idx[(size_t)t * k + j];
        g[j] = dw[(size_t)t * k + j];
        ps[j] = expf(lg[s[j]] - m) * inv;
        psel += ps[j];
    }
    if (renorm) {
        float dot = 0.0f;
        for (int j = 0; j < k; ++j) dot += (ps[j] / psel) * g[j];
        for (int e = 0; e < E; ++e) dl[e] = 0.0f;
        for (int j = 0; j < k; ++j) dl[s[j]] = (ps[j] / psel) * (g[j] - dot);
    } else {
        float gp = 0.0f;                        // sum_j dw_j p[s_j]
        for (int j = 0; j < k; ++j) gp += g[j] * ps[j];
        for (int e = 0; e < E; ++e) {
            float pe = expf(lg[e] - m) * inv;
            float v = -gp * pe;
            for (int j = 0; j < k; ++j) if (s[j] == e) v += g[j] * ps[j];
            dl[e] = v;
        }
    }
}

template <typename XT, int EC>
hipError_t run_gate(const moe_shape_t& s, const void* X, const float* Wg, const float* bg,
                    float* logits, int32_t* idx, float* w, hipStream_t st)
{
    constexpr int TOK = GATE_ACC / EC;
    const int tok_per_block = GATE_WAVES * TOK;
    const int grid = (s.T + tok_per_block - 1) / tok_per_block;
    const int e_pitch = s.E | 1;
    const size_t dyn = (size_t)GATE_WAVES * TOK * e_pitch * sizeof(float);
    hipLaunchKernelGGL((gate_topk_kernel<XT, EC>), dim3(grid), dim3(GATE_THREADS), dyn, st,
                       (const XT*)X, Wg, bg, logits, idx, w, s.T, s.d, s.E, s.k, s.renorm, e_pitch);
    return hipGetLastError();
}

template <typename XT>
hipError_t run_gate_t(const moe_shape_t& s, const void* X, const float* Wg, const float* bg,
                      float* logits, int32_t* idx, float* w, hipStream_t st)
{
    if (s.E <= 8) return run_gate<XT, 8>(s, X, Wg, bg, logits, idx, w, st);
    if (s.E <= 16) return run_gate<XT, 16>(s, X, Wg, bg, logits, idx, w, st);
    if (s.E <= 32) return run_gate<XT, 32>(s, X, Wg, bg, logits, idx, w, st);
    return run_gate<XT, 64>(s, X, Wg, bg, logits, idx, w, st);
}

}  // namespace

hipError_t launch_gate_topk(const moe_shape_t& s, const void* X, const float* Wg, const float* bg,
                            float* logits, int32_t* idx, float* w, hipStream_t st)
{
    if (s.T == 0) return hipSuccess;
    if (s.dtype == MOE_F32) return run_gate_t<float>(s, X, Wg, bg, logits, idx, w, st);
    return run_gate_t<bf16_t>(s, X, Wg, bg, logits, idx, w, st);
}

hipError_t launch_gate_bwd(const moe_shape_t& s, const float* dw, const float* logits, const int32_t* idx,
                           float* dlogits, hipStream_t st)
{
    if (s.T == 0) return hipSuccess;
    const int threads = 256;
    hipLaunchKernelGGL(gate_bwd_kernel, dim3((s.T + threads - 1) / threads), dim3(threads), 0, st,
                       dw, logits, idx, dlogits, s.T, s.E, s.k, s.renorm);
    return hipGetLastError();
}

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

// Fold the 64 partials of all 128 sums of a wave at once and store the logits (LDS + global).  At the
// step with offset `off`, register pair (2i, 2i+1) becomes register i: lanes with the `off` bit clear
// finish sum 2i (s_l + s_{l+off}), lanes with it set finish sum 2i+1.  These are exactly the additions
// of the fixed order; only which lane performs them differs.
template <int EC>
__device__ __forceinline__ void fold_and_store(float (&acc)[GATE_ACC], int lane, int wave, int tok0, int ec0,
                                               int T, int E, int e_pitch, const float* __restrict__ bg,
                                               float* logit_lds, float* __restrict__ logits)
{
    constexpr int TOK = GATE_ACC / EC;
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

// Top-k, softmax and gate weights: one lane per token of the wave, reading the logits from LDS.
template <int TOK>
__device__ __forceinline__ void route_tokens(int lane, int wave, int tok0, int T, int E, int k, int renorm, int e_pitch,
                                             const float* logit_lds, int32_t* __restrict__ idx, float* __restrict__ wout)
{
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

        fold_and_store<EC>(acc, lane, wave, tok0, ec0, T, E, e_pitch, bg, logit_lds, logits);
    }
    __syncthreads();
    route_tokens<GATE_ACC / EC>(lane, wave, tok0, T, E, k, renorm, e_pitch, logit_lds, idx, wout);
}

// ---- fast path: bf16 X, E == EC in {16, 32, 64}, d a multiple of the chunk depth -------------------
// Both the gate matrix and the tokens stream through a 3-deep LDS ring filled by buffer loads that
// write LDS directly (16 bytes per lane, whole rows), so HBM sees each token row once in 512-byte
// pieces and no address arithmetic or conversion runs in the FMA loop.  Same summation order.
typedef __attribute__((ext_vector_type(4))) int gate_rsrc_t;
#define GATE_LDS_PTR(T) __attribute__((address_space(3))) T*

__device__ __forceinline__ gate_rsrc_t gate_make_rsrc(const void* base, unsigned long long bytes)
{
    if (bytes > 0xffffffffull) bytes = 0xffffffffull;
    const unsigned long long b = (unsigned long long)base;
    gate_rsrc_t r;
    r[0] = (int)(unsigned)(b & 0xffffffffull);
    r[1] = (int)(unsigned)((b >> 32) & 0xffffull);
    r[2] = (int)(unsigned)bytes;                           // reads past this limit return zero
    r[3] = 0x00020000;
    return r;
}
__device__ __forceinline__ void gate_dma16(gate_rsrc_t r, uint32_t lds_base, uint32_t voff, uint32_t soff)
{
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tbuffer_load_dwordx4 %1, %2, %3 offen lds"
                 :: "s"(lds_base), "v"(voff), "s"(r), "s"(soff) : "memory");
}

template <int EC>
__global__ __launch_bounds__(GATE_THREADS) void gate_topk_fast_kernel(
    const bf16_t* __restrict__ X, const float* __restrict__ Wg, const float* __restrict__ bg,
    float* __restrict__ logits, int32_t* __restrict__ idx, float* __restrict__ wout,
    int T, int d, int k, int renorm, int e_pitch)
{
    constexpr int E = EC;
    constexpr int TOK = GATE_ACC / EC;                     // tokens per wave
    constexpr int NTOK = GATE_WAVES * TOK;                 // tokens per block
    constexpr int RC = GATE_W_FLOATS / EC;                 // contraction depth of a chunk (256 / 128 / 64)
    constexpr int E4 = EC / 4;                             // 16-byte pieces per gate-matrix row
    constexpr int W_BYTES = GATE_W_FLOATS * 4;             // 16 KB
    constexpr int X_BYTES = NTOK * RC * 2;
    constexpr int STAGE = W_BYTES + X_BYTES;
    constexpr int NST = 3;
    constexpr int W_PIECES = W_BYTES / 1024 / GATE_WAVES;  // DMA instructions per wave per chunk
    constexpr int X_PIECES = (X_BYTES / 1024 + GATE_WAVES - 1) / GATE_WAVES;
    constexpr int SW_SHIFT = (E4 == 4) ? 2 : (E4 == 8 ? 1 : 0);

    extern __shared__ __attribute__((aligned(1024))) unsigned char gsm[];   // ring, then the logits
    const uint32_t lds0 = (uint32_t)(uintptr_t)(GATE_LDS_PTR(unsigned char))gsm;
    float* logit_lds = reinterpret_cast<float*>(gsm + NST * STAGE);

    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int blk_tok0 = blockIdx.x * NTOK;
    const int tok0 = blk_tok0 + wave * TOK;

    // gate matrix: row r is E floats = E4 pieces; piece p of row r lands in slot p ^ swz(r) of that row
    const gate_rsrc_t rW = gate_make_rsrc(Wg, (unsigned long long)d * E * 4);
    // tokens of this block: rows past T read as zero
    const long long xrows = (long long)T - blk_tok0;
    const gate_rsrc_t rX = gate_make_rsrc(X + (size_t)blk_tok0 * d, (unsigned long long)(xrows > 0 ? xrows : 0) * d * 2);
    uint32_t wv_off[W_PIECES], wl_off[W_PIECES], xv_off[X_PIECES], xl_off[X_PIECES];
#pragma unroll
    for (int i = 0; i < W_PIECES; ++i) {
        const int L = (wave * W_PIECES + i) * 64 + lane;   // 16-byte slot in the chunk
        const int r = L / E4, slot = L % E4;
        const int piece = slot ^ ((r >> SW_SHIFT) & (E4 - 1));
        wv_off[i] = (uint32_t)((r * E + piece * 4) * 4);
        wl_off[i] = (uint32_t)((wave * W_PIECES + i) * 1024);
    }
#pragma unroll
    for (int i = 0; i < X_PIECES; ++i) {
        const int L = (wave * X_PIECES + i) * 64 + lane;   // 16-byte slot: token L / (RC/8), piece L % (RC/8)
        const int tk = L / (RC / 8), piece = L % (RC / 8);
        xv_off[i] = (uint32_t)((tk * d + piece * 8) * 2);
        xl_off[i] = (uint32_t)(W_BYTES + (wave * X_PIECES + i) * 1024);
    }
    const int n_chunks = d / RC;
    const bool has_x = wave * X_PIECES * 1024 < X_BYTES;  // with few tokens per block only the first waves move X
    static_assert(X_PIECES == 1 || (X_BYTES / 1024) % GATE_WAVES == 0, "a wave moves all of its X pieces or none");
    auto issue = [&](int c) {
        const uint32_t st = lds0 + (uint32_t)(c % NST) * STAGE;
#pragma unroll
        for (int i = 0; i < W_PIECES; ++i) gate_dma16(rW, st + wl_off[i], wv_off[i], (uint32_t)c * (RC * E * 4));
#pragma unroll
        for (int i = 0; i < X_PIECES; ++i)
            if (has_x) gate_dma16(rX, st + xl_off[i], xv_off[i], (uint32_t)c * (RC * 2));
    };

    float acc[GATE_ACC];
#pragma unroll
    for (int i = 0; i < GATE_ACC; ++i) acc[i] = 0.0f;

    issue(0);
    if (n_chunks > 1) issue(1);
    for (int c = 0; c < n_chunks; ++c) {
        // everything but this wave's share of the next chunk must have landed
        if (c + 1 >= n_chunks) asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        else if (has_x) asm volatile("s_waitcnt vmcnt(%0)" :: "n"(W_PIECES + X_PIECES) : "memory");
        else asm volatile("s_waitcnt vmcnt(%0)" :: "n"(W_PIECES) : "memory");
        asm volatile("s_barrier" ::: "memory");
        if (c + 2 < n_chunks) issue(c + 2);
        // The reads of a 64-column step (TOK token values of the lane's column, the E weights of its row) are
        // issued together, one step ahead of the multiply-adds that use them, and waited for once: left to the
        // compiler every read is followed by a wait of its own.
        const uint32_t st = lds0 + (uint32_t)(c % NST) * STAGE;
        const uint32_t xa0 = st + W_BYTES + (uint32_t)((wave * TOK * RC + lane) * 2);
        typedef __attribute__((ext_vector_type(4))) float gate_f4;
        uint32_t xr[2][TOK];
        gate_f4 wr[2][E4];
        auto request = [&](int js, uint32_t (&xq)[TOK], gate_f4 (&wq)[E4]) {
            const uint32_t xa = xa0 + (uint32_t)js * 128;
#pragma unroll
            for (int tk = 0; tk < TOK; ++tk)
                asm volatile("ds_read_u16 %0, %1 offset:%2" : "=v"(xq[tk]) : "v"(xa), "n"(tk * RC * 2));
            const int r = js * 64 + lane;
            const int sw = (r >> SW_SHIFT) & (E4 - 1);
#pragma unroll
            for (int e4 = 0; e4 < E4; ++e4) {
                const uint32_t wa = st + (uint32_t)((r * E4 + (e4 ^ sw)) * 16);
                asm volatile("ds_read_b128 %0, %1" : "=v"(wq[e4]) : "v"(wa));
            }
        };
        auto arrive = [&](uint32_t (&xq)[TOK], gate_f4 (&wq)[E4]) {            // everything requested so far has landed
#pragma unroll
            for (int tk = 0; tk < TOK; ++tk) asm volatile("" : "+v"(xq[tk]));
            asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
#pragma unroll
            for (int tk = 0; tk < TOK; ++tk) asm volatile("" : "+v"(xq[tk]));
#pragma unroll
            for (int e4 = 0; e4 < E4; ++e4) asm volatile("" : "+v"(wq[e4]));
        };
        auto multiply = [&](const uint32_t (&xq)[TOK], const gate_f4 (&wq)[E4]) {
#pragma unroll
            for (int e4 = 0; e4 < E4; ++e4)
#pragma unroll
                for (int tk = 0; tk < TOK; ++tk) {
                    const float x = __uint_as_float(xq[tk] << 16);
                    float* a = &acc[tk * EC + e4 * 4];
                    a[0] = fmaf(x, wq[e4][0], a[0]);
                    a[1] = fmaf(x, wq[e4][1], a[1]);
                    a[2] = fmaf(x, wq[e4][2], a[2]);
                    a[3] = fmaf(x, wq[e4][3], a[3]);
                }
        };
        request(0, xr[0], wr[0]);
#pragma unroll
        for (int js = 0; js < RC / 64; ++js) {
            arrive(xr[js & 1], wr[js & 1]);
            if (js + 1 < RC / 64) request(js + 1, xr[(js + 1) & 1], wr[(js + 1) & 1]);
            multiply(xr[js & 1], wr[js & 1]);
        }
    }
    fold_and_store<EC>(acc, lane, wave, tok0, 0, T, E, e_pitch, bg, logit_lds, logits);
    __syncthreads();
    route_tokens<TOK>(lane, wave, tok0, T, E, k, renorm, e_pitch, logit_lds, idx, wout);
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

template <int EC>
hipError_t run_gate_fast(const moe_shape_t& s, const void* X, const float* Wg, const float* bg,
                         float* logits, int32_t* idx, float* w, hipStream_t st)
{
    constexpr int TOK = GATE_ACC / EC, NTOK = GATE_WAVES * TOK, RC = GATE_W_FLOATS / EC;
    constexpr int STAGE = GATE_W_FLOATS * 4 + NTOK * RC * 2;
    const int e_pitch = s.E | 1;
    const size_t lds = (size_t)3 * STAGE + (size_t)NTOK * e_pitch * sizeof(float);
    auto kern = gate_topk_fast_kernel<EC>;
    static bool configured = false;
    if (!configured) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        if (e != hipSuccess) return e;
        configured = true;
    }
    const int grid = (s.T + NTOK - 1) / NTOK;
    hipLaunchKernelGGL(kern, dim3(grid), dim3(GATE_THREADS), lds, st, (const bf16_t*)X, Wg, bg, logits, idx, w,
                       s.T, s.d, s.k, s.renorm, e_pitch);
    return hipGetLastError();
}

}  // namespace

hipError_t launch_gate_topk(const moe_shape_t& s, const void* X, const float* Wg, const float* bg,
                            float* logits, int32_t* idx, float* w, hipStream_t st)
{
    if (s.T == 0) return hipSuccess;
    if (s.dtype == MOE_BF16 && (long long)s.T * s.d * 2 < (1ll << 32)) {
        if (s.E == 16 && s.d % 256 == 0) return run_gate_fast<16>(s, X, Wg, bg, logits, idx, w, st);
        if (s.E == 32 && s.d % 128 == 0) return run_gate_fast<32>(s, X, Wg, bg, logits, idx, w, st);
        if (s.E == 64 && s.d % 64 == 0) return run_gate_fast<64>(s, X, Wg, bg, logits, idx, w, st);
    }
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

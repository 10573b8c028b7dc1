// Gate logits in a fixed fp32 summation order, top-k routing and gate weights (Section 2.1 of
// the paper: the gate relates every input to all experts and routes it to the top-k), and the
// gradient of the gate weights with respect to the logits.
//
// Summation order of logit[t,e] (what makes routing reproducible bit for bit): two partial sums; the
// columns are taken in blocks of 32 and block B belongs to partial B mod 2; inside a block the columns
// are visited as c = 32B + 8q + j with j = 0..7 outer and q = 0..3 inner, one fused multiply-add each;
// logit = (s0 + s1) + bias.  This is the order in which the 16x16x4 fp32 matrix instruction accumulates
// (four fused multiply-adds in ascending k, denormals kept) when a lane feeds it the 8 consecutive
// columns it loaded with one 16-byte request, so the whole contraction runs on the matrix cores.
#include "internal.h"
#include <type_traits>

namespace {

constexpr int GATE_WAVES = 4;                 // waves per block, 16 tokens each
constexpr int GATE_THREADS = GATE_WAVES * 64;
constexpr int GATE_TOK = GATE_WAVES * 16;     // tokens per block

typedef float gate_f4 __attribute__((ext_vector_type(4)));
typedef unsigned gate_u4 __attribute__((ext_vector_type(4)));

// Eight consecutive columns of one token, as loaded.
template <typename XT> struct XPiece;
template <> struct XPiece<bf16_t> { uint4 v; };
template <> struct XPiece<float> { float4 a, b; };

// Loads.  FULL (d % 64 == 0, every staged expert exists): a request is either inside the matrix or belongs to a
// chunk past the end that is never multiplied, so its address is clamped and nothing is selected; the request stays
// unconditional, which matters: a load under a condition makes the compiler drain all outstanding requests at the
// join.  Otherwise columns at or past d and experts at or past E are replaced by zeros.
template <bool VEC, bool FULL>
__device__ __forceinline__ void load_piece(XPiece<bf16_t>& p, const bf16_t* row, int c, int d)
{
    // bf16 shapes have d % 64 == 0: a piece is inside the row or past it
    const uint4 v = *reinterpret_cast<const uint4*>(row + (c < d ? c : 0));
    if (FULL) p.v = v;
    else p.v = (c < d) ? v : make_uint4(0u, 0u, 0u, 0u);
}
template <bool VEC, bool FULL>
__device__ __forceinline__ void load_piece(XPiece<float>& p, const float* row, int c, int d)
{
    if (FULL) {
        p.a = *reinterpret_cast<const float4*>(row + (c < d ? c : 0));
        p.b = *reinterpret_cast<const float4*>(row + (c < d ? c + 4 : 0));
    } else if (VEC) {                           // d % 4 == 0: each half is inside the row or past it
        const float4 a = *reinterpret_cast<const float4*>(row + (c < d ? c : 0));
        const float4 b = *reinterpret_cast<const float4*>(row + (c + 4 < d ? c + 4 : 0));
        p.a = (c < d) ? a : make_float4(0.0f, 0.0f, 0.0f, 0.0f);
        p.b = (c + 4 < d) ? b : make_float4(0.0f, 0.0f, 0.0f, 0.0f);
    } else {
        float v[8];
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            const float x = row[c + j < d ? c + j : 0];
            v[j] = (c + j < d) ? x : 0.0f;
        }
        p.a = make_float4(v[0], v[1], v[2], v[3]);
        p.b = make_float4(v[4], v[5], v[6], v[7]);
    }
}
template <int J> __device__ __forceinline__ float piece_get(const XPiece<bf16_t>& p)
{
    const uint32_t w = (J / 2 == 0) ? p.v.x : (J / 2 == 1) ? p.v.y : (J / 2 == 2) ? p.v.z : p.v.w;
    return __uint_as_float((J & 1) ? (w & 0xffff0000u) : (w << 16));
}
template <int J> __device__ __forceinline__ float piece_get(const XPiece<float>& p)
{
    const float4& h = (J < 4) ? p.a : p.b;
    return (J % 4 == 0) ? h.x : (J % 4 == 1) ? h.y : (J % 4 == 2) ? h.z : h.w;
}

// Top-k, softmax and gate weights of one token from its E logits.
__device__ __forceinline__ void route_one(const float* lg, int t, int E, int k, int renorm,
                                          int32_t* __restrict__ idx, float* __restrict__ wout)
{
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

// The same routing by four lanes per token (lane = 4 * token + part; part takes the experts e = part, part + 4, ...):
// every lane proposes its best remaining logit, two exchange steps pick the winner by (value descending, index
// ascending), which is the order of the serial scan; the softmax sum is folded the same way.  All 64 lanes take part
// in the exchanges; `store` says whether the token exists.
__device__ __forceinline__ void route_four(const float* lg, int part, int t, bool store, int E, int k, int renorm,
                                           int32_t* __restrict__ idx, float* __restrict__ wout)
{
    int sel[8];
    float selv[8];
    for (int j = 0; j < k; ++j) {
        int best = 0x7fffffff;
        float bv = -INFINITY;
        for (int e = part; e < E; e += 4) {
            bool taken = false;
            for (int q = 0; q < j; ++q) taken |= (sel[q] == e);
            if (taken) continue;
            float v = lg[e];
            v = (v != v) ? -INFINITY : v;
            if (best == 0x7fffffff || v > bv) { best = e; bv = v; }
        }
#pragma unroll
        for (int off = 1; off <= 2; off <<= 1) {
            const float ov = __shfl_xor(bv, off, 64);
            const int oi = __shfl_xor(best, off, 64);
            if (oi != 0x7fffffff && (best == 0x7fffffff || ov > bv || (ov == bv && oi < best))) { bv = ov; best = oi; }
        }
        sel[j] = best;
        selv[j] = bv;
    }
    const float m = selv[0];
    float sum = 0.0f;
    for (int e = part; e < E; e += 4) {
        float v = lg[e];
        v = (v != v) ? -INFINITY : v;
        sum += expf(v - m);
    }
    sum += __shfl_xor(sum, 1, 64);
    sum += __shfl_xor(sum, 2, 64);
    float ps[8], psum = 0.0f;
    for (int j = 0; j < k; ++j) { ps[j] = expf(selv[j] - m) / sum; psum += ps[j]; }
    if (store && part == 0)
        for (int j = 0; j < k; ++j) {
            idx[(size_t)t * k + j] = sel[j];
            wout[(size_t)t * k + j] = renorm ? ps[j] / psum : ps[j];
        }
}

// One block = 64 tokens, wave w = tokens 16w..16w+15 over the whole contraction; NT tiles of 16 experts per
// pass.  MFMA roles: rows = experts (A operand: the gate matrix, staged through LDS in chunks of 64 columns
// shared by the four waves), columns = tokens (B operand: the lane's own 16-byte pieces of X, NXP chunks
// requested ahead).  Lane l = (q = l / 16, i = l % 16) feeds expert 16*tile + i and token i with column
// 32B + 8q + j in the j-th instruction of block B; the two blocks of a chunk go to the two partial sums.
// ROUTE: E <= 16 NT, one pass, routing fused; otherwise passes of 16 NT experts write logits only.
template <typename XT, int NT, int NXP, bool ROUTE, bool VEC, bool FULL, bool EVEN>
__global__ __launch_bounds__(GATE_THREADS) void gate_mfma_kernel(
    const XT* __restrict__ X, const float* __restrict__ Wg, const float* __restrict__ bg,
    float* __restrict__ logits, int32_t* __restrict__ idx, float* __restrict__ wout,
    int T, int d, int E, int k, int renorm, int e_pitch)
{
    constexpr int CHF = 1024 * NT;             // floats of one staged chunk: 64 columns x 16 NT experts
    __shared__ float w_lds[2 * CHF];           // [buffer][block s][q][tile][j / 4][i][j % 4]
    extern __shared__ float logit_lds[];       // ROUTE: [GATE_TOK][e_pitch]

    const int lane = threadIdx.x & 63;
    const int wave = threadIdx.x >> 6;
    const int q = lane >> 4, i16 = lane & 15;
    const int tok0w = blockIdx.x * GATE_TOK + wave * 16;
    const int tok = tok0w + i16;
    const XT* xrow = X + (size_t)(tok < T ? tok : T - 1) * d;     // rows past the end recompute the last token; never stored
    const int npairs = (d + 63) / 64;

    for (int ec0 = 0; ec0 < E; ec0 += 16 * NT) {
        gate_f4 acc[2][NT];
#pragma unroll
        for (int s = 0; s < 2; ++s)
#pragma unroll
            for (int tl = 0; tl < NT; ++tl) acc[s][tl] = gate_f4{0.0f, 0.0f, 0.0f, 0.0f};

        XPiece<XT> xb[NXP][2];
        auto load_pair = [&](int p, XPiece<XT> (&dst)[2]) {
            load_piece<VEC, FULL>(dst[0], xrow, p * 64 + 8 * q, d);
            load_piece<VEC, FULL>(dst[1], xrow, p * 64 + 32 + 8 * q, d);
        };
        // gate-matrix chunk p: item n of a thread = 4 consecutive experts of one column
        auto load_w = [&](int p, float4 (&wr)[NT]) {
#pragma unroll
            for (int n = 0; n < NT; ++n) {
                const int it = n * GATE_THREADS + threadIdx.x;
                const int c = p * 64 + it / (4 * NT), e = ec0 + 4 * (it % (4 * NT));
                const bool in_c = c < d;
                const float* src = Wg + (size_t)(in_c ? c : 0) * E;
                float4 v;
                if (FULL) {
                    v = *reinterpret_cast<const float4*>(src + e);
                } else if (VEC) {                       // E % 4 == 0: the four experts are inside the row or past it
                    v = *reinterpret_cast<const float4*>(src + (e < E ? e : 0));
                    if (!(in_c && e < E)) v = make_float4(0.0f, 0.0f, 0.0f, 0.0f);
                } else {
                    const float x0 = src[e + 0 < E ? e + 0 : 0], x1 = src[e + 1 < E ? e + 1 : 0];
                    const float x2 = src[e + 2 < E ? e + 2 : 0], x3 = src[e + 3 < E ? e + 3 : 0];
                    v.x = (in_c && e + 0 < E) ? x0 : 0.0f;
                    v.y = (in_c && e + 1 < E) ? x1 : 0.0f;
                    v.z = (in_c && e + 2 < E) ? x2 : 0.0f;
                    v.w = (in_c && e + 3 < E) ? x3 : 0.0f;
                }
                wr[n] = v;
            }
        };
        auto store_w = [&](int buf, const float4 (&wr)[NT]) {
#pragma unroll
            for (int n = 0; n < NT; ++n) {
                const int it = n * GATE_THREADS + threadIdx.x;
                const int cc = it / (4 * NT), e4 = it % (4 * NT);
                const int s = cc >> 5, qq = (cc >> 3) & 3, jh = (cc >> 2) & 1, j4 = cc & 3;
                const int tl = e4 >> 2, i0 = (e4 & 3) * 4;
                float* dst = w_lds + buf * CHF + (((((s * 4 + qq) * NT + tl) * 2 + jh) * 16 + i0) * 4 + j4);
                dst[0] = wr[n].x;
                dst[4] = wr[n].y;
                dst[8] = wr[n].z;
                dst[12] = wr[n].w;
            }
        };
        // Ring slot u holds the tokens' columns of chunk p and the gate-matrix chunk p + 1, requested together
        // NXP chunks ahead: the memory counter retires in order, so whatever is needed soon must not have been
        // requested after something that is needed late.
        float4 wreg[NXP][NT];
        load_w(0, wreg[0]);
        store_w(0, wreg[0]);
#pragma unroll
        for (int u = 0; u < NXP; ++u) {
            load_pair(u, xb[u]);                                  // past the row: zeros, no access
            load_w(u + 1, wreg[u]);
        }
        __syncthreads();

        for (int p0 = 0; p0 < npairs; p0 += NXP) {
#pragma unroll
            for (int u = 0; u < NXP; ++u) {
                const int p = p0 + u;
                if (EVEN || p < npairs) {       // EVEN: the chunk count is a multiple of NXP (no branch in the ring)
                    const float* wb = w_lds + (p & 1) * CHF;
                    gate_f4 wf[2][NT][2];
#pragma unroll
                    for (int s = 0; s < 2; ++s)
#pragma unroll
                        for (int tl = 0; tl < NT; ++tl)
#pragma unroll
                            for (int jh = 0; jh < 2; ++jh)
                                wf[s][tl][jh] = *reinterpret_cast<const gate_f4*>(
                                    wb + (((((s * 4 + q) * NT + tl) * 2 + jh) * 16 + i16) * 4));
                    auto step = [&](auto J) {
                        constexpr int j = decltype(J)::value;
                        const float x0 = piece_get<j>(xb[u][0]), x1 = piece_get<j>(xb[u][1]);
#pragma unroll
                        for (int tl = 0; tl < NT; ++tl) {
                            acc[0][tl] = __builtin_amdgcn_mfma_f32_16x16x4f32(wf[0][tl][j / 4][j % 4], x0, acc[0][tl], 0, 0, 0);
                            acc[1][tl] = __builtin_amdgcn_mfma_f32_16x16x4f32(wf[1][tl][j / 4][j % 4], x1, acc[1][tl], 0, 0, 0);
                        }
                    };
                    step(std::integral_constant<int, 0>{}); step(std::integral_constant<int, 1>{});
                    step(std::integral_constant<int, 2>{}); step(std::integral_constant<int, 3>{});
                    step(std::integral_constant<int, 4>{}); step(std::integral_constant<int, 5>{});
                    step(std::integral_constant<int, 6>{}); step(std::integral_constant<int, 7>{});
                    if (p + 1 < npairs) store_w((p + 1) & 1, wreg[u]);
                    load_pair(p + NXP, xb[u]);
                    load_w(p + NXP + 1, wreg[u]);
                    __syncthreads();
                }
            }
        }

        // lane l, register r of tile tl: expert ec0 + 16 tl + 4q + r, token i16
#pragma unroll
        for (int tl = 0; tl < NT; ++tl)
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                const int e = ec0 + 16 * tl + 4 * q + r;
                if (e < E) {
                    const float v = (acc[0][tl][r] + acc[1][tl][r]) + bg[e];
                    if (ROUTE) logit_lds[(wave * 16 + i16) * e_pitch + e] = v;
                    else if (tok < T) logits[(size_t)tok * E + e] = v;
                }
            }
    }
    if (ROUTE) {
        __syncthreads();
        for (int i = lane; i < 16 * E; i += 64) {                 // the wave's 16 rows of logits are contiguous
            const int tk = i / E, e = i - tk * E;
            if (tok0w + tk < T) logits[(size_t)tok0w * E + i] = logit_lds[(wave * 16 + tk) * e_pitch + e];
        }
        route_four(logit_lds + (wave * 16 + (lane >> 2)) * e_pitch, lane & 3, tok0w + (lane >> 2), tok0w + (lane >> 2) < T, E, k, renorm, idx, wout);
    }
}

// ---- bf16 tokens, d % 64 == 0, every staged expert exists: the same contraction with both operands delivered by
// buffer loads that write LDS directly, so that nothing asynchronous ever targets a register and the waits can be
// written by hand (the compiler's own counts allow a third of the requests that may be outstanding).
// Per wave a ring of NXP token chunks (its 16 tokens x 64 columns, 2 KB: lane l's two 16-byte pieces at l * 16);
// per block a ring of NXP + 1 gate-matrix chunks (64 columns x 16 NT experts), every wave fetching a quarter.
// A gate-matrix piece (4 consecutive experts of one column) lands where the instruction that uses it finds the 64
// values of its lanes side by side: piece (block s, j, tile, q, i / 4) at 16 * ((((8 s + j) NT + tile) 4 + q) 4 + i / 4),
// so the A operand of instruction (s, j, tile) is one `ds_read_b32` at lane * 4 plus a constant.
typedef __attribute__((ext_vector_type(4))) int gate_rsrc_t;
#define GATE_LDS_PTR(T) __attribute__((address_space(3))) T*

__device__ __forceinline__ gate_rsrc_t gate_make_rsrc(const void* base, unsigned long long bytes)
{
    if (bytes > 0xffffffffull) bytes = 0xffffffffull;
    const unsigned long long b = (unsigned long long)base;
    gate_rsrc_t r;
    r[0] = (int)(unsigned)(b & 0xffffffffull);
    r[1] = (int)(unsigned)((b >> 32) & 0xffffull);
    r[2] = (int)(unsigned)bytes;                           // reads at or past this limit return zero
    r[3] = 0x00020000;
    return r;
}
__device__ __forceinline__ void gate_dma16(gate_rsrc_t r, uint32_t lds_base, uint32_t voff, uint32_t soff)
{
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tbuffer_load_dwordx4 %1, %2, %3 offen lds"
                 :: "s"(lds_base), "v"(voff), "s"(r), "s"(soff) : "memory");
}

constexpr int GATE_NXP = 5;                                // token chunks requested ahead
constexpr int GATE_NW = GATE_NXP + 1;                      // gate-matrix chunks in the ring
constexpr int GATE_XSLOT = 2048;                           // bytes of one wave's token chunk
constexpr int GATE_XRING = GATE_WAVES * GATE_NXP * GATE_XSLOT;

template <int NT, bool ROUTE>
__global__ __launch_bounds__(GATE_THREADS) void gate_mfma_dma_kernel(
    const bf16_t* __restrict__ X, const float* __restrict__ Wg, const float* __restrict__ bg,
    float* __restrict__ logits, int32_t* __restrict__ idx, float* __restrict__ wout,
    int T, int d, int E, int k, int renorm, int e_pitch)
{
    constexpr int NXP = GATE_NXP, NW = GATE_NW, XSLOT = GATE_XSLOT, XRING = GATE_XRING;
    constexpr int WCH = 4096 * NT;                         // bytes of one gate-matrix chunk
    constexpr int LPS = 2 + NT;                            // requests of one wave per chunk
    extern __shared__ __attribute__((aligned(1024))) unsigned char gsm[];   // token rings | gate-matrix ring | logits
    const uint32_t lds0 = (uint32_t)(uintptr_t)(GATE_LDS_PTR(unsigned char))gsm;
    float* logit_lds = reinterpret_cast<float*>(gsm + XRING + NW * WCH);

    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int q = lane >> 4, i16 = lane & 15;
    const int blk_tok0 = blockIdx.x * GATE_TOK;
    const int tok0w = blk_tok0 + wave * 16;
    const int tok = tok0w + i16;
    const int npairs = d / 64;

    // tokens: rows of this block onwards; a token past the end reads the last one (never stored); a chunk past the
    // end of a row reads into the next rows or, after the last row, zeros: never multiplied
    const gate_rsrc_t rX = gate_make_rsrc(X + (size_t)blk_tok0 * d, (unsigned long long)(T - blk_tok0) * d * 2);
    const int rowrel = (tok < T ? tok : T - 1) - blk_tok0;
    const uint32_t xv0 = (uint32_t)((rowrel * d + 8 * q) * 2), xv1 = xv0 + 64;
    const uint32_t xl_w = lds0 + (uint32_t)(wave * NXP * XSLOT);
    // gate matrix: this wave's NT requests of a chunk
    uint32_t wv[NT];
#pragma unroll
    for (int n = 0; n < NT; ++n) {
        const int L = (wave * NT + n) * 64 + lane;         // 16-byte slot of the chunk
        const int e4l = L & 3, qq = (L >> 2) & 3, tl = (L >> 4) % NT, sj = L / (16 * NT);
        const int c_local = 32 * (sj >> 3) + 8 * qq + (sj & 7);
        wv[n] = (uint32_t)((c_local * E + 16 * tl + 4 * e4l) * 4);
    }
    const uint32_t wl_w = lds0 + (uint32_t)(XRING + wave * NT * 1024);

    for (int ec0 = 0; ec0 < E; ec0 += 16 * NT) {
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");          // the stores of the previous pass do not count below
        // columns at or past d are at or past the limit: zeros
        const gate_rsrc_t rW = gate_make_rsrc(Wg + ec0, ((unsigned long long)d * E - ec0) * 4);
        auto issue = [&](int P, int xslot, int wstage) {
            gate_dma16(rX, xl_w + (uint32_t)(xslot * XSLOT), xv0, (uint32_t)P * 128u);
            gate_dma16(rX, xl_w + (uint32_t)(xslot * XSLOT + 1024), xv1, (uint32_t)P * 128u);
#pragma unroll
            for (int n = 0; n < NT; ++n)
                gate_dma16(rW, wl_w + (uint32_t)(wstage * WCH + n * 1024), wv[n], (uint32_t)P * (uint32_t)(64 * E * 4));
        };
        gate_f4 acc[2][NT];
#pragma unroll
        for (int s = 0; s < 2; ++s)
#pragma unroll
            for (int tl = 0; tl < NT; ++tl) acc[s][tl] = gate_f4{0.0f, 0.0f, 0.0f, 0.0f};

#pragma unroll
        for (int P = 0; P < NXP; ++P) issue(P, P, P);
        int xslot = 0, wstage = 0;
        for (int p = 0; p < npairs; ++p) {
            // this wave's requests for chunk p have landed (NXP - 1 younger groups may be pending); after the barrier
            // so have everybody's quarters of the gate-matrix chunk, and everybody is done with chunk p - 1
            asm volatile("s_waitcnt vmcnt(%0)" :: "n"((NXP - 1) * LPS) : "memory");
            asm volatile("s_barrier" ::: "memory");
            const unsigned char* xs = gsm + (wave * NXP + xslot) * XSLOT + lane * 16;
            const gate_u4 x0 = *reinterpret_cast<const gate_u4*>(xs);
            const gate_u4 x1 = *reinterpret_cast<const gate_u4*>(xs + 1024);
            const float* wsb = reinterpret_cast<const float*>(gsm + XRING + wstage * WCH) + lane;
            float wf[2][8][NT];
#pragma unroll
            for (int s = 0; s < 2; ++s)
#pragma unroll
                for (int j = 0; j < 8; ++j)
#pragma unroll
                    for (int tl = 0; tl < NT; ++tl) wf[s][j][tl] = wsb[((s * 8 + j) * NT + tl) * 64];
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                const uint32_t w0 = x0[j / 2], w1 = x1[j / 2];
                const float a0 = __uint_as_float((j & 1) ? (w0 & 0xffff0000u) : (w0 << 16));
                const float a1 = __uint_as_float((j & 1) ? (w1 & 0xffff0000u) : (w1 << 16));
#pragma unroll
                for (int tl = 0; tl < NT; ++tl) {
                    acc[0][tl] = __builtin_amdgcn_mfma_f32_16x16x4f32(wf[0][j][tl], a0, acc[0][tl], 0, 0, 0);
                    acc[1][tl] = __builtin_amdgcn_mfma_f32_16x16x4f32(wf[1][j][tl], a1, acc[1][tl], 0, 0, 0);
                }
            }
            // the reads of this chunk have returned before its slot is requested again
            asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
            issue(p + NXP, xslot, wstage == 0 ? NW - 1 : wstage - 1);
            xslot = (xslot + 1 == NXP) ? 0 : xslot + 1;
            wstage = (wstage + 1 == NW) ? 0 : wstage + 1;
        }
        // requests past the end are still on their way into the rings: nothing may reuse LDS before they land
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        __syncthreads();

        // lane l, register r of tile tl: expert ec0 + 16 tl + 4q + r, token i16
#pragma unroll
        for (int tl = 0; tl < NT; ++tl)
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                const int e = ec0 + 16 * tl + 4 * q + r;
                const float v = (acc[0][tl][r] + acc[1][tl][r]) + bg[e];
                if (ROUTE) logit_lds[(wave * 16 + i16) * e_pitch + e] = v;
                else if (tok < T) logits[(size_t)tok * E + e] = v;
            }
    }
    if (ROUTE) {
        __syncthreads();
        for (int i = lane; i < 16 * E; i += 64) {                 // the wave's 16 rows of logits are contiguous
            const int tk = i / E, e = i - tk * E;
            if (tok0w + tk < T) logits[(size_t)tok0w * E + i] = logit_lds[(wave * 16 + tk) * e_pitch + e];
        }
        route_four(logit_lds + (wave * 16 + (lane >> 2)) * e_pitch, lane & 3, tok0w + (lane >> 2), tok0w + (lane >> 2) < T, E, k, renorm, idx, wout);
    }
}

// Routing from logits in global memory (E > 64: the logits were written in passes).
__global__ void gate_route_kernel(const float* __restrict__ logits, int32_t* __restrict__ idx, float* __restrict__ wout,
                                  int T, int E, int k, int renorm)
{
    const int t = blockIdx.x * blockDim.x + threadIdx.x;
    if (t < T) route_one(logits + (size_t)t * E, t, E, k, renorm, idx, wout);
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

template <typename XT, int NT, int NXP, bool VEC, bool FULL, bool EVEN>
hipError_t run_gate(const moe_shape_t& s, const void* X, const float* Wg, const float* bg,
                    float* logits, int32_t* idx, float* w, hipStream_t st)
{
    const int grid = (s.T + GATE_TOK - 1) / GATE_TOK;
    if (s.E <= 16 * NT) {
        const int e_pitch = s.E | 1;
        const size_t dyn = (size_t)GATE_TOK * e_pitch * sizeof(float);
        hipLaunchKernelGGL((gate_mfma_kernel<XT, NT, NXP, true, VEC, FULL, EVEN>), dim3(grid), dim3(GATE_THREADS), dyn, st,
                           (const XT*)X, Wg, bg, logits, idx, w, s.T, s.d, s.E, s.k, s.renorm, e_pitch);
        return hipGetLastError();
    }
    hipLaunchKernelGGL((gate_mfma_kernel<XT, NT, NXP, false, VEC, FULL, EVEN>), dim3(grid), dim3(GATE_THREADS), 0, st,
                       (const XT*)X, Wg, bg, logits, idx, w, s.T, s.d, s.E, s.k, s.renorm, 0);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(gate_route_kernel, dim3((s.T + 255) / 256), dim3(256), 0, st, logits, idx, w, s.T, s.E, s.k, s.renorm);
    return hipGetLastError();
}

template <int NT>
hipError_t run_gate_dma(const moe_shape_t& s, const void* X, const float* Wg, const float* bg,
                        float* logits, int32_t* idx, float* w, hipStream_t st)
{
    const int grid = (s.T + GATE_TOK - 1) / GATE_TOK;
    const bool route = s.E <= 16 * NT;
    const int e_pitch = s.E | 1;
    const size_t lds = (size_t)GATE_XRING + (size_t)GATE_NW * 4096 * NT + (route ? (size_t)GATE_TOK * e_pitch * sizeof(float) : 0);
    auto kr = gate_mfma_dma_kernel<NT, true>;
    auto kn = gate_mfma_dma_kernel<NT, false>;
    static PerDeviceOnce once;                             // per instantiation
    const int dev = current_device();
    if (!once.is_done(dev)) {
        const int most = GATE_XRING + GATE_NW * 4096 * NT + GATE_TOK * (16 * NT + 1) * (int)sizeof(float);
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kr), hipFuncAttributeMaxDynamicSharedMemorySize, most);
        if (e == hipSuccess) e = hipFuncSetAttribute(reinterpret_cast<const void*>(kn), hipFuncAttributeMaxDynamicSharedMemorySize, most);
        if (e != hipSuccess) return e;
        once.mark(dev);
    }
    if (route) {
        hipLaunchKernelGGL(kr, dim3(grid), dim3(GATE_THREADS), lds, st, (const bf16_t*)X, Wg, bg, logits, idx, w,
                           s.T, s.d, s.E, s.k, s.renorm, e_pitch);
        return hipGetLastError();
    }
    hipLaunchKernelGGL(kn, dim3(grid), dim3(GATE_THREADS), lds, st, (const bf16_t*)X, Wg, bg, logits, idx, w,
                       s.T, s.d, s.E, s.k, s.renorm, 0);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(gate_route_kernel, dim3((s.T + 255) / 256), dim3(256), 0, st, logits, idx, w, s.T, s.E, s.k, s.renorm);
    return hipGetLastError();
}

template <typename XT, int NT, int NXP>
hipError_t run_gate_n(const moe_shape_t& s, const void* X, const float* Wg, const float* bg,
                      float* logits, int32_t* idx, float* w, hipStream_t st)
{
    // 16-byte requests need whole pieces inside the rows: E % 4 == 0 for the gate matrix, d % 4 == 0 for fp32
    // tokens (bf16 shapes have d % 64 == 0); other shapes take the same kernel with 4-byte requests.
    if (s.d % (64 * NXP) == 0 && s.E % (16 * NT) == 0) return run_gate<XT, NT, NXP, true, true, true>(s, X, Wg, bg, logits, idx, w, st);
    if (s.d % 64 == 0 && s.E % (16 * NT) == 0) return run_gate<XT, NT, NXP, true, true, false>(s, X, Wg, bg, logits, idx, w, st);
    if (s.E % 4 == 0 && s.d % 4 == 0) return run_gate<XT, NT, NXP, true, false, false>(s, X, Wg, bg, logits, idx, w, st);
    return run_gate<XT, NT, NXP, false, false, false>(s, X, Wg, bg, logits, idx, w, st);
}

template <typename XT>
hipError_t run_gate_t(const moe_shape_t& s, const void* X, const float* Wg, const float* bg,
                      float* logits, int32_t* idx, float* w, hipStream_t st)
{
    if (s.E <= 16) return run_gate_n<XT, 1, 8>(s, X, Wg, bg, logits, idx, w, st);
    if (s.E <= 32) return run_gate_n<XT, 2, 4>(s, X, Wg, bg, logits, idx, w, st);
    return run_gate_n<XT, 4, 4>(s, X, Wg, bg, logits, idx, w, st);
}

}  // namespace

hipError_t launch_gate_topk(const moe_shape_t& s, const void* X, const float* Wg, const float* bg,
                            float* logits, int32_t* idx, float* w, hipStream_t st)
{
    if (s.T == 0) return hipSuccess;
    if (s.dtype == MOE_F32) return run_gate_t<float>(s, X, Wg, bg, logits, idx, w, st);
    // rows of 64 tokens must stay inside the 32-bit offsets of a buffer load
    if (s.d % 64 == 0 && (long long)s.d * 2 * (GATE_TOK + 1) < (1ll << 31) && (long long)s.d * s.E * 4 < (1ll << 31)) {
        if (s.E == 16) return run_gate_dma<1>(s, X, Wg, bg, logits, idx, w, st);
        if (s.E == 32) return run_gate_dma<2>(s, X, Wg, bg, logits, idx, w, st);
        if (s.E % 64 == 0) return run_gate_dma<4>(s, X, Wg, bg, logits, idx, w, st);
    }
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

// Grouped expert FFN in bf16 with fp32 accumulation on the gfx950 matrix cores (Section 4.2 of
// the paper: forward and backward expert computation over the inputs a device hosts).
//
// Every contraction of the forward and backward pass is one launch of the same tiled kernel:
//   fwd1  Z(,U) = Xp W1(,W3)        epilogue: Z, U, Act = act(Z)(*U)
//   fwd2  Yp    = Act W2
//   bwd1  dA    = dYp W2^T          epilogue: dZ (,dU), Act recomputed from the saved Z (,U)
//   bwd2  dXp   = dZ W1^T (+ dU W3^T)
//   wgrad dW1 = Xp^T dZ, dW3 = Xp^T dU, dW2 = Act^T dYp over the rows of each group
// Groups are ragged and may be empty; row tiles start at the group's first row and the last one
// is masked, so nothing is padded to the largest load.  The kernel is persistent: one block per
// CU walks its share of the tiles, which it derives on the device from the group offsets (the
// host never reads the counts).
//
// Tiling: 256 x 256 output tile per block, 32-deep contraction slices moved from HBM/L2 straight
// into a 5-deep ring of LDS buffers by buffer loads (no register staging; rows outside a ragged
// group arrive as zeros because they lie past the end of the buffer resource), 32x32x16 bf16 MFMA
// with the accumulators in AGPRs.  An operand whose contraction index is contiguous in memory is
// kept row-major in LDS and read with 16-byte loads; one whose contraction index is the slow one
// is kept as it is and read with the transposing LDS load, so no operand is ever transposed in
// HBM.  Both layouts are XOR-swizzled so that fragment reads are free of bank conflicts.  Every
// request to L2 is a whole 128-byte line: a K-contiguous operand is therefore fetched two slices
// at a time for half of the tile's rows (128 rows x 64 steps per ring buffer), a K-major one a
// slice at a time (32 steps x 256 columns); the L2 channels, not HBM, are what the loop queues at
// when the same bytes are asked for in 64-byte pieces.  The MFMA
// is issued with the operands swapped, which leaves every lane with four consecutive output
// columns of one row.  The two rows of waves of a block alternate between fetching fragments and
// multiplying, half an iteration apart.
#include "internal.h"
#include <type_traits>

// Where the main loop starts relative to a 256-byte boundary of the code, in 4-byte steps.  The loop is one basic
// block that every wave runs tens of thousands of times; how its two phases fall into the instruction fetch
// windows changes the time of the weight-gradient contraction by 6 % from the best to the worst placement (period:
// 32 bytes) and of the others by 1-2 %, so the placement is fixed instead of being left to what precedes the loop.
#ifndef LOOP_OFF
#define LOOP_OFF 4
#endif
#define LOOP_OFF_STR2(x) #x
#define LOOP_OFF_STR1(x) LOOP_OFF_STR2(x)
#define LOOP_OFF_STR LOOP_OFF_STR1(LOOP_OFF)
#ifndef LOOP_OFF_P
#define LOOP_OFF_P 4
#endif
#define LOOP_OFF_P_STR LOOP_OFF_STR1(LOOP_OFF_P)

namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(8))) short s16x8;
typedef __attribute__((ext_vector_type(4))) short s16x4;
typedef __attribute__((ext_vector_type(16))) float f32x16;
#define LDS_PTR(T) __attribute__((address_space(3))) T*

enum Kind { KIND_NN = 0, KIND_NT = 1, KIND_TN = 2 };
enum Epi { EPI_BF16 = 0, EPI_F32 = 1, EPI_FWD1_GELU = 2, EPI_FWD1_SWIGLU = 3, EPI_BWD1_GELU = 4, EPI_BWD1_SWIGLU = 5 };

struct GemmParams {
    // contraction segments (bwd2 of SwiGLU has two: dZ W1^T + dU W3^T)
    const bf16_t* A[2];
    const bf16_t* B[2];
    const bf16_t* B_dual;        // fwd1 SwiGLU: second weight matrix read beside B[0]
    long lda, ldb;               // leading dimensions in elements
    long b_group_stride;         // elements between the weight matrices of consecutive groups (0 for TN)
    int n_seg, Kseg;             // NN/NT: contraction length per segment
    int Mout, N;                 // TN: output rows; all kinds: output columns
    const int32_t *slot_offsets, *dest_slots;
    int self, Gcap;
    int row_tiles, col_tiles;    // tile counts (row_tiles is an upper bound for NN/NT)
    int band;                    // row tiles per band of the tile walk (a round of 32 tiles is band x 32/band)
    int n_tiles;
    // outputs
    bf16_t *O0, *O1, *O2;        // EPI_BF16: O0.  FWD1: Z, U, Act.  BWD1: dZ, dU, Act
    float* OF;                   // EPI_F32
    int accumulate;              // EPI_F32: add to the output instead of overwriting it
    long ldo, o_group_stride;
    const bf16_t *Zin, *Uin;     // BWD1: saved pre-activations
    int write_act;               // BWD1: recompute the activation into O2 (0: the forward pass's copy is still there)
    float* split_ws;             // NN/NT: partial tiles of the K-split last round, [unit][wave][128 registers][64 lanes]
    int split_cap;               // units that fit there
};

// GELU (Eq. 2 with the Gaussian CDF) and its derivative from one exponential and one reciprocal: erf by the
// five-term rational approximation of Abramowitz & Stegun 7.1.26 (absolute error below 1.5e-7, two orders under
// what a bf16 output resolves), whose exp(-x^2) at x = z / sqrt(2) is also the density the derivative needs.  The
// library erff is some thirty instructions with branches, per element of an epilogue that the matrix cores wait for.
struct gelu_parts { float cdf, pdf; };                     // Phi(z) and phi(z)
__device__ __forceinline__ gelu_parts gelu_terms(float z)
{
    const float x = z * 0.70710678118654752f, ax = __builtin_fabsf(x);
    const float t = __builtin_amdgcn_rcpf(__builtin_fmaf(0.3275911f, ax, 1.0f));
    const float e = __expf(-(ax * ax));                    // exp(-z^2 / 2)
    float y = __builtin_fmaf(1.061405429f, t, -1.453152027f);
    y = __builtin_fmaf(y, t, 1.421413741f);
    y = __builtin_fmaf(y, t, -0.284496736f);
    y = __builtin_fmaf(y, t, 0.254829592f);
    const float half_erfc = 0.5f * (y * t) * e;            // (1 - erf|x|) / 2
    gelu_parts r;
    r.cdf = z < 0.0f ? half_erfc : 1.0f - half_erfc;
    r.pdf = 0.3989422804014327f * e;
    return r;
}
__device__ __forceinline__ float gelu_f(float z) { return z * gelu_terms(z).cdf; }
__device__ __forceinline__ float gelu_grad_f(float z) { const gelu_parts g = gelu_terms(z); return __builtin_fmaf(z, g.pdf, g.cdf); }
// exp and reciprocal are one instruction each (1 ulp); a full-precision division would be a dozen per element of an
// epilogue whose vector instructions are what the matrix cores wait for between two tiles
__device__ __forceinline__ float sigmoid_f(float z) { return __builtin_amdgcn_rcpf(1.0f + __expf(-z)); }

// Tile geometry: 256 x 256 outputs per block, 8 waves of 128 x 64, contraction slices of 32
// staged through a 5-deep ring of LDS buffers (16 KB per operand and buffer): all 160 KB of LDS.
constexpr int BM = 256, BN = 256, BK = 32, STAGES = 5;
// Row tiles per band of the tile walk, per contraction (measured at d = 4096, h = 14336, SwiGLU; see launch()).
#ifndef BAND_FWD1
#define BAND_FWD1 16
#endif
#ifndef BAND_FWD2
#define BAND_FWD2 8
#endif
#ifndef BAND_BWD1
#define BAND_BWD1 8
#endif
#ifndef BAND_BWD2
#define BAND_BWD2 8
#endif
#ifndef BAND_WGRAD
#define BAND_WGRAD 8
#endif
constexpr int WGM = 2, WGN = 4, NWAVES = WGM * WGN, NT = NWAVES * 64;
constexpr int WM = BM / WGM, WN = BN / WGN, TM = WM / 32, TN = WN / 32;
constexpr int PIECES = 16 / NWAVES;         // 1-KB DMA pieces per wave per 16-KB operand slice
constexpr uint32_t OPER_BYTES = 16384, STAGE_BYTES = 2 * OPER_BYTES;
constexpr int EP_PITCH = WN * 4 + 16;       // epilogue patch: bytes per staged row of WN floats (padded against bank conflicts)
constexpr int EP_ROWS = 32;               // rows a wave stages at a time: one row of fragments
constexpr int EP_WAVE = EP_ROWS * EP_PITCH;
constexpr size_t RING_BYTES = (size_t)STAGES * STAGE_BYTES;
constexpr size_t LDS_BYTES = RING_BYTES > (size_t)NWAVES * EP_WAVE ? RING_BYTES : (size_t)NWAVES * EP_WAVE;

// ---- LDS layouts (byte offsets inside one operand buffer) --------------------------------------
// K-contiguous operand (NN and NT fetch it in whole 128-byte lines): a buffer holds 128 rows x 64 steps (two
// slices of 32), 128 bytes per row, its eight 16-byte pieces XOR-swizzled by the row so that 16 consecutive rows of
// one piece cover all banks.
__device__ __forceinline__ uint32_t halfpair_off(int row, int piece8) { return row * 128 + ((piece8 ^ ((row >> 1) & 7)) << 4); }
// K-major operand: [32 steps][COLS columns]; 64-byte granules of a row XOR-swizzled by the step so
// that the four steps a transposing load touches fall into different banks.
template <int COLS>
__device__ __forceinline__ uint32_t kmajor_off(int krow, int col) { return krow * (COLS * 2) + ((((col >> 5) ^ (krow & 3))) << 6) + (col & 31) * 2; }

// Fragment = 32 rows (or columns) x 16 contraction steps; lane l holds row l%32, steps 8*(l/32)..+7.
// Fragment reads are issued as assembly and waited for by hand (WAIT_FRAGS below): the compiler's
// own wait insertion cannot express "the set loaded one iteration ago is complete" and would stall
// every MFMA group on the fragments that were only just requested for the next iteration.
template <int IMM>
__device__ __forceinline__ void lds_frag_kcontig_at(bf16x8& f, uint32_t addr)
{
    asm volatile("ds_read_b128 %0, %1 offset:%2" : "=v"(f) : "v"(addr), "n"(IMM));
}
// The transposing load works on blocks of 16 lanes: lane s of a block points at 4 consecutive columns
// of step s/4; lane i of the block receives column i of steps 0..3.  Two loads give the 8 steps of a
// lane in the same order as the K-contiguous fragment.  IMM: a constant distance added to the address.
template <int ROW4_BYTES, int IMM>
__device__ __forceinline__ void lds_frag_kmajor_at(bf16x8& f, uint32_t addr)
{
    s16x4 lo, hi;
    asm volatile("ds_read_b64_tr_b16 %0, %2 offset:%3\n\tds_read_b64_tr_b16 %1, %2 offset:%4"
                 : "=&v"(lo), "=&v"(hi) : "v"(addr), "n"(IMM), "n"(IMM + ROW4_BYTES));
    const s16x8 v = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
    f = __builtin_bit_cast(bf16x8, v);
}

typedef __attribute__((ext_vector_type(4))) int rsrc_t;     // raw buffer resource (4 scalar registers)
typedef __amdgpu_buffer_rsrc_t buf_rsrc_t;                   // the same thing as the store builtin wants it
typedef __attribute__((ext_vector_type(4))) unsigned u32x4;

__device__ __forceinline__ rsrc_t make_rsrc(const void* base, long long bytes)
{
    if (bytes < 0) bytes = 0;
    if (bytes > 0xffffffffll) bytes = 0xffffffffll;
    const unsigned long long b = (unsigned long long)base;
    rsrc_t r;
    r[0] = (int)(unsigned)(b & 0xffffffffull);
    r[1] = (int)(unsigned)((b >> 32) & 0xffffull);         // stride 0: raw buffer, byte offsets
    r[2] = (int)(unsigned)bytes;                           // bytes past this limit read as zero
    r[3] = 0x00020000;
    return r;
}

// 16 bytes per lane from a buffer straight into LDS at lds_base + lane*16 (lds_base is uniform and
// goes through M0); bytes past the end of the buffer arrive as zeros.  Issued as assembly so that
// the compiler does not serialise later LDS reads of other ring slots behind it; completion is
// tracked by hand with WAIT_VMCNT before the barrier that publishes the slot.
__device__ __forceinline__ void dma16(rsrc_t r, uint32_t lds_base, uint32_t voff, uint32_t soff)
{
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tbuffer_load_dwordx4 %1, %2, %3 offen lds"
                 :: "s"(lds_base), "v"(voff), "s"(r), "s"(soff) : "memory");
}

#define WAIT_VMCNT(n) asm volatile("s_waitcnt vmcnt(%0)" :: "n"(n) : "memory")
#define BLOCK_BARRIER() asm volatile("s_barrier" ::: "memory")


// ---- the kernel ---------------------------------------------------------------------------------
template <int KIND, int EPI, bool FIN>
__global__ __launch_bounds__(NT) void grouped_gemm_kernel(const GemmParams p)
{
    constexpr bool A_KMAJOR = (KIND == KIND_TN);
    constexpr bool B_KMAJOR = (KIND != KIND_NT);
    constexpr bool DUAL = (EPI == EPI_FWD1_SWIGLU);
    static_assert(!DUAL || (TN % 2 == 0), "dual-B needs an even number of column fragments per wave");

    extern __shared__ __attribute__((aligned(1024))) unsigned char smem[];
    const uint32_t lds0 = (uint32_t)(uintptr_t)(LDS_PTR(unsigned char))smem;

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm = wave / WGN, wn = wave % WGN;

    // ---- group table, once per block: lane i of every wave holds hosted group i (at most 64 groups)
    int first_slot, n_groups;
    hosted_range(p.dest_slots, p.self, p.Gcap, first_slot, n_groups);
    int g_row0 = 0, g_rows = 0;
    if (lane < n_groups) {
        g_row0 = p.slot_offsets[first_slot + lane];
        g_rows = p.slot_offsets[first_slot + lane + 1] - g_row0;
    }
    const int g_nt = (g_rows + BM - 1) / BM;               // row tiles of the group (NN/NT)
    int g_incl = g_nt;                                     // inclusive prefix over groups
#pragma unroll
    for (int off = 1; off < 64; off <<= 1) {
        const int up = __shfl_up(g_incl, off, 64);
        if (lane >= off) g_incl += up;
    }
    const int total_rt = __builtin_amdgcn_readlane(g_incl, 63);
    const int g_excl = g_incl - g_nt;

    // ---- which tiles.  The kernel is persistent: one block per CU walks its share of the tiles, so a
    // tile's stores drain under the next tile's loads and nothing is relaunched.  Blocks go round-robin
    // over the 8 XCDs (block b runs on XCD b % 8), each with its own L2.  The tiles that actually exist
    // (the counts are only known here) are cut into rounds of as many tiles as an XCD has blocks, 8 row
    // tiles by 4 column tiles walked column by column inside a band of 8 row tiles, so that the tiles in
    // flight on an XCD share operand slices in its L2; consecutive rounds go to the 8 XCDs in turn, so
    // that at any time the XCDs work on neighbouring rounds and what one of them has fetched from HBM
    // the others find in the memory-side cache.
    const int xcd = blockIdx.x & 7, q0 = blockIdx.x >> 3, q_stride = gridDim.x >> 3;
    const int BAND = p.band;
    const int tiles_g = p.row_tiles * p.col_tiles;         // TN: tiles of one group
    const int n_act = total_rt * p.col_tiles;              // NN/NT: tiles that exist
    const int rpg = (tiles_g + q_stride - 1) / q_stride;   // TN: rounds per group
    // NN/NT: the tiles left over after the last full round of the chip (fewer than there are blocks) are cut
    // along the contraction into S parts, each an item of its own, so that the last round keeps S times as
    // many blocks busy for 1/S of a tile's time.  A part leaves its accumulators in the workspace; a second
    // launch (FIN) adds the parts of a tile in a fixed order and runs the tile's epilogue.
    const int nblk = gridDim.x;
    const int n_full = (KIND == KIND_TN) ? 0 : (n_act / nblk) * nblk, rem = n_act - n_full;
    int S = 1;
    if (KIND != KIND_TN && rem > 0 && p.split_ws != nullptr) {
        S = min(4, nblk / rem);
        S = min(S, max(1, p.n_seg * (p.Kseg / BK) / 64));   // a part is worth its 256-KB round trip from 64 slices on
        if (rem * S > p.split_cap) S = 1;
    }
    if (FIN && S == 1) return;
    const int n_items = n_full + rem * S;
    const int n_rounds = (KIND == KIND_TN) ? p.Gcap * rpg : (n_items + q_stride - 1) / q_stride;
    const int q_first = FIN ? (int)blockIdx.x : q0;
    const int q_step = FIN ? nblk : q_stride;
    const int q_end = FIN ? rem : ((n_rounds + 7) >> 3) * q_stride;

  for (int q = q_first; q < q_end; q += q_step) {
    int g, rt, ct;
    int part = 0, parts = 1, unit = 0;                     // K-split: which part of how many, and where it is kept
    long a_row0, a_row_end;      // valid rows of the A tile (NN/NT) or of the contraction (TN)
    int k_tiles;
    int m0;                      // first output row of the tile (global row for NN/NT, row of dW for TN)
    if (KIND == KIND_TN) {
        // every group has the same tile grid but its own contraction length: a round never mixes
        // groups, so the blocks of an XCD stay on the same contraction slices of shared operands
        const int R = ((q - q0) / q_stride) * 8 + xcd;
        g = R / rpg;
        if (g >= p.Gcap) break;
        const int t = (R - g * rpg) * q_stride + q0;
        if (t >= tiles_g) continue;
        const int band = t / (BAND * p.col_tiles);
        const int in_band = t - band * BAND * p.col_tiles;
        const int band_rows = min(BAND, p.row_tiles - band * BAND);
        rt = band * BAND + in_band % band_rows;
        ct = in_band / band_rows;
        const int row0 = __builtin_amdgcn_readlane(g_row0, g & 63);       // empty for unused groups
        const int rows = __builtin_amdgcn_readlane(g_rows, g & 63);
        a_row0 = row0; a_row_end = row0 + rows;
        k_tiles = (rows + BK - 1) / BK;
        m0 = rt * BM;
    } else {
        int t;
        if (FIN) {
            t = n_full + q; parts = S; unit = q * S;
        } else {
            const int item = (((q - q0) / q_stride) * 8 + xcd) * q_stride + q0;
            if (item >= n_items) break;
            t = item;
            if (item >= n_full) { t = n_full + (item - n_full) / S; part = (item - n_full) % S; parts = S; unit = item - n_full; }
        }
        const int band = t / (BAND * p.col_tiles);
        const int in_band = t - band * BAND * p.col_tiles;
        const int band_rows = min(BAND, total_rt - band * BAND);
        rt = band * BAND + in_band % band_rows;
        ct = in_band / band_rows;
        g = __popcll(__ballot(g_incl <= rt)) & 63;                         // first group whose tiles reach past rt
        const int gr0 = __builtin_amdgcn_readlane(g_row0, g);
        const int row0 = gr0 + (rt - __builtin_amdgcn_readlane(g_excl, g)) * BM;
        const int row_end = gr0 + __builtin_amdgcn_readlane(g_rows, g);
        a_row0 = row0; a_row_end = row_end;
        k_tiles = p.n_seg * (p.Kseg / BK);
        m0 = row0;
    }
    const int n0 = ct * (DUAL ? BN / 2 : BN);             // first output column (hidden unit for dual)
    const int k_per_seg = (KIND == KIND_TN) ? k_tiles : p.Kseg / BK;
    // slices of this item: all of them, or one part of a split tile; none in the finishing launch
    // (a K-contiguous operand is fetched two slices at a time: parts begin at even slices)
    const int k_lo = (int)((long)part * k_tiles / parts) & ~1;
    const int k_hi = (part + 1 == parts) ? k_tiles : ((int)((long)(part + 1) * k_tiles / parts) & ~1);
    const int k_cnt = FIN ? 0 : k_hi - k_lo;

    // ---- buffer resources: everything outside the valid rows of an operand reads as zero --------
    // Each wave moves two 1-KB pieces of the A slice and two of the B slice per contraction slice.
    rsrc_t rA[2], rB[2];                   // per segment (A), per segment or per dual half (B)
    uint32_t voffA[2], voffB[2];                           // per-lane byte offsets of this wave's two pieces
    uint32_t ldsA[2], ldsB[2];                             // LDS byte offsets of the pieces inside a stage
    uint32_t stepA, stepB;                                 // byte advance of the source per slice
    const bf16_t *tn_baseA = nullptr, *tn_baseB = nullptr; // TN: where the current resources start, and how many
    long tn_bytesA = 0, tn_bytesB = 0;                     // bytes of the group's rows lie behind that point
    {
        const long a_rows = a_row_end - a_row0;
        if (KIND == KIND_TN) {
            tn_baseA = p.A[0] + a_row0 * p.lda + m0; tn_bytesA = (a_rows * p.lda - m0) * 2;
            tn_baseB = p.B[0] + a_row0 * p.ldb + n0; tn_bytesB = (a_rows * p.ldb - n0) * 2;
            rA[0] = rA[1] = make_rsrc(tn_baseA, tn_bytesA);
            rB[0] = rB[1] = make_rsrc(tn_baseB, tn_bytesB);
            stepA = (uint32_t)(BK * p.lda * 2);
            stepB = (uint32_t)(BK * p.ldb * 2);
        } else {
            for (int s = 0; s < 2; ++s) {
                const int ss = s < p.n_seg ? s : 0;
                rA[s] = make_rsrc(p.A[ss] + a_row0 * p.lda, a_rows * p.lda * 2);
            }
            stepA = BK * 2;
            const long gofs = (long)g * p.b_group_stride;
            if (KIND == KIND_NN) {
                rB[0] = make_rsrc(p.B[0] + gofs + n0, ((long)p.Kseg * p.ldb - n0) * 2);
                rB[1] = DUAL ? make_rsrc(p.B_dual + gofs + n0, ((long)p.Kseg * p.ldb - n0) * 2) : rB[0];
                stepB = (uint32_t)(BK * p.ldb * 2);
            } else {
                for (int s = 0; s < 2; ++s) {
                    const int ss = s < p.n_seg ? s : 0;
                    rB[s] = make_rsrc(p.B[ss] + gofs + (long)n0 * p.ldb, (long)(p.N - n0) * p.ldb * 2);
                }
                stepB = BK * 2;
            }
        }
#pragma unroll
        for (int i = 0; i < PIECES; ++i) {
            const int blk = wave + NWAVES * i;             // piece index inside a 16-KB operand buffer
            const int L = blk * 64 + lane;                 // 16-byte slot inside the buffer
            ldsA[i] = blk * 1024;
            if (A_KMAJOR) {
                const int krow = L >> 5, pp = L & 31, col = (((pp >> 2) ^ (krow & 3)) << 5) + (pp & 3) * 8;
                voffA[i] = (uint32_t)((krow * p.lda + col) * 2);
            } else {
                // a 1-KB piece is 8 rows x 128 bytes of a 128-row half: lane l reads piece l%8 of row l/8, where the
                // swizzle of the buffer puts it
                const int row = blk * 8 + (lane >> 3), piece = (lane & 7) ^ ((row >> 1) & 7);
                voffA[i] = (uint32_t)((row * p.lda + piece * 8) * 2);
            }
            if (!B_KMAJOR) {
                ldsB[i] = blk * 1024;
                const int row = blk * 8 + (lane >> 3), piece = (lane & 7) ^ ((row >> 1) & 7);
                voffB[i] = (uint32_t)((row * p.ldb + piece * 8) * 2);
            } else if (DUAL) {
                // two sub-buffers of [32][128] (8 pieces each); this wave's pieces alternate between them
                const int half = i & 1, blk2 = wave + NWAVES * (i >> 1);
                const int L2 = blk2 * 64 + lane;
                ldsB[i] = half * 8192 + blk2 * 1024;
                const int krow = L2 >> 4, pp = L2 & 15, col = (((pp >> 2) ^ (krow & 3)) << 5) + (pp & 3) * 8;
                voffB[i] = (uint32_t)((krow * p.ldb + col) * 2);
            } else {
                ldsB[i] = blk * 1024;
                const int krow = L >> 5, pp = L & 31, col = (((pp >> 2) ^ (krow & 3)) << 5) + (pp & 3) * 8;
                voffB[i] = (uint32_t)((krow * p.ldb + col) * 2);
            }
        }
    }

    // Slices are requested strictly in order; the source offsets advance with the stream.
    int iss_stage = 0;
    int iss_seg = (KIND == KIND_TN) ? 0 : k_lo / k_per_seg, iss_in_seg = (KIND == KIND_TN) ? 0 : k_lo - iss_seg * k_per_seg;
    uint32_t soffA = (uint32_t)iss_in_seg * stepA, soffB = (uint32_t)iss_in_seg * stepB;
    // The requests of one slice into stage iss_stage, with the resources the caller has picked: no decision in it.
    auto issue_with = [&](const rsrc_t ra, const rsrc_t rb0, const rsrc_t rb1) {
        const uint32_t st = lds0 + (uint32_t)iss_stage * STAGE_BYTES;
        iss_stage = (iss_stage + 1 == STAGES) ? 0 : iss_stage + 1;
#pragma unroll
        for (int i = 0; i < PIECES; ++i) dma16(ra, st + ldsA[i], voffA[i], soffA);
#pragma unroll
        for (int i = 0; i < PIECES; ++i) dma16((DUAL && (i & 1)) ? rb1 : rb0, st + OPER_BYTES + ldsB[i], voffB[i], soffB);
        ++iss_in_seg;
        soffA += stepA; soffB += stepB;
    };
    // What may have to change between two slices: the next contraction segment (NN/NT), or, for TN, whose offset
    // runs over all rows of the group, the base of the resources: buffer offsets are 32 bits, so the resources are
    // moved up to the current slice long before that overflows (a group of 2^31 bytes and more).
    auto issue_fixups = [&]() {
        if (KIND != KIND_TN && iss_in_seg == k_per_seg) { iss_in_seg = 0; ++iss_seg; soffA = 0; soffB = 0; }
        if (KIND == KIND_TN && ((soffA | soffB) & 0xc0000000u)) {
            tn_baseA += soffA / 2; tn_bytesA -= soffA; soffA = 0;
            tn_baseB += soffB / 2; tn_bytesB -= soffB; soffB = 0;
            rA[0] = rA[1] = make_rsrc(tn_baseA, tn_bytesA);
            rB[0] = rB[1] = make_rsrc(tn_baseB, tn_bytesB);
        }
    };
    auto issue_next = [&]() {                              // one slice, strictly in order
        issue_with(iss_seg ? rA[1] : rA[0], (KIND == KIND_NT && iss_seg) ? rB[1] : rB[0], rB[1]);
        issue_fixups();
    };
    // how many slices can be requested from here without a fixup in between (at least one)
    auto issue_run = [&]() -> int {
        if (KIND != KIND_TN) return k_per_seg - iss_in_seg;
        const uint32_t hi = soffA > soffB ? soffA : soffB, st = stepA > stepB ? stepA : stepB;
        return (int)((0x3fffffffu - hi) / st) + 1;
    };

    // NN and NT fetch their K-contiguous operands in whole 128-byte lines: a request group carries, for such an
    // operand, 128 rows x 64 steps (two slices) instead of 256 rows x 32 steps: group n holds the upper (n even) or
    // lower (n odd) 128 rows of the tile for slices 2 (n / 2) and 2 (n / 2) + 1.  Same bytes and same number of
    // instructions per group as a slice, half as many requests to L2.  A K-major operand (the weights of NN) keeps
    // one slice per group.  PAR: the parity of the group, known where the loop is written out.
    constexpr bool A_PAIR = !A_KMAJOR, B_PAIR = !B_KMAJOR;
    const uint32_t halfA = (uint32_t)(128 * p.lda * 2), halfB = (uint32_t)(128 * p.ldb * 2);   // to the lower 128 rows
    auto issue_group = [&](auto PAR, const rsrc_t ra, const rsrc_t rb0, const rsrc_t rb1) {
        constexpr int par = decltype(PAR)::value;
        const uint32_t st = lds0 + (uint32_t)iss_stage * STAGE_BYTES;
        iss_stage = (iss_stage + 1 == STAGES) ? 0 : iss_stage + 1;
        const uint32_t oa = (A_PAIR && par) ? soffA + halfA : soffA;
        const uint32_t ob = (B_PAIR && par) ? soffB + halfB : soffB;
#pragma unroll
        for (int i = 0; i < PIECES; ++i) dma16(ra, st + ldsA[i], voffA[i], oa);
#pragma unroll
        for (int i = 0; i < PIECES; ++i) dma16((DUAL && (i & 1)) ? rb1 : rb0, st + OPER_BYTES + ldsB[i], voffB[i], ob);
        ++iss_in_seg;
        if (!A_PAIR || par) soffA += A_PAIR ? 2 * stepA : stepA;
        if (!B_PAIR || par) soffB += B_PAIR ? 2 * stepB : stepB;
    };
    // after an odd group (segments hold an even number of slices): the next contraction segment
    auto group_fixups = [&]() {
        if (iss_in_seg == k_per_seg) { iss_in_seg = 0; ++iss_seg; soffA = 0; soffB = 0; }
    };

    // ---- per-lane fragment addresses inside a ring buffer.  The buffer's base is the only part of a fragment
    // address that changes from slice to slice, and every vector instruction of the fetching wave takes an issue
    // slot from the matrix instructions of its partner: fragments that lie a constant distance apart share one
    // address register and differ in the instruction's immediate offset.
    static_assert(TM == 4 && TN == 2, "the fragment reads below are written out for 4 x 2 fragments");
    // K-major operands (step half 0; half 1 is 16 steps further down)
    uint32_t fa_addr[TM], fb_addr[TN];
    constexpr uint32_t A_HALF = 16 * (BM * 2);
    constexpr int BCOLS = DUAL ? BN / 2 : BN;
    constexpr uint32_t B_HALF = 16 * (BCOLS * 2);
#pragma unroll
    for (int i = 0; i < TM; ++i) {
        const int b = lane >> 4, s = lane & 15;
        fa_addr[i] = kmajor_off<BM>(8 * (b >> 1) + (s >> 2), wm * WM + i * 32 + 16 * (b & 1) + 4 * (s & 3));
    }
#pragma unroll
    for (int j = 0; j < TN; ++j) {
        const int b = lane >> 4, s = lane & 15;
        const int krow = 8 * (b >> 1) + (s >> 2), cofs = 16 * (b & 1) + 4 * (s & 3);
        if (DUAL)   // even fragments from the W1 sub-buffer, odd ones from the W3 sub-buffer
            fb_addr[j] = OPER_BYTES + (j & 1) * 8192 + kmajor_off<BN / 2>(krow, wn * (WN / 2) + (j >> 1) * 32 + cofs);
        else
            fb_addr[j] = OPER_BYTES + kmajor_off<BN>(krow, wn * WN + j * 32 + cofs);
    }
    // TN: both operands K-major, a slice per ring buffer
    auto load_frags = [&](bf16x8 (&fa)[TM], bf16x8 (&fb)[TN], int stage, auto HALF) {
        constexpr int half = decltype(HALF)::value;
        const uint32_t st = lds0 + (uint32_t)stage * STAGE_BYTES;
#pragma unroll
        for (int i = 0; i < TM; ++i) lds_frag_kmajor_at<4 * BM * 2, half * (int)A_HALF>(fa[i], st + fa_addr[i]);
#pragma unroll
        for (int j = 0; j < TN; ++j) lds_frag_kmajor_at<4 * BCOLS * 2, half * (int)B_HALF>(fb[j], st + fb_addr[j]);
    };
    // Operands fetched in 128-byte lines: fragment 0 of this wave in a 128-row buffer, at the four quarters (16
    // steps each) of the buffer's two slices; the wave's other fragments lie 32 rows = 4 KB further on.  The upper
    // row of waves (A) and the waves of the two left columns (B) read the buffer of an even group, the others that
    // of the odd group after it.
    uint32_t fpa[4], fpb[4];
#pragma unroll
    for (int v = 0; v < 4; ++v) {
        fpa[v] = halfpair_off(lane & 31, lane >> 5) ^ (uint32_t)(v << 5);
        fpb[v] = OPER_BYTES + (halfpair_off((wn & 1) * 64 + (lane & 31), lane >> 5) ^ (uint32_t)(v << 5));
    }
    auto load_group_frags = [&](bf16x8 (&fa)[TM], bf16x8 (&fb)[TN], uint32_t stA, uint32_t stB, auto Q) {
        constexpr int quarter = decltype(Q)::value;        // 2 * (slice of the pair) + (16-step half of the slice)
        {
            const uint32_t a = stA + fpa[quarter];
            lds_frag_kcontig_at<0>(fa[0], a);
            lds_frag_kcontig_at<4096>(fa[1], a);
            lds_frag_kcontig_at<8192>(fa[2], a);
            lds_frag_kcontig_at<12288>(fa[3], a);
        }
        if constexpr (B_KMAJOR) {                          // stB: the buffer of the slice
#pragma unroll
            for (int j = 0; j < TN; ++j) lds_frag_kmajor_at<4 * BCOLS * 2, (quarter & 1) * (int)B_HALF>(fb[j], stB + fb_addr[j]);
        } else {
            const uint32_t bb = stB + fpb[quarter];
            lds_frag_kcontig_at<0>(fb[0], bb);
            lds_frag_kcontig_at<4096>(fb[1], bb);
        }
    };
    auto wait_frags = [&]() {
        __builtin_amdgcn_sched_barrier(0);
        asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
        __builtin_amdgcn_sched_barrier(0);                 // no MFMA moves above the wait
    };

    // NN and NT start their accumulators with the first products of slice 0 (a matrix instruction that takes zero
    // as its addend) instead of clearing 128 registers per tile; TN, whose groups may be empty, clears them.
    f32x16 acc[TM][TN];
    if (KIND == KIND_TN || FIN) {
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int j = 0; j < TN; ++j)
#pragma unroll
                for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.0f;
    }

    // the TM*TN products of one 16-step.  The accumulators are pinned to AGPRs, which leaves the
    // VGPRs of the wave to fragments and addresses.
    auto mma = [&](const bf16x8 (&fa)[TM], const bf16x8 (&fb)[TN]) {
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int j = 0; j < TN; ++j)
                asm volatile("v_mfma_f32_32x32x16_bf16 %0, %1, %2, %0" : "+a"(acc[i][j]) : "v"(fb[j]), "v"(fa[i]));
    };

    // ---- main loop, two phases per slice.  In its fetch phase a wave reads the fragments of slice t
    // from LDS and requests its share of what lies three or four slices ahead; one barrier later, in its multiply phase, it issues
    // the 16 MFMAs of the slice back to back.  The upper row of waves runs one barrier interval behind
    // the lower one; waves w and w+4 share a SIMD, so while one of them feeds the matrix pipe the other
    // collects its operands.  With LDS reads and MFMAs alone this loop runs at the MFMA rate; what it
    // waits for in practice is the delivery of the slices from L2/HBM.  All fragment reads are issued
    // before the DMA requests so that a request held up by the memory system never delays them (a
    // request placed between MFMAs stalls the matrix pipe for several MFMA slots instead).
    static_assert(WGN == 4 && PIECES == 2, "the loop is written for 8 waves");
    if (!FIN && k_cnt > 0) {
      if constexpr (KIND == KIND_TN) {
        bf16x8 fa0[TM], fb0[TN], fa1[TM], fb1[TN];
        constexpr int L = STAGES - 1;                      // slices requested ahead
        constexpr int SLICE_OPS = 2 * PIECES;              // DMA instructions of one wave per slice
        // Every slice t is preceded by exactly t + L request groups of this wave (the prologue issues L of them,
        // every slice one more), so "my pieces of slice t + 1 have landed" is always "at most L - 1 groups are still
        // on their way": one fixed wait count for the whole contraction.  Where there is no slice left to request
        // (a contraction shorter than the lookahead, and the last L slices of any contraction) the group goes to a
        // resource of zero length: nothing is read, zeros land in a ring slot that nobody reads again.
        const rsrc_t rnull = make_rsrc(p.A[0], 0);
#pragma unroll
        for (int i = 0; i < L; ++i) {
            if (i < k_cnt) issue_next(); else issue_with(rnull, rnull, rnull);
        }
        WAIT_VMCNT((L - 1) * SLICE_OPS);                   // slice 0 has landed
        BLOCK_BARRIER();
        if (wm == 1) BLOCK_BARRIER();
        int cur = 0;
        asm volatile(".p2align 8\n\t.rept " LOOP_OFF_STR "\n\ts_nop 0\n\t.endr" ::: "memory");
        // One slice: fetch phase (fragments of slice t, then the requests for slice t + L, then the wait for this
        // wave's pieces of slice t + 1), barrier, multiply phase, barrier.  Ring slot (t+4) % 5 held slice t-1,
        // which every wave finished reading at least one barrier ago.  The loop has no decision in it: it runs
        // over stretches of slices that need no fixup between their requests (a whole contraction segment, or
        // all of a group's rows short of 2^30 bytes) with the resources of the stretch.
        int t = 0;
        while (t < k_cnt) {
            const bool more = t + L < k_cnt;               // slices left to request
            const int n = more ? min(k_cnt - L - t, issue_run()) : k_cnt - t;
            const rsrc_t ra = more ? (iss_seg ? rA[1] : rA[0]) : rnull;
            const rsrc_t rb0 = more ? ((KIND == KIND_NT && iss_seg) ? rB[1] : rB[0]) : rnull;
            const rsrc_t rb1 = more ? rB[1] : rnull;
            for (int i = 0; i < n; ++i) {
                load_frags(fa0, fb0, cur, std::integral_constant<int, 0>{});
                load_frags(fa1, fb1, cur, std::integral_constant<int, 1>{});
                __builtin_amdgcn_sched_barrier(0);
                issue_with(ra, rb0, rb1);
                WAIT_VMCNT((L - 1) * SLICE_OPS);
                wait_frags();
                BLOCK_BARRIER();
                __builtin_amdgcn_s_setprio(1);
                mma(fa0, fb0);
                mma(fa1, fb1);
                __builtin_amdgcn_s_setprio(0);
                __builtin_amdgcn_sched_barrier(0);
                BLOCK_BARRIER();
                cur = (cur + 1 == STAGES) ? 0 : cur + 1;
            }
            t += n;
            if (more) issue_fixups();
        }
        WAIT_VMCNT(0);                                     // the zero-length requests too: the epilogue reuses the ring
        if (wm == 0) BLOCK_BARRIER();                      // both rows have passed the same number of barriers
        BLOCK_BARRIER();                                   // and everybody's requests have landed
      } else {
        bf16x8 fa0[TM], fb0[TN], fa1[TM], fb1[TN];
        // NN and NT.  One request group per slice, three ahead: before slice t come the groups 0 .. t + 2, slice t adds
        // group t + 3 into ring slot (t + 3) % 5, which held group t - 2, last read in slice t - 1.  Slice 2p and 2p + 1
        // read the K-contiguous operands from the buffers of the groups 2p (upper 128 rows) and 2p + 1 (lower 128
        // rows), a K-major operand from the buffer of the slice's own group.  What a slice waits for before its
        // barrier is the data of the next slice: after an even slice the K-major operand's group t + 1 (two groups
        // may still be on their way), after an odd slice the groups t + 1 and t + 2 of the next pair (one group may).
        // Contractions have an even number of slices (d and h are multiples of 64; split parts begin at even slices),
        // so the loop is written out for pairs: slice 0, then pairs of an odd and an even slice, whose two groups are
        // the two halves of one later pair of slices and need no fixup between them, then the last slice.
        constexpr int L = 3;
        constexpr int SLICE_OPS = 2 * PIECES;              // DMA instructions of one wave per group
        const rsrc_t rnull = make_rsrc(p.A[0], 0);
        auto real_a = [&]() { return iss_seg ? rA[1] : rA[0]; };
        auto real_b0 = [&]() { return (KIND == KIND_NT && iss_seg) ? rB[1] : rB[0]; };
        // groups 0, 1, 2: a contraction has at least two slices
        issue_group(std::integral_constant<int, 0>{}, real_a(), real_b0(), rB[1]);
        issue_group(std::integral_constant<int, 1>{}, real_a(), real_b0(), rB[1]);
        group_fixups();
        if (k_cnt > 2) issue_group(std::integral_constant<int, 0>{}, real_a(), real_b0(), rB[1]);
        else issue_group(std::integral_constant<int, 0>{}, rnull, rnull, rnull);
        WAIT_VMCNT(SLICE_OPS);                             // groups 0 and 1 have landed: slices 0 and 1
        BLOCK_BARRIER();
        if (wm == 1) BLOCK_BARRIER();
        int cur = 0;                                       // ring slot of the slice's own group
        int pair0 = 0;                                     // ring slot of the even group of the slice's pair
        const int hA = wm, hB = wn >> 1;                   // which group of a pair holds this wave's rows of A and B
        auto slot_base = [&](int slot) { return lds0 + (uint32_t)(slot >= STAGES ? slot - STAGES : slot) * STAGE_BYTES; };
        // One slice of parity PAR; ra .. rb1: the resources of the group it requests (of the opposite parity).
        auto mma_first = [&](const bf16x8 (&fa)[TM], const bf16x8 (&fb)[TN]) {      // acc = products (+ 0)
#pragma unroll
            for (int i = 0; i < TM; ++i)
#pragma unroll
                for (int j = 0; j < TN; ++j)
                    asm volatile("v_mfma_f32_32x32x16_bf16 %0, %1, %2, 0" : "=a"(acc[i][j]) : "v"(fb[j]), "v"(fa[i]));
        };
        auto slice = [&](auto PAR, auto FIRST, const rsrc_t ra, const rsrc_t rb0, const rsrc_t rb1) {
            constexpr int par = decltype(PAR)::value;
            const uint32_t stA = slot_base(pair0 + hA);
            const uint32_t stB = B_KMAJOR ? slot_base(cur) : slot_base(pair0 + hB);
            load_group_frags(fa0, fb0, stA, stB, std::integral_constant<int, 2 * par>{});
            load_group_frags(fa1, fb1, stA, stB, std::integral_constant<int, 2 * par + 1>{});
            __builtin_amdgcn_sched_barrier(0);
            issue_group(std::integral_constant<int, 1 - par>{}, ra, rb0, rb1);
            WAIT_VMCNT(par ? SLICE_OPS : 2 * SLICE_OPS);
            wait_frags();
            BLOCK_BARRIER();
            __builtin_amdgcn_s_setprio(1);
            if constexpr (decltype(FIRST)::value) mma_first(fa0, fb0); else mma(fa0, fb0);
            mma(fa1, fb1);
            __builtin_amdgcn_s_setprio(0);
            __builtin_amdgcn_sched_barrier(0);
            BLOCK_BARRIER();
            cur = (cur + 1 == STAGES) ? 0 : cur + 1;
            if (par) pair0 = (pair0 + 2 >= STAGES) ? pair0 + 2 - STAGES : pair0 + 2;
        };
        // slice 0 requests group 3, the lower rows of slices 2 and 3
        if (k_cnt > 2) { slice(std::integral_constant<int, 0>{}, std::true_type{}, real_a(), real_b0(), rB[1]); group_fixups(); }
        else slice(std::integral_constant<int, 0>{}, std::true_type{}, rnull, rnull, rnull);
        asm volatile(".p2align 8\n\t.rept " LOOP_OFF_P_STR "\n\ts_nop 0\n\t.endr" ::: "memory");
        // slices 2i + 1 and 2i + 2 request the groups 2i + 4 and 2i + 5: slices 2i + 4 and 2i + 5, if there are any
        int t = 1;
        while (t < k_cnt - 1) {
            const bool more = t + L < k_cnt;               // the pair of slices t + 3, t + 4 exists
            const int n = more ? min((k_cnt - L - t + 1) / 2, (k_per_seg - iss_in_seg) / 2) : (k_cnt - 1 - t) / 2;
            const rsrc_t ra = more ? real_a() : rnull;
            const rsrc_t rb0 = more ? real_b0() : rnull;
            const rsrc_t rb1 = more ? rB[1] : rnull;
            for (int i = 0; i < n; ++i) {
                slice(std::integral_constant<int, 1>{}, std::false_type{}, ra, rb0, rb1);
                slice(std::integral_constant<int, 0>{}, std::false_type{}, ra, rb0, rb1);
            }
            t += 2 * n;
            if (more) group_fixups();
        }
        slice(std::integral_constant<int, 1>{}, std::false_type{}, rnull, rnull, rnull);      // the last slice
        WAIT_VMCNT(0);                                     // the zero-length requests too: the epilogue reuses the ring
        if (wm == 0) BLOCK_BARRIER();                      // both rows have passed the same number of barriers
        BLOCK_BARRIER();                                   // and everybody's requests have landed
      }
    }

    asm volatile("s_nop 15\n\ts_nop 15" ::: "memory");     // the last MFMAs have written back before the accumulators are read
    // partial tiles: [unit][wave][register / 4][lane] as float4, every instruction moves 1 KB
    if (KIND != KIND_TN && !FIN && parts > 1) {
        float4* ws4 = reinterpret_cast<float4*>(p.split_ws) + ((size_t)unit * NWAVES + wave) * (TM * TN * 4) * 64 + lane;
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int j = 0; j < TN; ++j) {
#pragma unroll
                for (int e4 = 0; e4 < 4; ++e4)
                    ws4[((i * TN + j) * 4 + e4) * 64] = make_float4(acc[i][j][e4 * 4], acc[i][j][e4 * 4 + 1], acc[i][j][e4 * 4 + 2], acc[i][j][e4 * 4 + 3]);
                __builtin_amdgcn_sched_barrier(0);
            }
        __syncthreads();
        continue;
    }
    // ---- epilogue.  A lane holds, per fragment, row l%32 and columns q*8 + (l/32)*4 + 0..3: storing
    // from there would touch 16-byte pieces of 32 different rows per instruction.  Instead every wave
    // passes its 128 x 64 accumulators through its own LDS patch (one row of fragments, 32 rows, at a time,
    // fp32) and reads them back row-major, 8 consecutive columns per lane, so that global loads and stores
    // move whole 128/256-byte row segments.  The patches lie at the top of LDS, above ring slots 0 and 1.
    unsigned char* patch = smem + (LDS_BYTES - (size_t)NWAVES * EP_WAVE) + wave * EP_WAVE;
    const int lrow = lane & 31, lcol = (lane >> 5) * 4;
    const long row_limit = (KIND == KIND_TN) ? (long)p.Mout : a_row_end;
    constexpr int CG = DUAL ? WN / 16 : WN / 8;            // 8-column groups per staged row that carry outputs
    const int erow = lane / CG, ecg = lane % CG;
    constexpr int ROWS_PER_PASS = 64 / CG;
    constexpr bool BWD1 = (EPI == EPI_BWD1_GELU || EPI == EPI_BWD1_SWIGLU);
    constexpr int N_PASS = EP_ROWS / ROWS_PER_PASS;        // passes per staged row of fragments
    // NN/NT: every store of the epilogue is issued whatever the tile looks like, as a buffer store whose resource
    // ends with the tile's last valid row (or has no length at all, for an output that is not written): the number
    // of memory instructions of an epilogue is then a constant of the instantiation, which the waits for the next
    // tile's first slices count on (see the main loop).  TN keeps ordinary predicated stores.
    constexpr bool UNCOND = (KIND != KIND_TN);
    const int wcol0 = n0 + (DUAL ? wn * (WN / 2) : wn * WN);           // first column of this wave: all of its columns exist or none
    buf_rsrc_t rO0 = buf_rsrc_t(), rO1 = buf_rsrc_t(), rO2 = buf_rsrc_t();
    if (UNCOND) {
        const bool cols = wcol0 < p.N;
        const long vrows = row_limit - m0 < BM ? row_limit - m0 : BM;       // the group may go on for millions of rows
        const int bytes = (int)(vrows * p.ldo * 2);
        auto out_rsrc = [&](bf16_t* base, bool on) {
            return __builtin_amdgcn_make_buffer_rsrc((void*)(base ? base + (long)m0 * p.ldo : p.O2), 0, (on && base && cols) ? bytes : 0, 0x00020000);
        };
        rO0 = out_rsrc(p.O0, true);
        rO1 = out_rsrc(p.O1, EPI == EPI_FWD1_SWIGLU || EPI == EPI_BWD1_SWIGLU);
        rO2 = out_rsrc(p.O2, BWD1 ? p.write_act != 0 : (EPI == EPI_FWD1_GELU || EPI == EPI_FWD1_SWIGLU));
    }
    // The saved pre-activations of the backward epilogue are requested a batch of passes ahead, into the second
    // of two register sets: a batch's loads are in flight while the batch before it is computed and stored, and,
    // memory operations completing in the order of issue, no load ever waits for a store issued before it.
#ifndef BWD1_BATCH
#define BWD1_BATCH 2
#endif
    constexpr int BATCH = BWD1 ? BWD1_BATCH : N_PASS;
    constexpr int NB = N_PASS / BATCH;                     // batches per staged row of fragments
    static_assert(N_PASS % BATCH == 0, "batches tile the passes of a staged row of fragments");
    uint4 zin[BWD1 ? 2 : 1][BWD1 ? BATCH : 1], uin[EPI == EPI_BWD1_SWIGLU ? 2 : 1][EPI == EPI_BWD1_SWIGLU ? BATCH : 1];
    auto request = [&](int fr, int pb, uint4* zi, uint4* ui) {
#pragma unroll
        for (int k = 0; k < BATCH; ++k) {
            // rows and columns past the end read the last valid ones (their results are not stored): no
            // predicate, no zero fill
            long row = (long)m0 + wm * WM + fr * EP_ROWS + (pb + k) * ROWS_PER_PASS + erow;
            row = row < row_limit ? row : row_limit - 1;
            const int col = min(n0 + wn * WN + ecg * 8, p.N - 8);
            zi[k] = *reinterpret_cast<const uint4*>(p.Zin + row * p.ldo + col);
            if (EPI == EPI_BWD1_SWIGLU) ui[k] = *reinterpret_cast<const uint4*>(p.Uin + row * p.ldo + col);
        }
    };
    if (BWD1) request(0, 0, zin[0], uin[0]);
#pragma unroll
    for (int fr = 0; fr < TM; ++fr) {
        asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
        __builtin_amdgcn_wave_barrier();
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const f32x16& a = acc[fr][j];
                float4 val = make_float4(a[q * 4 + 0], a[q * 4 + 1], a[q * 4 + 2], a[q * 4 + 3]);
                if (KIND != KIND_TN && FIN) {                  // the parts of a split tile, added in ascending order
                    const float4* ws4 = reinterpret_cast<const float4*>(p.split_ws) + ((size_t)unit * NWAVES + wave) * (TM * TN * 4) * 64 + lane;
                    float4 v[4];                               // at most 4 parts; all loads independent of each other
#pragma unroll
                    for (int s = 0; s < 4; ++s)
                        v[s] = (s < parts) ? ws4[(size_t)s * NWAVES * (TM * TN * 4) * 64 + ((fr * TN + j) * 4 + q) * 64]
                                           : make_float4(0.0f, 0.0f, 0.0f, 0.0f);
                    val = v[0];
#pragma unroll
                    for (int s = 1; s < 4; ++s) { val.x += v[s].x; val.y += v[s].y; val.z += v[s].z; val.w += v[s].w; }
                }
                *reinterpret_cast<float4*>(patch + lrow * EP_PITCH + (j * 32 + q * 8 + lcol) * 4) = val;
            }
        asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
        __builtin_amdgcn_wave_barrier();
#pragma unroll
        for (int b = 0; b < NB; ++b) {
        const int pb = b * BATCH, cur = (fr * NB + b) & 1;
        if (BWD1) {
            const int nxt = fr * NB + b + 1;
            if (nxt < TM * NB) request(nxt / NB, (nxt % NB) * BATCH, zin[cur ^ 1], uin[cur ^ 1]);
        }
#pragma unroll
        for (int pass = pb; pass < pb + BATCH; ++pass) {
            const int r = pass * ROWS_PER_PASS + erow;                     // row inside the patch
            const int trow = wm * WM + fr * EP_ROWS + r;                   // row inside the tile
            const long row = (long)m0 + trow;
            const int col = wcol0 + ecg * 8;
            if (!UNCOND && (row >= row_limit || col >= p.N)) continue;
            float v[8], u[8];
            {
                // dual: fragments alternate x W1 / x W3, 32 columns each; group ecg sits in pair ecg/4
                const int c0 = DUAL ? ((ecg >> 2) * 64 + (ecg & 3) * 8) * 4 : ecg * 32;
                const float4 x0 = *reinterpret_cast<const float4*>(patch + r * EP_PITCH + c0);
                const float4 x1 = *reinterpret_cast<const float4*>(patch + r * EP_PITCH + c0 + 16);
                v[0] = x0.x; v[1] = x0.y; v[2] = x0.z; v[3] = x0.w; v[4] = x1.x; v[5] = x1.y; v[6] = x1.z; v[7] = x1.w;
            }
            if (DUAL) {                                                    // the next 32 columns of the patch hold x W3
                const int c1 = ((ecg >> 2) * 64 + 32 + (ecg & 3) * 8) * 4;
                const float4 x0 = *reinterpret_cast<const float4*>(patch + r * EP_PITCH + c1);
                const float4 x1 = *reinterpret_cast<const float4*>(patch + r * EP_PITCH + c1 + 16);
                u[0] = x0.x; u[1] = x0.y; u[2] = x0.z; u[3] = x0.w; u[4] = x1.x; u[5] = x1.y; u[6] = x1.z; u[7] = x1.w;
            }
            const long o = row * p.ldo + col;
            const int bo = (int)(((long)trow * p.ldo + col) * 2);          // byte offset from the tile's first row
            auto pack8 = [](const float* f) {
                return make_uint4(pack_bf16x2(f[0], f[1]), pack_bf16x2(f[2], f[3]), pack_bf16x2(f[4], f[5]), pack_bf16x2(f[6], f[7]));
            };
            auto unpack8 = [](const uint4 w, float* f) {
                f[0] = __uint_as_float(w.x << 16); f[1] = __uint_as_float(w.x & 0xffff0000u);
                f[2] = __uint_as_float(w.y << 16); f[3] = __uint_as_float(w.y & 0xffff0000u);
                f[4] = __uint_as_float(w.z << 16); f[5] = __uint_as_float(w.z & 0xffff0000u);
                f[6] = __uint_as_float(w.w << 16); f[7] = __uint_as_float(w.w & 0xffff0000u);
            };
            auto put = [&](buf_rsrc_t r, const uint4 w) {      // rows past the tile's last one fall outside the resource
                __builtin_amdgcn_raw_buffer_store_b128(__builtin_bit_cast(u32x4, w), r, bo, 0, 0);
            };
            if (EPI == EPI_BF16) {
                put(rO0, pack8(v));
            } else if (EPI == EPI_F32) {
                float* dst = p.OF + (long)g * p.o_group_stride + o;
                if (p.accumulate) {
                    const float4 o0 = *reinterpret_cast<const float4*>(dst), o1 = *reinterpret_cast<const float4*>(dst + 4);
                    v[0] += o0.x; v[1] += o0.y; v[2] += o0.z; v[3] += o0.w;
                    v[4] += o1.x; v[5] += o1.y; v[6] += o1.z; v[7] += o1.w;
                }
                *reinterpret_cast<float4*>(dst) = make_float4(v[0], v[1], v[2], v[3]);
                *reinterpret_cast<float4*>(dst + 4) = make_float4(v[4], v[5], v[6], v[7]);
            } else if (EPI == EPI_FWD1_GELU) {
                float a[8];
#pragma unroll
                for (int e = 0; e < 8; ++e) a[e] = gelu_f(v[e]);
                put(rO0, pack8(v));                            // no length in a forward-only pass: Z is not kept
                put(rO2, pack8(a));
            } else if (EPI == EPI_FWD1_SWIGLU) {
                float a[8];
#pragma unroll
                for (int e = 0; e < 8; ++e) a[e] = v[e] * sigmoid_f(v[e]) * u[e];
                put(rO0, pack8(v));                            // no length in a forward-only pass: Z and U are not kept
                put(rO1, pack8(u));
                put(rO2, pack8(a));
            } else if (EPI == EPI_BWD1_GELU) {
                float z[8], dz[8];
                unpack8(zin[cur][pass - pb], z);
#pragma unroll
                for (int e = 0; e < 8; ++e) dz[e] = v[e] * gelu_grad_f(z[e]);
                uint4 aw = make_uint4(0, 0, 0, 0);
                if (p.write_act) {
                    float a[8];
#pragma unroll
                    for (int e = 0; e < 8; ++e) a[e] = gelu_f(z[e]);
                    aw = pack8(a);
                }
                put(rO0, pack8(dz));
                put(rO2, aw);                                  // no length when the forward pass's activation is still there
            } else if (EPI == EPI_BWD1_SWIGLU) {
                // silu(z) = z s and silu'(z) = s + z s (1 - s) with s = sigmoid(z): eight vector instructions and
                // two transcendentals per element (this epilogue is bound by its vector instructions)
                float z[8], uu[8], dz[8], du[8], zs[8];
                unpack8(zin[cur][pass - pb], z);
                unpack8(uin[cur][pass - pb], uu);
#pragma unroll
                for (int e = 0; e < 8; ++e) {
                    const float sg = sigmoid_f(z[e]);
                    zs[e] = z[e] * sg;
                    du[e] = v[e] * zs[e];
                    dz[e] = (v[e] * uu[e]) * __builtin_fmaf(zs[e], 1.0f - sg, sg);
                }
                uint4 aw = make_uint4(0, 0, 0, 0);
                if (p.write_act) {
                    float a[8];
#pragma unroll
                    for (int e = 0; e < 8; ++e) a[e] = zs[e] * uu[e];
                    aw = pack8(a);
                }
                put(rO0, pack8(dz));
                put(rO1, pack8(du));
                put(rO2, aw);                                  // no length when the forward pass's activation is still there
            }
        }
        }
    }
    __syncthreads();             // every wave is done with its patch before the next tile's DMA lands there
  }
}

// ---- host side ----------------------------------------------------------------------------------
template <int KIND, int EPI>
hipError_t launch(GemmParams p, int rows_upper, int n_groups_cap, hipStream_t st)
{
    constexpr bool DUAL = (EPI == EPI_FWD1_SWIGLU);
    const int bn = DUAL ? BN / 2 : BN;
    p.col_tiles = (p.N + bn - 1) / bn;
    if (KIND == KIND_TN) {
        p.row_tiles = (p.Mout + BM - 1) / BM;
        p.n_tiles = n_groups_cap * p.row_tiles * p.col_tiles;
    } else {
        p.row_tiles = (rows_upper + BM - 1) / BM + n_groups_cap;      // upper bound; the kernel counts the real ones
        p.n_tiles = p.row_tiles * p.col_tiles;
    }
    if (p.n_tiles == 0) return hipSuccess;
    // persistent: one block per CU (LDS allows no more), a multiple of 8.  The CU count and the kernels' dynamic
    // LDS limit are looked up / set once per device (per instantiation).
    static PerDeviceOnce once;
    static std::atomic<int> cus_of[64];
    const int dev = current_device();
    int cus = (dev >= 0 && dev < 64) ? cus_of[dev].load(std::memory_order_acquire) : 0;
    auto kern = grouped_gemm_kernel<KIND, EPI, false>;
    auto kern_fin = grouped_gemm_kernel<KIND, EPI, KIND != KIND_TN>;     // TN has no split round
    if (!once.is_done(dev) || cus == 0) {
        int n = 0;
        if (dev < 0 || hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || n < 8) n = 256;
        cus = n / 8 * 8;
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, (int)LDS_BYTES);
        if (e == hipSuccess && KIND != KIND_TN)
            e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern_fin), hipFuncAttributeMaxDynamicSharedMemorySize, (int)LDS_BYTES);
        if (e != hipSuccess) return e;
        if (dev >= 0 && dev < 64) cus_of[dev].store(cus, std::memory_order_release);
        once.mark(dev);
    }
    const int grid = cus;
    // short contractions gain less from the split than the second launch costs
    if (KIND == KIND_TN || p.n_seg * (p.Kseg / BK) < 128) p.split_ws = nullptr;
    p.split_cap = SPLIT_UNITS;
    hipLaunchKernelGGL(kern, dim3(grid), dim3(NT), LDS_BYTES, st, p);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess || KIND == KIND_TN || p.split_ws == nullptr) return e;
    // the tiles of a K-split last round: add their parts, run their epilogues
    hipLaunchKernelGGL(kern_fin, dim3(grid), dim3(NT), LDS_BYTES, st, p);
    return hipGetLastError();
}

GemmParams base_params(const moe_shape_t& s, const ffn_args& a)
{
    GemmParams p{};
    p.slot_offsets = a.slot_offsets; p.dest_slots = a.dest_slots;
    p.self = s.self; p.Gcap = s.G;
    p.n_seg = 1;
    p.split_ws = a.split_ws;
    return p;
}

}  // namespace



hipError_t launch_ffn_fwd_bf16(const moe_shape_t& s, const ffn_args& a, hipStream_t st)
{
    const int A = s.T * s.k;
    if (A == 0) return hipSuccess;
    const long d = s.d, h = s.h;
    hipError_t e;
    {   // fwd1: [rows, d] x W1[g] (d x h)
        GemmParams p = base_params(s, a);
        p.band = BAND_FWD1;
        p.A[0] = (const bf16_t*)a.Xp; p.B[0] = (const bf16_t*)a.W1; p.B_dual = (const bf16_t*)a.W3;
        p.lda = d; p.ldb = h; p.b_group_stride = d * h; p.Kseg = s.d; p.N = s.h;
        p.O0 = (bf16_t*)a.Z; p.O1 = (bf16_t*)a.U; p.O2 = (bf16_t*)a.Act; p.ldo = h;
        e = (s.act == MOE_ACT_SWIGLU) ? launch<KIND_NN, EPI_FWD1_SWIGLU>(p, A, s.G, st)
                                      : launch<KIND_NN, EPI_FWD1_GELU>(p, A, s.G, st);
        if (e != hipSuccess) return e;
    }
    {   // fwd2: Act [rows, h] x W2[g] (h x d)
        GemmParams p = base_params(s, a);
        p.band = BAND_FWD2;
        p.A[0] = (const bf16_t*)a.Act; p.B[0] = (const bf16_t*)a.W2;
        p.lda = h; p.ldb = d; p.b_group_stride = d * h; p.Kseg = s.h; p.N = s.d;
        p.O0 = (bf16_t*)a.Yp; p.ldo = d;
        e = launch<KIND_NN, EPI_BF16>(p, A, s.G, st);
    }
    return e;
}

hipError_t launch_ffn_bwd_bf16(const moe_shape_t& s, const ffn_args& a, hipStream_t st)
{
    const int A = s.T * s.k;
    const long d = s.d, h = s.h;
    const bool swiglu = s.act == MOE_ACT_SWIGLU;
    hipError_t e = hipSuccess;
    if (A > 0) {
        {   // bwd1: dA = dYp [rows, d] x W2[g]^T (W2 is h x d: contraction index contiguous)
            GemmParams p = base_params(s, a);
            p.band = BAND_BWD1;
            p.A[0] = (const bf16_t*)a.dYp; p.B[0] = (const bf16_t*)a.W2;
            p.lda = d; p.ldb = d; p.b_group_stride = d * h; p.Kseg = s.d; p.N = s.h;
            p.O0 = (bf16_t*)a.dZ; p.O1 = (bf16_t*)a.dU; p.O2 = (bf16_t*)a.Act; p.ldo = h;
            p.Zin = (const bf16_t*)a.Z; p.Uin = (const bf16_t*)a.U;
            p.write_act = a.act_saved ? 0 : 1;
            e = swiglu ? launch<KIND_NT, EPI_BWD1_SWIGLU>(p, A, s.G, st)
                       : launch<KIND_NT, EPI_BWD1_GELU>(p, A, s.G, st);
            if (e != hipSuccess) return e;
        }
        {   // bwd2: dXp = dZ [rows, h] x W1[g]^T (+ dU x W3[g]^T)
            GemmParams p = base_params(s, a);
            p.band = BAND_BWD2;
            p.A[0] = (const bf16_t*)a.dZ; p.B[0] = (const bf16_t*)a.W1;
            p.A[1] = (const bf16_t*)a.dU; p.B[1] = (const bf16_t*)a.W3;
            p.n_seg = swiglu ? 2 : 1;
            p.lda = h; p.ldb = h; p.b_group_stride = d * h; p.Kseg = s.h; p.N = s.d;
            p.O0 = (bf16_t*)a.dXp; p.ldo = d;
            e = launch<KIND_NT, EPI_BF16>(p, A, s.G, st);
            if (e != hipSuccess) return e;
        }
    }
    // weight gradients: contraction over the rows of each group
    auto wgrad = [&](const void* L, long ldl, int Mout, const void* R, long ldr, int N, float* out) {
        GemmParams p = base_params(s, a);
        p.band = BAND_WGRAD;
        p.A[0] = (const bf16_t*)L; p.B[0] = (const bf16_t*)R;
        p.lda = ldl; p.ldb = ldr; p.b_group_stride = 0; p.Mout = Mout; p.N = N;
        p.OF = out; p.ldo = N; p.o_group_stride = d * h; p.accumulate = a.accumulate ? 1 : 0;
        return launch<KIND_TN, EPI_F32>(p, A, s.G, st);
    };
    e = wgrad(a.Xp, d, s.d, a.dZ, h, s.h, a.dW1);
    if (e != hipSuccess) return e;
    if (swiglu) {
        e = wgrad(a.Xp, d, s.d, a.dU, h, s.h, a.dW3);
        if (e != hipSuccess) return e;
    }
    return wgrad(a.Act, h, s.h, a.dYp, d, s.d, a.dW2);
}

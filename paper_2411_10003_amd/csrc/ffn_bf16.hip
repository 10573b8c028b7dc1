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
// is masked, so nothing is padded to the largest load.  The grid is sized from an upper bound
// of the tile count (the host never reads the counts); surplus blocks exit at once.
//
// Tiling: BM x BN output tile per block, BK-deep slices staged through LDS (double buffered,
// next slice prefetched into registers while the current one is multiplied), 32x32x16 bf16 MFMA.
// An operand whose contraction index is contiguous in memory is kept row-major in LDS and read
// with 16-byte loads; one whose contraction index is the slow one is kept as it is and read with
// the transposing LDS load, so no operand is ever transposed in HBM.  The MFMA is issued with the
// operands swapped, which leaves every lane with four consecutive output columns of one row and
// gives 8/16-byte stores.
#include "internal.h"

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
    int n_tiles;
    // outputs
    bf16_t *O0, *O1, *O2;        // EPI_BF16: O0.  FWD1: Z, U, Act.  BWD1: dZ, dU, Act
    float* OF;                   // EPI_F32
    long ldo, o_group_stride;
    const bf16_t *Zin, *Uin;     // BWD1: saved pre-activations
};

__device__ __forceinline__ float gelu_f(float z) { return 0.5f * z * (1.0f + erff(z * 0.70710678118654752f)); }
__device__ __forceinline__ float gelu_grad_f(float z) {
    return 0.5f * (1.0f + erff(z * 0.70710678118654752f)) + z * 0.3989422804014327f * __expf(-0.5f * z * z);
}
__device__ __forceinline__ float sigmoid_f(float z) { return 1.0f / (1.0f + __expf(-z)); }

template <int BM_, int BN_, int BK_, int WGM_, int WGN_>
struct Tile {
    static constexpr int BM = BM_, BN = BN_, BK = BK_, WGM = WGM_, WGN = WGN_;
    static constexpr int NT = WGM * WGN * 64;
    static constexpr int WM = BM / WGM, WN = BN / WGN;
    static constexpr int TM = WM / 32, TN = WN / 32;
    static constexpr int PITCH_R = BK + 8;                 // K-contiguous tile: [rows][BK], padded
    static constexpr int PITCH_CM = BM + 32, PITCH_CN = BN + 32;   // K-major tile: [BK][cols], padded
    static constexpr int A_R = BM * PITCH_R, A_C = BK * PITCH_CM;
    static constexpr int B_R = BN * PITCH_R, B_C = BK * PITCH_CN;
};

// ---- global -> registers -> LDS -----------------------------------------------------------------
// A tile of ROWS x COLS elements, COLS contiguous in memory, moved as 16-byte pieces.
// Piece q = p * NT + tid sits at row q / (COLS/8), column 8 * (q % (COLS/8)).
template <int ROWS, int COLS, int NT>
struct Mover {
    static constexpr int PIECES = ROWS * COLS / 8;
    static constexpr int PER = (PIECES + NT - 1) / NT;
    static constexpr int CPR = COLS / 8;

    // rows [row0, row0+ROWS) x columns [col0, col0+COLS) of a matrix with leading dimension ld;
    // rows >= row_end and columns >= col_end read as zero.  With DUAL the right half of the tile
    // comes from `base2` at the same columns as the left half.
    template <bool DUAL>
    static __device__ __forceinline__ void load(uint4 (&r)[PER], const bf16_t* base, const bf16_t* base2, long ld,
                                                long row0, long row_end, int col0, int col_end, int tid)
    {
#pragma unroll
        for (int p = 0; p < PER; ++p) {
            const int q = p * NT + tid;
            const int row = q / CPR;
            int c = (q % CPR) * 8;
            const bf16_t* src = base;
            if (DUAL) {
                if (c >= COLS / 2) { src = base2; c -= COLS / 2; }
            }
            uint4 v = make_uint4(0, 0, 0, 0);
            if ((PIECES % NT == 0 || q < PIECES) && row0 + row < row_end && col0 + c < col_end)
                v = *reinterpret_cast<const uint4*>(src + (row0 + row) * ld + col0 + c);
            r[p] = v;
        }
    }
    template <int PITCH>
    static __device__ __forceinline__ void store(const uint4 (&r)[PER], bf16_t* tile, int tid)
    {
#pragma unroll
        for (int p = 0; p < PER; ++p) {
            const int q = p * NT + tid;
            if (PIECES % NT == 0 || q < PIECES)
                *reinterpret_cast<uint4*>(tile + (q / CPR) * PITCH + (q % CPR) * 8) = r[p];
        }
    }
};

// ---- LDS -> MFMA operand fragments --------------------------------------------------------------
// Fragment = 32 rows (or columns) x 16 contraction steps; lane l holds row l%32, steps 8*(l/32)..+7.
template <int PITCH>
__device__ __forceinline__ bf16x8 frag_kcontig(const bf16_t* tile, int row_base, int kk, int lane)
{
    const bf16_t* p = tile + (row_base + (lane & 31)) * PITCH + kk + 8 * (lane >> 5);
    return *reinterpret_cast<const bf16x8*>(p);
}
// Tile stored [contraction step][column].  The transposing load works on blocks of 16 lanes: lane s of
// a block points at 4 consecutive columns of step (s/4); lane i of the block receives column i of
// steps 0..3.  Two loads give the 8 steps of a lane in the same order as frag_kcontig.
template <int PITCH>
__device__ __forceinline__ bf16x8 frag_kmajor(const bf16_t* tile, int col_base, int kk, int lane)
{
    const int b = lane >> 4, s = lane & 15;
    const bf16_t* p = tile + (kk + 8 * (b >> 1) + (s >> 2)) * PITCH + col_base + 16 * (b & 1) + 4 * (s & 3);
    const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((LDS_PTR(s16x4))(p));
    const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((LDS_PTR(s16x4))(p + 4 * PITCH));
    const s16x8 v = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
    return __builtin_bit_cast(bf16x8, v);
}

__device__ __forceinline__ uint2 pack4(float a, float b, float c, float d)
{
    return make_uint2(pack_bf16x2(a, b), pack_bf16x2(c, d));
}
__device__ __forceinline__ void unpack4(uint2 v, float* f)
{
    f[0] = __uint_as_float(v.x << 16); f[1] = __uint_as_float(v.x & 0xffff0000u);
    f[2] = __uint_as_float(v.y << 16); f[3] = __uint_as_float(v.y & 0xffff0000u);
}

// ---- the kernel ---------------------------------------------------------------------------------
template <class TC, int KIND, int EPI>
__global__ __launch_bounds__(TC::NT) void grouped_gemm_kernel(const GemmParams p)
{
    constexpr int BM = TC::BM, BN = TC::BN, BK = TC::BK, NT = TC::NT;
    constexpr bool A_KMAJOR = (KIND == KIND_TN);
    constexpr bool B_KMAJOR = (KIND != KIND_NT);
    constexpr bool DUAL = (EPI == EPI_FWD1_SWIGLU);
    constexpr int A_ELEMS = A_KMAJOR ? TC::A_C : TC::A_R;
    constexpr int B_ELEMS = B_KMAJOR ? TC::B_C : TC::B_R;
    constexpr int STAGE = A_ELEMS + B_ELEMS;
    static_assert(!DUAL || (TC::TN % 2 == 0), "dual-B needs an even number of column fragments per wave");

    extern __shared__ __attribute__((aligned(16))) bf16_t smem[];

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave / TC::WGN, wn = wave % TC::WGN;

    // ---- which tile: spread consecutive tiles over one XCD (blocks go round-robin over 8 XCDs),
    //      then walk bands of 8 row tiles column by column so that neighbours share operands
    int tile_id;
    {
        const int nb = gridDim.x, per = nb >> 3;           // nb is a multiple of 8
        tile_id = (blockIdx.x & 7) * per + (blockIdx.x >> 3);
    }
    if (tile_id >= p.n_tiles) return;
    int first_slot, n_groups;
    hosted_range(p.dest_slots, p.self, p.Gcap, first_slot, n_groups);

    int g, rt, ct;
    {
        int rem = tile_id, row_tiles = p.row_tiles;
        g = 0;
        if (KIND == KIND_TN) {
            const int per_group = p.row_tiles * p.col_tiles;
            g = rem / per_group;
            rem -= g * per_group;
        }
        const int band = rem / (8 * p.col_tiles);
        const int in_band = rem - band * 8 * p.col_tiles;
        const int band_rows = min(8, row_tiles - band * 8);
        rt = band * 8 + in_band % band_rows;
        ct = in_band / band_rows;
    }

    long a_row0, a_row_end;      // valid rows of the A tile (NN/NT) or of the contraction (TN)
    int k_tiles;
    int m0;                      // first output row of the tile (global row for NN/NT, row of dW for TN)
    if (KIND == KIND_TN) {
        int row0 = 0, rows = 0;
        if (g < n_groups) { row0 = p.slot_offsets[first_slot + g]; rows = p.slot_offsets[first_slot + g + 1] - row0; }
        a_row0 = row0; a_row_end = row0 + rows;
        k_tiles = (rows + BK - 1) / BK;
        m0 = rt * BM;
    } else {
        int acc = 0;
        bool found = false;
        int gg = 0, row0 = 0, row_end = 0;
        for (; gg < n_groups; ++gg) {
            const int o = p.slot_offsets[first_slot + gg], e = p.slot_offsets[first_slot + gg + 1];
            const int nt = (e - o + BM - 1) / BM;
            if (rt < acc + nt) { row0 = o + (rt - acc) * BM; row_end = e; found = true; break; }
            acc += nt;
        }
        if (!found) return;
        g = gg;
        a_row0 = row0; a_row_end = row_end;
        k_tiles = p.n_seg * (p.Kseg / BK);
        m0 = row0;
    }
    const int n0 = ct * (DUAL ? BN / 2 : BN);             // first output column (hidden unit for dual)
    const int k_per_seg = (KIND == KIND_TN) ? k_tiles : p.Kseg / BK;

    using MovA = Mover<A_KMAJOR ? BK : BM, A_KMAJOR ? BM : BK, NT>;
    using MovB = Mover<B_KMAJOR ? BK : BN, B_KMAJOR ? BN : BK, NT>;
    uint4 ra[MovA::PER], rb[MovB::PER];

    auto load_slice = [&](int kt) {
        const int seg = (KIND == KIND_TN) ? 0 : kt / k_per_seg;
        const int k0 = (kt - seg * k_per_seg) * BK;
        const bf16_t* Ab = p.A[seg];
        const bf16_t* Bb = p.B[seg] + (long)g * p.b_group_stride;
        if (KIND == KIND_TN) {
            // A tile: contraction rows [a_row0 + k0, +BK) x output rows [m0, m0+BM) of a [rows, Mout] matrix
            MovA::template load<false>(ra, Ab, Ab, p.lda, a_row0 + k0, a_row_end, m0, p.Mout, tid);
            MovB::template load<false>(rb, Bb, Bb, p.ldb, a_row0 + k0, a_row_end, n0, p.N, tid);
        } else {
            MovA::template load<false>(ra, Ab, Ab, p.lda, a_row0, a_row_end, k0, p.Kseg, tid);
            if (KIND == KIND_NN) {
                const bf16_t* B2 = DUAL ? p.B_dual + (long)g * p.b_group_stride : Bb;
                MovB::template load<DUAL>(rb, Bb, B2, p.ldb, k0, p.Kseg, n0, p.N, tid);
            } else {
                MovB::template load<false>(rb, Bb, Bb, p.ldb, n0, p.N, k0, p.Kseg, tid);
            }
        }
    };
    auto store_slice = [&](int stage) {
        bf16_t* sa = smem + stage * STAGE;
        bf16_t* sb = sa + A_ELEMS;
        if (A_KMAJOR) MovA::template store<TC::PITCH_CM>(ra, sa, tid); else MovA::template store<TC::PITCH_R>(ra, sa, tid);
        if (B_KMAJOR) MovB::template store<TC::PITCH_CN>(rb, sb, tid); else MovB::template store<TC::PITCH_R>(rb, sb, tid);
    };

    f32x16 acc[TC::TM][TC::TN];
#pragma unroll
    for (int i = 0; i < TC::TM; ++i)
#pragma unroll
        for (int j = 0; j < TC::TN; ++j)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.0f;

    if (k_tiles > 0) {
        load_slice(0);
        store_slice(0);
    }
    __syncthreads();
    for (int kt = 0; kt < k_tiles; ++kt) {
        const int cur = kt & 1;
        const bool more = kt + 1 < k_tiles;
        if (more) load_slice(kt + 1);
        const bf16_t* sa = smem + cur * STAGE;
        const bf16_t* sb = sa + A_ELEMS;
#pragma unroll
        for (int kk = 0; kk < BK; kk += 16) {
            bf16x8 fa[TC::TM], fb[TC::TN];
#pragma unroll
            for (int i = 0; i < TC::TM; ++i) {
                const int r = wm * TC::WM + i * 32;
                fa[i] = A_KMAJOR ? frag_kmajor<TC::PITCH_CM>(sa, r, kk, lane) : frag_kcontig<TC::PITCH_R>(sa, r, kk, lane);
            }
#pragma unroll
            for (int j = 0; j < TC::TN; ++j) {
                // dual: even fragments come from the left half (W1), odd ones from the right half (W3)
                const int c = DUAL ? (j & 1) * (BN / 2) + wn * (TC::WN / 2) + (j >> 1) * 32 : wn * TC::WN + j * 32;
                fb[j] = B_KMAJOR ? frag_kmajor<TC::PITCH_CN>(sb, c, kk, lane) : frag_kcontig<TC::PITCH_R>(sb, c, kk, lane);
            }
#pragma unroll
            for (int i = 0; i < TC::TM; ++i)
#pragma unroll
                for (int j = 0; j < TC::TN; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fb[j], fa[i], acc[i][j], 0, 0, 0);
        }
        if (more) store_slice(cur ^ 1);
        __syncthreads();
    }

    // ---- epilogue: lane holds row (l%32) of each fragment and columns q*8 + (l/32)*4 + 0..3
    const int lrow = lane & 31, lcol = (lane >> 5) * 4;
    const long row_limit = (KIND == KIND_TN) ? (long)p.Mout : a_row_end;
#pragma unroll
    for (int i = 0; i < TC::TM; ++i) {
        const long row = (long)m0 + wm * TC::WM + i * 32 + lrow;
        if (row >= row_limit) continue;
        if (EPI == EPI_FWD1_SWIGLU) {
#pragma unroll
            for (int j = 0; j < TC::TN; j += 2) {
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    const int col = n0 + wn * (TC::WN / 2) + (j >> 1) * 32 + q * 8 + lcol;
                    if (col >= p.N) continue;
                    float z[4], u[4], a[4];
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        z[e] = acc[i][j][q * 4 + e];
                        u[e] = acc[i][j + 1][q * 4 + e];
                        a[e] = z[e] * sigmoid_f(z[e]) * u[e];
                    }
                    const long o = row * p.ldo + col;
                    *reinterpret_cast<uint2*>(p.O0 + o) = pack4(z[0], z[1], z[2], z[3]);
                    *reinterpret_cast<uint2*>(p.O1 + o) = pack4(u[0], u[1], u[2], u[3]);
                    *reinterpret_cast<uint2*>(p.O2 + o) = pack4(a[0], a[1], a[2], a[3]);
                }
            }
        } else {
#pragma unroll
            for (int j = 0; j < TC::TN; ++j) {
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    const int col = n0 + wn * TC::WN + j * 32 + q * 8 + lcol;
                    if (col >= p.N) continue;
                    float v[4];
#pragma unroll
                    for (int e = 0; e < 4; ++e) v[e] = acc[i][j][q * 4 + e];
                    const long o = row * p.ldo + col;
                    if (EPI == EPI_BF16) {
                        *reinterpret_cast<uint2*>(p.O0 + o) = pack4(v[0], v[1], v[2], v[3]);
                    } else if (EPI == EPI_F32) {
                        *reinterpret_cast<float4*>(p.OF + (long)g * p.o_group_stride + o) = make_float4(v[0], v[1], v[2], v[3]);
                    } else if (EPI == EPI_FWD1_GELU) {
                        *reinterpret_cast<uint2*>(p.O0 + o) = pack4(v[0], v[1], v[2], v[3]);
                        *reinterpret_cast<uint2*>(p.O2 + o) = pack4(gelu_f(v[0]), gelu_f(v[1]), gelu_f(v[2]), gelu_f(v[3]));
                    } else if (EPI == EPI_BWD1_GELU) {
                        float z[4];
                        unpack4(*reinterpret_cast<const uint2*>(p.Zin + o), z);
                        *reinterpret_cast<uint2*>(p.O0 + o) = pack4(v[0] * gelu_grad_f(z[0]), v[1] * gelu_grad_f(z[1]),
                                                                   v[2] * gelu_grad_f(z[2]), v[3] * gelu_grad_f(z[3]));
                        *reinterpret_cast<uint2*>(p.O2 + o) = pack4(gelu_f(z[0]), gelu_f(z[1]), gelu_f(z[2]), gelu_f(z[3]));
                    } else if (EPI == EPI_BWD1_SWIGLU) {
                        float z[4], u[4], dz[4], du[4], a[4];
                        unpack4(*reinterpret_cast<const uint2*>(p.Zin + o), z);
                        unpack4(*reinterpret_cast<const uint2*>(p.Uin + o), u);
#pragma unroll
                        for (int e = 0; e < 4; ++e) {
                            const float s = sigmoid_f(z[e]);
                            du[e] = v[e] * z[e] * s;
                            dz[e] = v[e] * u[e] * s * (1.0f + z[e] * (1.0f - s));
                            a[e] = z[e] * s * u[e];
                        }
                        *reinterpret_cast<uint2*>(p.O0 + o) = pack4(dz[0], dz[1], dz[2], dz[3]);
                        *reinterpret_cast<uint2*>(p.O1 + o) = pack4(du[0], du[1], du[2], du[3]);
                        *reinterpret_cast<uint2*>(p.O2 + o) = pack4(a[0], a[1], a[2], a[3]);
                    }
                }
            }
        }
    }
}

// ---- host side ----------------------------------------------------------------------------------
using TileMain = Tile<256, 256, 64, 2, 4>;     // 8 waves, 128 x 64 per wave

template <class TC, int KIND, int EPI>
hipError_t launch(GemmParams p, int rows_upper, int n_groups_cap, hipStream_t st)
{
    constexpr bool A_KMAJOR = (KIND == KIND_TN);
    constexpr bool B_KMAJOR = (KIND != KIND_NT);
    constexpr bool DUAL = (EPI == EPI_FWD1_SWIGLU);
    constexpr int STAGE = (A_KMAJOR ? TC::A_C : TC::A_R) + (B_KMAJOR ? TC::B_C : TC::B_R);
    constexpr size_t LDS = (size_t)2 * STAGE * sizeof(bf16_t);
    const int bn = DUAL ? TC::BN / 2 : TC::BN;
    p.col_tiles = (p.N + bn - 1) / bn;
    if (KIND == KIND_TN) {
        p.row_tiles = (p.Mout + TC::BM - 1) / TC::BM;
        p.n_tiles = n_groups_cap * p.row_tiles * p.col_tiles;
    } else {
        p.row_tiles = (rows_upper + TC::BM - 1) / TC::BM + n_groups_cap;
        p.n_tiles = p.row_tiles * p.col_tiles;
    }
    if (p.n_tiles == 0) return hipSuccess;
    const int grid = (p.n_tiles + 7) / 8 * 8;
    auto kern = grouped_gemm_kernel<TC, KIND, EPI>;
    static bool configured = false;      // per instantiation
    if (!configured) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, (int)LDS);
        if (e != hipSuccess) return e;
        configured = true;
    }
    hipLaunchKernelGGL(kern, dim3(grid), dim3(TC::NT), LDS, st, p);
    return hipGetLastError();
}

GemmParams base_params(const moe_shape_t& s, const ffn_args& a)
{
    GemmParams p{};
    p.slot_offsets = a.slot_offsets; p.dest_slots = a.dest_slots;
    p.self = s.self; p.Gcap = s.G;
    p.n_seg = 1;
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
        p.A[0] = (const bf16_t*)a.Xp; p.B[0] = (const bf16_t*)a.W1; p.B_dual = (const bf16_t*)a.W3;
        p.lda = d; p.ldb = h; p.b_group_stride = d * h; p.Kseg = s.d; p.N = s.h;
        p.O0 = (bf16_t*)a.Z; p.O1 = (bf16_t*)a.U; p.O2 = (bf16_t*)a.Act; p.ldo = h;
        e = (s.act == MOE_ACT_SWIGLU) ? launch<TileMain, KIND_NN, EPI_FWD1_SWIGLU>(p, A, s.G, st)
                                      : launch<TileMain, KIND_NN, EPI_FWD1_GELU>(p, A, s.G, st);
        if (e != hipSuccess) return e;
    }
    {   // fwd2: Act [rows, h] x W2[g] (h x d)
        GemmParams p = base_params(s, a);
        p.A[0] = (const bf16_t*)a.Act; p.B[0] = (const bf16_t*)a.W2;
        p.lda = h; p.ldb = d; p.b_group_stride = d * h; p.Kseg = s.h; p.N = s.d;
        p.O0 = (bf16_t*)a.Yp; p.ldo = d;
        e = launch<TileMain, KIND_NN, EPI_BF16>(p, A, s.G, st);
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
            p.A[0] = (const bf16_t*)a.dYp; p.B[0] = (const bf16_t*)a.W2;
            p.lda = d; p.ldb = d; p.b_group_stride = d * h; p.Kseg = s.d; p.N = s.h;
            p.O0 = (bf16_t*)a.dZ; p.O1 = (bf16_t*)a.dU; p.O2 = (bf16_t*)a.Act; p.ldo = h;
            p.Zin = (const bf16_t*)a.Z; p.Uin = (const bf16_t*)a.U;
            e = swiglu ? launch<TileMain, KIND_NT, EPI_BWD1_SWIGLU>(p, A, s.G, st)
                       : launch<TileMain, KIND_NT, EPI_BWD1_GELU>(p, A, s.G, st);
            if (e != hipSuccess) return e;
        }
        {   // bwd2: dXp = dZ [rows, h] x W1[g]^T (+ dU x W3[g]^T)
            GemmParams p = base_params(s, a);
            p.A[0] = (const bf16_t*)a.dZ; p.B[0] = (const bf16_t*)a.W1;
            p.A[1] = (const bf16_t*)a.dU; p.B[1] = (const bf16_t*)a.W3;
            p.n_seg = swiglu ? 2 : 1;
            p.lda = h; p.ldb = h; p.b_group_stride = d * h; p.Kseg = s.h; p.N = s.d;
            p.O0 = (bf16_t*)a.dXp; p.ldo = d;
            e = launch<TileMain, KIND_NT, EPI_BF16>(p, A, s.G, st);
            if (e != hipSuccess) return e;
        }
    }
    // weight gradients: contraction over the rows of each group
    auto wgrad = [&](const void* L, long ldl, int Mout, const void* R, long ldr, int N, float* out) {
        GemmParams p = base_params(s, a);
        p.A[0] = (const bf16_t*)L; p.B[0] = (const bf16_t*)R;
        p.lda = ldl; p.ldb = ldr; p.b_group_stride = 0; p.Mout = Mout; p.N = N;
        p.OF = out; p.ldo = N; p.o_group_stride = d * h;
        return launch<TileMain, KIND_TN, EPI_F32>(p, A, s.G, st);
    };
    e = wgrad(a.Xp, d, s.d, a.dZ, h, s.h, a.dW1);
    if (e != hipSuccess) return e;
    if (swiglu) {
        e = wgrad(a.Xp, d, s.d, a.dU, h, s.h, a.dW3);
        if (e != hipSuccess) return e;
    }
    return wgrad(a.Act, h, s.h, a.dYp, d, s.d, a.dW2);
}

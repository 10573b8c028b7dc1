// Expert FFN forward and backward in fp32 (Section 4.2 of the paper, FEC / BEC) for the small
// single-precision configuration.  Plain LDS-tiled fp32 contractions, one output element per
// thread; groups are ragged and may be empty.  Not the performance path (the bf16 MFMA kernels
// are); this one exists so that the fp32 workload meets a 1e-5 tolerance.
#include "internal.h"

namespace {

constexpr int TS = 16;   // tile side; block = TS x TS threads

__device__ __forceinline__ float gelu_f(float z) { return 0.5f * z * (1.0f + erff(z * 0.70710678118654752f)); }
__device__ __forceinline__ float gelu_grad_f(float z) {
    return 0.5f * (1.0f + erff(z * 0.70710678118654752f)) + z * 0.3989422804014327f * expf(-0.5f * z * z);
}
__device__ __forceinline__ float sigmoid_f(float z) { return 1.0f / (1.0f + expf(-z)); }

// A strided view: element (r, c) at p[r * rs + c * cs]
struct View { const float* p; long rs, cs; };

enum Mode { FWD1 = 0, FWD2 = 1, BWD1 = 2, BWD2 = 3, WGRAD = 4 };

struct F32Args {
    const int32_t *slot_offsets, *dest_slots;
    int self, Gcap, act, d, h;
    const float *Xp, *W1, *W2, *W3, *dYp, *Zc, *Uc, *Actc, *dZc, *dUc;
    float *Yp, *Z, *U, *Act, *dZ, *dU, *dXp, *dW1, *dW2, *dW3;
    int accumulate;
};

// acc (+acc2) = sum_k A(m,k) B(k,n) (+ A2(m,k) B2(k,n)) over a TS x TS output tile
__device__ __forceinline__ void tile_gemm(View A, View B, View A2, View B2, bool dual,
                                          int m, int n, int M, int N, int K, float& acc, float& acc2)
{
    __shared__ float As[TS][TS + 1], Bs[TS][TS + 1], A2s[TS][TS + 1], B2s[TS][TS + 1];
    const int tx = threadIdx.x, ty = threadIdx.y;
    acc = 0.0f; acc2 = 0.0f;
    for (int k0 = 0; k0 < K; k0 += TS) {
        As[ty][tx] = (m < M && k0 + tx < K) ? A.p[(long)m * A.rs + (long)(k0 + tx) * A.cs] : 0.0f;
        Bs[ty][tx] = (k0 + ty < K && n < N) ? B.p[(long)(k0 + ty) * B.rs + (long)n * B.cs] : 0.0f;
        if (dual) {
            A2s[ty][tx] = (m < M && k0 + tx < K) ? A2.p[(long)m * A2.rs + (long)(k0 + tx) * A2.cs] : 0.0f;
            B2s[ty][tx] = (k0 + ty < K && n < N) ? B2.p[(long)(k0 + ty) * B2.rs + (long)n * B2.cs] : 0.0f;
        }
        __syncthreads();
#pragma unroll
        for (int kk = 0; kk < TS; ++kk) {
            acc = fmaf(As[ty][kk], Bs[kk][tx], acc);
            if (dual) acc2 = fmaf(A2s[ty][kk], B2s[kk][tx], acc2);
        }
        __syncthreads();
    }
}

// grid: x = column tiles, y = row tiles (upper bound), z = group
template <int MODE>
__global__ __launch_bounds__(TS * TS) void ffn_f32_kernel(F32Args a)
{
    int first, ng;
    hosted_range(a.dest_slots, a.self, a.Gcap, first, ng);
    const int g = blockIdx.z;
    const int d = a.d, h = a.h;
    const bool swiglu = a.act == MOE_ACT_SWIGLU;
    int row0 = 0, rows = 0;
    if (g < ng) { row0 = a.slot_offsets[first + g]; rows = a.slot_offsets[first + g + 1] - row0; }
    const long wdh = (long)g * d * h;
    const int tx = threadIdx.x, ty = threadIdx.y;
    float acc, acc2;

    if (MODE == WGRAD) {
        // blockIdx.y selects which gradient and its row tile: [0,nt_d) dW1, [nt_d,2nt_d) dW3, then dW2
        const int nt_d = (d + TS - 1) / TS;
        int which, rt;
        if ((int)blockIdx.y < nt_d) { which = 1; rt = blockIdx.y; }
        else if ((int)blockIdx.y < 2 * nt_d) { which = 3; rt = blockIdx.y - nt_d; }
        else { which = 2; rt = blockIdx.y - 2 * nt_d; }
        if (which == 3 && !swiglu) return;
        const int Mo = (which == 2) ? h : d, No = (which == 2) ? d : h;
        const int m = rt * TS + ty, n = blockIdx.x * TS + tx;
        if (rt * TS >= Mo || (int)blockIdx.x * TS >= No) return;
        // out[m,n] = sum over the group's rows r of L[r,m] * R[r,n]
        const float* Lp = (which == 2) ? a.Actc : a.Xp;
        const float* Rp = (which == 1) ? a.dZc : (which == 3 ? a.dUc : a.dYp);
        View A{Lp + (long)row0 * Mo, 1, Mo};            // A(m, r) = L[row0 + r, m]
        View B{Rp + (long)row0 * No, No, 1};            // B(r, n) = R[row0 + r, n]
        tile_gemm(A, B, A, B, false, m, n, Mo, No, rows, acc, acc2);
        float* out = (which == 1) ? a.dW1 : (which == 3 ? a.dW3 : a.dW2);
        if (m < Mo && n < No) out[wdh + (long)m * No + n] = a.accumulate ? out[wdh + (long)m * No + n] + acc : acc;
        return;
    }

    if ((int)blockIdx.y * TS >= rows) return;
    const int m = blockIdx.y * TS + ty;                 // row inside the group
    const int n = blockIdx.x * TS + tx;
    const long r = (long)row0 + m;
    if (MODE == FWD1) {
        View A{a.Xp + (long)row0 * d, d, 1};
        View B{a.W1 + wdh, h, 1};
        View B2{swiglu ? a.W3 + wdh : a.W1 + wdh, h, 1};
        tile_gemm(A, B, A, B2, swiglu, m, n, rows, h, d, acc, acc2);
        if (m < rows && n < h) {
            if (a.Z) a.Z[r * h + n] = acc;              // forward only: the pre-activations are not kept
            if (swiglu) { if (a.U) a.U[r * h + n] = acc2; a.Act[r * h + n] = acc * sigmoid_f(acc) * acc2; }
            else a.Act[r * h + n] = gelu_f(acc);
        }
    } else if (MODE == FWD2) {
        View A{a.Actc + (long)row0 * h, h, 1};
        View B{a.W2 + wdh, d, 1};
        tile_gemm(A, B, A, B, false, m, n, rows, d, h, acc, acc2);
        if (m < rows && n < d) a.Yp[r * d + n] = acc;
    } else if (MODE == BWD1) {
        // dA[m, n] = sum_c dYp[m, c] * W2[n, c]
        View A{a.dYp + (long)row0 * d, d, 1};
        View B{a.W2 + wdh, 1, d};
        tile_gemm(A, B, A, B, false, m, n, rows, h, d, acc, acc2);
        if (m < rows && n < h) {
            const float z = a.Zc[r * h + n];
            if (swiglu) {
                const float u = a.Uc[r * h + n], s = sigmoid_f(z);
                a.dU[r * h + n] = acc * z * s;
                a.dZ[r * h + n] = acc * u * s * (1.0f + z * (1.0f - s));
                a.Act[r * h + n] = z * s * u;
            } else {
                a.dZ[r * h + n] = acc * gelu_grad_f(z);
                a.Act[r * h + n] = gelu_f(z);
            }
        }
    } else if (MODE == BWD2) {
        // dXp[m, n] = sum_j dZ[m, j] W1[n, j] (+ dU[m, j] W3[n, j])
        View A{a.dZc + (long)row0 * h, h, 1};
        View B{a.W1 + wdh, 1, h};
        View A2{swiglu ? a.dUc + (long)row0 * h : a.dZc, h, 1};
        View B2{swiglu ? a.W3 + wdh : a.W1 + wdh, 1, h};
        tile_gemm(A, B, A2, B2, swiglu, m, n, rows, d, h, acc, acc2);
        if (m < rows && n < d) a.dXp[r * d + n] = swiglu ? acc + acc2 : acc;
    }
}

F32Args make_args(const moe_shape_t& s, const ffn_args& a)
{
    F32Args f{};
    f.slot_offsets = a.slot_offsets; f.dest_slots = a.dest_slots;
    f.self = s.self; f.Gcap = s.G; f.act = (int)s.act; f.d = s.d; f.h = s.h;
    f.Xp = (const float*)a.Xp; f.W1 = (const float*)a.W1; f.W2 = (const float*)a.W2; f.W3 = (const float*)a.W3;
    f.dYp = (const float*)a.dYp;
    f.Zc = (const float*)a.Z; f.Uc = (const float*)a.U; f.Actc = (const float*)a.Act;
    f.dZc = (const float*)a.dZ; f.dUc = (const float*)a.dU;
    f.Yp = (float*)a.Yp; f.Z = (float*)a.Z; f.U = (float*)a.U; f.Act = (float*)a.Act;
    f.dZ = (float*)a.dZ; f.dU = (float*)a.dU; f.dXp = (float*)a.dXp;
    f.dW1 = a.dW1; f.dW2 = a.dW2; f.dW3 = a.dW3;
    f.accumulate = a.accumulate ? 1 : 0;
    return f;
}

inline int cdiv(int a, int b) { return (a + b - 1) / b; }

}  // namespace

hipError_t launch_ffn_fwd_f32(const moe_shape_t& s, const ffn_args& a, hipStream_t st)
{
    const int A = s.T * s.k;
    if (A == 0) return hipSuccess;
    const F32Args f = make_args(s, a);
    const dim3 b(TS, TS);
    hipLaunchKernelGGL(ffn_f32_kernel<FWD1>, dim3(cdiv(s.h, TS), cdiv(A, TS), s.G), b, 0, st, f);
    hipLaunchKernelGGL(ffn_f32_kernel<FWD2>, dim3(cdiv(s.d, TS), cdiv(A, TS), s.G), b, 0, st, f);
    return hipGetLastError();
}

hipError_t launch_ffn_bwd_f32(const moe_shape_t& s, const ffn_args& a, hipStream_t st)
{
    const int A = s.T * s.k;
    const F32Args f = make_args(s, a);
    const dim3 b(TS, TS);
    if (A > 0) {
        hipLaunchKernelGGL(ffn_f32_kernel<BWD1>, dim3(cdiv(s.h, TS), cdiv(A, TS), s.G), b, 0, st, f);
        hipLaunchKernelGGL(ffn_f32_kernel<BWD2>, dim3(cdiv(s.d, TS), cdiv(A, TS), s.G), b, 0, st, f);
    }
    const int nt_d = cdiv(s.d, TS), nt_h = cdiv(s.h, TS);
    const int xt = nt_d > nt_h ? nt_d : nt_h;
    hipLaunchKernelGGL(ffn_f32_kernel<WGRAD>, dim3(xt, 2 * nt_d + nt_h, s.G), b, 0, st, f);
    return hipGetLastError();
}

// Greedy search for a lightweight expert placement (Section 4.3, Algorithm 1 of the paper) with its
// performance model (Section 4.2, Eqs. 1-6; Section 5.3, Eq. 8), as one wavefront on the GPU: lane j
// is device j.  The search is a short serial loop over at most E selections; running it on the device
// keeps the host out of the loop between the counts of one iteration and the dispatch of the next.
// All decisions are integer except the comparison of two estimated times, which are IEEE doubles
// evaluated in one fixed association order (no contraction: the library is built with
// -ffp-contract=off).
#include "internal.h"

#include <cmath>

namespace {

constexpr int MAX_E = 1024;

__device__ __forceinline__ long long wave_max_ll(long long v)
{
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) { const long long o = __shfl_xor(v, off, 64); v = o > v ? o : v; }
    return v;
}
__device__ __forceinline__ long long wave_min_ll(long long v)
{
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) { const long long o = __shfl_xor(v, off, 64); v = o < v ? o : v; }
    return v;
}
__device__ __forceinline__ long long wave_sum_ll(long long v)
{
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) v += __shfl_xor(v, off, 64);
    return v;
}

// T'(R, H, s, n) from the largest R and H (Eq. 6, or Eq. 8 with overlap)
__device__ __forceinline__ double layer_time(const moe_planner_t& c, long long max_r, long long max_h, int s, int n)
{
    const double a2a = ((double)max_r * c.size_input) / c.B;                       // Eq. 1
    const double fec = (double)max_h / c.t;                                        // Eq. 2; Eq. 3 is twice this
    const double base = 4.0 * a2a + 3.0 * fec;
    const double tr = ((double)s * (double)(c.D - n) * c.size_params) / ((double)c.D * c.B);   // Eq. 4
    const double ag = ((double)s * (double)(c.D - n) * c.size_grads) / ((double)c.D * c.B);    // Eq. 5
    if (!c.overlap) return (base + tr) + ag;                                       // Eq. 6
    const double bec = 2.0 * fec;
    const double ptr = fmax(0.0, (tr - fec) - c.T_FNEC);                           // Eq. 8
    const double pag = fmax(0.0, (ag - bec) - c.T_BNEC);
    return (base + ptr) + pag;
}

__global__ __launch_bounds__(64) void plan_kernel(const moe_planner_t c, const int32_t* __restrict__ gating, const moe_plan_out_t out)
{
    __shared__ long long tot[MAX_E];                       // inputs per expert over all devices
    __shared__ int sel_rank[MAX_E];                        // rank of selection or -1
    __shared__ unsigned long long skip_of[MAX_E];          // devices skipped, by rank of selection
    const int lane = threadIdx.x;
    const int D = c.D, E = c.E, epd = E / D, n = c.n;

    for (int e = lane; e < E; e += 64) {
        long long s = 0;
        for (int j = 0; j < D; ++j) s += gating[j * E + e];
        tot[e] = s;
        sel_rank[e] = -1;
        out.selected[e] = -1;
        out.skipped[e] = 0ull;
        out.times[2 + e] = 0.0;
    }
    __syncthreads();

    // H, R without any replica: a device computes everything routed to the experts it owns
    const bool dev = lane < D;
    long long H = 0, R = 0;
    if (dev) {
        long long own = 0;
        for (int e = lane * epd; e < (lane + 1) * epd; ++e) { H += tot[e]; own += gating[lane * E + e]; }
        R = H - own;
    }
    const long long total = wave_sum_ll(H);
    const double T_base = layer_time(c, wave_max_ll(dev ? R : 0), wave_max_ll(dev ? H : 0), 0, 0);
    double T_out = T_base;
    long long H_best = H, R_best = R;
    int cnt = 0, s = 0;

    while (s < E) {
        const long long max_h = wave_max_ll(dev ? H : -1);
        const long long min_h = wave_min_ll(dev ? H : 0x7fffffffffffffffll);
        if ((double)(max_h - min_h) < (c.alpha * (double)total) / (double)E) break;        // Eq. 7: balanced
        const int i = __ffsll((unsigned long long)__ballot(dev && H == max_h)) - 1;        // heaviest device, lowest index
        int best = -1;
        for (int e = i * epd; e < (i + 1) * epd; ++e)
            if (sel_rank[e] < 0 && (best < 0 || tot[e] > tot[best])) best = e;
        if (best < 0) break;                                                               // the device has been used up

        // the n non-owners with the fewest inputs of the expert are skipped
        const long long cj = dev ? (long long)gating[lane * E + best] : 0;
        int rank = 0;
        for (int jj = 0; jj < D; ++jj) {
            const long long o = __shfl(cj, jj, 64);
            if (jj != i && (o < cj || (o == cj && jj < lane))) ++rank;
        }
        const bool skip = dev && lane != i && rank < n;
        const unsigned long long skip_mask = (unsigned long long)__ballot(skip);
        const long long delta = (dev && lane != i && !skip) ? cj : 0;                      // inputs that now stay at home
        const long long moved = wave_sum_ll(delta);
        H += delta;
        if (lane == i) { H -= moved; R -= moved; }

        if (lane == 0) { sel_rank[best] = s; skip_of[s] = skip_mask; out.selected[s] = best; out.skipped[s] = skip_mask; }
        __syncthreads();
        ++s;
        const double T = layer_time(c, wave_max_ll(dev ? R : 0), wave_max_ll(dev ? H : 0), s, n);
        if (lane == 0) out.times[2 + s - 1] = T;
        if (T < T_out) { T_out = T; cnt = s; H_best = H; R_best = R; }
    }

    if (dev) { out.H[lane] = H_best; out.R[lane] = R_best; }
    if (lane == 0) { out.times[0] = T_base; out.times[1] = T_out; out.info[0] = cnt; out.info[1] = s; }
    // Get_PoE: the first cnt selections, as one plan per device
    for (int idx = lane; idx < D * E; idx += 64) {
        const int j = idx / E, e = idx - j * E;
        const int r = sel_rank[e];
        int dest = e / epd;
        if (r >= 0 && r < cnt && !((skip_of[r] >> j) & 1ull)) dest = j;
        out.expert_dest[idx] = dest;
    }
}

}  // namespace

hipError_t launch_plan(const moe_planner_t& cfg, const int32_t* gating, const moe_plan_out_t& out, hipStream_t st)
{
    hipLaunchKernelGGL(plan_kernel, dim3(1), dim3(64), 0, st, cfg, gating, out);
    return hipGetLastError();
}

// Input distribution (Section 3 of the paper: inputs per expert), the send layout of a placement
// (Section 4.1) and the stable positions of the assignments inside it.  Integer work only; the
// per-wave histograms and ranks come from wavefront ballots, the offsets from prefix scans.
//
// Assignments are cut into chunks of ROUTE_CHUNK consecutive ids, one wavefront per chunk.
//   chunk_hist[c][e]  assignments of expert e in chunk c
//   chunk_base[c][e]  the same summed over all earlier chunks
//   pos[a] = slot_offsets[slot(e)] + chunk_base[c][e] + (rank of a among the chunk's earlier e's)
#include "internal.h"

namespace {

constexpr int ROUTE_WAVES = 4;

__device__ __forceinline__ unsigned long long lanemask_lt(int lane) {
    return (lane == 0) ? 0ull : (~0ull >> (64 - lane));
}

__global__ __launch_bounds__(ROUTE_WAVES * 64) void chunk_hist_kernel(
    const int32_t* __restrict__ idx, int32_t* __restrict__ chunk_hist, int A, int E, int n_chunks)
{
    extern __shared__ int32_t hist_lds[];          // [ROUTE_WAVES][E]
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int chunk = blockIdx.x * ROUTE_WAVES + wave;
    volatile int32_t* hist = hist_lds + wave * E;
    for (int e = lane; e < E; e += 64) hist[e] = 0;
    if (chunk < n_chunks) {
        for (int r = 0; r < ROUTE_CHUNK / 64; ++r) {
            const int a = chunk * ROUTE_CHUNK + r * 64 + lane;
            int e = -1;
            if (a < A) {
                e = idx[a];
                if (e < 0 || e >= E) e = -1;            // a corrupt index is not counted
            }
            unsigned long long active = __ballot(e >= 0);
            while (active) {
                const int leader = __ffsll((long long)active) - 1;
                const int e0 = __shfl(e, leader, 64);
                const unsigned long long m = __ballot(e == e0);
                if (lane == leader) hist[e0] = hist[e0] + __popcll(m);
                active &= ~m;
            }
        }
        for (int e = lane; e < E; e += 64) chunk_hist[(size_t)chunk * E + e] = hist[e];
    }
}

__global__ void counts_from_hist_kernel(const int32_t* __restrict__ chunk_hist, int n_chunks, int E,
                                        int32_t* __restrict__ counts)
{
    // one wavefront per expert: lanes stride over the chunks, then a butterfly sum
    const int lane = threadIdx.x & 63;
    const int e = blockIdx.x * (blockDim.x >> 6) + (threadIdx.x >> 6);
    if (e >= E) return;
    int s = 0;
    for (int c = lane; c < n_chunks; c += 64) s += chunk_hist[(size_t)c * E + e];
    for (int off = 32; off >= 1; off >>= 1) s += __shfl_xor(s, off, 64);
    if (lane == 0) counts[e] = s;
}

// One block.  Builds the layout from the counts and the placement, and the per-chunk bases.
__global__ __launch_bounds__(256) void layout_scan_kernel(
    const int32_t* __restrict__ expert_dest, const int32_t* __restrict__ counts,
    const int32_t* __restrict__ chunk_hist, int32_t* __restrict__ chunk_base, int n_chunks,
    int32_t* __restrict__ slot_of_expert, int32_t* __restrict__ slot_offsets,
    int32_t* __restrict__ dest_offsets, int32_t* __restrict__ dest_slots,
    int32_t* __restrict__ status, int E, int P, int self, int Gcap)
{
    extern __shared__ int32_t sm[];                // dest[E], slot_cnt[E], slot_off[E+1], flag
    int32_t* dest = sm;
    int32_t* slot_cnt = sm + E;
    int32_t* slot_off = sm + 2 * E;
    int32_t* flag = sm + 3 * E + 1;
    const int tid = threadIdx.x;
    if (tid == 0) *flag = 0;
    __syncthreads();
    for (int e = tid; e < E; e += blockDim.x) {
        int p = expert_dest[e];
        if (p < 0 || p >= P) { atomicOr(flag, 1); p = p < 0 ? 0 : P - 1; }
        dest[e] = p;
    }
    __syncthreads();
    // slot of expert e = number of experts ordered before it by (destination, id)
    for (int e = tid; e < E; e += blockDim.x) {
        const int p = dest[e];
        int s = 0;
        for (int f = 0; f < E; ++f) s += (dest[f] < p) || (dest[f] == p && f < e);
        slot_of_expert[e] = s;
        slot_cnt[s] = counts[e];
    }
    __syncthreads();
    if (tid == 0) {
        int row = 0;
        for (int s = 0; s < E; ++s) { slot_off[s] = row; row += slot_cnt[s]; }
        slot_off[E] = row;
        int hosted = 0;
        for (int e = 0; e < E; ++e) hosted += (dest[e] == self);
        if (hosted > Gcap) *flag = 1;
        *status = *flag ? (int32_t)MOE_ERR_PLAN : (int32_t)MOE_OK;
    }
    __syncthreads();
    for (int s = tid; s <= E; s += blockDim.x) slot_offsets[s] = slot_off[s];
    for (int p = tid; p <= P; p += blockDim.x) {
        int first = 0;                              // slots of destinations below p
        for (int f = 0; f < E; ++f) first += (dest[f] < p);
        dest_slots[p] = first;
        dest_offsets[p] = slot_off[first];
    }
    // exclusive prefix of chunk_hist over chunks, one wavefront per expert at a time
    const int lane = tid & 63, wave = tid >> 6, n_waves = blockDim.x >> 6;
    for (int e = wave; e < E; e += n_waves) {
        int carry = 0;
        for (int c0 = 0; c0 < n_chunks; c0 += 64) {
            const int c = c0 + lane;
            const int v = (c < n_chunks) ? chunk_hist[(size_t)c * E + e] : 0;
            int incl = v;
            for (int off = 1; off < 64; off <<= 1) {
                const int up = __shfl_up(incl, off, 64);
                if (lane >= off) incl += up;
            }
            if (c < n_chunks) chunk_base[(size_t)c * E + e] = carry + incl - v;
            carry += __shfl(incl, 63, 64);
        }
    }
}

__global__ __launch_bounds__(ROUTE_WAVES * 64) void positions_kernel(
    const int32_t* __restrict__ idx, const int32_t* __restrict__ chunk_base,
    const int32_t* __restrict__ slot_of_expert, const int32_t* __restrict__ slot_offsets,
    int32_t* __restrict__ pos, int32_t* __restrict__ perm, int A, int E, int n_chunks)
{
    extern __shared__ int32_t next_lds[];          // [ROUTE_WAVES][E] next free row per expert
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int chunk = blockIdx.x * ROUTE_WAVES + wave;
    if (chunk >= n_chunks) return;
    volatile int32_t* next = next_lds + wave * E;
    for (int e = lane; e < E; e += 64)
        next[e] = slot_offsets[slot_of_expert[e]] + chunk_base[(size_t)chunk * E + e];
    for (int r = 0; r < ROUTE_CHUNK / 64; ++r) {
        const int a = chunk * ROUTE_CHUNK + r * 64 + lane;
        int e = -1;
        if (a < A) {
            e = idx[a];
            if (e < 0 || e >= E) e = -1;
        }
        unsigned long long active = __ballot(e >= 0);
        while (active) {
            const int leader = __ffsll((long long)active) - 1;
            const int e0 = __shfl(e, leader, 64);
            const unsigned long long m = __ballot(e == e0);
            const int base = next[e0];
            if (e == e0) {
                const int row = base + __popcll(m & lanemask_lt(lane));
                pos[a] = row;
                perm[row] = a;
            }
            if (lane == leader) next[e0] = base + __popcll(m);
            active &= ~m;
        }
    }
}

// Layout and positions in one launch, for the common case of few chunks: every block rebuilds the
// (small) layout from the counts and the placement in LDS, block 0 publishes it, and every wave gets
// the base of its chunk by summing the histograms of the chunks before it instead of reading a
// prefix table that a separate single-block launch would have to write first.
constexpr int FUSED_MAX_E = 64, FUSED_MAX_CHUNKS = 1024;

__global__ __launch_bounds__(ROUTE_WAVES * 64) void layout_positions_kernel(
    const int32_t* __restrict__ idx, const int32_t* __restrict__ expert_dest, const int32_t* __restrict__ counts,
    const int32_t* __restrict__ chunk_hist,
    int32_t* __restrict__ slot_of_expert, int32_t* __restrict__ slot_offsets,
    int32_t* __restrict__ dest_offsets, int32_t* __restrict__ dest_slots, int32_t* __restrict__ status,
    int32_t* __restrict__ pos, int32_t* __restrict__ perm, int A, int E, int P, int self, int Gcap, int n_chunks)
{
    __shared__ int32_t dest[FUSED_MAX_E], slot_of[FUSED_MAX_E], slot_cnt[FUSED_MAX_E], slot_off[FUSED_MAX_E + 1];
    __shared__ int32_t next_all[ROUTE_WAVES][FUSED_MAX_E];
    __shared__ int32_t flag;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int chunk = blockIdx.x * ROUTE_WAVES + wave;
    // every load that does not depend on the layout is issued first, so that the kernel pays one memory
    // round trip and not one per stage: placement and counts, this wave's assignments, and the histograms of
    // the chunks before it
    int my_dest = 0, my_count = 0;
    if (tid < E) { my_dest = expert_dest[tid]; my_count = counts[tid]; }
    int e_of[ROUTE_CHUNK / 64];
#pragma unroll
    for (int r = 0; r < ROUTE_CHUNK / 64; ++r) {
        const int a = chunk * ROUTE_CHUNK + r * 64 + lane;
        int e = -1;
        if (chunk < n_chunks && a < A) {
            e = idx[a];
            if (e < 0 || e >= E) e = -1;
        }
        e_of[r] = e;
    }
    // rows of every expert in the chunks before this one.  The histograms of those chunks are one flat array
    // of 16-byte pieces, q = E/4 per chunk; q divides 64, so a lane striding by 64 always meets the same four
    // experts and all of its loads are independent.
    const int q = E >> 2;
    int4 acc = make_int4(0, 0, 0, 0);
    if (chunk < n_chunks) {
        const int4* hp = reinterpret_cast<const int4*>(chunk_hist);
        const int n4 = chunk * q;
#pragma unroll 4
        for (int i = lane; i < n4; i += 64) {
            const int4 v = hp[i];
            acc.x += v.x; acc.y += v.y; acc.z += v.z; acc.w += v.w;
        }
    }

    if (tid == 0) flag = 0;
    __syncthreads();
    if (tid < E) {
        int p = my_dest;
        if (p < 0 || p >= P) { atomicOr(&flag, 1); p = p < 0 ? 0 : P - 1; }
        dest[tid] = p;
    }
    __syncthreads();
    if (tid < E) {                                          // slot = rank by (destination, id)
        const int p = dest[tid];
        int sl = 0;
        for (int f = 0; f < E; ++f) sl += (dest[f] < p) || (dest[f] == p && f < tid);
        slot_of[tid] = sl;
        slot_cnt[sl] = my_count;
    }
    __syncthreads();
    if (wave == 0) {                                        // exclusive scan of the slot counts (E <= 64: one wave)
        const int v = lane < E ? slot_cnt[lane] : 0;
        int incl = v;
        for (int off = 1; off < 64; off <<= 1) {
            const int up = __shfl_up(incl, off, 64);
            if (lane >= off) incl += up;
        }
        if (lane < E) slot_off[lane] = incl - v;
        if (lane == 63) slot_off[E] = incl;
    }
    __syncthreads();
    if (blockIdx.x == 0) {                                  // one block publishes the layout
        if (tid < E) slot_of_expert[tid] = slot_of[tid];
        if (tid <= E) slot_offsets[tid] = slot_off[tid];
        if (tid <= P) {
            int first = 0;
            for (int f = 0; f < E; ++f) first += (dest[f] < tid);
            dest_slots[tid] = first;
            dest_offsets[tid] = slot_off[first];
        }
        if (tid == 0) {
            int hosted = 0;
            for (int e = 0; e < E; ++e) hosted += (dest[e] == self);
            *status = (flag || hosted > Gcap) ? (int32_t)MOE_ERR_PLAN : (int32_t)MOE_OK;
        }
    }
    if (chunk >= n_chunks) return;
    for (int off = q; off < 64; off <<= 1) {
        acc.x += __shfl_xor(acc.x, off, 64); acc.y += __shfl_xor(acc.y, off, 64);
        acc.z += __shfl_xor(acc.z, off, 64); acc.w += __shfl_xor(acc.w, off, 64);
    }
    // lane e keeps the next free row of expert e (E <= 64); lanes 0..q-1 hold the sums of experts 4l..4l+3
    int32_t* nx = next_all[wave];
    if (lane < q) { nx[4 * lane + 0] = acc.x; nx[4 * lane + 1] = acc.y; nx[4 * lane + 2] = acc.z; nx[4 * lane + 3] = acc.w; }
    __builtin_amdgcn_wave_barrier();
    int next_row = 0;
    if (lane < E) next_row = slot_off[slot_of[lane]] + reinterpret_cast<volatile int32_t*>(nx)[lane];
    // One ballot per expert instead of one per distinct expert met: no data-dependent loop and nothing that
    // waits on LDS inside it.
#pragma unroll
    for (int r = 0; r < ROUTE_CHUNK / 64; ++r) {
        const int a = chunk * ROUTE_CHUNK + r * 64 + lane;
        const int e = e_of[r];
        unsigned long long mine = 0ull;
        int add = 0;
        for (int e0 = 0; e0 < E; ++e0) {
            const unsigned long long m = __ballot(e == e0);
            if (e == e0) mine = m;
            if (lane == e0) add = __popcll(m);
        }
        const int base = __shfl(next_row, e < 0 ? 0 : e, 64);
        if (e >= 0) {
            const int row = base + __popcll(mine & lanemask_lt(lane));
            pos[a] = row;
            perm[row] = a;
        }
        next_row += add;
    }
}

// Layout of the rows a device receives for the experts it hosts: the same slots as the local layout, the row
// offsets of the receive buffer instead of those of the send buffer.
__global__ void recv_layout_kernel(const int32_t* __restrict__ local_dest_slots, const int32_t* __restrict__ recv_offsets,
                                   int32_t* __restrict__ slot_offsets, int32_t* __restrict__ dest_slots, int E, int P, int self, int G)
{
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    const int first = local_dest_slots[self];
    if (i <= E) {
        int g = i - first;
        g = g < 0 ? 0 : (g > G ? G : g);
        slot_offsets[i] = recv_offsets[g];
    }
    if (i <= P) dest_slots[i] = local_dest_slots[i];
}

}  // namespace

hipError_t launch_chunk_hist(const moe_shape_t& s, const int32_t* idx, int32_t* chunk_hist, int n_chunks, hipStream_t st)
{
    if (n_chunks == 0) return hipSuccess;
    const int grid = (n_chunks + ROUTE_WAVES - 1) / ROUTE_WAVES;
    hipLaunchKernelGGL(chunk_hist_kernel, dim3(grid), dim3(ROUTE_WAVES * 64), (size_t)ROUTE_WAVES * s.E * sizeof(int32_t), st,
                       idx, chunk_hist, s.T * s.k, s.E, n_chunks);
    return hipGetLastError();
}

hipError_t launch_counts_from_hist(const moe_shape_t& s, const int32_t* chunk_hist, int n_chunks, int32_t* counts, hipStream_t st)
{
    const int waves = 4;
    hipLaunchKernelGGL(counts_from_hist_kernel, dim3((s.E + waves - 1) / waves), dim3(waves * 64), 0, st,
                       chunk_hist, n_chunks, s.E, counts);
    return hipGetLastError();
}

hipError_t launch_layout_scan(const moe_shape_t& s, const int32_t* expert_dest, const int32_t* counts,
                              const int32_t* chunk_hist, int32_t* chunk_base, int n_chunks,
                              const moe_layout_t& L, int32_t* status, hipStream_t st)
{
    const size_t lds = (size_t)(3 * s.E + 2) * sizeof(int32_t);
    hipLaunchKernelGGL(layout_scan_kernel, dim3(1), dim3(256), lds, st, expert_dest, counts, chunk_hist, chunk_base,
                       n_chunks, L.slot_of_expert, L.slot_offsets, L.dest_offsets, L.dest_slots, status,
                       s.E, s.P, s.self, s.G);
    return hipGetLastError();
}

hipError_t launch_positions(const moe_shape_t& s, const int32_t* idx, const int32_t* chunk_base, int n_chunks,
                            const moe_layout_t& L, hipStream_t st)
{
    if (n_chunks == 0) return hipSuccess;
    const int grid = (n_chunks + ROUTE_WAVES - 1) / ROUTE_WAVES;
    hipLaunchKernelGGL(positions_kernel, dim3(grid), dim3(ROUTE_WAVES * 64), (size_t)ROUTE_WAVES * s.E * sizeof(int32_t), st,
                       idx, chunk_base, L.slot_of_expert, L.slot_offsets, L.pos, L.perm, s.T * s.k, s.E, n_chunks);
    return hipGetLastError();
}

bool layout_positions_fusable(const moe_shape_t& s, int n_chunks)
{
    const bool e_ok = s.E >= 4 && s.E <= FUSED_MAX_E && (s.E & (s.E - 1)) == 0;      // a power of two: E/4 divides 64
    return e_ok && s.P <= ROUTE_WAVES * 64 - 1 && n_chunks >= 1 && n_chunks <= FUSED_MAX_CHUNKS;
}

hipError_t launch_layout_positions(const moe_shape_t& s, const int32_t* idx, const int32_t* expert_dest, const int32_t* counts,
                                   const int32_t* chunk_hist, int n_chunks, const moe_layout_t& L, int32_t* status, hipStream_t st)
{
    const int grid = (n_chunks + ROUTE_WAVES - 1) / ROUTE_WAVES;
    hipLaunchKernelGGL(layout_positions_kernel, dim3(grid), dim3(ROUTE_WAVES * 64), 0, st, idx, expert_dest, counts, chunk_hist,
                       L.slot_of_expert, L.slot_offsets, L.dest_offsets, L.dest_slots, status, L.pos, L.perm,
                       s.T * s.k, s.E, s.P, s.self, s.G, n_chunks);
    return hipGetLastError();
}

hipError_t launch_recv_layout(const moe_shape_t& s, const int32_t* local_dest_slots, const int32_t* recv_offsets,
                              int32_t* slot_offsets, int32_t* dest_slots, hipStream_t st)
{
    const int n = (s.E > s.P ? s.E : s.P) + 1;
    hipLaunchKernelGGL(recv_layout_kernel, dim3((n + 255) / 256), dim3(256), 0, st, local_dest_slots, recv_offsets,
                       slot_offsets, dest_slots, s.E, s.P, s.self, s.G);
    return hipGetLastError();
}


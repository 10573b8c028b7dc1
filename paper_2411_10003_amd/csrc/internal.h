// Internal declarations shared by the translation units of libmoehot (gfx950 only).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stddef.h>
#include <atomic>

#include "../../include/moehot.h"

struct moe_ctx {
    moe_shape_t s;
    // workspace layout (byte offsets, all multiples of 256)
    size_t off_status;     // int32 status word(s)
    size_t off_chunk_hist; // int32 [n_chunks][E] per-chunk expert histograms
    size_t off_chunk_base; // int32 [n_chunks][E] exclusive prefix over chunks
    size_t off_act;        // elt [A,h]  activation output A (forward) / recomputed A (backward)
    size_t off_dz;         // elt [A,h]  dZ
    size_t off_du;         // elt [A,h]  dU (SwiGLU)
    size_t off_gate_part;  // float [partitions][d*E + E] partial sums of the gate parameter gradients
    size_t off_split;      // float [SPLIT_UNITS][256*256] partial tiles of the grouped GEMM's last, K-split round (bf16 path)
    size_t ws_bytes;
    int n_chunks;          // ceil(A / ROUTE_CHUNK)
    // apart from this setting (moe_set_act_saved) a handle is immutable: every call is a function of its arguments
    int act_saved = 0;     // backward may read the activation the forward pass left in the workspace
};

// One-time set-up of a kernel per device (its dynamic LDS limit, the device's CU count).  The set-up
// calls are idempotent, so threads that race simply both make them; devices past 63 are set up on every call.
struct PerDeviceOnce {
    std::atomic<uint64_t> done{0};
    bool is_done(int dev) const { return dev >= 0 && dev < 64 && ((done.load(std::memory_order_acquire) >> dev) & 1u); }
    void mark(int dev) { if (dev >= 0 && dev < 64) done.fetch_or(1ull << dev, std::memory_order_release); }
};
inline int current_device() { int d = 0; if (hipGetDevice(&d) != hipSuccess) d = -1; return d; }

// Assignments handled by one wave of the routing kernels.
constexpr int ROUTE_CHUNK = 256;

typedef uint16_t bf16_t;  // storage only

// MOE_OK, or MOE_ERR_HIP with the error remembered for moe_last_hip_error() (per thread).
int moe_hip_status(hipError_t e);

// ---- launchers (each returns a hipError_t; they enqueue on `st`) ----------------------------
hipError_t launch_gate_topk(const moe_shape_t& s, const void* X, const float* Wg, const float* bg,
                            float* logits, int32_t* idx, float* w, hipStream_t st);
hipError_t launch_gate_bwd(const moe_shape_t& s, const float* dw, const float* logits, const int32_t* idx,
                           float* dlogits, hipStream_t st);

hipError_t launch_chunk_hist(const moe_shape_t& s, const int32_t* idx, int32_t* chunk_hist, int n_chunks, hipStream_t st);
hipError_t launch_counts_from_hist(const moe_shape_t& s, const int32_t* chunk_hist, int n_chunks, int32_t* counts, hipStream_t st);
hipError_t launch_layout_scan(const moe_shape_t& s, const int32_t* expert_dest, const int32_t* counts,
                              const int32_t* chunk_hist, int32_t* chunk_base, int n_chunks,
                              const moe_layout_t& L, int32_t* status, hipStream_t st);
hipError_t launch_positions(const moe_shape_t& s, const int32_t* idx, const int32_t* chunk_base, int n_chunks,
                            const moe_layout_t& L, hipStream_t st);

hipError_t launch_scatter_rows(const moe_shape_t& s, const void* X, const int32_t* pos, void* Xp, hipStream_t st);
hipError_t launch_combine(const moe_shape_t& s, const void* Yp, const int32_t* pos, const float* w, void* out, hipStream_t st);
hipError_t launch_combine_bwd(const moe_shape_t& s, const void* dOut, const void* Yp, const int32_t* pos,
                              const float* w, void* dYp, float* dw, hipStream_t st);
bool layout_positions_fusable(const moe_shape_t& s, int n_chunks);
hipError_t launch_layout_positions(const moe_shape_t& s, const int32_t* idx, const int32_t* expert_dest, const int32_t* counts,
                                   const int32_t* chunk_hist, int n_chunks, const moe_layout_t& L, int32_t* status, hipStream_t st);
int gate_grad_partitions(const moe_shape_t& s);
hipError_t launch_input_grad(const moe_shape_t& s, const void* dXp, const int32_t* pos, const float* dlogits,
                             const float* Wg, void* dX, hipStream_t st);
hipError_t launch_gate_wgrad(const moe_shape_t& s, const void* X, const float* dlogits, float* partial, float* partial_b,
                             float* dWg, float* dbg, hipStream_t st);
hipError_t launch_trans_gather(const moe_shape_t& s, const int32_t* expert_dest, const int32_t* pool_version,
                               const int32_t* slot_expert, const int32_t* slot_version,
                               const void* pool, void* groups, long bytes_per_expert, hipStream_t st);
hipError_t launch_trans_commit(const moe_shape_t& s, const int32_t* expert_dest, const int32_t* pool_version,
                               int32_t* slot_expert, int32_t* slot_version, hipStream_t st);
hipError_t launch_agg_add(const moe_shape_t& s, const int32_t* expert_dest, const float* groups, float* pool,
                          long floats_per_expert, hipStream_t st);
hipError_t launch_recv_layout(const moe_shape_t& s, const int32_t* local_dest_slots, const int32_t* recv_offsets,
                              int32_t* slot_offsets, int32_t* dest_slots, hipStream_t st);
hipError_t launch_plan(const moe_planner_t& cfg, const int32_t* gating, const moe_plan_out_t& out, hipStream_t st);
hipError_t launch_dispatch_bwd(const moe_shape_t& s, const void* dXp, const int32_t* pos, void* dX, hipStream_t st);

constexpr int SPLIT_UNITS = 320;       // partial tiles the K-split of a last round may need: at most one per block
struct ffn_args {
    const void *Xp, *W1, *W2, *W3;
    const int32_t *slot_offsets, *dest_slots;
    void *Yp, *Z, *U, *Act;            // forward outputs (Act in workspace)
    const void* dYp;                   // backward
    void *dXp, *dZ, *dU;               // dZ, dU in workspace
    float *dW1, *dW2, *dW3;
    bool accumulate = false;           // weight gradients are added to what dW holds instead of overwriting it
    bool act_saved = false;            // backward: Act still holds the forward pass's activation (not recomputed)
    float* split_ws = nullptr;         // workspace for K-split partial tiles (SPLIT_UNITS tiles of 256 x 256 floats)
};
hipError_t launch_ffn_fwd_f32(const moe_shape_t& s, const ffn_args& a, hipStream_t st);
hipError_t launch_ffn_bwd_f32(const moe_shape_t& s, const ffn_args& a, hipStream_t st);
hipError_t launch_ffn_fwd_bf16(const moe_shape_t& s, const ffn_args& a, hipStream_t st);
hipError_t launch_ffn_bwd_bf16(const moe_shape_t& s, const ffn_args& a, hipStream_t st);

// ---- small device helpers ----------------------------------------------------------------
__device__ __forceinline__ float bf16_to_f32(bf16_t v) { return __uint_as_float(((uint32_t)v) << 16); }
// Two floats to a pair of bf16, round-to-nearest-even, NaN stays NaN: the hardware conversion of gfx950
// (v_cvt_pk_bf16_f32), one instruction per pair instead of a dozen with a branch for the NaN case.
typedef __attribute__((ext_vector_type(2))) float moe_f32x2_t;
typedef __attribute__((ext_vector_type(2))) __bf16 moe_bf16x2_t;
__device__ __forceinline__ uint32_t pack_bf16x2(float lo, float hi) {
    const moe_f32x2_t v = {lo, hi};
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, moe_bf16x2_t));
}
__device__ __forceinline__ bf16_t f32_to_bf16(float f) { return (bf16_t)(pack_bf16x2(f, 0.0f) & 0xffffu); }

// Group table of the hosted slots, rebuilt by every FFN block from the layout (G is small).
__device__ __forceinline__ void hosted_range(const int32_t* dest_slots, int self, int Gcap, int& first_slot, int& n_groups) {
    first_slot = dest_slots[self];
    int n = dest_slots[self + 1] - first_slot;
    n_groups = n < Gcap ? n : Gcap;
    if (n_groups < 0) n_groups = 0;
}

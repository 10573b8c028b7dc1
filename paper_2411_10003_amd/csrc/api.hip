// Host side of the C ABI: argument checks, workspace carving and kernel sequencing.
// Nothing here synchronises or allocates device memory (moe_read_status excepted).
#include "internal.h"

#include <cmath>

#include <new>

namespace {

thread_local int g_last_hip_error = 0;

inline size_t align256(size_t x) { return (x + 255) & ~(size_t)255; }

inline int hip_status(hipError_t e)
{
    if (e == hipSuccess) return MOE_OK;
    g_last_hip_error = (int)e;
    return MOE_ERR_HIP;
}

inline size_t elt_size(const moe_shape_t& s) { return s.dtype == MOE_BF16 ? 2 : 4; }

int check_shape(const moe_shape_t& s)
{
    if (s.dtype != MOE_F32 && s.dtype != MOE_BF16) return MOE_ERR_DTYPE;
    if (s.act != MOE_ACT_GELU && s.act != MOE_ACT_SWIGLU) return MOE_ERR_SHAPE;
    if (s.T < 1 || s.d < 1 || s.h < 1) return MOE_ERR_SHAPE;
    if (s.k < 1 || s.k > 8 || s.E < s.k || s.E > 1024) return MOE_ERR_SHAPE;
    if (s.P < 1 || s.P > s.E || s.self < 0 || s.self >= s.P) return MOE_ERR_SHAPE;
    if (s.G < 1 || s.G > s.E) return MOE_ERR_SHAPE;
    if (s.renorm != 0 && s.renorm != 1) return MOE_ERR_SHAPE;
    if ((long long)s.T * s.k >= (1ll << 31) / 2) return MOE_ERR_SHAPE;
    if (s.dtype == MOE_BF16 && (s.d % 64 != 0 || s.h % 64 != 0)) return MOE_ERR_SHAPE;
    // the bf16 epilogues address a 256-row tile of an output with 32-bit byte offsets
    if (s.dtype == MOE_BF16 && (s.d >= (1 << 22) || s.h >= (1 << 22))) return MOE_ERR_SHAPE;
    if (s.dtype == MOE_BF16 && s.G > 64) return MOE_ERR_SHAPE;      // the grouped GEMM keeps one group per lane
    if (s.dtype == MOE_BF16 && (long long)s.d * s.h >= (1ll << 30)) return MOE_ERR_SHAPE;   // 32-bit byte offsets inside one weight matrix
    if (s.dtype == MOE_F32 && (s.d % 4 != 0)) return MOE_ERR_SHAPE;
    if (s.dtype == MOE_F32 && (long long)s.T * s.k > 16ll * 65535) return MOE_ERR_SHAPE;
    return MOE_OK;
}

inline bool misaligned(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 255) != 0; }

struct Carve {
    char* base;
    const moe_ctx* c;
    int32_t* status() const { return reinterpret_cast<int32_t*>(base + c->off_status); }
    int32_t* chunk_hist() const { return reinterpret_cast<int32_t*>(base + c->off_chunk_hist); }
    int32_t* chunk_base() const { return reinterpret_cast<int32_t*>(base + c->off_chunk_base); }
    void* act() const { return base + c->off_act; }
    void* dz() const { return base + c->off_dz; }
    void* du() const { return base + c->off_du; }
    float* gate_part() const { return reinterpret_cast<float*>(base + c->off_gate_part); }
    float* split() const { return c->s.dtype == MOE_BF16 ? reinterpret_cast<float*>(base + c->off_split) : nullptr; }
};

}  // namespace

int moe_hip_status(hipError_t e) { return hip_status(e); }

extern "C" {

int moe_create(moe_handle_t* out, const moe_shape_t* shape)
{
    if (!out || !shape) return MOE_ERR_NULL;
    const int rc = check_shape(*shape);
    if (rc != MOE_OK) return rc;
    moe_ctx* c = new (std::nothrow) moe_ctx();
    if (!c) return MOE_ERR_NULL;
    c->s = *shape;
    const size_t A = (size_t)shape->T * shape->k;
    c->n_chunks = (int)((A + ROUTE_CHUNK - 1) / ROUTE_CHUNK);
    size_t off = 0;
    c->off_status = off;      off += 256;
    c->off_chunk_hist = off;  off += align256((size_t)c->n_chunks * shape->E * sizeof(int32_t));
    c->off_chunk_base = off;  off += align256((size_t)c->n_chunks * shape->E * sizeof(int32_t));
    const size_t ah = align256(A * shape->h * elt_size(*shape));
    c->off_act = off;         off += ah;
    c->off_dz = off;          off += ah;
    c->off_du = off;          off += (shape->act == MOE_ACT_SWIGLU) ? ah : 0;
    c->off_gate_part = off;   off += align256((size_t)gate_grad_partitions(*shape) * ((size_t)shape->d * shape->E + shape->E) * sizeof(float));
    c->off_split = off;       off += (shape->dtype == MOE_BF16) ? align256((size_t)SPLIT_UNITS * 256 * 256 * sizeof(float)) : 0;
    c->ws_bytes = off;
    *out = c;
    return MOE_OK;
}

int moe_destroy(moe_handle_t h)
{
    if (!h) return MOE_ERR_NULL;
    delete h;
    return MOE_OK;
}

int moe_workspace_bytes(moe_handle_t h, size_t* bytes)
{
    if (!h || !bytes) return MOE_ERR_NULL;
    *bytes = h->ws_bytes;
    return MOE_OK;
}

const char* moe_status_string(int status)
{
    switch (status) {
        case MOE_OK: return "ok";
        case MOE_ERR_NULL: return "null pointer";
        case MOE_ERR_SHAPE: return "unsupported or inconsistent shape";
        case MOE_ERR_PLAN: return "expert placement out of range";
        case MOE_ERR_WORKSPACE: return "workspace missing or misaligned";
        case MOE_ERR_DTYPE: return "unsupported dtype";
        case MOE_ERR_UNIMPLEMENTED: return "not implemented";
        case MOE_ERR_HIP: return "HIP error";
        case MOE_ERR_TOO_LARGE: return "input exceeds the capacity of the built-in scratch array";
        default: return "unknown status";
    }
}

int moe_last_hip_error(void) { return g_last_hip_error; }

int moe_read_status(moe_handle_t h, const void* ws, void* stream, int* status)
{
    if (!h || !status) return MOE_ERR_NULL;
    if (!ws || misaligned(ws)) return MOE_ERR_WORKSPACE;
    int32_t v = 0;
    hipError_t e = hipMemcpyAsync(&v, (const char*)ws + h->off_status, sizeof(v), hipMemcpyDeviceToHost, (hipStream_t)stream);
    if (e == hipSuccess) e = hipStreamSynchronize((hipStream_t)stream);
    if (e != hipSuccess) return hip_status(e);
    *status = (int)v;
    return MOE_OK;
}

int moe_gate_topk(moe_handle_t h, const void* X, const float* Wg, const float* bg,
                  float* logits, int32_t* idx, float* w, void* stream)
{
    if (!h || !X || !Wg || !bg || !logits || !idx || !w) return MOE_ERR_NULL;
    return hip_status(launch_gate_topk(h->s, X, Wg, bg, logits, idx, w, (hipStream_t)stream));
}

int moe_expert_counts(moe_handle_t h, const int32_t* idx, int32_t* counts, void* ws, void* stream)
{
    if (!h || !idx || !counts) return MOE_ERR_NULL;
    if (!ws || misaligned(ws)) return MOE_ERR_WORKSPACE;
    const Carve c{(char*)ws, h};
    hipStream_t st = (hipStream_t)stream;
    hipError_t e = launch_chunk_hist(h->s, idx, c.chunk_hist(), h->n_chunks, st);
    if (e == hipSuccess) e = launch_counts_from_hist(h->s, c.chunk_hist(), h->n_chunks, counts, st);
    return hip_status(e);
}

// fresh_hist: the per-chunk histograms of this idx are already in the workspace (the caller says so)
static int dispatch_impl(moe_handle_t h, const int32_t* expert_dest, const void* X, const int32_t* idx,
                         const int32_t* counts, const moe_layout_t* L, void* Xp, void* ws, void* stream, bool fresh_hist)
{
    if (!h || !expert_dest || !X || !idx || !counts || !L || !Xp) return MOE_ERR_NULL;
    if (!L->slot_of_expert || !L->slot_offsets || !L->dest_offsets || !L->dest_slots || !L->pos || !L->perm)
        return MOE_ERR_NULL;
    if (!ws || misaligned(ws)) return MOE_ERR_WORKSPACE;
    const Carve c{(char*)ws, h};
    hipStream_t st = (hipStream_t)stream;
    hipError_t e = hipSuccess;
    if (!fresh_hist) e = launch_chunk_hist(h->s, idx, c.chunk_hist(), h->n_chunks, st);
    if (e == hipSuccess && layout_positions_fusable(h->s, h->n_chunks)) {
        e = launch_layout_positions(h->s, idx, expert_dest, counts, c.chunk_hist(), h->n_chunks, *L, c.status(), st);
    } else {
        if (e == hipSuccess)
            e = launch_layout_scan(h->s, expert_dest, counts, c.chunk_hist(), c.chunk_base(), h->n_chunks, *L, c.status(), st);
        if (e == hipSuccess) e = launch_positions(h->s, idx, c.chunk_base(), h->n_chunks, *L, st);
    }
    if (e == hipSuccess) e = launch_scatter_rows(h->s, X, L->pos, Xp, st);
    return hip_status(e);
}

int moe_dispatch(moe_handle_t h, const int32_t* expert_dest, const void* X, const int32_t* idx,
                 const int32_t* counts, const moe_layout_t* L, void* Xp, void* ws, void* stream)
{
    return dispatch_impl(h, expert_dest, X, idx, counts, L, Xp, ws, stream, false);
}

int moe_dispatch_after_counts(moe_handle_t h, const int32_t* expert_dest, const void* X, const int32_t* idx,
                              const int32_t* counts, const moe_layout_t* L, void* Xp, void* ws, void* stream)
{
    return dispatch_impl(h, expert_dest, X, idx, counts, L, Xp, ws, stream, true);
}

int moe_set_act_saved(moe_handle_t h, int saved)
{
    if (!h) return MOE_ERR_NULL;
    if (saved != 0 && saved != 1) return MOE_ERR_SHAPE;
    h->act_saved = saved;
    return MOE_OK;
}

int moe_expert_ffn_fwd(moe_handle_t h, const void* Xp, const moe_layout_t* L,
                       const void* W1, const void* W2, const void* W3,
                       void* Yp, void* Z, void* U, void* ws, void* stream)
{
    if (!h || !Xp || !L || !W1 || !W2 || !Yp) return MOE_ERR_NULL;
    if (!L->slot_offsets || !L->dest_slots) return MOE_ERR_NULL;
    const bool swiglu = h->s.act == MOE_ACT_SWIGLU;
    if (swiglu && !W3) return MOE_ERR_NULL;
    if (swiglu && ((Z == nullptr) != (U == nullptr))) return MOE_ERR_NULL;     // kept together or not at all
    if (!ws || misaligned(ws)) return MOE_ERR_WORKSPACE;
    const Carve c{(char*)ws, h};
    ffn_args a{};
    a.Xp = Xp; a.W1 = W1; a.W2 = W2; a.W3 = W3;
    a.slot_offsets = L->slot_offsets; a.dest_slots = L->dest_slots;
    a.Yp = Yp; a.Z = Z; a.U = U; a.Act = c.act(); a.split_ws = c.split();
    hipStream_t st = (hipStream_t)stream;
    return hip_status(h->s.dtype == MOE_F32 ? launch_ffn_fwd_f32(h->s, a, st) : launch_ffn_fwd_bf16(h->s, a, st));
}

int moe_combine(moe_handle_t h, const void* Yp, const int32_t* pos, const float* w, void* out, void* stream)
{
    if (!h || !Yp || !pos || !w || !out) return MOE_ERR_NULL;
    return hip_status(launch_combine(h->s, Yp, pos, w, out, (hipStream_t)stream));
}

int moe_combine_bwd(moe_handle_t h, const void* dOut, const void* Yp, const int32_t* pos, const float* w,
                    void* dYp, float* dw, void* stream)
{
    if (!h || !dOut || !Yp || !pos || !w || !dYp || !dw) return MOE_ERR_NULL;
    return hip_status(launch_combine_bwd(h->s, dOut, Yp, pos, w, dYp, dw, (hipStream_t)stream));
}

static int ffn_bwd_impl(moe_handle_t h, const void* dYp, const void* Xp, const void* Z, const void* U,
                        const moe_layout_t* L, const void* W1, const void* W2, const void* W3,
                        void* dXp, float* dW1, float* dW2, float* dW3, void* ws, void* stream, bool accumulate)
{
    if (!h || !dYp || !Xp || !Z || !L || !W1 || !W2 || !dXp || !dW1 || !dW2) return MOE_ERR_NULL;
    if (!L->slot_offsets || !L->dest_slots) return MOE_ERR_NULL;
    const bool swiglu = h->s.act == MOE_ACT_SWIGLU;
    if (swiglu && (!W3 || !U || !dW3)) return MOE_ERR_NULL;
    if (!ws || misaligned(ws)) return MOE_ERR_WORKSPACE;
    const Carve c{(char*)ws, h};
    ffn_args a{};
    a.Xp = Xp; a.W1 = W1; a.W2 = W2; a.W3 = W3;
    a.slot_offsets = L->slot_offsets; a.dest_slots = L->dest_slots;
    a.Z = const_cast<void*>(Z); a.U = const_cast<void*>(U); a.Act = c.act();
    a.dYp = dYp; a.dXp = dXp; a.dZ = c.dz(); a.dU = c.du();
    a.dW1 = dW1; a.dW2 = dW2; a.dW3 = dW3;
    a.accumulate = accumulate; a.split_ws = c.split();
    a.act_saved = h->act_saved != 0;
    hipStream_t st = (hipStream_t)stream;
    return hip_status(h->s.dtype == MOE_F32 ? launch_ffn_bwd_f32(h->s, a, st) : launch_ffn_bwd_bf16(h->s, a, st));
}

int moe_expert_ffn_bwd(moe_handle_t h, const void* dYp, const void* Xp, const void* Z, const void* U,
                       const moe_layout_t* L, const void* W1, const void* W2, const void* W3,
                       void* dXp, float* dW1, float* dW2, float* dW3, void* ws, void* stream)
{
    return ffn_bwd_impl(h, dYp, Xp, Z, U, L, W1, W2, W3, dXp, dW1, dW2, dW3, ws, stream, false);
}

int moe_expert_ffn_bwd_acc(moe_handle_t h, const void* dYp, const void* Xp, const void* Z, const void* U,
                           const moe_layout_t* L, const void* W1, const void* W2, const void* W3,
                           void* dXp, float* dW1, float* dW2, float* dW3, void* ws, void* stream)
{
    return ffn_bwd_impl(h, dYp, Xp, Z, U, L, W1, W2, W3, dXp, dW1, dW2, dW3, ws, stream, true);
}

int moe_dispatch_bwd(moe_handle_t h, const void* dXp, const int32_t* pos, void* dX, void* stream)
{
    if (!h || !dXp || !pos || !dX) return MOE_ERR_NULL;
    return hip_status(launch_dispatch_bwd(h->s, dXp, pos, dX, (hipStream_t)stream));
}

int moe_gate_bwd(moe_handle_t h, const float* dw, const float* logits, const int32_t* idx,
                 float* dlogits, void* stream)
{
    if (!h || !dw || !logits || !idx || !dlogits) return MOE_ERR_NULL;
    return hip_status(launch_gate_bwd(h->s, dw, logits, idx, dlogits, (hipStream_t)stream));
}

int moe_gate_bwd_params(moe_handle_t h, const void* X, const float* dlogits, float* dWg, float* dbg, void* ws, void* stream)
{
    if (!h || !X || !dlogits || !dWg || !dbg) return MOE_ERR_NULL;
    if (!ws || misaligned(ws)) return MOE_ERR_WORKSPACE;
    const Carve c{(char*)ws, h};
    float* part = c.gate_part();
    float* part_b = part + (size_t)gate_grad_partitions(h->s) * h->s.d * h->s.E;
    return hip_status(launch_gate_wgrad(h->s, X, dlogits, part, part_b, dWg, dbg, (hipStream_t)stream));
}

int moe_input_grad(moe_handle_t h, const void* dXp, const int32_t* pos, const float* dlogits, const float* Wg,
                   void* dX, void* stream)
{
    if (!h || !dXp || !pos || !dlogits || !Wg || !dX) return MOE_ERR_NULL;
    return hip_status(launch_input_grad(h->s, dXp, pos, dlogits, Wg, dX, (hipStream_t)stream));
}

int moe_trans(moe_handle_t h, const int32_t* expert_dest, const int32_t* pool_version, int32_t* slot_expert,
              int32_t* slot_version, int n_tensors, const void* const* pools, void* const* groups,
              const size_t* bytes_per_expert, void* stream)
{
    if (!h || !expert_dest || !slot_expert || !pools || !groups || !bytes_per_expert) return MOE_ERR_NULL;
    if ((pool_version == nullptr) != (slot_version == nullptr)) return MOE_ERR_NULL;       // both or neither
    if (n_tensors < 1 || n_tensors > 8) return MOE_ERR_SHAPE;
    for (int i = 0; i < n_tensors; ++i) {
        if (!pools[i] || !groups[i]) return MOE_ERR_NULL;
        if (bytes_per_expert[i] == 0 || bytes_per_expert[i] % 16 != 0) return MOE_ERR_SHAPE;
        if ((reinterpret_cast<uintptr_t>(pools[i]) | reinterpret_cast<uintptr_t>(groups[i])) & 15) return MOE_ERR_SHAPE;
    }
    hipStream_t st = (hipStream_t)stream;
    hipError_t e = hipSuccess;
    for (int i = 0; i < n_tensors && e == hipSuccess; ++i)
        e = launch_trans_gather(h->s, expert_dest, pool_version, slot_expert, slot_version, pools[i], groups[i],
                                (long)bytes_per_expert[i], st);
    if (e == hipSuccess) e = launch_trans_commit(h->s, expert_dest, pool_version, slot_expert, slot_version, st);
    return hip_status(e);
}

int moe_agg(moe_handle_t h, const int32_t* expert_dest, int n_tensors, const float* const* group_grads,
            float* const* pool_grads, const size_t* floats_per_expert, void* stream)
{
    if (!h || !expert_dest || !group_grads || !pool_grads || !floats_per_expert) return MOE_ERR_NULL;
    if (n_tensors < 1 || n_tensors > 8) return MOE_ERR_SHAPE;
    for (int i = 0; i < n_tensors; ++i) {
        if (!group_grads[i] || !pool_grads[i]) return MOE_ERR_NULL;
        if (floats_per_expert[i] == 0 || floats_per_expert[i] % 4 != 0) return MOE_ERR_SHAPE;
        if ((reinterpret_cast<uintptr_t>(group_grads[i]) | reinterpret_cast<uintptr_t>(pool_grads[i])) & 15) return MOE_ERR_SHAPE;
    }
    hipError_t e = hipSuccess;
    for (int i = 0; i < n_tensors && e == hipSuccess; ++i)
        e = launch_agg_add(h->s, expert_dest, group_grads[i], pool_grads[i], (long)floats_per_expert[i], (hipStream_t)stream);
    return hip_status(e);
}

int moe_recv_layout(moe_handle_t h, const moe_layout_t* local, const int32_t* recv_offsets, const moe_layout_t* out, void* stream)
{
    if (!h || !local || !recv_offsets || !out) return MOE_ERR_NULL;
    if (!local->dest_slots || !out->slot_offsets || !out->dest_slots) return MOE_ERR_NULL;
    return hip_status(launch_recv_layout(h->s, local->dest_slots, recv_offsets, out->slot_offsets, out->dest_slots, (hipStream_t)stream));
}

int moe_plan(const moe_planner_t* cfg, const int32_t* gating, const moe_plan_out_t* out, void* stream)
{
    if (!cfg || !gating || !out) return MOE_ERR_NULL;
    if (!out->expert_dest || !out->selected || !out->skipped || !out->H || !out->R || !out->times || !out->info) return MOE_ERR_NULL;
    const moe_planner_t& c = *cfg;
    if (c.D < 1 || c.D > 64 || c.E < c.D || c.E > 1024 || c.E % c.D != 0) return MOE_ERR_SHAPE;
    if (c.n < 0 || c.n > c.D - 1 || (c.overlap != 0 && c.overlap != 1)) return MOE_ERR_SHAPE;
    const double pos[] = {c.B, c.t}, nonneg[] = {c.alpha, c.size_input, c.size_params, c.size_grads, c.T_FNEC, c.T_BNEC};
    for (double v : pos) if (!(v > 0.0) || !std::isfinite(v)) return MOE_ERR_SHAPE;
    for (double v : nonneg) if (!(v >= 0.0) || !std::isfinite(v)) return MOE_ERR_SHAPE;
    return hip_status(launch_plan(c, gating, *out, (hipStream_t)stream));
}

}  // extern "C"

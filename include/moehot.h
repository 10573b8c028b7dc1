/*
 * moehot.h -- C ABI of libmoehot: one GPU's share of an expert-parallel MoE layer on MI355X.
 *
 * The calls follow the workflow of an expert-parallel MoE layer as the Pro-Prophet paper
 * (arXiv 2411.10003) states it: the gate routes every input to its top-k experts (Section 2.1),
 * the number of inputs per expert is the "input distribution" the planner consumes (Section 3),
 * inputs are exchanged by an all-to-all according to an expert placement in which a device that
 * holds an expert's parameters computes its local inputs itself (Section 4.1), every device runs
 * the expert computation over the inputs it hosts (Section 4.2, Eq. 2-3), and a second all-to-all
 * returns the results to the inputs' original positions (Section 2.1, Fig. 2).  On one GPU the
 * all-to-all destinations are only a buffer layout.
 *
 * Conventions
 *   - Every pointer is DEVICE memory owned by the caller unless marked "host".  The library
 *     allocates no device memory; scratch comes from the caller's workspace (moe_workspace_bytes).
 *   - `stream` is a hipStream_t passed as void*.  Calls only enqueue work on it; they never
 *     synchronise and never read device data on the host (moe_read_status excepted).
 *   - Arguments are checked on the host before anything is launched.  Return value: MOE_OK or a
 *     negative moe_status_t; on an error nothing has been enqueued.
 *   - Outputs are overwritten, never accumulated into (the one exception, moe_expert_ffn_bwd_acc, says so in
 *     its name and adds to its weight gradients only).  Same inputs give the same bits.
 *   - A handle is an immutable description of the problem (moe_set_act_saved is its one setting): calls keep
 *     no state in it between them, so one handle may be used from several threads as long as calls that share
 *     a workspace do not overlap and moe_set_act_saved is not called while another call is running.
 *   - Row-major everywhere.  "elt" is the activation type of the handle: float (MOE_F32) or
 *     bfloat16 (MOE_BF16, upper half of an IEEE float, round-to-nearest-even).  Gate parameters,
 *     logits, gate weights and weight gradients are always float; indices are int32_t.
 *   - Notation: T tokens, d model width, h hidden width, E experts, k experts per token,
 *     P destinations, A = T*k assignments with id a = t*k + j, G hosted weight groups.
 *   - Calls that share a workspace must not overlap in time.
 */
#ifndef MOEHOT_H
#define MOEHOT_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    MOE_OK = 0,
    MOE_ERR_NULL = -1,          /* a required pointer is NULL */
    MOE_ERR_SHAPE = -2,         /* unsupported or inconsistent sizes */
    MOE_ERR_PLAN = -3,          /* placement out of range (reported by moe_read_status) */
    MOE_ERR_WORKSPACE = -4,     /* workspace missing or misaligned */
    MOE_ERR_DTYPE = -5,
    MOE_ERR_UNIMPLEMENTED = -6,
    MOE_ERR_HIP = -7,           /* a HIP call failed; see moe_last_hip_error() */
    MOE_ERR_TOO_LARGE = -8      /* moe_expert_counts_static: the input needs more than the built-in scratch array */
} moe_status_t;

typedef enum { MOE_F32 = 0, MOE_BF16 = 1 } moe_dtype_t;
typedef enum { MOE_ACT_GELU = 0, MOE_ACT_SWIGLU = 1 } moe_act_t;

/* Problem description, fixed per handle.
 *   self   : destination id of this GPU in [0, P).
 *   G      : capacity of the hosted weight arrays (owned + replicated experts), 1 <= G <= E.
 *   renorm : 1 = the k gate weights of a token are renormalised to sum to one.
 * Limits: 1 <= k <= 8, k <= E <= 1024, 1 <= P <= E; MOE_BF16 needs d % 64 == 0, h % 64 == 0,
 * G <= 64 (hosted weight groups), d*h < 2^30 (one weight matrix under 2 GiB) and d, h < 2^22;
 * T*k < 2^30; T*k*max(d, h) may exceed 2^31 (row offsets are 64-bit). */
typedef struct {
    int T, d, h, E, k, P, self, G;
    moe_dtype_t dtype;
    moe_act_t act;
    int renorm;
} moe_shape_t;

/* Send layout produced by moe_dispatch (all device pointers, int32_t):
 *   slot_of_expert[E]  slot index of each expert; slots are the experts ordered by
 *                      (expert_dest[e], e), so a destination's slots and rows are contiguous
 *   slot_offsets[E+1]  first row of each slot; slot_offsets[E] = A
 *   dest_offsets[P+1]  first row of each destination (the all-to-all send displacements)
 *   dest_slots[P+1]    first slot of each destination
 *   pos[A]             row of assignment a (stable: ascending a inside a slot)
 *   perm[A]            assignment held by each row; perm[pos[a]] = a
 * The hosted groups are the slots dest_slots[self] .. dest_slots[self+1]-1, in that order
 * (ascending expert id); group g uses W*[g].  At most G groups are computed. */
typedef struct {
    int32_t* slot_of_expert;
    int32_t* slot_offsets;
    int32_t* dest_offsets;
    int32_t* dest_slots;
    int32_t* pos;
    int32_t* perm;
} moe_layout_t;

typedef struct moe_ctx* moe_handle_t;

/* Create / destroy a handle (host objects only).  *out is written on success. */
int moe_create(moe_handle_t* out, const moe_shape_t* shape);
int moe_destroy(moe_handle_t h);

/* Bytes of workspace every call below may use (256-byte aligned device memory). */
int moe_workspace_bytes(moe_handle_t h, size_t* bytes);

const char* moe_status_string(int status);
/* Last hipError_t seen by this thread's calls, as an int (0 = hipSuccess). */
int moe_last_hip_error(void);

/* Synchronises `stream` and copies the device-side status word of the workspace to *status (host):
 * MOE_OK, or MOE_ERR_PLAN if the last moe_dispatch saw expert_dest outside [0,P) or more than G
 * hosted experts.  The only call that blocks. */
int moe_read_status(moe_handle_t h, const void* ws, void* stream, int* status);

/* Gate and routing (Section 2.1: the gate relates an input to all experts and routes it to the
 * top-k).  logits[t,e] = bg[e] + sum_c X[t,c] * Wg[c,e] in fp32 with a fixed summation order
 * (two partial sums fed by alternating blocks of 32 columns; inside a block the columns are visited
 * as 8q + j, j = 0..7 outer, q = 0..3 inner, one fused multiply-add each; logit = (s0 + s1) + bias)
 * so that routing is reproducible bit for bit.  This order is part of the interface: it is frozen, and any
 * kernel behind this call has to reproduce it.  idx[t,0..k) = the k largest logits, best
 * first, ties to the lowest index, NaN ranked as -inf.  p = softmax(logits[t,:]);
 * w[t,j] = p[idx[t,j]], divided by their sum over j when renorm = 1.
 *   in : X[T,d] elt, Wg[d,E] float, bg[E] float
 *   out: logits[T,E] float, idx[T,k] int32, w[T,k] float */
int moe_gate_topk(moe_handle_t h, const void* X, const float* Wg, const float* bg,
                  float* logits, int32_t* idx, float* w, void* stream);

/* Input distribution (Section 3: the number of inputs each expert processes; what the planner's
 * search consumes).  in: idx[A]; out: counts[E].  Uses the workspace. */
int moe_expert_counts(moe_handle_t h, const int32_t* idx, int32_t* counts, void* ws, void* stream);

/* moe_expert_counts for callers that cannot allocate or pass a workspace: code under HIP graph capture,
 * tight serving loops, harnesses that forbid hipMalloc.  Same inputs, same output, same kernels; the
 * per-chunk histograms live in an array built into the library (4 MiB of device memory per GPU the library
 * runs on, held until the process ends) instead of the workspace.  The call allocates and frees nothing.
 *   limit: ceil(T*k / 256) * E <= 2^20 words, else MOE_ERR_TOO_LARGE and nothing is enqueued
 *   Every call on a GPU uses that GPU's one array: calls that overlap in time on one GPU (two streams, two
 *   threads) race.  The array keeps the last call's contents; every word a call reads it has written first,
 *   so nothing needs clearing between calls. */
int moe_expert_counts_static(moe_handle_t h, const int32_t* idx, int32_t* counts, void* stream);

/* Placement-aware send buffer (Section 4.1: inputs of an expert whose parameters are on this
 * device are computed locally, the others go to the expert's owner; Fig. 2: first all-to-all).
 *   in : expert_dest[E] int32 in [0,P): destination that computes this GPU's inputs of expert e
 *        (== self for owned and replicated experts); X[T,d] elt; idx[A]; counts[E] as returned by
 *        moe_expert_counts for the same idx
 *   out: every array of *layout (host struct of device pointers); Xp[A,d] elt with
 *        Xp[r,:] = X[perm[r] / k, :] (bit copies)
 * Uses the workspace (it rebuilds the per-chunk histograms of idx there; nothing is carried over from
 * earlier calls). */
int moe_dispatch(moe_handle_t h, const int32_t* expert_dest, const void* X, const int32_t* idx,
                 const int32_t* counts, const moe_layout_t* layout, void* Xp, void* ws, void* stream);

/* As moe_dispatch, for the usual sequence counts -> plan -> dispatch: the caller states that the routing
 * part of `ws` still holds what moe_expert_counts(h, idx, counts, ws) left there, i.e. that call was made
 * with this idx, this workspace and a handle of the same T, k and E, idx has not been rewritten since, and
 * no other moe_expert_counts / moe_dispatch* call has used this workspace in between.  The histograms are
 * then not rebuilt.  If the statement is false the layout is wrong and no error is reported: when in
 * doubt call moe_dispatch. */
int moe_dispatch_after_counts(moe_handle_t h, const int32_t* expert_dest, const void* X, const int32_t* idx,
                              const int32_t* counts, const moe_layout_t* layout, void* Xp, void* ws, void* stream);

/* Forward expert computation over the hosted groups (Section 4.2, Eq. 2), ragged and possibly
 * empty, without padding:  GELU: Yp = gelu(Xp W1) W2;  SwiGLU: Yp = (silu(Xp W1) * (Xp W3)) W2,
 * gelu(z) = z/2 (1 + erf(z/sqrt 2)), silu(z) = z / (1 + exp(-z)), fp32 accumulation.
 *   in : Xp[A,d] elt; layout (slot_offsets, dest_slots are read); W1[G,d,h], W2[G,h,d] elt,
 *        W3[G,d,h] elt for SwiGLU (NULL otherwise)
 *   out: rows of the hosted groups only: Yp[A,d] elt, Z[A,h] elt (= Xp W1, kept for backward),
 *        U[A,h] elt (= Xp W3, SwiGLU only, else NULL).  Other rows are not touched.
 * Forward only (inference): Z = NULL and U = NULL; the pre-activations are then not written (a third of the
 * first contraction's stores for GELU, two thirds for SwiGLU) and Yp holds the same bits as with them.  Z and U
 * are given or left out together (MOE_ERR_NULL otherwise); a backward call needs a forward call that kept them. */
int moe_expert_ffn_fwd(moe_handle_t h, const void* Xp, const moe_layout_t* layout,
                       const void* W1, const void* W2, const void* W3,
                       void* Yp, void* Z, void* U, void* ws, void* stream);

/* Weighted return (Fig. 2: second all-to-all, then the sum at the input's original position):
 * out[t,:] = sum_j w[t,j] * Yp[pos[t*k+j],:], fp32 accumulation in ascending j, rounded once.
 *   in : Yp[A,d] elt (rows of other destinations are what the return all-to-all delivered),
 *        pos[A], w[T,k] float;  out: out[T,d] elt */
int moe_combine(moe_handle_t h, const void* Yp, const int32_t* pos, const float* w, void* out, void* stream);

/* Gradient of moe_combine: dYp[pos[a],:] = w[a] * dOut[t,:];  dw[t,j] = <dOut[t,:], Yp[pos[a],:]>.
 *   in : dOut[T,d] elt, Yp[A,d] elt, pos[A], w[T,k];  out: dYp[A,d] elt, dw[T,k] float */
int moe_combine_bwd(moe_handle_t h, const void* dOut, const void* Yp, const int32_t* pos, const float* w,
                    void* dYp, float* dw, void* stream);

/* Backward expert computation over the hosted groups (Section 4.2, Eq. 3).  With A = act(Z)(*U)
 * and dA = dYp W2^T:   GELU: dZ = dA * gelu'(Z);   SwiGLU: dU = dA * silu(Z), dZ = dA * U * silu'(Z);
 * dXp = dZ W1^T (+ dU W3^T);  dW1 = Xp^T dZ, dW3 = Xp^T dU, dW2 = A^T dYp, each over the group's rows.
 *   in : dYp[A,d], Xp[A,d], Z[A,h], U[A,h] (SwiGLU) elt; layout; W1, W2, W3 as in the forward call
 *   out: dXp[A,d] elt, rows of hosted groups only; dW1[G,d,h], dW2[G,h,d], dW3[G,d,h] float,
 *        written for all G groups (zeros for an empty or unused group)
 * The activation A is not a saved tensor: by default it is recomputed from Z (and U) into the workspace.
 * See moe_set_act_saved. */
int moe_expert_ffn_bwd(moe_handle_t h, const void* dYp, const void* Xp, const void* Z, const void* U,
                       const moe_layout_t* layout, const void* W1, const void* W2, const void* W3,
                       void* dXp, float* dW1, float* dW2, float* dW3, void* ws, void* stream);

/* saved = 1: the caller states that, whenever moe_expert_ffn_bwd(_acc) is called with this handle, the
 * workspace it is given still holds the activation A that moe_expert_ffn_fwd wrote there for the same rows
 * (same handle shape, same layout, same Xp and weights, and no other call has used that workspace since):
 * a layer that keeps its workspace from its forward to its backward pass.  The backward pass then reads A
 * instead of recomputing and rewriting it (a third of the bytes its first contraction writes).  saved = 0
 * (the default): A is recomputed from Z and U, and the workspace may be shared freely between calls.
 * MOE_F32 handles ignore the setting. */
int moe_set_act_saved(moe_handle_t h, int saved);

/* As moe_expert_ffn_bwd, but the weight gradients are added to what dW1, dW2, dW3 hold (all G groups;
 * an empty group adds zero): the form in which a device folds the gradient of a replicated expert into a
 * buffer that already holds another contribution, as the Agg primitive does across devices (Section 4.1),
 * and the form gradient accumulation over micro-batches needs.  dXp is overwritten as before. */
int moe_expert_ffn_bwd_acc(moe_handle_t h, const void* dYp, const void* Xp, const void* Z, const void* U,
                           const moe_layout_t* layout, const void* W1, const void* W2, const void* W3,
                           void* dXp, float* dW1, float* dW2, float* dW3, void* ws, void* stream);

/* Gradient of the send (the backward all-to-all of the dispatch): dX[t,:] = sum_j dXp[pos[t*k+j],:],
 * the expert-path gradient of the layer input.  in: dXp[A,d] elt, pos[A];  out: dX[T,d] elt */
int moe_dispatch_bwd(moe_handle_t h, const void* dXp, const int32_t* pos, void* dX, void* stream);

/* Gradient of the gate weights with respect to the logits, selection held fixed.
 *   renorm = 0: dlogits[t,e] = sum_j dw[t,j] p[s_j] ((e == s_j) - p[e])
 *   renorm = 1: dlogits[t,s_j] = w_j (dw_j - sum_i w_i dw_i), zero elsewhere
 *   in : dw[T,k] float, logits[T,E] float, idx[T,k];  out: dlogits[T,E] float */
int moe_gate_bwd(moe_handle_t h, const float* dw, const float* logits, const int32_t* idx,
                 float* dlogits, void* stream);

/* Gradients of the gate's parameters (the gate network of Section 2.1 is the linear map
 * logit[t,e] = bg[e] + sum_c X[t,c] Wg[c,e]):  dWg[c,e] = sum_t X[t,c] dlogits[t,e],  dbg[e] = sum_t dlogits[t,e].
 * fp32 sums in a fixed order (same bits every run).  Uses the workspace.
 *   in : X[T,d] elt, dlogits[T,E] float;  out: dWg[d,E] float, dbg[E] float */
int moe_gate_bwd_params(moe_handle_t h, const void* X, const float* dlogits, float* dWg, float* dbg,
                        void* ws, void* stream);

/* Complete gradient of the layer input: the backward of the send (as moe_dispatch_bwd) plus the gate
 * path, rounded once:  dX[t,:] = sum_j dXp[pos[t*k+j],:] + sum_e dlogits[t,e] Wg[:,e].
 *   in : dXp[A,d] elt, pos[A], dlogits[T,E] float, Wg[d,E] float;  out: dX[T,d] elt */
int moe_input_grad(moe_handle_t h, const void* dXp, const int32_t* pos, const float* dlogits, const float* Wg,
                   void* dX, void* stream);

/* Receive side (Eq. 2: H_i counts every input a device computes, its own and those the first all-to-all
 * delivers for the experts it owns).  The received rows of hosted group g lie in a receive buffer at rows
 * [recv_offsets[g], recv_offsets[g+1]); this call writes the two arrays of *out that the expert computation
 * reads (slot_offsets[E+1], dest_slots[P+1]) so that moe_expert_ffn_fwd / _bwd run over the receive buffer with
 * the same weight groups as over the send buffer: call them once per buffer, the second backward as
 * moe_expert_ffn_bwd_acc so that the weight gradients of both add up.
 *   in : local (the layout moe_dispatch wrote; dest_slots is read), recv_offsets[G+1] int32 device, non-decreasing,
 *        constant from the number of hosted groups on
 *   out: out->slot_offsets, out->dest_slots (the other members of *out are not touched)
 * The handle of the receive-side calls has the same E, P, self, G, d, h, dtype and act as the local one; its
 * T * k bounds the rows of the receive buffer. */
int moe_recv_layout(moe_handle_t h, const moe_layout_t* local, const int32_t* recv_offsets, const moe_layout_t* out,
                    void* stream);

/* Trans on one GPU (Section 4.1: the parameters of a selected expert are transferred to the devices that
 * compute its inputs; Section 5.1: an expert's parameters are updated before every such transfer).  With the
 * parameters of all E experts in pools in this GPU's memory, the transfer is a gather of the hosted experts
 * into the G group slots that moe_expert_ffn_fwd/bwd read, driven by the plan as it lies in device memory:
 * group g receives the g-th expert e (ascending) with expert_dest[e] == self.  A slot is not copied again
 * when it already holds that expert in the pool's current version.
 *   in    : expert_dest[E] int32 (device); pool_version[E] int32 (device): a number per expert that the caller
 *           changes whenever it has updated that expert's parameters in the pools (an optimizer step);
 *           n_tensors (1..8) and, on the HOST, arrays of n_tensors device pointers pools[i] ([E] experts of
 *           bytes_per_expert[i] bytes each, a multiple of 16, 16-byte aligned)
 *   in/out: slot_expert[G] int32 (device): the expert each slot holds, -1 for none; slot_version[G] int32
 *           (device): the version it was copied at; both updated after the copies
 *   out   : groups[i] ([G] slots of bytes_per_expert[i] bytes); slots beyond the hosted experts keep their contents
 * pool_version and slot_version may both be NULL: then every hosted slot is copied on every call.
 * More hosted experts than G is the caller's error (moe_dispatch reports it through moe_read_status). */
int moe_trans(moe_handle_t h, const int32_t* expert_dest, const int32_t* pool_version, int32_t* slot_expert,
              int32_t* slot_version, int n_tensors, const void* const* pools, void* const* groups,
              const size_t* bytes_per_expert, void* stream);

/* Agg on one GPU (Section 4.1: the gradients computed for a replicated expert are aggregated where the expert's
 * parameters live).  The inverse walk of moe_trans: the weight gradient of hosted group g, as moe_expert_ffn_bwd
 * wrote it, is ADDED to the entry of the g-th expert e (ascending) with expert_dest[e] == self in a pool of
 * per-expert gradients, so that gradients keep accumulating per expert while the plan, and with it the meaning of
 * a group slot, changes from one iteration to the next.
 *   in    : expert_dest[E] int32 (device); n_tensors (1..8) and, on the HOST, arrays of n_tensors device pointers
 *           group_grads[i] ([G] slots of floats_per_expert[i] floats, a multiple of 4, 16-byte aligned)
 *   in/out: pool_grads[i] ([E] experts of floats_per_expert[i] floats): pool[e] += group[g]; other experts untouched
 * Fixed order of additions (one per element): same bits every run. */
int moe_agg(moe_handle_t h, const int32_t* expert_dest, int n_tensors, const float* const* group_grads,
            float* const* pool_grads, const size_t* floats_per_expert, void* stream);

/* ---- planner (Sections 4.2-4.3 and 5.3 of the paper) ------------------------------------------
 *
 * moe_plan runs the paper's greedy search for a lightweight expert placement (Algorithm 1) on the
 * GPU, in one wavefront, from the matrix of routing counts of all devices, so that the plan of the
 * next iteration can be produced without the host reading any counts.  A placement is evaluated
 * with the performance model T'(R, H, s, n) = 4 T_A2A(R) + 3 T_FEC(H) + T_Trans(s, n) + T_Agg(s, n)
 * (Eqs. 1-6) or, with overlap = 1, with Trans and Agg reduced by the computation the scheduler hides
 * them behind (Eq. 8); the search runs while max(H) - min(H) >= alpha I / E (Eq. 7).
 *
 * Where Algorithm 1 is silent: loads are computed before the first evaluation; expert e belongs to
 * device e / (E/D); the heaviest device (ties: lowest index) contributes its unselected expert with
 * the most inputs (ties: lowest id) and the search stops when it has none left (the paper's
 * "i in Used" when E = D); the n devices that are skipped are the non-owners with the fewest inputs
 * of the expert (ties: lowest index); times are IEEE doubles, a new placement is kept only if its
 * time is strictly smaller.
 */
typedef struct {
    int D, E;                   /* devices, experts; 1 <= D <= 64, E <= 1024, E % D == 0 */
    int n;                      /* devices a selected expert is not transferred to, 0 <= n <= D-1 */
    int overlap;                /* 0: Eq. 6;  1: Eq. 8 */
    double alpha;               /* coefficient of the balance test, Eq. 7 */
    double size_input;          /* bytes of one input */
    double size_params;         /* bytes of one expert's parameters */
    double size_grads;          /* bytes of one expert's gradients */
    double B;                   /* average communication bandwidth, bytes/s, > 0 */
    double t;                   /* computation throughput, inputs/s, > 0 */
    double T_FNEC, T_BNEC;      /* forward/backward time of the non-MoE layer, s (Eq. 8 only) */
} moe_planner_t;

/* Outputs of moe_plan (all device memory, all written by every call):
 *   expert_dest[D][E] : row j is device j's plan in the form moe_dispatch takes: j where device j
 *                       holds the expert (owner or replica), the owner elsewhere
 *   selected[E]       : experts in the order the search selected them, -1 after the last
 *   skipped[E]        : bit j of entry r is set when device j does not receive the r-th selected expert
 *   H[D], R[D]        : inputs computed / received per device under the returned placement
 *   times[2 + E]      : T' without a placement, T' of the returned placement, T' after each selection
 *   info[2]           : cnt (selections kept in the placement), s (selections made by the search) */
typedef struct {
    int32_t* expert_dest;
    int32_t* selected;
    uint64_t* skipped;
    int64_t* H;
    int64_t* R;
    double* times;
    int32_t* info;
} moe_plan_out_t;

/* in: cfg (host), gating[D][E] int32 (device): inputs on device i routed to expert e, each >= 0
 * out: see moe_plan_out_t (struct on the host, pointers to device memory).
 * Errors: MOE_ERR_NULL, MOE_ERR_SHAPE (sizes, n, non-positive or non-finite model constants). */
int moe_plan(const moe_planner_t* cfg, const int32_t* gating, const moe_plan_out_t* out, void* stream);

/* ---- calibration (for the benchmark; nothing of the layer's path calls these) -----------------------------
 * moe_calib_copy: dst[0..bytes) = src[0..bytes) by a plain streaming kernel (device pointers, 16-byte aligned,
 * bytes a multiple of 16): what a copy sustains on this GPU, to set beside the published HBM bandwidth.
 * moe_calib_mfma: one block of 8 wavefronts per compute unit, every wavefront issues iters x 8 bf16 32x32x16
 * matrix instructions (32768 flop each) on operands held in registers: what the matrix cores sustain at this
 * GPU's power limit, to set beside the published peak.  out: device, out_floats floats of which the first
 * blocks x threads are written (so that the work cannot be optimised away; MOE_ERR_SHAPE if there are fewer:
 * 512 per compute unit are enough); *blocks and *threads (host) receive the launch shape.
 * moe_calib_round_bf16: out[i] = in[i] rounded to bf16 exactly as every bf16 output of the library is rounded
 * (round to nearest, ties to even; NaN stays NaN): n floats in, n 16-bit words out, device pointers. */
int moe_calib_copy(const void* src, void* dst, size_t bytes, void* stream);
int moe_calib_mfma(float* out, size_t out_floats, int iters, int* blocks, int* threads, void* stream);
int moe_calib_round_bf16(const float* in, uint16_t* out, size_t n, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* MOEHOT_H */

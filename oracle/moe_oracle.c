/*
 * moe_oracle.c -- TEST INFRASTRUCTURE, NOT PART OF THE PRODUCT.
 *
 * A plain, slow CPU statement of what one GPU's share of an expert-parallel MoE layer
 * computes: gate and top-k routing, the per-expert input distribution, the placement-aware
 * send layout, the expert FFN per routed input, the weighted return, and their gradients.
 * It exists so that the GPU library can be checked element by element.  It shares no code,
 * header, table or helper with the GPU library; only tests, the smoke check and the
 * benchmark's CPU-baseline leg may call it.
 *
 * Paper passages followed (arXiv 2411.10003):
 *   Section 2.1 (MoE layer: the gate relates every input to all experts and routes it to the
 *     top-k; EP workflow of Fig. 2: gate -> all-to-all -> expert computation -> all-to-all back)
 *   Section 3 / Fig. 4 (input distribution = number of inputs per expert)
 *   Section 4.1 (lightweight expert placement: a device that holds an expert's parameters
 *     computes its local inputs for that expert itself, the others go to the owner)
 *   Section 4.2, Eq. 2-3 (forward and backward expert computation over the inputs a device hosts)
 * The paper prints no formula for the gate, the activation or the buffer layout; the readings
 * used here (linear gate with bias and softmax, ties to the lowest index, exact-erf GELU or
 * SwiGLU without biases, stable token-major order, slots ordered by (destination, expert))
 * are listed in the repository's design notes.
 *
 * All floating inputs are fp32 arrays (for the bf16 workloads their values are already
 * bf16-representable).  Everything except the gate logits is evaluated in double.  The gate
 * logits are fp32 in one fixed summation order, because they decide integer results.
 *
 * Parity pins (tests/test_oracle_*.py): every function below is pinned by closed forms,
 * brute force, library routines or finite differences; none is "parity unpinned".
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#define ORC_ACT_GELU 0
#define ORC_ACT_SWIGLU 1

/* ---------------------------------------------------------------------------------------
 * Gate logits (Section 2.1: "computes the relationship between that input and all the
 * experts"), read as logit[t,e] = b[e] + sum_c X[t,c] * Wg[c,e] in fp32 with this order:
 * two partial sums; the columns are taken in blocks of 32, block B (columns 32B .. 32B+31)
 * belongs to partial B mod 2; inside a block the columns are visited as c = 32B + 8q + j with
 * j = 0..7 in the outer and q = 0..3 in the inner loop, each step one fused multiply-add
 * onto the partial; logit = (s0 + s1) + b[e].  Denormals are kept.
 */
void orc_gate_logits(const float* X, const float* Wg, const float* bg, int T, int d, int E, float* logits)
{
#pragma omp parallel for schedule(static)
    for (int t = 0; t < T; ++t) {
        for (int e = 0; e < E; ++e) {
            float s[2] = {0.0f, 0.0f};
            for (int B = 0; 32 * B < d; ++B)
                for (int j = 0; j < 8; ++j)
                    for (int q = 0; q < 4; ++q) {
                        const int c = 32 * B + 8 * q + j;
                        if (c < d) s[B & 1] = fmaf(X[(size_t)t * d + c], Wg[(size_t)c * E + e], s[B & 1]);
                    }
            logits[(size_t)t * E + e] = (s[0] + s[1]) + bg[e];
        }
    }
}

/* ---------------------------------------------------------------------------------------
 * Routing (Section 2.1: "routes the input to top-k expert(s)").  Selection: k passes, each
 * taking the largest remaining logit, a later index winning only when strictly greater, so
 * ties go to the lowest index; NaN counts as -inf.  p = softmax over all E logits.
 * Gate weights: renorm = 0: w_j = p[idx_j];  renorm = 1: w_j = p[idx_j] / sum_i p[idx_i].
 * probs may be NULL.
 */
void orc_topk(const float* logits, int T, int E, int k, int renorm, int32_t* idx, double* w, double* probs)
{
#pragma omp parallel for schedule(static)
    for (int t = 0; t < T; ++t) {
        double* v = (double*)malloc(sizeof(double) * (size_t)E);
        double* p = (double*)malloc(sizeof(double) * (size_t)E);
        char* taken = (char*)calloc((size_t)E, 1);
        for (int e = 0; e < E; ++e) {
            float x = logits[(size_t)t * E + e];
            v[e] = isnan(x) ? -INFINITY : (double)x;
        }
        for (int j = 0; j < k; ++j) {
            int best = -1;
            for (int e = 0; e < E; ++e) {
                if (taken[e]) continue;
                if (best < 0 || v[e] > v[best]) best = e;
            }
            taken[best] = 1;
            idx[(size_t)t * k + j] = best;
        }
        double m = -INFINITY;
        for (int e = 0; e < E; ++e) if (v[e] > m) m = v[e];
        double sum = 0.0;
        for (int e = 0; e < E; ++e) { p[e] = exp(v[e] - m); sum += p[e]; }
        for (int e = 0; e < E; ++e) p[e] /= sum;
        double sel = 0.0;
        for (int j = 0; j < k; ++j) sel += p[idx[(size_t)t * k + j]];
        for (int j = 0; j < k; ++j) {
            double pj = p[idx[(size_t)t * k + j]];
            w[(size_t)t * k + j] = renorm ? pj / sel : pj;
        }
        if (probs) for (int e = 0; e < E; ++e) probs[(size_t)t * E + e] = p[e];
        free(v); free(p); free(taken);
    }
}

/* Input distribution (Section 3): counts[e] = number of routed inputs (assignments) of expert e. */
void orc_counts(const int32_t* idx, int A, int E, int32_t* counts)
{
    for (int e = 0; e < E; ++e) counts[e] = 0;
    for (int a = 0; a < A; ++a) counts[idx[a]] += 1;
}

/* ---------------------------------------------------------------------------------------
 * Send layout for a placement (Section 4.1).  expert_dest[e] in [0,P) is the destination that
 * computes this device's inputs of expert e.  Slots are the experts ordered by
 * (expert_dest[e], e); a slot's rows are contiguous; a destination's slots are contiguous.
 * Outputs: slot_of_expert[E], slot_offsets[E+1] (first row of each slot, last = A),
 * dest_offsets[P+1] (first row of each destination), dest_slots[P+1] (first slot of each).
 * Returns 0, or -1 if a destination is out of range.
 */
int orc_layout(const int32_t* counts, const int32_t* expert_dest, int E, int P,
               int32_t* slot_of_expert, int32_t* slot_offsets, int32_t* dest_offsets, int32_t* dest_slots)
{
    for (int e = 0; e < E; ++e) if (expert_dest[e] < 0 || expert_dest[e] >= P) return -1;
    int slot = 0, row = 0;
    for (int p = 0; p < P; ++p) {
        dest_slots[p] = slot;
        dest_offsets[p] = row;
        for (int e = 0; e < E; ++e) {
            if (expert_dest[e] != p) continue;
            slot_of_expert[e] = slot;
            slot_offsets[slot] = row;
            row += counts[e];
            slot += 1;
        }
    }
    dest_slots[P] = slot;
    dest_offsets[P] = row;
    slot_offsets[E] = row;
    return 0;
}

/* Stable placement of assignments a = t*k + j (ascending) inside their slot:
 * pos[a] = row of assignment a, perm[row] = assignment. */
void orc_positions(const int32_t* idx, int A, int E, const int32_t* slot_of_expert, const int32_t* slot_offsets,
                   int32_t* pos, int32_t* perm)
{
    int32_t* next = (int32_t*)malloc(sizeof(int32_t) * (size_t)E);
    for (int s = 0; s < E; ++s) next[s] = slot_offsets[s];
    for (int a = 0; a < A; ++a) {
        int s = slot_of_expert[idx[a]];
        pos[a] = next[s];
        perm[next[s]] = a;
        next[s] += 1;
    }
    free(next);
}

/* Send buffer of the first all-to-all (Fig. 2): Xp[r,:] = X[perm[r] / k, :]. */
void orc_dispatch(const float* X, const int32_t* perm, int A, int d, int k, float* Xp)
{
    for (int r = 0; r < A; ++r)
        memcpy(Xp + (size_t)r * d, X + (size_t)(perm[r] / k) * d, sizeof(float) * (size_t)d);
}

/* --------------------------------------------------------------------------------------- */
static double gelu(double z) { return 0.5 * z * (1.0 + erf(z / sqrt(2.0))); }
static double gelu_grad(double z)
{
    const double inv_sqrt_2pi = 0.39894228040143267794;
    return 0.5 * (1.0 + erf(z / sqrt(2.0))) + z * inv_sqrt_2pi * exp(-0.5 * z * z);
}
static double sigmoid(double z) { return 1.0 / (1.0 + exp(-z)); }
static double silu(double z) { return z * sigmoid(z); }
static double silu_grad(double z) { double s = sigmoid(z); return s * (1.0 + z * (1.0 - s)); }

/* Hidden pre-activations of one input x with the weights of group g: z = x W1[g], u = x W3[g]. */
static void hidden_pre(const float* x, const float* W1g, const float* W3g, int d, int h, double* z, double* u)
{
    for (int j = 0; j < h; ++j) z[j] = 0.0;
    for (int c = 0; c < d; ++c) {
        double xc = (double)x[c];
        const float* row = W1g + (size_t)c * h;
        for (int j = 0; j < h; ++j) z[j] += xc * (double)row[j];
    }
    if (W3g) {
        for (int j = 0; j < h; ++j) u[j] = 0.0;
        for (int c = 0; c < d; ++c) {
            double xc = (double)x[c];
            const float* row = W3g + (size_t)c * h;
            for (int j = 0; j < h; ++j) u[j] += xc * (double)row[j];
        }
    }
}

/* ---------------------------------------------------------------------------------------
 * Forward expert computation (Section 4.2, FEC) for the listed assignments, each evaluated
 * with the weights of its own expert and without looking at the send layout.
 *   GELU  : y = gelu(x W1) W2               SwiGLU: y = (silu(x W1) * (x W3)) W2
 * X[T,d]; idx[A]; group_of_expert[E] (weight group of a hosted expert, -1 otherwise);
 * W1[G,d,h], W3[G,d,h], W2[G,h,d]; a_list[n] assignment ids.
 * Outputs (row i belongs to a_list[i]): Y[n,d]; Z[n,h], U[n,h], Act[n,h] may be NULL.
 * Returns 0, or -1 if a listed assignment's expert is not hosted.
 */
int orc_ffn_fwd(const float* X, const int32_t* idx, const int32_t* group_of_expert,
                const float* W1, const float* W2, const float* W3, int d, int h, int k, int act,
                const int32_t* a_list, int n, double* Y, double* Z, double* U, double* Act)
{
    for (int i = 0; i < n; ++i) if (group_of_expert[idx[a_list[i]]] < 0) return -1;
#pragma omp parallel for schedule(dynamic, 1)
    for (int i = 0; i < n; ++i) {
        int a = a_list[i];
        int g = group_of_expert[idx[a]];
        const float* x = X + (size_t)(a / k) * d;
        const float* W1g = W1 + (size_t)g * d * h;
        const float* W2g = W2 + (size_t)g * h * d;
        const float* W3g = (act == ORC_ACT_SWIGLU) ? W3 + (size_t)g * d * h : NULL;
        double* z = (double*)malloc(sizeof(double) * (size_t)h * 3);
        double* u = z + h;
        double* av = z + 2 * (size_t)h;
        hidden_pre(x, W1g, W3g, d, h, z, u);
        for (int j = 0; j < h; ++j) av[j] = (act == ORC_ACT_SWIGLU) ? silu(z[j]) * u[j] : gelu(z[j]);
        double* y = Y + (size_t)i * d;
        for (int c = 0; c < d; ++c) y[c] = 0.0;
        for (int j = 0; j < h; ++j) {
            const float* row = W2g + (size_t)j * d;
            double aj = av[j];
            for (int c = 0; c < d; ++c) y[c] += aj * (double)row[c];
        }
        if (Z) memcpy(Z + (size_t)i * h, z, sizeof(double) * (size_t)h);
        if (U && W3g) memcpy(U + (size_t)i * h, u, sizeof(double) * (size_t)h);
        if (Act) memcpy(Act + (size_t)i * h, av, sizeof(double) * (size_t)h);
        free(z);
    }
    return 0;
}

/* Weighted return (second all-to-all of Fig. 2 plus the sum at the source):
 * out[t,:] = sum_j w[t,j] * Yp[pos[t*k+j],:], j ascending.  t_list[n] lists the tokens. */
void orc_combine(const double* Yp, const int32_t* pos, const double* w, int d, int k,
                 const int32_t* t_list, int n, double* out)
{
#pragma omp parallel for schedule(static)
    for (int i = 0; i < n; ++i) {
        int t = t_list[i];
        double* o = out + (size_t)i * d;
        for (int c = 0; c < d; ++c) o[c] = 0.0;
        for (int j = 0; j < k; ++j) {
            const double* y = Yp + (size_t)pos[(size_t)t * k + j] * d;
            double wj = w[(size_t)t * k + j];
            for (int c = 0; c < d; ++c) o[c] += wj * y[c];
        }
    }
}

/* Gradient of the weighted return: dYp[pos[a],:] = w[a] * dOut[t,:] and
 * dw[t,j] = <dOut[t,:], Yp[pos[a],:]> with a = t*k + j, for all T tokens. */
void orc_combine_bwd(const float* dOut, const double* Yp, const int32_t* pos, const double* w,
                     int T, int d, int k, double* dYp, double* dw)
{
#pragma omp parallel for schedule(static)
    for (int t = 0; t < T; ++t) {
        const float* g = dOut + (size_t)t * d;
        for (int j = 0; j < k; ++j) {
            size_t a = (size_t)t * k + j;
            size_t r = (size_t)pos[a];
            double acc = 0.0;
            for (int c = 0; c < d; ++c) {
                dYp[r * d + c] = w[a] * (double)g[c];
                acc += (double)g[c] * Yp[r * d + c];
            }
            dw[a] = acc;
        }
    }
}

/* ---------------------------------------------------------------------------------------
 * Backward expert computation (Section 4.2, BEC), input gradient of the listed assignments.
 * dY[n,d] is aligned with a_list.  With z, u, A as in the forward pass and dA = dy W2^T:
 *   GELU  : dz = dA * gelu'(z);                       dx = dz W1^T
 *   SwiGLU: du = dA * silu(z); dz = dA * u * silu'(z); dx = dz W1^T + du W3^T
 */
int orc_ffn_bwd_rows(const float* X, const int32_t* idx, const int32_t* group_of_expert,
                     const float* W1, const float* W2, const float* W3, int d, int h, int k, int act,
                     const int32_t* a_list, int n, const double* dY, double* dX)
{
    for (int i = 0; i < n; ++i) if (group_of_expert[idx[a_list[i]]] < 0) return -1;
#pragma omp parallel for schedule(dynamic, 1)
    for (int i = 0; i < n; ++i) {
        int a = a_list[i];
        int g = group_of_expert[idx[a]];
        const float* x = X + (size_t)(a / k) * d;
        const float* W1g = W1 + (size_t)g * d * h;
        const float* W2g = W2 + (size_t)g * h * d;
        const float* W3g = (act == ORC_ACT_SWIGLU) ? W3 + (size_t)g * d * h : NULL;
        double* z = (double*)malloc(sizeof(double) * (size_t)h * 4);
        double* u = z + h;
        double* dz = z + 2 * (size_t)h;
        double* du = z + 3 * (size_t)h;
        hidden_pre(x, W1g, W3g, d, h, z, u);
        const double* dy = dY + (size_t)i * d;
        for (int j = 0; j < h; ++j) {
            const float* row = W2g + (size_t)j * d;
            double dA = 0.0;
            for (int c = 0; c < d; ++c) dA += dy[c] * (double)row[c];
            if (act == ORC_ACT_SWIGLU) {
                du[j] = dA * silu(z[j]);
                dz[j] = dA * u[j] * silu_grad(z[j]);
            } else {
                dz[j] = dA * gelu_grad(z[j]);
            }
        }
        double* dx = dX + (size_t)i * d;
        for (int c = 0; c < d; ++c) {
            const float* r1 = W1g + (size_t)c * h;
            double s = 0.0;
            for (int j = 0; j < h; ++j) s += dz[j] * (double)r1[j];
            if (W3g) {
                const float* r3 = W3g + (size_t)c * h;
                for (int j = 0; j < h; ++j) s += du[j] * (double)r3[j];
            }
            dx[c] = s;
        }
        free(z);
    }
    return 0;
}

/* ---------------------------------------------------------------------------------------
 * Weight gradients of group g restricted to hidden unit j, summed over every assignment
 * routed to that group (the FFN is a sum over hidden units, so the full gradient is this
 * for j = 0..h-1):
 *   dW2[g][j,:] = sum_a A_a[j] * dy_a        (row j of dW2[g],    length d)
 *   dW1[g][:,j] = sum_a x_a   * dz_a[j]      (column j of dW1[g], length d)
 *   dW3[g][:,j] = sum_a x_a   * du_a[j]      (SwiGLU only)
 * dYa[A,d] holds dy by assignment id (rows of other groups are not read).
 */
void orc_ffn_bwd_hidden(const float* X, const int32_t* idx, const int32_t* group_of_expert,
                        const float* W1, const float* W2, const float* W3, int d, int h, int k, int A, int act,
                        const float* dYa, int g, int j, double* dW2row, double* dW1col, double* dW3col)
{
    const float* W1g = W1 + (size_t)g * d * h;
    const float* W2g = W2 + (size_t)g * h * d;
    const float* W3g = (act == ORC_ACT_SWIGLU) ? W3 + (size_t)g * d * h : NULL;
    for (int c = 0; c < d; ++c) { dW2row[c] = 0.0; dW1col[c] = 0.0; if (W3g) dW3col[c] = 0.0; }
    for (int a = 0; a < A; ++a) {
        if (group_of_expert[idx[a]] != g) continue;
        const float* x = X + (size_t)(a / k) * d;
        const float* dy = dYa + (size_t)a * d;
        double z = 0.0, u = 0.0, dA = 0.0;
        for (int c = 0; c < d; ++c) z += (double)x[c] * (double)W1g[(size_t)c * h + j];
        if (W3g) for (int c = 0; c < d; ++c) u += (double)x[c] * (double)W3g[(size_t)c * h + j];
        for (int c = 0; c < d; ++c) dA += (double)dy[c] * (double)W2g[(size_t)j * d + c];
        double av, dz, du = 0.0;
        if (W3g) { av = silu(z) * u; du = dA * silu(z); dz = dA * u * silu_grad(z); }
        else { av = gelu(z); dz = dA * gelu_grad(z); }
        for (int c = 0; c < d; ++c) {
            dW2row[c] += av * (double)dy[c];
            dW1col[c] += (double)x[c] * dz;
            if (W3g) dW3col[c] += (double)x[c] * du;
        }
    }
}

/* The same for a list of hidden units of one group, one unit per thread: every unit is the call above,
 * unchanged (outer loop only).  Row i of each output belongs to hidden unit js[i]. */
void orc_ffn_bwd_hidden_many(const float* X, const int32_t* idx, const int32_t* group_of_expert,
                             const float* W1, const float* W2, const float* W3, int d, int h, int k, int A, int act,
                             const float* dYa, int g, const int32_t* js, int n_js,
                             double* dW2rows, double* dW1cols, double* dW3cols)
{
#pragma omp parallel for schedule(dynamic, 1)
    for (int i = 0; i < n_js; ++i)
        orc_ffn_bwd_hidden(X, idx, group_of_expert, W1, W2, W3, d, h, k, A, act, dYa, g, js[i],
                           dW2rows + (size_t)i * d, dW1cols + (size_t)i * d, dW3cols ? dW3cols + (size_t)i * d : NULL);
}

/* Gradient of the send (fourth all-to-all): dX[t,:] = sum_j dXp[pos[t*k+j],:]. */
void orc_dispatch_bwd(const double* dXp, const int32_t* pos, int T, int d, int k, double* dX)
{
#pragma omp parallel for schedule(static)
    for (int t = 0; t < T; ++t)
        for (int c = 0; c < d; ++c) {
            double s = 0.0;
            for (int j = 0; j < k; ++j) s += dXp[(size_t)pos[(size_t)t * k + j] * d + c];
            dX[(size_t)t * d + c] = s;
        }
}

/* ---------------------------------------------------------------------------------------
 * Gradient of the gate weights with respect to the logits, selection held fixed.
 *   renorm = 0 (w_j = p[s_j]):         dl[e]   = sum_j dw_j * p[s_j] * ((e == s_j) - p[e])
 *   renorm = 1 (w = softmax over the selected logits):
 *                                      dl[s_j] = w_j * (dw_j - sum_i w_i dw_i), 0 elsewhere
 */
void orc_gate_bwd(const double* dw, const float* logits, const int32_t* idx, int T, int E, int k, int renorm,
                  double* dlogits)
{
#pragma omp parallel for schedule(static)
    for (int t = 0; t < T; ++t) {
        double* p = (double*)malloc(sizeof(double) * (size_t)E);
        double m = -INFINITY, sum = 0.0;
        for (int e = 0; e < E; ++e) { double v = (double)logits[(size_t)t * E + e]; if (v > m) m = v; }
        for (int e = 0; e < E; ++e) { p[e] = exp((double)logits[(size_t)t * E + e] - m); sum += p[e]; }
        for (int e = 0; e < E; ++e) p[e] /= sum;
        double* dl = dlogits + (size_t)t * E;
        for (int e = 0; e < E; ++e) dl[e] = 0.0;
        const int32_t* s = idx + (size_t)t * k;
        const double* g = dw + (size_t)t * k;
        if (renorm) {
            double sel = 0.0, dot = 0.0;
            for (int j = 0; j < k; ++j) sel += p[s[j]];
            for (int j = 0; j < k; ++j) dot += (p[s[j]] / sel) * g[j];
            for (int j = 0; j < k; ++j) dl[s[j]] = (p[s[j]] / sel) * (g[j] - dot);
        } else {
            for (int j = 0; j < k; ++j)
                for (int e = 0; e < E; ++e)
                    dl[e] += g[j] * p[s[j]] * ((e == s[j] ? 1.0 : 0.0) - p[e]);
        }
        free(p);
    }
}

/* ---------------------------------------------------------------------------------------
 * Backward of the gate's linear map logit[t,e] = b[e] + sum_c X[t,c] Wg[c,e] (the gate network of
 * Section 2.1), given dlogits:
 *   dWg[c,e] = sum_t X[t,c] dlogits[t,e],   dbg[e] = sum_t dlogits[t,e]
 */
void orc_gate_bwd_params(const float* X, const double* dlogits, int T, int d, int E, double* dWg, double* dbg)
{
#pragma omp parallel for schedule(static)
    for (int c = 0; c < d; ++c)
        for (int e = 0; e < E; ++e) {
            double s = 0.0;
            for (int t = 0; t < T; ++t) s += (double)X[(size_t)t * d + c] * dlogits[(size_t)t * E + e];
            dWg[(size_t)c * E + e] = s;
        }
    for (int e = 0; e < E; ++e) {
        double s = 0.0;
        for (int t = 0; t < T; ++t) s += dlogits[(size_t)t * E + e];
        dbg[e] = s;
    }
}

/* Gradient of the layer input: the expert path (the backward of the send, see orc_dispatch_bwd) plus
 * the gate path dlogits Wg^T:  dX[t,c] = sum_j dXp[pos[t*k+j],c] + sum_e dlogits[t,e] Wg[c,e]. */
void orc_input_grad(const double* dXp, const int32_t* pos, const double* dlogits, const float* Wg,
                    int T, int d, int E, int k, double* dX)
{
#pragma omp parallel for schedule(static)
    for (int t = 0; t < T; ++t)
        for (int c = 0; c < d; ++c) {
            double s = 0.0;
            for (int j = 0; j < k; ++j) s += dXp[(size_t)pos[(size_t)t * k + j] * d + c];
            double g = 0.0;
            for (int e = 0; e < E; ++e) g += dlogits[(size_t)t * E + e] * (double)Wg[(size_t)c * E + e];
            dX[(size_t)t * d + c] = s + g;
        }
}


/*
 * CPU oracle for the binary-masked MoE layer forward (BEAM, Sec. 3.1-3.2).
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, plain definition that the
 * GPU library is checked against.  Only the test-suite, the smoke check and
 * the benchmark's cpu_baseline leg may call it; the product never does.  It
 * shares no code, header, table or helper with the HIP path.
 *
 * Everything is evaluated per token, straight from the equations, with every
 * floating-point sum carried in fp64.  Inputs are fp32 arrays (for bf16
 * workloads: the bf16 values, upcast exactly).  There is no blocking, fusion
 * or reordering: one dot product at a time.
 *
 * Layouts (row-major, last index contiguous), paper notation x W with W stored
 * transposed:
 *   x [T,H]; w_router, w_mask [N,H]; w_gate_up [N,2I,H] (rows 0..I-1 gate,
 *   rows I..2I-1 up); w_down [N,H,I].
 *
 * Readings of the paper taken here:
 *   - Top-K order: logit descending, equal logits -> lower expert index first;
 *     slot k holds the (k+1)-th ranked expert (Sec. 3.2 Step 1 leaves it open).
 *   - Routing weights: softmax over the K surviving logits (Eq. 4: softmax of
 *     the vector whose other entries are -inf).
 *   - Mask: m = 1 iff sigma(a) >= 0.5 iff a >= 0 (Eq. 6); the comparison is
 *     taken on the pre-activation a, never on sigma(a).  a == 0 keeps, which is
 *     what makes a zero-initialised mask router reproduce Top-K (Sec. 3.3.1).
 *   - The decision values r and a are rounded to fp32 before comparing: that
 *     is the precision the GPU kernels decide in.
 *   - No renormalisation after masking (Eq. 7 is a bare product); a token with
 *     no kept expert yields an exactly zero row (Sec. 3.2 Step 3, App. A.3).
 *   - delta in the GLU expert (Eq. 3) is SiLU.
 *   - Pairs are grouped by expert with a stable order (ascending flat pair
 *     index t*K+k inside an expert); dropped pairs carry id -1 (App. A.4).
 *   - Other activation rules on the same Top-K slots (Sec. 4.1 baselines, Sec. 4.4
 *     ablation), each yielding masked ids; the routing weights stay those of
 *     Eq. 4 and are never renormalised:
 *       threshold tau: keep iff sigma(a) >= tau iff a >= theta = ln(tau/(1-tau));
 *         the caller passes theta as an fp32 number and the comparison is a >= theta;
 *       cumulative probability phi: with p = softmax of r over ALL N experts,
 *         experts are activated in rank order until their cumulative p exceeds
 *         phi, i.e. slot k is kept iff sum_{j<k} p_ids[j] <= phi (the first slot
 *         always is); at most the K slots exist.  The paper names the rule and
 *         its threshold only; this is the reading taken.
 *   - Training (Sec. 3.3): every Top-K expert is evaluated whatever the mask says
 *     and the output uses the binary mask; the mask router's gradient is Eq. 12
 *     with dL_lm/dg^_i = <dL/dy, E_i(x)> (y is linear in g^); L_reg is returned
 *     per token, and the coefficient c that multiplies 1/K in Eq. 12 is an
 *     input (beta, or beta/T for a batch mean: the paper fixes no reduction).
 *   - Whole block (App. A.3): the layer input x is the already normalised
 *     hidden state, the residual h is a separate input; the shared expert is
 *     one GLU expert of its own width; its weight g_sh, for which the paper
 *     gives no formula, is 1, or sigma(x . w) when a gate vector w is given.
 *
 * Parity pins: every function here is pinned by the CPU tests (closed-form
 * micro case, all-ones / all-zero mask, dense library evaluation, brute force
 * over mask patterns, special cases K=1 / K=N / N=K=1, permutation invariants;
 * for the whole block: the zero-activation forms of App. A.3, a dense library
 * evaluation and the micro case extended by a shared expert and a residual;
 * for the mask-router gradient: central differences of the soft surrogate
 * under a linear loss, the zero rows of Theorem 1, and a closed form).
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

int beam_oracle_max_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/* Pre-activations of a linear head: out[t,e] = x[t,:] . w[e,:] (+ bias[e]).
 * Used for the router logits r (Sec. 3.2 Step 1) and the mask-router
 * pre-activation a = x W_m (Eq. 5, Sec. 3.4).  fp64 sum, one rounding to fp32. */
void beam_oracle_logits(int T, int H, int N, const float *x, const float *w,
                        const float *bias, float *out)
{
#ifdef _OPENMP
#pragma omp parallel for schedule(static) if (T >= 64)
#endif
    for (int t = 0; t < T; ++t) {
        for (int e = 0; e < N; ++e) {
            double acc = 0.0;
            for (int h = 0; h < H; ++h)
                acc += (double)x[(size_t)t * H + h] * (double)w[(size_t)e * H + h];
            if (bias)
                acc += (double)bias[e];
            out[(size_t)t * N + e] = (float)acc;
        }
    }
}

/* Steps 1, 3 and 4 of Sec. 3.2 for one token, from its N router logits r and N
 * mask pre-activations a:
 *   ids[k]     = expert with the (k+1)-th largest r           (Top-K, Step 1)
 *   g[k]       = exp(r_ids[k]) / sum_j exp(r_ids[j])          (Eq. 4)
 *   masked[k]  = a[ids[k]] >= 0 ? ids[k] : -1                 (Eq. 6, App. A.4)
 * g is NOT changed by the mask (Eq. 7 multiplies by m later).           */
static void route_mask_token(int N, int K, const float *r, const float *a,
                             int32_t *ids, double *g, int32_t *masked)
{
    char *taken = (char *)calloc((size_t)N, 1);
    for (int k = 0; k < K; ++k) {
        int best = -1;
        for (int e = 0; e < N; ++e) {
            if (taken[e])
                continue;
            if (best < 0 || r[e] > r[best])   /* strict >: lower index wins ties */
                best = e;
        }
        taken[best] = 1;
        ids[k] = best;
    }
    free(taken);
    double top = (double)r[ids[0]];
    double denom = 0.0;
    for (int k = 0; k < K; ++k) {
        g[k] = exp((double)r[ids[k]] - top);
        denom += g[k];
    }
    for (int k = 0; k < K; ++k)
        g[k] /= denom;
    for (int k = 0; k < K; ++k)
        masked[k] = (a[ids[k]] >= 0.0f) ? ids[k] : -1;
}

void beam_oracle_route_mask(int T, int N, int K, const float *router_logits,
                            const float *mask_logits, int32_t *topk_ids,
                            double *topk_weights, int32_t *masked_ids)
{
    for (int t = 0; t < T; ++t)
        route_mask_token(N, K, router_logits + (size_t)t * N, mask_logits + (size_t)t * N,
                         topk_ids + (size_t)t * K, topk_weights + (size_t)t * K,
                         masked_ids + (size_t)t * K);
}

/* Expert-wise grouping of the kept pairs (App. A.4: entries equal to -1 are
 * ignored).  Any id outside [0,N) counts as dropped.
 *   counts[e]      number of kept pairs of expert e
 *   offsets[0..N]  exclusive prefix sums, offsets[N] = P
 *   perm[i]        flat pair index f = t*K+k sitting at grouped row i (i < P),
 *                  -1 for i >= P; inside an expert f ascends (stable)
 *   inv_perm[f]    grouped row of pair f, or -1 if dropped                 */
void beam_oracle_permute(int TK, int N, const int32_t *masked_ids, int32_t *counts,
                         int32_t *offsets, int32_t *perm, int32_t *inv_perm,
                         int32_t *num_pairs)
{
    for (int e = 0; e < N; ++e)
        counts[e] = 0;
    for (int f = 0; f < TK; ++f) {
        int32_t e = masked_ids[f];
        if (e >= 0 && e < N)
            counts[e] += 1;
    }
    offsets[0] = 0;
    for (int e = 0; e < N; ++e)
        offsets[e + 1] = offsets[e] + counts[e];
    *num_pairs = offsets[N];
    for (int i = 0; i < TK; ++i)
        perm[i] = -1;
    for (int f = 0; f < TK; ++f)
        inv_perm[f] = -1;
    /* one expert at a time, pairs in ascending f: stable by construction */
    int32_t row = 0;
    for (int e = 0; e < N; ++e) {
        for (int f = 0; f < TK; ++f) {
            if (masked_ids[f] == e) {
                perm[row] = f;
                inv_perm[f] = row;
                ++row;
            }
        }
    }
}

/* One GLU expert on one token (Eq. 3 with delta = SiLU):
 *   gate_j = x . W_gate[:,j],  up_j = x . W_up[:,j]
 *   hid_j  = gate_j / (1 + exp(-gate_j)) * up_j
 *   y_c    = sum_j hid_j * W_down[j,c]
 * w_gate_up points at this expert's [2I,H] block, w_down at its [H,I] block. */
void beam_oracle_expert_ffn(int H, int I, const float *x, const float *w_gate_up,
                            const float *w_down, double *y)
{
    double *hid = (double *)malloc(sizeof(double) * (size_t)I);
    for (int j = 0; j < I; ++j) {
        double gate = 0.0, up = 0.0;
        const float *wg = w_gate_up + (size_t)j * H;
        const float *wu = w_gate_up + (size_t)(I + j) * H;
        for (int h = 0; h < H; ++h) {
            gate += (double)x[h] * (double)wg[h];
            up += (double)x[h] * (double)wu[h];
        }
        hid[j] = gate / (1.0 + exp(-gate)) * up;
    }
    for (int c = 0; c < H; ++c) {
        double acc = 0.0;
        const float *wd = w_down + (size_t)c * I;
        for (int j = 0; j < I; ++j)
            acc += hid[j] * (double)wd[j];
        y[c] = acc;
    }
    free(hid);
}

/* E_e(x_t) for every kept slot: y_slots[f,:] = expert masked_ids[f] applied to
 * token f / K; rows of dropped slots are zero.  Returns the number of expert
 * evaluations performed (= kept pairs).                                     */
int64_t beam_oracle_pair_outputs(int T, int H, int N, int K, int I, const float *x,
                                 const float *w_gate_up, const float *w_down,
                                 const int32_t *masked_ids, double *y_slots, int nthreads)
{
    int64_t evals = 0;
    (void)nthreads;
#ifdef _OPENMP
    if (nthreads < 1)
        nthreads = omp_get_max_threads();
#pragma omp parallel for schedule(dynamic, 1) num_threads(nthreads) reduction(+ : evals)
#endif
    for (int f = 0; f < T * K; ++f) {
        int32_t e = masked_ids[f];
        double *y = y_slots + (size_t)f * H;
        if (e < 0 || e >= N) {
            for (int c = 0; c < H; ++c)
                y[c] = 0.0;
            continue;
        }
        beam_oracle_expert_ffn(H, I, x + (size_t)(f / K) * H,
                               w_gate_up + (size_t)e * 2 * I * H, w_down + (size_t)e * H * I, y);
        evals += 1;
    }
    return evals;
}

/* The whole layer (Eq. 4-8), one token at a time:
 *   r = x W_r (+b_r), a = x W_m (+b_m); Top-K, g, mask as above;
 *   out[t,:] = sum over kept slots k, in slot order, of g[k] * E_ids[k](x_t).
 * Optional outputs may be NULL.  Returns the number of expert evaluations,
 * which is the layer's FLOP count divided by 6*H*I (Sec. 4.3: compute scales
 * with the activated experts).                                              */
int64_t beam_oracle_moe_forward(int T, int H, int N, int K, int I, const float *x,
                                const float *w_router, const float *b_router,
                                const float *w_mask, const float *b_mask,
                                const float *w_gate_up, const float *w_down, double *out,
                                int32_t *topk_ids, double *topk_weights, int32_t *masked_ids,
                                int nthreads)
{
    int64_t evals = 0;
    (void)nthreads;
#ifdef _OPENMP
    if (nthreads < 1)
        nthreads = omp_get_max_threads();
#pragma omp parallel for schedule(dynamic, 1) num_threads(nthreads) reduction(+ : evals)
#endif
    for (int t = 0; t < T; ++t) {
        float *r = (float *)malloc(sizeof(float) * (size_t)N);
        float *a = (float *)malloc(sizeof(float) * (size_t)N);
        int32_t *ids = (int32_t *)malloc(sizeof(int32_t) * (size_t)K);
        int32_t *msk = (int32_t *)malloc(sizeof(int32_t) * (size_t)K);
        double *g = (double *)malloc(sizeof(double) * (size_t)K);
        double *y = (double *)malloc(sizeof(double) * (size_t)H);
        const float *xt = x + (size_t)t * H;

        beam_oracle_logits(1, H, N, xt, w_router, b_router, r);
        beam_oracle_logits(1, H, N, xt, w_mask, b_mask, a);
        route_mask_token(N, K, r, a, ids, g, msk);

        double *o = out + (size_t)t * H;
        for (int c = 0; c < H; ++c)
            o[c] = 0.0;
        for (int k = 0; k < K; ++k) {
            if (msk[k] < 0)
                continue;
            int e = msk[k];
            beam_oracle_expert_ffn(H, I, xt, w_gate_up + (size_t)e * 2 * I * H,
                                   w_down + (size_t)e * H * I, y);
            for (int c = 0; c < H; ++c)
                o[c] += g[k] * y[c];
            evals += 1;
        }
        for (int k = 0; k < K; ++k) {
            if (topk_ids)
                topk_ids[(size_t)t * K + k] = ids[k];
            if (topk_weights)
                topk_weights[(size_t)t * K + k] = g[k];
            if (masked_ids)
                masked_ids[(size_t)t * K + k] = msk[k];
        }
        free(r); free(a); free(ids); free(msk); free(g); free(y);
    }
    return evals;
}

/* Activation rules other than the default mask (see the header): kind 0 =
 * threshold on the mask pre-activation, param = theta; kind 1 = cumulative
 * routing probability, param = phi.  Same outputs as beam_oracle_route_mask;
 * kind 0 with theta = 0 is that function.                                   */
static void route_rule_token(int N, int K, const float *r, const float *a, int kind,
                             float param, int32_t *ids, double *g, int32_t *masked)
{
    route_mask_token(N, K, r, a, ids, g, masked);   /* Top-K order and Eq. 4 weights */
    if (kind == 0) {
        for (int k = 0; k < K; ++k)
            masked[k] = (a[ids[k]] >= param) ? ids[k] : -1;
    } else {
        double top = (double)r[ids[0]];
        double z = 0.0;
        for (int e = 0; e < N; ++e)
            z += exp((double)r[e] - top);
        double cum = 0.0;                            /* probability of the ranks before k */
        for (int k = 0; k < K; ++k) {
            masked[k] = (cum <= (double)param) ? ids[k] : -1;
            cum += exp((double)r[ids[k]] - top) / z;
        }
    }
}

void beam_oracle_route_rule(int T, int N, int K, const float *router_logits,
                            const float *mask_logits, int kind, float param,
                            int32_t *topk_ids, double *topk_weights, int32_t *masked_ids)
{
    for (int t = 0; t < T; ++t)
        route_rule_token(N, K, router_logits + (size_t)t * N, mask_logits + (size_t)t * N, kind,
                         param, topk_ids + (size_t)t * K, topk_weights + (size_t)t * K,
                         masked_ids + (size_t)t * K);
}

/* The layer of beam_oracle_moe_forward under one of those rules.            */
int64_t beam_oracle_moe_forward_rule(int T, int H, int N, int K, int I, const float *x,
                                     const float *w_router, const float *b_router,
                                     const float *w_mask, const float *b_mask,
                                     const float *w_gate_up, const float *w_down, int kind,
                                     float param, double *out, int32_t *topk_ids,
                                     double *topk_weights, int32_t *masked_ids, int nthreads)
{
    int64_t evals = 0;
    (void)nthreads;
#ifdef _OPENMP
    if (nthreads < 1)
        nthreads = omp_get_max_threads();
#pragma omp parallel for schedule(dynamic, 1) num_threads(nthreads) reduction(+ : evals)
#endif
    for (int t = 0; t < T; ++t) {
        float *r = (float *)malloc(sizeof(float) * (size_t)N);
        float *a = (float *)malloc(sizeof(float) * (size_t)N);
        int32_t *ids = (int32_t *)malloc(sizeof(int32_t) * (size_t)K);
        int32_t *msk = (int32_t *)malloc(sizeof(int32_t) * (size_t)K);
        double *g = (double *)malloc(sizeof(double) * (size_t)K);
        double *y = (double *)malloc(sizeof(double) * (size_t)H);
        const float *xt = x + (size_t)t * H;
        beam_oracle_logits(1, H, N, xt, w_router, b_router, r);
        beam_oracle_logits(1, H, N, xt, w_mask, b_mask, a);
        route_rule_token(N, K, r, a, kind, param, ids, g, msk);
        double *o = out + (size_t)t * H;
        for (int c = 0; c < H; ++c)
            o[c] = 0.0;
        for (int k = 0; k < K; ++k) {
            if (msk[k] < 0)
                continue;
            int e = msk[k];
            beam_oracle_expert_ffn(H, I, xt, w_gate_up + (size_t)e * 2 * I * H,
                                   w_down + (size_t)e * H * I, y);
            for (int c = 0; c < H; ++c)
                o[c] += g[k] * y[c];
            evals += 1;
        }
        for (int k = 0; k < K; ++k) {
            if (topk_ids)
                topk_ids[(size_t)t * K + k] = ids[k];
            if (topk_weights)
                topk_weights[(size_t)t * K + k] = g[k];
            if (masked_ids)
                masked_ids[(size_t)t * K + k] = msk[k];
        }
        free(r); free(a); free(ids); free(msk); free(g); free(y);
    }
    return evals;
}

/* The whole MoE block with residual and shared expert (App. A.3):
 *   out[t,:] = h[t,:] + sum over kept slots of g[k] * E_ids[k](x_t)
 *                     + g_sh[t] * E_sh(x_t)
 * x is the normalised hidden state N(h); h (residual) may be NULL (no residual
 * term).  The shared expert is a GLU expert of width I_sh with weights
 * w_sh_gate_up [2*I_sh,H] and w_sh_down [H,I_sh]; I_sh = 0 means delta_sh = 0.
 * g_sh[t] = 1 / (1 + exp(-(x_t . w_sh_gate))) if w_sh_gate is given, else 1.
 * With every routed expert masked the sum over slots is empty and the block
 * reduces to the second form in App. A.3.  Returns the number of routed expert
 * evaluations (the shared expert is not counted: it is never skipped).      */
int64_t beam_oracle_block_forward(int T, int H, int N, int K, int I, const float *x,
                                  const float *w_router, const float *b_router,
                                  const float *w_mask, const float *b_mask,
                                  const float *w_gate_up, const float *w_down, int I_sh,
                                  const float *w_sh_gate_up, const float *w_sh_down,
                                  const float *w_sh_gate, const float *residual, double *out,
                                  int32_t *topk_ids, double *topk_weights, int32_t *masked_ids,
                                  double *g_shared, int nthreads)
{
    int64_t evals = beam_oracle_moe_forward(T, H, N, K, I, x, w_router, b_router, w_mask, b_mask,
                                            w_gate_up, w_down, out, topk_ids, topk_weights,
                                            masked_ids, nthreads);
    (void)nthreads;
#ifdef _OPENMP
    if (nthreads < 1)
        nthreads = omp_get_max_threads();
#pragma omp parallel for schedule(dynamic, 1) num_threads(nthreads)
#endif
    for (int t = 0; t < T; ++t) {
        const float *xt = x + (size_t)t * H;
        double *o = out + (size_t)t * H;
        double gsh = 1.0;
        if (w_sh_gate) {
            double z = 0.0;
            for (int h = 0; h < H; ++h)
                z += (double)xt[h] * (double)w_sh_gate[h];
            gsh = 1.0 / (1.0 + exp(-z));
        }
        if (I_sh > 0) {
            double *y = (double *)malloc(sizeof(double) * (size_t)H);
            beam_oracle_expert_ffn(H, I_sh, xt, w_sh_gate_up, w_sh_down, y);
            for (int c = 0; c < H; ++c)
                o[c] += gsh * y[c];
            free(y);
        }
        if (residual)
            for (int c = 0; c < H; ++c)
                o[c] += (double)residual[(size_t)t * H + c];
        if (g_shared)
            g_shared[t] = gsh;
    }
    return evals;
}

/* Training mode (Sec. 3.3), one batch.
 * Forward: Top-K, g and the binary mask as in inference, but E_i(x_t) is
 * evaluated for EVERY Top-K slot (Sec. 3.3.1); out[t] = sum_k m_k g_k E_k(x_t).
 * Backward for the mask router under the straight-through estimator (Eq. 9):
 *   dL/dg^_k  = <grad_out[t,:], E_k(x_t)>                       (y = sum g^_k E_k)
 *   grad_a[t,k] = (dL/dg^_k * g_k + c / K) * sigma'(a_k)        (Eq. 12, i in T_K)
 *   grad_w_mask[e,:] = sum over (t,k) with ids[t,k] = e of grad_a[t,k] * x[t,:]
 *   loss_reg[t] = (1/K) * sum_k sigma(a_k)                      (Eq. 10)
 * with a_k the mask pre-activation of the slot's expert, sigma'(a) =
 * sigma(a)(1 - sigma(a)).  Experts outside the Top-K set of a token get no
 * gradient from it (Theorem 1).  Outputs: out [T,H], grad_a [T,K],
 * grad_w_mask [N,H], loss_reg [T], all fp64; topk_ids / masked_ids optional. */
void beam_oracle_train_step(int T, int H, int N, int K, int I, const float *x,
                            const float *w_router, const float *b_router, const float *w_mask,
                            const float *b_mask, const float *w_gate_up, const float *w_down,
                            const float *grad_out, double reg_coeff, double *out,
                            double *grad_a, double *grad_w_mask, double *loss_reg,
                            int32_t *topk_ids, int32_t *masked_ids)
{
    for (size_t i = 0; i < (size_t)N * H; ++i)
        grad_w_mask[i] = 0.0;
    float *r = (float *)malloc(sizeof(float) * (size_t)N);
    float *a = (float *)malloc(sizeof(float) * (size_t)N);
    int32_t *ids = (int32_t *)malloc(sizeof(int32_t) * (size_t)K);
    int32_t *msk = (int32_t *)malloc(sizeof(int32_t) * (size_t)K);
    double *g = (double *)malloc(sizeof(double) * (size_t)K);
    double *y = (double *)malloc(sizeof(double) * (size_t)H);
    for (int t = 0; t < T; ++t) {
        const float *xt = x + (size_t)t * H;
        const float *dy = grad_out + (size_t)t * H;
        beam_oracle_logits(1, H, N, xt, w_router, b_router, r);
        beam_oracle_logits(1, H, N, xt, w_mask, b_mask, a);
        route_mask_token(N, K, r, a, ids, g, msk);
        double *o = out + (size_t)t * H;
        for (int c = 0; c < H; ++c)
            o[c] = 0.0;
        double reg = 0.0;
        for (int k = 0; k < K; ++k) {
            int e = ids[k];
            beam_oracle_expert_ffn(H, I, xt, w_gate_up + (size_t)e * 2 * I * H,
                                   w_down + (size_t)e * H * I, y);
            if (msk[k] >= 0)
                for (int c = 0; c < H; ++c)
                    o[c] += g[k] * y[c];
            double dot = 0.0;
            for (int c = 0; c < H; ++c)
                dot += (double)dy[c] * y[c];
            double sig = 1.0 / (1.0 + exp(-(double)a[e]));
            double ga = (dot * g[k] + reg_coeff / (double)K) * sig * (1.0 - sig);
            grad_a[(size_t)t * K + k] = ga;
            reg += sig;
            for (int h = 0; h < H; ++h)
                grad_w_mask[(size_t)e * H + h] += ga * (double)xt[h];
            if (topk_ids)
                topk_ids[(size_t)t * K + k] = ids[k];
            if (masked_ids)
                masked_ids[(size_t)t * K + k] = msk[k];
        }
        loss_reg[t] = reg / (double)K;
    }
    free(r); free(a); free(ids); free(msk); free(g); free(y);
}

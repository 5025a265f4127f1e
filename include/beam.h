/*
 * beam.h -- C ABI of libbeam: the binary-masked Mixture-of-Experts layer
 * forward of BEAM (Binary Expert Activation Masking) as hand-written HIP
 * kernels for AMD MI355X (gfx950).
 *
 * The layer (paper Sec. 3.2, Steps 1-4, one token x in R^H at a time):
 *   r = x W_r                      router logits over N experts
 *   T_K = the K largest entries of r;  g = softmax over those K        (Eq. 4)
 *   a = x W_m ;  m_i = 1 iff sigma(a_i) >= 0.5  iff  a_i >= 0          (Eq. 5-6)
 *   g^ = g (.) m    -- not renormalised                                (Eq. 7)
 *   y = sum_i g^_i E_i(x),  E_i(x) = (SiLU(x W_gate) (.) (x W_up)) W_down
 *                                                                  (Eq. 3, 8)
 * A token may keep 0..K experts; with 0 its output row is exactly +0.
 * Dropped (token, expert) pairs are marked with expert id -1 and never reach
 * the expert GEMMs (paper App. A.4).
 *
 * Conventions for every entry point
 *   - All pointers except the beam_shape are DEVICE pointers (HBM) unless
 *     stated otherwise.  The caller owns every buffer, including the
 *     workspace; the library never allocates, frees, copies to the host or
 *     synchronises.  Work is enqueued on `hip_stream` (a hipStream_t passed
 *     as void*; NULL = the default stream) and the call returns at once.
 *   - Row-major, last index contiguous.  Weights are "output-feature major,
 *     reduction dimension contiguous": the paper's x W with W stored
 *     transposed.
 *       x          [T, H]       dtype
 *       w_router   [N, H]       dtype      W_r^T
 *       w_mask     [N, H]       dtype      W_m^T
 *       w_gate_up  [N, 2I, H]   dtype      rows 0..I-1 = W_gate^T, I..2I-1 = W_up^T
 *       w_down     [N, H, I]    dtype      W_down^T
 *       out        [T, H]       dtype
 *     dtype is BEAM_F32 (4-byte IEEE) or BEAM_BF16 (2-byte bfloat16).  Logits,
 *     routing weights and y_pairs are always fp32; indices are int32.
 *   - Biases are optional fp32 [N] vectors added to the logits (NULL = none,
 *     which is the paper's parametrisation).  They exist so synthetic
 *     workloads can set a keep rate and an expert-popularity skew.
 *   - Inputs must be finite.  Top-K order is logit descending, equal logits
 *     by ascending expert index; slot k holds rank k+1.
 *   - Errors are return codes only.  Argument checks happen on the host
 *     before anything is enqueued:
 *       BEAM_ERR_INVALID_ARG  NULL required pointer, T < 0, K < 1, K > N,
 *                             H/N/I < 1, unknown dtype or layout, misaligned pointer
 *                             (16 bytes for x, weights, out, y_pairs, workspace)
 *       BEAM_ERR_UNSUPPORTED  outside the envelope: N <= 256, K <= 64,
 *                             H % 8 == 0, I % 8 == 0, T*K < 2^24; packed weights
 *                             need bf16, H % 256 == 0 and I % 128 == 0
 *       BEAM_ERR_WORKSPACE    workspace smaller than beam_workspace_bytes()
 *       BEAM_ERR_HIP          a launch failed (hipGetLastError() != success)
 *     T == 0 returns BEAM_OK without launching anything.
 *   - Calls that share a workspace must be ordered on one stream.
 */
#ifndef BEAM_H
#define BEAM_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    BEAM_OK = 0,
    BEAM_ERR_INVALID_ARG = 1,
    BEAM_ERR_UNSUPPORTED = 2,
    BEAM_ERR_WORKSPACE = 3,
    BEAM_ERR_HIP = 4
} beam_status;

typedef enum { BEAM_F32 = 0, BEAM_BF16 = 1 } beam_dtype;

/* Memory order of the expert weights w_gate_up and w_down.
 *   BEAM_WEIGHTS_PLAIN   row-major [N,2I,H] and [N,H,I] as described above.
 *   BEAM_WEIGHTS_PACKED  the same numbers in matrix-core fragment order, written
 *                        once by beam_pack_weights (bf16 only).  Per expert, a
 *                        matrix W[R][Kd] (R output features, Kd reduction) is cut
 *                        into blocks of 32 rows x 16 reduction indices; block
 *                        (rb, ks) is 1 KiB at element offset (rb*(Kd/16) + ks)*512
 *                        and holds, for l = 0..63 and i = 0..7, at l*8 + i the
 *                        value W[row(rb, l & 31)][ks*16 + (l >> 5)*8 + i].
 *                        w_down: row(rb, c) = rb*32 + c.  w_gate_up: blocks
 *                        alternate gate and up: row(2q, c) = gate feature
 *                        q*32 + c, row(2q+1, c) = up feature q*32 + c.
 *                        A wavefront then reads the B operand of a 32x32x16 MFMA
 *                        with one fully coalesced 1 KiB load.  Prefill-sized
 *                        batches run about 1.4x as fast from this layout and
 *                        decode-sized ones as fast as from the plain one, so a
 *                        server needs only the packed copy. */
typedef enum { BEAM_WEIGHTS_PLAIN = 0, BEAM_WEIGHTS_PACKED = 1 } beam_weight_layout;

/* T tokens, H hidden size (d_h), N experts, K experts per token, I expert
 * intermediate size; dtype of x, of every weight and of out; layout of the
 * expert weights.  Host struct. */
typedef struct {
    int32_t T, H, N, K, I;
    int32_t dtype;         /* beam_dtype */
    int32_t weight_layout; /* beam_weight_layout */
} beam_shape;

/* Bytes of device workspace sufficient for any entry point at this shape
 * (worst case: every Top-K pair kept).  Pure host function; returns 0 for an
 * invalid or unsupported shape. */
size_t beam_workspace_bytes(const beam_shape *shape);

/* Static description of a status code (host string, never NULL). */
const char *beam_status_string(beam_status status);

/* Library ABI version (bumped when a signature or struct changes). */
int32_t beam_abi_version(void);

/*
 * One-time repack of static expert weights (Eq. 3's W_gate, W_up, W_down) from
 * BEAM_WEIGHTS_PLAIN into BEAM_WEIGHTS_PACKED order; a pure permutation, so the
 * packed buffers have the size of the plain ones ([N,2I,H] and [N,H,I] elements)
 * and must not overlap them.  bf16 only, H % 32 == 0 and I % 32 == 0, else
 * BEAM_ERR_UNSUPPORTED.  Not part of the per-layer hot path.  shape->T and
 * shape->weight_layout are ignored.
 */
beam_status beam_pack_weights(const beam_shape *shape, const void *w_gate_up, const void *w_down,
                              void *w_gate_up_packed, void *w_down_packed, void *hip_stream);

/*
 * Steps 1-3 of Sec. 3.2: router logits, Top-K + softmax (Eq. 4), mask
 * pre-activation (Eq. 5) and binarisation (Eq. 6) written as the -1 sentinel
 * (App. A.4).
 *   out  topk_ids     [T,K] int32  expert of rank k+1
 *   out  topk_weights [T,K] fp32   g over the K survivors; NOT touched by the mask
 *   out  masked_ids   [T,K] int32  topk_ids where a >= 0, else -1
 *   out  router_logits_dbg, mask_logits_dbg  [T,N] fp32, each may be NULL
 * Logits are accumulated and compared in fp32 (never rounded to bf16).
 */
beam_status beam_route_mask(const beam_shape *shape, const void *x, const void *w_router,
                            const float *router_bias, const void *w_mask, const float *mask_bias,
                            int32_t *topk_ids, float *topk_weights, int32_t *masked_ids,
                            float *router_logits_dbg, float *mask_logits_dbg, void *workspace,
                            size_t workspace_bytes, void *hip_stream);

/*
 * Expert-wise grouping of the kept pairs (App. A.4): a stable counting sort of
 * the flat pair indices f = t*K + k by expert.  Any id outside [0,N) is treated
 * as dropped.  Deterministic: placement uses prefix sums only.
 *   in   masked_ids     [T,K]
 *   out  expert_counts  [N]     kept pairs per expert
 *   out  expert_offsets [N+1]   exclusive prefix sums; [N] = P
 *   out  perm           [T*K]   perm[i] = f of grouped row i for i < P (f ascending
 *                               inside an expert), -1 for i >= P
 *   out  inv_perm       [T*K]   grouped row of pair f, or -1 if dropped
 *   out  num_pairs      [1]     P (stays on the device)
 */
beam_status beam_permute(const beam_shape *shape, const int32_t *masked_ids, int32_t *expert_counts,
                         int32_t *expert_offsets, int32_t *perm, int32_t *inv_perm,
                         int32_t *num_pairs, void *workspace, size_t workspace_bytes,
                         void *hip_stream);

/*
 * The GLU experts of Eq. 3 on the kept pairs only: for grouped row i with
 * pair f = perm[i], token t = f / K and expert e (the segment of
 * expert_offsets that holds i),
 *   y_pairs[i,:] = (SiLU(x_t W_gate^e) (.) (x_t W_up^e)) W_down^e.
 *   out  y_pairs [T*K, H] fp32; rows 0..P-1 are written, the rest untouched.
 * bf16 shapes multiply bf16 operands on the matrix cores with fp32
 * accumulation; the hidden activation is rounded once to bf16 between the two
 * GEMMs.  P is read on the device; the host never learns it.
 */
beam_status beam_expert_ffn(const beam_shape *shape, const void *x, const void *w_gate_up,
                            const void *w_down, const int32_t *expert_offsets, const int32_t *perm,
                            const int32_t *num_pairs, float *y_pairs, void *workspace,
                            size_t workspace_bytes, void *hip_stream);

/*
 * Masked aggregation (Eq. 7-8):
 *   out[t,:] = sum over slots k with masked_ids[t,k] >= 0, in slot order, of
 *              topk_weights[t,k] * y_pairs[inv_perm[t*K+k], :]
 * accumulated in fp32 and rounded once to dtype.  A token with no kept expert
 * gets an exactly +0 row (App. A.3: the layer contributes nothing).
 */
beam_status beam_combine(const beam_shape *shape, const float *y_pairs, const float *topk_weights,
                         const int32_t *masked_ids, const int32_t *inv_perm, void *out,
                         void *hip_stream);

/*
 * The whole layer, Eq. 4-8, in one call: route + mask, group, expert FFNs on
 * the kept pairs, combine.  Intermediates live in the workspace.  The four
 * *_opt outputs may each be NULL: topk_ids_opt [T,K], topk_weights_opt [T,K],
 * masked_ids_opt [T,K], num_pairs_opt [1] (device).
 * Same indices as the staged calls; the output may differ from theirs in the
 * last bits where the fused call orders its fp32 sums differently (few experts
 * with a long reduction: the down projection is summed in four parts) or keeps
 * the pair rows of a very large batch in half precision between the down
 * projection and the aggregation (beam_fused_pair_row_bits), within the same
 * tolerance, and is the same on every run.
 */
beam_status beam_moe_forward(const beam_shape *shape, const void *x, const void *w_router,
                             const float *router_bias, const void *w_mask, const float *mask_bias,
                             const void *w_gate_up, const void *w_down, void *out,
                             int32_t *topk_ids_opt, float *topk_weights_opt,
                             int32_t *masked_ids_opt, int32_t *num_pairs_opt, void *workspace,
                             size_t workspace_bytes, void *hip_stream);

/*
 * beam_moe_forward for callers that cannot allocate device memory or hand in a
 * workspace: code running under HIP graph capture, tight serving loops, harnesses
 * that forbid hipMalloc.  Same arguments (without the optional outputs and the
 * workspace), same kernels, same bits in `out`.  The intermediates live in a device
 * array of BEAM_NOALLOC_WORKSPACE_BYTES that belongs to the library's code object: every
 * GPU the library runs on holds that much memory from the first call on it until the
 * process ends.  The call allocates and frees nothing and does not synchronise; the
 * first call on a device looks up the array's device address (do it once outside a
 * graph capture).
 *   - A shape whose beam_workspace_bytes() exceeds BEAM_NOALLOC_WORKSPACE_BYTES returns
 *     BEAM_ERR_WORKSPACE before anything is enqueued (Qwen3-shaped layer, H 2048,
 *     I 768, top-8: up to 395 tokens; H 4096, I 1536, top-8: up to 186).
 *   - All calls on one GPU share the one array and it keeps the last call's contents:
 *     calls that overlap in time on one GPU (two streams, two threads) race.  Calls on
 *     one stream are ordered and safe.  Nothing in the array needs clearing between
 *     calls.
 */
#define BEAM_NOALLOC_WORKSPACE_BYTES (32u << 20)
beam_status beam_moe_forward_noalloc(const beam_shape *shape, const void *x, const void *w_router,
                                     const float *router_bias, const void *w_mask,
                                     const float *mask_bias, const void *w_gate_up,
                                     const void *w_down, void *out, void *hip_stream);

/*
 * Other activation rules on the same Top-K slots (the paper's ablation on the
 * binarisation threshold, Sec. 4.4, and the cumulative-probability baseline of
 * Sec. 4.1).  A rule only decides which of the K ranked slots are kept, i.e. what
 * masked_ids holds; topk_ids and topk_weights (Eq. 4) are the same under every
 * rule and the weights are never renormalised.
 *   BEAM_RULE_MASK     keep iff a >= param.  For a threshold tau on sigma(a) pass
 *                      param = ln(tau / (1 - tau)); param = 0 is Eq. 6 (tau = 0.5),
 *                      i.e. what the entry points without a rule do.
 *   BEAM_RULE_CUMPROB  with p the softmax of the router logits over all N experts,
 *                      ranks are activated in order until their cumulative p
 *                      exceeds param = phi: slot k is kept iff the slots before
 *                      it sum to at most phi (the first always is; at most the K
 *                      slots exist).  The mask head is not used: w_mask may be
 *                      NULL.  Sums are fp32.
 * "Reduce K at inference" needs no rule: call any entry point with the smaller K.
 * beam_route_rule / beam_moe_forward_rule are beam_route_mask / beam_moe_forward
 * with the rule as second argument (NULL rule: BEAM_ERR_INVALID_ARG; unknown kind
 * or NaN param: BEAM_ERR_INVALID_ARG).
 */
typedef enum { BEAM_RULE_MASK = 0, BEAM_RULE_CUMPROB = 1 } beam_rule_kind;
typedef struct {
    int32_t kind; /* beam_rule_kind */
    float param;
} beam_rule;

beam_status beam_route_rule(const beam_shape *shape, const beam_rule *rule, const void *x,
                            const void *w_router, const float *router_bias, const void *w_mask,
                            const float *mask_bias, int32_t *topk_ids, float *topk_weights,
                            int32_t *masked_ids, float *router_logits_dbg,
                            float *mask_logits_dbg, void *workspace, size_t workspace_bytes,
                            void *hip_stream);
beam_status beam_moe_forward_rule(const beam_shape *shape, const beam_rule *rule, const void *x,
                                  const void *w_router, const float *router_bias,
                                  const void *w_mask, const float *mask_bias,
                                  const void *w_gate_up, const void *w_down, void *out,
                                  int32_t *topk_ids_opt, float *topk_weights_opt,
                                  int32_t *masked_ids_opt, int32_t *num_pairs_opt,
                                  void *workspace, size_t workspace_bytes, void *hip_stream);

/*
 * The whole MoE block of App. A.3 in one call: residual, routed experts under the
 * binary mask, and the shared expert,
 *   out[t,:] = h[t,:] + sum_i g^_i E_i(x_t) + g_sh[t] E_sh(x_t),
 * where x is the already normalised hidden state and h the residual.
 *   shape          N routed experts, K of them per token (as everywhere else)
 *   num_shared     S >= 0.  The shared expert is a GLU expert of width S*I, stored
 *                  as S further experts of width I after the routed ones:
 *                  w_gate_up [N+S, 2I, H], w_down [N+S, H, I]; block j holds
 *                  the shared expert's gate/up rows and down columns j*I .. j*I+I-1
 *                  (a GLU expert is the sum of its column blocks).  For packed
 *                  weights call beam_pack_weights with N+S experts.  S = 0: no
 *                  shared expert (delta_sh = 0).
 *   w_shared_gate  [H] dtype or NULL.  The paper gives no formula for g_sh: NULL
 *                  means g_sh = 1, otherwise g_sh[t] = sigma(x_t . w_shared_gate).
 *                  Must be NULL when S = 0.
 *   residual       [T,H] dtype or NULL (no residual term); its bytes must not overlap
 *                  those of out (BEAM_ERR_INVALID_ARG otherwise).
 *                  The sum starts from h in fp32 and is rounded once.
 *   *_opt          as in beam_moe_forward but with K+S slots per token:
 *                  [T,K+S]; slots K .. K+S-1 are the shared blocks (ids N .. N+S-1,
 *                  weight g_sh, never masked).  num_pairs_opt counts them too.
 * A token whose routed experts are all masked gets h + g_sh E_sh(x) (h itself
 * without a shared expert): the zero-activation case of App. A.3.
 * The workspace must hold beam_block_workspace_bytes(shape, num_shared) bytes
 * (0 = invalid or unsupported; N+S <= 256 and K+S <= 64).
 */
size_t beam_block_workspace_bytes(const beam_shape *shape, int32_t num_shared);
/*
 * Host-only query, for callers and tests that audit the workspace: where the fused
 * entry points keep the fp32 router and mask logits of Sec. 3.2 Step 1 (Eq. 5) inside
 * a workspace of beam_block_workspace_bytes(shape, num_shared) bytes.  Writes the
 * region's byte offset and size and the number of [T,2N] arrays of partial sums it has
 * room for (a prefill-sized logits product may cut its reduction into that many parts).
 * Nothing is enqueued.  Errors as beam_block_workspace_bytes (status instead of 0).
 */
beam_status beam_workspace_logits_region(const beam_shape *shape, int32_t num_shared,
                                         size_t *offset_host, size_t *bytes_host,
                                         int32_t *parts_host);
/*
 * Host-only query: the width in bits of the pair rows E_e(x_t) (Eq. 3, the terms of the sum
 * in Eq. 8) that the FUSED entry points (beam_moe_forward and its variants,
 * beam_moe_block_forward) keep in the workspace between the down projection and the
 * aggregation for this shape.  32: fp32.  16: IEEE half precision (11 significant bits,
 * saturating at +-65504), which the fused layer uses where the rows of a full batch fill the
 * GPU's 256 MiB last-level cache or more and their traffic bounds both kernels; the sum over a
 * token's slots is fp32, in slot order, rounded once, in either case.  The staged
 * beam_expert_ffn / beam_combine always exchange fp32 rows.  0: invalid or unsupported
 * shape.  Nothing is enqueued.
 */
int32_t beam_fused_pair_row_bits(const beam_shape *shape, int32_t num_shared);
beam_status beam_moe_block_forward(const beam_shape *shape, int32_t num_shared, const void *x,
                                   const void *w_router, const float *router_bias,
                                   const void *w_mask, const float *mask_bias,
                                   const void *w_gate_up, const void *w_down,
                                   const void *w_shared_gate, const void *residual, void *out,
                                   int32_t *topk_ids_opt, float *topk_weights_opt,
                                   int32_t *masked_ids_opt, int32_t *num_pairs_opt,
                                   void *workspace, size_t workspace_bytes, void *hip_stream);

/*
 * Training mode (Sec. 3.3).  The forward of training evaluates EVERY Top-K expert
 * whatever the mask says (Sec. 3.3.1) and applies the binary mask in the sum; it
 * composes from the entry points above: beam_route_mask, beam_permute on topk_ids
 * (not masked_ids), beam_expert_ffn, beam_combine with masked_ids and that
 * grouping's inv_perm.  This call is the mask router's backward under the
 * straight-through estimator (Eq. 9) with the sparsity regulariser (Eq. 10):
 *   dL/dg^_k       = <grad_out[t,:], y_pairs[inv_perm[t*K+k], :]>
 *   grad_a[t,k]    = (dL/dg^_k * topk_weights[t,k] + reg_coeff / K) * sigma'(a)   (Eq. 12)
 *                    with a = mask_logits[t, topk_ids[t,k]], sigma' = sigma (1 - sigma)
 *   grad_w_mask[e] = sum over the pairs (t,k) of expert e of grad_a[t,k] * x[t,:]
 *   loss_reg[t]    = (1/K) sum_k sigma(a)                                          (Eq. 10)
 * in   mask_logits [T,N] fp32 (beam_route_mask's mask_logits_dbg); y_pairs [T*K,H]
 *      fp32, expert_offsets [N+1], perm, inv_perm [T*K]: expert outputs and grouping
 *      of ALL Top-K pairs; grad_out [T,H] dtype = dL/dy; reg_coeff = the factor of
 *      L_reg in the loss (beta, or beta/T if the caller averages over tokens: the
 *      paper fixes no reduction).
 * out  grad_a [T,K] fp32; grad_w_mask [N,H] fp32 (rows of experts that no token
 *      selected are zero: Theorem 1); loss_reg [T] fp32.
 * fp32 arithmetic, fixed summation order (per 128-row tile, then per expert): the
 * result is reproducible run to run.  T = 0 writes nothing.
 */
beam_status beam_mask_router_backward(const beam_shape *shape, const void *x,
                                      const int32_t *topk_ids, const float *topk_weights,
                                      const float *mask_logits, const float *y_pairs,
                                      const int32_t *expert_offsets, const int32_t *perm,
                                      const int32_t *inv_perm, const void *grad_out,
                                      float reg_coeff, float *grad_a, float *grad_w_mask,
                                      float *loss_reg, void *workspace, size_t workspace_bytes,
                                      void *hip_stream);

/*
 * Measurement aid, not part of the layer: beam_moe_forward with a HIP event
 * recorded on `hip_stream` before and after every stage.  Unlike every other
 * entry point this one creates and destroys events and WAITS for the stream;
 * it then writes the elapsed milliseconds of the BEAM_NUM_STAGES stages to the
 * HOST array stage_ms_host, in this order:
 *   0 router + mask logits (Step 1-2)     1 Top-K / softmax / mask (Step 1, 3)
 *   2 grouping by expert (App. A.4)       3 gate/up GEMM + SiLU (Eq. 3)
 *   4 down GEMM (Eq. 3)                   5 masked aggregation (Eq. 7-8)
 * Each figure includes that stage's launch gaps.
 */
#define BEAM_NUM_STAGES 6
beam_status beam_moe_forward_timed(const beam_shape *shape, const void *x, const void *w_router,
                                   const float *router_bias, const void *w_mask,
                                   const float *mask_bias, const void *w_gate_up,
                                   const void *w_down, void *out, void *workspace,
                                   size_t workspace_bytes, void *hip_stream,
                                   float *stage_ms_host);

/*
 * Measurement aids, not part of the layer: what this GPU delivers, to read a
 * kernel's roofline fraction against.  Both only enqueue a kernel; the caller
 * times it (events on `hip_stream`).
 *   beam_probe_stream_read  reads `buf` (device, >= 64 MiB, 16-byte aligned) once
 *       with coalesced non-temporal 16-byte loads, eight in flight per lane; writes the
 *       number of bytes the kernel really reads (bytes rounded down to whole
 *       batches) to *bytes_read_host.  sink: >= 4 device bytes, left unchanged.
 *   beam_probe_mfma  runs iters x 4 back-to-back v_mfma_f32_32x32x16_bf16 per
 *       wavefront on 2048 workgroups with register operands that change every
 *       iteration; writes the flop count to *flops_host.
 */
beam_status beam_probe_stream_read(const void *buf, size_t bytes, void *sink, void *hip_stream,
                                   size_t *bytes_read_host);
beam_status beam_probe_mfma(int32_t iters, void *sink, void *hip_stream, double *flops_host);

/* The same measurement aid for beam_moe_block_forward (the shared-gate kernel,
 * if any, is counted in stage 0). */
beam_status beam_moe_block_forward_timed(const beam_shape *shape, int32_t num_shared,
                                         const void *x, const void *w_router,
                                         const float *router_bias, const void *w_mask,
                                         const float *mask_bias, const void *w_gate_up,
                                         const void *w_down, const void *w_shared_gate,
                                         const void *residual, void *out, void *workspace,
                                         size_t workspace_bytes, void *hip_stream,
                                         float *stage_ms_host);

#ifdef __cplusplus
}
#endif
#endif /* BEAM_H */

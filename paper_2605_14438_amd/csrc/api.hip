// The C ABI of libbeam (include/beam.h): argument checks on the host, the
// workspace carve-up, and the order in which the stage kernels are enqueued.
// Nothing here allocates, copies to the host or synchronises (the stage-timed
// measurement entry point excepted).
#include <atomic>

#include "common.hpp"

namespace beam {

bool stream_ffn_supported(const beam_shape &s);
bool tiled_ffn_supported(const beam_shape &s);
hipError_t launch_gate_up_generic(const beam_shape &s, const void *x, const void *w_gate_up,
                                  const int32_t *offsets, const int32_t *perm,
                                  const int32_t *num_pairs, void *hidden, hipStream_t st);
hipError_t launch_down_generic(const beam_shape &s, const void *hidden, const void *w_down,
                               const int32_t *offsets, const int32_t *num_pairs, float *y_pairs,
                               hipStream_t st);
// want: kRegimeAny, or the regime (work list hdr[2]) under which the kernel is to run at all
hipError_t launch_gate_up_stream(const beam_shape &s, const void *x, const void *w_gate_up,
                                 const int32_t *offsets, const int32_t *perm, const WorkList &wl,
                                 void *hidden, hipStream_t st, int want);
hipError_t launch_down_stream(const beam_shape &s, const void *hidden, const void *w_down,
                              const int32_t *offsets, const WorkList &wl, float *y_pairs,
                              hipStream_t st, int want);
hipError_t launch_gate_up_tiled(const beam_shape &s, const void *x, const void *w_gate_up,
                                const int32_t *offsets, const int32_t *perm, const WorkList &wl,
                                void *hidden, hipStream_t st, int want);
hipError_t launch_down_tiled(const beam_shape &s, const void *hidden, const void *w_down,
                             const int32_t *offsets, const WorkList &wl, float *y_pairs,
                             hipStream_t st, int k_split, int want, bool y16 = false);
hipError_t launch_pack_weights(const beam_shape &s, const void *w_gate_up, const void *w_down,
                               void *w_gate_up_packed, void *w_down_packed, hipStream_t st);

hipError_t launch_mask_router_backward(const beam_shape &s, const void *x,
                                       const int32_t *topk_ids, const float *topk_w,
                                       const float *mask_logits, const float *y_pairs,
                                       const int32_t *offsets, const int32_t *perm,
                                       const int32_t *inv_perm, const void *grad_out,
                                       float reg_coeff, const WorkList &wl, int max_tiles,
                                       float *partial, float *grad_a, float *grad_w_mask,
                                       float *loss_reg, hipStream_t st);

hipError_t launch_probe_stream_read(const void *buf, size_t bytes, void *sink, hipStream_t st);
hipError_t launch_probe_mfma(int iters, void *sink, hipStream_t st);

static inline size_t align_up(size_t v) { return (v + 255) & ~(size_t)255; }

static bool use_tiled(const beam_shape &s);

// Parts the fused layer cuts the down GEMM's reduction into.  The tiled GEMM has
// (row tiles) x H/256 items for 512 resident workgroups; a few experts with a long
// reduction (Mixtral-shaped: 8 experts, I = 14336) give fewer items than that, each
// hundreds of K-steps long, and most of the chip idles.  Decided from the shape alone
// (item count with every pair kept); the partial sums cost k_split x [T*K,H] fp32 of
// workspace and are added in part order by the aggregation.  Measured on the
// Mixtral-shaped layer, down GEMM: T = 256 384 -> 167 us, T = 512 404 -> 173,
// T = 1024 403 -> 250 (the aggregation gains 4-12 us); at T = 2048 (384 items of work
// already) four parts give 407 -> 352 us but the aggregation and the gate/up GEMM lose
// as much, and two parts give nothing, so it stays whole.
static int down_split_k_if_tiled(const beam_shape &s);
static int down_split_k(const beam_shape &s) {
    return use_tiled(s) ? down_split_k_if_tiled(s) : 1;
}

// `s` counts every expert and slot the grouped kernels see; the last S of them are the
// shared experts appended by the block entry point, which the router never scores.
WsLayout ws_layout(const beam_shape &s, int S) {
    WsLayout L;
    const size_t T = (size_t)s.T, N = (size_t)s.N, K = (size_t)s.K;
    const size_t TK = T * K;
    const size_t esz = s.dtype == BEAM_BF16 ? 2 : 4;
    L.max_tiles = (int)(TK / kTileM + N);  // sum over experts of ceil(c_e / kTileM)
    size_t off = 0;
    auto take = [&](size_t bytes) {
        const size_t at = off;
        off = align_up(off + bytes);
        return at;
    };
    // one allocation: the prefill logits kernel writes them as a single [T,2N] array, one
    // per part of its reduction.  The logits GEMM and Top-K run on the routed experts only
    // and cut the reduction by THEIR column count (2 * (N - S) can fit one column tile where
    // 2 * N needs two, which doubles the parts), so the parts are counted for that shape.
    beam_shape routed = s;
    routed.N = s.N - S;
    routed.K = s.K - S;
    const int parts_routed = logits_split_k(routed), parts_all = logits_split_k(s);
    L.logit_parts = parts_routed > parts_all ? parts_routed : parts_all;
    L.router_logits = take(2 * T * N * 4 * (size_t)L.logit_parts);
    L.router_logits_bytes = off - L.router_logits;
    L.mask_logits = L.router_logits + T * (N - S) * 4;
    L.packed_heads = take((2 * N + 255) / 256 * 256 * (size_t)s.H * esz);  // padded to a column tile
    L.topk_ids = take(TK * 4);
    L.topk_w = take(TK * 4);
    L.masked_ids = take(TK * 4);
    L.g_shared = take(T * 4);
    L.slice_counts = take((size_t)permute_slices((long)TK) * N * 4);
    L.counts = take(N * 4);
    L.offsets = take((N + 1) * 4);
    L.num_pairs = take(4);
    L.perm = take(TK * 4);
    L.inv_perm = take(TK * 4);
    L.work = take((16 + 3 * N + 2 * (size_t)L.max_tiles) * 4);
    L.hidden = take(TK * (size_t)s.I * esz);
    L.y_pairs = take(TK * (size_t)s.H * 4 * down_split_k(s));
    L.tile_partial = take((size_t)L.max_tiles * s.H * 4);
    L.total = off;
    return L;
}

WorkList work_list(void *base, const beam_shape &s, int max_tiles) {
    WorkList wl;
    int32_t *p = (int32_t *)base;
    wl.hdr = p;
    wl.active = p + 16;
    wl.active_beg = wl.active + s.N;
    wl.active_end = wl.active_beg + s.N;
    wl.tile_expert = wl.active_end + s.N;
    wl.tile_row0 = wl.tile_expert + max_tiles;
    return wl;
}

// What the shape alone says about the expert GEMMs.  Decode-sized batches (a handful of
// rows per expert whatever the keep rate) stream; from 256 rows per expert in the worst
// case the tiled GEMM it is; in between the right family depends on the keep rate and the
// routing skew, which only the device knows after grouping (work list hdr[2]): both
// families are enqueued and the one not chosen leaves at once (measured: a batch of 512
// tokens with every pair kept and a skewed router 419 us streamed against 226 us tiled, 15 %
// kept 130 against 143; 1024 tokens, uniform router, 15 % kept 248 against 270).
// A split down reduction (few experts, long reduction) is a host decision the aggregation
// shares, so those shapes stay with the host's rule.
static int down_split_k_if_tiled(const beam_shape &s) {
    if (!tiled_ffn_supported(s) || s.I < 4096) return 1;
    const long items = ((long)s.T * s.K / kTileM + s.N) * (s.H / 256);
    const int k_split = items <= 512 ? 4 : 1;
    return (s.I / 64) % k_split == 0 ? k_split : 1;   // whole 64-wide K-steps per part
}

Regime ffn_regime(const beam_shape &s) {
    const bool tiled_ok = tiled_ffn_supported(s), stream_ok = stream_ffn_supported(s);
    if (!tiled_ok && !stream_ok) return Regime::Generic;
    const long TK = (long)s.T * s.K;
    if (!stream_ok)   // packed weights outside the streaming envelope have no other reader
        return (s.weight_layout == BEAM_WEIGHTS_PACKED || TK > 32L * s.N) ? Regime::Tiled
                                                                          : Regime::Generic;
    if (!tiled_ok) return Regime::Stream;
    if (TK <= kChunk || TK <= 8L * s.N) return Regime::Stream;   // a few rows per expert at most
    if (TK >= 256L * s.N) return Regime::Tiled;
    if (down_split_k_if_tiled(s) > 1) return TK > 32L * s.N ? Regime::Tiled : Regime::Stream;
    return Regime::Auto;
}

static bool use_tiled(const beam_shape &s) { return ffn_regime(s) == Regime::Tiled; }

// Precision of the pair rows y = E_e(x_t) between the down GEMM and the aggregation INSIDE
// the fused entry points.  The staged beam_expert_ffn / beam_combine always exchange fp32.
// Where the rows of a full batch fill the 256 MiB last-level cache or more (so that the down GEMM
// writes them to HBM and the aggregation reads them back from there, which is what bounds
// both kernels at a high keep rate: 2 x 1.07 GB for the Qwen3-shaped layer at 16384 tokens)
// the fused layer keeps them in IEEE half precision: 11 significant bits, a rounding eight
// times finer than that of the bf16 output and of the bf16 hidden activation h before it,
// saturating at +-65504.  The sum over a token's slots is still fp32, in slot order, rounded
// once.  Decided from the shape alone (the aggregation must know the format when it is
// enqueued): the tiled GEMM on the host's word, whole reduction, bf16 layer.
static bool pair_rows_16bit(const beam_shape &s) {
    return s.dtype == BEAM_BF16 && use_tiled(s) && down_split_k_if_tiled(s) == 1 &&
           s.H % 256 == 0 && (size_t)s.T * s.K * s.H * sizeof(float) >= kStreamBytes;
}

hipError_t launch_gate_up(const beam_shape &s, const void *x, const void *w_gate_up,
                          const int32_t *offsets, const int32_t *perm, const int32_t *num_pairs,
                          const WorkList &wl, void *hidden, hipStream_t st) {
    switch (ffn_regime(s)) {
        case Regime::Tiled:
            return launch_gate_up_tiled(s, x, w_gate_up, offsets, perm, wl, hidden, st, kRegimeAny);
        case Regime::Stream:
            return launch_gate_up_stream(s, x, w_gate_up, offsets, perm, wl, hidden, st, kRegimeAny);
        case Regime::Auto: {
            const hipError_t e = launch_gate_up_stream(s, x, w_gate_up, offsets, perm, wl, hidden,
                                                       st, kRegimeStream);
            if (e != hipSuccess) return e;
            return launch_gate_up_tiled(s, x, w_gate_up, offsets, perm, wl, hidden, st,
                                        kRegimeTiled);
        }
        default:
            return launch_gate_up_generic(s, x, w_gate_up, offsets, perm, num_pairs, hidden, st);
    }
}

hipError_t launch_down(const beam_shape &s, const void *hidden, const void *w_down,
                       const int32_t *offsets, const int32_t *num_pairs, const WorkList &wl,
                       float *y_pairs, hipStream_t st, int k_split, bool y16) {
    if (y16 && ffn_regime(s) != Regime::Tiled) return hipErrorInvalidValue;
    switch (ffn_regime(s)) {
        case Regime::Tiled:
            return launch_down_tiled(s, hidden, w_down, offsets, wl, y_pairs, st, k_split,
                                     kRegimeAny, y16);
        case Regime::Stream:
            return launch_down_stream(s, hidden, w_down, offsets, wl, y_pairs, st, kRegimeAny);
        case Regime::Auto: {
            const hipError_t e =
                launch_down_stream(s, hidden, w_down, offsets, wl, y_pairs, st, kRegimeStream);
            if (e != hipSuccess) return e;
            return launch_down_tiled(s, hidden, w_down, offsets, wl, y_pairs, st, 1, kRegimeTiled);
        }
        default:
            return launch_down_generic(s, hidden, w_down, offsets, num_pairs, y_pairs, st);
    }
}

static beam_status check_shape(const beam_shape *s) {
    if (!s) return BEAM_ERR_INVALID_ARG;
    if (s->dtype != BEAM_F32 && s->dtype != BEAM_BF16) return BEAM_ERR_INVALID_ARG;
    if (s->weight_layout != BEAM_WEIGHTS_PLAIN && s->weight_layout != BEAM_WEIGHTS_PACKED)
        return BEAM_ERR_INVALID_ARG;
    if (s->T < 0 || s->H < 1 || s->N < 1 || s->I < 1 || s->K < 1 || s->K > s->N)
        return BEAM_ERR_INVALID_ARG;
    if (s->N > 256 || s->K > 64 || s->H % 8 != 0 || s->I % 8 != 0) return BEAM_ERR_UNSUPPORTED;
    if ((long)s->T * s->K >= (1L << 24)) return BEAM_ERR_UNSUPPORTED;
    if (s->weight_layout == BEAM_WEIGHTS_PACKED && !tiled_ffn_supported(*s))
        return BEAM_ERR_UNSUPPORTED;
    return BEAM_OK;
}

static inline bool misaligned(const void *p) { return ((uintptr_t)p & 15u) != 0; }

static beam_status check_ws(const beam_shape &s, void *ws, size_t bytes, const WsLayout &L) {
    (void)s;
    if (!ws || misaligned(ws)) return BEAM_ERR_INVALID_ARG;
    if (bytes < L.total) return BEAM_ERR_WORKSPACE;
    return BEAM_OK;
}

}  // namespace beam

using namespace beam;

#define BEAM_TRY_HIP(expr)                          \
    do {                                            \
        if ((expr) != hipSuccess) return BEAM_ERR_HIP; \
    } while (0)

extern "C" {

int32_t beam_abi_version(void) { return 3; }

const char *beam_status_string(beam_status status) {
    switch (status) {
        case BEAM_OK: return "ok";
        case BEAM_ERR_INVALID_ARG: return "invalid argument";
        case BEAM_ERR_UNSUPPORTED: return "shape outside the supported envelope";
        case BEAM_ERR_WORKSPACE: return "workspace too small";
        case BEAM_ERR_HIP: return "HIP launch failed";
    }
    return "unknown status";
}

size_t beam_workspace_bytes(const beam_shape *shape) {
    if (check_shape(shape) != BEAM_OK) return 0;
    return ws_layout(*shape).total;
}

beam_status beam_pack_weights(const beam_shape *shape, const void *w_gate_up, const void *w_down,
                              void *w_gate_up_packed, void *w_down_packed, void *hip_stream) {
    if (!shape) return BEAM_ERR_INVALID_ARG;
    beam_shape s = *shape;
    s.T = 0;
    s.weight_layout = BEAM_WEIGHTS_PLAIN;
    beam_status st = check_shape(&s);
    if (st != BEAM_OK) return st;
    if (!w_gate_up || !w_down || !w_gate_up_packed || !w_down_packed) return BEAM_ERR_INVALID_ARG;
    if (misaligned(w_gate_up) || misaligned(w_down) || misaligned(w_gate_up_packed) ||
        misaligned(w_down_packed) || w_gate_up == w_gate_up_packed || w_down == w_down_packed)
        return BEAM_ERR_INVALID_ARG;
    if (s.dtype != BEAM_BF16 || s.H % 32 != 0 || s.I % 32 != 0) return BEAM_ERR_UNSUPPORTED;
    BEAM_TRY_HIP(launch_pack_weights(s, w_gate_up, w_down, w_gate_up_packed, w_down_packed,
                                     (hipStream_t)hip_stream));
    return BEAM_OK;
}

static beam_status check_rule(const beam_rule *rule, RouteOpts *opt) {
    if (!rule) return BEAM_OK;  // Eq. 6: mask pre-activation >= 0
    if (rule->kind != BEAM_RULE_MASK && rule->kind != BEAM_RULE_CUMPROB)
        return BEAM_ERR_INVALID_ARG;
    if (!(rule->param == rule->param)) return BEAM_ERR_INVALID_ARG;  // NaN
    opt->rule = rule->kind;
    opt->param = rule->param;
    return BEAM_OK;
}

static beam_status route_impl(const beam_shape *shape, const beam_rule *rule, const void *x,
                              const void *w_router, const float *router_bias, const void *w_mask,
                              const float *mask_bias, int32_t *topk_ids, float *topk_weights,
                              int32_t *masked_ids, float *router_logits_dbg,
                              float *mask_logits_dbg, void *workspace, size_t workspace_bytes,
                              void *hip_stream) {
    beam_status st = check_shape(shape);
    if (st != BEAM_OK) return st;
    const beam_shape &s = *shape;
    RouteOpts opt;
    st = check_rule(rule, &opt);
    if (st != BEAM_OK) return st;
    if (!w_mask && opt.rule == BEAM_RULE_CUMPROB) w_mask = w_router;  // head computed, not used
    if (!x || !w_router || !w_mask || !topk_ids || !topk_weights || !masked_ids)
        return BEAM_ERR_INVALID_ARG;
    if (misaligned(x) || misaligned(w_router) || misaligned(w_mask)) return BEAM_ERR_INVALID_ARG;
    const WsLayout L = ws_layout(s);
    st = check_ws(s, workspace, workspace_bytes, L);
    if (st != BEAM_OK) return st;
    if (s.T == 0) return BEAM_OK;
    char *ws = (char *)workspace;
    hipStream_t stream = (hipStream_t)hip_stream;
    if (logits_tiled_supported(s)) {
        // prefill-sized: both heads as one tiled GEMM into [T,2N]; biases join at Top-K and
        // in the optional copies
        float *l2 = (float *)(ws + L.router_logits);
        BEAM_TRY_HIP(launch_logits_tiled(s, x, w_router, w_mask, ws + L.packed_heads, l2, stream));
        const int parts = logits_split_k(s);
        BEAM_TRY_HIP(launch_topk_mask(s, l2, l2 + s.N, router_bias, mask_bias, 2 * s.N, opt,
                                      topk_ids, topk_weights, masked_ids, stream, parts));
        if (router_logits_dbg || mask_logits_dbg)
            BEAM_TRY_HIP(launch_split_logits(s, l2, router_bias, mask_bias, router_logits_dbg,
                                             mask_logits_dbg, stream, parts));
        return BEAM_OK;
    }
    float *rl = router_logits_dbg ? router_logits_dbg : (float *)(ws + L.router_logits);
    float *ml = mask_logits_dbg ? mask_logits_dbg : (float *)(ws + L.mask_logits);
    BEAM_TRY_HIP(launch_logits(s, x, w_router, router_bias, w_mask, mask_bias, rl, ml, stream));
    BEAM_TRY_HIP(launch_topk_mask(s, rl, ml, nullptr, nullptr, s.N, opt, topk_ids, topk_weights,
                                  masked_ids, stream));
    return BEAM_OK;
}

beam_status beam_route_mask(const beam_shape *shape, const void *x, const void *w_router,
                            const float *router_bias, const void *w_mask, const float *mask_bias,
                            int32_t *topk_ids, float *topk_weights, int32_t *masked_ids,
                            float *router_logits_dbg, float *mask_logits_dbg, void *workspace,
                            size_t workspace_bytes, void *hip_stream) {
    return route_impl(shape, nullptr, x, w_router, router_bias, w_mask, mask_bias, topk_ids,
                      topk_weights, masked_ids, router_logits_dbg, mask_logits_dbg, workspace,
                      workspace_bytes, hip_stream);
}

beam_status beam_route_rule(const beam_shape *shape, const beam_rule *rule, const void *x,
                            const void *w_router, const float *router_bias, const void *w_mask,
                            const float *mask_bias, int32_t *topk_ids, float *topk_weights,
                            int32_t *masked_ids, float *router_logits_dbg,
                            float *mask_logits_dbg, void *workspace, size_t workspace_bytes,
                            void *hip_stream) {
    if (!rule) return BEAM_ERR_INVALID_ARG;
    return route_impl(shape, rule, x, w_router, router_bias, w_mask, mask_bias, topk_ids,
                      topk_weights, masked_ids, router_logits_dbg, mask_logits_dbg, workspace,
                      workspace_bytes, hip_stream);
}

beam_status beam_permute(const beam_shape *shape, const int32_t *masked_ids, int32_t *expert_counts,
                         int32_t *expert_offsets, int32_t *perm, int32_t *inv_perm,
                         int32_t *num_pairs, void *workspace, size_t workspace_bytes,
                         void *hip_stream) {
    beam_status st = check_shape(shape);
    if (st != BEAM_OK) return st;
    const beam_shape &s = *shape;
    if (!masked_ids || !expert_counts || !expert_offsets || !perm || !inv_perm || !num_pairs)
        return BEAM_ERR_INVALID_ARG;
    const WsLayout L = ws_layout(s);
    st = check_ws(s, workspace, workspace_bytes, L);
    if (st != BEAM_OK) return st;
    char *ws = (char *)workspace;
    const WorkList wl = work_list(ws + L.work, s, L.max_tiles);
    // T == 0 still defines the outputs: no pairs
    BEAM_TRY_HIP(launch_permute(s, masked_ids, expert_counts, expert_offsets, perm, inv_perm,
                                num_pairs, (int32_t *)(ws + L.slice_counts), wl,
                                (hipStream_t)hip_stream, !use_tiled(s)));
    return BEAM_OK;
}

beam_status beam_expert_ffn(const beam_shape *shape, const void *x, const void *w_gate_up,
                            const void *w_down, const int32_t *expert_offsets, const int32_t *perm,
                            const int32_t *num_pairs, float *y_pairs, void *workspace,
                            size_t workspace_bytes, void *hip_stream) {
    beam_status st = check_shape(shape);
    if (st != BEAM_OK) return st;
    const beam_shape &s = *shape;
    if (!x || !w_gate_up || !w_down || !expert_offsets || !perm || !num_pairs || !y_pairs)
        return BEAM_ERR_INVALID_ARG;
    if (misaligned(x) || misaligned(w_gate_up) || misaligned(w_down) || misaligned(y_pairs))
        return BEAM_ERR_INVALID_ARG;
    const WsLayout L = ws_layout(s);
    st = check_ws(s, workspace, workspace_bytes, L);
    if (st != BEAM_OK) return st;
    if (s.T == 0) return BEAM_OK;
    char *ws = (char *)workspace;
    hipStream_t stream = (hipStream_t)hip_stream;
    const WorkList wl = work_list(ws + L.work, s, L.max_tiles);
    BEAM_TRY_HIP(launch_work_list(s, expert_offsets, wl, stream, !use_tiled(s)));
    BEAM_TRY_HIP(launch_gate_up(s, x, w_gate_up, expert_offsets, perm, num_pairs, wl,
                                ws + L.hidden, stream));
    BEAM_TRY_HIP(launch_down(s, ws + L.hidden, w_down, expert_offsets, num_pairs, wl, y_pairs,
                             stream));
    return BEAM_OK;
}

beam_status beam_combine(const beam_shape *shape, const float *y_pairs, const float *topk_weights,
                         const int32_t *masked_ids, const int32_t *inv_perm, void *out,
                         void *hip_stream) {
    beam_status st = check_shape(shape);
    if (st != BEAM_OK) return st;
    const beam_shape &s = *shape;
    if (!y_pairs || !topk_weights || !masked_ids || !inv_perm || !out) return BEAM_ERR_INVALID_ARG;
    if (misaligned(y_pairs) || misaligned(out)) return BEAM_ERR_INVALID_ARG;
    if (s.T == 0) return BEAM_OK;
    BEAM_TRY_HIP(launch_combine(s, y_pairs, topk_weights, masked_ids, inv_perm, nullptr, out,
                                (hipStream_t)hip_stream));
    return BEAM_OK;
}

// The fused layer.  `shape` counts the routed experts (N, K per token); S shared
// experts (App. A.3) follow them in the weight arrays and ride the same grouped
// kernels as experts N .. N+S-1 with S always-kept slots per token, so from
// grouping on everything runs at N+S experts and K+S slots.
static beam_status moe_forward_impl(const beam_shape *shape, int S, const beam_rule *rule,
                                    const void *x, const void *w_router, const float *router_bias,
                                    const void *w_mask, const float *mask_bias,
                                    const void *w_gate_up, const void *w_down,
                                    const void *w_shared_gate, const void *residual, void *out,
                                    int32_t *topk_ids_opt, float *topk_weights_opt,
                                    int32_t *masked_ids_opt, int32_t *num_pairs_opt,
                                    void *workspace, size_t workspace_bytes, void *hip_stream,
                                    hipEvent_t *ev) {
    beam_status st = check_shape(shape);
    if (st != BEAM_OK) return st;
    const beam_shape &s = *shape;
    if (S < 0) return BEAM_ERR_INVALID_ARG;
    RouteOpts opt;
    st = check_rule(rule, &opt);
    if (st != BEAM_OK) return st;
    if (!w_mask && opt.rule == BEAM_RULE_CUMPROB) w_mask = w_router;  // head computed, not used
    beam_shape se = s;  // experts and slots including the shared ones
    se.N = s.N + S;
    se.K = s.K + S;
    if (S > 0) {
        // K <= N holds for the routed part; the slot count may exceed N + S never
        if (se.N > 256 || se.K > 64) return BEAM_ERR_UNSUPPORTED;
        if ((long)se.T * se.K >= (1L << 24)) return BEAM_ERR_UNSUPPORTED;
        if (se.weight_layout == BEAM_WEIGHTS_PACKED && !tiled_ffn_supported(se))
            return BEAM_ERR_UNSUPPORTED;
    }
    if (!x || !w_router || !w_mask || !w_gate_up || !w_down || !out) return BEAM_ERR_INVALID_ARG;
    if (misaligned(x) || misaligned(w_router) || misaligned(w_mask) || misaligned(w_gate_up) ||
        misaligned(w_down) || misaligned(out) || misaligned(residual) ||
        misaligned(w_shared_gate))
        return BEAM_ERR_INVALID_ARG;
    if (w_shared_gate && S == 0) return BEAM_ERR_INVALID_ARG;
    if (residual) {
        // both are __restrict__ in the kernels: the byte ranges must not overlap
        const size_t nbytes = (size_t)s.T * s.H * (s.dtype == BEAM_BF16 ? 2 : 4);
        const uintptr_t r0 = (uintptr_t)residual, o0 = (uintptr_t)out;
        if (r0 < o0 + nbytes && o0 < r0 + nbytes) return BEAM_ERR_INVALID_ARG;
    }
    const WsLayout L = ws_layout(se, S);
    st = check_ws(se, workspace, workspace_bytes, L);
    if (st != BEAM_OK) return st;
    if (s.T == 0) return BEAM_OK;
    char *ws = (char *)workspace;
    hipStream_t stream = (hipStream_t)hip_stream;
    float *rl = (float *)(ws + L.router_logits);
    float *ml = rl + (size_t)s.T * s.N;
    int32_t *ids = topk_ids_opt ? topk_ids_opt : (int32_t *)(ws + L.topk_ids);
    float *gw = topk_weights_opt ? topk_weights_opt : (float *)(ws + L.topk_w);
    int32_t *mids = masked_ids_opt ? masked_ids_opt : (int32_t *)(ws + L.masked_ids);
    int32_t *np = num_pairs_opt ? num_pairs_opt : (int32_t *)(ws + L.num_pairs);
    int32_t *counts = (int32_t *)(ws + L.counts);
    int32_t *offsets = (int32_t *)(ws + L.offsets);
    int32_t *perm = (int32_t *)(ws + L.perm);
    int32_t *inv = (int32_t *)(ws + L.inv_perm);
    float *y_pairs = (float *)(ws + L.y_pairs);
    float *g_shared = w_shared_gate ? (float *)(ws + L.g_shared) : nullptr;
    const WorkList wl = work_list(ws + L.work, se, L.max_tiles);
    opt.S = S;
    opt.g_shared = g_shared;

#define BEAM_STAGE_MARK(i)                                      \
    do {                                                        \
        if (ev) BEAM_TRY_HIP(hipEventRecord(ev[i], stream));    \
    } while (0)
    BEAM_STAGE_MARK(0);
    if (g_shared) BEAM_TRY_HIP(launch_shared_gate(s, x, w_shared_gate, g_shared, stream));
    if (tiny_decode_supported(se, 0) && stream_ffn_supported(s)) {
        // A handful of pairs: three kernels, routing recomputed where it is needed,
        // pairs addressed by flat index, aggregation folded into the down projection.
        BEAM_TRY_HIP(launch_logits(s, x, w_router, router_bias, w_mask, mask_bias, rl, ml, stream,
                                   num_pairs_opt));
        for (int i = 1; i <= 3; ++i) BEAM_STAGE_MARK(i);
        BEAM_TRY_HIP(launch_tiny_gate_up(s, opt, x, rl, ml, w_gate_up, ws + L.hidden, stream));
        BEAM_STAGE_MARK(4);
        BEAM_TRY_HIP(launch_tiny_down_combine(s, opt, rl, ml, ws + L.hidden, w_down, residual,
                                              out, topk_ids_opt, topk_weights_opt,
                                              masked_ids_opt, num_pairs_opt, stream));
        for (int i = 5; i <= 6; ++i) BEAM_STAGE_MARK(i);
        return BEAM_OK;
    }
    bool grouped = false;
    if (logits_tiled_supported(s)) {
        // prefill: both heads as one tiled GEMM into a [T,2N] array; biases join at Top-K
        BEAM_TRY_HIP(launch_logits_tiled(s, x, w_router, w_mask, ws + L.packed_heads, rl, stream));
        BEAM_STAGE_MARK(1);
        BEAM_TRY_HIP(launch_topk_mask(s, rl, rl + s.N, router_bias, mask_bias, 2 * s.N, opt, ids,
                                      gw, mids, stream, logits_split_k(s)));
    } else {
        BEAM_TRY_HIP(launch_logits(s, x, w_router, router_bias, w_mask, mask_bias, rl, ml, stream));
        BEAM_STAGE_MARK(1);
        if (route_permute_supported(s, opt, rl, ml)) {
            // decode: Top-K, mask and grouping in one launch of one workgroup
            BEAM_TRY_HIP(launch_route_permute(s, rl, ml, opt, ids, gw, mids, counts, offsets, perm,
                                              inv, np, wl, stream));
            grouped = true;
        } else {
            BEAM_TRY_HIP(launch_topk_mask(s, rl, ml, nullptr, nullptr, s.N, opt, ids, gw, mids,
                                          stream));
        }
    }
    BEAM_STAGE_MARK(2);
    if (!grouped)
        BEAM_TRY_HIP(launch_permute(se, mids, counts, offsets, perm, inv, np,
                                    (int32_t *)(ws + L.slice_counts), wl, stream,
                                    !use_tiled(se)));
    BEAM_STAGE_MARK(3);
    BEAM_TRY_HIP(launch_gate_up(se, x, w_gate_up, offsets, perm, np, wl, ws + L.hidden, stream));
    BEAM_STAGE_MARK(4);
    const int k_split = down_split_k(se);
    const bool y16 = pair_rows_16bit(se);
    BEAM_TRY_HIP(launch_down(se, ws + L.hidden, w_down, offsets, np, wl, y_pairs, stream,
                             k_split, y16));
    BEAM_STAGE_MARK(5);
    BEAM_TRY_HIP(launch_combine(se, y_pairs, gw, mids, inv, residual, out, stream, np, k_split,
                                y16));
    BEAM_STAGE_MARK(6);
#undef BEAM_STAGE_MARK
    return BEAM_OK;
}

beam_status beam_moe_forward(const beam_shape *shape, const void *x, const void *w_router,
                             const float *router_bias, const void *w_mask, const float *mask_bias,
                             const void *w_gate_up, const void *w_down, void *out,
                             int32_t *topk_ids_opt, float *topk_weights_opt,
                             int32_t *masked_ids_opt, int32_t *num_pairs_opt, void *workspace,
                             size_t workspace_bytes, void *hip_stream) {
    return moe_forward_impl(shape, 0, nullptr, x, w_router, router_bias, w_mask, mask_bias,
                            w_gate_up, w_down, nullptr, nullptr, out, topk_ids_opt,
                            topk_weights_opt, masked_ids_opt, num_pairs_opt, workspace,
                            workspace_bytes, hip_stream, nullptr);
}

// ---------------------------------------------------------------------------
// beam_moe_forward for callers that cannot allocate: the intermediates live in a
// device array that is part of this library's code object instead of a caller's
// workspace.  In host code the array's name is only a stand-in for the symbol;
// its device address is looked up once per device (hipGetSymbolAddress, with that
// device current) and only that address is ever handed to the kernels.
// ---------------------------------------------------------------------------
static __device__ __align__(256) unsigned char scratch[BEAM_NOALLOC_WORKSPACE_BYTES];

constexpr int kMaxDevices = 64;
static std::atomic<void *> g_scratch_addr[kMaxDevices];

// Device address of `scratch` on the current device, or NULL on a HIP error.
static void *scratch_on_current_device() {
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return nullptr;
    void *p = g_scratch_addr[dev].load(std::memory_order_acquire);
    if (p) return p;
    void *found = nullptr;
    if (hipGetSymbolAddress(&found, HIP_SYMBOL(scratch)) != hipSuccess || !found) return nullptr;
    // every thread that races here gets the same address from the runtime
    g_scratch_addr[dev].store(found, std::memory_order_release);
    return found;
}

beam_status beam_moe_forward_noalloc(const beam_shape *shape, const void *x, const void *w_router,
                                     const float *router_bias, const void *w_mask,
                                     const float *mask_bias, const void *w_gate_up,
                                     const void *w_down, void *out, void *hip_stream) {
    beam_status st = check_shape(shape);
    if (st != BEAM_OK) return st;
    // the size check comes before anything touches the device
    if (ws_layout(*shape).total > (size_t)BEAM_NOALLOC_WORKSPACE_BYTES) return BEAM_ERR_WORKSPACE;
    if (!x || !w_router || !w_mask || !w_gate_up || !w_down || !out) return BEAM_ERR_INVALID_ARG;
    if (shape->T == 0) return BEAM_OK;
    void *ws = scratch_on_current_device();
    if (!ws) return BEAM_ERR_HIP;
    // Nothing in the workspace has to start at zero: every kernel of the layer writes what a
    // later one reads (the one counter of the small-batch path is reset by the logits kernel).
    return moe_forward_impl(shape, 0, nullptr, x, w_router, router_bias, w_mask, mask_bias,
                            w_gate_up, w_down, nullptr, nullptr, out, nullptr, nullptr, nullptr,
                            nullptr, ws, (size_t)BEAM_NOALLOC_WORKSPACE_BYTES, hip_stream, nullptr);
}

beam_status beam_moe_forward_rule(const beam_shape *shape, const beam_rule *rule, const void *x,
                                  const void *w_router, const float *router_bias,
                                  const void *w_mask, const float *mask_bias,
                                  const void *w_gate_up, const void *w_down, void *out,
                                  int32_t *topk_ids_opt, float *topk_weights_opt,
                                  int32_t *masked_ids_opt, int32_t *num_pairs_opt,
                                  void *workspace, size_t workspace_bytes, void *hip_stream) {
    if (!rule) return BEAM_ERR_INVALID_ARG;
    return moe_forward_impl(shape, 0, rule, x, w_router, router_bias, w_mask, mask_bias,
                            w_gate_up, w_down, nullptr, nullptr, out, topk_ids_opt,
                            topk_weights_opt, masked_ids_opt, num_pairs_opt, workspace,
                            workspace_bytes, hip_stream, nullptr);
}

size_t beam_block_workspace_bytes(const beam_shape *shape, int32_t num_shared) {
    if (check_shape(shape) != BEAM_OK || num_shared < 0) return 0;
    beam_shape se = *shape;
    se.N += num_shared;
    se.K += num_shared;
    if (se.N > 256 || se.K > 64 || (long)se.T * se.K >= (1L << 24)) return 0;
    if (se.weight_layout == BEAM_WEIGHTS_PACKED && !tiled_ffn_supported(se)) return 0;
    return ws_layout(se, num_shared).total;
}

beam_status beam_workspace_logits_region(const beam_shape *shape, int32_t num_shared,
                                         size_t *offset_host, size_t *bytes_host,
                                         int32_t *parts_host) {
    if (!offset_host || !bytes_host || !parts_host) return BEAM_ERR_INVALID_ARG;
    if (beam_block_workspace_bytes(shape, num_shared) == 0)
        return check_shape(shape) != BEAM_OK ? check_shape(shape) : BEAM_ERR_UNSUPPORTED;
    beam_shape se = *shape;
    se.N += num_shared;
    se.K += num_shared;
    const WsLayout L = ws_layout(se, num_shared);
    *offset_host = L.router_logits;
    *bytes_host = L.router_logits_bytes;
    *parts_host = L.logit_parts;
    return BEAM_OK;
}

int32_t beam_fused_pair_row_bits(const beam_shape *shape, int32_t num_shared) {
    if (beam_block_workspace_bytes(shape, num_shared) == 0) return 0;
    beam_shape se = *shape;
    se.N += num_shared;
    se.K += num_shared;
    return pair_rows_16bit(se) ? 16 : 32;
}

beam_status beam_moe_block_forward(const beam_shape *shape, int32_t num_shared, const void *x,
                                   const void *w_router, const float *router_bias,
                                   const void *w_mask, const float *mask_bias,
                                   const void *w_gate_up, const void *w_down,
                                   const void *w_shared_gate, const void *residual, void *out,
                                   int32_t *topk_ids_opt, float *topk_weights_opt,
                                   int32_t *masked_ids_opt, int32_t *num_pairs_opt,
                                   void *workspace, size_t workspace_bytes, void *hip_stream) {
    return moe_forward_impl(shape, num_shared, nullptr, x, w_router, router_bias, w_mask,
                            mask_bias, w_gate_up, w_down, w_shared_gate, residual, out, topk_ids_opt,
                            topk_weights_opt, masked_ids_opt, num_pairs_opt, workspace,
                            workspace_bytes, hip_stream, nullptr);
}

beam_status beam_mask_router_backward(const beam_shape *shape, const void *x,
                                      const int32_t *topk_ids, const float *topk_weights,
                                      const float *mask_logits, const float *y_pairs,
                                      const int32_t *expert_offsets, const int32_t *perm,
                                      const int32_t *inv_perm, const void *grad_out,
                                      float reg_coeff, float *grad_a, float *grad_w_mask,
                                      float *loss_reg, void *workspace, size_t workspace_bytes,
                                      void *hip_stream) {
    beam_status st = check_shape(shape);
    if (st != BEAM_OK) return st;
    const beam_shape &s = *shape;
    if (!x || !topk_ids || !topk_weights || !mask_logits || !y_pairs || !expert_offsets || !perm ||
        !inv_perm || !grad_out || !grad_a || !grad_w_mask || !loss_reg)
        return BEAM_ERR_INVALID_ARG;
    if (misaligned(x) || misaligned(y_pairs) || misaligned(grad_out) || misaligned(grad_w_mask))
        return BEAM_ERR_INVALID_ARG;
    if (!(reg_coeff == reg_coeff)) return BEAM_ERR_INVALID_ARG;
    const WsLayout L = ws_layout(s);
    st = check_ws(s, workspace, workspace_bytes, L);
    if (st != BEAM_OK) return st;
    if (s.T == 0) return BEAM_OK;  // nothing selected: grad_w_mask is left untouched
    char *ws = (char *)workspace;
    hipStream_t stream = (hipStream_t)hip_stream;
    const WorkList wl = work_list(ws + L.work, s, L.max_tiles);
    BEAM_TRY_HIP(launch_work_list(s, expert_offsets, wl, stream));
    BEAM_TRY_HIP(launch_mask_router_backward(s, x, topk_ids, topk_weights, mask_logits, y_pairs,
                                             expert_offsets, perm, inv_perm, grad_out, reg_coeff,
                                             wl, L.max_tiles, (float *)(ws + L.tile_partial), grad_a,
                                             grad_w_mask, loss_reg, stream));
    return BEAM_OK;
}

beam_status beam_probe_stream_read(const void *buf, size_t bytes, void *sink, void *hip_stream,
                                   size_t *bytes_read_host) {
    if (!buf || !sink || !bytes_read_host || misaligned(buf) || bytes < (1u << 26))
        return BEAM_ERR_INVALID_ARG;
    const size_t per_block = bytes / 16 / 2048 / 2048 * 2048;  // as the launcher cuts it
    *bytes_read_host = per_block * 16 * 2048;
    BEAM_TRY_HIP(launch_probe_stream_read(buf, bytes, sink, (hipStream_t)hip_stream));
    return BEAM_OK;
}

beam_status beam_probe_mfma(int32_t iters, void *sink, void *hip_stream, double *flops_host) {
    if (iters < 1 || !sink || !flops_host) return BEAM_ERR_INVALID_ARG;
    // 2048 workgroups x 4 wavefronts x 4 MFMAs per iteration x 2*32*32*16 flops
    *flops_host = 2048.0 * 4.0 * 4.0 * (double)iters * 32768.0;
    BEAM_TRY_HIP(launch_probe_mfma(iters, sink, (hipStream_t)hip_stream));
    return BEAM_OK;
}

static beam_status timed_impl(const beam_shape *shape, int32_t num_shared, const void *x,
                              const void *w_router, const float *router_bias, const void *w_mask,
                              const float *mask_bias, const void *w_gate_up, const void *w_down,
                              const void *w_shared_gate, const void *residual, void *out,
                              void *workspace, size_t workspace_bytes, void *hip_stream,
                              float *stage_ms_host) {
    if (!stage_ms_host) return BEAM_ERR_INVALID_ARG;
    hipEvent_t ev[BEAM_NUM_STAGES + 1];
    for (int i = 0; i <= BEAM_NUM_STAGES; ++i) {
        if (hipEventCreate(&ev[i]) != hipSuccess) {
            while (--i >= 0) (void)hipEventDestroy(ev[i]);
            return BEAM_ERR_HIP;
        }
    }
    beam_status st = moe_forward_impl(shape, num_shared, nullptr, x, w_router, router_bias, w_mask,
                                      mask_bias, w_gate_up, w_down, w_shared_gate, residual, out,
                                      nullptr, nullptr, nullptr, nullptr, workspace,
                                      workspace_bytes, hip_stream, ev);
    if (st == BEAM_OK && shape->T > 0) {
        if (hipEventSynchronize(ev[BEAM_NUM_STAGES]) != hipSuccess) st = BEAM_ERR_HIP;
        for (int i = 0; st == BEAM_OK && i < BEAM_NUM_STAGES; ++i)
            if (hipEventElapsedTime(&stage_ms_host[i], ev[i], ev[i + 1]) != hipSuccess)
                st = BEAM_ERR_HIP;
    } else {
        for (int i = 0; i < BEAM_NUM_STAGES; ++i) stage_ms_host[i] = 0.0f;
    }
    for (int i = 0; i <= BEAM_NUM_STAGES; ++i) (void)hipEventDestroy(ev[i]);
    return st;
}

beam_status beam_moe_forward_timed(const beam_shape *shape, const void *x, const void *w_router,
                                   const float *router_bias, const void *w_mask,
                                   const float *mask_bias, const void *w_gate_up,
                                   const void *w_down, void *out, void *workspace,
                                   size_t workspace_bytes, void *hip_stream,
                                   float *stage_ms_host) {
    return timed_impl(shape, 0, x, w_router, router_bias, w_mask, mask_bias, w_gate_up, w_down,
                      nullptr, nullptr, out, workspace, workspace_bytes, hip_stream,
                      stage_ms_host);
}

beam_status beam_moe_block_forward_timed(const beam_shape *shape, int32_t num_shared,
                                         const void *x, const void *w_router,
                                         const float *router_bias, const void *w_mask,
                                         const float *mask_bias, const void *w_gate_up,
                                         const void *w_down, const void *w_shared_gate,
                                         const void *residual, void *out, void *workspace,
                                         size_t workspace_bytes, void *hip_stream,
                                         float *stage_ms_host) {
    return timed_impl(shape, num_shared, x, w_router, router_bias, w_mask, mask_bias, w_gate_up,
                      w_down, w_shared_gate, residual, out, workspace, workspace_bytes,
                      hip_stream, stage_ms_host);
}

}  // extern "C"

// Steps 1-3 of the masked-MoE layer (paper Sec. 3.2): router logits r = x W_r,
// mask pre-activations a = x W_m (Eq. 5), Top-K with softmax over the K
// survivors (Eq. 4) and the binary mask a >= 0 (Eq. 6) written as the -1
// sentinel (App. A.4).
//
// Both heads are one [T,H] x [H,2N] product.  Logits are accumulated in fp32
// and stay fp32: rounding them to bf16 would change the Top-K order.
#include "common.hpp"
#include "topk.hpp"

namespace beam {

// ---------------------------------------------------------------------------
// Logits, any dtype: one wavefront per (token, column), lanes stride over H
// four elements at a time.  Used for fp32 inputs and for shapes the MFMA
// kernel does not take.
// ---------------------------------------------------------------------------
template <typename T>
__global__ __launch_bounds__(256) void logits_generic_kernel(
    const T *__restrict__ x, const T *__restrict__ w_router, const float *__restrict__ b_router,
    const T *__restrict__ w_mask, const float *__restrict__ b_mask,
    float *__restrict__ router_logits, float *__restrict__ mask_logits, int Tn, int H, int N) {
    const int lane = threadIdx.x & 63;
    const int t = blockIdx.x;
    const int c = blockIdx.y * 4 + (threadIdx.x >> 6);
    if (c >= 2 * N) return;
    const bool is_router = c < N;
    const int e = is_router ? c : c - N;
    const T *xr = x + (size_t)t * H;
    const T *wr = (is_router ? w_router : w_mask) + (size_t)e * H;
    float acc = 0.0f;
    for (int h = lane * 4; h < H; h += 256) {
#pragma unroll
        for (int j = 0; j < 4; ++j) acc = fmaf(load_f32(xr + h + j), load_f32(wr + h + j), acc);
    }
    acc = wave_sum(acc);
    if (lane == 0) {
        const float *b = is_router ? b_router : b_mask;
        if (b) acc += b[e];
        (is_router ? router_logits : mask_logits)[(size_t)t * N + e] = acc;
    }
}

// ---------------------------------------------------------------------------
// Logits, bf16 on the matrix cores.  v_mfma_f32_16x16x32_bf16: A = 16 tokens
// x 32 k, B = 32 k x 16 logit columns, D = 16x16 fp32.  Operands go straight
// from global memory into the MFMA registers: lane l owns row/column (l & 15)
// and the 8 reduction indices 8*(l >> 4).. of every 32-wide MFMA step (one
// 16-byte load; the four lanes of a row read 64 contiguous bytes).
//
// A workgroup is WAVES_N x KSPLIT wavefronts: KSPLIT of them share one output
// tile and split the reduction (decode: few tokens, the kernel is one latency
// chain, so the chain is cut short); WAVES_N tile the columns.  MT x NT MFMA
// tiles per wavefront.
// ---------------------------------------------------------------------------
template <int MT, int NT, int WAVES_N, int KSPLIT>
__global__ __launch_bounds__(64 * WAVES_N * KSPLIT) void logits_mfma_kernel(
    const bf16_t *__restrict__ x, const bf16_t *__restrict__ w_router,
    const float *__restrict__ b_router, const bf16_t *__restrict__ w_mask,
    const float *__restrict__ b_mask, float *__restrict__ router_logits,
    float *__restrict__ mask_logits, int Tn, int H, int N, int32_t *__restrict__ zero_word) {
    // a counter a later kernel of the same call accumulates into (NULL: none)
    if (zero_word && blockIdx.x == 0 && blockIdx.y == 0 && threadIdx.x == 0) *zero_word = 0;
    const int lane = threadIdx.x & 63;
    const int wave = threadIdx.x >> 6;
    const int wn = wave % WAVES_N;
    const int ks = wave / WAVES_N;
    const int l16 = lane & 15;
    const int g = lane >> 4;
    const int t0 = blockIdx.x * (MT * 16);
    const int c0 = blockIdx.y * (WAVES_N * NT * 16) + wn * (NT * 16);
    const int klen = H / KSPLIT;
    const int kbeg = ks * klen + g * 8;

    const bf16_t *arow[MT];
    const bf16_t *brow[NT];
#pragma unroll
    for (int m = 0; m < MT; ++m) {
        int t = t0 + m * 16 + l16;
        t = t < Tn ? t : Tn - 1;
        arow[m] = x + (size_t)t * H + kbeg;
    }
#pragma unroll
    for (int n = 0; n < NT; ++n) {
        int c = c0 + n * 16 + l16;
        c = c < 2 * N ? c : 2 * N - 1;
        brow[n] = (c < N ? w_router + (size_t)c * H : w_mask + (size_t)(c - N) * H) + kbeg;
    }

    f32x4 acc[MT][NT];
#pragma unroll
    for (int m = 0; m < MT; ++m)
#pragma unroll
        for (int n = 0; n < NT; ++n) acc[m][n] = f32x4{0.f, 0.f, 0.f, 0.f};

    for (int k = 0; k < klen; k += 128) {
        uint4 a[MT][4], b[NT][4];
#pragma unroll
        for (int m = 0; m < MT; ++m)
#pragma unroll
            for (int j = 0; j < 4; ++j) a[m][j] = *(const uint4 *)(arow[m] + k + j * 32);
#pragma unroll
        for (int n = 0; n < NT; ++n)
#pragma unroll
            for (int j = 0; j < 4; ++j) b[n][j] = *(const uint4 *)(brow[n] + k + j * 32);
#pragma unroll
        for (int j = 0; j < 4; ++j)
#pragma unroll
            for (int m = 0; m < MT; ++m)
#pragma unroll
                for (int n = 0; n < NT; ++n)
                    acc[m][n] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(
                        __builtin_bit_cast(bf16x8, a[m][j]), __builtin_bit_cast(bf16x8, b[n][j]),
                        acc[m][n], 0, 0, 0);
    }

    if constexpr (KSPLIT > 1) {
        __shared__ float red[KSPLIT - 1][WAVES_N][MT * NT * 4][64];
        if (ks > 0) {
#pragma unroll
            for (int m = 0; m < MT; ++m)
#pragma unroll
                for (int n = 0; n < NT; ++n)
#pragma unroll
                    for (int r = 0; r < 4; ++r)
                        red[ks - 1][wn][(m * NT + n) * 4 + r][lane] = acc[m][n][r];
        }
        __syncthreads();
        if (ks > 0) return;
#pragma unroll
        for (int s = 0; s < KSPLIT - 1; ++s)
#pragma unroll
            for (int m = 0; m < MT; ++m)
#pragma unroll
                for (int n = 0; n < NT; ++n)
#pragma unroll
                    for (int r = 0; r < 4; ++r)
                        acc[m][n][r] += red[s][wn][(m * NT + n) * 4 + r][lane];
    }

    // D layout: lane l, register r -> token row 4*(l>>4)+r, column l&15.
#pragma unroll
    for (int n = 0; n < NT; ++n) {
        const int c = c0 + n * 16 + l16;
        if (c >= 2 * N) continue;
        const bool is_router = c < N;
        const int e = is_router ? c : c - N;
        const float *bp = is_router ? b_router : b_mask;
        const float bias = bp ? bp[e] : 0.0f;
        float *dst = is_router ? router_logits : mask_logits;
#pragma unroll
        for (int m = 0; m < MT; ++m)
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                const int t = t0 + m * 16 + g * 4 + r;
                if (t < Tn) dst[(size_t)t * N + e] = acc[m][n][r] + bias;
            }
    }
}

hipError_t launch_logits(const beam_shape &s, const void *x, const void *w_router,
                         const float *b_router, const void *w_mask, const float *b_mask,
                         float *router_logits, float *mask_logits, hipStream_t st,
                         int32_t *zero_word) {
    const int T = s.T, H = s.H, N = s.N;
    if (s.dtype == BEAM_BF16 && H % 128 == 0) {
        const bf16_t *xb = (const bf16_t *)x;
        const bf16_t *wr = (const bf16_t *)w_router;
        const bf16_t *wm = (const bf16_t *)w_mask;
        if (T <= 512 && H % 2048 == 0) {
            dim3 grid((T + 15) / 16, (2 * N + 15) / 16);
            logits_mfma_kernel<1, 1, 1, 16><<<grid, 1024, 0, st>>>(
                xb, wr, b_router, wm, b_mask, router_logits, mask_logits, T, H, N, zero_word);
        } else if (T <= 512 && H % 512 == 0) {
            dim3 grid((T + 15) / 16, (2 * N + 15) / 16);
            logits_mfma_kernel<1, 1, 1, 4><<<grid, 256, 0, st>>>(
                xb, wr, b_router, wm, b_mask, router_logits, mask_logits, T, H, N, zero_word);
        } else {
            dim3 grid((T + 31) / 32, (2 * N + 255) / 256);
            logits_mfma_kernel<2, 4, 4, 1><<<grid, 256, 0, st>>>(
                xb, wr, b_router, wm, b_mask, router_logits, mask_logits, T, H, N, zero_word);
        }
    } else {
        dim3 grid(T, (2 * N + 3) / 4);
        if (s.dtype == BEAM_BF16)
            logits_generic_kernel<bf16_t><<<grid, 256, 0, st>>>(
                (const bf16_t *)x, (const bf16_t *)w_router, b_router, (const bf16_t *)w_mask,
                b_mask, router_logits, mask_logits, T, H, N);
        else
            logits_generic_kernel<float><<<grid, 256, 0, st>>>(
                (const float *)x, (const float *)w_router, b_router, (const float *)w_mask, b_mask,
                router_logits, mask_logits, T, H, N);
    }
    return hipGetLastError();
}

// ---------------------------------------------------------------------------
// [T,2N] logits without biases (what the tiled GEMM writes) -> the two [T,N]
// arrays with biases that callers of the staged entry point may ask for.
// ---------------------------------------------------------------------------
__global__ __launch_bounds__(256) void split_logits_kernel(
    const float *__restrict__ logits2, const float *__restrict__ b_router,
    const float *__restrict__ b_mask, float *__restrict__ router_logits,
    float *__restrict__ mask_logits, int Tn, int N, LogitParts parts) {
    const size_t total = (size_t)Tn * 2 * N;
    for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < total; i += (size_t)gridDim.x * 256) {
        const int c = (int)(i % (2 * N));
        const size_t t = i / (2 * N);
        const float v = sum_parts(logits2 + i, parts);
        if (c < N) {
            if (router_logits) router_logits[t * N + c] = b_router ? v + b_router[c] : v;
        } else {
            if (mask_logits) mask_logits[t * N + c - N] = b_mask ? v + b_mask[c - N] : v;
        }
    }
}

hipError_t launch_split_logits(const beam_shape &s, const float *logits2, const float *b_router,
                               const float *b_mask, float *router_logits, float *mask_logits,
                               hipStream_t st, int n_parts) {
    LogitParts parts;
    parts.n = n_parts;
    parts.stride = (size_t)s.T * 2 * s.N;
    const size_t total = (size_t)s.T * 2 * s.N;
    const int grid = (int)((total + 255) / 256 < 2048 ? (total + 255) / 256 : 2048);
    split_logits_kernel<<<grid, 256, 0, st>>>(logits2, b_router, b_mask, router_logits,
                                              mask_logits, s.T, s.N, parts);
    return hipGetLastError();
}

// ---------------------------------------------------------------------------
// Weight of the shared expert (App. A.3): g_sh[t] = sigma(x_t . w), one
// wavefront per token, fp32.
// ---------------------------------------------------------------------------
template <typename T>
__global__ __launch_bounds__(256) void shared_gate_kernel(const T *__restrict__ x,
                                                          const T *__restrict__ w,
                                                          float *__restrict__ g_shared, int Tn,
                                                          int H) {
    const int lane = threadIdx.x & 63;
    const int t = blockIdx.x * 4 + (threadIdx.x >> 6);
    if (t >= Tn) return;  // wave-uniform
    const T *xr = x + (size_t)t * H;
    float acc = 0.0f;
    for (int h = lane * 4; h < H; h += 256) {
#pragma unroll
        for (int j = 0; j < 4; ++j) acc = fmaf(load_f32(xr + h + j), load_f32(w + h + j), acc);
    }
    acc = wave_sum(acc);
    if (lane == 0) g_shared[t] = 1.0f / (1.0f + expf(-acc));
}

hipError_t launch_shared_gate(const beam_shape &s, const void *x, const void *w_shared_gate,
                              float *g_shared, hipStream_t st) {
    dim3 grid((s.T + 3) / 4);
    if (s.dtype == BEAM_BF16)
        shared_gate_kernel<bf16_t><<<grid, 256, 0, st>>>((const bf16_t *)x,
                                                         (const bf16_t *)w_shared_gate, g_shared,
                                                         s.T, s.H);
    else
        shared_gate_kernel<float><<<grid, 256, 0, st>>>((const float *)x,
                                                        (const float *)w_shared_gate, g_shared,
                                                        s.T, s.H);
    return hipGetLastError();
}

// ---------------------------------------------------------------------------
// Top-K, softmax over the K survivors, binary mask: one wavefront per token.
// S > 0 appends the shared-expert slots: output rows have K + S entries and
// g_shared (NULL = 1) holds the per-token weight of those slots.
// ---------------------------------------------------------------------------
template <int RULE>
__global__ __launch_bounds__(256) void topk_mask_kernel(
    const float *__restrict__ router_logits, const float *__restrict__ mask_logits,
    const float *__restrict__ b_router, const float *__restrict__ b_mask, int row_stride,
    const float *__restrict__ g_shared, float param, int32_t *__restrict__ topk_ids,
    float *__restrict__ topk_w, int32_t *__restrict__ masked_ids, int Tn, int N, int K, int S, LogitParts parts) {
    const int t = blockIdx.x * 4 + (threadIdx.x >> 6);
    if (t >= Tn) return;  // wave-uniform
    const size_t f = (size_t)t * (K + S);
    const float gs = (S > 0 && g_shared) ? g_shared[t] : 1.0f;
    wave_route_token<RULE>(router_logits + (size_t)t * row_stride,
                           mask_logits + (size_t)t * row_stride, b_router, b_mask, N, K, S, gs,
                           param, topk_ids + f, topk_w + f, masked_ids + f, parts);
}

// Large batches: four tokens per wavefront (one per 16-lane row), 16 per workgroup.
template <int NPL, int RULE>
__global__ __launch_bounds__(256) void topk_mask_rows_kernel(
    const float *__restrict__ router_logits, const float *__restrict__ mask_logits,
    const float *__restrict__ b_router, const float *__restrict__ b_mask, int row_stride,
    const float *__restrict__ g_shared, float param, int32_t *__restrict__ topk_ids,
    float *__restrict__ topk_w, int32_t *__restrict__ masked_ids, int Tn, int N, int K, int S, LogitParts parts) {
    const int t = blockIdx.x * 16 + (threadIdx.x >> 4);
    const bool valid = t < Tn;
    const int tc = valid ? t : Tn - 1;
    const size_t f = (size_t)tc * (K + S);
    const float gs = (S > 0 && g_shared) ? g_shared[tc] : 1.0f;
    row_route_token<NPL, RULE>(router_logits + (size_t)tc * row_stride,
                               mask_logits + (size_t)tc * row_stride, b_router, b_mask, N, K, S,
                               gs, param, valid, topk_ids + f, topk_w + f, masked_ids + f, parts);
}

// Logits live as two [T,N] arrays that already include the biases, or (row_stride
// = 2N, biases still to add) as one [T,2N] array: router columns, then mask columns.
// s.N and s.K count the routed experts; opt.S shared-expert slots are appended.
template <int RULE>
static hipError_t launch_topk_rule(const beam_shape &s, const float *router_logits,
                                   const float *mask_logits, const float *b_router,
                                   const float *b_mask, int row_stride, const RouteOpts &opt,
                                   int32_t *topk_ids, float *topk_w, int32_t *masked_ids,
                                   hipStream_t st, LogitParts parts) {
    // The row variant does four tokens per wavefront at about the cost of one; the
    // wave variant has the shorter latency chain for decode-sized batches.
    const bool aligned = ((uintptr_t)router_logits | (uintptr_t)mask_logits |
                          (uintptr_t)b_router | (uintptr_t)b_mask) % 16 == 0;
    const int S = opt.S;
#define BEAM_TOPK_ARGS                                                                          \
    router_logits, mask_logits, b_router, b_mask, row_stride, opt.g_shared, opt.param,          \
        topk_ids, topk_w, masked_ids, s.T, s.N, s.K, S, parts
    if (s.T >= 512 && s.K + S <= 16 && s.N % 4 == 0 && row_stride % 4 == 0 && s.N <= 256 &&
        aligned) {
        dim3 grid((s.T + 15) / 16);
        if (s.N <= 64) topk_mask_rows_kernel<4, RULE><<<grid, 256, 0, st>>>(BEAM_TOPK_ARGS);
        else if (s.N <= 128) topk_mask_rows_kernel<8, RULE><<<grid, 256, 0, st>>>(BEAM_TOPK_ARGS);
        else topk_mask_rows_kernel<16, RULE><<<grid, 256, 0, st>>>(BEAM_TOPK_ARGS);
        return hipGetLastError();
    }
    dim3 grid((s.T + 3) / 4);
    topk_mask_kernel<RULE><<<grid, 256, 0, st>>>(BEAM_TOPK_ARGS);
#undef BEAM_TOPK_ARGS
    return hipGetLastError();
}

hipError_t launch_topk_mask(const beam_shape &s, const float *router_logits,
                            const float *mask_logits, const float *b_router, const float *b_mask,
                            int row_stride, const RouteOpts &opt, int32_t *topk_ids,
                            float *topk_w, int32_t *masked_ids, hipStream_t st, int n_parts) {
    LogitParts parts;   // parts of a [T, row_stride] array each
    parts.n = n_parts;
    parts.stride = (size_t)s.T * row_stride;
    if (opt.rule == kRuleCumProb)
        return launch_topk_rule<kRuleCumProb>(s, router_logits, mask_logits, b_router, b_mask,
                                              row_stride, opt, topk_ids, topk_w, masked_ids, st,
                                              parts);
    return launch_topk_rule<kRuleMask>(s, router_logits, mask_logits, b_router, b_mask,
                                       row_stride, opt, topk_ids, topk_w, masked_ids, st, parts);
}

}  // namespace beam

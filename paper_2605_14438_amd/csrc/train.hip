// Training-mode backward of the mask router (paper Sec. 3.3): the straight-through
// estimator of Eq. 9 passes dL/dm to the raw mask m^ = sigma(a), which gives
// Eq. 12 for the gradient with respect to the pre-activation a = x W_m,
//   grad_a[t,k] = (dL/dg^_k * g_k + c / K) * sigma'(a_k),   k over the Top-K set,
// with dL/dg^_k = <dL/dy[t,:], E_k(x_t)> because y = sum_k g^_k E_k(x_t) is linear
// in g^, and c the coefficient of L_reg (Eq. 10, 11).  In training every Top-K
// expert is evaluated whatever the mask says (Sec. 3.3.1), so E_k(x_t) is a row
// of y_pairs for EVERY slot: the grouping here is that of topk_ids, not of
// masked_ids.  Then grad_W_m[e,:] = sum over the pairs of expert e of
// grad_a * x_t, a segmented sum over the expert-sorted rows: partial sums per
// 128-row tile of the work list, then one ordered pass per expert, so the result
// does not depend on scheduling (no floating-point atomics).
#include "common.hpp"

namespace beam {

__device__ __forceinline__ float4 ld4(const float *p) { return *(const float4 *)p; }
typedef float f32x4t __attribute__((ext_vector_type(4)));
__device__ __forceinline__ float4 ld4_stream(const float *p) {
    const f32x4t v = __builtin_nontemporal_load((const f32x4t *)p);
    return make_float4(v.x, v.y, v.z, v.w);
}
__device__ __forceinline__ float4 ld4(const bf16_t *p) {
    const uint2 q = *(const uint2 *)p;
    return make_float4(__uint_as_float(q.x << 16), __uint_as_float(q.x & 0xffff0000u),
                       __uint_as_float(q.y << 16), __uint_as_float(q.y & 0xffff0000u));
}

// One workgroup per token; its wavefronts take the K slots round-robin.
// H % 4 == 0 (the envelope has H % 8 == 0).
template <typename T>
__global__ __launch_bounds__(256) void mask_grad_pairs_kernel(
    const int32_t *__restrict__ topk_ids, const float *__restrict__ topk_w,
    const float *__restrict__ mask_logits, const float *__restrict__ y_pairs,
    const int32_t *__restrict__ inv_perm, const T *__restrict__ grad_out, float reg_over_k,
    float *__restrict__ grad_a, float *__restrict__ loss_reg, int H, int N, int K) {
    __shared__ float sig_s[64];
    const int t = blockIdx.x;
    const int lane = threadIdx.x & 63;
    const int wave = threadIdx.x >> 6;
    const T *dy = grad_out + (size_t)t * H;
    for (int k = wave; k < K; k += 4) {
        const size_t f = (size_t)t * K + k;
        const int row = inv_perm[f];
        float dot = 0.0f;
        if (row >= 0) {  // wave-uniform
            const float *y = y_pairs + (size_t)row * H;
            for (int h = lane * 4; h < H; h += 256) {
                const float4 a = ld4(dy + h);
                const float4 b = ld4_stream(y + h);   // read once, larger than the caches
                dot = fmaf(a.x, b.x, dot);
                dot = fmaf(a.y, b.y, dot);
                dot = fmaf(a.z, b.z, dot);
                dot = fmaf(a.w, b.w, dot);
            }
        }
        dot = wave_sum(dot);
        if (lane == 0) {
            const float a = mask_logits[(size_t)t * N + topk_ids[f]];
            const float sig = 1.0f / (1.0f + expf(-a));
            grad_a[f] = (dot * topk_w[f] + reg_over_k) * sig * (1.0f - sig);
            sig_s[k] = sig;
        }
    }
    __syncthreads();
    if (threadIdx.x == 0) {
        float s = 0.0f;
        for (int k = 0; k < K; ++k) s += sig_s[k];  // slot order: reproducible
        loss_reg[t] = s / (float)K;                 // Eq. 10
    }
}

// grid (tiles, ceil(H / 256)), one wavefront per workgroup: partial[tile, c] =
// sum over the tile's grouped rows, in row order, of grad_a[f] * x[t_f, c].
// Eight independent row loads are issued before the first add: the kernel is a
// gather and lives on memory-level parallelism.
template <typename T>
__global__ __launch_bounds__(64) void mask_grad_w_partial_kernel(
    const T *__restrict__ x, const float *__restrict__ grad_a, const int32_t *__restrict__ perm,
    const int32_t *__restrict__ offsets, WorkList wl, float *__restrict__ partial, int H, int K) {
    const int tile = blockIdx.x;
    if (tile >= wl.hdr[1]) return;
    const int c = (blockIdx.y * 64 + threadIdx.x) * 4;
    if (c >= H) return;
    const int e = wl.tile_expert[tile];
    const int row0 = wl.tile_row0[tile];
    const int row_end = min(row0 + kTileM, offsets[e + 1]);
    float4 acc = make_float4(0.f, 0.f, 0.f, 0.f);
    for (int r = row0; r < row_end; r += 8) {
        float4 xv[8];
        float ga[8];
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            const bool in = r + i < row_end;
            const int f = perm[in ? r + i : r];
            ga[i] = in ? grad_a[f] : 0.0f;
            xv[i] = ld4(x + (size_t)(f / K) * H + c);
        }
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            const bool in = r + i < row_end;
            acc.x = in ? fmaf(ga[i], xv[i].x, acc.x) : acc.x;
            acc.y = in ? fmaf(ga[i], xv[i].y, acc.y) : acc.y;
            acc.z = in ? fmaf(ga[i], xv[i].z, acc.z) : acc.z;
            acc.w = in ? fmaf(ga[i], xv[i].w, acc.w) : acc.w;
        }
    }
    *(float4 *)(partial + (size_t)tile * H + c) = acc;
}

// grid (N, ceil(H / 256)), one wavefront per workgroup: grad_w_mask[e, c] = sum
// over expert e's tiles, in tile order (loads batched by eight, adds in order);
// zero for an expert no token selected (Theorem 1: no gradient).
__global__ __launch_bounds__(64) void mask_grad_w_reduce_kernel(
    const float *__restrict__ partial, const int32_t *__restrict__ offsets,
    float *__restrict__ grad_w_mask, int H, int N) {
    const int e = blockIdx.x;
    // tiles of the experts before e: integer sum over the wavefront
    int mine = 0;
    for (int q = threadIdx.x; q < e; q += 64) mine += tiles_of(offsets[q + 1] - offsets[q]);
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) mine += __shfl_xor(mine, off);
    const int first_tile = mine;
    const int c = (blockIdx.y * 64 + threadIdx.x) * 4;
    if (c >= H) return;
    const int nt = tiles_of(offsets[e + 1] - offsets[e]);
    float4 acc = make_float4(0.f, 0.f, 0.f, 0.f);
    for (int i = 0; i < nt; i += 8) {
        float4 p[8];
#pragma unroll
        for (int j = 0; j < 8; ++j)
            p[j] = *(const float4 *)(partial + (size_t)(first_tile + (i + j < nt ? i + j : i)) * H + c);
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            const bool in = i + j < nt;
            acc.x += in ? p[j].x : 0.0f;
            acc.y += in ? p[j].y : 0.0f;
            acc.z += in ? p[j].z : 0.0f;
            acc.w += in ? p[j].w : 0.0f;
        }
    }
    *(float4 *)(grad_w_mask + (size_t)e * H + c) = acc;
}

hipError_t launch_mask_router_backward(const beam_shape &s, const void *x,
                                       const int32_t *topk_ids, const float *topk_w,
                                       const float *mask_logits, const float *y_pairs,
                                       const int32_t *offsets, const int32_t *perm,
                                       const int32_t *inv_perm, const void *grad_out,
                                       float reg_coeff, const WorkList &wl, int max_tiles,
                                       float *partial, float *grad_a, float *grad_w_mask,
                                       float *loss_reg, hipStream_t st) {
    const float rk = reg_coeff / (float)s.K;
    const dim3 gp(max_tiles, (s.H + 255) / 256);
    const dim3 gr(s.N, (s.H + 255) / 256);
    if (s.dtype == BEAM_BF16) {
        mask_grad_pairs_kernel<bf16_t><<<s.T, 256, 0, st>>>(
            topk_ids, topk_w, mask_logits, y_pairs, inv_perm, (const bf16_t *)grad_out, rk, grad_a,
            loss_reg, s.H, s.N, s.K);
        BEAM_CHECK_LAUNCH();
        mask_grad_w_partial_kernel<bf16_t><<<gp, 64, 0, st>>>((const bf16_t *)x, grad_a, perm,
                                                               offsets, wl, partial, s.H, s.K);
    } else {
        mask_grad_pairs_kernel<float><<<s.T, 256, 0, st>>>(
            topk_ids, topk_w, mask_logits, y_pairs, inv_perm, (const float *)grad_out, rk, grad_a,
            loss_reg, s.H, s.N, s.K);
        BEAM_CHECK_LAUNCH();
        mask_grad_w_partial_kernel<float><<<gp, 64, 0, st>>>((const float *)x, grad_a, perm,
                                                              offsets, wl, partial, s.H, s.K);
    }
    BEAM_CHECK_LAUNCH();
    mask_grad_w_reduce_kernel<<<gr, 64, 0, st>>>(partial, offsets, grad_w_mask, s.H, s.N);
    return hipGetLastError();
}

}  // namespace beam

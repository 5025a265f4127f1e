// Masked aggregation (paper Eq. 7-8): out[t] = sum_k m_k g_k E_{id_k}(x_t) over
// the kept slots of token t, in slot order, fp32 accumulate, one rounding.  A
// gather over the expert-sorted rows: every output element is written exactly
// once with coalesced 16-byte accesses and no atomics, and a token with no
// kept expert gets an exactly +0 row (App. A.3).
#include "common.hpp"

namespace beam {

template <typename T>
__global__ __launch_bounds__(256) void combine_kernel(
    const float *__restrict__ y_pairs, const float *__restrict__ topk_w,
    const int32_t *__restrict__ masked_ids, const int32_t *__restrict__ inv_perm,
    T *__restrict__ out, int Tn, int H, int K) {
    const int t = blockIdx.x;
    const int32_t *ids = masked_ids + (size_t)t * K;
    const int32_t *inv = inv_perm + (size_t)t * K;
    const float *w = topk_w + (size_t)t * K;
    for (int c = threadIdx.x * 4; c < H; c += 1024) {
        float4 acc = make_float4(0.f, 0.f, 0.f, 0.f);
        for (int k = 0; k < K; ++k) {
            const int row = inv[k];
            if (ids[k] < 0 || row < 0) continue;
            const float g = w[k];
            const float4 y = *(const float4 *)(y_pairs + (size_t)row * H + c);
            acc.x = fmaf(g, y.x, acc.x);
            acc.y = fmaf(g, y.y, acc.y);
            acc.z = fmaf(g, y.z, acc.z);
            acc.w = fmaf(g, y.w, acc.w);
        }
        T *o = out + (size_t)t * H + c;
        store_from_f32(o + 0, acc.x);
        store_from_f32(o + 1, acc.y);
        store_from_f32(o + 2, acc.z);
        store_from_f32(o + 3, acc.w);
    }
}

hipError_t launch_combine(const beam_shape &s, const float *y_pairs, const float *topk_w,
                          const int32_t *masked_ids, const int32_t *inv_perm, void *out,
                          hipStream_t st) {
    dim3 grid(s.T);
    if (s.dtype == BEAM_BF16)
        combine_kernel<bf16_t><<<grid, 256, 0, st>>>(y_pairs, topk_w, masked_ids, inv_perm,
                                                     (bf16_t *)out, s.T, s.H, s.K);
    else
        combine_kernel<float><<<grid, 256, 0, st>>>(y_pairs, topk_w, masked_ids, inv_perm,
                                                    (float *)out, s.T, s.H, s.K);
    return hipGetLastError();
}

}  // namespace beam

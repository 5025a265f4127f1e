// Masked aggregation (paper Eq. 7-8): out[t] = sum_k m_k g_k E_{id_k}(x_t) over
// the kept slots of token t, in slot order, fp32 accumulate, one rounding.  With
// a residual h (App. A.3) the sum starts from h[t] instead of zero.  A
// gather over the expert-sorted rows: every output element is written exactly
// once with coalesced accesses and no atomics, and a token with no kept expert
// gets an exactly +0 row (App. A.3).
#include <type_traits>

#include "common.hpp"

namespace beam {

__device__ __forceinline__ void store4(float *p, float4 v) { *(float4 *)p = v; }
__device__ __forceinline__ void store4(bf16_t *p, float4 v) {
    uint2 q;
    q.x = (uint32_t)f32_to_bf16(v.x) | ((uint32_t)f32_to_bf16(v.y) << 16);
    q.y = (uint32_t)f32_to_bf16(v.z) | ((uint32_t)f32_to_bf16(v.w) << 16);
    *(uint2 *)p = q;
}

__device__ __forceinline__ float4 load4(const float *p) { return *(const float4 *)p; }
typedef float f32x4n __attribute__((ext_vector_type(4)));
template <bool STREAM>
__device__ __forceinline__ float4 load_y4(const float *p) {
    if constexpr (STREAM) {
        const f32x4n v = __builtin_nontemporal_load((const f32x4n *)p);
        return make_float4(v.x, v.y, v.z, v.w);
    } else {
        return *(const float4 *)p;
    }
}
// half-precision pair rows (the fused layer's large batches): four values in eight bytes
typedef uint32_t u32x2n __attribute__((ext_vector_type(2)));
__device__ __forceinline__ float half_bits_to_float(uint32_t bits) {
    return (float)__builtin_bit_cast(_Float16, (unsigned short)bits);
}
template <bool STREAM>
__device__ __forceinline__ float4 load_y4(const _Float16 *p) {
    uint32_t lo, hi;
    if constexpr (STREAM) {
        const u32x2n q = __builtin_nontemporal_load((const u32x2n *)p);
        lo = q.x;
        hi = q.y;
    } else {
        const uint2 q = *(const uint2 *)p;
        lo = q.x;
        hi = q.y;
    }
    return make_float4(half_bits_to_float(lo & 0xffffu), half_bits_to_float(lo >> 16),
                       half_bits_to_float(hi & 0xffffu), half_bits_to_float(hi >> 16));
}
__device__ __forceinline__ float4 load4(const bf16_t *p) {
    const uint2 q = *(const uint2 *)p;
    return make_float4(__uint_as_float(q.x << 16), __uint_as_float(q.x & 0xffff0000u),
                       __uint_as_float(q.y << 16), __uint_as_float(q.y & 0xffff0000u));
}

__device__ __forceinline__ void axpy4(float g, const float4 &y, float4 &acc) {
    acc.x = fmaf(g, y.x, acc.x);
    acc.y = fmaf(g, y.y, acc.y);
    acc.z = fmaf(g, y.z, acc.z);
    acc.w = fmaf(g, y.w, acc.w);
}

// One wavefront per token, H % (256 * CH) == 0.  Lane k < K looks up slot k; a
// ballot gives the kept slots as a wave-uniform bit set that is walked in slot
// order, two slots at a time, each slot's row and weight broadcast from its
// lane.  A lane owns CH groups of four columns, 256 apart, so one slot is CH
// independent 16-byte loads per lane and a wavefront keeps up to 2 * CH KiB in
// flight: the kernel is a pure gather and lives on memory-level parallelism.
// Dropped slots cost nothing.
template <typename T, int CH, typename Y>
__global__ __launch_bounds__(256) void combine_wave_kernel(
    const Y *__restrict__ y_pairs, const float *__restrict__ topk_w,
    const int32_t *__restrict__ masked_ids, const int32_t *__restrict__ inv_perm,
    const T *__restrict__ residual, T *__restrict__ out, int Tn, int H, int K,
    const int32_t *__restrict__ num_pairs, int k_split, size_t slice_stride) {
    const int lane = threadIdx.x & 63;
    const int t = blockIdx.x * (blockDim.x >> 6) + (threadIdx.x >> 6);
    if (t >= Tn) return;  // wave-uniform
    int row = -1;
    float g = 0.0f;
    if (lane < K) {
        const size_t f = (size_t)t * K + lane;
        row = masked_ids[f] >= 0 ? inv_perm[f] : -1;
        g = topk_w[f];
    }
    const uint64_t kept = __ballot(row >= 0);
    auto sum_slots = [&](auto stream) {
        constexpr bool STREAM = decltype(stream)::value;
        for (int c0 = lane * 4; c0 < H; c0 += 256 * CH) {
            float4 acc[CH];
#pragma unroll
            for (int i = 0; i < CH; ++i)
                acc[i] = residual ? load4(residual + (size_t)t * H + c0 + i * 256)
                                  : make_float4(0.f, 0.f, 0.f, 0.f);
            for (int sl = 0; sl < k_split; ++sl) {   // parts of a split down projection, in order
            const Y *ys = y_pairs + sl * slice_stride;
            uint64_t m = kept;
            while (m) {
                const int ka = __builtin_ctzll(m);
                m &= m - 1;
                const Y *pa = ys + (size_t)__shfl(row, ka) * H + c0;
                const float ga = __shfl(g, ka);
                if (m) {
                    const int kb = __builtin_ctzll(m);
                    m &= m - 1;
                    const Y *pb = ys + (size_t)__shfl(row, kb) * H + c0;
                    const float gb = __shfl(g, kb);
                    float4 ya[CH], yb[CH];
#pragma unroll
                    for (int i = 0; i < CH; ++i) ya[i] = load_y4<STREAM>(pa + i * 256);
#pragma unroll
                    for (int i = 0; i < CH; ++i) yb[i] = load_y4<STREAM>(pb + i * 256);
#pragma unroll
                    for (int i = 0; i < CH; ++i) {
                        axpy4(ga, ya[i], acc[i]);
                        axpy4(gb, yb[i], acc[i]);
                    }
                } else {
                    float4 ya[CH];
#pragma unroll
                    for (int i = 0; i < CH; ++i) ya[i] = load_y4<STREAM>(pa + i * 256);
#pragma unroll
                    for (int i = 0; i < CH; ++i) axpy4(ga, ya[i], acc[i]);
                }
            }
            }
#pragma unroll
            for (int i = 0; i < CH; ++i) store4(out + (size_t)t * H + c0 + i * 256, acc[i]);
        }
    };
    // y_pairs too large to have stayed in cache since the down projection wrote it:
    // read it past the caches (same values, same order of additions)
    if (num_pairs && (size_t)*num_pairs * H * sizeof(Y) > kStreamBytes)
        sum_slots(std::true_type{});
    else
        sum_slots(std::false_type{});
}

// Any H % 4 == 0: one workgroup per token, a slot at a time.
template <typename T>
__global__ __launch_bounds__(256) void combine_generic_kernel(
    const float *__restrict__ y_pairs, const float *__restrict__ topk_w,
    const int32_t *__restrict__ masked_ids, const int32_t *__restrict__ inv_perm,
    const T *__restrict__ residual, T *__restrict__ out, int Tn, int H, int K) {
    const int t = blockIdx.x;
    const int32_t *ids = masked_ids + (size_t)t * K;
    const int32_t *inv = inv_perm + (size_t)t * K;
    const float *w = topk_w + (size_t)t * K;
    for (int c = threadIdx.x * 4; c < H; c += 1024) {
        float4 acc = residual ? load4(residual + (size_t)t * H + c)
                              : make_float4(0.f, 0.f, 0.f, 0.f);
        for (int k = 0; k < K; ++k) {
            const int row = inv[k];
            if (ids[k] < 0 || row < 0) continue;
            axpy4(w[k], *(const float4 *)(y_pairs + (size_t)row * H + c), acc);
        }
        store4(out + (size_t)t * H + c, acc);
    }
}

template <typename T>
static void launch_typed(const beam_shape &s, const float *y_pairs, const float *topk_w,
                         const int32_t *masked_ids, const int32_t *inv_perm, const T *residual,
                         T *out, hipStream_t st, const int32_t *num_pairs, int k_split,
                         bool y16) {
    // decode-sized batches: one wavefront per workgroup, to spread over the CUs
    const int wpb = s.T <= 1024 ? 1 : 4;
    const dim3 wave_grid((s.T + wpb - 1) / wpb);
#define BEAM_COMBINE_WAVE(CH)                                                                   \
    if (y16)                                                                                    \
        combine_wave_kernel<T, CH, _Float16><<<wave_grid, 64 * wpb, 0, st>>>(                   \
            (const _Float16 *)y_pairs, topk_w, masked_ids, inv_perm, residual, out, s.T, s.H,  \
            s.K, num_pairs, k_split, (size_t)s.T * s.K * s.H);                                 \
    else                                                                                        \
        combine_wave_kernel<T, CH, float><<<wave_grid, 64 * wpb, 0, st>>>(                      \
            y_pairs, topk_w, masked_ids, inv_perm, residual, out, s.T, s.H, s.K, num_pairs,   \
            k_split, (size_t)s.T * s.K * s.H)
    if (s.H % 2048 == 0) { BEAM_COMBINE_WAVE(8); }
    else if (s.H % 1280 == 0) { BEAM_COMBINE_WAVE(5); }
    else if (s.H % 1024 == 0) { BEAM_COMBINE_WAVE(4); }
    else if (s.H % 512 == 0) { BEAM_COMBINE_WAVE(2); }
    else if (s.H % 256 == 0) { BEAM_COMBINE_WAVE(1); }
    else
        combine_generic_kernel<T><<<dim3(s.T), 256, 0, st>>>(y_pairs, topk_w, masked_ids,
                                                             inv_perm, residual, out, s.T, s.H,
                                                             s.K);
#undef BEAM_COMBINE_WAVE
}

// y16: y_pairs holds half-precision rows (the tiled down GEMM wrote them so); H % 256 == 0
// and k_split == 1 then.
hipError_t launch_combine(const beam_shape &s, const float *y_pairs, const float *topk_w,
                          const int32_t *masked_ids, const int32_t *inv_perm,
                          const void *residual, void *out, hipStream_t st,
                          const int32_t *num_pairs, int k_split, bool y16) {
    if (y16 && (s.H % 256 != 0 || k_split != 1)) return hipErrorInvalidValue;
    if (s.dtype == BEAM_BF16)
        launch_typed<bf16_t>(s, y_pairs, topk_w, masked_ids, inv_perm, (const bf16_t *)residual,
                             (bf16_t *)out, st, num_pairs, k_split, y16);
    else
        launch_typed<float>(s, y_pairs, topk_w, masked_ids, inv_perm, (const float *)residual,
                            (float *)out, st, num_pairs, k_split, y16);
    return hipGetLastError();
}

}  // namespace beam

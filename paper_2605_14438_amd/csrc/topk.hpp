// Wave-level Top-K + softmax + binary mask for one token (paper Sec. 3.2 Step 1,
// Eq. 4, Eq. 6), shared by the routing kernels.
#pragma once

#include "common.hpp"

namespace beam {

template <int CTRL, int ROW_MASK>
__device__ __forceinline__ uint64_t dpp_move_u64(uint64_t v) {
    // lanes whose source lies outside the row / mask keep their own value
    const int lo = __builtin_amdgcn_update_dpp((int)(uint32_t)v, (int)(uint32_t)v, CTRL, ROW_MASK,
                                               0xf, false);
    const int hi = __builtin_amdgcn_update_dpp((int)(uint32_t)(v >> 32), (int)(uint32_t)(v >> 32),
                                               CTRL, ROW_MASK, 0xf, false);
    return ((uint64_t)(uint32_t)hi << 32) | (uint32_t)lo;
}

template <int CTRL, int ROW_MASK>
__device__ __forceinline__ void max_step(uint64_t &key) {
    const uint64_t other = dpp_move_u64<CTRL, ROW_MASK>(key);
    key = other > key ? other : key;
}

// Largest key of the wavefront, returned in every lane.  DPP lane moves (quad
// swaps, half-row and row mirrors, row broadcasts into lane 63) cost a cycle or
// two each where an LDS-routed shuffle costs tens; routing is one latency chain.
__device__ __forceinline__ uint64_t wave_max_u64(uint64_t key) {
    max_step<0xB1, 0xf>(key);   // quad_perm [1,0,3,2]
    max_step<0x4E, 0xf>(key);   // quad_perm [2,3,0,1]
    max_step<0x141, 0xf>(key);  // row_half_mirror
    max_step<0x140, 0xf>(key);  // row_mirror: every lane of a 16-lane row holds the row's best
    max_step<0x142, 0xa>(key);  // row_bcast:15 into rows 1 and 3
    max_step<0x143, 0xc>(key);  // row_bcast:31 into rows 2 and 3: lane 63 holds the best
    const uint32_t lo = __builtin_amdgcn_readlane((int)(uint32_t)key, 63);
    const uint32_t hi = __builtin_amdgcn_readlane((int)(uint32_t)(key >> 32), 63);
    return ((uint64_t)hi << 32) | lo;
}

// One sortable key per candidate: the logit mapped to an unsigned integer that
// orders like the float, then the complemented expert index, so that a single
// unsigned compare realises "logit descending, equal logits by ascending expert
// index".  -0 is folded into +0 first (they compare equal as floats).  The
// lowest bit carries the candidate's mask decision (a >= 0) along, so the
// winner's mask needs no second, dependent memory access; it sits below the
// index and cannot change the order.  Key 0 marks "no candidate".
__device__ __forceinline__ uint64_t topk_key(float v, int e, bool keep) {
    uint32_t u = __float_as_uint(v + 0.0f);
    u = (u & 0x80000000u) ? ~u : (u | 0x80000000u);
    const uint32_t low = ((0x7FFFFFFFu - (uint32_t)e) << 1) | (keep ? 1u : 0u);
    return ((uint64_t)u << 32) | low;
}
__device__ __forceinline__ int key_expert(uint64_t key) {
    return (int)(0x7FFFFFFFu - ((uint32_t)key >> 1));
}
__device__ __forceinline__ bool key_keep(uint64_t key) { return ((uint32_t)key & 1u) != 0; }
__device__ __forceinline__ float key_logit(uint64_t key) {
    uint32_t u = (uint32_t)(key >> 32);
    u = (u & 0x80000000u) ? (u & 0x7FFFFFFFu) : ~u;
    return __uint_as_float(u);
}

// Whole wavefront, one token: lane l holds logits l, l+64, l+128, l+192
// (N <= 256) of both heads.  K rounds of wave arg-max; after round k lane k
// keeps the winner, so slot k = rank k+1.  Lanes k < K then write ids, softmax
// weights over the K survivors and the masked id (a >= 0 keeps, otherwise -1).
// br / bm: optional biases still to be added to r / a (NULL if the logits already
// include them).
// Shared experts (App. A.3): lanes K .. K+S-1 append S always-kept slots for the
// experts N .. N+S-1 with weight g_shared; the three outputs are rows of K+S.
// RULE picks what decides "kept" (the routing weights are Eq. 4's either way):
//   kRuleMask     a >= param; param = ln(tau/(1-tau)) for a threshold tau on
//                 sigma(a), 0 for the paper's tau = 0.5 (Eq. 6, Sec. 4.4)
//   kRuleCumProb  the cumulative-probability baseline of Sec. 4.1: with p the
//                 softmax of r over all N experts, slot k is kept iff the ranks
//                 before it sum to at most param (= phi)
constexpr int kRuleMask = 0;
constexpr int kRuleCumProb = 1;

// The logits may arrive as several arrays of partial sums (a logits GEMM whose
// reduction was cut into parts): part p of an entry sits p * stride floats after
// part 0.  The parts are added in order wherever logits are read, so every
// reader sees the same fp32 value.
struct LogitParts {
    int n = 1;
    size_t stride = 0;
};
__device__ __forceinline__ float sum_parts(const float *p, LogitParts parts) {
    float v = p[0];
    for (int q = 1; q < parts.n; ++q) v += p[q * parts.stride];
    return v;
}
__device__ __forceinline__ float4 sum_parts4(const float *p, LogitParts parts) {
    float4 v = *(const float4 *)p;
    for (int q = 1; q < parts.n; ++q) {
        const float4 u = *(const float4 *)(p + q * parts.stride);
        v.x += u.x, v.y += u.y, v.z += u.z, v.w += u.w;
    }
    return v;
}

template <int RULE>
__device__ __forceinline__ void wave_route_token(const float *__restrict__ r,
                                                 const float *__restrict__ a,
                                                 const float *__restrict__ br,
                                                 const float *__restrict__ bm, int N, int K,
                                                 int S, float g_shared, float param,
                                                 int32_t *__restrict__ ids_out,
                                                 float *__restrict__ w_out,
                                                 int32_t *__restrict__ masked_out,
                                                 LogitParts parts = LogitParts()) {
    const int lane = threadIdx.x & 63;
    uint64_t key[4];
    float logit[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int e = lane + 64 * i;
        key[i] = 0ull;
        logit[i] = -INFINITY;
        if (e < N) {
            const float r0 = sum_parts(r + e, parts), a0 = sum_parts(a + e, parts);
            const float rv = br ? r0 + br[e] : r0;
            const float av = bm ? a0 + bm[e] : a0;
            key[i] = topk_key(rv, e, av >= param);
            logit[i] = rv;
        }
    }
    uint64_t mine = 0;
    for (int k = 0; k < K; ++k) {
        uint64_t best = key[0];
#pragma unroll
        for (int i = 1; i < 4; ++i) best = key[i] > best ? key[i] : best;
        best = wave_max_u64(best);
#pragma unroll
        for (int i = 0; i < 4; ++i) key[i] = key[i] == best ? 0ull : key[i];
        mine = lane == k ? best : mine;
    }
    const int my_id = key_expert(mine);
    const float my_r = key_logit(mine);
    const float top = __shfl(my_r, 0);
    const float ex = lane < K ? expf(my_r - top) : 0.0f;
    const float denom = wave_sum(ex);
    bool keep = key_keep(mine);
    if constexpr (RULE == kRuleCumProb) {
        float zl = 0.0f;
#pragma unroll
        for (int i = 0; i < 4; ++i) zl += expf(logit[i] - top);   // exp(-inf) = 0 past N
        const float p = ex / wave_sum(zl);
        float before = 0.0f;                 // probability of the ranks ahead of this slot
        for (int q = 0; q < K; ++q) {
            const float pq = __shfl(p, q);
            before += q < lane ? pq : 0.0f;
        }
        keep = before <= param;
    }
    if (lane < K) {
        ids_out[lane] = my_id;
        w_out[lane] = ex / denom;
        masked_out[lane] = keep ? my_id : -1;
    } else if (lane < K + S) {
        ids_out[lane] = N + lane - K;
        w_out[lane] = g_shared;
        masked_out[lane] = N + lane - K;
    }
}

// Throughput variant for large batches: one token per 16-lane row, four tokens
// per wavefront.  Lane j of a row holds candidates j*NPL .. j*NPL+NPL-1 (N <=
// 16*NPL), so the arg-max reductions stay inside a row: four DPP steps, no
// cross-row traffic, and every lane of the row ends up with the row's best key.
// Same keys, same K rounds, same softmax and shared-expert slots as
// wave_route_token; needs K + S <= 16.
// `valid` is row-uniform (false for the rows past the last token).  Returns the
// masked id that lane j wrote for slot j (-1: dropped, or no slot j).
__device__ __forceinline__ uint64_t row_max_u64(uint64_t key) {
    max_step<0xB1, 0xf>(key);   // quad_perm [1,0,3,2]
    max_step<0x4E, 0xf>(key);   // quad_perm [2,3,0,1]
    max_step<0x141, 0xf>(key);  // row_half_mirror
    max_step<0x140, 0xf>(key);  // row_mirror
    return key;
}

__device__ __forceinline__ float row_sum_f32(float v) {
    v += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), 0xB1, 0xf, 0xf, false));
    v += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), 0x4E, 0xf, 0xf, false));
    v += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), 0x141, 0xf, 0xf, false));
    v += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), 0x140, 0xf, 0xf, false));
    return v;
}

template <int NPL, int RULE>
__device__ __forceinline__ int row_route_token(const float *__restrict__ r,
                                                const float *__restrict__ a,
                                                const float *__restrict__ br,
                                                const float *__restrict__ bm, int N, int K,
                                                int S, float g_shared, float param, bool valid,
                                                int32_t *__restrict__ ids_out,
                                                float *__restrict__ w_out,
                                                int32_t *__restrict__ masked_out,
                                               LogitParts parts = LogitParts()) {
    static_assert(NPL % 4 == 0, "candidates are loaded four at a time");
    const int j = threadIdx.x & 15;
    uint64_t key[NPL];
    float logit[RULE == kRuleCumProb ? NPL : 1];  // kRuleCumProb needs the softmax over all N
#pragma unroll
    for (int q = 0; q < NPL / 4; ++q) {
        const int e0 = j * NPL + q * 4;
        float4 rv = make_float4(0.f, 0.f, 0.f, 0.f), av = rv;
        const bool in = valid && e0 < N;  // N % 4 == 0: a group of four is all in or all out
        if (in) {
            rv = sum_parts4(r + e0, parts);
            av = sum_parts4(a + e0, parts);
            if (br) {
                const float4 b = *(const float4 *)(br + e0);
                rv.x += b.x, rv.y += b.y, rv.z += b.z, rv.w += b.w;
            }
            if (bm) {
                const float4 b = *(const float4 *)(bm + e0);
                av.x += b.x, av.y += b.y, av.z += b.z, av.w += b.w;
            }
        }
        key[q * 4 + 0] = in ? topk_key(rv.x, e0 + 0, av.x >= param) : 0ull;
        key[q * 4 + 1] = in ? topk_key(rv.y, e0 + 1, av.y >= param) : 0ull;
        key[q * 4 + 2] = in ? topk_key(rv.z, e0 + 2, av.z >= param) : 0ull;
        key[q * 4 + 3] = in ? topk_key(rv.w, e0 + 3, av.w >= param) : 0ull;
        if constexpr (RULE == kRuleCumProb) {
            logit[q * 4 + 0] = in ? rv.x : -INFINITY;
            logit[q * 4 + 1] = in ? rv.y : -INFINITY;
            logit[q * 4 + 2] = in ? rv.z : -INFINITY;
            logit[q * 4 + 3] = in ? rv.w : -INFINITY;
        }
    }
    uint64_t mine = 0;
    for (int k = 0; k < K; ++k) {
        uint64_t best = key[0];
#pragma unroll
        for (int i = 1; i < NPL; ++i) best = key[i] > best ? key[i] : best;
        best = row_max_u64(best);
#pragma unroll
        for (int i = 0; i < NPL; ++i) key[i] = key[i] == best ? 0ull : key[i];
        mine = j == k ? best : mine;
    }
    const int my_id = key_expert(mine);
    const float my_r = key_logit(mine);
    const float top = __shfl(my_r, threadIdx.x & 48);  // lane 0 of this row (wave-relative)
    const float ex = j < K ? expf(my_r - top) : 0.0f;
    const float denom = row_sum_f32(ex);
    bool keep = key_keep(mine);
    if constexpr (RULE == kRuleCumProb) {
        float zl = 0.0f;
#pragma unroll
        for (int i = 0; i < NPL; ++i) zl += expf(logit[i] - top);   // exp(-inf) = 0 past N
        const float p = ex / row_sum_f32(zl);
        float before = 0.0f;
        for (int q = 0; q < K; ++q) {
            const float pq = __shfl(p, (threadIdx.x & 48) + q);
            before += q < j ? pq : 0.0f;
        }
        keep = before <= param;
    }
    int kept_id = -1;  // what lane j wrote to masked_out; -1 also for the lanes that wrote nothing
    if (valid && j < K) {
        kept_id = keep ? my_id : -1;
        ids_out[j] = my_id;
        w_out[j] = ex / denom;
        masked_out[j] = kept_id;
    } else if (valid && j < K + S) {
        kept_id = N + j - K;
        ids_out[j] = kept_id;
        w_out[j] = g_shared;
        masked_out[j] = kept_id;
    }
    return kept_id;
}

}  // namespace beam

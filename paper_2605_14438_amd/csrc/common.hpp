// Internal declarations shared by the HIP translation units of libbeam.
// gfx950 only: 64-wide wavefronts, bf16 MFMA with fp32 accumulation.
#pragma once

#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include "beam.h"

namespace beam {

constexpr int kWave = 64;

// Pairs handled by the one workgroup of the decode grouping kernel (one wavefront
// walks kGroupsPerChunk groups of 64 flat pair indices in order).
constexpr int kGroupsPerChunk = 8;
constexpr int kChunk = kWave * kGroupsPerChunk;

// Row tile of the prefill grouped GEMM.  Every expert segment is cut into row
// tiles of this many grouped rows (the last one ragged): the paper's "block
// alignment" (App. A.4), done with a tile list instead of padding the index
// array, so at most kTileM - 1 padded rows per expert are ever multiplied.
constexpr int kTileM = 128;
// y_pairs [P,H] fp32 is written once by the down projection and read once by the
// aggregation.  Beyond this size (the 256 MiB last-level cache) it cannot stay
// on chip between the two, and both sides use non-temporal accesses so that it
// does not displace the weights and activations that are reused: measured at
// P*H*4 = 1.07 GB down 556 -> 536 us and aggregation 241 -> 194 us; below it the
// plain accesses are faster (the aggregation finds y_pairs in cache).
constexpr size_t kStreamBytes = (size_t)256 << 20;

__host__ __device__ inline int tiles_of(int count) { return (count + kTileM - 1) / kTileM; }

typedef uint16_t bf16_t;
typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(4 * sizeof(float)))) float f32x4;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float f32x16;

__device__ __forceinline__ float bf16_to_f32(bf16_t v) {
    return __uint_as_float(((uint32_t)v) << 16);
}
// Round-to-nearest-even (gfx950 has a hardware conversion; the compiler emits
// it for the __bf16 cast).
__device__ __forceinline__ bf16_t f32_to_bf16(float f) {
    return __builtin_bit_cast(bf16_t, (__bf16)f);
}

__device__ __forceinline__ float load_f32(const float *p) { return *p; }
__device__ __forceinline__ float load_f32(const bf16_t *p) { return bf16_to_f32(*p); }
__device__ __forceinline__ void store_from_f32(float *p, float v) { *p = v; }
__device__ __forceinline__ void store_from_f32(bf16_t *p, float v) { *p = f32_to_bf16(v); }

// SiLU with the hardware exponential and reciprocal (about 1 ulp each) instead
// of an IEEE division: the result is rounded to bf16 (8 bits) right after, and a
// GEMM epilogue evaluates 128 of these per lane.
__device__ __forceinline__ float silu(float g) {
    return g * __builtin_amdgcn_rcpf(1.0f + __expf(-g));
}

__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) v += __shfl_xor(v, off);
    return v;
}

// Device workspace carve-up.  Every offset is a multiple of 256 bytes.
struct WsLayout {
    size_t router_logits;  // [T,N] f32
    size_t mask_logits;    // [T,N] f32 (router_logits and mask_logits are contiguous)
    size_t packed_heads;   // [2N,H] dtype : router and mask heads in MFMA fragment order
    size_t topk_ids;       // [T,K] i32
    size_t topk_w;         // [T,K] f32
    size_t masked_ids;     // [T,K] i32
    size_t g_shared;       // [T] f32 : weight of the shared-expert slots (block entry point)
    size_t slice_counts;   // [slices,N] i32 : kept pairs per (slice of the pair list, expert)
    size_t counts;         // [N] i32
    size_t offsets;        // [N+1] i32
    size_t num_pairs;      // [1] i32
    size_t perm;           // [T*K] i32
    size_t inv_perm;       // [T*K] i32
    size_t work;           // work list, see WorkList
    size_t hidden;         // [T*K, I] dtype : SiLU(gate)*up of every grouped row
    size_t y_pairs;        // [T*K, H] f32
    size_t tile_partial;   // [max_tiles, H] f32 : per-tile sums of the mask-router backward
    size_t total;
    size_t router_logits_bytes;  // size of the logits region (router + mask, every part)
    int logit_parts;             // [T,2N] arrays the region has room for
    int max_tiles;
};
WsLayout ws_layout(const beam_shape &s, int S = 0);

// Work list written on the device after the prefix sums:
//   hdr[0] = number of experts with at least one kept pair (U)
//   hdr[1] = number of row tiles
//   hdr[2] = which expert GEMM kernels suit the realised counts (kRegimeStream / kRegimeTiled);
//            where the host cannot tell from the shape it launches both families and each
//            kernel leaves at once unless it is the one chosen here
//   active[u]      expert id of the u-th non-empty expert (most rows first where the list
//                  is built from counts; descending id in the single-chunk grouping)
//   active_beg[u], active_end[u]  its grouped rows [beg, end)
//   tile_expert[i] expert of row tile i,  tile_row0[i] its first grouped row
// A workgroup that serves active expert u fetches all four words in one round
// trip instead of chasing hdr -> active -> offsets.
constexpr int kRegimeStream = 0;
constexpr int kRegimeTiled = 1;
constexpr int kRegimeAny = -1;     // kernel argument: run whatever hdr[2] says
// rows of one expert that the streaming kernels cover in one pass over its weights
constexpr int kStreamRows = 32;
struct WorkList {
    int32_t *hdr;
    int32_t *active;
    int32_t *active_beg;
    int32_t *active_end;
    int32_t *tile_expert;
    int32_t *tile_row0;
};
WorkList work_list(void *base, const beam_shape &s, int max_tiles);

// Between the launches of a multi-kernel sequence: return at the first launch that
// failed (a later successful launch may clear what hipGetLastError reports).
#define BEAM_CHECK_LAUNCH()                                   \
    do {                                                      \
        const hipError_t launch_err_ = hipGetLastError();     \
        if (launch_err_ != hipSuccess) return launch_err_;    \
    } while (0)

// ---- launchers (each returns hipGetLastError() after enqueueing) ----------
// What the Top-K stage appends and decides beyond Eq. 4: S shared-expert slots
// with per-token weight g_shared (NULL = 1), and the activation rule (0: mask
// pre-activation >= param; 1: cumulative routing probability, param = phi).
struct RouteOpts {
    int S = 0;
    const float *g_shared = nullptr;
    int rule = 0;
    float param = 0.0f;
};
// zero_word: an int32 the MFMA logits kernels reset to 0 (bf16, H % 128 == 0 only;
// NULL: none), for a counter that a later kernel of the same call adds to
hipError_t launch_logits(const beam_shape &s, const void *x, const void *w_router,
                         const float *b_router, const void *w_mask, const float *b_mask,
                         float *router_logits, float *mask_logits, hipStream_t st,
                         int32_t *zero_word = nullptr);
hipError_t launch_split_logits(const beam_shape &s, const float *logits2, const float *b_router,
                               const float *b_mask, float *router_logits, float *mask_logits,
                               hipStream_t st, int n_parts = 1);
bool tiny_decode_supported(const beam_shape &s, int S);
hipError_t launch_tiny_gate_up(const beam_shape &s, const RouteOpts &opt, const void *x,
                               const float *router_logits, const float *mask_logits,
                               const void *w_gate_up, void *hidden, hipStream_t st);
hipError_t launch_tiny_down_combine(const beam_shape &s, const RouteOpts &opt,
                                    const float *router_logits, const float *mask_logits,
                                    const void *hidden, const void *w_down, const void *residual,
                                    void *out, int32_t *topk_ids_opt, float *topk_w_opt,
                                    int32_t *masked_ids_opt, int32_t *num_pairs_opt,
                                    hipStream_t st);
hipError_t launch_shared_gate(const beam_shape &s, const void *x, const void *w_shared_gate,
                              float *g_shared, hipStream_t st);
hipError_t launch_topk_mask(const beam_shape &s, const float *router_logits,
                            const float *mask_logits, const float *b_router, const float *b_mask,
                            int row_stride, const RouteOpts &opt, int32_t *topk_ids,
                            float *topk_w, int32_t *masked_ids, hipStream_t st, int n_parts = 1);
bool logits_tiled_supported(const beam_shape &s);
// parts the tiled logits GEMM cuts its reduction into (its output is that many [T,2N] arrays)
int logits_split_k(const beam_shape &s);
hipError_t launch_logits_tiled(const beam_shape &s, const void *x, const void *w_router,
                               const void *w_mask, void *packed_heads, float *logits2,
                               hipStream_t st);
hipError_t launch_permute(const beam_shape &s, const int32_t *masked_ids, int32_t *counts,
                          int32_t *offsets, int32_t *perm, int32_t *inv_perm, int32_t *num_pairs,
                          int32_t *slice_counts, const WorkList &wl, hipStream_t st,
                          bool longest_first = false);
int permute_slices(long TK);   // rows of slice_counts the grouping of TK pairs needs
bool route_permute_supported(const beam_shape &s, const RouteOpts &opt, const float *router_logits,
                             const float *mask_logits);
hipError_t launch_route_permute(const beam_shape &s, const float *router_logits,
                                const float *mask_logits, const RouteOpts &opt,
                                int32_t *topk_ids, float *topk_w, int32_t *masked_ids,
                                int32_t *counts, int32_t *offsets, int32_t *perm,
                                int32_t *inv_perm, int32_t *num_pairs, const WorkList &wl,
                                hipStream_t st);
// longest_first: order the active-expert list by row count, most rows first (for the
// streaming kernels, which walk it)
hipError_t launch_work_list(const beam_shape &s, const int32_t *offsets, const WorkList &wl,
                            hipStream_t st, bool longest_first = false);
// What the host can tell about the expert GEMMs from the shape alone.
enum class Regime { Stream, Tiled, Auto, Generic };
Regime ffn_regime(const beam_shape &s);
hipError_t launch_gate_up(const beam_shape &s, const void *x, const void *w_gate_up,
                          const int32_t *offsets, const int32_t *perm, const int32_t *num_pairs,
                          const WorkList &wl, void *hidden, hipStream_t st);
// k_split > 1 (tiled path only): y_pairs is k_split arrays [T*K,H] of partial sums
// y16 (tiled path with k_split == 1 only): y_pairs is an array of half-precision rows
hipError_t launch_down(const beam_shape &s, const void *hidden, const void *w_down,
                       const int32_t *offsets, const int32_t *num_pairs, const WorkList &wl,
                       float *y_pairs, hipStream_t st, int k_split = 1, bool y16 = false);
// num_pairs (device, may be NULL): lets the kernel see how large y_pairs is
hipError_t launch_combine(const beam_shape &s, const float *y_pairs, const float *topk_w,
                          const int32_t *masked_ids, const int32_t *inv_perm,
                          const void *residual, void *out, hipStream_t st,
                          const int32_t *num_pairs = nullptr, int k_split = 1, bool y16 = false);

}  // namespace beam

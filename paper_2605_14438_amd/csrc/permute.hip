// Expert-wise grouping of the kept (token, expert) pairs (paper App. A.4: ids
// equal to -1 are skipped when tokens are grouped by expert).  A stable
// counting sort of the flat pair index f = t*K+k by expert id.  The pair list is
// cut into slices of 2048 to 8192 pairs, one workgroup of 16 wavefronts each,
// every wavefront a contiguous run of pairs:
//   1. count    per slice, the kept pairs per expert (per-wavefront LDS rows,
//               summed over the wavefronts)
//   2. scatter  every slice counts its wavefronts' pairs again, adds up the
//               slices' counts per expert (all of them for the expert's start,
//               the earlier ones for its own start inside the expert) and
//               places each kept pair at start + (rank among equal ids so far);
//               one more workgroup writes the per-expert arrays and the work
//               list the FFN kernels walk
// Placement uses only prefix sums and wavefront ballots, never atomics, so the
// result is the same on every run.  Up to one slice the two steps are one launch
// of one workgroup; decode batches (up to 512 pairs) have a shorter kernel still.

#include "common.hpp"
#include "topk.hpp"

namespace beam {

// Lanes of the wavefront that hold the same id (ids < 2^nbits <= 256), restricted
// to valid lanes: one ballot per id bit.
__device__ __forceinline__ int id_bits(int N) { return N > 1 ? 32 - __builtin_clz(N - 1) : 0; }

__device__ __forceinline__ uint64_t match_id(int id, bool valid, int nbits) {
    uint64_t peers = __ballot(valid);
#pragma unroll
    for (int b = 0; b < 8; ++b) {
        if (b >= nbits) break;   // uniform
        const bool bit = (id >> b) & 1;
        const uint64_t m = __ballot(valid && bit);
        peers &= bit ? m : ~m;
    }
    return peers;
}

// Exclusive prefix sum over 256 entries held one per thread by the first 256
// threads of a workgroup (every thread of the workgroup must call it; threads
// >= 256 pass 0 and only take part in the barriers); returns the exclusive
// value, *total gets the sum.  Wavefront shuffles plus four wavefront totals in
// scratch: two barriers.
__device__ __forceinline__ int block_exclusive_scan_256(int v, int *scratch /*[>= 4]*/, int *total) {
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = tid >> 6;
    int incl = v;
#pragma unroll
    for (int off = 1; off < 64; off <<= 1) {
        const int t = __shfl_up(incl, off);
        if (lane >= off) incl += t;
    }
    if (tid < 256 && lane == 63) scratch[wave] = incl;
    __syncthreads();
    int run = incl - v;
    int sum = 0;
#pragma unroll
    for (int w = 0; w < 4; ++w) {
        const int s = scratch[w];
        run += w < wave ? s : 0;
        sum += s;
    }
    *total = sum;
    __syncthreads();   // scratch may be written again
    return tid < 256 ? run : 0;
}

// Work list from the per-expert counts (thread e < 256 owns expert e; threads past
// 256, if any, pass e >= N and count 0 and help with the barriers and the tile list).
// The row tiles are written by all threads together, tile t by thread t % 256,
// which finds its expert by bisection over the tile prefix: with a skewed router
// one expert can own most of the tiles, and its thread would otherwise write
// them one by one.
__device__ __forceinline__ void emit_work_list(int e, int N, int count, int offset,
                                               const WorkList &wl, int *scratch,
                                               bool longest_first) {
    __shared__ int tile_end[256];   // inclusive prefix of the experts' tile counts
    __shared__ int row_beg[256];
    // Order of the active-expert list, which the streaming kernels walk one workgroup set
    // per entry.  longest_first (asked for when those kernels may run): experts that need
    // several passes over their weights come first (more than four passes, then more than
    // one, then the rest; expert order inside a class), so that the long-running workgroup
    // sets (a shared expert's above all) start first instead of forming the tail.  One scan
    // of the three class flags packed ten bits apiece gives every expert its position.
    const int has = (e < N && count > 0) ? 1 : 0;
    int cls = 2;
    if (longest_first) cls = count > 4 * kStreamRows ? 0 : (count > kStreamRows ? 1 : 2);
    int packed_total;
    const int packed_before = block_exclusive_scan_256(has << (10 * cls), scratch, &packed_total);
    const int t0 = packed_total & 1023, t1 = (packed_total >> 10) & 1023;
    const int n_active = t0 + t1 + (packed_total >> 20);
    if (has) {
        const int within = (packed_before >> (10 * cls)) & 1023;
        const int slot = within + (cls > 0 ? t0 : 0) + (cls > 1 ? t1 : 0);
        wl.active[slot] = e;
        wl.active_beg[slot] = offset;
        wl.active_end[slot] = offset + count;
    }
    if (threadIdx.x == 0) wl.hdr[0] = n_active;
    // Regime of the expert GEMMs, from the realised counts: the streaming kernels read an
    // expert's weights once per pass of kStreamRows rows, the tiled GEMM about once; measured
    // on the Qwen3-shaped layer (T = 128 .. 4096, keep 15 % .. 100 %, uniform and skewed
    // routing) the streaming kernels win while the passes stay within 1.3 per active expert
    // and no expert has more than four passes (its workgroups would run them back to back
    // while the rest of the chip idles: a shared expert from 129 tokens on).
    int passes;
    (void)block_exclusive_scan_256(e < N ? (count + kStreamRows - 1) / kStreamRows : 0, scratch,
                                   &passes);
    if (threadIdx.x == 0)
        wl.hdr[2] = (10 * passes > 13 * n_active || (longest_first && t0 > 0)) ? kRegimeTiled
                                                                               : kRegimeStream;
    int total;
    const int nt = e < N ? tiles_of(count) : 0;
    const int tbase = block_exclusive_scan_256(nt, scratch, &total);
    if (threadIdx.x < 256) {
        tile_end[e] = tbase + nt;
        row_beg[e] = offset;
    }
    __syncthreads();
    for (int t = threadIdx.x; t < total; t += blockDim.x) {
        int lo = 0, hi = 255;   // first expert whose tiles end after t
        while (lo < hi) {
            const int mid = (lo + hi) >> 1;
            if (tile_end[mid] > t) hi = mid;
            else lo = mid + 1;
        }
        const int first = lo == 0 ? 0 : tile_end[lo - 1];
        wl.tile_expert[t] = lo;
        wl.tile_row0[t] = row_beg[lo] + (t - first) * kTileM;
    }
    if (threadIdx.x == 0) wl.hdr[1] = total;
}

// Work list alone, for callers that hand in expert_offsets directly.
__global__ __launch_bounds__(256) void work_list_kernel(const int32_t *__restrict__ offsets, int N,
                                                        WorkList wl, int longest_first) {
    __shared__ int scratch[256];
    const int e = threadIdx.x;
    int off = 0, cnt = 0;
    if (e < N) {
        off = offsets[e];
        cnt = offsets[e + 1] - off;
        if (cnt < 0) cnt = 0;
    }
    emit_work_list(e, N, cnt, off, wl, scratch, longest_first != 0);
}

// Decode batches: the whole pair list is one chunk (T*K <= kChunk).  The first
// 256 threads of the workgroup do count, scans, work list and scatter with
// four barriers (every thread of the workgroup must call this; `ids` may live
// in LDS or in global memory).  Wavefront w < 4 ranks the pairs of groups w and
// w+4 (64 pairs each) with ballots; thread e < 256 then owns expert e.
struct ChunkShared {
    int grp[kGroupsPerChunk][256];  // kept pairs per (group, expert), then their prefix
    int offs[256];
    int wtot[4][3];
};

__device__ __forceinline__ void permute_chunk_body(const int32_t *ids, ChunkShared &sh,
                                                   int32_t *__restrict__ counts,
                                                   int32_t *__restrict__ offsets,
                                                   int32_t *__restrict__ perm,
                                                   int32_t *__restrict__ inv_perm,
                                                   int32_t *__restrict__ num_pairs, int TK, int N,
                                                   const WorkList &wl) {
    static_assert(kGroupsPerChunk == 8, "two groups per wavefront");
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = tid >> 6;
    const bool worker = tid < 256;  // wave-uniform
    if (worker) {
#pragma unroll
        for (int g = 0; g < kGroupsPerChunk; ++g) sh.grp[g][tid] = 0;
    }
    __syncthreads();
    int id2[2] = {-1, -1}, rank2[2] = {0, 0};
    if (worker) {
#pragma unroll
        for (int q = 0; q < 2; ++q) {
            const int g = wave + 4 * q;
            const int f = g * 64 + lane;
            const int id = f < TK ? ids[f] : -1;
            const bool valid = id >= 0 && id < N;
            const uint64_t peers = match_id(id, valid, id_bits(N));
            id2[q] = valid ? id : -1;
            rank2[q] = __popcll(peers & ((1ull << lane) - 1ull));
            if (valid && rank2[q] == 0) sh.grp[g][id] = __popcll(peers);
        }
    }
    __syncthreads();
    int cnt = 0, s_cnt = 0, s_has = 0, s_tiles = 0, nt = 0;
    if (worker) {  // thread tid owns expert tid
#pragma unroll
        for (int g = 0; g < kGroupsPerChunk; ++g) {
            const int c = sh.grp[g][tid];
            sh.grp[g][tid] = cnt;
            cnt += c;
        }
        s_cnt = cnt;
        s_has = cnt > 0 ? 1 : 0;
        nt = tiles_of(cnt);
        s_tiles = nt;
#pragma unroll
        for (int off = 1; off < 64; off <<= 1) {
            const int ta = __shfl_up(s_cnt, off);
            const int tb = __shfl_up(s_has, off);
            const int tc = __shfl_up(s_tiles, off);
            if (lane >= off) {
                s_cnt += ta;
                s_has += tb;
                s_tiles += tc;
            }
        }
        if (lane == 63) {
            sh.wtot[wave][0] = s_cnt;
            sh.wtot[wave][1] = s_has;
            sh.wtot[wave][2] = s_tiles;
        }
    }
    __syncthreads();
    int total = 0;
    if (worker) {
        int t_has = 0, t_tiles = 0;
#pragma unroll
        for (int w = 0; w < 4; ++w) {
            if (w < wave) {
                s_cnt += sh.wtot[w][0];
                s_has += sh.wtot[w][1];
                s_tiles += sh.wtot[w][2];
            }
            total += sh.wtot[w][0];
            t_has += sh.wtot[w][1];
            t_tiles += sh.wtot[w][2];
        }
        const int has = cnt > 0 ? 1 : 0;
        const int excl = s_cnt - cnt;
        sh.offs[tid] = excl;
        if (tid < N) {
            counts[tid] = cnt;
            offsets[tid] = excl;
        }
        if (tid == 0) {
            offsets[N] = total;
            *num_pairs = total;
            wl.hdr[0] = t_has;
            wl.hdr[1] = t_tiles;
            wl.hdr[2] = kRegimeStream;   // a handful of pairs: never the tiled GEMM's case
        }
        if (has) {
            // descending expert id: the shared experts (the last ids, every token's rows)
            // come first in the list the streaming kernels walk
            wl.active[t_has - s_has] = tid;
            wl.active_beg[t_has - s_has] = excl;
            wl.active_end[t_has - s_has] = excl + cnt;
        }
        for (int i = 0; i < nt; ++i) {
            wl.tile_expert[s_tiles - nt + i] = tid;
            wl.tile_row0[s_tiles - nt + i] = excl + i * kTileM;
        }
    }
    __syncthreads();
    if (worker) {
#pragma unroll
        for (int q = 0; q < 2; ++q) {
            const int g = wave + 4 * q;
            const int f = g * 64 + lane;
            if (f >= TK) continue;
            if (id2[q] >= 0) {
                const int pos = sh.offs[id2[q]] + sh.grp[g][id2[q]] + rank2[q];
                perm[pos] = f;
                inv_perm[f] = pos;
            } else {
                inv_perm[f] = -1;
            }
            if (f >= total) perm[f] = -1;
        }
    }
}

__global__ __launch_bounds__(256) void permute_single_chunk_kernel(
    const int32_t *__restrict__ masked_ids, int32_t *__restrict__ counts,
    int32_t *__restrict__ offsets, int32_t *__restrict__ perm, int32_t *__restrict__ inv_perm,
    int32_t *__restrict__ num_pairs, int TK, int N, WorkList wl) {
    __shared__ ChunkShared sh;
    permute_chunk_body(masked_ids, sh, counts, offsets, perm, inv_perm, num_pairs, TK, N, wl);
}

// Decode batches, fused layer: Top-K + softmax + mask of all tokens (one per
// 16-lane row, up to 32 tokens) and the single-chunk grouping in one launch of
// one workgroup; the masked ids go to the grouping through LDS.  Same token and
// chunk code as the separate kernels, so the same bits; one launch and one
// global round trip of the ids less on a path that is a chain of latencies.
template <int NPL, int RULE>
__global__ __launch_bounds__(512) void route_permute_kernel(
    const float *__restrict__ router_logits, const float *__restrict__ mask_logits,
    const float *__restrict__ g_shared, float param, int32_t *__restrict__ topk_ids,
    float *__restrict__ topk_w, int32_t *__restrict__ masked_ids, int32_t *__restrict__ counts,
    int32_t *__restrict__ offsets, int32_t *__restrict__ perm, int32_t *__restrict__ inv_perm,
    int32_t *__restrict__ num_pairs, int Tn, int N, int K, int S, WorkList wl) {
    __shared__ ChunkShared sh;
    __shared__ int32_t ids[kChunk];
    const int slots = K + S;
    const int t = threadIdx.x >> 4;
    const int j = threadIdx.x & 15;
    const bool valid = t < Tn;
    const int tc = valid ? t : Tn - 1;
    const size_t f = (size_t)tc * slots;
    const float gs = (S > 0 && g_shared) ? g_shared[tc] : 1.0f;
    const int kept = row_route_token<NPL, RULE>(
        router_logits + (size_t)tc * N, mask_logits + (size_t)tc * N, nullptr, nullptr, N, K, S,
        gs, param, valid, topk_ids + f, topk_w + f, masked_ids + f);
    if (valid && j < slots) ids[t * slots + j] = kept;
    __syncthreads();
    permute_chunk_body(ids, sh, counts, offsets, perm, inv_perm, num_pairs, Tn * slots, N + S, wl);
}

// s.N, s.K: routed experts and slots; opt.S shared slots follow.  Logits include the biases.
// Up to 32 tokens: measured 1.4-1.5 us per layer faster than the two launches at T = 4
// and 8, 0.8 at T = 32, but 0.7 slower at T = 64, where the one workgroup's Top-K work
// outweighs the launch it saves.
bool route_permute_supported(const beam_shape &s, const RouteOpts &opt, const float *router_logits,
                             const float *mask_logits) {
    return s.T <= 32 && s.T * (s.K + opt.S) <= kChunk && s.K + opt.S <= 16 && s.N % 4 == 0 &&
           s.N <= 256 && ((uintptr_t)router_logits | (uintptr_t)mask_logits) % 16 == 0;
}

hipError_t launch_route_permute(const beam_shape &s, const float *router_logits,
                                const float *mask_logits, const RouteOpts &opt,
                                int32_t *topk_ids, float *topk_w, int32_t *masked_ids,
                                int32_t *counts, int32_t *offsets, int32_t *perm,
                                int32_t *inv_perm, int32_t *num_pairs, const WorkList &wl,
                                hipStream_t st) {
    // one 16-lane row per token; the grouping needs the first 256 threads
    const int threads = s.T * 16 <= 256 ? 256 : (s.T * 16 + 63) / 64 * 64;
#define BEAM_LAUNCH_RP(NPL_, RULE_)                                                            \
    route_permute_kernel<NPL_, RULE_><<<1, threads, 0, st>>>(                                  \
        router_logits, mask_logits, opt.g_shared, opt.param, topk_ids, topk_w, masked_ids,     \
        counts, offsets, perm, inv_perm, num_pairs, s.T, s.N, s.K, opt.S, wl)
#define BEAM_LAUNCH_RP_RULE(RULE_)                                                             \
    do {                                                                                       \
        if (s.N <= 64) BEAM_LAUNCH_RP(4, RULE_);                                               \
        else if (s.N <= 128) BEAM_LAUNCH_RP(8, RULE_);                                         \
        else BEAM_LAUNCH_RP(16, RULE_);                                                        \
    } while (0)
    if (opt.rule == kRuleCumProb) BEAM_LAUNCH_RP_RULE(kRuleCumProb);
    else BEAM_LAUNCH_RP_RULE(kRuleMask);
#undef BEAM_LAUNCH_RP_RULE
#undef BEAM_LAUNCH_RP
    return hipGetLastError();
}

// One slice of the pair list in a workgroup of 16 wavefronts.  Wavefront w owns a
// contiguous run of `per_wave` 64-pair groups starting at pair f0 - lane; it counts its
// pairs per expert into its own LDS row (slice_count), thread e then turns the rows into
// start positions, and every wavefront walks its run again in order, placing each kept
// pair at its expert's running position (slice_place): stable, no atomics.
constexpr int kOneWgWaves = 16;
constexpr int kOneWgGroups = 8;   // 64-pair groups per wavefront, held in registers
constexpr int kOneWgMaxPairs = 64 * kOneWgWaves * kOneWgGroups;

struct SlicePairs {
    int ids[kOneWgGroups];          // -1: masked, past the run or past the input
    uint64_t peers[kOneWgGroups];   // lanes of the group with the same id
};

// Every thread of the workgroup must call it (two barriers).  Afterwards pos[w][e] is the
// number of kept pairs of expert e in wavefront w's run.
__device__ __forceinline__ void slice_count(const int32_t *__restrict__ masked_ids, int TK, int N,
                                            int f0, int per_wave, int (*pos)[256],
                                            SlicePairs &sp) {
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = tid >> 6;
    // all loads of the run in flight at once
#pragma unroll
    for (int q = 0; q < kOneWgGroups; ++q) {
        const int f = f0 + q * 64;
        const int id = (q < per_wave && f < TK) ? masked_ids[f] : -1;
        sp.ids[q] = (id >= 0 && id < N) ? id : -1;
    }
    for (int i = tid; i < kOneWgWaves * 256; i += 64 * kOneWgWaves) (&pos[0][0])[i] = 0;
    __syncthreads();
    const int nbits = id_bits(N);
#pragma unroll
    for (int q = 0; q < kOneWgGroups; ++q) {
        sp.peers[q] = 0;
        if (q >= per_wave) continue;   // uniform: small inputs use the first groups only
        const bool valid = sp.ids[q] >= 0;
        sp.peers[q] = match_id(sp.ids[q], valid, nbits);
        if (valid && (sp.peers[q] & ((1ull << lane) - 1ull)) == 0)
            pos[wave][sp.ids[q]] += __popcll(sp.peers[q]);
    }
    __syncthreads();
}

// pos[w][e] holds the position of the first pair of expert e in wavefront w's run; `total`
// is the number of kept pairs of the whole input (rows from there on carry no pair).
__device__ __forceinline__ void slice_place(const SlicePairs &sp, int TK, int f0, int per_wave,
                                            int total, int (*pos)[256],
                                            int32_t *__restrict__ perm,
                                            int32_t *__restrict__ inv_perm) {
    const int lane = threadIdx.x & 63;
    const int wave = threadIdx.x >> 6;
#pragma unroll
    for (int q = 0; q < kOneWgGroups; ++q) {
        if (q >= per_wave) continue;
        const int f = f0 + q * 64;
        const bool valid = sp.ids[q] >= 0;
        const int rank = __popcll(sp.peers[q] & ((1ull << lane) - 1ull));
        const int base = valid ? pos[wave][sp.ids[q]] : 0;
        if (valid && rank == 0) pos[wave][sp.ids[q]] = base + __popcll(sp.peers[q]);
        if (f < TK) {
            if (valid) {
                perm[base + rank] = f;
                inv_perm[f] = base + rank;
            } else {
                inv_perm[f] = -1;
            }
            if (f >= total) perm[f] = -1;  // rows [P, T*K) carry no pair
        }
    }
}

// A few thousand pairs (prefill chunks of up to about 1000 tokens): the whole counting
// sort in one launch of one workgroup.
__global__ __launch_bounds__(64 * kOneWgWaves) void permute_one_workgroup_kernel(
    const int32_t *__restrict__ masked_ids, int32_t *__restrict__ counts,
    int32_t *__restrict__ offsets, int32_t *__restrict__ perm, int32_t *__restrict__ inv_perm,
    int32_t *__restrict__ num_pairs, int TK, int N, WorkList wl, int longest_first) {
    __shared__ int pos[kOneWgWaves][256];   // per wavefront and expert: count, then next position
    __shared__ int scratch[256];
    const int tid = threadIdx.x;
    const int groups = (TK + 63) >> 6;
    const int per_wave = (groups + kOneWgWaves - 1) / kOneWgWaves;   // <= kOneWgGroups
    const int f0 = (tid >> 6) * per_wave * 64 + (tid & 63);
    SlicePairs sp;
    slice_count(masked_ids, TK, N, f0, per_wave, pos, sp);
    int cnt = 0;
    if (tid < 256) {   // thread e: exclusive prefix of expert e's counts over the wavefronts
#pragma unroll
        for (int w = 0; w < kOneWgWaves; ++w) {
            const int c = pos[w][tid];
            pos[w][tid] = cnt;
            cnt += c;
        }
    }
    int total;
    const int excl = block_exclusive_scan_256(cnt, scratch, &total);
    if (tid < 256) {
#pragma unroll
        for (int w = 0; w < kOneWgWaves; ++w) pos[w][tid] += excl;
        if (tid < N) {
            counts[tid] = cnt;
            offsets[tid] = excl;
        }
    }
    if (tid == 0) {
        offsets[N] = total;
        *num_pairs = total;
    }
    emit_work_list(tid, N, cnt, excl, wl, scratch, longest_first != 0);
    __syncthreads();
    slice_place(sp, TK, f0, per_wave, total, pos, perm, inv_perm);
}

// More than one workgroup's worth of pairs: slices of 16 * per_wave groups, short ones while
// that keeps the slices few (the ballots that rank equal ids are scalar work, which the
// wavefronts of a compute unit do one after the other: many short slices on many compute
// units finish sooner than a few long ones).
static int slice_groups_per_wave(long TK) {
    int g = 2;
    while (g < kOneWgGroups && TK > 128L * 64 * kOneWgWaves * g) g *= 2;
    return g;
}

// First launch: slice_counts[slice][e] = kept pairs of expert e.
__global__ __launch_bounds__(64 * kOneWgWaves) void slice_count_kernel(
    const int32_t *__restrict__ masked_ids, int32_t *__restrict__ slice_counts, int TK, int N,
    int per_wave) {
    __shared__ int pos[kOneWgWaves][256];
    const int tid = threadIdx.x;
    const int f0 = (blockIdx.x * kOneWgWaves + (tid >> 6)) * per_wave * 64 + (tid & 63);
    SlicePairs sp;
    slice_count(masked_ids, TK, N, f0, per_wave, pos, sp);
    if (tid < N) {
        int cnt = 0;
#pragma unroll
        for (int w = 0; w < kOneWgWaves; ++w) cnt += pos[w][tid];
        slice_counts[(size_t)blockIdx.x * N + tid] = cnt;
    }
}

// Second launch, nslice + 1 workgroups.  Workgroup b < nslice places the pairs of slice b:
// thread e adds up expert e's counts over all slices (the expert's total) and over the
// slices before b, a scan of the totals gives the expert's first row, and the wavefronts'
// own counts, taken again from the ids, give every wavefront its first row inside that.
// Workgroup nslice reads no ids: it writes the per-expert arrays and the work list.
__global__ __launch_bounds__(64 * kOneWgWaves) void slice_scatter_kernel(
    const int32_t *__restrict__ masked_ids, const int32_t *__restrict__ slice_counts,
    int32_t *__restrict__ counts, int32_t *__restrict__ offsets, int32_t *__restrict__ perm,
    int32_t *__restrict__ inv_perm, int32_t *__restrict__ num_pairs, int TK, int N, int nslice,
    int per_wave, WorkList wl, int longest_first) {
    __shared__ int pos[kOneWgWaves][256];
    __shared__ int scratch[256];
    const int tid = threadIdx.x;
    const int b = blockIdx.x;
    const bool lister = b == nslice;   // uniform over the workgroup
    const int f0 = (b * kOneWgWaves + (tid >> 6)) * per_wave * 64 + (tid & 63);
    // the other slices' counts are requested first: their latency passes under the counting
    int cnt = 0, before = 0;
    if (tid < N) {
#pragma unroll 8
        for (int sl = 0; sl < nslice; ++sl) {
            const int c = slice_counts[(size_t)sl * N + tid];
            before += sl < b ? c : 0;
            cnt += c;
        }
    }
    SlicePairs sp;
    if (!lister) slice_count(masked_ids, TK, N, f0, per_wave, pos, sp);
    int total;
    const int excl = block_exclusive_scan_256(cnt, scratch, &total);
    if (lister) {
        if (tid < N) {
            counts[tid] = cnt;
            offsets[tid] = excl;
        }
        if (tid == 0) {
            offsets[N] = total;
            *num_pairs = total;
        }
        emit_work_list(tid, N, cnt, excl, wl, scratch, longest_first != 0);
        return;
    }
    if (tid < 256) {
        int run = excl + before;
#pragma unroll
        for (int w = 0; w < kOneWgWaves; ++w) {
            const int c = pos[w][tid];
            pos[w][tid] = run;
            run += c;
        }
    }
    __syncthreads();
    slice_place(sp, TK, f0, per_wave, total, pos, perm, inv_perm);
}

int permute_slices(long TK) {
    const long slice = 64L * kOneWgWaves * slice_groups_per_wave(TK);
    const long n = (TK + slice - 1) / slice;
    return n < 1 ? 1 : (int)n;
}

hipError_t launch_permute(const beam_shape &s, const int32_t *masked_ids, int32_t *counts,
                          int32_t *offsets, int32_t *perm, int32_t *inv_perm, int32_t *num_pairs,
                          int32_t *slice_counts, const WorkList &wl, hipStream_t st,
                          bool longest_first) {
    const int TK = s.T * s.K;
    const int lf = longest_first ? 1 : 0;
    if (TK <= kChunk) {
        permute_single_chunk_kernel<<<1, 256, 0, st>>>(masked_ids, counts, offsets, perm, inv_perm,
                                                       num_pairs, TK, s.N, wl);
        return hipGetLastError();
    }
    if (TK <= kOneWgMaxPairs) {
        permute_one_workgroup_kernel<<<1, 64 * kOneWgWaves, 0, st>>>(
            masked_ids, counts, offsets, perm, inv_perm, num_pairs, TK, s.N, wl, lf);
        return hipGetLastError();
    }
    const int nslice = permute_slices(TK);
    const int per_wave = slice_groups_per_wave(TK);
    slice_count_kernel<<<nslice, 64 * kOneWgWaves, 0, st>>>(masked_ids, slice_counts, TK, s.N,
                                                             per_wave);
    BEAM_CHECK_LAUNCH();
    slice_scatter_kernel<<<nslice + 1, 64 * kOneWgWaves, 0, st>>>(
        masked_ids, slice_counts, counts, offsets, perm, inv_perm, num_pairs, TK, s.N, nslice,
        per_wave, wl, lf);
    return hipGetLastError();
}

hipError_t launch_work_list(const beam_shape &s, const int32_t *offsets, const WorkList &wl,
                            hipStream_t st, bool longest_first) {
    const int lf = longest_first ? 1 : 0;
    work_list_kernel<<<1, 256, 0, st>>>(offsets, s.N, wl, lf);
    return hipGetLastError();
}

}  // namespace beam

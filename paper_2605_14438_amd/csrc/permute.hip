// Expert-wise grouping of the kept (token, expert) pairs (paper App. A.4: ids
// equal to -1 are skipped when tokens are grouped by expert).  A stable
// counting sort of the flat pair index f = t*K+k by expert id:
//   1. count    per chunk of kChunk pairs, an LDS histogram over experts
//   2. scan     per expert, exclusive prefix over chunks; then exclusive prefix
//               over experts; plus the work list the FFN kernels walk
//   3. scatter  every chunk re-reads its ids and places each kept pair at
//               offset[e] + base[chunk][e] + (rank among equal ids so far)
// Placement uses only prefix sums and wavefront ballots, never atomics on the
// destination, so the result is the same on every run.  When the whole input
// is one chunk (decode batches) the three steps run as one launch.
#include "common.hpp"

namespace beam {

// Lanes of the wavefront that hold the same id (ids < 256), restricted to
// valid lanes: eight ballots, one per id bit.
__device__ __forceinline__ uint64_t match_id(int id, bool valid) {
    uint64_t peers = __ballot(valid);
#pragma unroll
    for (int b = 0; b < 8; ++b) {
        const bool bit = (id >> b) & 1;
        const uint64_t m = __ballot(valid && bit);
        peers &= bit ? m : ~m;
    }
    return peers;
}

// Exclusive prefix sum over the first n (<= 256) entries held one per thread of
// a 256-thread workgroup; returns the exclusive value, *total gets the sum.
__device__ __forceinline__ int block_exclusive_scan_256(int v, int *scratch /*[256]*/, int *total) {
    const int tid = threadIdx.x;
    scratch[tid] = v;
    __syncthreads();
    for (int off = 1; off < 256; off <<= 1) {
        const int add = tid >= off ? scratch[tid - off] : 0;
        __syncthreads();
        scratch[tid] += add;
        __syncthreads();
    }
    const int incl = scratch[tid];
    *total = scratch[255];
    __syncthreads();
    return incl - v;
}

// One wavefront counts the kept pairs of one chunk per expert.
__global__ __launch_bounds__(64) void count_kernel(const int32_t *__restrict__ masked_ids,
                                                   int32_t *__restrict__ blk_counts, int TK,
                                                   int N) {
    __shared__ int hist[256];
    const int lane = threadIdx.x;
    for (int e = lane; e < 256; e += 64) hist[e] = 0;
    __syncthreads();
    const int f0 = blockIdx.x * kChunk;
#pragma unroll
    for (int gidx = 0; gidx < kGroupsPerChunk; ++gidx) {
        const int f = f0 + gidx * 64 + lane;
        const int id = f < TK ? masked_ids[f] : -1;
        const bool valid = id >= 0 && id < N;
        const uint64_t peers = match_id(id, valid);
        // the lowest lane of every group of equal ids adds the group size
        if (valid && (peers & ((1ull << lane) - 1ull)) == 0) hist[id] += __popcll(peers);
        __syncthreads();
    }
    for (int e = lane; e < N; e += 64) blk_counts[(size_t)blockIdx.x * N + e] = hist[e];
}

// Work list from the per-expert counts (thread e owns expert e; 256 threads).
__device__ __forceinline__ void emit_work_list(int e, int N, int count, int offset,
                                               const WorkList &wl, int *scratch) {
    int total;
    const int has = (e < N && count > 0) ? 1 : 0;
    const int slot = block_exclusive_scan_256(has, scratch, &total);
    if (has) wl.active[slot] = e;
    if (threadIdx.x == 0) wl.hdr[0] = total;
    const int ntile = (e < N) ? (count + kTileM - 1) / kTileM : 0;
    const int tbase = block_exclusive_scan_256(ntile, scratch, &total);
    for (int i = 0; i < ntile; ++i) {
        wl.tile_expert[tbase + i] = e;
        wl.tile_row0[tbase + i] = offset + i * kTileM;
    }
    if (threadIdx.x == 0) wl.hdr[1] = total;
}

__global__ __launch_bounds__(256) void scan_kernel(const int32_t *__restrict__ blk_counts,
                                                   int32_t *__restrict__ blk_base,
                                                   int32_t *__restrict__ counts,
                                                   int32_t *__restrict__ offsets,
                                                   int32_t *__restrict__ num_pairs, int nchunk,
                                                   int N, WorkList wl) {
    __shared__ int scratch[256];
    const int e = threadIdx.x;
    int run = 0;
    if (e < N) {
        for (int b = 0; b < nchunk; ++b) {
            const int c = blk_counts[(size_t)b * N + e];
            blk_base[(size_t)b * N + e] = run;
            run += c;
        }
        counts[e] = run;
    }
    int total;
    const int excl = block_exclusive_scan_256(e < N ? run : 0, scratch, &total);
    if (e < N) offsets[e] = excl;
    if (e == 0) {
        offsets[N] = total;
        *num_pairs = total;
    }
    emit_work_list(e, N, run, excl, wl, scratch);
}

// Work list alone, for callers that hand in expert_offsets directly.
__global__ __launch_bounds__(256) void work_list_kernel(const int32_t *__restrict__ offsets, int N,
                                                        WorkList wl) {
    __shared__ int scratch[256];
    const int e = threadIdx.x;
    int off = 0, cnt = 0;
    if (e < N) {
        off = offsets[e];
        cnt = offsets[e + 1] - off;
        if (cnt < 0) cnt = 0;
    }
    emit_work_list(e, N, cnt, off, wl, scratch);
}

__global__ __launch_bounds__(64) void scatter_kernel(const int32_t *__restrict__ masked_ids,
                                                     const int32_t *__restrict__ offsets,
                                                     const int32_t *__restrict__ blk_base,
                                                     int32_t *__restrict__ perm,
                                                     int32_t *__restrict__ inv_perm, int TK, int N) {
    __shared__ int run[256];
    const int lane = threadIdx.x;
    for (int e = lane; e < N; e += 64) run[e] = offsets[e] + blk_base[(size_t)blockIdx.x * N + e];
    __syncthreads();
    const int P = offsets[N];
    const int f0 = blockIdx.x * kChunk;
#pragma unroll
    for (int gidx = 0; gidx < kGroupsPerChunk; ++gidx) {
        const int f = f0 + gidx * 64 + lane;
        const int id = f < TK ? masked_ids[f] : -1;
        const bool valid = id >= 0 && id < N;
        const uint64_t peers = match_id(id, valid);
        const int rank = __popcll(peers & ((1ull << lane) - 1ull));
        const int base = valid ? run[id] : 0;
        __syncthreads();
        if (valid && rank == 0) run[id] = base + __popcll(peers);
        __syncthreads();
        if (f < TK) {
            if (valid) {
                perm[base + rank] = f;
                inv_perm[f] = base + rank;
            } else {
                inv_perm[f] = -1;
            }
            if (f >= P) perm[f] = -1;  // rows [P, T*K) carry no pair
        }
    }
}

// Decode batches: the whole pair list is one chunk.  One workgroup of 256
// threads does count, scan, work list and scatter; wavefront 0 walks the ids.
__global__ __launch_bounds__(256) void permute_single_chunk_kernel(
    const int32_t *__restrict__ masked_ids, int32_t *__restrict__ counts,
    int32_t *__restrict__ offsets, int32_t *__restrict__ perm, int32_t *__restrict__ inv_perm,
    int32_t *__restrict__ num_pairs, int TK, int N, WorkList wl) {
    __shared__ int hist[256];
    __shared__ int run[256];
    __shared__ int scratch[256];
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const bool walker = tid < 64;
    hist[tid] = 0;
    __syncthreads();
    int ids[kGroupsPerChunk];
    uint64_t peers[kGroupsPerChunk];
#pragma unroll
    for (int gidx = 0; gidx < kGroupsPerChunk; ++gidx) {
        ids[gidx] = -1;
        peers[gidx] = 0;
        if (walker) {
            const int f = gidx * 64 + lane;
            const int id = f < TK ? masked_ids[f] : -1;
            const bool valid = id >= 0 && id < N;
            ids[gidx] = valid ? id : -1;
            peers[gidx] = match_id(id, valid);
            if (valid && (peers[gidx] & ((1ull << lane) - 1ull)) == 0)
                hist[id] += __popcll(peers[gidx]);
        }
        __syncthreads();
    }
    const int cnt = tid < N ? hist[tid] : 0;
    int total;
    const int excl = block_exclusive_scan_256(cnt, scratch, &total);
    if (tid < N) {
        counts[tid] = cnt;
        offsets[tid] = excl;
    }
    if (tid == 0) {
        offsets[N] = total;
        *num_pairs = total;
    }
    run[tid] = excl;
    emit_work_list(tid, N, cnt, excl, wl, scratch);
    __syncthreads();
#pragma unroll
    for (int gidx = 0; gidx < kGroupsPerChunk; ++gidx) {
        const int f = gidx * 64 + lane;
        const bool valid = walker && ids[gidx] >= 0;
        const int rank = __popcll(peers[gidx] & ((1ull << lane) - 1ull));
        const int base = valid ? run[ids[gidx]] : 0;
        __syncthreads();
        if (valid && rank == 0) run[ids[gidx]] = base + __popcll(peers[gidx]);
        __syncthreads();
        if (walker && f < TK) {
            if (valid) {
                perm[base + rank] = f;
                inv_perm[f] = base + rank;
            } else {
                inv_perm[f] = -1;
            }
            if (f >= total) perm[f] = -1;
        }
    }
}

hipError_t launch_permute(const beam_shape &s, const int32_t *masked_ids, int32_t *counts,
                          int32_t *offsets, int32_t *perm, int32_t *inv_perm, int32_t *num_pairs,
                          int32_t *blk_counts, int32_t *blk_base, int nchunk, const WorkList &wl,
                          hipStream_t st) {
    const int TK = s.T * s.K;
    if (nchunk == 1) {
        permute_single_chunk_kernel<<<1, 256, 0, st>>>(masked_ids, counts, offsets, perm, inv_perm,
                                                       num_pairs, TK, s.N, wl);
        return hipGetLastError();
    }
    count_kernel<<<nchunk, 64, 0, st>>>(masked_ids, blk_counts, TK, s.N);
    scan_kernel<<<1, 256, 0, st>>>(blk_counts, blk_base, counts, offsets, num_pairs, nchunk, s.N,
                                   wl);
    scatter_kernel<<<nchunk, 64, 0, st>>>(masked_ids, offsets, blk_base, perm, inv_perm, TK, s.N);
    return hipGetLastError();
}

hipError_t launch_work_list(const beam_shape &s, const int32_t *offsets, const WorkList &wl,
                            hipStream_t st) {
    work_list_kernel<<<1, 256, 0, st>>>(offsets, s.N, wl);
    return hipGetLastError();
}

}  // namespace beam

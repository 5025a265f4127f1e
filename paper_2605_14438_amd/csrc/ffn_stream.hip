// GLU experts (paper Eq. 3, delta = SiLU) for decode-sized batches, bf16.
//
// With a handful of kept rows per expert the cost is reading each touched
// expert's weights from HBM once: 6*H*I bytes per expert against 6*H*I flops
// per row.  So the weights are the streamed operand: every wavefront owns 16
// (or 2x16) weight rows and pulls them through the MFMA A operand straight
// from global memory with 16-byte loads, while the few activation rows, which
// every workgroup of the same expert shares and which stay in L2, feed the B
// operand.  v_mfma_f32_16x16x32_bf16: D[i][j] = sum_k A[i][k] B[k][j] with
// A row i = weight row (output feature), B column j = grouped activation row.
//
//   lane l:  A/B row or column  l & 15,  k = 8*(l >> 4) .. +7 of each 32-step
//   D:       lane l, register r -> feature 4*(l >> 4) + r, activation row l & 15
//
// More than 16 rows in an expert loops over row tiles (weights re-read through
// L2); the tiled GEMM takes over when that becomes the common case.
#include "common.hpp"
#include "topk.hpp"

namespace beam {

// Packed expert weights are read once per pass, a whole 1 KiB fragment per load
// instruction, and never again soon: loading them with the non-temporal hint keeps
// them from being installed in the caches on their way through, which on this GPU
// raises a plain streaming read from 6.1 to 7.0 TB/s (decode layer from packed
// weights 123.7 -> 114.4 us).  Not for row-major weights: there one instruction
// takes half of each 128-byte line and the next one the other half, which the hint
// turns into two trips to memory (123.3 -> 130.6 us).  The activation rows, which
// every workgroup of an expert shares, keep the default policy.
typedef uint32_t u32x4w __attribute__((ext_vector_type(4)));
__device__ __forceinline__ u32x4w load_weights16v(const bf16_t *p) {
    return __builtin_nontemporal_load((const u32x4w *)p);
}

// Rows [row_beg, row_end) of the hidden activation for the 16 gate and 16 up
// features j0.. of expert e:  hidden[row, j] = bf16(SiLU(x_t . W_gate[j]) * (x_t . W_up[j])),
// t = token_of(row).  The workgroup's 4 wavefronts split the reduction over H.
// RT row tiles of 16 rows share one pass over the weights (RT = 2 for experts
// with more than 16 rows, a shared expert above all: one pass per 32 rows
// instead of two; RT = 4 would halve the occupancy of every workgroup).  red: LDS, 3 * 8 * RT * 64 floats.
template <int RT, typename TokenOf>
__device__ __forceinline__ void gate_up_rows(const bf16_t *__restrict__ x,
                                             const bf16_t *__restrict__ w_gate_up, int e,
                                             int row_beg, int row_end, TokenOf token_of,
                                             bf16_t *__restrict__ hidden, int H, int I, int j0,
                                             float *red) {
    const int lane = threadIdx.x & 63;
    const int ks = threadIdx.x >> 6;
    const int l16 = lane & 15;
    const int g = lane >> 4;
    const int klen = H >> 2;
    const int kbeg = ks * klen + g * 8;
    const bf16_t *gp = w_gate_up + ((size_t)e * 2 * I + j0 + l16) * H + kbeg;
    const bf16_t *up = gp + (size_t)I * H;
    auto red_at = [&](int s, int v, int l) -> float & { return red[(s * 8 * RT + v) * 64 + l]; };

    for (int row0 = row_beg; row0 < row_end; row0 += 16 * RT) {
        const bf16_t *xp[RT];
#pragma unroll
        for (int rt = 0; rt < RT; ++rt) {
            int row = row0 + rt * 16 + l16;
            row = row < row_end ? row : row_end - 1;
            xp[rt] = x + (size_t)token_of(row) * H + kbeg;
        }
        f32x4 ag[RT], au[RT];
#pragma unroll
        for (int rt = 0; rt < RT; ++rt) {
            ag[rt] = f32x4{0.f, 0.f, 0.f, 0.f};
            au[rt] = f32x4{0.f, 0.f, 0.f, 0.f};
        }
        // Software pipeline over chunks of 128 reduction indices: the loads of
        // chunk c+1 are issued before the MFMAs of chunk c, so a wavefront always
        // has 12 KB in flight.  sched_barrier keeps the compiler from sinking the
        // loads back behind the MFMAs to save registers.
        uint4 wg[2][4], wu[2][4], xv[2][RT][4];
        auto load = [&](int b, int k) {
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                wg[b][j] = *(const uint4 *)(gp + k + j * 32);
                wu[b][j] = *(const uint4 *)(up + k + j * 32);
            }
#pragma unroll
            for (int rt = 0; rt < RT; ++rt)
#pragma unroll
                for (int j = 0; j < 4; ++j) xv[b][rt][j] = *(const uint4 *)(xp[rt] + k + j * 32);
        };
        auto mma = [&](int b) {
#pragma unroll
            for (int j = 0; j < 4; ++j)
#pragma unroll
                for (int rt = 0; rt < RT; ++rt) {
                    ag[rt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(
                        __builtin_bit_cast(bf16x8, wg[b][j]),
                        __builtin_bit_cast(bf16x8, xv[b][rt][j]), ag[rt], 0, 0, 0);
                    au[rt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(
                        __builtin_bit_cast(bf16x8, wu[b][j]),
                        __builtin_bit_cast(bf16x8, xv[b][rt][j]), au[rt], 0, 0, 0);
                }
        };
        // steady state without conditionals, so the wait before each MFMA group
        // counts only the older chunk's loads; the last one or two chunks are peeled
        load(0, 0);
        int k = 0;
        for (; k + 256 < klen; k += 256) {
            load(1, k + 128);
            __builtin_amdgcn_sched_barrier(0);
            mma(0);
            __builtin_amdgcn_sched_barrier(0);
            load(0, k + 256);
            __builtin_amdgcn_sched_barrier(0);
            mma(1);
            __builtin_amdgcn_sched_barrier(0);
        }
        if (k + 128 < klen) {
            load(1, k + 128);
            __builtin_amdgcn_sched_barrier(0);
            mma(0);
            mma(1);
        } else {
            mma(0);
        }
        if (ks > 0) {
#pragma unroll
            for (int rt = 0; rt < RT; ++rt)
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                    red_at(ks - 1, rt * 8 + r, lane) = ag[rt][r];
                    red_at(ks - 1, rt * 8 + 4 + r, lane) = au[rt][r];
                }
        }
        __syncthreads();
        if (ks == 0) {
#pragma unroll
            for (int rt = 0; rt < RT; ++rt) {
#pragma unroll
                for (int s = 0; s < 3; ++s)
#pragma unroll
                    for (int r = 0; r < 4; ++r) {
                        ag[rt][r] += red_at(s, rt * 8 + r, lane);
                        au[rt][r] += red_at(s, rt * 8 + 4 + r, lane);
                    }
                const int row = row0 + rt * 16 + l16;
                if (row < row_end) {
                    uint32_t lo = (uint32_t)f32_to_bf16(silu(ag[rt][0]) * au[rt][0]) |
                                  ((uint32_t)f32_to_bf16(silu(ag[rt][1]) * au[rt][1]) << 16);
                    uint32_t hi = (uint32_t)f32_to_bf16(silu(ag[rt][2]) * au[rt][2]) |
                                  ((uint32_t)f32_to_bf16(silu(ag[rt][3]) * au[rt][3]) << 16);
                    *(uint2 *)(hidden + (size_t)row * I + j0 + g * 4) = make_uint2(lo, hi);
                }
            }
        }
        __syncthreads();
    }
}

// grid (I/16, max active experts): expert-sorted rows from the work list.
__global__ __launch_bounds__(256) void gate_up_stream_kernel(
    const bf16_t *__restrict__ x, const bf16_t *__restrict__ w_gate_up,
    const int32_t *__restrict__ perm, WorkList wl, bf16_t *__restrict__ hidden, int H, int K,
    int I, int want) {
    const int u = blockIdx.y;
    // one round trip: the words are independent loads.  Not the regime chosen on the
    // device: no active expert for this kernel, every workgroup leaves.
    const int n_active = (want != kRegimeAny && wl.hdr[2] != want) ? 0 : wl.hdr[0];
    const int e = wl.active[u];
    const int row_beg = wl.active_beg[u];
    const int row_end = wl.active_end[u];
    if (u >= n_active) return;
    __shared__ float red[3 * 8 * 2 * 64];
    auto token_of = [&](int row) { return perm[row] / K; };
    if (row_end - row_beg > 16)  // uniform over the workgroup
        gate_up_rows<2>(x, w_gate_up, e, row_beg, row_end, token_of, hidden, H, I,
                        blockIdx.x * 16, red);
    else
        gate_up_rows<1>(x, w_gate_up, e, row_beg, row_end, token_of, hidden, H, I,
                        blockIdx.x * 16, red);
}

// ---------------------------------------------------------------------------
// Tiny batches (T * slots <= kTinySlots, single-token decode above all): the layer is
// bound by the number of kernels, each a few microseconds of launch, drain and
// first-touch latency however little it does.  So the Top-K / mask / grouping
// kernels are dropped: every workgroup that needs a routing decision recomputes
// it from the logits (one wavefront, about a microsecond), pairs are addressed
// by their flat index f = t * slots + k instead of being sorted by expert, and
// the aggregation is folded into the down projection.  Three kernels instead of
// six.  An expert kept by two tokens is streamed twice, which at these sizes
// (about one pair per touched expert) costs less than a kernel does.
//
// gate_up_slot_kernel: grid (I/16, T * slots); hidden[f, :] for kept pair f.
// ---------------------------------------------------------------------------
template <int RULE>
__global__ __launch_bounds__(256) void gate_up_slot_kernel(
    const bf16_t *__restrict__ x, const bf16_t *__restrict__ w_gate_up,
    const float *__restrict__ router_logits, const float *__restrict__ mask_logits,
    const float *__restrict__ g_shared, float param, bf16_t *__restrict__ hidden, int H, int N,
    int K, int S, int I) {
    __shared__ float red[3 * 8 * 64];
    __shared__ int32_t ids_s[64], masked_s[64];
    __shared__ float w_s[64];
    const int slots = K + S;
    const int f = blockIdx.y;
    const int t = f / slots;
    if (threadIdx.x < 64)
        wave_route_token<RULE>(router_logits + (size_t)t * N, mask_logits + (size_t)t * N, nullptr,
                               nullptr, N, K, S, (S > 0 && g_shared) ? g_shared[t] : 1.0f, param,
                               ids_s, w_s, masked_s);
    __syncthreads();
    const int e = masked_s[f - t * slots];
    if (e < 0) return;  // uniform over the workgroup
    gate_up_rows<1>(x, w_gate_up, e, f, f + 1, [&](int) { return t; }, hidden, H, I,
                    blockIdx.x * 16, red);
}

// down_combine_token_kernel: grid (H / (16*FT), T); a workgroup owns 16*FT
// output features of one token.  out[t, c] = (h[t, c] +) sum over the token's kept
// slots, in slot order, of g_k * (hidden[f_k, :] . W_down[e_k][c, :]).  The four
// wavefronts take the kept slots round-robin (each runs the reduction of
// down_stream_kernel for its slot) and park the fp32 results in LDS; wavefront 0
// then adds them up in slot order, exactly the running sum of the combine kernel,
// and rounds once.  Every wavefront recomputes the token's routing; workgroup 0
// of a token also reports it.
template <int FT, int RULE>
__global__ __launch_bounds__(256) void down_combine_token_kernel(
    const bf16_t *__restrict__ hidden, const bf16_t *__restrict__ w_down,
    const float *__restrict__ router_logits, const float *__restrict__ mask_logits,
    const float *__restrict__ g_shared, float param, const bf16_t *__restrict__ residual,
    bf16_t *__restrict__ out, int32_t *__restrict__ topk_ids_opt, float *__restrict__ topk_w_opt,
    int32_t *__restrict__ masked_ids_opt, int32_t *__restrict__ num_pairs_opt, int H, int N, int K,
    int S, int I) {
    __shared__ int32_t ids_s[4][64], masked_s[4][64];
    __shared__ float w_s[4][64];
    __shared__ float y_s[64][FT][4][4];  // [kept slot ordinal][tile][feature group g][r]
    const int slots = K + S;
    const int t = blockIdx.y;
    const int lane = threadIdx.x & 63;
    const int wave = threadIdx.x >> 6;
    const int l16 = lane & 15;
    const int g = lane >> 4;
    wave_route_token<RULE>(router_logits + (size_t)t * N, mask_logits + (size_t)t * N, nullptr,
                           nullptr, N, K, S, (S > 0 && g_shared) ? g_shared[t] : 1.0f, param,
                           ids_s[wave], w_s[wave], masked_s[wave]);
    __builtin_amdgcn_wave_barrier();  // a wavefront reads back only its own copy
    const bool in = lane < slots;
    const uint64_t kept = __ballot(in && masked_s[wave][in ? lane : 0] >= 0);
    if (blockIdx.x == 0 && wave == 0) {
        const size_t f = (size_t)t * slots + lane;
        if (in && topk_ids_opt) topk_ids_opt[f] = ids_s[0][lane];
        if (in && topk_w_opt) topk_w_opt[f] = w_s[0][lane];
        if (in && masked_ids_opt) masked_ids_opt[f] = masked_s[0][lane];
        // the logits kernel of this call has zeroed the counter
        if (num_pairs_opt && lane == 0) atomicAdd(num_pairs_opt, __popcll(kept));
    }
    const int c0 = blockIdx.x * (16 * FT);
    const bf16_t *wrow[FT];
#pragma unroll
    for (int f = 0; f < FT; ++f) {
        int c = c0 + f * 16 + l16;
        c = c < H ? c : H - 1;
        wrow[f] = w_down + (size_t)c * I + g * 8;
    }
    // One or two kept slots and a long reduction: the wavefronts that would idle take
    // parts of the reduction (four parts of one slot, two of each of two), added in order
    // below; a short reduction stays whole and bit-identical to the staged path.
    const int nkept = __popcll(kept);
    int parts = 1;
    if (I >= 4096 && nkept >= 1 && nkept <= 2 && I % ((4 / nkept) * 128) == 0) parts = 4 / nkept;
    const int len = I / parts;
    int ord = 0;
    for (uint64_t m = kept; m; m &= m - 1, ++ord) {
        int part = 0;
        if (parts == 1) {
            if ((ord & 3) != wave) continue;  // wave-uniform
        } else {
            if (wave % nkept != ord) continue;
            part = wave / nkept;
        }
        const int k = __builtin_ctzll(m);
        const int e = masked_s[wave][k];
        const bf16_t *hp = hidden + ((size_t)t * slots + k) * I + g * 8 + part * len;
        const size_t eoff = (size_t)e * H * I + (size_t)part * len;
        f32x4 acc[FT];
#pragma unroll
        for (int f = 0; f < FT; ++f) acc[f] = f32x4{0.f, 0.f, 0.f, 0.f};
        // same two-deep software pipeline as the streaming kernels
        uint4 w[2][FT][4], hv[2][4];
        auto load = [&](int b, int kk) {
#pragma unroll
            for (int j = 0; j < 4; ++j) {
#pragma unroll
                for (int f = 0; f < FT; ++f)
                    w[b][f][j] = *(const uint4 *)(wrow[f] + eoff + kk + j * 32);
                hv[b][j] = *(const uint4 *)(hp + kk + j * 32);
            }
        };
        auto mma = [&](int b) {
#pragma unroll
            for (int j = 0; j < 4; ++j)
#pragma unroll
                for (int f = 0; f < FT; ++f)
                    acc[f] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(
                        __builtin_bit_cast(bf16x8, w[b][f][j]), __builtin_bit_cast(bf16x8, hv[b][j]),
                        acc[f], 0, 0, 0);
        };
        load(0, 0);
        int kk = 0;
        for (; kk + 256 < len; kk += 256) {
            load(1, kk + 128);
            __builtin_amdgcn_sched_barrier(0);
            mma(0);
            __builtin_amdgcn_sched_barrier(0);
            load(0, kk + 256);
            __builtin_amdgcn_sched_barrier(0);
            mma(1);
            __builtin_amdgcn_sched_barrier(0);
        }
        if (kk + 128 < len) {
            load(1, kk + 128);
            __builtin_amdgcn_sched_barrier(0);
            mma(0);
            mma(1);
        } else {
            mma(0);
        }
        // every column of the MFMA result is the same hidden row: lanes with l16 == 0
        // hold features 4*g .. 4*g+3 of each tile
        if (l16 == 0) {
#pragma unroll
            for (int f = 0; f < FT; ++f)
#pragma unroll
                for (int r = 0; r < 4; ++r) y_s[ord * parts + part][f][g][r] = acc[f][r];
        }
    }
    __syncthreads();
    if (wave == 0 && l16 == 0) {
#pragma unroll
        for (int f = 0; f < FT; ++f) {
            const int c = c0 + f * 16 + g * 4;
            if (c >= H) continue;
            float tot[4] = {0.f, 0.f, 0.f, 0.f};
            if (residual) {
                const uint2 q = *(const uint2 *)(residual + (size_t)t * H + c);
                tot[0] = __uint_as_float(q.x << 16);
                tot[1] = __uint_as_float(q.x & 0xffff0000u);
                tot[2] = __uint_as_float(q.y << 16);
                tot[3] = __uint_as_float(q.y & 0xffff0000u);
            }
            int j = 0;
            for (uint64_t m = kept; m; m &= m - 1, ++j) {
                const float gk = w_s[0][__builtin_ctzll(m)];
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                    float y = y_s[j * parts][f][g][r];
                    for (int p = 1; p < parts; ++p) y += y_s[j * parts + p][f][g][r];
                    tot[r] = fmaf(gk, y, tot[r]);
                }
            }
            uint2 q;
            q.x = (uint32_t)f32_to_bf16(tot[0]) | ((uint32_t)f32_to_bf16(tot[1]) << 16);
            q.y = (uint32_t)f32_to_bf16(tot[2]) | ((uint32_t)f32_to_bf16(tot[3]) << 16);
            *(uint2 *)(out + (size_t)t * H + c) = q;
        }
    }
}

// y_pairs[row, c] = hidden[row, :] . W_down[c, :]
// grid (H / (64*FT), max active experts); each wavefront owns FT tiles of 16
// output features and runs the whole reduction over I.
// rows [row_beg, row_end) of expert e, RT row tiles of 16 per pass over the weights
template <int FT, int RT>
__device__ __forceinline__ void down_rows(const bf16_t *__restrict__ hidden,
                                          const bf16_t *const (&wp)[FT], int row_beg, int row_end,
                                          float *__restrict__ y_pairs, int H, int I, int c0) {
    const int lane = threadIdx.x & 63;
    const int l16 = lane & 15;
    const int g = lane >> 4;
    for (int row0 = row_beg; row0 < row_end; row0 += 16 * RT) {
        const bf16_t *hp[RT];
#pragma unroll
        for (int rt = 0; rt < RT; ++rt) {
            int row = row0 + rt * 16 + l16;
            row = row < row_end ? row : row_end - 1;
            hp[rt] = hidden + (size_t)row * I + g * 8;
        }
        f32x4 acc[RT][FT];
#pragma unroll
        for (int rt = 0; rt < RT; ++rt)
#pragma unroll
            for (int f = 0; f < FT; ++f) acc[rt][f] = f32x4{0.f, 0.f, 0.f, 0.f};
        // same two-deep software pipeline as the gate/up kernel
        uint4 w[2][FT][4], hv[2][RT][4];
        auto load = [&](int b, int k) {
#pragma unroll
            for (int j = 0; j < 4; ++j) {
#pragma unroll
                for (int f = 0; f < FT; ++f) w[b][f][j] = *(const uint4 *)(wp[f] + k + j * 32);
#pragma unroll
                for (int rt = 0; rt < RT; ++rt) hv[b][rt][j] = *(const uint4 *)(hp[rt] + k + j * 32);
            }
        };
        auto mma = [&](int b) {
#pragma unroll
            for (int j = 0; j < 4; ++j)
#pragma unroll
                for (int rt = 0; rt < RT; ++rt)
#pragma unroll
                    for (int f = 0; f < FT; ++f)
                        acc[rt][f] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(
                            __builtin_bit_cast(bf16x8, w[b][f][j]),
                            __builtin_bit_cast(bf16x8, hv[b][rt][j]), acc[rt][f], 0, 0, 0);
        };
        // steady state without conditionals, so the wait before each MFMA group
        // counts only the older chunk's loads; the last one or two chunks are peeled
        load(0, 0);
        int k = 0;
        for (; k + 256 < I; k += 256) {
            load(1, k + 128);
            __builtin_amdgcn_sched_barrier(0);
            mma(0);
            __builtin_amdgcn_sched_barrier(0);
            load(0, k + 256);
            __builtin_amdgcn_sched_barrier(0);
            mma(1);
            __builtin_amdgcn_sched_barrier(0);
        }
        if (k + 128 < I) {
            load(1, k + 128);
            __builtin_amdgcn_sched_barrier(0);
            mma(0);
            mma(1);
        } else {
            mma(0);
        }
#pragma unroll
        for (int rt = 0; rt < RT; ++rt) {
            const int row = row0 + rt * 16 + l16;
            if (row < row_end) {
#pragma unroll
                for (int f = 0; f < FT; ++f) {
                    const int c = c0 + f * 16 + g * 4;
                    if (c < H)
                        *(float4 *)(y_pairs + (size_t)row * H + c) = make_float4(
                            acc[rt][f][0], acc[rt][f][1], acc[rt][f][2], acc[rt][f][3]);
                }
            }
        }
    }
}

template <int FT>
__global__ __launch_bounds__(256) void down_stream_kernel(
    const bf16_t *__restrict__ hidden, const bf16_t *__restrict__ w_down, WorkList wl,
    float *__restrict__ y_pairs, int H, int I, int want) {
    const int u = blockIdx.y;
    const int n_active = (want != kRegimeAny && wl.hdr[2] != want) ? 0 : wl.hdr[0];
    const int e = wl.active[u];
    const int row_beg = wl.active_beg[u];
    const int row_end = wl.active_end[u];
    if (u >= n_active) return;
    const int lane = threadIdx.x & 63;
    const int wave = threadIdx.x >> 6;
    const int l16 = lane & 15;
    const int g = lane >> 4;
    const int c0 = (blockIdx.x * 4 + wave) * (16 * FT);
    if (c0 >= H) return;
    const bf16_t *wp[FT];
#pragma unroll
    for (int f = 0; f < FT; ++f) {
        int c = c0 + f * 16 + l16;
        c = c < H ? c : H - 1;
        wp[f] = w_down + ((size_t)e * H + c) * I + g * 8;
    }
    if (row_end - row_beg > 16)  // uniform over the workgroup
        down_rows<FT, 2>(hidden, wp, row_beg, row_end, y_pairs, H, I, c0);
    else
        down_rows<FT, 1>(hidden, wp, row_beg, row_end, y_pairs, H, I, c0);
}

// ---------------------------------------------------------------------------
// The same two streaming kernels for BEAM_WEIGHTS_PACKED (a server keeps one
// copy of the weights, packed for prefill, and decodes from it too).  The packed
// order is the A operand of v_mfma_f32_32x32x16_bf16: one fully coalesced 1 KiB
// load per 32 weight rows x 16 reduction indices.
//   A/B lane l: row/column l & 31, k = 8*(l >> 5)..+7
//   D register r of lane l: feature 8*(r >> 2) + 4*(l >> 5) + (r & 3),
//                           activation row l & 31
// so up to 32 activation rows share a pass and a lane ends up with runs of four
// consecutive features of its row.
// ---------------------------------------------------------------------------
typedef uint32_t u32x4s __attribute__((ext_vector_type(4)));
// MFMA k-steps (16 indices each) per pipeline chunk: 8 for the down kernel; 4 for
// gate/up, whose two weight streams would otherwise take every register and
// leave one workgroup per CU
constexpr int kPackedChunk = 8;
constexpr int kGateUpPackedChunk = 4;

// hidden rows [row_beg, row_end) x the 32 features of block q of expert e; the 4
// wavefronts share the reduction over H, chunk by chunk in turn (measured against four
// contiguous quarters, Qwen3-shaped decode layer at T = 64: this kernel 66.9 -> 59.7 us,
// 0.74 -> 0.83 of the HBM peak; with eight read points per workgroup instead of two the
// chip kept four times as many streams open in DRAM).  red: LDS, 3 * 32 * 64 floats.
// STREAM: weights with the non-temporal hint (not for the single-token kernels, where
// it measured 2 us slower per layer: a handful of workgroups, nothing to displace).
template <int CH, bool STREAM, typename TokenOf>
__device__ __forceinline__ void gate_up_rows_packed(const bf16_t *__restrict__ x,
                                                    const bf16_t *__restrict__ w_gate_up, int e,
                                                    int row_beg, int row_end, TokenOf token_of,
                                                    bf16_t *__restrict__ hidden, int H, int I,
                                                    int q, float *red) {
    const int lane = threadIdx.x & 63;
    const int ks4 = threadIdx.x >> 6;
    const int l32 = lane & 31;
    const int kh = lane >> 5;
    const int ksteps = H >> 4;
    const int kper = ksteps >> 2;  // k-steps of this wavefront
    // The wavefronts take the chunks of CH k-steps in turn (wavefront w: chunks w, w + 4,
    // ...), so the workgroup reads each of its two row blocks as one sequential stream
    // instead of four streams a quarter of the block apart.
    const int k0 = ks4 * CH;
    // blocks 2q (gate) and 2q + 1 (up) of this expert's 2I/32 row blocks
    const bf16_t *gp =
        w_gate_up + (((size_t)e * ((2 * I) >> 5) + 2 * q) * ksteps + k0) * 512 + lane * 8;
    const bf16_t *up = gp + (size_t)ksteps * 512;

    for (int row0 = row_beg; row0 < row_end; row0 += 32) {
        int row = row0 + l32;
        row = row < row_end ? row : row_end - 1;
        const bf16_t *xp = x + (size_t)token_of(row) * H + k0 * 16 + kh * 8;
        f32x16 ag, au;
#pragma unroll
        for (int r = 0; r < 16; ++r) ag[r] = au[r] = 0.0f;
        u32x4s wg[2][CH], wu[2][CH], xv[2][CH];
        auto load = [&](int b, int k) {
#pragma unroll
            for (int j = 0; j < CH; ++j) {
                if constexpr (STREAM) {
                    wg[b][j] = load_weights16v(gp + (size_t)(4 * k + j) * 512);
                    wu[b][j] = load_weights16v(up + (size_t)(4 * k + j) * 512);
                } else {
                    wg[b][j] = *(const u32x4s *)(gp + (size_t)(4 * k + j) * 512);
                    wu[b][j] = *(const u32x4s *)(up + (size_t)(4 * k + j) * 512);
                }
            }
#pragma unroll
            for (int j = 0; j < CH; ++j) xv[b][j] = *(const u32x4s *)(xp + (4 * k + j) * 16);
        };
        auto mma = [&](int b) {
#pragma unroll
            for (int j = 0; j < CH; ++j) {
                ag = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, wg[b][j]),
                                                             __builtin_bit_cast(bf16x8, xv[b][j]),
                                                             ag, 0, 0, 0);
                au = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, wu[b][j]),
                                                             __builtin_bit_cast(bf16x8, xv[b][j]),
                                                             au, 0, 0, 0);
            }
        };
        // two chunks in flight, steady state without conditionals (see gate_up_rows)
        load(0, 0);
        int k = 0;
        for (; k + 2 * CH < kper; k += 2 * CH) {
            load(1, k + CH);
            __builtin_amdgcn_sched_barrier(0);
            mma(0);
            __builtin_amdgcn_sched_barrier(0);
            load(0, k + 2 * CH);
            __builtin_amdgcn_sched_barrier(0);
            mma(1);
            __builtin_amdgcn_sched_barrier(0);
        }
        if (k + CH < kper) {
            load(1, k + CH);
            __builtin_amdgcn_sched_barrier(0);
            mma(0);
            mma(1);
        } else {
            mma(0);
        }
        if (ks4 > 0) {
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                red[((ks4 - 1) * 32 + r) * 64 + lane] = ag[r];
                red[((ks4 - 1) * 32 + 16 + r) * 64 + lane] = au[r];
            }
        }
        __syncthreads();
        if (ks4 == 0) {
#pragma unroll
            for (int s = 0; s < 3; ++s)
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    ag[r] += red[(s * 32 + r) * 64 + lane];
                    au[r] += red[(s * 32 + 16 + r) * 64 + lane];
                }
            if (row0 + l32 < row_end) {
                bf16_t *orow = hidden + (size_t)(row0 + l32) * I + q * 32 + kh * 4;
#pragma unroll
                for (int rg = 0; rg < 4; ++rg) {
                    const int r = rg * 4;
                    const uint32_t lo = (uint32_t)f32_to_bf16(silu(ag[r]) * au[r]) |
                                        ((uint32_t)f32_to_bf16(silu(ag[r + 1]) * au[r + 1]) << 16);
                    const uint32_t hi = (uint32_t)f32_to_bf16(silu(ag[r + 2]) * au[r + 2]) |
                                        ((uint32_t)f32_to_bf16(silu(ag[r + 3]) * au[r + 3]) << 16);
                    *(uint2 *)(orow + rg * 8) = make_uint2(lo, hi);
                }
            }
        }
        __syncthreads();
    }
}

// grid (I/32, max active experts)
__global__ __launch_bounds__(256, 2) void gate_up_stream_packed_kernel(
    const bf16_t *__restrict__ x, const bf16_t *__restrict__ w_gate_up,
    const int32_t *__restrict__ perm, WorkList wl, bf16_t *__restrict__ hidden, int H, int K,
    int I, int want) {
    const int u = blockIdx.y;
    const int n_active = (want != kRegimeAny && wl.hdr[2] != want) ? 0 : wl.hdr[0];
    const int e = wl.active[u];
    const int row_beg = wl.active_beg[u];
    const int row_end = wl.active_end[u];
    if (u >= n_active) return;
    __shared__ float red[3 * 32 * 64];
    gate_up_rows_packed<kGateUpPackedChunk, true>(x, w_gate_up, e, row_beg, row_end,
                                            [&](int row) { return perm[row] / K; }, hidden, H, I,
                                            blockIdx.x, red);
}

// y rows [row_beg, row_end) x the 32 output features of row block rb of expert e;
// one wavefront runs the whole reduction over I.
__device__ __forceinline__ void down_rows_packed(const bf16_t *__restrict__ hidden,
                                                 const bf16_t *__restrict__ w_down, int e, int rb,
                                                 int row_beg, int row_end,
                                                 float *__restrict__ y_pairs, int H, int I) {
    constexpr int CH = kPackedChunk;
    const int lane = threadIdx.x & 63;
    const int l32 = lane & 31;
    const int kh = lane >> 5;
    const int ksteps = I >> 4;
    const bf16_t *wp = w_down + (((size_t)e * (H >> 5) + rb) * ksteps) * 512 + lane * 8;
    for (int row0 = row_beg; row0 < row_end; row0 += 32) {
        int row = row0 + l32;
        row = row < row_end ? row : row_end - 1;
        const bf16_t *hp = hidden + (size_t)row * I + kh * 8;
        f32x16 acc;
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[r] = 0.0f;
        u32x4s w[2][CH], hv[2][CH];
        auto load = [&](int b, int k) {
#pragma unroll
            for (int j = 0; j < CH; ++j) {
                w[b][j] = load_weights16v(wp + (size_t)(k + j) * 512);
                hv[b][j] = *(const u32x4s *)(hp + (k + j) * 16);
            }
        };
        auto mma = [&](int b) {
#pragma unroll
            for (int j = 0; j < CH; ++j)
                acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, w[b][j]),
                                                              __builtin_bit_cast(bf16x8, hv[b][j]),
                                                              acc, 0, 0, 0);
        };
        load(0, 0);
        int k = 0;
        for (; k + 2 * CH < ksteps; k += 2 * CH) {
            load(1, k + CH);
            __builtin_amdgcn_sched_barrier(0);
            mma(0);
            __builtin_amdgcn_sched_barrier(0);
            load(0, k + 2 * CH);
            __builtin_amdgcn_sched_barrier(0);
            mma(1);
            __builtin_amdgcn_sched_barrier(0);
        }
        if (k + CH < ksteps) {
            load(1, k + CH);
            __builtin_amdgcn_sched_barrier(0);
            mma(0);
            mma(1);
        } else {
            mma(0);
        }
        if (row0 + l32 < row_end) {
            float *orow = y_pairs + (size_t)(row0 + l32) * H + rb * 32 + kh * 4;
#pragma unroll
            for (int rg = 0; rg < 4; ++rg)
                *(float4 *)(orow + rg * 8) = make_float4(acc[rg * 4], acc[rg * 4 + 1],
                                                         acc[rg * 4 + 2], acc[rg * 4 + 3]);
        }
    }
}

// grid (H/128, max active experts): each wavefront one block of 32 output features
__global__ __launch_bounds__(256) void down_stream_packed_kernel(
    const bf16_t *__restrict__ hidden, const bf16_t *__restrict__ w_down, WorkList wl,
    float *__restrict__ y_pairs, int H, int I, int want) {
    const int u = blockIdx.y;
    const int n_active = (want != kRegimeAny && wl.hdr[2] != want) ? 0 : wl.hdr[0];
    const int e = wl.active[u];
    const int row_beg = wl.active_beg[u];
    const int row_end = wl.active_end[u];
    if (u >= n_active) return;
    const int rb = blockIdx.x * 4 + (threadIdx.x >> 6);
    if (rb * 32 >= H) return;
    down_rows_packed(hidden, w_down, e, rb, row_beg, row_end, y_pairs, H, I);
}

// The tiny-batch kernels (see gate_up_slot_kernel) for packed weights.
// grid (I/32, T * slots)
template <int RULE>
__global__ __launch_bounds__(256, 2) void gate_up_slot_packed_kernel(
    const bf16_t *__restrict__ x, const bf16_t *__restrict__ w_gate_up,
    const float *__restrict__ router_logits, const float *__restrict__ mask_logits,
    const float *__restrict__ g_shared, float param, bf16_t *__restrict__ hidden, int H, int N,
    int K, int S, int I) {
    __shared__ float red[3 * 32 * 64];
    __shared__ int32_t ids_s[64], masked_s[64];
    __shared__ float w_s[64];
    const int slots = K + S;
    const int f = blockIdx.y;
    const int t = f / slots;
    if (threadIdx.x < 64)
        wave_route_token<RULE>(router_logits + (size_t)t * N, mask_logits + (size_t)t * N, nullptr,
                               nullptr, N, K, S, (S > 0 && g_shared) ? g_shared[t] : 1.0f, param,
                               ids_s, w_s, masked_s);
    __syncthreads();
    const int e = masked_s[f - t * slots];
    if (e < 0) return;  // uniform over the workgroup
    gate_up_rows_packed<kGateUpPackedChunk, false>(x, w_gate_up, e, f, f + 1, [&](int) { return t; },
                                            hidden, H, I, blockIdx.x, red);
}

// grid (H/32, T): a workgroup owns one block of 32 output features of one token;
// otherwise as down_combine_token_kernel.  Every column of the MFMA result is the
// same hidden row, so lanes 0 and 32 hold the 32 features between them.
template <int RULE>
__global__ __launch_bounds__(256) void down_combine_token_packed_kernel(
    const bf16_t *__restrict__ hidden, const bf16_t *__restrict__ w_down,
    const float *__restrict__ router_logits, const float *__restrict__ mask_logits,
    const float *__restrict__ g_shared, float param, const bf16_t *__restrict__ residual,
    bf16_t *__restrict__ out, int32_t *__restrict__ topk_ids_opt, float *__restrict__ topk_w_opt,
    int32_t *__restrict__ masked_ids_opt, int32_t *__restrict__ num_pairs_opt, int H, int N, int K,
    int S, int I) {
    constexpr int CH = kPackedChunk;
    __shared__ int32_t ids_s[4][64], masked_s[4][64];
    __shared__ float w_s[4][64];
    __shared__ float y_s[64][2][16];  // [kept slot ordinal][lane half][register]
    const int slots = K + S;
    const int t = blockIdx.y;
    const int rb = blockIdx.x;
    const int lane = threadIdx.x & 63;
    const int wave = threadIdx.x >> 6;
    const int l32 = lane & 31;
    const int kh = lane >> 5;
    wave_route_token<RULE>(router_logits + (size_t)t * N, mask_logits + (size_t)t * N, nullptr,
                           nullptr, N, K, S, (S > 0 && g_shared) ? g_shared[t] : 1.0f, param,
                           ids_s[wave], w_s[wave], masked_s[wave]);
    __builtin_amdgcn_wave_barrier();  // a wavefront reads back only its own copy
    const bool in = lane < slots;
    const uint64_t kept = __ballot(in && masked_s[wave][in ? lane : 0] >= 0);
    if (blockIdx.x == 0 && wave == 0) {
        const size_t f = (size_t)t * slots + lane;
        if (in && topk_ids_opt) topk_ids_opt[f] = ids_s[0][lane];
        if (in && topk_w_opt) topk_w_opt[f] = w_s[0][lane];
        if (in && masked_ids_opt) masked_ids_opt[f] = masked_s[0][lane];
        // the logits kernel of this call has zeroed the counter
        if (num_pairs_opt && lane == 0) atomicAdd(num_pairs_opt, __popcll(kept));
    }
    const int ksteps = I >> 4;
    // One or two kept slots and a long reduction (a few experts with a wide FFN): the
    // wavefronts that would idle take parts of the reduction instead, four parts of one
    // slot or two parts of each of two; the parts are added in order below.  (A short
    // reduction stays whole, which keeps this path bit-identical to the staged one there.)
    const int nkept = __popcll(kept);
    int parts = 1;
    if (I >= 4096 && nkept >= 1 && nkept <= 2 && ksteps % ((4 / nkept) * CH) == 0) parts = 4 / nkept;
    const int len = ksteps / parts;
    int ord = 0;
    for (uint64_t m = kept; m; m &= m - 1, ++ord) {
        int part = 0;
        if (parts == 1) {
            if ((ord & 3) != wave) continue;  // wave-uniform
        } else {
            if (wave % nkept != ord) continue;
            part = wave / nkept;
        }
        const int k = __builtin_ctzll(m);
        const int e = masked_s[wave][k];
        const bf16_t *hp = hidden + ((size_t)t * slots + k) * I + kh * 8 + (size_t)part * len * 16;
        const bf16_t *wp = w_down + (((size_t)e * (H >> 5) + rb) * ksteps + (size_t)part * len) * 512 +
                           lane * 8;
        f32x16 acc;
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[r] = 0.0f;
        u32x4s w[2][CH], hv[2][CH];
        auto load = [&](int b, int kk) {
#pragma unroll
            for (int j = 0; j < CH; ++j) {
                w[b][j] = *(const u32x4s *)(wp + (size_t)(kk + j) * 512);
                hv[b][j] = *(const u32x4s *)(hp + (kk + j) * 16);
            }
        };
        auto mma = [&](int b) {
#pragma unroll
            for (int j = 0; j < CH; ++j)
                acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, w[b][j]),
                                                              __builtin_bit_cast(bf16x8, hv[b][j]),
                                                              acc, 0, 0, 0);
        };
        load(0, 0);
        int kk = 0;
        for (; kk + 2 * CH < len; kk += 2 * CH) {
            load(1, kk + CH);
            __builtin_amdgcn_sched_barrier(0);
            mma(0);
            __builtin_amdgcn_sched_barrier(0);
            load(0, kk + 2 * CH);
            __builtin_amdgcn_sched_barrier(0);
            mma(1);
            __builtin_amdgcn_sched_barrier(0);
        }
        if (kk + CH < len) {
            load(1, kk + CH);
            __builtin_amdgcn_sched_barrier(0);
            mma(0);
            mma(1);
        } else {
            mma(0);
        }
        if (l32 == 0) {
#pragma unroll
            for (int r = 0; r < 16; ++r) y_s[ord * parts + part][kh][r] = acc[r];
        }
    }
    __syncthreads();
    if (wave == 0 && l32 == 0) {
        // register 4*rg + i of lane half kh is feature 8*rg + 4*kh + i of the block
        const size_t base = (size_t)t * H + rb * 32 + kh * 4;
#pragma unroll
        for (int rg = 0; rg < 4; ++rg) {
            float tot[4] = {0.f, 0.f, 0.f, 0.f};
            if (residual) {
                const uint2 q = *(const uint2 *)(residual + base + rg * 8);
                tot[0] = __uint_as_float(q.x << 16);
                tot[1] = __uint_as_float(q.x & 0xffff0000u);
                tot[2] = __uint_as_float(q.y << 16);
                tot[3] = __uint_as_float(q.y & 0xffff0000u);
            }
            int j = 0;
            for (uint64_t m = kept; m; m &= m - 1, ++j) {
                const float gk = w_s[0][__builtin_ctzll(m)];
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    float y = y_s[j * parts][kh][rg * 4 + i];
                    for (int p = 1; p < parts; ++p) y += y_s[j * parts + p][kh][rg * 4 + i];
                    tot[i] = fmaf(gk, y, tot[i]);
                }
            }
            uint2 q;
            q.x = (uint32_t)f32_to_bf16(tot[0]) | ((uint32_t)f32_to_bf16(tot[1]) << 16);
            q.y = (uint32_t)f32_to_bf16(tot[2]) | ((uint32_t)f32_to_bf16(tot[3]) << 16);
            *(uint2 *)(out + base + rg * 8) = q;
        }
    }
}

bool stream_ffn_supported(const beam_shape &s) {
    return s.dtype == BEAM_BF16 && s.H % 512 == 0 && s.I % 128 == 0;
}

static int max_active(const beam_shape &s) {
    const long TK = (long)s.T * s.K;
    return (int)(TK < s.N ? TK : s.N);
}

hipError_t launch_gate_up_stream(const beam_shape &s, const void *x, const void *w_gate_up,
                                 const int32_t *offsets, const int32_t *perm, const WorkList &wl,
                                 void *hidden, hipStream_t st, int want) {
    (void)offsets;
    if (s.weight_layout == BEAM_WEIGHTS_PACKED)
        gate_up_stream_packed_kernel<<<dim3(s.I / 32, max_active(s)), 256, 0, st>>>(
            (const bf16_t *)x, (const bf16_t *)w_gate_up, perm, wl, (bf16_t *)hidden, s.H, s.K,
            s.I, want);
    else
        gate_up_stream_kernel<<<dim3(s.I / 16, max_active(s)), 256, 0, st>>>(
            (const bf16_t *)x, (const bf16_t *)w_gate_up, perm, wl, (bf16_t *)hidden, s.H, s.K,
            s.I, want);
    return hipGetLastError();
}

hipError_t launch_down_stream(const beam_shape &s, const void *hidden, const void *w_down,
                              const int32_t *offsets, const WorkList &wl, float *y_pairs,
                              hipStream_t st, int want) {
    constexpr int FT = 2;
    (void)offsets;
    if (s.weight_layout == BEAM_WEIGHTS_PACKED)
        down_stream_packed_kernel<<<dim3(s.H / 128, max_active(s)), 256, 0, st>>>(
            (const bf16_t *)hidden, (const bf16_t *)w_down, wl, y_pairs, s.H, s.I, want);
    else
        down_stream_kernel<FT><<<dim3((s.H + 64 * FT - 1) / (64 * FT), max_active(s)), 256, 0,
                                 st>>>((const bf16_t *)hidden, (const bf16_t *)w_down, wl, y_pairs,
                                       s.H, s.I, want);
    return hipGetLastError();
}

// The three-kernel path above.  Logits [T,N] x 2 with biases already added.
constexpr int kTinySlots = 24;
bool tiny_decode_supported(const beam_shape &s, int S) {
    // Measured against the six-kernel path (Qwen3-shaped layer, 8 slots per token): 19.6 vs
    // 28.9 us at T = 1, 27.4 vs 30.6 at T = 3, level at T = 4, slower from there on, because
    // every slot's workgroups pay for a routing pass before most of them find their slot
    // masked.
    return stream_ffn_supported(s) && (long)s.T * (s.K + S) <= kTinySlots && s.K + S <= 64;
}

hipError_t launch_tiny_gate_up(const beam_shape &s, const RouteOpts &opt, const void *x,
                               const float *router_logits, const float *mask_logits,
                               const void *w_gate_up, void *hidden, hipStream_t st) {
    const bool packed = s.weight_layout == BEAM_WEIGHTS_PACKED;
    const dim3 grid(s.I / (packed ? 32 : 16), s.T * (s.K + opt.S));
#define BEAM_TINY(KERNEL, RULE)                                                                 \
    KERNEL<RULE><<<grid, 256, 0, st>>>((const bf16_t *)x, (const bf16_t *)w_gate_up,            \
                                       router_logits, mask_logits, opt.g_shared, opt.param,     \
                                       (bf16_t *)hidden, s.H, s.N, s.K, opt.S, s.I)
    if (packed && opt.rule == kRuleCumProb) BEAM_TINY(gate_up_slot_packed_kernel, kRuleCumProb);
    else if (packed) BEAM_TINY(gate_up_slot_packed_kernel, kRuleMask);
    else if (opt.rule == kRuleCumProb) BEAM_TINY(gate_up_slot_kernel, kRuleCumProb);
    else BEAM_TINY(gate_up_slot_kernel, kRuleMask);
#undef BEAM_TINY
    return hipGetLastError();
}

hipError_t launch_tiny_down_combine(const beam_shape &s, const RouteOpts &opt,
                                    const float *router_logits, const float *mask_logits,
                                    const void *hidden, const void *w_down, const void *residual,
                                    void *out, int32_t *topk_ids_opt, float *topk_w_opt,
                                    int32_t *masked_ids_opt, int32_t *num_pairs_opt,
                                    hipStream_t st) {
    constexpr int FT = 2;  // plain: 16 * FT = 32 features per workgroup, as one packed block
    const dim3 grid(s.H / 32, s.T);
#define BEAM_TINY_ARGS                                                                          \
    (const bf16_t *)hidden, (const bf16_t *)w_down, router_logits, mask_logits, opt.g_shared,   \
        opt.param, (const bf16_t *)residual, (bf16_t *)out, topk_ids_opt, topk_w_opt,           \
        masked_ids_opt, num_pairs_opt, s.H, s.N, s.K, opt.S, s.I
    const bool packed = s.weight_layout == BEAM_WEIGHTS_PACKED;
    if (packed && opt.rule == kRuleCumProb)
        down_combine_token_packed_kernel<kRuleCumProb><<<grid, 256, 0, st>>>(BEAM_TINY_ARGS);
    else if (packed)
        down_combine_token_packed_kernel<kRuleMask><<<grid, 256, 0, st>>>(BEAM_TINY_ARGS);
    else if (opt.rule == kRuleCumProb)
        down_combine_token_kernel<FT, kRuleCumProb><<<grid, 256, 0, st>>>(BEAM_TINY_ARGS);
    else
        down_combine_token_kernel<FT, kRuleMask><<<grid, 256, 0, st>>>(BEAM_TINY_ARGS);
#undef BEAM_TINY_ARGS
    return hipGetLastError();
}

}  // namespace beam

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

namespace beam {

// hidden[row, j] = bf16( SiLU(x_t . W_gate[j]) * (x_t . W_up[j]) )
// grid (I/16, max active experts); 4 wavefronts split the reduction over H.
__global__ __launch_bounds__(256) void gate_up_stream_kernel(
    const bf16_t *__restrict__ x, const bf16_t *__restrict__ w_gate_up,
    const int32_t *__restrict__ perm, WorkList wl, bf16_t *__restrict__ hidden, int H, int K,
    int I) {
    const int u = blockIdx.y;
    // one round trip: the four words are independent loads
    const int n_active = wl.hdr[0];
    const int e = wl.active[u];
    const int row_beg = wl.active_beg[u];
    const int row_end = wl.active_end[u];
    if (u >= n_active) return;
    const int lane = threadIdx.x & 63;
    const int ks = threadIdx.x >> 6;
    const int l16 = lane & 15;
    const int g = lane >> 4;
    const int j0 = blockIdx.x * 16;
    const int klen = H >> 2;
    const int kbeg = ks * klen + g * 8;
    const bf16_t *gp = w_gate_up + ((size_t)e * 2 * I + j0 + l16) * H + kbeg;
    const bf16_t *up = gp + (size_t)I * H;
    __shared__ float red[3][8][64];

    for (int row0 = row_beg; row0 < row_end; row0 += 16) {
        int row = row0 + l16;
        row = row < row_end ? row : row_end - 1;
        const int t = perm[row] / K;
        const bf16_t *xp = x + (size_t)t * H + kbeg;
        f32x4 ag = {0.f, 0.f, 0.f, 0.f};
        f32x4 au = {0.f, 0.f, 0.f, 0.f};
        // Software pipeline over chunks of 128 reduction indices: the loads of
        // chunk c+1 are issued before the MFMAs of chunk c, so a wavefront always
        // has 12 KB in flight.  sched_barrier keeps the compiler from sinking the
        // loads back behind the MFMAs to save registers.
        uint4 wg[2][4], wu[2][4], xv[2][4];
        auto load = [&](int b, int k) {
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                wg[b][j] = *(const uint4 *)(gp + k + j * 32);
                wu[b][j] = *(const uint4 *)(up + k + j * 32);
            }
#pragma unroll
            for (int j = 0; j < 4; ++j) xv[b][j] = *(const uint4 *)(xp + k + j * 32);
        };
        auto mma = [&](int b) {
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                ag = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, wg[b][j]),
                                                             __builtin_bit_cast(bf16x8, xv[b][j]),
                                                             ag, 0, 0, 0);
                au = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, wu[b][j]),
                                                             __builtin_bit_cast(bf16x8, xv[b][j]),
                                                             au, 0, 0, 0);
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
            for (int r = 0; r < 4; ++r) {
                red[ks - 1][r][lane] = ag[r];
                red[ks - 1][4 + r][lane] = au[r];
            }
        }
        __syncthreads();
        if (ks == 0) {
#pragma unroll
            for (int s = 0; s < 3; ++s)
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                    ag[r] += red[s][r][lane];
                    au[r] += red[s][4 + r][lane];
                }
            if (row0 + l16 < row_end) {
                uint32_t lo = (uint32_t)f32_to_bf16(silu(ag[0]) * au[0]) |
                              ((uint32_t)f32_to_bf16(silu(ag[1]) * au[1]) << 16);
                uint32_t hi = (uint32_t)f32_to_bf16(silu(ag[2]) * au[2]) |
                              ((uint32_t)f32_to_bf16(silu(ag[3]) * au[3]) << 16);
                *(uint2 *)(hidden + (size_t)(row0 + l16) * I + j0 + g * 4) = make_uint2(lo, hi);
            }
        }
        __syncthreads();
    }
}

// y_pairs[row, c] = hidden[row, :] . W_down[c, :]
// grid (H / (64*FT), max active experts); each wavefront owns FT tiles of 16
// output features and runs the whole reduction over I.
template <int FT>
__global__ __launch_bounds__(256) void down_stream_kernel(
    const bf16_t *__restrict__ hidden, const bf16_t *__restrict__ w_down, WorkList wl,
    float *__restrict__ y_pairs, int H, int I) {
    const int u = blockIdx.y;
    const int n_active = wl.hdr[0];
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

    for (int row0 = row_beg; row0 < row_end; row0 += 16) {
        int row = row0 + l16;
        row = row < row_end ? row : row_end - 1;
        const bf16_t *hp = hidden + (size_t)row * I + g * 8;
        f32x4 acc[FT];
#pragma unroll
        for (int f = 0; f < FT; ++f) acc[f] = f32x4{0.f, 0.f, 0.f, 0.f};
        // same two-deep software pipeline as the gate/up kernel
        uint4 w[2][FT][4], hv[2][4];
        auto load = [&](int b, int k) {
#pragma unroll
            for (int j = 0; j < 4; ++j) {
#pragma unroll
                for (int f = 0; f < FT; ++f) w[b][f][j] = *(const uint4 *)(wp[f] + k + j * 32);
                hv[b][j] = *(const uint4 *)(hp + k + j * 32);
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
        if (row0 + l16 < row_end) {
#pragma unroll
            for (int f = 0; f < FT; ++f) {
                const int c = c0 + f * 16 + g * 4;
                if (c < H)
                    *(float4 *)(y_pairs + (size_t)(row0 + l16) * H + c) =
                        make_float4(acc[f][0], acc[f][1], acc[f][2], acc[f][3]);
            }
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
                                 void *hidden, hipStream_t st) {
    dim3 grid(s.I / 16, max_active(s));
    (void)offsets;
    gate_up_stream_kernel<<<grid, 256, 0, st>>>((const bf16_t *)x, (const bf16_t *)w_gate_up, perm,
                                                wl, (bf16_t *)hidden, s.H, s.K, s.I);
    return hipGetLastError();
}

hipError_t launch_down_stream(const beam_shape &s, const void *hidden, const void *w_down,
                              const int32_t *offsets, const WorkList &wl, float *y_pairs,
                              hipStream_t st) {
    constexpr int FT = 2;
    dim3 grid((s.H + 64 * FT - 1) / (64 * FT), max_active(s));
    (void)offsets;
    down_stream_kernel<FT><<<grid, 256, 0, st>>>((const bf16_t *)hidden, (const bf16_t *)w_down, wl,
                                                 y_pairs, s.H, s.I);
    return hipGetLastError();
}

}  // namespace beam

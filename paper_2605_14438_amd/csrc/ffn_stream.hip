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
    const int32_t *__restrict__ offsets, const int32_t *__restrict__ perm,
    const int32_t *__restrict__ wl_hdr, const int32_t *__restrict__ wl_active,
    bf16_t *__restrict__ hidden, int H, int K, int I) {
    const int u = blockIdx.y;
    if (u >= wl_hdr[0]) return;
    const int e = wl_active[u];
    const int row_beg = offsets[e];
    const int row_end = offsets[e + 1];
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
        for (int k = 0; k < klen; k += 128) {
            uint4 wg[4], wu[4], xv[4];
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                wg[j] = *(const uint4 *)(gp + k + j * 32);
                wu[j] = *(const uint4 *)(up + k + j * 32);
                xv[j] = *(const uint4 *)(xp + k + j * 32);
            }
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                ag = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, wg[j]),
                                                             __builtin_bit_cast(bf16x8, xv[j]), ag,
                                                             0, 0, 0);
                au = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, wu[j]),
                                                             __builtin_bit_cast(bf16x8, xv[j]), au,
                                                             0, 0, 0);
            }
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
    const bf16_t *__restrict__ hidden, const bf16_t *__restrict__ w_down,
    const int32_t *__restrict__ offsets, const int32_t *__restrict__ wl_hdr,
    const int32_t *__restrict__ wl_active, float *__restrict__ y_pairs, int H, int I) {
    const int u = blockIdx.y;
    if (u >= wl_hdr[0]) return;
    const int e = wl_active[u];
    const int row_beg = offsets[e];
    const int row_end = offsets[e + 1];
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
        for (int k = 0; k < I; k += 128) {
            uint4 w[FT][4], hv[4];
#pragma unroll
            for (int j = 0; j < 4; ++j) {
#pragma unroll
                for (int f = 0; f < FT; ++f) w[f][j] = *(const uint4 *)(wp[f] + k + j * 32);
                hv[j] = *(const uint4 *)(hp + k + j * 32);
            }
#pragma unroll
            for (int j = 0; j < 4; ++j)
#pragma unroll
                for (int f = 0; f < FT; ++f)
                    acc[f] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(
                        __builtin_bit_cast(bf16x8, w[f][j]), __builtin_bit_cast(bf16x8, hv[j]),
                        acc[f], 0, 0, 0);
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
    gate_up_stream_kernel<<<grid, 256, 0, st>>>((const bf16_t *)x, (const bf16_t *)w_gate_up,
                                                offsets, perm, wl.hdr, wl.active,
                                                (bf16_t *)hidden, s.H, s.K, s.I);
    return hipGetLastError();
}

hipError_t launch_down_stream(const beam_shape &s, const void *hidden, const void *w_down,
                              const int32_t *offsets, const WorkList &wl, float *y_pairs,
                              hipStream_t st) {
    constexpr int FT = 2;
    dim3 grid((s.H + 64 * FT - 1) / (64 * FT), max_active(s));
    down_stream_kernel<FT><<<grid, 256, 0, st>>>((const bf16_t *)hidden, (const bf16_t *)w_down,
                                                 offsets, wl.hdr, wl.active, y_pairs, s.H, s.I);
    return hipGetLastError();
}

}  // namespace beam

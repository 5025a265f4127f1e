// GLU experts (paper Eq. 3, delta = SiLU) for prefill-sized batches, bf16: a
// grouped GEMM over the expert-sorted rows on the matrix cores.
//
// The kept pairs of expert e are the grouped rows [offsets[e], offsets[e+1]).
// Each segment is cut into row tiles of BM rows (the work list; this is the
// "block alignment" of App. A.4 without padding the index array: rows past the
// end of a segment are clamped on load and masked on store).  One workgroup
// computes a BM x BN output tile, K-loop in steps of 64:
//
//   GATE_UP:  A = x rows gathered through perm (token = perm[row] / K),
//             B = BN/2 gate rows and the BN/2 matching up rows of W_gate_up[e],
//             interleaved in blocks of 32 so that MFMA column tile 2q holds
//             gate features and tile 2q+1 the same features of up; the
//             epilogue forms SiLU(gate)*up in registers and writes bf16.
//   DOWN:     A = hidden rows (contiguous), B = BN rows of W_down[e]; the
//             epilogue writes fp32 y_pairs.
//
// Both operands are "reduction dimension contiguous", which is the order the
// MFMA wants, so tiles travel global -> registers -> LDS in 16-byte pieces,
// double buffered: the global loads of k-step i+1 are in flight while k-step i
// is multiplied out of the other LDS stage.  LDS rows hold 8 pieces (64 bf16);
// piece c of row r is stored at c ^ (r & 7) so that the 16-byte operand reads
// of 8 consecutive rows fall in 8 different bank groups.
//
// Work order.  Workgroups are handed to the 8 XCDs round-robin by linear id,
// and each XCD has its own L2.  Linear id b is therefore remapped to work item
// (b % 8) * ceil(W/8) + b / 8: every XCD walks one contiguous eighth of the
// (expert, row tile, column tile) list, column tile fastest, so the workgroups
// that run together on an XCD share their A tile and their expert's weights
// through that XCD's L2 instead of each pulling them from HBM.
//
// v_mfma_f32_32x32x16_bf16 layouts (wave64): A/B lane l -> row/col l & 31,
// k = 8*(l >> 5)..+7;  D register r of lane l -> row 8*(r >> 2) + 4*(l >> 5) +
// (r & 3), col l & 31.
#include "common.hpp"

namespace beam {

template <int BM, int BN, int WM, int WN, bool GATE_UP>
__global__ __launch_bounds__(64 * WM * WN) void ffn_tile_kernel(
    const bf16_t *__restrict__ a_src,   // GATE_UP: x [T,H];  DOWN: hidden [P,I]
    const bf16_t *__restrict__ w,       // GATE_UP: w_gate_up [N,2I,H];  DOWN: w_down [N,H,I]
    const int32_t *__restrict__ offsets, const int32_t *__restrict__ perm,
    const int32_t *__restrict__ wl_hdr, const int32_t *__restrict__ tile_expert,
    const int32_t *__restrict__ tile_row0, bf16_t *__restrict__ hidden_out,
    float *__restrict__ y_out, int H, int K, int I, int n_col_tiles) {
    constexpr int NT = 64 * WM * WN;
    constexpr int RPP = NT / 8;          // tile rows copied per pass
    constexpr int AP = BM / RPP;
    constexpr int BP = BN / RPP;
    constexpr int WTM = BM / WM / 32;    // MFMA tiles per wavefront
    constexpr int WTN = BN / WN / 32;
    static_assert(BM % RPP == 0 && BN % RPP == 0, "tile/loader mismatch");
    static_assert(!GATE_UP || WTN % 2 == 0, "gate/up tiles must pair inside a wavefront");

    // XCD-aware work order
    const int n_work = wl_hdr[1] * n_col_tiles;
    const int per_xcd = (n_work + 7) >> 3;
    const int slot = blockIdx.x >> 3;
    const int work = (blockIdx.x & 7) * per_xcd + slot;
    if (slot >= per_xcd || work >= n_work) return;
    const int tile = work / n_col_tiles;
    const int col_tile = work - tile * n_col_tiles;

    const int e = tile_expert[tile];
    const int row0 = tile_row0[tile];
    const int row_end = offsets[e + 1];
    const int n0 = col_tile * (GATE_UP ? BN / 2 : BN);
    const int kdim = GATE_UP ? H : I;

    __shared__ uint4 As[2][BM * 8];
    __shared__ uint4 Bs[2][BN * 8];

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = tid >> 6;
    const int wm = wave / WN;
    const int wn = wave % WN;
    const int piece = tid & 7;
    const int lr = tid >> 3;

    const bf16_t *ap[AP];
    const bf16_t *bp[BP];
#pragma unroll
    for (int p = 0; p < AP; ++p) {
        int grow = row0 + lr + p * RPP;
        grow = grow < row_end ? grow : row_end - 1;
        if constexpr (GATE_UP) {
            const int tok = perm[grow] / K;
            ap[p] = a_src + (size_t)tok * H + piece * 8;
        } else {
            ap[p] = a_src + (size_t)grow * I + piece * 8;
        }
    }
#pragma unroll
    for (int p = 0; p < BP; ++p) {
        const int r = lr + p * RPP;
        if constexpr (GATE_UP) {
            const int blk = r >> 5;
            const int feat = n0 + (blk >> 1) * 32 + (r & 31);
            const int wrow = (blk & 1) ? I + feat : feat;
            bp[p] = w + ((size_t)e * 2 * I + wrow) * H + piece * 8;
        } else {
            bp[p] = w + ((size_t)e * H + n0 + r) * I + piece * 8;
        }
    }

    f32x16 acc[WTM][WTN];
#pragma unroll
    for (int m = 0; m < WTM; ++m)
#pragma unroll
        for (int n = 0; n < WTN; ++n)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[m][n][r] = 0.0f;

    uint4 ra[AP], rb[BP];
    auto gload = [&](int ko) {
#pragma unroll
        for (int p = 0; p < AP; ++p) ra[p] = *(const uint4 *)(ap[p] + ko);
#pragma unroll
        for (int p = 0; p < BP; ++p) rb[p] = *(const uint4 *)(bp[p] + ko);
    };
    auto lstore = [&](int st) {
#pragma unroll
        for (int p = 0; p < AP; ++p) {
            const int r = lr + p * RPP;
            As[st][r * 8 + (piece ^ (r & 7))] = ra[p];
        }
#pragma unroll
        for (int p = 0; p < BP; ++p) {
            const int r = lr + p * RPP;
            Bs[st][r * 8 + (piece ^ (r & 7))] = rb[p];
        }
    };

    const int l32 = lane & 31;
    const int kh = lane >> 5;
    const int nk = kdim / 64;

    gload(0);
    lstore(0);
    __syncthreads();
    for (int kt = 0; kt < nk; ++kt) {
        const int st = kt & 1;
        const bool more = kt + 1 < nk;
        if (more) gload((kt + 1) * 64);
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int kk = 0; kk < 4; ++kk) {
            const int pc = kk * 2 + kh;
            uint4 af[WTM], bf[WTN];
#pragma unroll
            for (int m = 0; m < WTM; ++m) {
                const int r = wm * (BM / WM) + m * 32 + l32;
                af[m] = As[st][r * 8 + (pc ^ (r & 7))];
            }
#pragma unroll
            for (int n = 0; n < WTN; ++n) {
                const int r = wn * (BN / WN) + n * 32 + l32;
                bf[n] = Bs[st][r * 8 + (pc ^ (r & 7))];
            }
#pragma unroll
            for (int m = 0; m < WTM; ++m)
#pragma unroll
                for (int n = 0; n < WTN; ++n)
                    acc[m][n] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(
                        __builtin_bit_cast(bf16x8, af[m]), __builtin_bit_cast(bf16x8, bf[n]),
                        acc[m][n], 0, 0, 0);
        }
        __builtin_amdgcn_sched_barrier(0);
        // the other stage was last read in iteration kt-1; the barrier that
        // closed that iteration makes it free to overwrite now
        if (more) lstore(st ^ 1);
        __syncthreads();
    }

    // epilogue
#pragma unroll
    for (int m = 0; m < WTM; ++m) {
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            const int trow = wm * (BM / WM) + m * 32 + (r >> 2) * 8 + kh * 4 + (r & 3);
            const int grow = row0 + trow;
            if (grow >= row_end) continue;
            if constexpr (GATE_UP) {
#pragma unroll
                for (int q = 0; q < WTN / 2; ++q) {
                    const int blk = wn * WTN + 2 * q;
                    const int feat = n0 + (blk >> 1) * 32 + l32;
                    const float hv = silu(acc[m][2 * q][r]) * acc[m][2 * q + 1][r];
                    hidden_out[(size_t)grow * I + feat] = f32_to_bf16(hv);
                }
            } else {
#pragma unroll
                for (int n = 0; n < WTN; ++n) {
                    const int c = n0 + (wn * WTN + n) * 32 + l32;
                    y_out[(size_t)grow * H + c] = acc[m][n][r];
                }
            }
        }
    }
}

// Row-tile size for a shape, decided on the host from the worst-case average
// segment length (the host never learns the real counts).
int ffn_tile_m(const beam_shape &s) {
    return ((long)s.T * s.K >= 512L * s.N && s.I % 128 == 0 && s.H % 256 == 0) ? 256 : 128;
}

bool tiled_ffn_supported(const beam_shape &s) {
    return s.dtype == BEAM_BF16 && s.H % 128 == 0 && s.I % 64 == 0;
}

static int max_tiles(const beam_shape &s, int tile_m) {
    return (int)((long)s.T * s.K / tile_m + s.N);
}

hipError_t launch_gate_up_tiled(const beam_shape &s, const void *x, const void *w_gate_up,
                                const int32_t *offsets, const int32_t *perm, const WorkList &wl,
                                void *hidden, hipStream_t st) {
    const int tm = ffn_tile_m(s);
    if (tm == 256) {
        const int nct = s.I / 128;
        ffn_tile_kernel<256, 256, 2, 4, true><<<max_tiles(s, tm) * nct, 512, 0, st>>>(
            (const bf16_t *)x, (const bf16_t *)w_gate_up, offsets, perm, wl.hdr, wl.tile_expert,
            wl.tile_row0, (bf16_t *)hidden, nullptr, s.H, s.K, s.I, nct);
    } else {
        const int nct = s.I / 64;
        ffn_tile_kernel<128, 128, 2, 2, true><<<max_tiles(s, tm) * nct, 256, 0, st>>>(
            (const bf16_t *)x, (const bf16_t *)w_gate_up, offsets, perm, wl.hdr, wl.tile_expert,
            wl.tile_row0, (bf16_t *)hidden, nullptr, s.H, s.K, s.I, nct);
    }
    return hipGetLastError();
}

hipError_t launch_down_tiled(const beam_shape &s, const void *hidden, const void *w_down,
                             const int32_t *offsets, const WorkList &wl, float *y_pairs,
                             hipStream_t st) {
    const int tm = ffn_tile_m(s);
    if (tm == 256) {
        const int nct = s.H / 256;
        ffn_tile_kernel<256, 256, 2, 4, false><<<max_tiles(s, tm) * nct, 512, 0, st>>>(
            (const bf16_t *)hidden, (const bf16_t *)w_down, offsets, nullptr, wl.hdr,
            wl.tile_expert, wl.tile_row0, nullptr, y_pairs, s.H, s.K, s.I, nct);
    } else {
        const int nct = s.H / 128;
        ffn_tile_kernel<128, 128, 2, 2, false><<<max_tiles(s, tm) * nct, 256, 0, st>>>(
            (const bf16_t *)hidden, (const bf16_t *)w_down, offsets, nullptr, wl.hdr,
            wl.tile_expert, wl.tile_row0, nullptr, y_pairs, s.H, s.K, s.I, nct);
    }
    return hipGetLastError();
}

}  // namespace beam

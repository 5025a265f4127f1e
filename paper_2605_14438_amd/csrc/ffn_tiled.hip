// GLU experts (paper Eq. 3, delta = SiLU) for prefill-sized batches, bf16: a
// grouped GEMM over the expert-sorted rows on the matrix cores.
//
// The kept pairs of expert e are the grouped rows [offsets[e], offsets[e+1]).
// Each segment is cut into row tiles of BM = 128 rows (the work list; this is
// the "block alignment" of App. A.4 without padding the index array: rows past
// the end of a segment are clamped on load and masked on store).  One workgroup
// of NW = 4 or 8 wavefronts side by side computes a BM x (64 NW) output tile, each
// wavefront all BM rows of 64 columns as 32x32 MFMA tiles, K-loop in steps of 16*KS
// (column counts below are for NW = 4; with eight wavefronts a tile is twice as wide):
//
//   GATE_UP:  A = x rows gathered through perm (token = perm[row] / K),
//             B = 128 gate rows and the 128 matching up rows of W_gate_up[e],
//             interleaved in blocks of 32 so that MFMA column tile 2q holds
//             gate features and tile 2q+1 the same features of up; the
//             epilogue forms SiLU(gate)*up in registers and writes bf16.
//   DOWN:     A = hidden rows (contiguous), B = 256 rows of W_down[e]; the
//             epilogue writes fp32 y_pairs.
//
// Operand paths.  On gfx950 the MFMA rate is twice MI300's while the LDS still
// delivers 128 B/clk/CU on reads and about half that on writes, so a kernel
// that stages both operands through LDS is LDS bound.  Here only the
// activations (A) go global -> registers -> LDS (double buffered, 16-byte
// pieces, piece c of row r stored at c ^ (r & 7) so the operand reads of 8
// consecutive rows fall in 8 different bank groups).  The weights (B) never
// touch LDS; they go from global memory straight into the MFMA B registers,
// refilled on a rolling basis about three quarters of a K-step ahead.
//   PACKED weights (beam_pack_weights) are stored in MFMA fragment order: the B
//   operand of one 32x32x16 MFMA is one contiguous 1 KiB block, lane l reading
//   bytes 16*l, so every weight load is fully coalesced and a wavefront's
//   stream through an expert is sequential.
//   PLAIN row-major weights are also "reduction dimension contiguous", which is
//   the order the MFMA wants, so they can be fed directly too: every lane loads
//   the 64 contiguous bytes of its weight row that it needs for the four MFMA
//   k-steps of a K-step.  To make them contiguous, step j of lane-half h uses
//   k = 32*h + 8*j..+7 on BOTH operands (a permutation of the reduction index,
//   which leaves the dot product unchanged): A piece 4*h + j from LDS.  But
//   adjacent lanes then sit in different weight rows, and the vector memory
//   path serves such 16-byte pieces at about one per clock: this variant runs
//   at roughly half the speed of the packed one.
//
// Work order.  Workgroups are handed to the 8 XCDs round-robin by linear id,
// and each XCD has its own L2.  The grid is persistent: 512 workgroups, two per
// CU (256 of eight wavefronts, one per CU, in the wide schedule), workgroup b on XCD
// b % 8 as its member b / 8.  The (row tile, column
// tile) items are ordered by groups of up to four row tiles of one expert,
// inside a group by column tile, then by row tile, and this sequence
// is cut into chunks of 64 consecutive items; chunk c goes to XCD c % 8, one
// item per resident workgroup.  So the 64 workgroups that run together on an
// XCD hold four row tiles times 16 column tiles (or, when an expert has fewer
// column tiles, all of them for about ten row tiles): they share their A tiles
// and that expert's weights through the XCD's L2 instead of each pulling them
// from HBM, while the chunks deal the work evenly over the XCDs.
//
// v_mfma_f32_32x32x16_bf16 layouts (wave64): A/B lane l -> row/col l & 31,
// k = 8*(l >> 5)..+7; D register r of lane l -> row 8*(r >> 2) + 4*(l >> 5) +
// (r & 3), col l & 31.  In the gate/up GEMM the weights are passed as the MFMA
// "A" operand (result rows = output features) and the activations as "B" (result
// columns = grouped rows), so a lane ends up with runs of four consecutive
// features of one row; the down GEMM passes them the other way round.
#include <type_traits>

#include "common.hpp"

namespace beam {

constexpr int kTileN = 256;
constexpr int kWorkgroupsPerCU = 2;
// row tiles that share a column tile's weights back to back in the work order
constexpr int kRowGroup = 4;
// wavefront grid inside a workgroup: 1 x 4 (each weight fragment is loaded by exactly one wavefront)
constexpr int kWavesM = 1;
// MFMA k-steps per K-step of the main loop
constexpr int kKSteps = 4;

// KS = MFMA k-steps (16 reduction indices each) per K-step of the main loop: one
// K-step is the prefetch distance.  With two workgroups per CU the register
// budget is 256 per lane (128 of them accumulators), which fits KS = 4; the
// other workgroup's MFMAs cover what a 64-wide prefetch distance does not.
// One item of work: output tile rows [row0, min(row0 + BM, row_end)) of expert
// e, column tile col_tile.
// 16 bytes as a native vector: register arrays of it are promoted reliably,
// which arrays of the uint4 struct are not once they live across items
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

struct TileItem {
    int e, row0, row_end, col_tile;
    int slice;  // which part of the reduction (down roles with a split reduction), else 0
};

// The persistent tile loop of one workgroup.  next_item(seq, it) advances seq to
// this workgroup's next item at or after position seq and fills `it`, or returns
// false when there is none; it must be uniform over the workgroup.
// As: 2 * BM * 2 * KS uint4 of LDS.
//
// CHAIN: items are chained without a pipeline bubble: the last K-step of an item
// already issues the next item's first weight fragments and, behind its MFMAs,
// the next item's first activation tile, which then lands during the epilogue's
// stores; only the very first item of a workgroup pays a prologue.  That keeps
// one K-step of operands live across the epilogue (48 more registers with 128-row
// tiles), which the schedule with two workgroups per CU cannot afford: there
// CHAIN is off, every item starts with its own prologue, and the other
// workgroup's MFMAs cover it.
// COL_GUARD (down roles only): the output is narrower than the last column tile;
// columns >= H are computed from zero padding and not stored.
// stream_out (down roles only, uniform): the output goes past the caches.
// y16 (down roles only, uniform, k_split == 1): the output rows are stored as IEEE half
// precision (11 significant bits, saturating at +-65504) instead of fp32; y_out then points
// to an array of that type.
// k_split (down roles only): the reduction is cut into k_split equal parts; an
// item multiplies part `slice` and writes its partial sums to y_out + slice *
// slice_stride (elements).  With few, long items (a handful of experts with a
// long reduction) this is what fills the chip and evens out its last round;
// the aggregation adds the parts in slice order.
template <int BM, int WM, int KS, bool GATE_UP, bool PACKED, bool CHAIN, bool COL_GUARD, int NW,
          typename NextItem>
__device__ __forceinline__ void ffn_tile_run(
    u32x4 *As, const bf16_t *__restrict__ a_src, const bf16_t *__restrict__ w,
    const int32_t *__restrict__ perm, bf16_t *__restrict__ hidden_out, float *__restrict__ y_out,
    int H, int K, int I, bool stream_out, bool y16, int k_split, size_t slice_stride,
    NextItem next_item) {
    constexpr int PR = 2 * KS;           // 16-byte pieces per LDS row (K-step of 16*KS indices)
    constexpr int NT = 64 * NW;          // threads; NW wavefronts, each 64 columns wide with WM == 1
    constexpr int TN = kTileN * NW / 4;  // columns of the output tile
    constexpr int RPP = NT / PR;         // tile rows copied per pass of the workgroup's threads
    constexpr int AP = BM / RPP;         // A rows per thread
    constexpr int WN = NW / WM;
    constexpr int WTM = BM / WM / 32;    // MFMA row tiles per wavefront
    constexpr int WTN = (TN / 32) / WN;  // MFMA column tiles per wavefront (TN columns in all)
    static_assert(WM == 1 || WM == 2, "wavefront grid is 1x4 or 2x2");
    constexpr int kStage = BM * PR;      // uint4 per LDS stage

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = tid >> 6;
    const int wm = wave / WN;
    const int wn = wave % WN;
    const int piece = tid % PR;
    const int lr = tid / PR;
    const int l32 = lane & 31;
    const int kh = lane >> 5;
    const int kdim = GATE_UP ? H : I;
    const int nk = kdim / (16 * KS) / k_split;   // K-steps per item
    // element stride between the weight pieces of consecutive MFMA k-steps,
    // and between consecutive K-steps
    constexpr int kBStep = PACKED ? 512 : 8;
    constexpr int kBKStep = PACKED ? 512 * KS : 16 * KS;

    int seq = 0;
    TileItem cur;
    if (!next_item(seq, cur)) return;

    // element offsets of this thread's A rows (32 bits: T*H and T*K*I < 2^32,
    // checked on the host); pointers would cost twice the registers
    uint32_t ao[AP];
    const bf16_t *bp[WTN];
// operand addresses of item `it`
#define BEAM_SETUP(it)                                                                          \
    _Pragma("unroll") for (int p = 0; p < AP; ++p) {                                            \
        int grow = (it).row0 + lr + p * RPP;                                                    \
        grow = grow < (it).row_end ? grow : (it).row_end - 1;                                   \
        if constexpr (GATE_UP) {                                                                \
            const int tok = perm[grow] / K;                                                     \
            ao[p] = (uint32_t)tok * (uint32_t)H + piece * 8;                                    \
        } else {                                                                                \
            ao[p] = (uint32_t)grow * (uint32_t)I + piece * 8 + (it).slice * nk * (16 * KS);     \
        }                                                                                       \
    }                                                                                           \
    _Pragma("unroll") for (int n = 0; n < WTN; ++n) {                                           \
        const int nb = wn * WTN + n;                                                            \
        if constexpr (PACKED) {                                                                 \
            /* 32-row block rb of this expert: (kdim/16) fragments of 512 elements */           \
            const int rows32 = (GATE_UP ? 2 * I : H) >> 5;                                      \
            const int rb = (it).col_tile * (TN / 32) + nb;                                      \
            bp[n] = w + ((size_t)(it).e * rows32 + rb) * (size_t)(kdim >> 4) * 512 + lane * 8;  \
        } else if constexpr (GATE_UP) {                                                         \
            const int feat = (it).col_tile * (TN / 2) + (nb >> 1) * 32 + l32;                   \
            const int wrow = (nb & 1) ? I + feat : feat;                                        \
            bp[n] = w + ((size_t)(it).e * 2 * I + wrow) * H + kh * (8 * KS);                    \
        } else {                                                                                \
            bp[n] = w + ((size_t)(it).e * H + (it).col_tile * TN + nb * 32 + l32) * I +         \
                    kh * (8 * KS);                                                              \
        }                                                                                       \
        if constexpr (!GATE_UP) bp[n] += (size_t)(it).slice * nk * kBKStep;                     \
    }

    f32x16 acc[WTM][WTN];
#define BEAM_ZERO_ACC                                                                           \
    _Pragma("unroll") for (int m = 0; m < WTM; ++m)                                             \
        _Pragma("unroll") for (int n = 0; n < WTN; ++n)                                         \
            _Pragma("unroll") for (int r = 0; r < 16; ++r) acc[m][n][r] = 0.0f;

    u32x4 ra[AP];
    u32x4 bq[WTN][KS];
// activation tile: global -> registers, registers -> swizzled LDS stage
#define BEAM_GLOAD_A(ko)                                                         \
    _Pragma("unroll") for (int p = 0; p < AP; ++p) ra[p] = *(const u32x4 *)(a_src + ao[p] + (ko));
#define BEAM_LSTORE_A(st)                                                        \
    _Pragma("unroll") for (int p = 0; p < AP; ++p) {                             \
        const int r_ = lr + p * RPP;                                             \
        As[(st) * kStage + r_ * PR + (piece ^ (r_ & 7))] = ra[p];                \
    }
    // One K-step out of LDS stage st.  The weight registers are a single
    // buffer refilled on a rolling basis: as soon as the MFMAs of k-step j
    // have been issued, bq[.][j] is reloaded for the next K-step, so every
    // weight load has about three quarters of a K-step to arrive.
    // A fragments are double buffered at half-step granularity: a k-step j is
    // done in two halves of GH row tiles; the fragments of the next half are
    // read from LDS before the MFMAs of the current half are issued.
    constexpr int GH = WTM / 2;
    auto read_a = [&](int st, int hstep, u32x4 *af) {
        const int j = hstep >> 1;
        const int g = hstep & 1;
        const int pc = PACKED ? j * 2 + kh : kh * KS + j;
#pragma unroll
        for (int m = 0; m < GH; ++m) {
            const int r = wm * (BM / WM) + (g * GH + m) * 32 + l32;
            af[m] = As[st * kStage + r * PR + (pc ^ (r & 7))];
        }
    };
    auto compute = [&](int st, auto prefetch, int kt_next) {
        constexpr bool PF = decltype(prefetch)::value;
        u32x4 af[2][GH];
        read_a(st, 0, af[0]);
#pragma unroll
        for (int hs = 0; hs < 2 * KS; ++hs) {
            const int j = hs >> 1;
            const int g = hs & 1;
            if (hs + 1 < 2 * KS) read_a(st, hs + 1, af[(hs + 1) & 1]);
#pragma unroll
            for (int m = 0; m < GH; ++m)
#pragma unroll
                for (int n = 0; n < WTN; ++n)
                    if constexpr (GATE_UP)
                        acc[g * GH + m][n] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(
                            __builtin_bit_cast(bf16x8, bq[n][j]),
                            __builtin_bit_cast(bf16x8, af[hs & 1][m]), acc[g * GH + m][n], 0, 0, 0);
                    else
                        acc[g * GH + m][n] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(
                            __builtin_bit_cast(bf16x8, af[hs & 1][m]),
                            __builtin_bit_cast(bf16x8, bq[n][j]), acc[g * GH + m][n], 0, 0, 0);
            if constexpr (PF) {
                if (g == 1) {
#pragma unroll
                    for (int n = 0; n < WTN; ++n)
                        bq[n][j] = *(const u32x4 *)(bp[n] + kt_next * kBKStep + j * kBStep);
                }
            }
        }
    };
    // The same K-step for an item whose tile holds at most 32*MT rows (the ragged last tile
    // of an expert; MT = 1 or 2): only the first MT row tiles are multiplied, one fragment
    // set per k-step, double buffered at k-step granularity.  The other accumulators stay
    // at zero and their rows are masked on store.
    auto compute_short = [&](int st, auto mt_c, auto prefetch, int kt_next) {
        constexpr int MT = decltype(mt_c)::value;
        constexpr bool PF = decltype(prefetch)::value;
        u32x4 af[2][MT];
        auto read_s = [&](int j, u32x4 *f) {
            const int pc = PACKED ? j * 2 + kh : kh * KS + j;
#pragma unroll
            for (int m = 0; m < MT; ++m) {
                const int r = wm * (BM / WM) + m * 32 + l32;
                f[m] = As[st * kStage + r * PR + (pc ^ (r & 7))];
            }
        };
        read_s(0, af[0]);
#pragma unroll
        for (int j = 0; j < KS; ++j) {
            if (j + 1 < KS) read_s(j + 1, af[(j + 1) & 1]);
#pragma unroll
            for (int m = 0; m < MT; ++m)
#pragma unroll
                for (int n = 0; n < WTN; ++n)
                    if constexpr (GATE_UP)
                        acc[m][n] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(
                            __builtin_bit_cast(bf16x8, bq[n][j]),
                            __builtin_bit_cast(bf16x8, af[j & 1][m]), acc[m][n], 0, 0, 0);
                    else
                        acc[m][n] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(
                            __builtin_bit_cast(bf16x8, af[j & 1][m]),
                            __builtin_bit_cast(bf16x8, bq[n][j]), acc[m][n], 0, 0, 0);
            if constexpr (PF) {
#pragma unroll
                for (int n = 0; n < WTN; ++n)
                    bq[n][j] = *(const u32x4 *)(bp[n] + kt_next * kBKStep + j * kBStep);
            }
        }
    };
    // K-loop of such an item: only the rows that can hold data are loaded and stored
    // (the prologue has filled the whole first stage).
    auto k_loop_short = [&](auto mt_c, int par_) {
        constexpr int MT = decltype(mt_c)::value;
        constexpr int APS = (32 * MT + RPP - 1) / RPP < AP ? (32 * MT + RPP - 1) / RPP : AP;
        for (int kt = 0; kt + 1 < nk; ++kt) {
            const int st = (par_ + kt) & 1;
#pragma unroll
            for (int p = 0; p < APS; ++p)
                ra[p] = *(const u32x4 *)(a_src + ao[p] + (kt + 1) * (16 * KS));
            compute_short(st, mt_c, std::true_type{}, kt + 1);
#pragma unroll
            for (int p = 0; p < APS; ++p) {
                const int r_ = lr + p * RPP;
                As[(st ^ 1) * kStage + r_ * PR + (piece ^ (r_ & 7))] = ra[p];
            }
            __builtin_amdgcn_sched_group_barrier(0x020, APS, 0);           // VMEM read
            __builtin_amdgcn_sched_group_barrier(0x100, 2 * MT, 0);        // DS read
#pragma unroll
            for (int j = 0; j < KS; ++j) {
                __builtin_amdgcn_sched_group_barrier(0x008, MT * WTN, 0);  // MFMA
                __builtin_amdgcn_sched_group_barrier(0x020, WTN, 0);       // refill
                if (j < KS - 2) __builtin_amdgcn_sched_group_barrier(0x100, MT, 0);
                if (j >= KS - APS) __builtin_amdgcn_sched_group_barrier(0x200, 1, 0);
            }
            __syncthreads();
        }
        compute_short((par_ + nk - 1) & 1, mt_c, std::false_type{}, 0);
    };
// The order the scheduler is to build for one K-step (left alone it sinks every
// load to just before its first use to save registers): per half k-step the
// MFMAs, the refill of the weight registers they consumed and the LDS fragment
// reads of the next half.
#define BEAM_SCHED_HALF_STEP(hs)                                                                \
    __builtin_amdgcn_sched_group_barrier(0x008, GH * WTN, 0);             /* MFMA */            \
    if ((hs) & 1) __builtin_amdgcn_sched_group_barrier(0x020, WTN, 0);    /* refill */          \
    if ((hs) < 2 * KS - 2) __builtin_amdgcn_sched_group_barrier(0x100, GH, 0);

    int par = 0;  // LDS stage that holds K-step 0 of the current item
    bool prologue = true;
    for (;;) {
        if (prologue) {  // the workgroup's first item; without CHAIN, every item
            BEAM_ZERO_ACC
            BEAM_SETUP(cur)
            BEAM_GLOAD_A(0)
#pragma unroll
            for (int n = 0; n < WTN; ++n)
#pragma unroll
                for (int j = 0; j < KS; ++j) bq[n][j] = *(const u32x4 *)(bp[n] + j * kBStep);
            BEAM_LSTORE_A(0)
            __syncthreads();
            prologue = !CHAIN;
        }
        TileItem nxt;
        int seq_next = seq + 1;
        const bool has_next = next_item(seq_next, nxt);

        // ragged last tiles of an expert with at most 64 / 32 rows: a quarter or half of the MFMAs
        const int valid_rows = cur.row_end - cur.row0;
        const int short_mt = (CHAIN || WM != 1 || valid_rows > 64) ? 0 : (valid_rows > 32 ? 2 : 1);
        if (short_mt == 1) k_loop_short(std::integral_constant<int, 1>{}, par);
        else if (short_mt == 2) k_loop_short(std::integral_constant<int, 2>{}, par);
        // steady state without conditionals, so each wait counts only older loads
        for (int kt = 0; short_mt == 0 && kt + 1 < nk; ++kt) {
            const int st = (par + kt) & 1;
            BEAM_GLOAD_A((kt + 1) * (16 * KS))
            compute(st, std::true_type{}, kt + 1);
            BEAM_LSTORE_A(st ^ 1)
            // activation loads first; the LDS stores of the next activation tile are
            // spread over the last four half-steps, so the matrix cores keep running
            // while the (half-rate) LDS writes drain instead of idling through a
            // store phase.
            __builtin_amdgcn_sched_group_barrier(0x020, AP, 0);            // VMEM read
            __builtin_amdgcn_sched_group_barrier(0x100, 2 * GH, 0);        // DS read
#pragma unroll
            for (int hs = 0; hs < 2 * KS; ++hs) {
                BEAM_SCHED_HALF_STEP(hs)
                if (hs >= 2 * KS - (AP < 4 ? AP : 4))
                    __builtin_amdgcn_sched_group_barrier(0x200, AP < 4 ? 1 : AP / 4, 0);
            }
            __syncthreads();
        }
        const int lst = (par + nk - 1) & 1;
        const TileItem done = cur;
        if (CHAIN && has_next) {
            // Last K-step: operand addresses of the next item (for the gate/up GEMM a
            // lookup through perm, whose latency the MFMAs cover), its first weight
            // fragments as the refills, its first activation tile last.
            BEAM_SETUP(nxt)
            compute(lst, std::true_type{}, 0);
            BEAM_GLOAD_A(0)
            if constexpr (GATE_UP) __builtin_amdgcn_sched_group_barrier(0x020, AP, 0);  // perm
            __builtin_amdgcn_sched_group_barrier(0x100, 2 * GH, 0);
#pragma unroll
            for (int hs = 0; hs < 2 * KS; ++hs) { BEAM_SCHED_HALF_STEP(hs) }
            __builtin_amdgcn_sched_group_barrier(0x020, AP, 0);
        } else if (short_mt == 0) {
            compute(lst, std::false_type{}, 0);
        }

        // Epilogue of item `done`.
        const int n0 = done.col_tile * (GATE_UP ? TN / 2 : TN);
        if constexpr (GATE_UP) {
            // The weights were the MFMA A operand and the activations the B operand,
            // so in a 32x32 result tile lane l holds activation row l & 31 and, in
            // registers 4q..4q+3, the four consecutive features 8q + 4*(l >> 5) +
            // 0..3: one row pointer per tile, SiLU(gate)*up in registers, 8-byte
            // stores of four bf16.
#pragma unroll
            for (int m = 0; m < WTM; ++m) {
                const int grow = done.row0 + wm * (BM / WM) + m * 32 + l32;
                if (grow >= done.row_end) continue;
                bf16_t *orow = hidden_out + (size_t)grow * I + n0 + kh * 4;
#pragma unroll
                for (int q = 0; q < WTN / 2; ++q) {
                    const int nb = wn * WTN + 2 * q;
#pragma unroll
                    for (int rg = 0; rg < 4; ++rg) {
                        uint32_t pk[2];
#pragma unroll
                        for (int h2 = 0; h2 < 2; ++h2) {
                            const int r = rg * 4 + h2 * 2;
                            const float v0 = silu(acc[m][2 * q][r]) * acc[m][2 * q + 1][r];
                            const float v1 = silu(acc[m][2 * q][r + 1]) * acc[m][2 * q + 1][r + 1];
                            pk[h2] = (uint32_t)f32_to_bf16(v0) | ((uint32_t)f32_to_bf16(v1) << 16);
                        }
                        *(uint2 *)(orow + (nb >> 1) * 32 + rg * 8) = make_uint2(pk[0], pk[1]);
                    }
                }
            }
        } else {
            // Activations were the A operand: register r of lane l is row
            // 8*(r >> 2) + 4*(l >> 5) + (r & 3), column l & 31 of the tile, so each
            // store instruction writes two full 128-byte row segments of fp32.
            // The address is split into a part that is the same for the whole wavefront (one
            // 64-bit pointer per item), a 32-bit part per lane and a multiple of the row pitch
            // per register, so that a store costs one 32-bit add; blocks of 32 rows that lie
            // inside the expert's segment are stored without the per-row test.
            auto store_tile = [&](auto stream, auto half) {
                using Y = std::conditional_t<decltype(half)::value, _Float16, float>;
                constexpr uint32_t ysz = sizeof(Y);
                char *base = (char *)y_out +
                             ((size_t)done.slice * slice_stride +
                              (size_t)(done.row0 + wm * (BM / WM)) * H + n0 + wn * WTN * 32) * ysz;
                const uint32_t pitch = (uint32_t)H * ysz;
                const int rows = done.row_end - done.row0 - wm * (BM / WM);   // uniform
                const int lane_rows = rows - kh * 4;
                const uint32_t lane_off = (uint32_t)(kh * 4) * pitch + (uint32_t)l32 * ysz;
                auto store_row = [&](int m, int r, uint32_t pitch_m) {
                    const uint32_t off =
                        lane_off + (uint32_t)(m * 32 + (r >> 2) * 8 + (r & 3)) * pitch_m;
#pragma unroll
                    for (int n = 0; n < WTN; ++n) {
                        if (COL_GUARD && n0 + l32 + (wn * WTN + n) * 32 >= H) continue;
                        Y v;
                        if constexpr (decltype(half)::value)
                            v = (Y)__builtin_amdgcn_fmed3f(acc[m][n][r], -65504.0f, 65504.0f);
                        else
                            v = acc[m][n][r];
                        Y *dst = (Y *)(base + off) + n * 32;
                        if constexpr (decltype(stream)::value) __builtin_nontemporal_store(v, dst);
                        else *dst = v;
                    }
                };
#pragma unroll
                for (int m = 0; m < WTM; ++m) {
                    if (m * 32 >= rows) break;   // uniform
                    // The pitch passes through an empty asm per block so that the row offsets
                    // are formed where they are used, one scalar multiply and one add each; left
                    // alone the compiler forms all of them ahead of the item and spills them.
                    uint32_t pitch_m = pitch;
                    asm volatile("" : "+s"(pitch_m));
                    if ((m + 1) * 32 <= rows) {
#pragma unroll
                        for (int r = 0; r < 16; ++r) store_row(m, r, pitch_m);
                    } else {
#pragma unroll
                        for (int r = 0; r < 16; ++r)
                            if (m * 32 + (r >> 2) * 8 + (r & 3) < lane_rows) store_row(m, r, pitch_m);
                    }
                }
            };
            if (y16 && stream_out) store_tile(std::true_type{}, std::true_type{});
            else if (y16) store_tile(std::false_type{}, std::true_type{});
            else if (stream_out) store_tile(std::true_type{}, std::false_type{});
            else store_tile(std::false_type{}, std::false_type{});
        }
        if (!has_next) break;
        cur = nxt;
        seq = seq_next;
        if constexpr (CHAIN) {
            // The next item's first activation tile goes into the stage that the
            // K-step before last used (every wavefront left it at that K-step's barrier).
            BEAM_LSTORE_A(lst ^ 1)
            BEAM_ZERO_ACC
            par = lst ^ 1;
        }
        __syncthreads();  // CHAIN: the tile is visible; else: both stages are free again
    }
#undef BEAM_SETUP
#undef BEAM_ZERO_ACC
#undef BEAM_GLOAD_A
#undef BEAM_LSTORE_A
#undef BEAM_SCHED_HALF_STEP
}

// Persistent kernel over the work list: kWorkgroupsPerCU resident workgroups
// per CU, each walking (row tile, column tile) items.  Two 128-row workgroups
// per CU measured faster than one 256-row workgroup (the second workgroup's
// MFMAs cover the first one's prologue, epilogue and barriers) and than three
// 64-row ones (more weight traffic per flop).  NW = 8: the two workgroups fused into
// one of eight wavefronts on a tile twice as wide (see launch_tile).
template <int WM, int KS, int OCC, bool GATE_UP, bool PACKED, int NW>
__global__ __launch_bounds__(64 * NW, OCC) void ffn_tile_kernel(
    const bf16_t *__restrict__ a_src,   // GATE_UP: x [T,H];  DOWN: hidden [P,I]
    const bf16_t *__restrict__ w,       // GATE_UP: w_gate_up [N,2I,H];  DOWN: w_down [N,H,I]
    const int32_t *__restrict__ offsets, const int32_t *__restrict__ perm,
    const int32_t *__restrict__ wl_hdr, const int32_t *__restrict__ tile_expert,
    const int32_t *__restrict__ tile_row0, bf16_t *__restrict__ hidden_out,
    float *__restrict__ y_out, int H, int K, int I, int n_col_tiles, int k_split,
    size_t slice_stride, int want, int y16, int tiles_lo, int tiles_hi) {
    __shared__ u32x4 As[2 * kTileM * 2 * KS];
    // Item order: the row tiles of an expert in groups of up to kRowGroup (a group
    // never spans two experts); inside a group the column tile is the slow index
    // and the row tile the fast one, so neighbouring items multiply different rows
    // by the SAME weight fragments and an expert's weights leave HBM about once.
    // The items of a group are the range [F * n_col_tiles, (F + size) * n_col_tiles)
    // with F the list index of its first row tile, so item / n_col_tiles is always
    // a row tile of the item's own group, from which the group is reconstructed.
    // not the regime chosen on the device: no tiles for this kernel, every workgroup leaves
    // tiles_lo, tiles_hi: the kernel runs for work lists of tiles_lo .. tiles_hi row tiles only
    // (two schedules enqueued for one GEMM: the tile count, known on the device, picks one)
    int n_tiles = (want != kRegimeAny && wl_hdr[2] != want) ? 0 : wl_hdr[1];
    if (n_tiles < tiles_lo || n_tiles > tiles_hi) n_tiles = 0;
    // with a split reduction: all items of part 0, then all of part 1, ...
    const int n_base = n_tiles * n_col_tiles;
    const int n_work = n_base * k_split;
    const int xcd = blockIdx.x & 7;
    const int member = blockIdx.x >> 3;  // gridDim.x / 8 workgroups per XCD
    const int per_xcd = gridDim.x >> 3;
    auto next_item = [&](int &round, TileItem &it) -> bool {
        const int item_s = (round * 8 + xcd) * per_xcd + member;
        if (item_s >= n_work) return false;  // uniform over the workgroup
        const int slice = item_s / n_base;
        const int item = item_s - slice * n_base;
        const int q = item / n_col_tiles;
        const int e = tile_expert[q];
        const int beg = offsets[e];
        const int end = offsets[e + 1];
        const int j = (tile_row0[q] - beg) / kTileM;   // q among the expert's row tiles
        const int g0 = j - j % kRowGroup;              // first row tile of the group
        const int left = tiles_of(end - beg) - g0;
        const int size = left < kRowGroup ? left : kRowGroup;
        const int rem = item - (q - (j - g0)) * n_col_tiles;
        const int col_tile = rem / size;
        it.e = e;
        it.row0 = beg + (g0 + rem - col_tile * size) * kTileM;
        it.row_end = end;
        it.col_tile = col_tile;
        it.slice = slice;
        return true;
    };
    // more rows of y_pairs than the last-level cache can hold until they are read again
    const bool stream_out =
        !GATE_UP && (size_t)n_tiles * kTileM * H * (y16 ? 2 : sizeof(float)) > kStreamBytes;
    ffn_tile_run<kTileM, WM, KS, GATE_UP, PACKED, OCC == 1 && NW == 4, false, NW>(
        As, a_src, w, perm, hidden_out, y_out, H, K, I, stream_out, !GATE_UP && y16 != 0, k_split,
        slice_stride,
        next_item);
}

bool tiled_ffn_supported(const beam_shape &s) {
    return s.dtype == BEAM_BF16 && s.H % 256 == 0 && s.I % 128 == 0 &&
           (long)s.T * s.H < (1L << 32) && (long)s.T * s.K * s.I < (1L << 32);
}


template <bool GATE_UP>
static void launch_tile(const beam_shape &s, const bf16_t *a, const bf16_t *w,
                        const int32_t *offsets, const int32_t *perm, const WorkList &wl,
                        bf16_t *hidden, float *y, int nct, int k_split, hipStream_t st, int want,
                        int y16 = 0) {
    const bool packed = s.weight_layout == BEAM_WEIGHTS_PACKED;
    int tiles_lo = 0, tiles_hi = 0x7fffffff;
#define BEAM_LAUNCH_TILE(KS_, OCC_, PK)                                                        \
    ffn_tile_kernel<kWavesM, KS_, OCC_, GATE_UP, PK, 4><<<256 * OCC_, 256, 0, st>>>(           \
        a, w, offsets, perm, wl.hdr, wl.tile_expert, wl.tile_row0, hidden, y, s.H, s.K, s.I, nct, \
        k_split, (size_t)s.T * s.K * s.H, want, y16, tiles_lo, tiles_hi)
    // Three schedules of the same tile body.  "Dense": 64-wide K-steps, two
    // workgroups per CU, whose MFMAs cover each other's prologue, epilogue and
    // barriers; the faster one when the reduction is short and the work MFMA
    // bound.  "Deep": 128-wide K-steps, one workgroup per CU with twice the
    // bytes in flight per barrier and items chained without a prologue;
    // measured 8-17 % faster for the gate/up GEMM
    // when the reduction is long (H >= 4096) or when there are so few rows per
    // expert that the kernel can only be bound by streaming the weights
    // (at most 256 per expert even with every pair kept).
    const bool wide_fits = packed && k_split == 1 &&
                           (GATE_UP ? (2 * s.I) % 512 == 0 : s.H % 512 == 0);
    if constexpr (GATE_UP) {
        const long TK = (long)s.T * s.K;
        if (packed && s.H < 4096 && wide_fits && TK >= 64L * s.N && TK <= 512L * s.N) {
            // In between, which of the deep and the wide schedule is faster follows the number
            // of row tiles, which depends on the keep rate and the routing skew: the wide one
            // needs more than about 1.25 items per workgroup to fill the chip evenly (Qwen3
            // shape, deep / wide gate/up in us: T = 4096 keep 15 %, 103 tiles, 124 / 143;
            // keep 25 % 153 / 144, keep 100 % 292 / 269; T = 2048 keep 50 % 157 / 145;
            // T = 1024 keep 50 % 130 / 149, keep 100 % 158 / 148).  Both are enqueued and the
            // one whose range the tile count is not in leaves at once (whole layer, deep /
            // wide / both enqueued: T = 4096 keep 15 % 232 / 246 / 232, keep 25 % 280 / 264 /
            // 266, keep 100 % 517 / 486 / 489; T = 2048 keep 50 % 299 / 278 / 281).
            const int max_deep = 640 / nct;   // nct column tiles of 256; the wide tile spans two
            tiles_hi = max_deep;
            BEAM_LAUNCH_TILE(8, 1, true);
            if (hipPeekAtLastError() != hipSuccess) return;   // the caller reads and reports it
            tiles_lo = max_deep + 1;
            tiles_hi = 0x7fffffff;
        } else if (packed && s.H >= 4096 && wide_fits && TK >= 64L * s.N) {
            // Long reduction: the deep schedule's 128-wide K-steps halve the barriers per
            // byte, and it keeps the lead while the wide schedule's items make fewer than
            // about five rounds over the workgroups, i.e. while what the last, partial round
            // wastes outweighs the wide tile's fewer load bytes.  Measured gate/up, deep / wide
            // in us, by rounds of the wide items: large layer T = 4096 (128 tiles, 3.0 rounds)
            // 566 / 567, T = 8192 (131 tiles, 3.1) 626 / 648, T = 16384 (256 tiles, 6.0)
            // 858 / 785; Mixtral shape T = 2048 (24 tiles of 56 column tiles, 5.25) 650 / 613,
            // with every pair kept (7.0) 1000 / 895, T = 4096 1127 / 1028.  Both are enqueued
            // and the tile count picks one, as above.
            const int max_deep = (5 * 256 - 1) * 2 / nct;
            tiles_hi = max_deep;
            BEAM_LAUNCH_TILE(8, 1, true);
            if (hipPeekAtLastError() != hipSuccess) return;   // the caller reads and reports it
            tiles_lo = max_deep + 1;
            tiles_hi = 0x7fffffff;
        } else if (packed && (s.H >= 4096 || TK <= 256L * s.N)) {
            BEAM_LAUNCH_TILE(8, 1, true);
            return;
        }
    }
    // "Wide": where the output width allows, the two workgroups of a CU become one of eight
    // wavefronts side by side on a 128 x 512 tile: the same registers, LDS and MFMA work per
    // CU, but the activation tile is loaded (and gathered) once for twice the columns, a sixth
    // fewer load bytes per MFMA, which is what the K-step's time follows.  Measured against
    // the dense schedule (Qwen3 shape): gate/up 799 -> 767 us at T = 16384 with every pair
    // kept, 210 -> 197 at 15 %, 456 -> 441 at T = 8192; down 317 -> 305 at T = 8192,
    // Mixtral shape T = 2048 419 -> 391, large layer T = 8192 349 -> 330.
    if (wide_fits) {
        ffn_tile_kernel<kWavesM, kKSteps, 1, GATE_UP, true, 8><<<256, 512, 0, st>>>(
            a, w, offsets, perm, wl.hdr, wl.tile_expert, wl.tile_row0, hidden, y, s.H, s.K, s.I,
            nct / 2, k_split, (size_t)s.T * s.K * s.H, want, y16, tiles_lo, tiles_hi);
        return;
    }
    if (packed) BEAM_LAUNCH_TILE(kKSteps, kWorkgroupsPerCU, true);
    else BEAM_LAUNCH_TILE(kKSteps, kWorkgroupsPerCU, false);
#undef BEAM_LAUNCH_TILE
}

hipError_t launch_gate_up_tiled(const beam_shape &s, const void *x, const void *w_gate_up,
                                const int32_t *offsets, const int32_t *perm, const WorkList &wl,
                                void *hidden, hipStream_t st, int want) {
    launch_tile<true>(s, (const bf16_t *)x, (const bf16_t *)w_gate_up, offsets, perm, wl,
                      (bf16_t *)hidden, nullptr, s.I / (kTileN / 2), 1, st, want);
    return hipGetLastError();
}

// k_split > 1: y_pairs holds k_split arrays [T*K,H] of partial sums, one per part of
// the reduction; I / (16 * kKSteps) must be a multiple of k_split.
// y16 (with k_split == 1 only): y_pairs is an array of half-precision rows.
hipError_t launch_down_tiled(const beam_shape &s, const void *hidden, const void *w_down,
                             const int32_t *offsets, const WorkList &wl, float *y_pairs,
                             hipStream_t st, int k_split, int want, bool y16) {
    if (y16 && k_split != 1) return hipErrorInvalidValue;
    launch_tile<false>(s, (const bf16_t *)hidden, (const bf16_t *)w_down, offsets, nullptr, wl,
                       nullptr, y_pairs, s.H / kTileN, k_split, st, want, y16 ? 1 : 0);
    return hipGetLastError();
}

// ---------------------------------------------------------------------------
// Router and mask heads for prefill batches (paper Sec. 3.2 Step 1, Eq. 5): the
// [T,H] x [H,2N] product is the same problem as a down GEMM of one "expert" with
// 2N output features, so it runs on the tile body above: x tiles through LDS,
// the 2N head rows, repacked into fragment order at every call (they are 1 MB;
// the caller's layout stays plain), straight into the MFMA registers.  Output:
// fp32 [T,2N], router columns first.
// ---------------------------------------------------------------------------
__global__ __launch_bounds__(256) void pack_heads_kernel(const uint4 *__restrict__ w_router,
                                                         const uint4 *__restrict__ w_mask,
                                                         uint4 *__restrict__ dst, int N, int H) {
    const int ksteps = H >> 4;
    const int rows = (2 * N + kTileN - 1) / kTileN * kTileN;  // zero rows pad the last column tile
    const int total = rows * (H >> 3);
    for (int o = blockIdx.x * 256 + threadIdx.x; o < total; o += gridDim.x * 256) {
        const int l = o & 63;
        const int frag = o >> 6;
        const int ks = frag % ksteps;
        const int rb = frag / ksteps;
        const int row = rb * 32 + (l & 31);
        uint4 v = make_uint4(0u, 0u, 0u, 0u);
        if (row < 2 * N) {
            const uint4 *src = row < N ? w_router + (size_t)row * (H >> 3)
                                       : w_mask + (size_t)(row - N) * (H >> 3);
            v = src[ks * 2 + (l >> 5)];
        }
        dst[o] = v;
    }
}

// 64-row tiles: the output is only 2N wide, so the row tiles alone have to fill
// the chip (T = 16384 gives 256 of them).
constexpr int kLogitsM = 64;
// 128-wide K-steps: with at most one item per workgroup the kernel is one latency
// chain per K-step, so fewer, larger steps
constexpr int kLogitsKS = 8;

__global__ __launch_bounds__(256, 2) void logits_tile_kernel(
    const bf16_t *__restrict__ x, const bf16_t *__restrict__ packed_heads,
    float *__restrict__ logits2, int Tn, int H, int N2, int k_split) {
    __shared__ u32x4 As[2 * kLogitsM * 2 * kLogitsKS];
    const int nct = (N2 + kTileN - 1) / kTileN;
    const int n_base = ((Tn + kLogitsM - 1) / kLogitsM) * nct;
    const int n_work = n_base * k_split;
    auto next_item = [&](int &round, TileItem &it) -> bool {
        const int item_s = blockIdx.x + round * gridDim.x;
        if (item_s >= n_work) return false;
        const int slice = item_s / n_base;
        const int item = item_s - slice * n_base;
        const int tile = item / nct;
        it.e = 0;
        it.row0 = tile * kLogitsM;
        it.row_end = Tn;
        it.col_tile = item - tile * nct;
        it.slice = slice;
        return true;
    };
    // down-GEMM roles: output width N2, reduction length H, a single expert
    ffn_tile_run<kLogitsM, kWavesM, kLogitsKS, false, true, true, true, 4>(
        As, x, packed_heads, nullptr, nullptr, logits2, N2, 1, H, false, false, k_split,
        (size_t)Tn * N2, next_item);
}

bool logits_tiled_supported(const beam_shape &s) {
    return s.dtype == BEAM_BF16 && s.T > 512 && s.H % 256 == 0 &&
           (long)s.T * s.H < (1L << 32);
}

// With 64-row tiles and at most two column tiles a batch of a few thousand tokens gives
// fewer items than CUs, and an item is one latency chain per K-step (load the x tile,
// store it to LDS, barrier, multiply).  Cutting the reduction into parts gives every CU
// an item: each part writes its own [T,2N] array and every reader of the logits adds the
// parts in order (LogitParts).  Up to one item per CU: beyond that (measured at 512
// items) the kernel gains nothing, all workgroups pull the same 1 MB of head weights
// through L2, and the readers pay for the extra parts.
int logits_split_k(const beam_shape &s) {
    if (!logits_tiled_supported(s)) return 1;
    const long items = ((s.T + kLogitsM - 1) / kLogitsM) * ((2L * s.N + kTileN - 1) / kTileN);
    int k = 1;
    while (k < 4 && items * k * 2 <= 256 && (s.H / (16 * kLogitsKS)) % (2 * k) == 0) k *= 2;
    return k;
}

hipError_t launch_logits_tiled(const beam_shape &s, const void *x, const void *w_router,
                               const void *w_mask, void *packed_heads, float *logits2,
                               hipStream_t st) {
    pack_heads_kernel<<<256, 256, 0, st>>>((const uint4 *)w_router, (const uint4 *)w_mask,
                                           (uint4 *)packed_heads, s.N, s.H);
    BEAM_CHECK_LAUNCH();
    const int k_split = logits_split_k(s);
    const int n_work =
        ((s.T + kLogitsM - 1) / kLogitsM) * ((2 * s.N + kTileN - 1) / kTileN) * k_split;
    const int grid = n_work < 512 ? n_work : 512;
    logits_tile_kernel<<<grid, 256, 0, st>>>((const bf16_t *)x, (const bf16_t *)packed_heads,
                                             logits2, s.T, s.H, 2 * s.N, k_split);
    return hipGetLastError();
}

// ---------------------------------------------------------------------------
// One-time repack of plain row-major expert weights into MFMA fragment order
// (see BEAM_WEIGHTS_PACKED in beam.h).  One thread per 16-byte piece; writes are
// contiguous.  rows32 = blocks of 32 output rows per expert, ksteps = Kd / 16.
// ---------------------------------------------------------------------------
template <bool GATE_UP>
__global__ __launch_bounds__(256) void pack_weights_kernel(const uint4 *__restrict__ src,
                                                           uint4 *__restrict__ dst, int N,
                                                           int rows, int kd, int I) {
    const size_t total = (size_t)N * rows * (kd >> 3);
    const int ksteps = kd >> 4;
    const int rows32 = rows >> 5;
    for (size_t o = (size_t)blockIdx.x * 256 + threadIdx.x; o < total;
         o += (size_t)gridDim.x * 256) {
        const int l = (int)(o & 63);
        size_t frag = o >> 6;
        const int ks = (int)(frag % ksteps);
        frag /= ksteps;
        const int rb = (int)(frag % rows32);
        const int e = (int)(frag / rows32);
        const int c = l & 31;
        int row;
        if constexpr (GATE_UP) {
            row = (rb & 1) ? I + (rb >> 1) * 32 + c : (rb >> 1) * 32 + c;
        } else {
            row = rb * 32 + c;
        }
        dst[o] = src[((size_t)e * rows + row) * (kd >> 3) + ks * 2 + (l >> 5)];
    }
}

hipError_t launch_pack_weights(const beam_shape &s, const void *w_gate_up, const void *w_down,
                               void *w_gate_up_packed, void *w_down_packed, hipStream_t st) {
    pack_weights_kernel<true><<<4096, 256, 0, st>>>((const uint4 *)w_gate_up,
                                                    (uint4 *)w_gate_up_packed, s.N, 2 * s.I, s.H,
                                                    s.I);
    BEAM_CHECK_LAUNCH();
    pack_weights_kernel<false><<<4096, 256, 0, st>>>((const uint4 *)w_down, (uint4 *)w_down_packed,
                                                     s.N, s.H, s.I, s.I);
    return hipGetLastError();
}

}  // namespace beam

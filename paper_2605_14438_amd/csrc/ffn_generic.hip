// GLU experts (paper Eq. 3, delta = SiLU) on the kept pairs, any dtype, plain
// fp32 FMAs: one wavefront per output element, lanes stride over the reduction
// dimension.  This is the path for fp32 layers and for bf16 shapes outside the
// MFMA kernels' envelope; it is correct for every supported shape, not fast.
#include "common.hpp"

namespace beam {

// Expert that owns grouped row p: the e with offsets[e] <= p < offsets[e+1].
__device__ __forceinline__ int expert_of_row(const int32_t *offsets, int N, int p) {
    int lo = 0, hi = N;  // invariant: offsets[lo] <= p < offsets[hi]
    while (hi - lo > 1) {
        const int mid = (lo + hi) >> 1;
        if (offsets[mid] <= p) lo = mid; else hi = mid;
    }
    return lo;
}

// hidden[p, j] = SiLU(x_t . W_gate[j]) * (x_t . W_up[j]); one workgroup per row.
template <typename T>
__global__ __launch_bounds__(256) void gate_up_generic_kernel(
    const T *__restrict__ x, const T *__restrict__ w_gate_up, const int32_t *__restrict__ offsets,
    const int32_t *__restrict__ perm, const int32_t *__restrict__ num_pairs,
    T *__restrict__ hidden, int H, int N, int K, int I) {
    const int p = blockIdx.x;
    if (p >= *num_pairs) return;
    const int lane = threadIdx.x & 63;
    const int wave = threadIdx.x >> 6;
    const int e = expert_of_row(offsets, N, p);
    const int t = perm[p] / K;
    const T *xr = x + (size_t)t * H;
    const T *wg = w_gate_up + (size_t)e * 2 * I * H;
    for (int j = blockIdx.y * 4 + wave; j < I; j += 4 * gridDim.y) {
        const T *g_row = wg + (size_t)j * H;
        const T *u_row = wg + (size_t)(I + j) * H;
        float ag = 0.0f, au = 0.0f;
        for (int h = lane * 4; h < H; h += 256) {
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const float xv = load_f32(xr + h + q);
                ag = fmaf(xv, load_f32(g_row + h + q), ag);
                au = fmaf(xv, load_f32(u_row + h + q), au);
            }
        }
        ag = wave_sum(ag);
        au = wave_sum(au);
        if (lane == 0) store_from_f32(hidden + (size_t)p * I + j, silu(ag) * au);
    }
}

// y_pairs[p, c] = hidden[p, :] . W_down[c, :]
template <typename T>
__global__ __launch_bounds__(256) void down_generic_kernel(
    const T *__restrict__ hidden, const T *__restrict__ w_down,
    const int32_t *__restrict__ offsets, const int32_t *__restrict__ num_pairs,
    float *__restrict__ y_pairs, int H, int N, int I) {
    const int p = blockIdx.x;
    if (p >= *num_pairs) return;
    const int lane = threadIdx.x & 63;
    const int wave = threadIdx.x >> 6;
    const int e = expert_of_row(offsets, N, p);
    const T *hr = hidden + (size_t)p * I;
    const T *wd = w_down + (size_t)e * H * I;
    for (int c = blockIdx.y * 4 + wave; c < H; c += 4 * gridDim.y) {
        const T *row = wd + (size_t)c * I;
        float acc = 0.0f;
        for (int j = lane * 4; j < I; j += 256) {
#pragma unroll
            for (int q = 0; q < 4; ++q) acc = fmaf(load_f32(hr + j + q), load_f32(row + j + q), acc);
        }
        acc = wave_sum(acc);
        if (lane == 0) y_pairs[(size_t)p * H + c] = acc;
    }
}

static dim3 generic_grid(const beam_shape &s) {
    const long TK = (long)s.T * s.K;
    // grid.y splits the output features of a row so small batches still fill the chip
    int split = 1;
    while (split < 64 && TK * split < 2048) split *= 2;
    return dim3((unsigned)TK, split);
}

hipError_t launch_gate_up_generic(const beam_shape &s, const void *x, const void *w_gate_up,
                                  const int32_t *offsets, const int32_t *perm,
                                  const int32_t *num_pairs, void *hidden, hipStream_t st) {
    const dim3 grid = generic_grid(s);
    if (s.dtype == BEAM_BF16)
        gate_up_generic_kernel<bf16_t><<<grid, 256, 0, st>>>(
            (const bf16_t *)x, (const bf16_t *)w_gate_up, offsets, perm, num_pairs,
            (bf16_t *)hidden, s.H, s.N, s.K, s.I);
    else
        gate_up_generic_kernel<float><<<grid, 256, 0, st>>>(
            (const float *)x, (const float *)w_gate_up, offsets, perm, num_pairs, (float *)hidden,
            s.H, s.N, s.K, s.I);
    return hipGetLastError();
}

hipError_t launch_down_generic(const beam_shape &s, const void *hidden, const void *w_down,
                               const int32_t *offsets, const int32_t *num_pairs, float *y_pairs,
                               hipStream_t st) {
    const dim3 grid = generic_grid(s);
    if (s.dtype == BEAM_BF16)
        down_generic_kernel<bf16_t><<<grid, 256, 0, st>>>((const bf16_t *)hidden,
                                                          (const bf16_t *)w_down, offsets,
                                                          num_pairs, y_pairs, s.H, s.N, s.I);
    else
        down_generic_kernel<float><<<grid, 256, 0, st>>>((const float *)hidden,
                                                         (const float *)w_down, offsets, num_pairs,
                                                         y_pairs, s.H, s.N, s.I);
    return hipGetLastError();
}

}  // namespace beam

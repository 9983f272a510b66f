// ELL SpMV (Section II-B: at most K entries per row, one K-wide value slab and one K-wide column slab).
// Slot-major storage, one row per lane: value and column reads are contiguous across the wave.  Rows are packed
// from slot 0, so the first padding marker (col = -1) ends a row.
#include "dev_common.hpp"
#include "mo_internal.hpp"

namespace mo {

constexpr int ELL_B = 256;
// The slot-split kernel pays off while one-row-per-lane blocks cannot fill the chip (measured: faster up to about
// 260 000 rows at K = 27, slower beyond; no gain for K < 16).
constexpr int64_t ELL_SPLIT_MAX_ROWS = 300000;
constexpr int64_t ELL_SPLIT_MIN_K = 16;

template <typename T>
__global__ __launch_bounds__(ELL_B) void k_ell(const int32_t *__restrict__ col, const T *__restrict__ val, int64_t m, int64_t K,
                                                int64_t ld, const T *__restrict__ x, T *__restrict__ y)
{
    const int64_t lb = xcd_block(blockIdx.x, gridDim.x);
    const int64_t row = lb * ELL_B + threadIdx.x;
    if (row >= m) return;
    T sum = (T)0;
    const int32_t *c = col + row;
    const T *v = val + row;
#pragma unroll 4
    for (int64_t s = 0; s < K; ++s) {
        const int32_t j = ld_stream(c + s * ld);
        if (j >= 0) sum += ld_stream(v + s * ld) * x[j];
    }
    st_stream(y + row, sum);
}

// Small matrices: one row per lane leaves most of the chip idle and makes every lane walk all K slots in sequence.
// Here a block owns 64 rows and its four waves take the slots s = w, w + 4, ...; the four partial sums of a row are
// added in wave order through LDS (fixed order, so reruns are bit-identical).
template <typename T>
__global__ __launch_bounds__(ELL_B) void k_ell_split(const int32_t *__restrict__ col, const T *__restrict__ val, int64_t m, int64_t K,
                                                      int64_t ld, const T *__restrict__ x, T *__restrict__ y)
{
    constexpr int NW = ELL_B / WAVE;
    __shared__ T part[NW][WAVE];
    const int lane = lane_id(), w = threadIdx.x / WAVE;
    const int64_t row = (int64_t)blockIdx.x * WAVE + lane;
    T sum = (T)0;
    if (row < m) {
        const int32_t *c = col + row;
        const T *v = val + row;
#pragma unroll 4
        for (int64_t s = w; s < K; s += NW) {
            const int32_t j = ld_stream(c + s * ld);
            if (j >= 0) sum += ld_stream(v + s * ld) * x[j];
        }
    }
    part[w][lane] = sum;
    __syncthreads();
    if (w == 0 && row < m) {
        T t = part[0][lane];
#pragma unroll
        for (int q = 1; q < NW; ++q) t += part[q][lane];
        y[row] = t;
    }
}

template <typename T>
static mo_status ell_typed(const mo_matrix &a, const void *x, void *y, hipStream_t s)
{
    if (a.m <= ELL_SPLIT_MAX_ROWS && a.k >= ELL_SPLIT_MIN_K) {
        const unsigned g = (unsigned)((a.m + WAVE - 1) / WAVE);
        hipLaunchKernelGGL(k_ell_split<T>, dim3(g), dim3(ELL_B), 0, s, a.ell_col, (const T *)a.ell_val, a.m, a.k, a.ld, (const T *)x, (T *)y);
        MO_LAUNCH_CHECK();
        return MO_OK;
    }
    const unsigned grid = (unsigned)((a.m + ELL_B - 1) / ELL_B);
    hipLaunchKernelGGL(k_ell<T>, dim3(grid), dim3(ELL_B), 0, s, a.ell_col, (const T *)a.ell_val, a.m, a.k, a.ld, (const T *)x, (T *)y);
    MO_LAUNCH_CHECK();
    return MO_OK;
}

mo_status spmv_ell(const mo_matrix &a, const void *x, void *y, hipStream_t s)
{
    return a.dtype == MO_F32 ? ell_typed<float>(a, x, y, s) : ell_typed<double>(a, x, y, s);
}

}  // namespace mo

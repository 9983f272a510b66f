// ELL SpMV (Section II-B: at most K entries per row, one K-wide value slab and one K-wide column slab).
// Slot-major storage, one row per lane: value and column reads are contiguous across the wave.  Rows are packed
// from slot 0, so the first padding marker (col = -1) ends a row.
#include "dev_common.hpp"
#include "mo_internal.hpp"

namespace mo {

constexpr int ELL_B = 256;
constexpr int ELL_U = 8;   // slots fetched together

// sum += A(row, slots s, s + step, ...) * x over the slots [s0, s1) of one row.  The loads of ELL_U slots are issued
// together and unconditionally (a padded slot reads x[0] twice and is masked out of the sum), so that no load waits
// for a branch on the one before it.  The order of the additions is the slot order.
template <typename T>
__device__ __forceinline__ T ell_row_sum(const int32_t *__restrict__ c, const T *__restrict__ v, int64_t ld, int64_t s0, int64_t s1,
                                         int64_t step, const T *__restrict__ x)
{
    T sum = (T)0;
    int64_t s = s0;
    for (; s + (ELL_U - 1) * step < s1; s += ELL_U * step) {
        int32_t j[ELL_U];
        T a[ELL_U], xv[ELL_U];
#pragma unroll
        for (int u = 0; u < ELL_U; ++u) j[u] = ld_stream(c + (s + u * step) * ld);
#pragma unroll
        for (int u = 0; u < ELL_U; ++u) {   // a padded slot reads x[0] in place of its value: no slab traffic for padding
            a[u] = ld_stream(j[u] >= 0 ? v + (s + u * step) * ld : x);
            xv[u] = x[j[u] >= 0 ? j[u] : 0];
        }
#pragma unroll
        for (int u = 0; u < ELL_U; ++u) sum += j[u] >= 0 ? a[u] * xv[u] : (T)0;
    }
    for (; s < s1; s += step) {
        const int32_t j = ld_stream(c + s * ld);
        const T a = ld_stream(j >= 0 ? v + s * ld : x);
        const T xv = x[j >= 0 ? j : 0];
        sum += j >= 0 ? a * xv : (T)0;
    }
    return sum;
}

template <typename T>
__global__ __launch_bounds__(ELL_B) void k_ell(const int32_t *__restrict__ col, const T *__restrict__ val, int64_t m, int64_t K,
                                                int64_t ld, const T *__restrict__ x, T *__restrict__ y)
{
    const int64_t lb = xcd_block(blockIdx.x, gridDim.x);
    const int64_t row = lb * ELL_B + threadIdx.x;
    if (row >= m) return;
    st_stream(y + row, ell_row_sum<T>(col + row, val + row, ld, 0, K, 1, x));
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
    if (row < m) sum = ell_row_sum<T>(col + row, val + row, ld, w, K, NW, x);
    part[w][lane] = sum;
    __syncthreads();
    if (w == 0 && row < m) {
        T t = part[0][lane];
#pragma unroll
        for (int q = 1; q < NW; ++q) t += part[q][lane];
        y[row] = t;
    }
}

// HYB whose rows keep only a few entries in the COO part: the row's lane adds its own COO run (found through the
// positions of the row runs that the handle keeps) right after its ELL slots, so y is written once by one kernel
// instead of being written by the ELL kernel and read, updated and written again by the COO kernel.
template <typename T>
__global__ __launch_bounds__(ELL_B) void k_ell_hyb(const int32_t *__restrict__ col, const T *__restrict__ val, int64_t m, int64_t K,
                                                    int64_t ld, const int32_t *__restrict__ coo_rp, const int32_t *__restrict__ ccol,
                                                    const T *__restrict__ cval, const T *__restrict__ x, T *__restrict__ y)
{
    const int64_t lb = xcd_block(blockIdx.x, gridDim.x);
    const int64_t row = lb * ELL_B + threadIdx.x;
    if (row >= m) return;
    const int32_t p0 = coo_rp[row], p1 = coo_rp[row + 1];
    T sum = ell_row_sum<T>(col + row, val + row, ld, 0, K, 1, x);
    for (int32_t p = p0; p < p1; ++p) sum += cval[p] * x[ccol[p]];
    st_stream(y + row, sum);
}

template <typename T>
static mo_status hyb_fused_typed(const mo_matrix &a, const void *x, void *y, hipStream_t s)
{
    const unsigned grid = (unsigned)((a.m + ELL_B - 1) / ELL_B);
    hipLaunchKernelGGL(k_ell_hyb<T>, dim3(grid), dim3(ELL_B), 0, s, a.ell_col, (const T *)a.ell_val, a.m, a.k, a.ld, a.coo_rp, a.coo_col,
                       (const T *)a.coo_val, (const T *)x, (T *)y);
    MO_LAUNCH_CHECK();
    return MO_OK;
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

mo_status spmv_hyb_fused(const mo_matrix &a, const void *x, void *y, hipStream_t s)
{
    return a.dtype == MO_F32 ? hyb_fused_typed<float>(a, x, y, s) : hyb_fused_typed<double>(a, x, y, s);
}

mo_status spmv_ell(const mo_matrix &a, const void *x, void *y, hipStream_t s)
{
    return a.dtype == MO_F32 ? ell_typed<float>(a, x, y, s) : ell_typed<double>(a, x, y, s);
}

}  // namespace mo

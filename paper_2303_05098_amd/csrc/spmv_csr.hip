// CSR SpMV (Section II-B: values and column indices stored row after row, row_ptr marks the row boundaries).
//
// Vector kernel: an aligned group of LANES lanes (2..64, chosen from the mean row length at conversion time) owns
// one row, strides over its entries with coalesced loads and reduces with shuffles.  The association order is
// fixed by LANES, so results are bit-identical from run to run.  Neighbouring rows are kept on the same XCD so that
// the part of x a band or stencil touches stays in that XCD's L2.
#include "dev_common.hpp"
#include "mo_internal.hpp"

namespace mo {

constexpr int CSR_B = 256;

template <typename T, int LANES, bool ACC>
__global__ __launch_bounds__(CSR_B) void k_csr_vector(const int32_t *__restrict__ row_ptr, const int32_t *__restrict__ col_idx,
                                                       const T *__restrict__ val, int64_t m, const T *__restrict__ x, T *__restrict__ y)
{
    constexpr int ROWS = CSR_B / LANES;
    const int64_t lb = xcd_block(blockIdx.x, gridDim.x);
    const int64_t row = lb * ROWS + threadIdx.x / LANES;
    const int sub = threadIdx.x % LANES;
    T sum = (T)0;
    if (row < m) {
        const int64_t lo = row_ptr[row], hi = row_ptr[row + 1];
        for (int64_t p = lo + sub; p < hi; p += LANES) sum += val[p] * x[col_idx[p]];
    }
    sum = group_sum_down(sum, LANES);
    if (sub == 0 && row < m) {
        if (ACC) y[row] += sum; else y[row] = sum;
    }
}

template <typename T, int LANES>
static mo_status launch_vec(const mo_matrix &a, const T *x, T *y, bool acc, hipStream_t s)
{
    constexpr int ROWS = CSR_B / LANES;
    const unsigned grid = (unsigned)((a.m + ROWS - 1) / ROWS);
    if (acc)
        hipLaunchKernelGGL((k_csr_vector<T, LANES, true>), dim3(grid), dim3(CSR_B), 0, s, a.csr_row_ptr, a.csr_col, (const T *)a.csr_val, a.m, x, y);
    else
        hipLaunchKernelGGL((k_csr_vector<T, LANES, false>), dim3(grid), dim3(CSR_B), 0, s, a.csr_row_ptr, a.csr_col, (const T *)a.csr_val, a.m, x, y);
    MO_LAUNCH_CHECK();
    return MO_OK;
}

template <typename T>
static mo_status csr_typed(const mo_matrix &a, const void *xv, void *yv, bool acc, hipStream_t s)
{
    const T *x = (const T *)xv;
    T *y = (T *)yv;
    switch (a.csr_lanes) {
    case 2: return launch_vec<T, 2>(a, x, y, acc, s);
    case 4: return launch_vec<T, 4>(a, x, y, acc, s);
    case 8: return launch_vec<T, 8>(a, x, y, acc, s);
    case 16: return launch_vec<T, 16>(a, x, y, acc, s);
    case 32: return launch_vec<T, 32>(a, x, y, acc, s);
    default: return launch_vec<T, 64>(a, x, y, acc, s);
    }
}

mo_status spmv_csr(const mo_matrix &a, const void *x, void *y, bool accumulate, hipStream_t s)
{
    return a.dtype == MO_F32 ? csr_typed<float>(a, x, y, accumulate, s) : csr_typed<double>(a, x, y, accumulate, s);
}

}  // namespace mo

// ELL SpMV (Section II-B: at most K entries per row, one K-wide value slab and one K-wide column slab).
// Slot-major storage, one row per lane: value and column reads are contiguous across the wave.  Rows are packed
// from slot 0, so the first padding marker (col = -1) ends a row.
#include "dev_common.hpp"
#include "mo_internal.hpp"

namespace mo {

constexpr int ELL_B = 256;

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

template <typename T>
static mo_status ell_typed(const mo_matrix &a, const void *x, void *y, hipStream_t s)
{
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

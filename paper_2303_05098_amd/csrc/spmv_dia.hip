// DIA SpMV (Section II-B: one dense slab per stored diagonal plus an integer offset per diagonal).
// y_i = sum_k val[k*ld + i] * x[i + off_k]; positions whose column falls outside [0, n) hold +0 and are skipped.
// One row per lane: slab reads and x reads are both contiguous across the wave; no index traffic at all.
#include "dev_common.hpp"
#include "mo_internal.hpp"

namespace mo {

constexpr int DIA_B = 256;

template <typename T>
__global__ __launch_bounds__(DIA_B) void k_dia(const int32_t *__restrict__ off, const T *__restrict__ val, int64_t m, int64_t n,
                                                int64_t nd, int64_t ld, const T *__restrict__ x, T *__restrict__ y)
{
    const int64_t lb = xcd_block(blockIdx.x, gridDim.x);
    const int64_t row = lb * DIA_B + threadIdx.x;
    if (row >= m) return;
    T sum = (T)0;
    const T *v = val + row;
#pragma unroll 4
    for (int64_t k = 0; k < nd; ++k) {
        const int64_t j = row + off[k];
        if (j >= 0 && j < n) sum += v[k * ld] * x[j];
    }
    y[row] = sum;
}

template <typename T>
static mo_status dia_typed(const mo_matrix &a, const void *x, void *y, hipStream_t s)
{
    const unsigned grid = (unsigned)((a.m + DIA_B - 1) / DIA_B);
    hipLaunchKernelGGL(k_dia<T>, dim3(grid), dim3(DIA_B), 0, s, a.dia_off, (const T *)a.dia_val, a.m, a.n, a.nd, a.ld, (const T *)x, (T *)y);
    MO_LAUNCH_CHECK();
    return MO_OK;
}

mo_status spmv_dia(const mo_matrix &a, const void *x, void *y, hipStream_t s)
{
    return a.dtype == MO_F32 ? dia_typed<float>(a, x, y, s) : dia_typed<double>(a, x, y, s);
}

}  // namespace mo

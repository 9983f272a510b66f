// Y = A X for k right-hand sides at once, in every format: a second operation under the tuning interface, which the
// paper defines for SpMV and leaves open for further operations (Section VI-B).  X is n x k and Y is m x k, both
// row-major, so the k values a matrix entry needs are contiguous.
//
// The product is computed in column panels of width 8, 4, 2 or 1 (k = 13 is 8 + 4 + 1): one row per lane as in the
// SpMV kernels, so the matrix is streamed coalesced once per panel, the panel's accumulators live in registers and
// the panel's values of a row of X are fetched with wide loads.  Panels are no wider than 8 because the rows of X a
// block touches must stay in the 4 MB L2 of its XCD between their uses by neighbouring rows: at 16 columns the
// 27-point stencil on 128^3 points fell out of L2 and a single pass took 3.6 times as long as at 8.
// Rows given by a row pointer (CSR, the CSR remainder of HDC, the sorted COO arrays with the positions of their row
// runs) reach the lanes through a per-wave LDS stage filled with coalesced loads, as in the conversion kernels.
// Every output is summed by one thread in a fixed order: results are bit-identical from run to run.  HYB and HDC run
// their second part in accumulate mode.
#include "dev_common.hpp"
#include "mo_internal.hpp"

namespace mo {

constexpr int MB = 256;
constexpr int RCAP = 1024;   // entries a wave stages at a time in the row-pointer kernel
constexpr int SPMM_LONG_ROW = 64;   // rows longer than this are walked by the whole wave

template <typename T, int K>
__device__ __forceinline__ void fma_row(T (&acc)[K], T a, const T *__restrict__ xr)
{
#pragma unroll
    for (int v = 0; v < K; ++v) acc[v] += a * xr[v];
}

template <typename T, int K, bool ACC>
__device__ __forceinline__ void store_row(T *__restrict__ yr, const T (&acc)[K])
{
#pragma unroll
    for (int v = 0; v < K; ++v) yr[v] = ACC ? yr[v] + acc[v] : acc[v];
}

// x and y point at the first column of the panel; ldk = k is the distance between rows of X and of Y.
template <typename T, int K>
__global__ __launch_bounds__(MB) void k_spmm_dia(const int32_t *__restrict__ off, const T *__restrict__ val, int64_t nd, int64_t ld,
                                                  int64_t m, int64_t n, int64_t ldk, const T *__restrict__ x, T *__restrict__ y)
{
    const int64_t i = xcd_block(blockIdx.x, gridDim.x) * MB + threadIdx.x;
    if (i >= m) return;
    T acc[K];
#pragma unroll
    for (int v = 0; v < K; ++v) acc[v] = (T)0;
    for (int64_t d = 0; d < nd; ++d) {
        const int64_t j = i + off[d];
        if (j >= 0 && j < n) fma_row<T, K>(acc, ld_stream(val + d * ld + i), x + j * ldk);
    }
    store_row<T, K, false>(y + i * ldk, acc);
}

template <typename T, int K>
__global__ __launch_bounds__(MB) void k_spmm_ell(const int32_t *__restrict__ col, const T *__restrict__ val, int64_t W, int64_t ld,
                                                  int64_t m, int64_t ldk, const T *__restrict__ x, T *__restrict__ y)
{
    const int64_t i = xcd_block(blockIdx.x, gridDim.x) * MB + threadIdx.x;
    if (i >= m) return;
    T acc[K];
#pragma unroll
    for (int v = 0; v < K; ++v) acc[v] = (T)0;
    for (int64_t s = 0; s < W; ++s) {
        const int32_t j = ld_stream(col + s * ld + i);
        if (j >= 0) fma_row<T, K>(acc, ld_stream(val + s * ld + i), x + (int64_t)j * ldk);
    }
    store_row<T, K, false>(y + i * ldk, acc);
}

// Rows by row pointer.  The entries of a wave's 64 rows are one contiguous run: it is staged in LDS in chunks of whole
// rows (as many consecutive rows as fit RCAP entries) and every lane walks its own row out of LDS.  Rows of more
// than SPMM_LONG_ROW entries are left to the whole wave, so that one long row does not keep 63 lanes waiting.  rp
// comes from a validated CSR or was built by the conversions, so it is non-decreasing; the conditions below still
// keep every LDS index inside the chunk.
template <typename T, int K, bool ACC>
__global__ __launch_bounds__(MB) void k_spmm_rows(const int32_t *__restrict__ rp, const int32_t *__restrict__ col,
                                                   const T *__restrict__ val, int64_t m, int64_t ldk, const T *__restrict__ x,
                                                   T *__restrict__ y)
{
    __shared__ int32_t s_col_all[(MB / WAVE) * RCAP];
    __shared__ T s_val_all[(MB / WAVE) * RCAP];
    int32_t *s_col = s_col_all + (threadIdx.x / WAVE) * RCAP;
    T *s_val = s_val_all + (threadIdx.x / WAVE) * RCAP;
    const int lane = lane_id();
    const int64_t i = xcd_block(blockIdx.x, gridDim.x) * MB + threadIdx.x;
    const bool rv = i < m;
    const int lo = rv ? rp[i] : 0, hi = rv ? rp[i + 1] : 0;
    T acc[K];
#pragma unroll
    for (int v = 0; v < K; ++v) acc[v] = (T)0;
    const bool is_long = rv && hi - lo > SPMM_LONG_ROW;
    const int nvalid = __popcll(ballot64(rv));
    int first = 0;
    while (first < nvalid) {
        const int start = __builtin_amdgcn_readlane(lo, first);
        const uint64_t fits = ballot64(rv && lo >= start && hi >= lo && hi - start <= RCAP) >> first;
        const int nrun = ~fits ? __ffsll((unsigned long long)~fits) - 1 : WAVE;
        if (nrun <= 0) { ++first; continue; }   // longer than a chunk: a long row, walked by the whole wave below
        const int last = first + nrun - 1;
        const int end = __builtin_amdgcn_readlane(hi, last);
        const int total = end - start;   // 0 .. RCAP
        if (total > 0) {
            stage_to_lds(col + start, s_col, total, lane);
            stage_to_lds(val + start, s_val, total, lane);
        }
        if (!is_long && lane >= first && lane <= last && hi <= end)
            for (int p = lo - start; p < hi - start; ++p) fma_row<T, K>(acc, s_val[p], x + (int64_t)s_col[p] * ldk);
        first = last + 1;
    }
    // Long rows: the 64 lanes share the row's entries (coalesced loads straight from memory), the K partial sums of
    // every lane are added across the wave in a fixed order, and the row's own lane keeps the result.
    uint64_t longmask = ballot64(is_long);
    while (longmask) {
        const int l = __ffsll((unsigned long long)longmask) - 1;
        longmask &= longmask - 1;
        const int rlo = __builtin_amdgcn_readlane(lo, l), rhi = __builtin_amdgcn_readlane(hi, l);
        T part[K];
#pragma unroll
        for (int v = 0; v < K; ++v) part[v] = (T)0;
        for (int p = rlo + lane; p < rhi; p += WAVE) fma_row<T, K>(part, val[p], x + (int64_t)col[p] * ldk);
#pragma unroll
        for (int v = 0; v < K; ++v) {
            const T t = wave_sum(part[v]);
            if (lane == l) acc[v] = t;
        }
    }
    if (rv && (!ACC || hi > lo)) store_row<T, K, ACC>(y + i * ldk, acc);
}

template <typename T, int K>
static mo_status spmm_panel(const mo_matrix &a, const T *x, T *y, int64_t ldk, hipStream_t s)
{
    const unsigned grid = (unsigned)((a.m + MB - 1) / MB);
    const bool dia = a.fmt == MO_DIA || (a.fmt == MO_HDC && a.nd > 0);
    if (dia) {
        hipLaunchKernelGGL((k_spmm_dia<T, K>), dim3(grid), dim3(MB), 0, s, a.dia_off, (const T *)a.dia_val, a.nd, a.ld, a.m, a.n, ldk, x, y);
        MO_LAUNCH_CHECK();
    }
    switch (a.fmt) {
    case MO_DIA:
        return MO_OK;
    case MO_ELL:
    case MO_HYB:
        hipLaunchKernelGGL((k_spmm_ell<T, K>), dim3(grid), dim3(MB), 0, s, a.ell_col, (const T *)a.ell_val, a.k, a.ld, a.m, ldk, x, y);
        MO_LAUNCH_CHECK();
        if (a.fmt == MO_HYB && a.nnz_coo > 0) {
            hipLaunchKernelGGL((k_spmm_rows<T, K, true>), dim3(grid), dim3(MB), 0, s, a.coo_rp, a.coo_col, (const T *)a.coo_val, a.m, ldk, x, y);
            MO_LAUNCH_CHECK();
        }
        return MO_OK;
    case MO_COO:
        hipLaunchKernelGGL((k_spmm_rows<T, K, false>), dim3(grid), dim3(MB), 0, s, a.coo_rp, a.coo_col, (const T *)a.coo_val, a.m, ldk, x, y);
        MO_LAUNCH_CHECK();
        return MO_OK;
    case MO_CSR:
        hipLaunchKernelGGL((k_spmm_rows<T, K, false>), dim3(grid), dim3(MB), 0, s, a.csr_row_ptr, a.csr_col, (const T *)a.csr_val, a.m, ldk, x, y);
        MO_LAUNCH_CHECK();
        return MO_OK;
    case MO_HDC:
        if (!dia) {
            hipLaunchKernelGGL((k_spmm_rows<T, K, false>), dim3(grid), dim3(MB), 0, s, a.csr_row_ptr, a.csr_col, (const T *)a.csr_val, a.m, ldk, x, y);
            MO_LAUNCH_CHECK();
        } else if (a.nnz_csr > 0) {
            hipLaunchKernelGGL((k_spmm_rows<T, K, true>), dim3(grid), dim3(MB), 0, s, a.csr_row_ptr, a.csr_col, (const T *)a.csr_val, a.m, ldk, x, y);
            MO_LAUNCH_CHECK();
        }
        return MO_OK;
    }
    return MO_E_FORMAT;
}

template <typename T>
static mo_status spmm_typed(const mo_matrix &a, const T *x, T *y, int k, hipStream_t s)
{
    int v0 = 0;
    while (v0 < k) {
        const int left = k - v0;
        if (left >= 8) { MO_TRY((spmm_panel<T, 8>(a, x + v0, y + v0, k, s))); v0 += 8; }
        else if (left >= 4) { MO_TRY((spmm_panel<T, 4>(a, x + v0, y + v0, k, s))); v0 += 4; }
        else if (left >= 2) { MO_TRY((spmm_panel<T, 2>(a, x + v0, y + v0, k, s))); v0 += 2; }
        else { MO_TRY((spmm_panel<T, 1>(a, x + v0, y + v0, k, s))); v0 += 1; }
    }
    return MO_OK;
}

mo_status spmm(const mo_matrix &a, const void *x, void *y, int k, hipStream_t s)
{
    return a.dtype == MO_F32 ? spmm_typed<float>(a, (const float *)x, (float *)y, k, s)
                             : spmm_typed<double>(a, (const double *)x, (double *)y, k, s);
}

}  // namespace mo

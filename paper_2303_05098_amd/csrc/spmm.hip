// Y = A X for k right-hand sides at once, in every format: a second operation under the tuning interface, which the
// paper defines for SpMV and leaves open for further operations (Section VI-B).  X is n x k and Y is m x k, both
// row-major, so the k values a matrix entry needs are contiguous.
//
// The product is computed in column panels of width 8, 4, 2 or 1 (k = 13 is 8 + 4 + 1): one row per lane as in the
// SpMV kernels, so the matrix is streamed coalesced once per panel, the panel's accumulators live in registers and
// the panel's values of a row of X are fetched with wide loads.  Wider panels would not help: what limits the
// product beyond 8 columns is the footprint of the rows of X that neighbouring matrix rows share, which at 16 columns
// (128-byte rows) no longer fits the 4 MB L2 of an XCD for a 27-point stencil on 128^3 points.
// Rows given by a row pointer (CSR, the CSR remainder of HDC, the sorted COO arrays with the positions of their row
// runs) reach the lanes through a per-wave LDS stage filled with coalesced loads, as in the conversion kernels.
// Every output is summed by one thread in a fixed order: results are bit-identical from run to run.  HYB and HDC run
// their second part in accumulate mode.
#include "dev_common.hpp"
#include "mo_internal.hpp"

namespace mo {

constexpr int MB = 256;
constexpr int RCAP = 1024;   // entries a wave stages at a time in the row-pointer kernel
constexpr size_t SPMM_DIA_LDS = 80 * 1024;   // LDS a block may spend on staged rows of X: two blocks per CU (one block per CU
                                             // measured 1.7x slower than the direct kernel on the banded matrix)
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

// DIA with the window plan of the SpMV kernel (offsets closer than one block of rows share a window of x): the
// block stages the windows' rows of X, K values each, in LDS once and serves every diagonal from there, instead of
// fetching K values per row and diagonal through the L1 / texture path.  One row per thread, blockDim.x rows per
// block (the block size the plan was made for).
template <typename T, int K>
__global__ __launch_bounds__(1024) void k_spmm_dia_lds(const int32_t *__restrict__ xpos, const int32_t *__restrict__ cl, int ncl,
                                                        const T *__restrict__ val, int64_t nd, int64_t ld, int64_t m, int64_t n,
                                                        int64_t ldk, const T *__restrict__ x, T *__restrict__ y)
{
    extern __shared__ __align__(16) unsigned char s_raw[];
    T *xs = reinterpret_cast<T *>(s_raw);
    const int rows = blockDim.x;
    const int64_t row0 = xcd_block(blockIdx.x, gridDim.x) * rows;
    for (int c = 0; c < ncl; ++c) {
        const int64_t first = row0 + cl[3 * c];
        const int len = cl[3 * c + 1], base = cl[3 * c + 2];
        for (int i = threadIdx.x; i < len * K; i += rows) {
            const int e = i / K, v = i - e * K;
            const int64_t j = first + e;
            xs[(base + e) * K + v] = (j >= 0 && j < n) ? x[j * ldk + v] : (T)0;
        }
    }
    __syncthreads();
    const int64_t i = row0 + threadIdx.x;
    if (i >= m) return;
    T acc[K];
#pragma unroll
    for (int v = 0; v < K; ++v) acc[v] = (T)0;
    const T *vp = val + i;
    const T *xl = xs + (int64_t)threadIdx.x * K;
#pragma unroll 4
    for (int64_t d = 0; d < nd; ++d) fma_row<T, K>(acc, ld_stream(vp + d * ld), xl + (int64_t)xpos[d] * K);
    store_row<T, K, false>(y + i * ldk, acc);
}

// coo_rp != nullptr: a HYB handle whose rows keep few entries in the COO part; the row's lane adds its own COO run.
template <typename T, int K>
__global__ __launch_bounds__(MB) void k_spmm_ell(const int32_t *__restrict__ col, const T *__restrict__ val, int64_t W, int64_t ld,
                                                  int64_t m, int64_t ldk, const int32_t *__restrict__ coo_rp,
                                                  const int32_t *__restrict__ ccol, const T *__restrict__ cval,
                                                  const T *__restrict__ x, T *__restrict__ y)
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
    if (coo_rp) {
        const int32_t p1 = coo_rp[i + 1];
        for (int32_t p = coo_rp[i]; p < p1; ++p) fma_row<T, K>(acc, cval[p], x + (int64_t)ccol[p] * ldk);
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
        if (!is_long && lane >= first && lane <= last && hi <= end) {
            constexpr int ROWS_U = K >= 8 ? 4 : 8;   // entries fetched together; fewer for wide panels (registers)
            int p = lo - start;
            const int pe = hi - start;
            for (; p + ROWS_U <= pe; p += ROWS_U) {   // ROWS_U entries at a time: their LDS reads and their gathers of X overlap
                int32_t cj[ROWS_U];
                T aj[ROWS_U];
#pragma unroll
                for (int u = 0; u < ROWS_U; ++u) { cj[u] = s_col[p + u]; aj[u] = s_val[p + u]; }
                if constexpr (K == 1) {
                    T xj[ROWS_U];
#pragma unroll
                    for (int u = 0; u < ROWS_U; ++u) xj[u] = x[(int64_t)cj[u] * ldk];
#pragma unroll
                    for (int u = 0; u < ROWS_U; ++u) acc[0] += aj[u] * xj[u];
                } else {
#pragma unroll
                    for (int u = 0; u < ROWS_U; ++u) fma_row<T, K>(acc, aj[u], x + (int64_t)cj[u] * ldk);
                }
            }
            for (; p < pe; ++p) fma_row<T, K>(acc, s_val[p], x + (int64_t)s_col[p] * ldk);
        }
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

// One column panel of the DIA part (DIA, or HDC with kept diagonals).  use_lds: the window kernel.
template <typename T, int K>
static mo_status dia_panel(const mo_matrix &a, const T *x, T *y, int64_t ldk, bool use_lds, hipStream_t s)
{
    if (use_lds) {
        const int64_t rows = (int64_t)a.dia_block * a.dia_rows;   // rows per block the window plan was made for
        const size_t lds = (size_t)a.dia_lds_elems * K * sizeof(T);
        static bool raised = false;   // more than 64 KB of dynamic LDS has to be asked for, once per kernel
        if (!raised) {
            MO_HIP(hipFuncSetAttribute((const void *)k_spmm_dia_lds<T, K>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)SPMM_DIA_LDS));
            raised = true;
        }
        hipLaunchKernelGGL((k_spmm_dia_lds<T, K>), dim3((unsigned)((a.m + rows - 1) / rows)), dim3((unsigned)rows), lds, s, a.dia_xpos,
                           a.dia_clusters, (int)a.dia_ncl, (const T *)a.dia_val, a.nd, a.ld, a.m, a.n, ldk, x, y);
    } else {
        hipLaunchKernelGGL((k_spmm_dia<T, K>), dim3((unsigned)((a.m + MB - 1) / MB)), dim3(MB), 0, s, a.dia_off, (const T *)a.dia_val, a.nd,
                           a.ld, a.m, a.n, ldk, x, y);
    }
    MO_LAUNCH_CHECK();
    return MO_OK;
}

// One column panel of everything that is not a DIA part.  after_dia: the DIA part of an HDC handle has already
// written this panel of Y, the remainder is added to it.
template <typename T, int K>
static mo_status rest_panel(const mo_matrix &a, const T *x, T *y, int64_t ldk, bool after_dia, hipStream_t s)
{
    const unsigned grid = (unsigned)((a.m + MB - 1) / MB);
    switch (a.fmt) {
    case MO_DIA:
        return MO_OK;
    case MO_ELL:
    case MO_HYB:
    {
        const bool fused = a.fmt == MO_HYB && a.nnz_coo > 0 && a.hyb_max_surplus <= HYB_FUSED_MAX_SURPLUS && a.coo_rp;
        hipLaunchKernelGGL((k_spmm_ell<T, K>), dim3(grid), dim3(MB), 0, s, a.ell_col, (const T *)a.ell_val, a.k, a.ld, a.m, ldk,
                           fused ? a.coo_rp : (const int32_t *)nullptr, a.coo_col, (const T *)a.coo_val, x, y);
        MO_LAUNCH_CHECK();
        if (a.fmt == MO_HYB && a.nnz_coo > 0 && !fused) {
            hipLaunchKernelGGL((k_spmm_rows<T, K, true>), dim3(grid), dim3(MB), 0, s, a.coo_rp, a.coo_col, (const T *)a.coo_val, a.m, ldk, x, y);
            MO_LAUNCH_CHECK();
        }
        return MO_OK;
    }
    case MO_COO:
        hipLaunchKernelGGL((k_spmm_rows<T, K, false>), dim3(grid), dim3(MB), 0, s, a.coo_rp, a.coo_col, (const T *)a.coo_val, a.m, ldk, x, y);
        MO_LAUNCH_CHECK();
        return MO_OK;
    case MO_CSR:
        hipLaunchKernelGGL((k_spmm_rows<T, K, false>), dim3(grid), dim3(MB), 0, s, a.csr_row_ptr, a.csr_col, (const T *)a.csr_val, a.m, ldk, x, y);
        MO_LAUNCH_CHECK();
        return MO_OK;
    case MO_HDC:
        if (!after_dia) {
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
    const bool dia = a.fmt == MO_DIA || (a.fmt == MO_HDC && a.nd > 0);
    if (dia) {
        // The window kernel is worth it when a panel of at least 4 columns (or all k of them) fits its LDS budget;
        // otherwise the slabs would be streamed too many times and the direct kernel with 8-column panels is used.
        int widest = 8;
        const int64_t rows = (int64_t)a.dia_block * a.dia_rows;
        bool use_lds = rows > 0 && rows <= 1024;
        if (use_lds) {
            while (widest > 1 && (size_t)a.dia_lds_elems * widest * sizeof(T) > SPMM_DIA_LDS) widest >>= 1;
            if ((size_t)a.dia_lds_elems * widest * sizeof(T) > SPMM_DIA_LDS || widest < (k < 4 ? k : 4)) { use_lds = false; widest = 8; }
        }
        for (int v0 = 0; v0 < k;) {
            const int left = k - v0 < widest ? k - v0 : widest;
            if (left >= 8) { MO_TRY((dia_panel<T, 8>(a, x + v0, y + v0, k, use_lds, s))); v0 += 8; }
            else if (left >= 4) { MO_TRY((dia_panel<T, 4>(a, x + v0, y + v0, k, use_lds, s))); v0 += 4; }
            else if (left >= 2) { MO_TRY((dia_panel<T, 2>(a, x + v0, y + v0, k, use_lds, s))); v0 += 2; }
            else { MO_TRY((dia_panel<T, 1>(a, x + v0, y + v0, k, use_lds, s))); v0 += 1; }
        }
    }
    for (int v0 = 0; v0 < k;) {
        const int left = k - v0;
        if (left >= 8) { MO_TRY((rest_panel<T, 8>(a, x + v0, y + v0, k, dia, s))); v0 += 8; }
        else if (left >= 4) { MO_TRY((rest_panel<T, 4>(a, x + v0, y + v0, k, dia, s))); v0 += 4; }
        else if (left >= 2) { MO_TRY((rest_panel<T, 2>(a, x + v0, y + v0, k, dia, s))); v0 += 2; }
        else { MO_TRY((rest_panel<T, 1>(a, x + v0, y + v0, k, dia, s))); v0 += 1; }
    }
    return MO_OK;
}

mo_status spmm(const mo_matrix &a, const void *x, void *y, int k, hipStream_t s)
{
    return a.dtype == MO_F32 ? spmm_typed<float>(a, (const float *)x, (float *)y, k, s)
                             : spmm_typed<double>(a, (const double *)x, (double *)y, k, s);
}

}  // namespace mo

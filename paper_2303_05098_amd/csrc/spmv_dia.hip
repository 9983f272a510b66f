// DIA SpMV (Section II-B: one dense slab per stored diagonal plus an integer offset per diagonal), and the fused
// HDC kernel (true diagonals as DIA, the remainder as CSR).
//
// y_i = sum_k val[k*ld + i] * x[i + off_k].  One row per lane, so slab reads are contiguous across the wave and are
// streamed past the caches; no index traffic at all.  The x operand is what limits a naive version: every diagonal
// re-reads a B-row window of x through L1/L2, which doubles the traffic below the CU.  Diagonals whose offsets are
// close (a stencil's dx = -1, 0, +1; a band's -2..2) read almost the same window, so at conversion time the offsets
// are grouped into clusters and each block stages one window per cluster in LDS, once, and serves all diagonals of
// the cluster from there.  Columns outside [0, n) are staged as 0; the matching slab positions hold +0 by
// construction, so the inner loop needs no bounds test.
#include "dev_common.hpp"
#include "mo_internal.hpp"

namespace mo {

constexpr int DIA_B = 256;

// ---------------------------------------------------------------------------------------------- direct kernels
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
    for (int64_t k = 0; k < nd; ++k) {   // loads without conditions (x index clamped), so that the unrolled ones overlap
        const int64_t j = row + off[k];
        const bool in = j >= 0 && j < n;
        const T a = ld_stream(v + k * ld);
        const T xv = x[in ? j : 0];
        sum += in ? a * xv : (T)0;
    }
    st_stream(y + row, sum);
}

template <typename T>
__global__ __launch_bounds__(DIA_B) void k_hdc_fused(const int32_t *__restrict__ off, const T *__restrict__ val, int64_t m, int64_t n,
                                                      int64_t nd, int64_t ld, const int32_t *__restrict__ row_ptr,
                                                      const int32_t *__restrict__ col_idx, const T *__restrict__ cval,
                                                      const T *__restrict__ x, T *__restrict__ y)
{
    const int64_t lb = xcd_block(blockIdx.x, gridDim.x);
    const int64_t row = lb * DIA_B + threadIdx.x;
    if (row >= m) return;
    const int32_t lo = row_ptr[row], hi = row_ptr[row + 1];
    T sum = (T)0;
    const T *v = val + row;
#pragma unroll 4
    for (int64_t k = 0; k < nd; ++k) {   // loads without conditions (x index clamped), so that the unrolled ones overlap
        const int64_t j = row + off[k];
        const bool in = j >= 0 && j < n;
        const T a = ld_stream(v + k * ld);
        const T xv = x[in ? j : 0];
        sum += in ? a * xv : (T)0;
    }
    for (int32_t p = lo; p < hi; ++p) sum += cval[p] * x[col_idx[p]];
    st_stream(y + row, sum);
}

// ---------------------------------------------------------------------------------------------- LDS-staged kernels
// cl[3c] = lowest offset of cluster c, cl[3c+1] = staged length (span + rows per block), cl[3c+2] = LDS base.
// xpos[k] = LDS position of x[row0 + off_k] for the block's first row.
//
// Every thread owns R consecutive rows (R = 1 for fp64, 2 for fp32 so that a lane still moves 8 bytes per load).
//
// HDC: the CSR remainder of the block's rows is one contiguous run of entries.  It is handled entry-parallel, not
// row by row: the block multiplies those entries with their gathered x values into an LDS buffer (in chunks of
// HDC_CHUNK entries, normally a single one), and each row then adds its own slice of that buffer to its diagonal
// sum, in entry order.  A row-by-row loop would spend most of its memory instructions on the few lanes whose row
// has a remainder at all.
constexpr int HDC_CHUNK = 1024;

template <typename T, int R> struct RowVec;
template <> struct RowVec<double, 1> { using type = double; };
template <> struct RowVec<float, 1> { using type = float; };
template <> struct RowVec<double, 2> { using type = dbl2v; };
template <> struct RowVec<float, 2> { using type = flt2v; };

template <typename T, int R>
__device__ __forceinline__ void load_rows(const T *p, T (&out)[R])
{
    if constexpr (R == 1) out[0] = ld_stream(p);
    else {
        const typename RowVec<T, 2>::type v = ld_stream(reinterpret_cast<const typename RowVec<T, 2>::type *>(p));
        out[0] = v.x; out[1] = v.y;
    }
}

template <typename T, int B, int R, bool HDC>
__global__ __launch_bounds__(B) void k_dia_lds(const int32_t *__restrict__ xpos, const int32_t *__restrict__ cl, int ncl,
                                               const T *__restrict__ val, int64_t m, int64_t n, int64_t nd, int64_t ld,
                                               const int32_t *__restrict__ row_ptr, const int32_t *__restrict__ col_idx,
                                               const T *__restrict__ cval, const T *__restrict__ x, T *__restrict__ y)
{
    constexpr int ROWS = B * R;
    extern __shared__ __align__(16) unsigned char s_raw[];
    T *xs = reinterpret_cast<T *>(s_raw);
    __shared__ int32_t rps[HDC ? ROWS + 1 : 1];
    __shared__ T prod[HDC ? HDC_CHUNK : 1];
    const int64_t lb = xcd_block(blockIdx.x, gridDim.x);
    const int64_t row0 = lb * ROWS;
    const int64_t row = row0 + (int64_t)threadIdx.x * R;
    // HDC: the remainder entries of this block are [blk_lo, blk_lo + nrem).  The first chunk's columns and values are
    // requested right away, their x values right after the barrier, and the products are only needed after the
    // diagonal stream, so none of these latencies is exposed on its own.
    int32_t blk_lo = 0, nrem = 0, first_c = 0;
    T first_v = (T)0;
    bool first_on = false;
    if (HDC) {
        const int64_t rend = row0 + ROWS < m ? row0 + ROWS : m;
        blk_lo = row_ptr[row0];
        nrem = row_ptr[rend] - blk_lo;
        first_on = (int)threadIdx.x < nrem && (int)threadIdx.x < HDC_CHUNK;
        if (first_on) { first_c = col_idx[blk_lo + threadIdx.x]; first_v = cval[blk_lo + threadIdx.x]; }
    }
    for (int c = 0; c < ncl; ++c) {
        const int64_t first = row0 + cl[3 * c];
        const int len = cl[3 * c + 1], base = cl[3 * c + 2];
        for (int i = threadIdx.x; i < len; i += B) {
            const int64_t j = first + i;
            xs[base + i] = (j >= 0 && j < n) ? x[j] : (T)0;
        }
    }
    if (HDC) {
        for (int i = threadIdx.x; i <= ROWS; i += B) {
            const int64_t r = row0 + i;
            rps[i] = row_ptr[r < m ? r : m];
        }
    }
    __syncthreads();
    T sum[R];
#pragma unroll
    for (int j = 0; j < R; ++j) sum[j] = (T)0;
    T p_first = (T)0;
    if (HDC && first_on) p_first = first_v * x[first_c];
    if (row < m) {   // ld is a multiple of 64 and row a multiple of R, so a vector of R rows never leaves the slab
        const T *v = val + row;
        const T *xl = xs + threadIdx.x * R;
#pragma unroll 4
        for (int64_t k = 0; k < nd; ++k) {
            T a[R];
            load_rows<T, R>(v + k * ld, a);
            const T *xk = xl + xpos[k];
#pragma unroll
            for (int j = 0; j < R; ++j) sum[j] += a[j] * xk[j];
        }
    }
    if (HDC && nrem > 0) {   // nrem is uniform across the block
        for (int32_t c0 = 0; c0 < nrem; c0 += HDC_CHUNK) {
            if (c0 == 0) {
                if ((int)threadIdx.x < nrem && (int)threadIdx.x < HDC_CHUNK) prod[threadIdx.x] = p_first;
                for (int e = threadIdx.x + B; e < HDC_CHUNK && e < nrem; e += B) prod[e] = cval[blk_lo + e] * x[col_idx[blk_lo + e]];
            } else {
                for (int e = threadIdx.x; e < HDC_CHUNK && c0 + e < nrem; e += B) prod[e] = cval[blk_lo + c0 + e] * x[col_idx[blk_lo + c0 + e]];
            }
            __syncthreads();
#pragma unroll
            for (int j = 0; j < R; ++j) {
                int lo = rps[threadIdx.x * R + j] - blk_lo - c0, hi = rps[threadIdx.x * R + j + 1] - blk_lo - c0;
                lo = lo < 0 ? 0 : lo;
                hi = hi > HDC_CHUNK ? HDC_CHUNK : hi;
                for (int e = lo; e < hi; ++e) sum[j] += prod[e];
            }
            __syncthreads();
        }
    }
    if (row < m) {
        if constexpr (R == 1) st_stream(y + row, sum[0]);
        else {
            // m need not be even: the last thread may own a single row
            if (row + 1 < m) {
                typename RowVec<T, 2>::type o;
                o.x = sum[0]; o.y = sum[1];
                st_stream(reinterpret_cast<typename RowVec<T, 2>::type *>(y + row), o);
            } else st_stream(y + row, sum[0]);
        }
    }
}

template <typename T, int B, int R, bool HDC>
static mo_status launch_lds(const mo_matrix &a, const void *x, void *y, hipStream_t s)
{
    const int64_t rows = (int64_t)B * R;
    const unsigned grid = (unsigned)((a.m + rows - 1) / rows);
    const size_t lds = (size_t)a.dia_lds_elems * sizeof(T);
    hipLaunchKernelGGL((k_dia_lds<T, B, R, HDC>), dim3(grid), dim3(B), lds, s, a.dia_xpos, a.dia_clusters, (int)a.dia_ncl,
                       (const T *)a.dia_val, a.m, a.n, a.nd, a.ld, a.csr_row_ptr, a.csr_col, (const T *)a.csr_val, (const T *)x, (T *)y);
    MO_LAUNCH_CHECK();
    return MO_OK;
}

// ---------------------------------------------------------------------------------------------- batched kernel
// Large matrices with at most DIA_PRE diagonals (a band, a 2-D or 7-point stencil, the true diagonals of an HDC
// matrix): the same windows and the same sums as k_dia_lds, but a block issues all its loads as one batch before its
// barrier: the window positions (WB per thread; more go in further batches, which is rare), the slab values of all ND
// diagonals, the row offsets of the remainder and the first chunk of the remainder's columns and values, whose x
// gathers follow as soon as the columns are there.  A block of such a matrix is short-lived (a few thousand slab
// values), and k_dia_lds, which stages its windows one piece at a time (load, wait, store) and streams the
// diagonals four at a time, keeps almost nothing in flight for much of a block's life.  Measured: 9 diagonals + 3 %
// scattered entries on 4.2 M rows (HDC) 82.8 -> 75.0 us in fp64 and 56.4 -> 48.0 us in fp32, 5 diagonals on 1.8 M rows
// 20.3 -> 17.2 us.  Not for small matrices or many diagonals: below about half a million rows the larger kernel
// (arguments, code) costs more than the batch saves (5 diagonals on 367 000 rows: 4.4 -> 4.9 us), and 27 diagonals need
// more than one batch of slab loads, which gains nothing over the four-at-a-time stream (2.1 M rows: the same 77 us).
//
// The launch plan (DiaPlan) travels in the kernel arguments, so a block reads it from scalar registers and no load
// waits for a table.  The windows are contiguous in LDS, so staging is one flat loop over positions, B at a time; such
// a run of positions lies in at most two windows, and the plan names, per run, where the second one starts and
// which x each of them holds.  xpos[k] is the LDS position of x[row0 + off_k] for the block's first row.  ND, the
// number of diagonals, is a template parameter: with it the loads and sums need no conditions, the compiler keeps
// every load of the batch in flight at once and counts exactly how many it may leave behind at each wait.
//
// HDC: the remainder's row pointers are read as 2-byte offsets relative to the block's first remainder entry, which
// a table with one entry per block names (launch data, built at conversion): half the bytes of the row pointers,
// and the block's range comes from a table that stays in cache instead of a cold line of row_ptr.
template <typename T, int B, int R, int ND, bool HDC>
__global__ __launch_bounds__(B) void k_dia_batch(const DiaPlan pl, const T *__restrict__ val, int64_t m, int64_t n, int64_t ld,
                                                 const int32_t *__restrict__ blk_ptr, const uint16_t *__restrict__ rp16,
                                                 const int32_t *__restrict__ col_idx, const T *__restrict__ cval,
                                                 const T *__restrict__ x, T *__restrict__ y)
{
    constexpr int ROWS = B * R;
    constexpr int WB = sizeof(T) == 8 ? 8 : 12;   // window positions per thread and batch
    extern __shared__ __align__(16) unsigned char s_raw[];
    T *xs = reinterpret_cast<T *>(s_raw);
    __shared__ int32_t rps[HDC ? ROWS + 1 : 1];
    __shared__ T prod[HDC ? HDC_CHUNK : 1];
    const int tid = (int)threadIdx.x;
    const int64_t lb = xcd_block(blockIdx.x, gridDim.x);
    const int64_t row0 = lb * ROWS;
    const int64_t row = row0 + (int64_t)tid * R;
    const int64_t rl = row < m ? row : 0;   // rows past the end load row 0's slab values and drop them
    // HDC: the remainder entries of this block are [blk_lo, blk_lo + nrem)
    int32_t blk_lo = 0, nrem = 0;
    if (HDC) {
        blk_lo = blk_ptr[lb];
        nrem = blk_ptr[lb + 1] - blk_lo;
    }
    T w[WB];          // x for the window positions tid + u * B of the current batch of runs
    uint32_t w_in = 0;
    // Issue order (loads return in order): the remainder's columns first, so that their x gathers can follow as
    // soon as they arrive and while everything else is still on its way.
    uint32_t first_c = 0;
    T first_v = (T)0;
    const bool first_on = HDC && tid < nrem;
    if (HDC && nrem > 0) {   // entry e0 for this thread (clamped: every thread loads, the surplus ones drop it)
        const int e0 = tid < nrem ? tid : nrem - 1;
        first_c = (uint32_t)col_idx[blk_lo + e0];
        first_v = cval[blk_lo + e0];
    }
    __builtin_amdgcn_sched_barrier(0);
    window_loads<T, B, WB>(pl.win, 0, tid, row0, n, x, w, &w_in);
    int32_t rp_mine[R];
    if (HDC) {
#pragma unroll
        for (int u = 0; u < R; ++u) {
            const int64_t r = row0 + tid + u * B;
            rp_mine[u] = r < m ? (int32_t)rp16[r] : nrem;   // relative to blk_lo
        }
    }
    T a[ND][R];
    const T *v0 = val + rl;
#pragma unroll
    for (int k = 0; k < ND; ++k) load_rows<T, R>(v0 + k * ld, a[k]);
    __builtin_amdgcn_sched_barrier(0);
    T x_first = (T)0;
    if (HDC && nrem > 0) {
        // the column passes through an empty statement the compiler cannot look into, so that nothing derived from it
        // (the address of the gather) is computed, and waited for, before the loads above have been issued
        asm volatile("" : "+v"(first_c));
        x_first = x[first_c];
    }
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll 1
    for (int u0 = WB; u0 * B < pl.win.elems; u0 += WB) {   // more window positions than one batch holds: rare
        window_stores<T, B, WB>(pl.win, u0 - WB, tid, w, w_in, xs);
        window_loads<T, B, WB>(pl.win, u0, tid, row0, n, x, w, &w_in);
    }
    window_stores<T, B, WB>(pl.win, ((pl.win.elems + B - 1) / B - 1) / WB * WB, tid, w, w_in, xs);
    if (HDC) {
#pragma unroll
        for (int u = 0; u < R; ++u) rps[tid + u * B] = rp_mine[u];
        if (tid == 0) rps[ROWS] = nrem;
    }
    __syncthreads();
    T sum[R];
#pragma unroll
    for (int j = 0; j < R; ++j) sum[j] = (T)0;
    const T *xl = xs + tid * R;
#pragma unroll
    for (int k = 0; k < ND; ++k) {
        const T *xk = xl + pl.xpos[k];
#pragma unroll
        for (int j = 0; j < R; ++j) sum[j] += a[k][j] * xk[j];
    }
    if (HDC && nrem > 0) {   // nrem is uniform across the block
        for (int32_t c0 = 0; c0 < nrem; c0 += HDC_CHUNK) {
            if (c0 == 0) {
                if (first_on) prod[tid] = first_v * x_first;
                for (int e = tid + B; e < HDC_CHUNK && e < nrem; e += B) prod[e] = cval[blk_lo + e] * x[col_idx[blk_lo + e]];
            } else {
                for (int e = tid; e < HDC_CHUNK && c0 + e < nrem; e += B) prod[e] = cval[blk_lo + c0 + e] * x[col_idx[blk_lo + c0 + e]];
            }
            __syncthreads();
#pragma unroll
            for (int j = 0; j < R; ++j) {
                int lo = rps[tid * R + j] - c0, hi = rps[tid * R + j + 1] - c0;
                lo = lo < 0 ? 0 : lo;
                hi = hi > HDC_CHUNK ? HDC_CHUNK : hi;
                for (int e = lo; e < hi; ++e) sum[j] += prod[e];
            }
            if (c0 + HDC_CHUNK < nrem) __syncthreads();   // the products are replaced by the next chunk's
        }
    }
    if (row < m) {
        if constexpr (R == 1) st_stream(y + row, sum[0]);
        else {
            // m need not be even: the last thread may own a single row
            if (row + 1 < m) {
                typename RowVec<T, 2>::type o;
                o.x = sum[0]; o.y = sum[1];
                st_stream(reinterpret_cast<typename RowVec<T, 2>::type *>(y + row), o);
            } else st_stream(y + row, sum[0]);
        }
    }
}

template <typename T, int ND, bool HDC>
static mo_status launch_batch(const mo_matrix &a, const void *x, void *y, hipStream_t s)
{
    constexpr int B = DIA_BATCH_BLOCK, R = DIA_ROWS_PER_LANE<T>;
    const int64_t rows = (int64_t)B * R;
    const unsigned grid = (unsigned)((a.m + rows - 1) / rows);
    const size_t lds = (size_t)a.dia_plan.win.elems * sizeof(T);
    hipLaunchKernelGGL((k_dia_batch<T, B, R, ND, HDC>), dim3(grid), dim3(B), lds, s, a.dia_plan, (const T *)a.dia_val, a.m, a.n, a.ld,
                       a.hdc_blk, a.hdc_rp16, a.csr_col, (const T *)a.csr_val, (const T *)x, (T *)y);
    MO_LAUNCH_CHECK();
    return MO_OK;
}

template <typename T, bool HDC>
static mo_status dia_batch(const mo_matrix &a, const void *x, void *y, hipStream_t s)
{
    static_assert(DIA_PRE == 12, "one case per number of diagonals");
    if (HDC && (!a.hdc_blk || !a.hdc_rp16)) return MO_E_NULL;   // the conversion builds them whenever this kernel is chosen
    switch (a.nd) {
    case 1: return launch_batch<T, 1, HDC>(a, x, y, s);
    case 2: return launch_batch<T, 2, HDC>(a, x, y, s);
    case 3: return launch_batch<T, 3, HDC>(a, x, y, s);
    case 4: return launch_batch<T, 4, HDC>(a, x, y, s);
    case 5: return launch_batch<T, 5, HDC>(a, x, y, s);
    case 6: return launch_batch<T, 6, HDC>(a, x, y, s);
    case 7: return launch_batch<T, 7, HDC>(a, x, y, s);
    case 8: return launch_batch<T, 8, HDC>(a, x, y, s);
    case 9: return launch_batch<T, 9, HDC>(a, x, y, s);
    case 10: return launch_batch<T, 10, HDC>(a, x, y, s);
    case 11: return launch_batch<T, 11, HDC>(a, x, y, s);
    case 12: return launch_batch<T, 12, HDC>(a, x, y, s);
    default: return MO_E_SHAPE;
    }
}

template <typename T, bool HDC>
static mo_status dia_any(const mo_matrix &a, const void *x, void *y, hipStream_t s)
{
    if (a.dia_batch) return dia_batch<T, HDC>(a, x, y, s);
    constexpr int R = DIA_ROWS_PER_LANE<T>;
    if (a.dia_block == 256 && a.dia_rows == R) return launch_lds<T, 256, R, HDC>(a, x, y, s);
    if (a.dia_block == 512 && a.dia_rows == R) return launch_lds<T, 512, R, HDC>(a, x, y, s);
    const unsigned grid = (unsigned)((a.m + DIA_B - 1) / DIA_B);
    if (HDC)
        hipLaunchKernelGGL(k_hdc_fused<T>, dim3(grid), dim3(DIA_B), 0, s, a.dia_off, (const T *)a.dia_val, a.m, a.n, a.nd, a.ld,
                           a.csr_row_ptr, a.csr_col, (const T *)a.csr_val, (const T *)x, (T *)y);
    else
        hipLaunchKernelGGL(k_dia<T>, dim3(grid), dim3(DIA_B), 0, s, a.dia_off, (const T *)a.dia_val, a.m, a.n, a.nd, a.ld, (const T *)x, (T *)y);
    MO_LAUNCH_CHECK();
    return MO_OK;
}

mo_status spmv_hdc_fused(const mo_matrix &a, const void *x, void *y, hipStream_t s)
{
    if (a.nnz_csr == 0) return spmv_dia(a, x, y, s);   // nothing beside the diagonals: no row pointers to read
    return a.dtype == MO_F32 ? dia_any<float, true>(a, x, y, s) : dia_any<double, true>(a, x, y, s);
}

mo_status spmv_dia(const mo_matrix &a, const void *x, void *y, hipStream_t s)
{
    return a.dtype == MO_F32 ? dia_any<float, false>(a, x, y, s) : dia_any<double, false>(a, x, y, s);
}

// Groups ascending offsets into clusters for a block of `block` rows: neighbours closer than `block` share a window
// (staging the gap costs less than staging a second window).  Returns false when the windows do not fit `max_elems`.
bool plan_dia_clusters(const std::vector<int32_t> &off, int block, int64_t max_elems, std::vector<int32_t> *xpos,
                       std::vector<int32_t> *clusters, int64_t *total_elems)
{
    xpos->assign(off.size(), 0);
    clusters->clear();
    int64_t base = 0;
    size_t k = 0;
    while (k < off.size()) {
        size_t e = k;
        while (e + 1 < off.size() && (int64_t)off[e + 1] - (int64_t)off[e] < block) ++e;
        const int64_t len = (int64_t)off[e] - (int64_t)off[k] + block;
        if (base + len > max_elems) return false;
        for (size_t q = k; q <= e; ++q) (*xpos)[q] = (int32_t)(base + ((int64_t)off[q] - (int64_t)off[k]));
        clusters->push_back(off[k]);
        clusters->push_back((int32_t)len);
        clusters->push_back((int32_t)base);
        base += len;
        k = e + 1;
    }
    *total_elems = base;
    return true;
}

}  // namespace mo

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
// The launch plan (DiaPlan) travels in the kernel arguments, so a block reads it from scalar registers.  The windows
// are contiguous in LDS, so staging is one flat loop over positions, B at a time; such a run of positions lies in at
// most two windows, and the plan names, per run, where the second one starts and which x each of them holds.
// xpos[k] is the LDS position of x[row0 + off_k] for the block's first row.
//
// Every thread owns R consecutive rows (R = 1 for fp64, 2 for fp32 so that a lane still moves 8 bytes per load).
//
// A block's loads are issued as one batch before its barrier: the first WB positions per thread of the windows,
// the row offsets of the remainder (HDC: 2 bytes per row, relative to the block's first remainder entry, which a
// table with one entry per block names), the slab values of the first DIA_PRE diagonals, and the first chunk of the
// HDC remainder with its x gathers.  A block then pays one memory latency for all of them instead of one per window
// piece and per group of four diagonals; blocks are short-lived (a few thousand slab values), so a block that waits
// for one load at a time keeps almost nothing in flight for much of its life.  Further diagonals follow in batches
// of DIA_PRE after the barrier.
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
__global__ __launch_bounds__(B) void k_dia_lds(const DiaPlan pl, const int32_t *__restrict__ xpos, const T *__restrict__ val, int64_t m,
                                               int64_t n, int64_t nd, int64_t ld, const int32_t *__restrict__ blk_ptr,
                                               const uint16_t *__restrict__ rp16, const int32_t *__restrict__ col_idx, const T *__restrict__ cval,
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
    T a[DIA_PRE][R];
    const T *v0 = val + rl;
#pragma unroll
    for (int k = 0; k < DIA_PRE; ++k)
        if (k < nd) load_rows<T, R>(v0 + k * ld, a[k]);
    __builtin_amdgcn_sched_barrier(0);
    T x_first = (T)0;
    if (HDC && nrem > 0) x_first = x[first_c];
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
    for (int k = 0; k < DIA_PRE; ++k) {
        if (k < nd) {
            const T *xk = xl + pl.xpos[k];
#pragma unroll
            for (int j = 0; j < R; ++j) sum[j] += a[k][j] * xk[j];
        }
    }
    for (int64_t k0 = DIA_PRE; k0 < nd; k0 += DIA_PRE) {
#pragma unroll
        for (int k = 0; k < DIA_PRE; ++k)
            if (k0 + k < nd) load_rows<T, R>(v0 + (k0 + k) * ld, a[k]);
#pragma unroll
        for (int k = 0; k < DIA_PRE; ++k) {
            if (k0 + k < nd) {
                const T *xk = xl + xpos[k0 + k];
#pragma unroll
                for (int j = 0; j < R; ++j) sum[j] += a[k][j] * xk[j];
            }
        }
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

template <typename T, int B, int R, bool HDC>
static mo_status launch_lds(const mo_matrix &a, const void *x, void *y, hipStream_t s)
{
    const int64_t rows = (int64_t)B * R;
    const unsigned grid = (unsigned)((a.m + rows - 1) / rows);
    const size_t lds = (size_t)a.dia_plan.win.elems * sizeof(T);
    hipLaunchKernelGGL((k_dia_lds<T, B, R, HDC>), dim3(grid), dim3(B), lds, s, a.dia_plan, a.dia_xpos, (const T *)a.dia_val, a.m, a.n, a.nd,
                       a.ld, a.hdc_blk, a.hdc_rp16, a.csr_col, (const T *)a.csr_val, (const T *)x, (T *)y);
    MO_LAUNCH_CHECK();
    return MO_OK;
}

template <typename T, bool HDC>
static mo_status dia_any(const mo_matrix &a, const void *x, void *y, hipStream_t s)
{
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
    if (a.dia_block && (!a.hdc_blk || !a.hdc_rp16)) return MO_E_NULL;   // the conversion builds them whenever this path is taken
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

// COO SpMV (Section II-B: one (row, col, value) triple per stored entry).  The library always produces
// (row, col)-sorted COO, so y[row] = sum over the run of equal rows.  The reduction is a segmented sum with a fixed
// association order and no floating-point atomics, so results are bit-identical from run to run:
//   1. every thread owns COO_STRIP consecutive entries, loads them with wide loads, gathers x and reduces the runs
//      inside its strip in registers;
//   2. runs that cross strips are finished through a small LDS table by the thread that holds the head of the run;
//   3. a run that crosses a tile boundary leaves its continuation in a per-tile carry slot, added by k_coo_fixup.
// Exactly one thread of the whole grid writes y[row] in step 1/2, and one thread adds the carries in step 3.
// y is zeroed first only when the matrix has rows without entries (known from the conversion's row statistics).
#include "dev_common.hpp"
#include "mo_internal.hpp"

namespace mo {

constexpr int COO_B = 256;
// Entries per thread (COO_STRIP): 8, 4 or 2, chosen at conversion time from the size of the part.

template <typename T>
__global__ void k_zero(T *__restrict__ p, int64_t n)
{
    int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    for (; i < n; i += stride) p[i] = (T)0;
}


template <typename T, int COO_STRIP, bool ACC>
__global__ __launch_bounds__(COO_B) void k_coo_tile(const int32_t *__restrict__ row, const int32_t *__restrict__ col,
                                                     const T *__restrict__ val, int64_t nnz, const T *__restrict__ x,
                                                     T *__restrict__ y, int32_t *__restrict__ carry_row, T *__restrict__ carry_val)
{
    __shared__ int s_first[COO_B + 1];
    __shared__ int s_last[COO_B];
    __shared__ int s_closed[COO_B];
    __shared__ T s_lead[COO_B];

    constexpr int TILE = COO_B * COO_STRIP;
    const int64_t tile = xcd_block(blockIdx.x, gridDim.x);
    const int64_t base = tile * TILE;
    const int t = threadIdx.x;

    // Entries are fetched with consecutive lanes on consecutive entries (entry base + t + q * 256 in load q), so that a
    // wave's x gathers cover 64 neighbouring entries - a few rows, whose columns share cache lines - and not every
    // fourth entry of 256; the products and row indices then change hands through LDS, after which every thread owns
    // COO_STRIP consecutive entries.  (With 16-byte loads of 4 consecutive entries per lane the gathers of one
    // instruction spread over four times as many rows: 125 against 107 us for this stream-and-gather step on the
    // 27-point stencil's pattern.)
    __shared__ int s_row[TILE];
    __shared__ T s_prod[TILE];
    // the row of the entry before the tile (thread 0 needs it at the very end to tell whether the tile's first run
    // started earlier): requested with everything else, not when it is needed
    int row_before = -1;
    if (t == 0 && base > 0) row_before = row[base - 1];
    {
        int rr[COO_STRIP], cc[COO_STRIP];
        T vv[COO_STRIP], xx[COO_STRIP];
        const int64_t left = nnz - base;                       // > 0
        const int lim = (int)(left < TILE ? left : TILE);      // entries of this tile
#pragma unroll
        for (int q = 0; q < COO_STRIP; ++q) {                  // unconditional loads, index clamped into the tile
            const int i = t + q * COO_B;
            const int64_t p = base + (i < lim ? i : lim - 1);
            rr[q] = ld_stream(row + p);
            cc[q] = ld_stream(col + p);
        }
#pragma unroll
        for (int q = 0; q < COO_STRIP; ++q) {
            const int i = t + q * COO_B;
            vv[q] = ld_stream(val + base + (i < lim ? i : lim - 1));
        }
#pragma unroll
        for (int q = 0; q < COO_STRIP; ++q) xx[q] = x[cc[q]];
#pragma unroll
        for (int q = 0; q < COO_STRIP; ++q) {
            const int i = t + q * COO_B;
            s_row[i] = i < lim ? rr[q] : -1;
            s_prod[i] = i < lim ? vv[q] * xx[q] : (T)0;
        }
    }
    __syncthreads();
    int r[COO_STRIP];
    T pr[COO_STRIP];
#pragma unroll
    for (int q = 0; q < COO_STRIP; ++q) { r[q] = s_row[t * COO_STRIP + q]; pr[q] = s_prod[t * COO_STRIP + q]; }

    // runs inside the strip
    int cur = r[0];
    T acc = pr[0];
    bool leading = true, lead_closed = false, has_tail = false;
    T lead_sum = (T)0;
#pragma unroll
    for (int q = 1; q < COO_STRIP; ++q) {
        if (r[q] == cur) {
            acc += pr[q];
        } else {
            if (leading) { lead_sum = acc; lead_closed = true; leading = false; }
            else if (cur >= 0) { if (ACC) y[cur] += acc; else y[cur] = acc; }   // a run that starts and ends in this strip
            cur = r[q];
            acc = pr[q];
        }
    }
    if (leading) lead_sum = acc; else has_tail = true;
    const int tail_row = cur;
    const T tail_sum = acc;

    s_first[t] = r[0];
    s_last[t] = r[COO_STRIP - 1];
    s_closed[t] = lead_closed ? 1 : 0;
    s_lead[t] = lead_sum;
    if (t == 0) s_first[COO_B] = -2;
    __syncthreads();

    // the run that reaches the end of this strip and started inside it
    if (has_tail && tail_row >= 0) {
        T total = tail_sum;
        for (int u = t + 1; s_first[u] == tail_row; ++u) {
            total += s_lead[u];
            if (s_closed[u]) break;
        }
        if (ACC) y[tail_row] += total; else y[tail_row] = total;
    }
    // the run at the start of this strip, when its head is here (or, for thread 0, possibly in an earlier tile)
    const int before = (t == 0) ? row_before : s_last[t - 1];
    const bool head_here = r[0] != before;
    if (r[0] >= 0 && (head_here || t == 0)) {
        T total = lead_sum;
        if (!lead_closed) {
            for (int u = t + 1; s_first[u] == r[0]; ++u) {
                total += s_lead[u];
                if (s_closed[u]) break;
            }
        }
        if (head_here) { if (ACC) y[r[0]] += total; else y[r[0]] = total; }
        else { carry_val[tile] = total; }
    }
    if (t == 0) carry_row[tile] = (r[0] >= 0 && !head_here) ? r[0] : -1;
}

// Adds the carries: a chain of consecutive tiles with the same carry row is summed in tile order by the thread of
// its first tile.
template <typename T>
__global__ void k_coo_fixup(const int32_t *__restrict__ carry_row, const T *__restrict__ carry_val, int64_t tiles, T *__restrict__ y)
{
    const int64_t k = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (k >= tiles) return;
    const int r = carry_row[k];
    if (r < 0) return;
    if (k > 0 && carry_row[k - 1] == r) return;
    T total = carry_val[k];
    // the same sum in the same order, with the loads of FU tiles in flight together: a row that crosses a thousand tiles
    // is otherwise a thousand dependent loads
    constexpr int FU = 16;
    bool more = true;
    for (int64_t u0 = k + 1; more && u0 < tiles; u0 += FU) {
        int32_t rr[FU];
        T vv[FU];
#pragma unroll
        for (int j = 0; j < FU; ++j) {
            const int64_t u = u0 + j < tiles ? u0 + j : tiles - 1;
            rr[j] = carry_row[u];
            vv[j] = carry_val[u];
        }
#pragma unroll
        for (int j = 0; j < FU; ++j) {
            more = more && u0 + j < tiles && rr[j] == r;
            if (more) total += vv[j];
        }
    }
    y[r] += total;
}

template <typename T>
static mo_status zero_typed(void *p, int64_t n, hipStream_t s)
{
    if (n <= 0) return MO_OK;
    int64_t g = (n + 2047) / 2048;
    if (g > 4096) g = 4096;
    hipLaunchKernelGGL(k_zero<T>, dim3((unsigned)g), dim3(256), 0, s, (T *)p, n);
    MO_LAUNCH_CHECK();
    return MO_OK;
}

mo_status fill_zero(void *p, int64_t n_elems, mo_dtype dt, hipStream_t s)
{
    return dt == MO_F32 ? zero_typed<float>(p, n_elems, s) : zero_typed<double>(p, n_elems, s);
}

template <typename T, int STRIP>
static mo_status coo_launch(const mo_matrix &a, const T *x, T *y, bool accumulate, hipStream_t s)
{
    const unsigned tiles = (unsigned)a.coo_tiles;
    if (accumulate)
        hipLaunchKernelGGL((k_coo_tile<T, STRIP, true>), dim3(tiles), dim3(COO_B), 0, s, a.coo_row, a.coo_col, (const T *)a.coo_val,
                           a.nnz_coo, x, y, a.coo_carry_row, (T *)a.coo_carry_val);
    else
        hipLaunchKernelGGL((k_coo_tile<T, STRIP, false>), dim3(tiles), dim3(COO_B), 0, s, a.coo_row, a.coo_col, (const T *)a.coo_val,
                           a.nnz_coo, x, y, a.coo_carry_row, (T *)a.coo_carry_val);
    MO_LAUNCH_CHECK();
    if (tiles > 1) {
        hipLaunchKernelGGL(k_coo_fixup<T>, dim3((tiles + 255) / 256), dim3(256), 0, s, a.coo_carry_row, (const T *)a.coo_carry_val,
                           (int64_t)tiles, y);
        MO_LAUNCH_CHECK();
    }
    return MO_OK;
}

template <typename T>
static mo_status coo_typed(const mo_matrix &a, const void *x, void *y, bool accumulate, hipStream_t s)
{
    // y[row] is stored by the one thread that holds the head of the row's run, so only rows without entries need zeros
    if (!accumulate && !(a.fmt == MO_COO && a.coo_every_row)) MO_TRY(zero_typed<T>(y, a.m, s));
    if (a.nnz_coo <= 0) return MO_OK;
    if (a.coo_strip == 2) return coo_launch<T, 2>(a, (const T *)x, (T *)y, accumulate, s);
    if (a.coo_strip == 8) return coo_launch<T, 8>(a, (const T *)x, (T *)y, accumulate, s);
    return coo_launch<T, 4>(a, (const T *)x, (T *)y, accumulate, s);
}

mo_status carry_fixup(const int32_t *carry_row, const void *carry_val, int64_t tiles, void *y, mo_dtype dt, hipStream_t s)
{
    const unsigned g = (unsigned)((tiles + 255) / 256);
    if (dt == MO_F32) hipLaunchKernelGGL(k_coo_fixup<float>, dim3(g), dim3(256), 0, s, carry_row, (const float *)carry_val, tiles, (float *)y);
    else hipLaunchKernelGGL(k_coo_fixup<double>, dim3(g), dim3(256), 0, s, carry_row, (const double *)carry_val, tiles, (double *)y);
    MO_LAUNCH_CHECK();
    return MO_OK;
}

mo_status spmv_coo(const mo_matrix &a, const void *x, void *y, bool accumulate, hipStream_t s)
{
    return a.dtype == MO_F32 ? coo_typed<float>(a, x, y, accumulate, s) : coo_typed<double>(a, x, y, accumulate, s);
}

}  // namespace mo

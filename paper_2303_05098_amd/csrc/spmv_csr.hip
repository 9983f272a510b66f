// CSR SpMV (Section II-B: values and column indices stored row after row, row_ptr marks the row boundaries).
//
// Two kernels, chosen per matrix at conversion time, both with a fixed association order (bit-identical reruns):
//
//  * tiled (no row longer than CSR_TILE_SLACK): the entry array is cut into tiles of CSR_TILE entries; tile k owns
//    the rows that START inside it (the first such row and its entry position are precomputed, 8 bytes per tile).
//    A block streams the entries of its rows with fully coalesced non-temporal loads, independent of the row
//    structure, multiplies them with the gathered x values and parks the products in LDS; the rows are then summed
//    out of LDS.  Measured against staging (col, val) in LDS and gathering row by row, this keeps every global load
//    of a tile in flight at once and was 20-30 % faster on the stencil and band configurations.
//  * vector (skewed matrices): an aligned group of LANES lanes strides over one row, shuffle reduction.
//
// Neighbouring tiles / rows are kept on the same XCD so that the part of x a band touches stays in that XCD's L2.
#include "dev_common.hpp"
#include "mo_internal.hpp"

namespace mo {

constexpr int CSR_B = 256;

// ---------------------------------------------------------------------------------------------- vector kernel
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
        for (int64_t p = lo + sub; p < hi; p += LANES) sum += ld_stream(val + p) * x[ld_stream(col_idx + p)];
    }
    sum = group_sum_down(sum, LANES);
    if (sub == 0 && row < m) {
        if (ACC) y[row] += sum; else y[row] = sum;
    }
}

// ---------------------------------------------------------------------------------------------- tiled kernel
// tile_rp[2k] = first row whose start lies in tile k (or later), tile_rp[2k+1] = row_ptr of that row.
__global__ __launch_bounds__(256) void k_csr_tiles(const int32_t *__restrict__ row_ptr, int64_t m, int64_t nnz, int64_t ntiles,
                                                    int64_t tile_size, int32_t *__restrict__ tile_rp)
{
    const int64_t k = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (k > ntiles) return;
    int64_t r = m;
    if (k < ntiles) {
        const int64_t target = k * tile_size;   // first row with row_ptr[row] >= target
        int64_t lo = 0, hi = m;                // answer in [0, m]
        while (lo < hi) {
            const int64_t mid = (lo + hi) >> 1;
            if ((int64_t)row_ptr[mid] >= target) hi = mid; else lo = mid + 1;
        }
        r = lo;
    }
    tile_rp[2 * k] = (int32_t)r;
    tile_rp[2 * k + 1] = (r < m) ? row_ptr[r] : (int32_t)nnz;
}

// Every thread gathers x for the entries it streams (entry order, all loads of a tile in flight together) and stores
// the products in LDS; the rows are then summed from LDS, G lanes per row, without touching global memory again.
template <typename T, int TILE, int G, bool ACC>
__global__ __launch_bounds__(CSR_B) void k_csr_tiled(const int32_t *__restrict__ tile_rp, const int32_t *__restrict__ row_ptr,
                                                     const int32_t *__restrict__ col_idx, const T *__restrict__ val,
                                                     const T *__restrict__ x, T *__restrict__ y)
{
    constexpr int CAP = TILE + CSR_TILE_SLACK;
    constexpr int EPT = (CAP + CSR_B - 1) / CSR_B;
    constexpr int RPB = CSR_B / G;
    __shared__ T ps[CAP];
    const int64_t tile = xcd_block(blockIdx.x, gridDim.x);
    const int2v a = *reinterpret_cast<const int2v *>(tile_rp + 2 * tile);
    const int2v b = *reinterpret_cast<const int2v *>(tile_rp + 2 * tile + 2);
    const int64_t ra = a.x, rb = b.x;
    const int64_t p0 = a.y;
    int cnt = b.y - a.y;
    cnt = cnt < CAP ? cnt : CAP;
    const int sub = threadIdx.x % G;
    const int64_t nrows = rb - ra;
    int lo = 0, hi = 0;
    {
        const int64_t r = ra + threadIdx.x / G;
        if (r < rb) { lo = row_ptr[r] - (int32_t)p0; hi = row_ptr[r + 1] - (int32_t)p0; }
    }
    int32_t c[EPT];
    T v[EPT];
#pragma unroll
    for (int j = 0; j < EPT; ++j) {
        const int i = threadIdx.x + j * CSR_B;
        c[j] = 0; v[j] = (T)0;
        if (i < cnt) { c[j] = ld_stream(col_idx + p0 + i); v[j] = ld_stream(val + p0 + i); }
    }
#pragma unroll
    for (int j = 0; j < EPT; ++j) {
        const int i = threadIdx.x + j * CSR_B;
        if (i < cnt) ps[i] = v[j] * x[c[j]];
    }
    __syncthreads();
    for (int64_t base = 0; base < nrows; base += RPB) {
        const int64_t r = ra + base + threadIdx.x / G;
        if (base > 0) {
            lo = hi = 0;
            if (r < rb) { lo = row_ptr[r] - (int32_t)p0; hi = row_ptr[r + 1] - (int32_t)p0; }
        }
        T sum = (T)0;
        for (int e = lo + sub; e < hi; e += G) sum += ps[e];
        if (G > 1) sum = group_sum_down(sum, G);
        if (sub == 0 && r < rb) {
            if (ACC) y[r] += sum; else st_stream(y + r, sum);
        }
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

template <typename T, int TILE, int G>
static mo_status launch_tiled(const mo_matrix &a, const T *x, T *y, bool acc, hipStream_t s)
{
    const unsigned grid = (unsigned)a.csr_tiles;
    if (acc)
        hipLaunchKernelGGL((k_csr_tiled<T, TILE, G, true>), dim3(grid), dim3(CSR_B), 0, s, a.csr_tile_rp, a.csr_row_ptr, a.csr_col, (const T *)a.csr_val, x, y);
    else
        hipLaunchKernelGGL((k_csr_tiled<T, TILE, G, false>), dim3(grid), dim3(CSR_B), 0, s, a.csr_tile_rp, a.csr_row_ptr, a.csr_col, (const T *)a.csr_val, x, y);
    MO_LAUNCH_CHECK();
    return MO_OK;
}

template <typename T, int TILE>
static mo_status launch_tiled_g(const mo_matrix &a, const T *x, T *y, bool acc, hipStream_t s)
{
    switch (a.csr_group) {
    case 1: return launch_tiled<T, TILE, 1>(a, x, y, acc, s);
    case 2: return launch_tiled<T, TILE, 2>(a, x, y, acc, s);
    case 4: return launch_tiled<T, TILE, 4>(a, x, y, acc, s);
    case 8: return launch_tiled<T, TILE, 8>(a, x, y, acc, s);
    default: return launch_tiled<T, TILE, 16>(a, x, y, acc, s);
    }
}

template <typename T>
static mo_status csr_typed(const mo_matrix &a, const void *xv, void *yv, bool acc, hipStream_t s)
{
    const T *x = (const T *)xv;
    T *y = (T *)yv;
    if (a.csr_tiles > 0) return launch_tiled_g<T, CSR_TILE>(a, x, y, acc, s);
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

// Launch plan for a CSR part: tiled when no row exceeds the LDS slack, vector otherwise.  tile_rp must hold
// 2 * (tiles + 1) ints when the tiled kernel is chosen.
int64_t csr_tile_count(int64_t nnz, int64_t max_row, int tile_size)
{
    if (max_row > CSR_TILE_SLACK) return 0;
    const int64_t t = (nnz + tile_size - 1) / tile_size;
    return t > 0 ? t : 1;
}

mo_status csr_build_tiles(const int32_t *row_ptr, int64_t m, int64_t nnz, int64_t ntiles, int tile_size, int32_t *tile_rp, hipStream_t s)
{
    hipLaunchKernelGGL(k_csr_tiles, dim3((unsigned)((ntiles + 1 + 255) / 256)), dim3(256), 0, s, row_ptr, m, nnz, ntiles,
                       (int64_t)tile_size, tile_rp);
    MO_LAUNCH_CHECK();
    return MO_OK;
}

}  // namespace mo

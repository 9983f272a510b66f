// CSR SpMV (Section II-B: values and column indices stored row after row, row_ptr marks the row boundaries).
//
// The entry array is cut into tiles of 2048 entries (512 for parts of fewer than 2^20 entries, which would otherwise
// occupy too few blocks: 5.0 -> 3.8 us on matrices of some 10^5 entries), one block per tile, so the work per block is
// the same whatever the row lengths are.  A block streams its entries with fully coalesced non-temporal loads, multiplies them
// with the gathered x values and parks the products in LDS; rows are then summed out of LDS, G lanes per row (G from
// the mean row length).  Both kernels have a fixed association order (bit-identical reruns, no float atomics):
//
//  * k_csr_tiled (no row longer than CSR_TILE_SLACK): tile k owns the rows that START inside it and also streams
//    their tails (at most CSR_TILE_SLACK extra entries), so every row is summed by one block and y is written once.
//    The first such row and its entry position are precomputed: 8 bytes of launch data per tile.
//  * k_csr_split (longer rows exist): tile k is exactly entries [k*CSR_TILE, (k+1)*CSR_TILE); the part of a row that
//    spills into later tiles goes through per-tile carry slots and a tiny fix-up kernel.  On the lognormal
//    configuration (rows up to 1802 entries) this runs at 186 us against 236 us for a lanes-per-row vector kernel.
//
// Measured against staging (col, val) in LDS and gathering row by row, multiplying while streaming keeps every
// global load of a tile in flight at once and was 20-30 % faster on the stencil and band configurations.
// Neighbouring tiles are kept on the same XCD so that the part of x a band touches stays in that XCD's L2.
#include "dev_common.hpp"
#include "mo_internal.hpp"

namespace mo {

constexpr int CSR_B = 256;

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
    // x is gathered for every slot, used or not (an unused slot holds column 0), so that the gathers of a thread are
    // all in flight together: behind a per-slot condition each one waited for the one before it
    T xv[EPT];
#pragma unroll
    for (int j = 0; j < EPT; ++j) xv[j] = x[c[j]];
#pragma unroll
    for (int j = 0; j < EPT; ++j) {
        const int i = threadIdx.x + j * CSR_B;
        if (i < cnt) ps[i] = v[j] * xv[j];
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

// Sum of one value per thread over the block, in a fixed order (xor butterfly inside a wave, waves added in order).
template <typename T>
__device__ __forceinline__ T block_sum(T v, T *s_red)
{
    v = wave_sum(v);
    if (lane_id() == 0) s_red[threadIdx.x / WAVE] = v;
    __syncthreads();
    T t = s_red[0];
#pragma unroll
    for (int w = 1; w < CSR_B / WAVE; ++w) t += s_red[w];
    __syncthreads();
    return t;
}

// Tiled kernel for matrices with rows of any length: tile k is exactly the entries [k*TILE, (k+1)*TILE), so the work
// per block does not depend on the row structure at all.  The head of the tile that belongs to a row started in an
// earlier tile is reduced by the whole block into a per-tile carry slot (added to y by the carry fix-up kernel, in
// tile order); rows that start in the tile are summed from the LDS products up to the tile end, G lanes per row,
// except rows with more than CSR_LONG_SEG entries inside the tile, which the whole block reduces one after another.
constexpr int CSR_LONG_SEG = 256;

template <typename T, int TILE, int G, bool ACC>
__global__ __launch_bounds__(CSR_B) void k_csr_split(const int32_t *__restrict__ tile_rp, const int32_t *__restrict__ row_ptr,
                                                     const int32_t *__restrict__ col_idx, const T *__restrict__ val, int64_t nnz,
                                                     const T *__restrict__ x, T *__restrict__ y, int32_t *__restrict__ carry_row,
                                                     T *__restrict__ carry_val)
{
    constexpr int EPT = TILE / CSR_B;
    constexpr int RPB = CSR_B / G;
    __shared__ T ps[TILE];
    __shared__ T s_red[CSR_B / WAVE];
    __shared__ int s_long[TILE / CSR_LONG_SEG + 1];
    __shared__ int s_nlong;
    const int64_t tile = xcd_block(blockIdx.x, gridDim.x);
    const int64_t t0 = tile * TILE;
    const int cnt = (int)((t0 + TILE < nnz ? t0 + TILE : nnz) - t0);
    const int2v a = *reinterpret_cast<const int2v *>(tile_rp + 2 * tile);
    const int2v b = *reinterpret_cast<const int2v *>(tile_rp + 2 * tile + 2);
    const int64_t ra = a.x, rb = b.x;
    int seg = (int)((int64_t)a.y - t0);          // entries at the head of the tile that continue row ra - 1
    seg = seg < cnt ? seg : cnt;
    const int sub = threadIdx.x % G;
    const int64_t nrows = rb - ra;
    int lo = 0, hi = 0;
    {
        const int64_t r = ra + threadIdx.x / G;
        if (r < rb) { lo = row_ptr[r] - (int32_t)t0; hi = row_ptr[r + 1] - (int32_t)t0; }
    }
    int32_t c[EPT];
    T v[EPT];
#pragma unroll
    for (int j = 0; j < EPT; ++j) {
        const int i = threadIdx.x + j * CSR_B;
        c[j] = 0; v[j] = (T)0;
        if (i < cnt) { c[j] = ld_stream(col_idx + t0 + i); v[j] = ld_stream(val + t0 + i); }
    }
    T xv[EPT];   // gathered for every slot, used or not (an unused slot holds column 0): all in flight together
#pragma unroll
    for (int j = 0; j < EPT; ++j) xv[j] = x[c[j]];
#pragma unroll
    for (int j = 0; j < EPT; ++j) {
        const int i = threadIdx.x + j * CSR_B;
        if (i < cnt) ps[i] = v[j] * xv[j];
    }
    if (threadIdx.x == 0) s_nlong = 0;
    __syncthreads();
    if (seg > 0) {   // uniform
        T part = (T)0;
        for (int i = threadIdx.x; i < seg; i += CSR_B) part += ps[i];
        const T total = block_sum(part, s_red);
        if (threadIdx.x == 0) carry_val[tile] = total;
    }
    if (threadIdx.x == 0) carry_row[tile] = seg > 0 ? (int32_t)(ra - 1) : -1;
    for (int64_t base = 0; base < nrows; base += RPB) {
        const int64_t r = ra + base + threadIdx.x / G;
        if (base > 0) {
            lo = hi = 0;
            if (r < rb) { lo = row_ptr[r] - (int32_t)t0; hi = row_ptr[r + 1] - (int32_t)t0; }
        }
        hi = hi < cnt ? hi : cnt;
        const bool is_long = hi - lo > CSR_LONG_SEG;
        T sum = (T)0;
        if (!is_long)
            for (int e = lo + sub; e < hi; e += G) sum += ps[e];
        if (G > 1) sum = group_sum_down(sum, G);
        if (sub == 0 && r < rb) {
            if (is_long) s_long[atomicAdd(&s_nlong, 1)] = (int)(r - ra);
            else if (ACC) y[r] += sum;
            else y[r] = sum;
        }
    }
    __syncthreads();
    const int nlong = s_nlong;   // at most TILE / CSR_LONG_SEG rows; each sum is order-fixed, so the list order does not matter
    for (int q = 0; q < nlong; ++q) {
        const int64_t r = ra + s_long[q];
        const int l0 = row_ptr[r] - (int32_t)t0;
        int h0 = row_ptr[r + 1] - (int32_t)t0;
        h0 = h0 < cnt ? h0 : cnt;
        T part = (T)0;
        for (int i = l0 + threadIdx.x; i < h0; i += CSR_B) part += ps[i];
        const T total = block_sum(part, s_red);
        if (threadIdx.x == 0) { if (ACC) y[r] += total; else y[r] = total; }
    }
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

template <typename T, int TILE, int G>
static mo_status launch_split(const mo_matrix &a, const T *x, T *y, bool acc, hipStream_t s)
{
    const unsigned grid = (unsigned)a.csr_tiles;
    if (acc)
        hipLaunchKernelGGL((k_csr_split<T, TILE, G, true>), dim3(grid), dim3(CSR_B), 0, s, a.csr_tile_rp, a.csr_row_ptr, a.csr_col,
                           (const T *)a.csr_val, a.nnz_csr, x, y, a.csr_carry_row, (T *)a.csr_carry_val);
    else
        hipLaunchKernelGGL((k_csr_split<T, TILE, G, false>), dim3(grid), dim3(CSR_B), 0, s, a.csr_tile_rp, a.csr_row_ptr, a.csr_col,
                           (const T *)a.csr_val, a.nnz_csr, x, y, a.csr_carry_row, (T *)a.csr_carry_val);
    MO_LAUNCH_CHECK();
    return grid > 1 ? carry_fixup(a.csr_carry_row, a.csr_carry_val, (int64_t)grid, y, a.dtype, s) : MO_OK;
}

template <typename T, int TILE>
static mo_status launch_tiled_g(const mo_matrix &a, const T *x, T *y, bool acc, hipStream_t s)
{
    if (a.csr_split) {
        switch (a.csr_group) {
        case 1: return launch_split<T, TILE, 1>(a, x, y, acc, s);
        case 2: return launch_split<T, TILE, 2>(a, x, y, acc, s);
        case 4: return launch_split<T, TILE, 4>(a, x, y, acc, s);
        case 8: return launch_split<T, TILE, 8>(a, x, y, acc, s);
        default: return launch_split<T, TILE, 16>(a, x, y, acc, s);
        }
    }
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
    return a.csr_tile == CSR_TILE_SMALL ? launch_tiled_g<T, CSR_TILE_SMALL>(a, x, y, acc, s) : launch_tiled_g<T, CSR_TILE>(a, x, y, acc, s);
}

mo_status spmv_csr(const mo_matrix &a, const void *x, void *y, bool accumulate, hipStream_t s)
{
    return a.dtype == MO_F32 ? csr_typed<float>(a, x, y, accumulate, s) : csr_typed<double>(a, x, y, accumulate, s);
}

// Launch plan for a CSR part: tiled when no row exceeds the LDS slack, vector otherwise.  tile_rp must hold
// 2 * (tiles + 1) ints when the tiled kernel is chosen.
int64_t csr_tile_count(int64_t nnz, int tile_size)
{
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

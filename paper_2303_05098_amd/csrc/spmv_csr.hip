// CSR SpMV (Section II-B: values and column indices stored row after row, row_ptr marks the row boundaries).
//
// The entry array is cut into tiles of 2048 entries (4096 in fp32 or when rows average 16 entries or more; 512 for
// parts of fewer than 2^20 entries, which would otherwise occupy too few blocks), one block per tile, so the work per
// block is the same whatever the row lengths are.  A block streams its entries with fully coalesced non-temporal
// loads, multiplies them with the gathered x values and parks the products in LDS; rows are then summed out of LDS,
// G lanes per row (G from the mean row length).  Both kernels have a fixed association order (bit-identical reruns,
// no float atomics):
//
//  * k_csr_tiled (no row longer than CSR_MAX_ROW): tile k owns the rows that START at or after entry k * TILE (first
//    row rounded up to a whole cache line of y where the slack allows it) and streams them to the end of the last
//    one, so every row is summed by one block and y is written once, in whole lines.  The first row and its entry
//    position are precomputed: 8 bytes of launch data per tile.
//  * k_csr_split (longer rows exist): tile k is exactly entries [k*CSR_TILE, (k+1)*CSR_TILE); the part of a row that
//    spills into later tiles goes through per-tile carry slots and a tiny fix-up kernel.  On the lognormal
//    configuration (rows up to 1802 entries) this runs at 186 us against 236 us for a lanes-per-row vector kernel.
//
// What the tile kernel costs beyond its entry stream was measured step by step on the stencil's access pattern
// (stand-alone kernels, 679 MB of columns and values): stream alone 95 us (7.1 TB/s); + x gathers 107 - 110 us; +
// products through LDS and row sums 115 - 119 us; + y written 128 us when a tile's rows begin and end on lines of
// y, 144 us when they do not (partial lines, merged in DRAM); and 165 us when the tile's entry stream also starts off
// a line boundary, as it does when it starts at the first owned row.  Hence the two alignments above.  Kernels that
// keep a block alive over several tiles (with or without the next tile's loads in flight) were slower than one
// short-lived block per tile, and so was a variant that served x from LDS windows staged per tile.
// Neighbouring tiles are kept on the same XCD so that the part of x a band touches stays in that XCD's L2.
#include "dev_common.hpp"
#include "mo_internal.hpp"

namespace mo {

constexpr int CSR_B = 256;

// ---------------------------------------------------------------------------------------------- tiled kernel
// tile_rp[2k] = first row of tile k, tile_rp[2k+1] = row_ptr of that row.  The first row is the first one whose start
// lies at or after entry k * tile_size, rounded up to a multiple of row_align (so that the y values a tile writes
// begin and end on cache-line boundaries; 1 = no rounding).  Tile k owns the rows up to the first row of tile k + 1.
__global__ __launch_bounds__(256) void k_csr_tiles(const int32_t *__restrict__ row_ptr, int64_t m, int64_t nnz, int64_t ntiles,
                                                    int64_t tile_size, int64_t row_align, int32_t *__restrict__ tile_rp)
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
        r = (lo + row_align - 1) / row_align * row_align;
        r = r < m ? r : m;
    }
    tile_rp[2 * k] = (int32_t)r;
    tile_rp[2 * k + 1] = (r < m) ? row_ptr[r] : (int32_t)nnz;
}

// Every thread fetches x for the entries it streams (entry order, all loads of a tile in flight together) and stores
// the products in LDS; the rows are then summed from LDS, G lanes per row, without touching global memory again.
//
// The life of a block is a chain of memory round trips, and the order of the requests is chosen so that the chain is
// as short as it can be: tile header (scalar load) -> [all column indices, all values, the row pointers of the first
// two passes of rows: one batch, nothing in it waits for anything else] -> x gathers as soon as the columns are there
// (loads return in order of issue and the columns were issued first, so the values and row pointers are still on
// their way) -> products to LDS -> sums.  Loads are unconditional, with the entry index clamped into the tile, so that
// no branch and no wait separates them.
template <typename T, int TILE, int G, bool ACC>
__global__ __launch_bounds__(CSR_B) void k_csr_tiled(const int32_t *__restrict__ tile_rp, const int32_t *__restrict__ row_ptr,
                                                     const int32_t *__restrict__ col_idx, const T *__restrict__ val,
                                                     const T *__restrict__ x, T *__restrict__ y, int64_t m)
{
    constexpr int CAP = TILE + CSR_TILE_SLACK + CSR_HEAD;
    constexpr int FULL = TILE / CSR_B;                   // loads every thread of every tile issues
    constexpr int EPT = (CAP + CSR_B - 1) / CSR_B;       // the rest only where the tile reaches that far
    constexpr int RPB = CSR_B / G;
    constexpr int RU = 4;   // LDS reads of a lane that are in flight together while a row is summed
    __shared__ T ps[CAP];
    const int64_t tile = xcd_block(blockIdx.x, gridDim.x);
    const int2v a = *reinterpret_cast<const int2v *>(tile_rp + 2 * tile);
    const int2v b = *reinterpret_cast<const int2v *>(tile_rp + 2 * tile + 2);
    const int64_t ra = a.x, rb = b.x;
    // the stream starts on a 128-byte boundary of the column array (256 of the value array) at or below the first
    // owned entry: every wave then reads whole cache lines; the up to CSR_HEAD - 1 entries before the first owned
    // one belong to the previous tile and are not used
    const int32_t p0 = a.y & ~(CSR_HEAD - 1);
    int cnt = b.y - p0;
    cnt = cnt < CAP ? cnt : CAP;
    const int sub = threadIdx.x % G;
    const int64_t nrows = rb - ra;
    const int last = cnt > 0 ? cnt - 1 : 0;
    const int32_t *cbase = col_idx + p0;
    const T *vbase = val + p0;
    int32_t c[EPT];
    T v[EPT];
    int32_t rp[4];
    if (cnt > 0) {   // uniform
#pragma unroll
        for (int j = 0; j < EPT; ++j) {
            const int i = threadIdx.x + j * CSR_B;
            if (j < FULL) c[j] = ld_stream(cbase + (i < cnt ? i : last));
            else { c[j] = 0; if (i < cnt) c[j] = ld_stream(cbase + i); }
        }
#pragma unroll
        for (int j = 0; j < EPT; ++j) {
            const int i = threadIdx.x + j * CSR_B;
            if (j < FULL) v[j] = ld_stream(vbase + (i < cnt ? i : last));
            else { v[j] = (T)0; if (i < cnt) v[j] = ld_stream(vbase + i); }
        }
    }
    {   // row pointers of the rows this thread sums in the first two passes (clamped: row_ptr has m + 1 entries)
        const int64_t r0 = ra + threadIdx.x / G, r1 = r0 + RPB;
        rp[0] = row_ptr[r0 < m ? r0 : m]; rp[1] = row_ptr[r0 + 1 < m ? r0 + 1 : m];
        rp[2] = row_ptr[r1 < m ? r1 : m]; rp[3] = row_ptr[r1 + 1 < m ? r1 + 1 : m];
    }
    if (cnt > 0) {
        T xv[EPT];
#pragma unroll
        for (int j = 0; j < EPT; ++j) {
            const int i = threadIdx.x + j * CSR_B;
            if (j < FULL) xv[j] = x[c[j]];
            else { xv[j] = (T)0; if (i < cnt) xv[j] = x[c[j]]; }
        }
#pragma unroll
        for (int j = 0; j < EPT; ++j) {
            const int i = threadIdx.x + j * CSR_B;
            if (i < cnt) ps[i] = v[j] * xv[j];
        }
    }
    __syncthreads();
    for (int64_t base = 0; base < nrows; base += RPB) {
        const int64_t r = ra + base + threadIdx.x / G;
        int lo, hi;
        if (base == 0) { lo = rp[0] - p0; hi = rp[1] - p0; }
        else if (base == RPB) { lo = rp[2] - p0; hi = rp[3] - p0; }
        else { lo = row_ptr[r < m ? r : m] - p0; hi = row_ptr[r + 1 < m ? r + 1 : m] - p0; }
        if (r >= rb) lo = hi = 0;
        T sum = (T)0;
        int e = lo + sub;
        for (; e + (RU - 1) * G < hi; e += RU * G) {
            T t[RU];
#pragma unroll
            for (int u = 0; u < RU; ++u) t[u] = ps[e + u * G];
#pragma unroll
            for (int u = 0; u < RU; ++u) sum += t[u];
        }
        for (; e < hi; e += G) sum += ps[e];
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
    // A tile that owns far more rows than it has entries (a long stretch of empty rows: the remainder of an HDC matrix
    // whose scattered entries sit in a few rows) walks only the rows between its first and its last entry; the empty
    // rows around them are zeroed without a look at row_ptr, or left alone when accumulating (half a million of them
    // in one tile took 1.8 ms).
    int64_t r_lo = ra, r_hi = rb;
    if (nrows > 4 * (int64_t)TILE) {   // uniform
        __shared__ int64_t s_rng[2];
        if (threadIdx.x == 0) {
            if (cnt > seg) {
                s_rng[0] = row_of_entry(row_ptr, ra, rb - 1, t0 + seg);
                s_rng[1] = row_of_entry(row_ptr, ra, rb - 1, t0 + cnt - 1) + 1;
            } else {
                s_rng[0] = rb; s_rng[1] = rb;
            }
        }
        __syncthreads();
        r_lo = s_rng[0]; r_hi = s_rng[1];
        if (!ACC) {
            for (int64_t r = ra + threadIdx.x; r < r_lo; r += CSR_B) y[r] = (T)0;
            for (int64_t r = r_hi + threadIdx.x; r < rb; r += CSR_B) y[r] = (T)0;
        }
    }
    for (int64_t base = 0; base < r_hi - r_lo; base += RPB) {
        const int64_t r = r_lo + base + threadIdx.x / G;
        if (base > 0 || r_lo != ra) {
            lo = hi = 0;
            if (r < r_hi) { lo = row_ptr[r] - (int32_t)t0; hi = row_ptr[r + 1] - (int32_t)t0; }
        }
        hi = hi < cnt ? hi : cnt;
        const bool is_long = hi - lo > CSR_LONG_SEG;
        T sum = (T)0;
        if (!is_long)
            for (int e = lo + sub; e < hi; e += G) sum += ps[e];
        if (G > 1) sum = group_sum_down(sum, G);
        if (sub == 0 && r < r_hi) {
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
    if (acc) hipLaunchKernelGGL((k_csr_tiled<T, TILE, G, true>), dim3(grid), dim3(CSR_B), 0, s, a.csr_tile_rp, a.csr_row_ptr, a.csr_col,
                                (const T *)a.csr_val, x, y, a.m);
    else hipLaunchKernelGGL((k_csr_tiled<T, TILE, G, false>), dim3(grid), dim3(CSR_B), 0, s, a.csr_tile_rp, a.csr_row_ptr, a.csr_col,
                            (const T *)a.csr_val, x, y, a.m);
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
static mo_status launch_split_g(const mo_matrix &a, const T *x, T *y, bool acc, hipStream_t s)
{
    switch (a.csr_group) {
    case 1: return launch_split<T, TILE, 1>(a, x, y, acc, s);
    case 2: return launch_split<T, TILE, 2>(a, x, y, acc, s);
    case 4: return launch_split<T, TILE, 4>(a, x, y, acc, s);
    case 8: return launch_split<T, TILE, 8>(a, x, y, acc, s);
    default: return launch_split<T, TILE, 16>(a, x, y, acc, s);
    }
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
    if (a.csr_split)
        return a.csr_tile == CSR_TILE_SMALL ? launch_split_g<T, CSR_TILE_SMALL>(a, x, y, acc, s) : launch_split_g<T, CSR_TILE>(a, x, y, acc, s);
    if (a.csr_tile == CSR_TILE_LARGE) return launch_tiled_g<T, CSR_TILE_LARGE>(a, x, y, acc, s);
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

mo_status csr_build_tiles(const int32_t *row_ptr, int64_t m, int64_t nnz, int64_t ntiles, int tile_size, int row_align, int32_t *tile_rp,
                          hipStream_t s)
{
    hipLaunchKernelGGL(k_csr_tiles, dim3((unsigned)((ntiles + 1 + 255) / 256)), dim3(256), 0, s, row_ptr, m, nnz, ntiles,
                       (int64_t)tile_size, (int64_t)row_align, tile_rp);
    MO_LAUNCH_CHECK();
    return MO_OK;
}

}  // namespace mo

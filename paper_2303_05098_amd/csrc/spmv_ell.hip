// ELL SpMV (Section II-B: at most K entries per row, one K-wide value slab and one K-wide column slab).
// Slot-major storage, one row per lane: value and column reads are contiguous across the wave.  Rows are packed
// from slot 0, so the first padding marker (col = -1) ends a row.
#include "dev_common.hpp"
#include "mo_internal.hpp"

#include <type_traits>

namespace mo {

constexpr int ELL_B = 256;
constexpr int ELL_U = 8;   // slots fetched together
constexpr int ELL_WIN_B = 512;                      // rows per block of the kernel with x windows
constexpr int64_t ELL_WIN_LDS_BYTES = 40 * 1024;    // LDS budget of its windows
constexpr int ELL_WIN_RUNS = (int)(ELL_WIN_LDS_BYTES / 4 / ELL_WIN_B);   // runs of ELL_WIN_B staged positions at most

// sum += A(row, slots s, s + step, ...) * x over the slots [s0, s1) of one row.  The loads of ELL_U slots are issued
// together (a padded slot reads x[0] twice and is masked out of the sum; a slot past s1, in the last group, is skipped
// by a condition that is the same for every lane), so that no load waits for a branch on the one before it, and the
// column indices of the next ELL_U slots are requested before the values and x entries of the current ones are waited
// for: a group of slots costs one memory round trip instead of two, and the ragged end of a row costs one group, not
// two round trips per slot.  The order of the additions is the slot order.
//
// RUN: the row also owns the entries [p0, p1) of a COO part (HYB), which are added after the slots, in order.  The
// first of them travels with the slots: its column and value are requested with the first group's values, its x entry
// with the second group's, so a row with a single such entry (the usual case) pays no round trip of its own.
template <typename T, bool RUN = false>
__device__ __forceinline__ T ell_row_sum(const int32_t *__restrict__ c, const T *__restrict__ v, int64_t ld, int64_t s0, int64_t s1,
                                         int64_t step, const T *__restrict__ x, const int32_t *__restrict__ ccol = nullptr,
                                         const T *__restrict__ cval = nullptr, int32_t p0 = 0, int32_t p1 = 0)
{
    T sum = (T)0;
    int32_t jn[ELL_U];
    // column indices of the group that starts at slot s: unguarded when the whole group lies below s1
    auto request_columns = [&](int64_t s) {
        if (s + (ELL_U - 1) * step < s1) {
#pragma unroll
            for (int u = 0; u < ELL_U; ++u) jn[u] = ld_stream(c + (s + u * step) * ld);
        } else {
#pragma unroll
            for (int u = 0; u < ELL_U; ++u) {
                jn[u] = -1;
                if (s + u * step < s1) jn[u] = ld_stream(c + (s + u * step) * ld);
            }
        }
    };
    uint32_t cc = 0;
    T cv = (T)0, xg = (T)0;
    int groups = 0;
    int64_t s = s0;
    auto group = [&](auto ragged) {
        constexpr bool RG = decltype(ragged)::value;
        int32_t j[ELL_U];
        T a[ELL_U], xv[ELL_U];
#pragma unroll
        for (int u = 0; u < ELL_U; ++u) { j[u] = jn[u]; a[u] = (T)0; xv[u] = (T)0; }
        if (RUN && groups == 1) xg = x[cc];
#pragma unroll
        for (int u = 0; u < ELL_U; ++u) {   // a padded slot reads x[0] in place of its value: no slab traffic for padding
            if (!RG || s + u * step < s1) {
                a[u] = ld_stream(j[u] >= 0 ? v + (s + u * step) * ld : x);
                xv[u] = x[j[u] >= 0 ? j[u] : 0];
            }
        }
        if (RUN && groups == 0) {   // entry p0 of the run, or entry 0 of the part for a row without run (dropped later)
            const int32_t pc = p0 < p1 ? p0 : 0;
            cc = (uint32_t)ccol[pc];
            cv = cval[pc];
        }
        if (!RG && s + ELL_U * step < s1) request_columns(s + ELL_U * step);
#pragma unroll
        for (int u = 0; u < ELL_U; ++u) sum += j[u] >= 0 ? a[u] * xv[u] : (T)0;
        ++groups;
    };
    if (s < s1) request_columns(s);
    for (; s + (ELL_U - 1) * step < s1; s += ELL_U * step) group(std::false_type{});
    if (s < s1) group(std::true_type{});
    if (RUN) {
        if (groups == 0) {
            const int32_t pc = p0 < p1 ? p0 : 0;
            cc = (uint32_t)ccol[pc];
            cv = cval[pc];
        }
        if (groups < 2) xg = x[cc];
        if (p0 < p1) sum += cv * xg;
        for (int32_t p = p0 + 1; p < p1; ++p) sum += cval[p] * x[ccol[p]];
    }
    return sum;
}
template <typename T>
__global__ __launch_bounds__(ELL_B) void k_ell(const int32_t *__restrict__ col, const T *__restrict__ val, int64_t m, int64_t K,
                                                int64_t ld, const T *__restrict__ x, T *__restrict__ y)
{
    const int64_t lb = xcd_block(blockIdx.x, gridDim.x);
    const int64_t row = lb * ELL_B + threadIdx.x;
    if (row >= m) return;
    st_stream(y + row, ell_row_sum<T>(col + row, val + row, ld, 0, K, 1, x));
}

// One row per lane with x served from LDS windows (matrices with a window plan: most entries on a few groups of
// diagonals).  The rows [row0, row0 + B) of a block read x almost only inside x[row0 + lo_q, row0 + B - 1 + lo_q +
// span_q) for the groups q of the plan; the block fetches those windows once, coalesced, and every entry then finds
// its x value by comparing its column with the window bounds, which are the same for all lanes (scalar registers).
// An entry outside every window is gathered from global memory.  Measured on the 27-point stencil: the x gathers of
// k_ell cost 19 of its 129 us although consecutive lanes read consecutive x entries (every slot is one more memory
// instruction per wave; with x from a fixed LDS table the kernel ran in 110 us); the windows replace 27 gathers per row
// by 5 staged x entries per row, and the lookup costs part of that again: 123 us with 512-row blocks, 127 with 256.
// HYB: the row's lane also adds its run of the COO part (see k_ell_hyb).
template <typename T, int B, bool HYB>
__global__ __launch_bounds__(B) void k_ell_win(const int32_t *__restrict__ col, const T *__restrict__ val, int64_t m, int64_t n, int64_t K,
                                               int64_t ld, const int32_t *__restrict__ coo_rp, const int32_t *__restrict__ ccol,
                                               const T *__restrict__ cval, const T *__restrict__ x, T *__restrict__ y, const XPlan xp,
                                               const WinRuns<ELL_WIN_RUNS> runs)
{
    extern __shared__ __align__(16) unsigned char s_raw[];
    T *xs = reinterpret_cast<T *>(s_raw);
    const int64_t lb = xcd_block(blockIdx.x, gridDim.x);
    const int64_t row0 = lb * B;
    const int64_t row = row0 + threadIdx.x;
    const bool rv = row < m;
    const int64_t rr = rv ? row : m - 1;   // lanes past the end walk the last row and store nothing
    const int32_t *c = col + rr;
    const T *v = val + rr;
    // the first group of column indices is requested before the windows, so that both are on their way together; so
    // are the bounds of the row's run in the COO part (HYB)
    int32_t jn[ELL_U];
    auto request_columns = [&](int64_t s) {   // unguarded when the whole group lies below K
        if (s + ELL_U <= K) {
#pragma unroll
            for (int u = 0; u < ELL_U; ++u) jn[u] = ld_stream(c + (s + u) * ld);
        } else {
#pragma unroll
            for (int u = 0; u < ELL_U; ++u) {
                jn[u] = -1;
                if (s + u < K) jn[u] = ld_stream(c + (s + u) * ld);
            }
        }
    };
    if (K > 0) request_columns(0);
    int32_t p0 = 0, p1 = 0;
    if (HYB) { p0 = coo_rp[rr]; p1 = coo_rp[rr + 1]; }
    // the windows: all loads of a batch of runs issued before the first is stored (one memory latency per batch, and a
    // single batch is the rule)
    {
        constexpr int WB = 8;
        const int tid = (int)threadIdx.x;
        T w[WB];
        uint32_t w_in = 0;
        window_loads<T, B, WB>(runs, 0, tid, row0, n, x, w, &w_in);
#pragma unroll 1
        for (int u0 = WB; u0 * B < runs.elems; u0 += WB) {
            window_stores<T, B, WB>(runs, u0 - WB, tid, w, w_in, xs);
            window_loads<T, B, WB>(runs, u0, tid, row0, n, x, w, &w_in);
        }
        window_stores<T, B, WB>(runs, ((runs.elems + B - 1) / B - 1) / WB * WB, tid, w, w_in, xs);
    }
    __syncthreads();
    // window bounds of this block: the same for all lanes (scalar registers)
    int shift[XP_MAX_CL], wlen[XP_MAX_CL], wbase[XP_MAX_CL];
    {
        int base = 0;
#pragma unroll
        for (int q = 0; q < XP_MAX_CL; ++q) {
            const bool on = q < xp.ncl;
            wlen[q] = on ? xp.span[q] + B - 1 : 0;               // an unused group matches nothing
            shift[q] = on ? (int)row0 + xp.lo[q] : 0;            // row0 + lo fits 32 bits: |lo| < m + n < 2^31
            wbase[q] = base;
            base += wlen[q];
        }
    }
    T sum = (T)0;
    uint32_t cc = 0;   // HYB: the first entry of the row's COO run travels with the slots (see ell_row_sum)
    T cv = (T)0, xg = (T)0;
    int groups = 0;
    int64_t s = 0;
    auto group = [&](auto ragged) {   // ragged: the last group of a row whose K is no multiple of ELL_U skips the slots past K
        constexpr bool RG = decltype(ragged)::value;
        int32_t j[ELL_U];
        T a[ELL_U], xv[ELL_U];
        int pos[ELL_U];
        bool hit[ELL_U];
#pragma unroll
        for (int u = 0; u < ELL_U; ++u) { j[u] = jn[u]; pos[u] = 0; hit[u] = false; a[u] = (T)0; xv[u] = (T)0; }
        if (HYB && groups == 1) xg = x[cc];
#pragma unroll
        for (int u = 0; u < ELL_U; ++u)
            if (!RG || s + u < K) a[u] = ld_stream(j[u] >= 0 ? v + (s + u) * ld : x);   // padding: no slab traffic
        if (HYB && groups == 0) {
            const int32_t pc = p0 < p1 ? p0 : 0;
            cc = (uint32_t)ccol[pc];
            cv = cval[pc];
        }
        for (int q = 0; q < xp.ncl; ++q) {                    // uniform trip count
            const int sh = shift[q], ln = wlen[q], bs = wbase[q];
#pragma unroll
            for (int u = 0; u < ELL_U; ++u) {
                const unsigned idx = (unsigned)(j[u] - sh);
                const bool in = idx < (unsigned)ln;
                pos[u] = in ? bs + (int)idx : pos[u];
                hit[u] = hit[u] || in;
            }
        }
        bool all = true;
#pragma unroll
        for (int u = 0; u < ELL_U; ++u) all = all && (hit[u] || j[u] < 0);
        if (!all) {
#pragma unroll
            for (int u = 0; u < ELL_U; ++u) xv[u] = x[(j[u] >= 0 && !hit[u]) ? j[u] : 0];
        }
        if (!RG && s + ELL_U < K) request_columns(s + ELL_U);
#pragma unroll
        for (int u = 0; u < ELL_U; ++u) {
            const T xl = xs[pos[u]];
            const T xu = hit[u] ? xl : (all ? (T)0 : xv[u]);
            sum += j[u] >= 0 ? a[u] * xu : (T)0;
        }
        ++groups;
    };
    for (; s + ELL_U <= K; s += ELL_U) group(std::false_type{});
    if (s < K) group(std::true_type{});
    if (HYB) {
        if (groups == 0) {
            const int32_t pc = p0 < p1 ? p0 : 0;
            cc = (uint32_t)ccol[pc];
            cv = cval[pc];
        }
        if (groups < 2) xg = x[cc];
        if (p0 < p1) sum += cv * xg;
        for (int32_t p = p0 + 1; p < p1; ++p) sum += cval[p] * x[ccol[p]];
    }
    if (rv) st_stream(y + row, sum);
}

// Small matrices: one row per lane leaves most of the chip idle and makes every lane walk all K slots in sequence.
// Here a block owns 64 rows and its four waves take the slots s = w, w + 4, ...; the four partial sums of a row are
// added in wave order through LDS (fixed order, so reruns are bit-identical).
template <typename T>
__global__ __launch_bounds__(ELL_B) void k_ell_split(const int32_t *__restrict__ col, const T *__restrict__ val, int64_t m, int64_t K,
                                                      int64_t ld, const T *__restrict__ x, T *__restrict__ y)
{
    constexpr int NW = ELL_B / WAVE;
    __shared__ T part[NW][WAVE];
    const int lane = lane_id(), w = threadIdx.x / WAVE;
    const int64_t row = (int64_t)blockIdx.x * WAVE + lane;
    T sum = (T)0;
    if (row < m) sum = ell_row_sum<T>(col + row, val + row, ld, w, K, NW, x);
    part[w][lane] = sum;
    __syncthreads();
    if (w == 0 && row < m) {
        T t = part[0][lane];
#pragma unroll
        for (int q = 1; q < NW; ++q) t += part[q][lane];
        y[row] = t;
    }
}

// HYB whose rows keep only a few entries in the COO part: the row's lane adds its own COO run (found through the
// positions of the row runs that the handle keeps) right after its ELL slots, so y is written once by one kernel
// instead of being written by the ELL kernel and read, updated and written again by the COO kernel.
template <typename T>
__global__ __launch_bounds__(ELL_B) void k_ell_hyb(const int32_t *__restrict__ col, const T *__restrict__ val, int64_t m, int64_t K,
                                                    int64_t ld, const int32_t *__restrict__ coo_rp, const int32_t *__restrict__ ccol,
                                                    const T *__restrict__ cval, const T *__restrict__ x, T *__restrict__ y)
{
    const int64_t lb = xcd_block(blockIdx.x, gridDim.x);
    const int64_t row = lb * ELL_B + threadIdx.x;
    if (row >= m) return;
    const int32_t p0 = coo_rp[row], p1 = coo_rp[row + 1];
    st_stream(y + row, ell_row_sum<T, true>(col + row, val + row, ld, 0, K, 1, x, ccol, cval, p0, p1));
}

// LDS bytes of the windows for blocks of B rows, or 0 when the plan does not pay: no plan, windows beyond the budget,
// or more staged x entries than a third of the entries a block multiplies (then the gathers are the cheaper way).
template <typename T>
static size_t ell_window_bytes(const mo_matrix &a, int B)
{
    if (a.xplan.ncl <= 0 || a.m <= ELL_SPLIT_MAX_ROWS) return 0;   // 512-row blocks leave a small matrix on too few CUs
    int64_t elems = 0;
    for (int q = 0; q < a.xplan.ncl; ++q) elems += (int64_t)a.xplan.span[q] + B - 1;
    if (elems * (int64_t)sizeof(T) > ELL_WIN_LDS_BYTES) return 0;
    const double per_block = (double)B * ((double)a.nnz / (double)a.m);
    if ((double)elems * 3.0 > per_block) return 0;
    return (size_t)elems * sizeof(T);
}

template <typename T, bool HYB>
static mo_status ell_win_launch(const mo_matrix &a, const void *x, void *y, size_t lds, hipStream_t s)
{
    constexpr int B = ELL_WIN_B;
    const unsigned grid = (unsigned)((a.m + B - 1) / B);
    WinRuns<ELL_WIN_RUNS> runs;   // the staging order of the windows, from the plan (a few dozen integer operations)
    int32_t wlen[XP_MAX_CL];
    for (int q = 0; q < a.xplan.ncl; ++q) wlen[q] = a.xplan.span[q] + B - 1;
    if (!plan_window_runs(a.xplan.lo, wlen, a.xplan.ncl, B, &runs) || (size_t)runs.elems * sizeof(T) != lds) return MO_E_SHAPE;
    hipLaunchKernelGGL((k_ell_win<T, B, HYB>), dim3(grid), dim3(B), lds, s, a.ell_col, (const T *)a.ell_val, a.m, a.n, a.k, a.ld, a.coo_rp,
                       a.coo_col, (const T *)a.coo_val, (const T *)x, (T *)y, a.xplan, runs);
    MO_LAUNCH_CHECK();
    return MO_OK;
}

template <typename T>
static mo_status hyb_fused_typed(const mo_matrix &a, const void *x, void *y, hipStream_t s)
{
    if (const size_t lds = ell_window_bytes<T>(a, ELL_WIN_B)) return ell_win_launch<T, true>(a, x, y, lds, s);
    const unsigned grid = (unsigned)((a.m + ELL_B - 1) / ELL_B);
    hipLaunchKernelGGL(k_ell_hyb<T>, dim3(grid), dim3(ELL_B), 0, s, a.ell_col, (const T *)a.ell_val, a.m, a.k, a.ld, a.coo_rp, a.coo_col,
                       (const T *)a.coo_val, (const T *)x, (T *)y);
    MO_LAUNCH_CHECK();
    return MO_OK;
}

template <typename T>
static mo_status ell_typed(const mo_matrix &a, const void *x, void *y, hipStream_t s)
{
    if (a.m <= ELL_SPLIT_MAX_ROWS && a.k >= ELL_SPLIT_MIN_K) {
        const unsigned g = (unsigned)((a.m + WAVE - 1) / WAVE);
        hipLaunchKernelGGL(k_ell_split<T>, dim3(g), dim3(ELL_B), 0, s, a.ell_col, (const T *)a.ell_val, a.m, a.k, a.ld, (const T *)x, (T *)y);
        MO_LAUNCH_CHECK();
        return MO_OK;
    }
    if (const size_t lds = ell_window_bytes<T>(a, ELL_WIN_B)) return ell_win_launch<T, false>(a, x, y, lds, s);
    const unsigned grid = (unsigned)((a.m + ELL_B - 1) / ELL_B);
    hipLaunchKernelGGL(k_ell<T>, dim3(grid), dim3(ELL_B), 0, s, a.ell_col, (const T *)a.ell_val, a.m, a.k, a.ld, (const T *)x, (T *)y);
    MO_LAUNCH_CHECK();
    return MO_OK;
}

bool ell_uses_windows(const mo_matrix &a)
{
    return (a.dtype == MO_F32 ? ell_window_bytes<float>(a, ELL_WIN_B) : ell_window_bytes<double>(a, ELL_WIN_B)) > 0;
}

mo_status spmv_hyb_fused(const mo_matrix &a, const void *x, void *y, hipStream_t s)
{
    return a.dtype == MO_F32 ? hyb_fused_typed<float>(a, x, y, s) : hyb_fused_typed<double>(a, x, y, s);
}

mo_status spmv_ell(const mo_matrix &a, const void *x, void *y, hipStream_t s)
{
    return a.dtype == MO_F32 ? ell_typed<float>(a, x, y, s) : ell_typed<double>(a, x, y, s);
}

}  // namespace mo

// Switching away from any format, and features of a matrix in whatever format it is held.
//
// The paper's tuner inspects the active format of the matrix without converting it back (Section VI-C: statistics
// per format, no transfers between memory spaces), and the container can switch between any two formats at run time
// (Section II-C).  Here:
//   * row lengths and diagonal counts are gathered straight from the arrays of each format (DIA slabs, ELL slabs,
//     COO triples, CSR remainder), with the same two-level merging of diagonal counts as the CSR kernels;
//   * any -> CSR rebuilds row_ptr from the row lengths (exclusive scan) and writes each row's entries in ascending
//     column order (DIA and CSR parts of HDC are merged by column; the COO part of HYB follows its ELL part);
//   * any -> any is any -> CSR followed by the CSR -> format conversion.
// A DIA slab cannot tell a stored zero from padding: positions holding exactly 0 are not entries on the way back.
#include "dev_common.hpp"
#include "feat_common.hpp"
#include "mo_internal.hpp"

#include <cmath>

namespace mo {

// Everything a kernel needs to walk a handle, by value.
template <typename T>
struct View {
    int64_t m, n, ld, nd, k, nnz_coo;
    const int32_t *dia_off;
    const T *dia_val;
    const int32_t *ell_col;
    const T *ell_val;
    const int32_t *coo_row, *coo_col;
    const T *coo_val;
    const int32_t *csr_row_ptr, *csr_col;
    const T *csr_val;
};

template <typename T>
static View<T> make_view(const mo_matrix &a)
{
    View<T> v{};
    v.m = a.m; v.n = a.n; v.ld = a.ld;
    const bool dia = a.fmt == MO_DIA || a.fmt == MO_HDC, ell = a.fmt == MO_ELL || a.fmt == MO_HYB;
    const bool coo = a.fmt == MO_COO || a.fmt == MO_HYB, csr = a.fmt == MO_CSR || a.fmt == MO_HDC;
    v.nd = dia ? a.nd : 0; v.dia_off = a.dia_off; v.dia_val = (const T *)a.dia_val;
    v.k = ell ? a.k : 0; v.ell_col = a.ell_col; v.ell_val = (const T *)a.ell_val;
    v.nnz_coo = coo ? a.nnz_coo : 0; v.coo_row = a.coo_row; v.coo_col = a.coo_col; v.coo_val = (const T *)a.coo_val;
    v.csr_row_ptr = csr ? a.csr_row_ptr : nullptr; v.csr_col = a.csr_col; v.csr_val = (const T *)a.csr_val;
    return v;
}

// First position p in [lo, hi) of the sorted COO row array with coo_row[p] >= r (hi if there is none).
__device__ __forceinline__ int64_t coo_lower_bound(const int32_t *__restrict__ coo_row, int64_t lo, int64_t hi, int64_t r)
{
    while (lo < hi) {
        const int64_t mid = (lo + hi) >> 1;
        if ((int64_t)coo_row[mid] < r) lo = mid + 1; else hi = mid;
    }
    return lo;
}

// ------------------------------------------------------------------ row lengths of any format
template <typename T>
__global__ __launch_bounds__(FB) void k_len_any(View<T> v, int32_t *__restrict__ len)
{
    // the block's rows own one contiguous range of the sorted COO part: two threads find it in the whole array,
    // then every lane searches only inside it
    __shared__ int64_t s_coo[2];
    const int64_t row0 = (int64_t)blockIdx.x * FB;
    if (v.nnz_coo > 0 && threadIdx.x < 2) {
        const int64_t rend = row0 + FB < v.m ? row0 + FB : v.m;
        s_coo[threadIdx.x] = coo_lower_bound(v.coo_row, 0, v.nnz_coo, threadIdx.x == 0 ? row0 : rend);
    }
    __syncthreads();
    const int64_t row = row0 + threadIdx.x;
    if (row >= v.m) return;
    int c = 0;
    for (int64_t k = 0; k < v.nd; ++k) {
        const int64_t j = row + v.dia_off[k];
        if (j >= 0 && j < v.n && v.dia_val[k * v.ld + row] != (T)0) ++c;
    }
    for (int64_t s = 0; s < v.k; ++s)
        if (v.ell_col[s * v.ld + row] >= 0) ++c;
    if (v.nnz_coo > 0) {
        const int64_t q = coo_lower_bound(v.coo_row, s_coo[0], s_coo[1], row);
        c += (int)(coo_lower_bound(v.coo_row, q, s_coo[1], row + 1) - q);
    }
    if (v.csr_row_ptr) c += v.csr_row_ptr[row + 1] - v.csr_row_ptr[row];
    len[row] = c;
}

// max, min, sum, sum of squares of the row lengths (one set of atomics per block).
__global__ __launch_bounds__(FB) void k_len_stats(const int32_t *__restrict__ len, int64_t m, Counters *ctr, unsigned long long *total)
{
    unsigned long long mx = 0ull, mn = ~0ull, sq = 0ull, sm = 0ull;
    const int64_t stride = (int64_t)gridDim.x * FB;
    for (int64_t i = (int64_t)blockIdx.x * FB + threadIdx.x; i < m; i += stride) {
        const unsigned long long l = (unsigned long long)len[i];
        mx = l > mx ? l : mx; mn = l < mn ? l : mn; sq += l * l; sm += l;
    }
    mx = wave_max(mx); mn = wave_min(mn); sq = wave_sum(sq); sm = wave_sum(sm);
    __shared__ unsigned long long s_mx[FB / WAVE], s_mn[FB / WAVE], s_sq[FB / WAVE], s_sm[FB / WAVE];
    if (lane_id() == 0) { const int w = threadIdx.x / WAVE; s_mx[w] = mx; s_mn[w] = mn; s_sq[w] = sq; s_sm[w] = sm; }
    __syncthreads();
    if (threadIdx.x == 0) {
        for (int w = 1; w < FB / WAVE; ++w) {
            mx = s_mx[w] > mx ? s_mx[w] : mx; mn = s_mn[w] < mn ? s_mn[w] : mn; sq += s_sq[w]; sm += s_sm[w];
        }
        atomicMax(&ctr->max_row, mx); atomicMin(&ctr->min_row, mn); atomicAdd(&ctr->sum_sq, sq); atomicAdd(total, sm);
    }
}

// ------------------------------------------------------------------ diagonal counts of any format
// DIA part: the count of diagonal off_k is the number of in-matrix, non-zero positions of slab k.
// blockIdx.x = diagonal, blockIdx.y = chunk of rows; one atomic per block.
template <typename T>
__global__ __launch_bounds__(FB) void k_hist_dia(View<T> v, uint32_t *__restrict__ hist)
{
    const int64_t k = blockIdx.x;
    const int64_t off = v.dia_off[k];
    unsigned int c = 0;
    const int64_t stride = (int64_t)gridDim.y * FB;
    for (int64_t row = (int64_t)blockIdx.y * FB + threadIdx.x; row < v.m; row += stride) {
        const int64_t j = row + off;
        if (j >= 0 && j < v.n && v.dia_val[k * v.ld + row] != (T)0) ++c;
    }
    c = wave_sum(c);
    __shared__ unsigned int s_c[FB / WAVE];
    if (lane_id() == 0) s_c[threadIdx.x / WAVE] = c;
    __syncthreads();
    if (threadIdx.x == 0) {
        for (int w = 1; w < FB / WAVE; ++w) c += s_c[w];
        if (c) atomicAdd(&hist[off + (v.m - 1)], c);
    }
}

// ELL, COO and CSR parts: one row per lane for the slabs and the CSR remainder (equal diagonals meet in the same
// step and are merged by ballot), one entry per lane for COO; everything goes through the block's LDS hash table.
template <typename T>
__global__ __launch_bounds__(FB) void k_hist_parts(View<T> v, int64_t rows_per_block, int64_t coo_per_block, uint32_t *__restrict__ hist)
{
    __shared__ int ht_key[HT_SIZE];
    __shared__ uint32_t ht_cnt[HT_SIZE];
    __shared__ int ht_full;
    if (threadIdx.x == 0) ht_full = 0;
    for (int i = threadIdx.x; i < HT_SIZE; i += FB) { ht_key[i] = -1; ht_cnt[i] = 0u; }
    __syncthreads();
    const int lane = lane_id();
    auto merged = [&](bool ok, int key) {   // called by whole waves
        uint64_t todo = ballot64(ok);
        int rounds = 0;
        while (todo) {
            if (rounds == MERGE_ROUNDS) {
                if ((todo >> lane) & 1ull) count_key(key, 1u, ht_key, ht_cnt, &ht_full, hist);
                break;
            }
            const int leader = __ffsll((unsigned long long)todo) - 1;
            const int lkey = __shfl(key, leader, WAVE);
            const uint64_t same = ballot64(ok && key == lkey) & todo;
            if (lane == leader) count_key(lkey, (uint32_t)__popcll(same), ht_key, ht_cnt, &ht_full, hist);
            todo &= ~same;
            ++rounds;
        }
    };
    const int64_t row_begin = (int64_t)blockIdx.x * rows_per_block;
    int64_t row_end = row_begin + rows_per_block;
    row_end = row_end < v.m ? row_end : v.m;
    for (int64_t base = row_begin; base < row_end; base += FB) {   // uniform trip count across the block
        const int64_t row = base + threadIdx.x;
        const bool rv = row < row_end;
        for (int64_t s = 0; s < v.k; ++s) {
            const int c = rv ? v.ell_col[s * v.ld + row] : -1;
            merged(c >= 0, (int)((int64_t)c - row + (v.m - 1)));
        }
        if (v.csr_row_ptr) {
            const int lo = rv ? v.csr_row_ptr[row] : 0, hi = rv ? v.csr_row_ptr[row + 1] : 0;
            const int wmax = wave_max(hi - lo);
            for (int q = 0; q < wmax; ++q) {
                const bool act = q < hi - lo;
                const int c = act ? v.csr_col[lo + q] : 0;
                merged(act, (int)((int64_t)c - row + (v.m - 1)));
            }
        }
    }
    const int64_t p_begin = (int64_t)blockIdx.x * coo_per_block;
    int64_t p_end = p_begin + coo_per_block;
    p_end = p_end < v.nnz_coo ? p_end : v.nnz_coo;
    for (int64_t base = p_begin; base < p_end; base += FB) {   // uniform trip count: merged() is a wave operation
        const int64_t p = base + threadIdx.x;
        const bool act = p < p_end;
        merged(act, act ? (int)((int64_t)v.coo_col[p] - v.coo_row[p] + (v.m - 1)) : 0);
    }
    __syncthreads();
    for (int i = threadIdx.x; i < HT_SIZE; i += FB) {
        const uint32_t c = ht_cnt[i];
        if (c) atomicAdd(&hist[ht_key[i]], c);
    }
}

// ------------------------------------------------------------------ any -> CSR
// One row per lane; the row's entries leave in ascending column order.  A block's 256 rows own one contiguous range
// of the output, which is staged through LDS in chunks of FILL_CH entries so that the global writes are coalesced
// (a lane writing its row directly would scatter 4- and 8-byte stores one row length apart).
constexpr int FILL_CH = 2048;

// MODE 0: any mix of parts, one entry at a time.  MODE 1: DIA part merged by column with the CSR part, if there is
// one (DIA, HDC); MODE 2: ELL part followed by the COO part (ELL, HYB): the slab is read FILL_U slots at a time with
// unconditional loads, so that a lane has FILL_U lines in flight instead of one per memory latency.  These two modes
// walk the row from its start for every chunk and keep what falls into the chunk; rpb (rows per block) is chosen on
// the host so that a block normally needs one chunk.
constexpr int FILL_U = 8;

template <typename T, int MODE>
__global__ __launch_bounds__(FB) void k_fill_csr_any(View<T> v, const int32_t *__restrict__ out_ptr, int32_t *__restrict__ ocol,
                                                      T *__restrict__ oval, int rpb)
{
    __shared__ int32_t s_col[FILL_CH];
    __shared__ T s_val[FILL_CH];
    __shared__ int64_t s_coo[2];
    const int64_t row0 = (int64_t)blockIdx.x * rpb;
    const int64_t row = row0 + threadIdx.x;
    const bool rv = (int)threadIdx.x < rpb && row < v.m;
    const int64_t rend = row0 + rpb < v.m ? row0 + rpb : v.m;
    if (v.nnz_coo > 0 && threadIdx.x < 2) s_coo[threadIdx.x] = coo_lower_bound(v.coo_row, 0, v.nnz_coo, threadIdx.x == 0 ? row0 : rend);
    __syncthreads();
    const int64_t out_lo = out_ptr[row0], out_hi = out_ptr[rend];
    const int64_t pos_begin = rv ? (int64_t)out_ptr[row] : out_hi;
    const int64_t pos_end = rv ? (int64_t)out_ptr[row + 1] : out_hi;
    int64_t pos = pos_begin;
    // cursors into the four possible sources of this row
    int64_t kd = 0, sl = 0, q = 0, qe = 0;
    int p = 0, pe = 0;
    if (rv && v.csr_row_ptr) { p = v.csr_row_ptr[row]; pe = v.csr_row_ptr[row + 1]; }
    if (rv && v.nnz_coo > 0) {
        q = coo_lower_bound(v.coo_row, s_coo[0], s_coo[1], row);
        qe = coo_lower_bound(v.coo_row, q, s_coo[1], row + 1);
    }
    // Next entry of the row: the DIA part and the CSR part (HDC holds both) are two ascending column sequences and
    // are merged; then the ELL part; then the COO part (HYB: the COO entries of a row come after its ELL entries).
    auto next = [&](int32_t &col, T &val) -> bool {
        int64_t jd = -1;
        T ad = (T)0;
        while (kd < v.nd) {
            const int64_t j = row + v.dia_off[kd];
            const T a = (j >= 0 && j < v.n) ? v.dia_val[kd * v.ld + row] : (T)0;
            if (a != (T)0) { jd = j; ad = a; break; }
            ++kd;
        }
        const bool has_d = jd >= 0, has_c = p < pe;
        if (has_d && (!has_c || jd < (int64_t)v.csr_col[p])) { col = (int32_t)jd; val = ad; ++kd; return true; }
        if (has_c) { col = v.csr_col[p]; val = v.csr_val[p]; ++p; return true; }
        if (sl < v.k) {
            const int c = v.ell_col[sl * v.ld + row];
            if (c >= 0) { col = c; val = v.ell_val[sl * v.ld + row]; ++sl; return true; }
            sl = v.k;   // padding only follows the last entry of a row
        }
        if (q < qe) { col = v.coo_col[q]; val = v.coo_val[q]; ++q; return true; }
        return false;
    };
    const int64_t rc = rv ? row : (v.m - 1);                  // a row every lane may load from
    for (int64_t c0 = out_lo; c0 < out_hi; c0 += FILL_CH) {   // uniform trip count across the block
        const int64_t c1 = c0 + FILL_CH < out_hi ? c0 + FILL_CH : out_hi;
        if constexpr (MODE == 0) {
            while (pos < pos_end && pos < c1) {
                int32_t col = 0;
                T val = (T)0;
                if (!next(col, val)) { pos = pos_end; break; }   // cannot happen: the lengths were counted from the same arrays
                s_col[pos - c0] = col;
                s_val[pos - c0] = val;
                ++pos;
            }
        } else {
            const bool touch = rv && pos_begin < c1 && pos_end > c0;
            pos = pos_begin;
            auto emit = [&](int32_t col, T val) {
                if (pos >= c0 && pos < c1) { s_col[pos - c0] = col; s_val[pos - c0] = val; }
                ++pos;
            };
            if constexpr (MODE == 1) {
                // HDC: the row's CSR entries (ascending columns, as the diagonals are) are slipped in before the first
                // DIA entry of a larger column
                int pc = p;
                int32_t cc = (touch && pc < pe) ? v.csr_col[pc] : 0x7fffffff;
                for (int64_t k0 = 0; k0 < v.nd && ballot64(touch && pos < pos_end && pos < c1) != 0ull; k0 += FILL_U) {
                    T a[FILL_U];
#pragma unroll
                    for (int u = 0; u < FILL_U; ++u) a[u] = v.dia_val[(k0 + u < v.nd ? k0 + u : v.nd - 1) * v.ld + rc];
#pragma unroll
                    for (int u = 0; u < FILL_U; ++u) {
                        if (k0 + u >= v.nd) break;
                        const int64_t j = row + v.dia_off[k0 + u];
                        if (touch && j >= 0 && j < v.n && a[u] != (T)0) {
                            while ((int64_t)cc < j) {
                                emit(cc, v.csr_val[pc]);
                                ++pc;
                                cc = pc < pe ? v.csr_col[pc] : 0x7fffffff;
                            }
                            emit((int32_t)j, a[u]);
                        }
                    }
                }
                if (touch)
                    for (; pc < pe; ++pc) emit(v.csr_col[pc], v.csr_val[pc]);
            } else {
                for (int64_t s0 = 0; s0 < v.k && ballot64(touch && pos < pos_end && pos < c1) != 0ull; s0 += FILL_U) {
                    int32_t c[FILL_U];
                    T a[FILL_U];
#pragma unroll
                    for (int u = 0; u < FILL_U; ++u) {
                        const int64_t at = (s0 + u < v.k ? s0 + u : v.k - 1) * v.ld + rc;
                        c[u] = v.ell_col[at];
                        a[u] = v.ell_val[at];
                    }
#pragma unroll
                    for (int u = 0; u < FILL_U; ++u)
                        if (touch && s0 + u < v.k && c[u] >= 0) emit(c[u], a[u]);
                }
                if (touch)
                    for (int64_t t = q; t < qe; ++t) emit(v.coo_col[t], v.coo_val[t]);
            }
        }
        __syncthreads();
        for (int64_t i = c0 + threadIdx.x; i < c1; i += FB) {
            ocol[i] = s_col[i - c0];
            oval[i] = s_val[i - c0];
        }
        __syncthreads();
    }
}

// ------------------------------------------------------------------ host side
struct TempCsr {   // device arrays of a rebuilt CSR; freed unless handed over
    hipStream_t s;
    int32_t *row_ptr = nullptr, *col = nullptr;
    void *val = nullptr;
    int64_t nnz = 0;
    explicit TempCsr(hipStream_t st) : s(st) {}
    ~TempCsr() { dev_free(row_ptr, s); dev_free(col, s); dev_free(val, s); }
    void release() { row_ptr = nullptr; col = nullptr; val = nullptr; }
};

template <typename T>
static mo_status rebuild_csr(const mo_matrix &a, TempCsr &out, hipStream_t s)
{
    const View<T> v = make_view<T>(a);
    Scratch scr(s);
    int32_t *len = (int32_t *)scr.get((size_t)a.m * 4);
    void *tmp = scr.get(scan_tmp_bytes(a.m));
    out.row_ptr = (int32_t *)dev_alloc((size_t)(a.m + 1) * 4, s);
    if (!len || !tmp || !out.row_ptr) return MO_E_ALLOC;
    const unsigned rb = (unsigned)((a.m + FB - 1) / FB);
    hipLaunchKernelGGL(k_len_any<T>, dim3(rb), dim3(FB), 0, s, v, len);
    MO_LAUNCH_CHECK();
    MO_TRY(exclusive_scan_i32(len, out.row_ptr, a.m, tmp, s));
    int32_t total = 0;
    MO_HIP(hipMemcpyAsync(&total, out.row_ptr + a.m, 4, hipMemcpyDeviceToHost, s));
    MO_HIP(hipStreamSynchronize(s));
    out.nnz = total;
    out.col = (int32_t *)dev_alloc((size_t)(total > 0 ? total : 1) * 4, s);
    out.val = dev_alloc((size_t)(total > 0 ? total : 1) * sizeof(T), s);
    if (!out.col || !out.val) return MO_E_ALLOC;
    if (a.fmt == MO_COO || a.fmt == MO_CSR) {
        // COO is sorted by (row, col): its column and value arrays already are the CSR ones
        const int32_t *src_col = a.fmt == MO_COO ? a.coo_col : a.csr_col;
        const void *src_val = a.fmt == MO_COO ? a.coo_val : a.csr_val;
        if (total > 0) {
            MO_HIP(hipMemcpyAsync(out.col, src_col, (size_t)total * 4, hipMemcpyDeviceToDevice, s));
            MO_HIP(hipMemcpyAsync(out.val, src_val, (size_t)total * sizeof(T), hipMemcpyDeviceToDevice, s));
        }
    } else {
        // rows per block: as many as keep the block's output within one LDS chunk at the mean row length
        int rpb = FB;
        while (rpb > 32 && (double)total / (double)a.m * rpb > 0.9 * FILL_CH) rpb >>= 1;
        const dim3 grid((unsigned)((a.m + rpb - 1) / rpb));
        if (v.nd > 0 && v.k == 0 && v.nnz_coo == 0)
            hipLaunchKernelGGL((k_fill_csr_any<T, 1>), grid, dim3(FB), 0, s, v, out.row_ptr, out.col, (T *)out.val, rpb);
        else if (v.k > 0 && v.nd == 0 && !v.csr_row_ptr)
            hipLaunchKernelGGL((k_fill_csr_any<T, 2>), grid, dim3(FB), 0, s, v, out.row_ptr, out.col, (T *)out.val, rpb);
        else
            hipLaunchKernelGGL((k_fill_csr_any<T, 0>), grid, dim3(FB), 0, s, v, out.row_ptr, out.col, (T *)out.val, rpb);
        MO_LAUNCH_CHECK();
    }
    MO_HIP(hipStreamSynchronize(s));   // scratch is released on return
    return MO_OK;
}

static mo_status switch_impl(const mo_matrix &a, mo_format fmt, const mo_params &p, mo_matrix **out, hipStream_t s)
{
    TempCsr t(s);
    MO_TRY(a.dtype == MO_F32 ? rebuild_csr<float>(a, t, s) : rebuild_csr<double>(a, t, s));
    mo_csr view{a.m, a.n, t.nnz, t.row_ptr, t.col, t.val, a.dtype};
    Scratch scr(s);
    Analysis an;
    MO_TRY(analyse(view, p, fmt == MO_DIA || fmt == MO_HDC, &an, scr, s));
    mo_matrix *h = nullptr;
    MO_TRY(convert_impl(view, fmt, p, an, &h, s));
    if (fmt == MO_CSR) {   // the CSR handle borrows these arrays: hand them over
        h->owned.push_back(t.row_ptr); h->owned.push_back(t.col); h->owned.push_back(t.val);
        t.release();
    }
    *out = h;
    return MO_OK;
}

template <typename T>
static mo_status features_any(const mo_matrix &a, const mo_params &p, Counters *h_out, unsigned long long *nnz_out, hipStream_t s)
{
    const View<T> v = make_view<T>(a);
    Scratch scr(s);
    const int64_t ndiag = a.m + a.n - 1;
    // one block of scratch: [counters, 256 bytes | entry total, 256 bytes | diagonal counters | row lengths]
    char *base = (char *)scr.get(512 + (size_t)ndiag * 4 + (size_t)a.m * 4);
    if (!base) return MO_E_ALLOC;
    Counters *ctr = (Counters *)base;
    unsigned long long *total = (unsigned long long *)(base + 256);
    uint32_t *hist = (uint32_t *)(base + 512);
    int32_t *len = (int32_t *)(base + 512 + (size_t)ndiag * 4);
    // the total and the histogram are contiguous: one launch zeroes both and resets the counters
    hipLaunchKernelGGL(k_zero_and_reset, dim3(grid_for(ndiag + 64, FB * 4, 4096)), dim3(FB), 0, s, (uint32_t *)total, ndiag + 64, ctr, (uint32_t *)nullptr, 0);
    MO_LAUNCH_CHECK();
    const unsigned rb = (unsigned)((a.m + FB - 1) / FB);
    hipLaunchKernelGGL(k_len_any<T>, dim3(rb), dim3(FB), 0, s, v, len);
    MO_LAUNCH_CHECK();
    hipLaunchKernelGGL(k_len_stats, dim3(grid_for(a.m, FB * 4, 512)), dim3(FB), 0, s, len, a.m, ctr, total);
    MO_LAUNCH_CHECK();
    if (v.nd > 0) {
        hipLaunchKernelGGL(k_hist_dia<T>, dim3((unsigned)v.nd, grid_for(a.m, FB * 8, 256)), dim3(FB), 0, s, v, hist);
        MO_LAUNCH_CHECK();
    }
    if (v.k > 0 || v.nnz_coo > 0 || v.csr_row_ptr) {
        constexpr int64_t BLOCKS = 2048;
        int64_t rpb = (a.m + BLOCKS - 1) / BLOCKS;
        rpb = ((rpb + FB - 1) / FB) * FB;
        const int64_t nblk = (a.m + rpb - 1) / rpb;
        const int64_t cpb = (v.nnz_coo + nblk - 1) / nblk;
        hipLaunchKernelGGL(k_hist_parts<T>, dim3((unsigned)nblk), dim3(FB), 0, s, v, rpb, cpb, hist);
        MO_LAUNCH_CHECK();
    }
    const int64_t mn = a.m < a.n ? a.m : a.n;
    hipLaunchKernelGGL(k_diag_count, dim3(grid_for(ndiag, FB * 4, 512)), dim3(FB), 0, s, hist, ndiag,
                       (unsigned long long)mn * (unsigned long long)p.td_num, (unsigned long long)p.td_den, ctr, (const uint32_t *)nullptr, (const uint32_t *)nullptr);
    MO_LAUNCH_CHECK();
    struct { Counters c; char pad[256 - sizeof(Counters)]; unsigned long long total; } host;   // mirrors the head of the block
    static_assert(sizeof(host) == 264, "counters in the first 256 bytes, the total right after");
    MO_HIP(hipMemcpyAsync(&host, base, sizeof(host), hipMemcpyDeviceToHost, s));
    MO_HIP(hipStreamSynchronize(s));
    *h_out = host.c;
    *nnz_out = host.total;
    return MO_OK;
}

}  // namespace mo

using namespace mo;

extern "C" {

mo_status mo_switch(const mo_matrix *a, mo_format fmt, const mo_params *params, mo_matrix **out, void *stream)
{
    if (!out) return MO_E_NULL;
    *out = nullptr;
    if (!a) return MO_E_NULL;
    if ((int)fmt < 0 || (int)fmt >= MO_NUM_FORMATS) return MO_E_FORMAT;
    mo_params p;
    MO_TRY(check_params(params, &p));
    const mo_status rc = no_throw([&] { return switch_impl(*a, fmt, p, out, (hipStream_t)stream); });
    if (rc != MO_OK) *out = nullptr;
    return rc;
}

mo_status mo_matrix_features(const mo_matrix *a, const mo_params *params, double out[MO_NUM_FEATURES], mo_feature_ints *ints_opt,
                             void *stream)
{
    if (!a || !out) return MO_E_NULL;
    if (a->fmt == MO_CSR) {   // the CSR kernels stage columns through LDS and are the faster walk of these arrays
        const mo_csr view{a->m, a->n, a->nnz_csr, a->csr_row_ptr, a->csr_col, a->csr_val, a->dtype};
        return mo_features(&view, params, out, ints_opt, stream);
    }
    mo_params p;
    MO_TRY(check_params(params, &p));
    Counters c;
    unsigned long long nnz = 0;
    MO_TRY(a->dtype == MO_F32 ? features_any<float>(*a, p, &c, &nnz, (hipStream_t)stream)
                              : features_any<double>(*a, p, &c, &nnz, (hipStream_t)stream));
    mo_feature_ints ints;
    ints.m = a->m; ints.n = a->n; ints.nnz = (int64_t)nnz;
    ints.max_row = (int64_t)c.max_row; ints.min_row = (int64_t)c.min_row;
    ints.n_diag = (int64_t)c.n_diag; ints.n_true_diag = (int64_t)c.n_true;
    ints.sum_sq_row = c.sum_sq;
    if (ints_opt) *ints_opt = ints;
    return mo_features_finalize(&ints, out);   // the same finalisation as mo_features (Table I)
}

}  // extern "C"

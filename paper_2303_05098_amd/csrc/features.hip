// Feature extraction kernels (Table I; Sections IV-A and VI-C) and CSR validation.
//
// Two traversals give every integer the ten features need: one over row_ptr (max, min, sum of squares of the row
// lengths, all in one pass as Section VI-C asks) and one over col_idx (entries per diagonal d = col - row).  Both
// also check the CSR precondition, and both clamp what they read so that a malformed matrix can never make a kernel
// index outside the arrays it was given.  All arithmetic is integer, so results do not depend on scheduling.
#include "dev_common.hpp"
#include "feat_common.hpp"
#include "mo_internal.hpp"

namespace mo {

// F1: one pass over row_ptr.
__global__ __launch_bounds__(FB) void k_row_stats(const int32_t *__restrict__ row_ptr, int64_t m, int64_t nnz, Counters *ctr)
{
    unsigned long long mx = 0ull, mn = ~0ull, sq = 0ull;
    bool err = false;
    const int64_t stride = (int64_t)gridDim.x * FB;
    for (int64_t i = (int64_t)blockIdx.x * FB + threadIdx.x; i < m; i += stride) {
        const int64_t a = row_ptr[i], b = row_ptr[i + 1];
        if (i == 0 && a != 0) err = true;
        if (i == m - 1 && b != nnz) err = true;
        if (b < a || a < 0 || b > nnz) err = true;
        const unsigned long long len = b > a ? (unsigned long long)(b - a) : 0ull;
        mx = len > mx ? len : mx;
        mn = len < mn ? len : mn;
        sq += len * len;
    }
    mx = wave_max(mx); mn = wave_min(mn); sq = wave_sum(sq);
    __shared__ unsigned long long s_mx[FB / WAVE], s_mn[FB / WAVE], s_sq[FB / WAVE];
    __shared__ int s_err;
    if (threadIdx.x == 0) s_err = 0;
    __syncthreads();
    if (err) s_err = 1;
    if (lane_id() == 0) { s_mx[threadIdx.x / WAVE] = mx; s_mn[threadIdx.x / WAVE] = mn; s_sq[threadIdx.x / WAVE] = sq; }
    __syncthreads();
    if (threadIdx.x == 0) {
        for (int w = 1; w < FB / WAVE; ++w) {
            mx = s_mx[w] > mx ? s_mx[w] : mx;
            mn = s_mn[w] < mn ? s_mn[w] : mn;
            sq += s_sq[w];
        }
        atomicMax(&ctr->max_row, mx);
        atomicMin(&ctr->min_row, mn);
        atomicAdd(&ctr->sum_sq, sq);
        if (s_err) atomicOr(&ctr->err, 1u);
    }
}

// F2: one pass over col_idx.  Lane l of a wave owns row r0 + l and walks its entries (rows of at most SHORT_ROW
// entries; the columns reach the lanes through LDS so that global loads stay coalesced), so for banded and stencil
// matrices all lanes meet the same diagonal in the same step.  Counts are merged twice before they reach
// memory: equal keys inside a wave by ballot (one update per distinct key, at most MERGE_ROUNDS rounds, then one
// update per lane), and across the whole block in a small LDS hash table that is flushed once at the end.  A block
// owns a contiguous run of rows, so a stencil's 27 diagonals cost 27 global atomics per block instead of one per
// wave and step (same-address atomics serialise in L2: that was 1.6 ms on the 128^3 stencil).  Keys that find no
// free slot within a few probes (matrices with many distinct diagonals) go straight to global memory.
// A row longer than SHORT_ROW is walked by the whole wave with coalesced loads; entries of one row lie on distinct
// diagonals, so they are counted directly.
template <bool DO_HIST>
__global__ __launch_bounds__(FB) void k_diag_hist(const int32_t *__restrict__ row_ptr, const int32_t *__restrict__ col_idx,
                                                   int64_t m, int64_t n, int64_t nnz, int64_t rows_per_block,
                                                   uint32_t *__restrict__ hist, Counters *ctr)
{
    __shared__ int ht_key[DO_HIST ? HT_SIZE : 1];
    __shared__ uint32_t ht_cnt[DO_HIST ? HT_SIZE : 1];
    __shared__ int ht_full;
    __shared__ int32_t s_col_all[(FB / WAVE) * FCAP];
    int32_t *s_col = s_col_all + (threadIdx.x / WAVE) * FCAP;
    if (threadIdx.x == 0) ht_full = 0;
    if (DO_HIST) {
        for (int i = threadIdx.x; i < HT_SIZE; i += FB) { ht_key[i] = -1; ht_cnt[i] = 0u; }
        __syncthreads();
    }
    const int lane = lane_id();
    bool err = false;
    const int64_t row_begin = (int64_t)blockIdx.x * rows_per_block;
    int64_t row_end = row_begin + rows_per_block;
    row_end = row_end < m ? row_end : m;
    for (int64_t base = row_begin; base < row_end; base += FB) {   // uniform trip count across the block
        const int64_t row = base + threadIdx.x;
        const bool rv = row < row_end;
        int64_t lo = 0, hi = 0;
        if (rv) {
            lo = row_ptr[row]; hi = row_ptr[row + 1];
            lo = lo < 0 ? 0 : (lo > nnz ? nnz : lo);
            hi = hi < lo ? lo : (hi > nnz ? nnz : hi);
        }
        const int64_t len = hi - lo;
        // The entries of the wave's 64 rows are one contiguous run: stream it through the wave's LDS region with
        // coalesced loads (FCAP entries at a time) and let every lane pick the entries of its own row out of LDS.
        const bool is_short = rv && len <= SHORT_ROW;
        const int64_t wb = wave_min(rv ? lo : (int64_t)0x7fffffffffffll);
        const int64_t we = wave_max(rv ? hi : (int64_t)0);
        int64_t prev = -1;
        for (int64_t c0 = wb; c0 < we; c0 += FCAP) {
            const int64_t c1 = c0 + FCAP < we ? c0 + FCAP : we;
            for (int i = lane; i < (int)(c1 - c0); i += WAVE) s_col[i] = ld_stream(col_idx + c0 + i);
            const int64_t ea = lo > c0 ? lo : c0, eb = hi < c1 ? hi : c1;
            const int cnt = (is_short && eb > ea) ? (int)(eb - ea) : 0;
            const int wmax = wave_max(cnt);
            for (int k = 0; k < wmax; ++k) {
                const bool act = k < cnt;
                const int64_t c = act ? (int64_t)s_col[ea + k - c0] : 0;
                const bool ok = act && c >= 0 && c < n && c > prev;
                if (act && !ok) err = true;
                if (act) prev = c;
                if (DO_HIST) {
                    const int key = ok ? (int)(c - row + (m - 1)) : -1;
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
                }
            }
        }
        uint64_t longmask = ballot64(rv && len > SHORT_ROW);
        while (longmask) {
            const int l = __ffsll((unsigned long long)longmask) - 1;
            longmask &= longmask - 1;
            const int64_t r = __shfl(row, l, WAVE);
            const int64_t rlo = __shfl(lo, l, WAVE);
            const int64_t rhi = __shfl(hi, l, WAVE);
            for (int64_t q = rlo + lane; q < rhi; q += WAVE) {
                const int64_t c = col_idx[q], cp = q > rlo ? (int64_t)col_idx[q - 1] : (int64_t)-1;
                const bool ok = c >= 0 && c < n && c > cp;
                if (!ok) err = true;
                else if (DO_HIST) atomicAdd(&hist[c - r + (m - 1)], 1u);
            }
        }
    }
    if (DO_HIST) {
        __syncthreads();
        for (int i = threadIdx.x; i < HT_SIZE; i += FB) {
            const uint32_t c = ht_cnt[i];
            if (c) atomicAdd(&hist[ht_key[i]], c);
        }
    }
    if (err) atomicOr(&ctr->err, 2u);
}

mo_status analyse(const mo_csr &a, const mo_params &p, bool want_hist, Analysis *out, Scratch &scratch, hipStream_t s)
{
    Counters *ctr = (Counters *)scratch.get(sizeof(Counters));
    if (!ctr) return MO_E_ALLOC;
    const int64_t ndiag = a.m + a.n - 1;
    uint32_t *hist = nullptr;
    if (want_hist) {
        hist = (uint32_t *)scratch.get((size_t)ndiag * sizeof(uint32_t));
        if (!hist) return MO_E_ALLOC;
    }
    hipLaunchKernelGGL(k_init_counters, dim3(1), dim3(64), 0, s, ctr);
    MO_LAUNCH_CHECK();
    if (want_hist) {
        hipLaunchKernelGGL(k_fill_u32, dim3(grid_for(ndiag, FB * 4, 4096)), dim3(FB), 0, s, hist, ndiag, 0u);
        MO_LAUNCH_CHECK();
    }
    hipLaunchKernelGGL(k_row_stats, dim3(grid_for(a.m, FB * 4, 512)), dim3(FB), 0, s, a.row_ptr, a.m, a.nnz, ctr);
    MO_LAUNCH_CHECK();
    // at most HIST_BLOCKS blocks, each owning a contiguous run of rows (a multiple of the block size)
    constexpr int64_t HIST_BLOCKS = 2048;
    int64_t rows_per_block = (a.m + HIST_BLOCKS - 1) / HIST_BLOCKS;
    rows_per_block = ((rows_per_block + FB - 1) / FB) * FB;
    const int64_t row_blocks = (a.m + rows_per_block - 1) / rows_per_block;
    if (want_hist)
        hipLaunchKernelGGL(k_diag_hist<true>, dim3((unsigned)row_blocks), dim3(FB), 0, s, a.row_ptr, a.col_idx, a.m, a.n, a.nnz,
                           rows_per_block, hist, ctr);
    else
        hipLaunchKernelGGL(k_diag_hist<false>, dim3((unsigned)row_blocks), dim3(FB), 0, s, a.row_ptr, a.col_idx, a.m, a.n, a.nnz,
                           rows_per_block, hist, ctr);
    MO_LAUNCH_CHECK();
    if (want_hist) {
        const int64_t mn = a.m < a.n ? a.m : a.n;
        hipLaunchKernelGGL(k_diag_count, dim3(grid_for(ndiag, FB * 4, 512)), dim3(FB), 0, s, hist, ndiag,
                           (unsigned long long)mn * (unsigned long long)p.td_num, (unsigned long long)p.td_den, ctr);
        MO_LAUNCH_CHECK();
    }
    Counters h;
    MO_HIP(hipMemcpyAsync(&h, ctr, sizeof(Counters), hipMemcpyDeviceToHost, s));
    MO_HIP(hipStreamSynchronize(s));
    if (h.err) return MO_E_CSR_INVALID;
    out->max_row = (int64_t)h.max_row;
    out->min_row = (int64_t)h.min_row;
    out->sum_sq = h.sum_sq;
    out->n_diag = (int64_t)h.n_diag;
    out->n_true = (int64_t)h.n_true;
    out->hist = hist;
    return MO_OK;
}

}  // namespace mo

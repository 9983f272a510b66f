// Feature extraction kernels (Table I; Sections IV-A and VI-C) and CSR validation.
//
// One traversal gives every integer the ten features need: max, min and sum of squares of the row lengths from
// row_ptr and the entries per diagonal d = col - row from col_idx (all statistics in one pass, as Section VI-C
// asks).  The same pass checks the CSR precondition and clamps what it reads, so that a malformed matrix can never
// make a kernel index outside the arrays it was given.  All arithmetic is integer: results do not depend on
// scheduling.
#include "dev_common.hpp"
#include "feat_common.hpp"
#include "mo_internal.hpp"

#include <mutex>

namespace mo {

// One traversal of the matrix gives every integer the features need ("multiple statistics at the same time",
// Section VI-C): row lengths (max, min, sum of squares) from row_ptr and entries per diagonal from col_idx.
//
// Lane l of a wave owns row r0 + l and walks its entries (rows of at most SHORT_ROW entries; the columns reach the
// lanes through LDS so that global loads stay coalesced), so for banded and stencil matrices all lanes meet the
// same diagonal in the same step.  Counts are merged three times before they reach memory:
//   1. registers: for step k of the walk, lanes k and k + 32 of two register pairs remember four diagonals and
//      their running counts (a four-way cache per step, private to the wave).  A banded matrix meets the same few
//      diagonals at the same step in every group of 64 rows, so the common case is four compares, ballots and
//      popcounts, no memory at all;
//   2. LDS: keys that miss the cache either replace its least used way (whose count moves to the block's hash
//      table) or, when they were met once only or the rows share no diagonals at all, go to the table directly;
//   3. the table is flushed to the global histogram once per block (same-address atomics serialise in L2: a
//      stencil's 27 diagonals cost 27 global atomics per block, not one per wave and step).
// Keys that find no free slot within a few probes (matrices with many distinct diagonals) go straight to memory.
// A row longer than SHORT_ROW is walked by the whole wave with coalesced loads; entries of one row lie on distinct
// diagonals, so they are counted directly.
static_assert(2 * SHORT_ROW <= WAVE, "the per-step cache lives in lanes k and k + SHORT_ROW");

constexpr int TB = 512;           // threads per block of the traversal: 8 waves share one hash table
constexpr int TCAP = 2 * FCAP;    // entries a wave stages at a time: 64 rows of SHORT_ROW entries, so that the rows of a
                                  // wave are walked in one go whenever they are all short
constexpr int TRAV_BLOCKS = 512;  // at most this many blocks: every block ends with one atomic per distinct
                                  // diagonal it met, and same-address atomics are served one after the other

// Row statistics of one block (no atomics: the host reduces the few hundred partial results).
struct RowPart {
    unsigned long long max_row, min_row, sum_sq, err;
};

template <bool DO_HIST>
__global__ __launch_bounds__(TB) void k_traverse(const int32_t *__restrict__ row_ptr, const int32_t *__restrict__ col_idx,
                                                  int64_t m, int64_t n, int64_t nnz, int64_t rows_per_block,
                                                  uint32_t *__restrict__ hist, RowPart *__restrict__ part, Counters *reset)
{
    if (reset && blockIdx.x == 0 && threadIdx.x == 0) {   // for the diagonal count that follows on the same stream
        reset->max_row = 0ull; reset->min_row = ~0ull; reset->sum_sq = 0ull; reset->n_diag = 0ull; reset->n_true = 0ull;
        reset->err = 0u; reset->pad = 0u;
    }
    __shared__ int ht_key[DO_HIST ? HT_SIZE : 1];
    __shared__ uint32_t ht_cnt[DO_HIST ? HT_SIZE : 1];
    __shared__ int ht_full;
    __shared__ int32_t s_col_all[(TB / WAVE) * TCAP];
    int32_t *s_col = s_col_all + (threadIdx.x / WAVE) * TCAP;
    if (threadIdx.x == 0) ht_full = 0;
    if (DO_HIST) {
        for (int i = threadIdx.x; i < HT_SIZE; i += TB) { ht_key[i] = -1; ht_cnt[i] = 0u; }
    }
    __syncthreads();
    const int lane = lane_id();
    bool err = false;
    uint64_t errm = 0ull;   // lanes of this wave that met a column out of range or out of order
    unsigned long long mx = 0ull, mn = ~0ull, sq = 0ull;
    // per-step cache of (diagonal, count): step k owns lanes k and k + SHORT_ROW of the pairs A and B (four ways)
    int ckeyA = -1, ckeyB = -1;
    int ccntA = 0, ccntB = 0;
    const int kbias = (int)(m - 1);
    const int64_t row_begin = (int64_t)blockIdx.x * rows_per_block;
    int64_t row_end = row_begin + rows_per_block;
    row_end = row_end < m ? row_end : m;
    for (int64_t base = row_begin; base < row_end; base += TB) {   // uniform trip count across the block
        const int64_t row = base + threadIdx.x;
        const bool rv = row < row_end;
        int lo = 0, hi = 0;   // nnz < 2^31: positions fit 32 bits
        if (rv) {
            const int64_t a = row_ptr[row], b = row_ptr[row + 1];
            if (row == 0 && a != 0) err = true;
            if (row == m - 1 && b != nnz) err = true;
            if (b < a || a < 0 || b > nnz) err = true;
            // clamped copies: a malformed row_ptr can never make this kernel index outside col_idx
            lo = (int)(a < 0 ? 0 : (a > nnz ? nnz : a));
            hi = (int)(b < lo ? lo : (b > nnz ? nnz : b));
            const unsigned long long l = b > a ? (unsigned long long)(b - a) : 0ull;
            mx = l > mx ? l : mx;
            mn = l < mn ? l : mn;
            sq += l * l;
        }
        const int len = hi - lo;
        // The entries of the wave's 64 rows are one contiguous run of col_idx.  It is streamed through the wave's LDS
        // region with coalesced loads, in chunks that hold whole rows (as many consecutive rows as fit TCAP entries),
        // and every lane picks the entries of its own row out of LDS.  Whole rows per chunk keep step k of the walk
        // at the k-th entry of every row, which is what makes the per-step cache below hit.  The conditions on lo
        // and hi keep every LDS index inside the chunk whatever row_ptr holds.
        const bool is_short = rv && len <= SHORT_ROW;
        const int nvalid = __popcll(ballot64(rv));
        const int krow = kbias - (int)row;   // key = col + krow
        int first = 0;
        while (first < nvalid) {
            const int start = __builtin_amdgcn_readlane(lo, first);
            const uint64_t fits = ballot64(rv && lo >= start && hi - start <= TCAP) >> first;
            const int nrun = ~fits ? __ffsll((unsigned long long)~fits) - 1 : WAVE;   // consecutive lanes from `first` that fit
            if (nrun <= 0) { ++first; continue; }   // this row alone exceeds the chunk: it is a long row, walked below
            const int last = first + nrun - 1;
            const int end = __builtin_amdgcn_readlane(hi, last);
            const int total = end - start;   // 0 .. TCAP
            if (total > 0) stage_to_lds(col_idx + start, s_col, total, lane);
            const bool mine_now = is_short && lane >= first && lane <= last && hi <= end;
            const int cnt = mine_now ? len : 0;   // <= SHORT_ROW
            const int32_t *mine = s_col + (mine_now ? lo - start : 0);
            int prev = -1;
            const int cm1 = cnt > 0 ? cnt - 1 : 0;
            // Lane masks are built from the compare instructions' own 64-bit results and combined with scalar
            // operations: every per-lane boolean that is turned into a mask costs two more vector instructions.
            for (int k = 0;; ++k) {
                const uint64_t actm = __builtin_amdgcn_sicmp(k, cnt, 40 /* signed < */);
                if (!actm) break;
                const int ks = __builtin_amdgcn_readfirstlane(k);
                const int c = mine[k < cm1 ? k : cm1];   // lanes past their row end re-read their last entry (unused)
                const uint64_t okm = actm & __builtin_amdgcn_uicmp((unsigned)c, (unsigned)n, 36 /* unsigned < */) &
                                     __builtin_amdgcn_sicmp(c, prev, 38 /* signed > */);
                errm |= actm & ~okm;
                prev = c;                                 // a lane past its row end never becomes active again in this chunk
                if (DO_HIST) {
                    const int key = c + krow;
                    // the four cached diagonals of step k: lanes k and k + SHORT_ROW of two register pairs; the
                    // second pair is only looked at when the first does not cover the step
                    const int k0 = __builtin_amdgcn_readlane(ckeyA, ks), k1 = __builtin_amdgcn_readlane(ckeyA, ks + SHORT_ROW);
                    const uint64_t h0 = okm & __builtin_amdgcn_sicmp(key, k0, 32 /* == */);
                    const uint64_t h1 = okm & __builtin_amdgcn_sicmp(key, k1, 32);
                    ccntA += lane == ks ? __popcll(h0) : (lane == ks + SHORT_ROW ? __popcll(h1) : 0);
                    uint64_t todo = okm & ~(h0 | h1);
                    if (todo) {
                        const int k2 = __builtin_amdgcn_readlane(ckeyB, ks), k3 = __builtin_amdgcn_readlane(ckeyB, ks + SHORT_ROW);
                        const uint64_t h2 = okm & __builtin_amdgcn_sicmp(key, k2, 32);
                        const uint64_t h3 = okm & __builtin_amdgcn_sicmp(key, k3, 32);
                        ccntB += lane == ks ? __popcll(h2) : (lane == ks + SHORT_ROW ? __popcll(h3) : 0);
                        todo &= ~(h2 | h3);
                    }
                    if (todo) {
                        // Keys the cache does not hold: each takes the place of the way with the smallest count when
                        // it was met at least twice in this step or a way is still empty (single meetings are mostly
                        // diagonals that do not repeat and must not push out ones that do).  Rows that share no
                        // diagonals leave this loop at its first round.
                        int rounds = 4;
                        while (todo && rounds-- > 0) {
                            const int leader = __ffsll((unsigned long long)todo) - 1;
                            const int lkey = __builtin_amdgcn_readlane(key, leader);
                            const uint64_t same = __builtin_amdgcn_sicmp(key, lkey, 32) & todo;   // todo holds valid lanes only
                            const int mult = __popcll(same);
                            const int n0 = __builtin_amdgcn_readlane(ccntA, ks), n1 = __builtin_amdgcn_readlane(ccntA, ks + SHORT_ROW);
                            const int n2 = __builtin_amdgcn_readlane(ccntB, ks), n3 = __builtin_amdgcn_readlane(ccntB, ks + SHORT_ROW);
                            int way = 0, nmin = n0;
                            if (n1 < nmin) { way = 1; nmin = n1; }
                            if (n2 < nmin) { way = 2; nmin = n2; }
                            if (n3 < nmin) { way = 3; nmin = n3; }
                            if (mult >= 2 || nmin == 0) {
                                const int wl = ks + (way & 1) * SHORT_ROW;
                                if (way < 2) {
                                    if (lane == wl) {
                                        if (ccntA) count_key(ckeyA, (uint32_t)ccntA, ht_key, ht_cnt, &ht_full, hist);
                                        ckeyA = lkey; ccntA = mult;
                                    }
                                } else {
                                    if (lane == wl) {
                                        if (ccntB) count_key(ckeyB, (uint32_t)ccntB, ht_key, ht_cnt, &ht_full, hist);
                                        ckeyB = lkey; ccntB = mult;
                                    }
                                }
                                todo &= ~same;
                            } else {
                                break;   // a single meeting and no empty way: it and the rest go to the table below
                            }
                        }
                        if ((todo >> lane) & 1ull) count_key(key, 1u, ht_key, ht_cnt, &ht_full, hist);
                    }
                }
            }
            first = last + 1;
        }
        uint64_t longmask = ballot64(rv && len > SHORT_ROW);
        while (longmask) {
            const int l = __ffsll((unsigned long long)longmask) - 1;
            longmask &= longmask - 1;
            const int64_t r = base + (threadIdx.x - lane) + l;
            const int rlo = __builtin_amdgcn_readlane(lo, l), rhi = __builtin_amdgcn_readlane(hi, l);
            for (int q = rlo + lane; q < rhi; q += WAVE) {
                const int64_t c = col_idx[q], cp = q > rlo ? (int64_t)col_idx[q - 1] : (int64_t)-1;
                const bool ok = c >= 0 && c < n && c > cp;
                if (!ok) err = true;
                else if (DO_HIST) atomicAdd(&hist[c - r + (m - 1)], 1u);
            }
        }
    }
    if (DO_HIST) {
        if (ccntA) count_key(ckeyA, (uint32_t)ccntA, ht_key, ht_cnt, &ht_full, hist);
        if (ccntB) count_key(ckeyB, (uint32_t)ccntB, ht_key, ht_cnt, &ht_full, hist);
        __syncthreads();
        for (int i = threadIdx.x; i < HT_SIZE; i += TB) {
            const uint32_t c = ht_cnt[i];
            if (c) atomicAdd(&hist[ht_key[i]], c);
        }
    }
    // row-length statistics and the error flag of this block
    if (errm) err = true;
    mx = wave_max(mx); mn = wave_min(mn); sq = wave_sum(sq);
    __shared__ unsigned long long s_mx[TB / WAVE], s_mn[TB / WAVE], s_sq[TB / WAVE];
    __shared__ int s_err;
    if (threadIdx.x == 0) s_err = 0;
    __syncthreads();
    if (err) s_err = 1;
    if (lane == 0) { s_mx[threadIdx.x / WAVE] = mx; s_mn[threadIdx.x / WAVE] = mn; s_sq[threadIdx.x / WAVE] = sq; }
    __syncthreads();
    if (threadIdx.x == 0) {
        for (int w = 1; w < TB / WAVE; ++w) {
            mx = s_mx[w] > mx ? s_mx[w] : mx;
            mn = s_mn[w] < mn ? s_mn[w] : mn;
            sq += s_sq[w];
        }
        part[blockIdx.x] = RowPart{mx, mn, sq, s_err ? 1ull : 0ull};
    }
}

mo_status analyse(const mo_csr &a, const mo_params &p, bool want_hist, Analysis *out, Scratch &scratch, hipStream_t s)
{
    // blocks own contiguous runs of rows (a multiple of the block size)
    int64_t rows_per_block = (a.m + TRAV_BLOCKS - 1) / TRAV_BLOCKS;
    rows_per_block = ((rows_per_block + TB - 1) / TB) * TB;
    const int64_t row_blocks = (a.m + rows_per_block - 1) / rows_per_block;   // 1 .. TRAV_BLOCKS
    // one allocation: [diagonal counters | row partials | histogram]
    const int64_t ndiag = a.m + a.n - 1;
    const size_t head = 256 + (size_t)TRAV_BLOCKS * sizeof(RowPart);
    static_assert(sizeof(Counters) <= 256, "the counters own the first 256 bytes");
    char *base = (char *)scratch.get(head + (want_hist ? (size_t)ndiag * sizeof(uint32_t) : 0));
    if (!base) return MO_E_ALLOC;
    Counters *ctr = (Counters *)base;
    RowPart *part = (RowPart *)(base + 256);
    uint32_t *hist = want_hist ? (uint32_t *)(base + head) : nullptr;
    if (want_hist) {
        hipLaunchKernelGGL(k_zero_and_reset, dim3(grid_for(ndiag, FB * 4, 4096)), dim3(FB), 0, s, hist, ndiag, ctr);
        MO_LAUNCH_CHECK();
        hipLaunchKernelGGL(k_traverse<true>, dim3((unsigned)row_blocks), dim3(TB), 0, s, a.row_ptr, a.col_idx, a.m, a.n, a.nnz,
                           rows_per_block, hist, part, (Counters *)nullptr);
        MO_LAUNCH_CHECK();
        const int64_t mn = a.m < a.n ? a.m : a.n;
        hipLaunchKernelGGL(k_diag_count, dim3(grid_for(ndiag, FB * 4, 512)), dim3(FB), 0, s, hist, ndiag,
                           (unsigned long long)mn * (unsigned long long)p.td_num, (unsigned long long)p.td_den, ctr);
        MO_LAUNCH_CHECK();
    } else {
        hipLaunchKernelGGL(k_traverse<false>, dim3((unsigned)row_blocks), dim3(TB), 0, s, a.row_ptr, a.col_idx, a.m, a.n, a.nnz,
                           rows_per_block, hist, part, (Counters *)nullptr);
        MO_LAUNCH_CHECK();
    }
    struct { Counters c; char pad[256 - sizeof(Counters)]; RowPart part[TRAV_BLOCKS]; } h;
    static_assert(sizeof(h) == 256 + TRAV_BLOCKS * sizeof(RowPart), "host mirror of the head of the scratch block");
    const size_t bytes = 256 + (size_t)row_blocks * sizeof(RowPart);
    MO_HIP(hipMemcpyAsync(&h, base, bytes, hipMemcpyDeviceToHost, s));
    MO_HIP(hipStreamSynchronize(s));
    unsigned long long mx = 0ull, mnr = ~0ull, sq = 0ull, err = 0ull;
    for (int64_t b = 0; b < row_blocks; ++b) {
        mx = h.part[b].max_row > mx ? h.part[b].max_row : mx;
        mnr = h.part[b].min_row < mnr ? h.part[b].min_row : mnr;
        sq += h.part[b].sum_sq;
        err |= h.part[b].err;
    }
    if (err) return MO_E_CSR_INVALID;
    out->max_row = (int64_t)mx;
    out->min_row = (int64_t)mnr;
    out->sum_sq = sq;
    out->n_diag = want_hist ? (int64_t)h.c.n_diag : 0;
    out->n_true = want_hist ? (int64_t)h.c.n_true : 0;
    out->hist = hist;
    return MO_OK;
}

// ------------------------------------------------------------------ the tuner's hot call
// mo_features is what a deployed tuner pays per matrix, and on small matrices its cost is launches and allocator
// calls, not kernels.  It therefore keeps one scratch block between calls (grown on demand, through the installed
// allocator) and a pinned host block for the results, under these rules:
//   * on entry the histogram part of the block is all zero: the counting kernel clears what it reads, so no fill
//     kernel runs after the first call;
//   * the traversal resets the diagonal counters itself;
//   * `clean` is dropped before the first launch and set again only after the final synchronisation, so an error on
//     the way makes the next call zero the block again;
//   * one call at a time owns the block (try-lock); a concurrent call, or a failed allocation, takes the ordinary
//     path with per-call scratch.
// mo_set_allocator releases the block through the allocator it came from.
namespace {

__global__ __launch_bounds__(FB) void k_diag_count_clear(uint32_t *__restrict__ hist, int64_t nd, unsigned long long thr_rhs,
                                                          unsigned long long td_den, Counters *ctr)
{
    unsigned long long c_nd = 0, c_td = 0;
    const int64_t stride = (int64_t)gridDim.x * FB;
    for (int64_t i = (int64_t)blockIdx.x * FB + threadIdx.x; i < nd; i += stride) {
        const unsigned long long c = hist[i];
        if (c >= 1ull) {
            hist[i] = 0u;
            ++c_nd;
            if (c * td_den >= thr_rhs) ++c_td;
        }
    }
    c_nd = wave_sum(c_nd); c_td = wave_sum(c_td);
    __shared__ unsigned long long s_nd[FB / WAVE], s_td[FB / WAVE];
    if (lane_id() == 0) { s_nd[threadIdx.x / WAVE] = c_nd; s_td[threadIdx.x / WAVE] = c_td; }
    __syncthreads();
    if (threadIdx.x == 0) {
        for (int w = 1; w < FB / WAVE; ++w) { c_nd += s_nd[w]; c_td += s_td[w]; }
        if (c_nd) atomicAdd(&ctr->n_diag, c_nd);
        if (c_td) atomicAdd(&ctr->n_true, c_td);
    }
}

constexpr size_t HEAD_BYTES = 256 + (size_t)TRAV_BLOCKS * sizeof(RowPart);

struct FeatureCache {
    std::mutex mu;
    char *dev = nullptr;     // [Counters in 256 bytes | RowPart x TRAV_BLOCKS | histogram of hist_cap counters]
    int64_t hist_cap = 0;
    bool clean = false;
    void *host = nullptr;    // pinned, HEAD_BYTES
    int device = -1;
};
FeatureCache g_fc;

}  // namespace

void release_feature_cache()
{
    std::lock_guard<std::mutex> lk(g_fc.mu);
    if (g_fc.dev) dev_free(g_fc.dev, nullptr);
    g_fc.dev = nullptr; g_fc.hist_cap = 0; g_fc.clean = false;
}

mo_status analyse_cached(const mo_csr &a, const mo_params &p, Analysis *out, hipStream_t s)
{
    std::unique_lock<std::mutex> lk(g_fc.mu, std::try_to_lock);
    int dev_now = -1;
    bool usable = lk.owns_lock() && hipGetDevice(&dev_now) == hipSuccess;
    if (usable && !g_fc.host && hipHostMalloc(&g_fc.host, HEAD_BYTES, hipHostMallocDefault) != hipSuccess) {
        g_fc.host = nullptr;
        usable = false;
    }
    const int64_t ndiag = a.m + a.n - 1;
    if (usable && (g_fc.hist_cap < ndiag || g_fc.device != dev_now)) {
        if (g_fc.dev) dev_free(g_fc.dev, s);
        g_fc.hist_cap = ndiag + ndiag / 2;
        g_fc.dev = (char *)dev_alloc(HEAD_BYTES + (size_t)g_fc.hist_cap * sizeof(uint32_t), s);
        g_fc.clean = false;
        g_fc.device = dev_now;
        if (!g_fc.dev) { g_fc.hist_cap = 0; usable = false; }
    }
    if (!usable) {
        if (lk.owns_lock()) lk.unlock();
        Scratch scr(s);
        MO_TRY(analyse(a, p, true, out, scr, s));
        out->hist = nullptr;   // gone with the scratch
        return MO_OK;
    }
    Counters *ctr = (Counters *)g_fc.dev;
    RowPart *part = (RowPart *)(g_fc.dev + 256);
    uint32_t *hist = (uint32_t *)(g_fc.dev + HEAD_BYTES);
    const bool was_clean = g_fc.clean;
    g_fc.clean = false;
    if (!was_clean) {
        hipLaunchKernelGGL(k_zero_and_reset, dim3(grid_for(g_fc.hist_cap, FB * 4, 4096)), dim3(FB), 0, s, hist, g_fc.hist_cap, ctr);
        MO_LAUNCH_CHECK();
    }
    int64_t rows_per_block = (a.m + TRAV_BLOCKS - 1) / TRAV_BLOCKS;
    rows_per_block = ((rows_per_block + TB - 1) / TB) * TB;
    const int64_t row_blocks = (a.m + rows_per_block - 1) / rows_per_block;
    hipLaunchKernelGGL(k_traverse<true>, dim3((unsigned)row_blocks), dim3(TB), 0, s, a.row_ptr, a.col_idx, a.m, a.n, a.nnz,
                       rows_per_block, hist, part, ctr);
    MO_LAUNCH_CHECK();
    const int64_t mn = a.m < a.n ? a.m : a.n;
    hipLaunchKernelGGL(k_diag_count_clear, dim3(grid_for(ndiag, FB * 4, 512)), dim3(FB), 0, s, hist, ndiag,
                       (unsigned long long)mn * (unsigned long long)p.td_num, (unsigned long long)p.td_den, ctr);
    MO_LAUNCH_CHECK();
    const size_t bytes = 256 + (size_t)row_blocks * sizeof(RowPart);
    MO_HIP(hipMemcpyAsync(g_fc.host, g_fc.dev, bytes, hipMemcpyDeviceToHost, s));
    MO_HIP(hipStreamSynchronize(s));
    g_fc.clean = true;
    const Counters *hc = (const Counters *)g_fc.host;
    const RowPart *hp = (const RowPart *)((const char *)g_fc.host + 256);
    unsigned long long mx = 0ull, mnr = ~0ull, sq = 0ull, err = 0ull;
    for (int64_t b = 0; b < row_blocks; ++b) {
        mx = hp[b].max_row > mx ? hp[b].max_row : mx;
        mnr = hp[b].min_row < mnr ? hp[b].min_row : mnr;
        sq += hp[b].sum_sq;
        err |= hp[b].err;
    }
    if (err) return MO_E_CSR_INVALID;
    out->max_row = (int64_t)mx;
    out->min_row = (int64_t)mnr;
    out->sum_sq = sq;
    out->n_diag = (int64_t)hc->n_diag;
    out->n_true = (int64_t)hc->n_true;
    out->hist = nullptr;
    return MO_OK;
}

}  // namespace mo

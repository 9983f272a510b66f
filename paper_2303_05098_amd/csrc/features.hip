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

#include <cstring>
#include <mutex>
#include <vector>

namespace mo {

// One traversal of the matrix gives every integer the features need ("multiple statistics at the same time",
// Section VI-C): row lengths (max, min, sum of squares) from row_ptr and entries per diagonal from col_idx.
//
// Lane l of a wave owns row r0 + l and walks its entries (rows of at most SHORT_ROW entries; the columns reach the
// lanes through LDS so that global loads stay coalesced).  Counts are merged three times before they reach memory:
//   1. registers: the wave keeps a list of candidate diagonals, ascending, one per lane, with a running count each
//      (taken from the longest row it has staged: in a banded or stencil matrix every other row holds a subset of
//      that row's diagonals).  Columns ascend inside a row, so every row is merged against the list: the loop runs
//      over the candidates, the same for all lanes; a lane whose current entry lies on the candidate is counted by
//      ballot and moves on to its next entry.  One compare, one ballot and one add count a diagonal for 64 rows,
//      whether or not the rows are aligned step by step (boundary rows of a stencil hold fewer entries);
//   2. LDS: entries the merge steps over (diagonals not in the list) go to the block's hash table one by one; when
//      they are more than a quarter of a chunk the list is written to the table and rebuilt from the next chunk,
//      and after two lists in a row that did not fit (rows that share no diagonals) the wave goes without one;
//   3. the table is flushed to the global histogram once per block (same-address atomics serialise in L2: a
//      stencil's 27 diagonals cost 27 global atomics per block, not one per wave and step).
// Keys that find no free slot within a few probes (matrices with many distinct diagonals) go straight to memory.
// A row longer than SHORT_ROW is walked by the whole wave with coalesced loads; entries of one row lie on distinct
// diagonals, so the lanes of one step never meet in a table slot.
static_assert(SHORT_ROW <= WAVE, "one candidate diagonal per lane");

constexpr int TB = 512;           // threads per block of the traversal: 8 waves share one hash table
constexpr int TCAP = 1920;        // entries a wave stages at a time: 64 rows of up to 30 entries are walked in one go.  Not
                                  // 2048 (64 rows of SHORT_ROW entries): with the hash table that made 82 120 bytes of LDS per
                                  // block, 200 bytes too many for two blocks per CU, and the kernel ran with 8 waves per CU
constexpr int HV_SIZE = 256;      // slots of the block's second, small table: diagonals that came out of a candidate list
constexpr int HV_PROBES = 4;
static_assert((TB / WAVE) * TCAP * 4 + HT_SIZE * 8 + HV_SIZE * 8 + 1024 <= 80 * 1024, "two traversal blocks must fit one CU's 160 KB of LDS");

// A diagonal that a candidate list has counted is a frequent one.  When its list is given up (rows that hold too many
// entries off the list) its entries come one by one, and they must not end as global atomics on one address (served
// one after the other: a 4 M-row band with 30 % scattered entries took 38 ms that way, the hash table being full of
// scattered diagonals by the time the lists failed).  Such diagonals therefore get a table of their own, which
// single entries look up first.
__device__ __forceinline__ bool heavy_insert_add(int key, uint32_t n, int *hv_key, uint32_t *hv_cnt)
{
    const uint32_t h = ((uint32_t)key * 2654435761u) >> 24;   // 8 bits
    for (int p = 0; p < HV_PROBES; ++p) {
        const int s = (int)((h + p) & (HV_SIZE - 1));
        const int old = atomicCAS(&hv_key[s], -1, key);
        if (old == -1 || old == key) { atomicAdd(&hv_cnt[s], n); return true; }
    }
    return false;
}
__device__ __forceinline__ bool heavy_find_add(int key, const int *hv_key, uint32_t *hv_cnt)
{
    const uint32_t h = ((uint32_t)key * 2654435761u) >> 24;
    for (int p = 0; p < HV_PROBES; ++p) {
        const int s = (int)((h + p) & (HV_SIZE - 1));
        const int k = hv_key[s];
        if (k == key) { atomicAdd(&hv_cnt[s], 1u); return true; }
        if (k == -1) return false;   // nothing is ever removed: the key is not there (or is being put there: counted elsewhere then)
    }
    return false;
}
constexpr int TSTAGE = 16;        // column loads a lane has in flight while a chunk is staged: two round trips to memory per
                                  // full chunk (8: four round trips, with the few waves this kernel runs each one shows)
constexpr size_t SAMPLE_WORDS = 1088;   // >= partition_sample_bytes() / 4, a multiple of 64: what follows starts on a 256-byte boundary
constexpr int TRAV_BLOCKS = 512;  // at most this many blocks: every block ends with one atomic per distinct
                                  // diagonal it met, and same-address atomics are served one after the other

// Row statistics of one block (no atomics: the host reduces the few hundred partial results).
struct RowPart {
    unsigned long long max_row, min_row, sum_sq, err;
};

template <bool DO_HIST>
__global__ __launch_bounds__(TB) void k_traverse(const int32_t *__restrict__ row_ptr, const int32_t *__restrict__ col_idx,
                                                  int64_t m, int64_t n, int64_t nnz, int64_t rows_per_block,
                                                  uint32_t *__restrict__ hist, RowPart *__restrict__ part,
                                                  const uint32_t *__restrict__ skip, LongRows *__restrict__ lr,
                                                  uint32_t *__restrict__ lr_flag)
{
    if (skip && *skip) return;   // a kernel ahead in the stream has decided that another path counts this matrix
    __shared__ int ht_key[DO_HIST ? HT_SIZE : 1];
    __shared__ uint32_t ht_cnt[DO_HIST ? HT_SIZE : 1];
    __shared__ int hv_key[DO_HIST ? HV_SIZE : 1];
    __shared__ uint32_t hv_cnt[DO_HIST ? HV_SIZE : 1];
    __shared__ int ht_full;
    __shared__ int32_t s_col_all[(TB / WAVE) * TCAP];
    int32_t *s_col = s_col_all + (threadIdx.x / WAVE) * TCAP;
    if (threadIdx.x == 0) ht_full = 0;
    if (DO_HIST) {
        for (int i = threadIdx.x; i < HT_SIZE; i += TB) { ht_key[i] = -1; ht_cnt[i] = 0u; }
        for (int i = threadIdx.x; i < HV_SIZE; i += TB) { hv_key[i] = -1; hv_cnt[i] = 0u; }
    }
    __syncthreads();
    const int lane = lane_id();
    bool err = false;
    uint64_t errm = 0ull;   // lanes of this wave that met a column out of range or out of order
    unsigned long long mx = 0ull, mn = ~0ull, sq = 0ull;
    // candidate diagonals of this wave: lane d holds the d-th key (ascending; NONE beyond ncand) and its count
    constexpr int NONE = 0x7fffffff;
    int cand = NONE, ccnt = 0;
    int ncand = 0, tmpl_fail = 0, chunks = 0;   // wave-uniform
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
        // A very long row is noted for k_long_rows and not walked here (its length has been counted above).
        bool deferred = false;
        if (lr && rv && len > VLONG_ROW) {
            const uint32_t slot = atomicAdd(&lr->count, 1u);
            if (slot < (uint32_t)LR_CAP) {
                lr->rows[slot] = (int32_t)row;
                if (lr_flag) *lr_flag = 1u;
                deferred = true;
            }
        }
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
            if (total > 0) stage_to_lds<int32_t, TSTAGE>(col_idx + start, s_col, total, lane);
            const bool mine_now = is_short && lane >= first && lane <= last && hi <= end;
            const int cnt = mine_now ? len : 0;   // <= SHORT_ROW
            const int32_t *mine = s_col + (mine_now ? lo - start : 0);
            int prev = -1;
            const int cm1 = cnt > 0 ? cnt - 1 : 0;
            if constexpr (!DO_HIST) {
                // validation only.  Lane masks are built from the compare instructions' own 64-bit results and
                // combined with scalar operations.
                for (int k = 0;; ++k) {
                    const uint64_t actm = __builtin_amdgcn_sicmp(k, cnt, 40 /* signed < */);
                    if (!actm) break;
                    const int c = mine[k < cm1 ? k : cm1];   // lanes past their row end re-read their last entry (unused)
                    const uint64_t okm = actm & __builtin_amdgcn_uicmp((unsigned)c, (unsigned)n, 36 /* unsigned < */) &
                                         __builtin_amdgcn_sicmp(c, prev, 38 /* signed > */);
                    errm |= actm & ~okm;
                    prev = c;                                 // a lane past its row end never becomes active again in this chunk
                }
            } else {
                if ((chunks++ & 31) == 0) tmpl_fail = 0;      // a wave that gave up on candidate lists tries again now and then
                if (ncand == 0 && tmpl_fail < 2) {
                    // the longest row of the chunk becomes the candidate list, if it is well-formed
                    const int best = __builtin_amdgcn_readfirstlane(wave_max(cnt));
                    if (best > 0) {
                        const int L = __ffsll((unsigned long long)ballot64(cnt == best)) - 1;
                        const int offL = __builtin_amdgcn_readlane((int)(mine - s_col), L);
                        const int krowL = __builtin_amdgcn_readlane(krow, L);
                        const int j = lane < best ? lane : best - 1;
                        const int cj = s_col[offL + j];
                        const int cp = s_col[offL + (j > 0 ? j - 1 : 0)];
                        const bool okj = (unsigned)cj < (unsigned)n && (j == 0 || cj > cp);
                        if (ballot64(!okj) == 0ull) {
                            cand = lane < best ? cj + krowL : NONE;
                            ccnt = 0;
                            ncand = best;
                        }
                    }
                }
                // The lane's current entry as a key (NONE when the row is used up or malformed), checked as it is
                // fetched: inside [0, n) and above its predecessor.
                int e = 0;
                int c = mine[0];
                bool ok = cnt > 0 && (unsigned)c < (unsigned)n;
                if (cnt > 0 && !ok) err = true;
                int cur = ok ? c + krow : NONE;
                prev = c;
                auto advance = [&]() {
                    ++e;
                    const int cn = mine[e < cm1 ? e : cm1];
                    const bool okn = e < cnt && (unsigned)cn < (unsigned)n && cn > prev;
                    if (e < cnt && !okn) err = true;
                    prev = cn;
                    cur = okn ? cn + krow : NONE;
                };
                int nhit = 0, nmiss = 0;
                const int nc = __builtin_amdgcn_readfirstlane(ncand);
                for (int d = 0; d < nc; ++d) {
                    const int target = __builtin_amdgcn_readlane(cand, d);
                    uint64_t below = __builtin_amdgcn_sicmp(cur, target, 40 /* signed < */);
                    while (below) {                            // entries on diagonals that are not in the list
                        nmiss += (int)__popcll(below);
                        if (cur < target) {
                            if (!heavy_find_add(cur, hv_key, hv_cnt)) count_key(cur, 1u, ht_key, ht_cnt, &ht_full, hist);
                            advance();
                        }
                        below = __builtin_amdgcn_sicmp(cur, target, 40);
                    }
                    const uint64_t hit = __builtin_amdgcn_sicmp(cur, target, 32 /* == */);
                    if (hit) {
                        const int nh = (int)__popcll(hit);
                        nhit += nh;
                        ccnt += lane == d ? nh : 0;
                        if (cur == target) advance();
                    }
                }
                uint64_t left = __builtin_amdgcn_sicmp(cur, NONE, 33 /* != */);
                while (left) {                                 // entries beyond the last candidate
                    nmiss += (int)__popcll(left);
                    if (cur != NONE) {
                        if (!heavy_find_add(cur, hv_key, hv_cnt)) count_key(cur, 1u, ht_key, ht_cnt, &ht_full, hist);
                        advance();
                    }
                    left = __builtin_amdgcn_sicmp(cur, NONE, 33);
                }
                if (nc > 0) {
                    if (nmiss * 4 > nhit + nmiss) {            // the list does not fit these rows: write it out, start over
                        if (lane < ncand && ccnt && !heavy_insert_add(cand, (uint32_t)ccnt, hv_key, hv_cnt)) count_key(cand, (uint32_t)ccnt, ht_key, ht_cnt, &ht_full, hist);
                        cand = NONE; ccnt = 0; ncand = 0;
                        ++tmpl_fail;
                    } else {
                        tmpl_fail = 0;
                    }
                }
            }
            first = last + 1;
        }
        uint64_t longmask = ballot64(rv && len > SHORT_ROW && !deferred);
        while (longmask) {
            const int l = __ffsll((unsigned long long)longmask) - 1;
            longmask &= longmask - 1;
            const int64_t r = base + (threadIdx.x - lane) + l;
            const int rlo = __builtin_amdgcn_readlane(lo, l), rhi = __builtin_amdgcn_readlane(hi, l);
            for (int q = rlo + lane; q < rhi; q += WAVE) {
                const int64_t c = col_idx[q], cp = q > rlo ? (int64_t)col_idx[q - 1] : (int64_t)-1;
                const bool ok = c >= 0 && c < n && c > cp;
                if (!ok) err = true;
                else if (DO_HIST) {
                    // through the block's tables like every other entry: the rows of a wide band hold the same diagonals,
                    // and one atomic per entry on a few hundred addresses took 50 - 100 CSR SpMVs
                    const int key = (int)(c - r + (m - 1));
                    if (!heavy_find_add(key, hv_key, hv_cnt)) count_key(key, 1u, ht_key, ht_cnt, &ht_full, hist);
                }
            }
        }
    }
    if (DO_HIST) {
        if (lane < ncand && ccnt && !heavy_insert_add(cand, (uint32_t)ccnt, hv_key, hv_cnt)) count_key(cand, (uint32_t)ccnt, ht_key, ht_cnt, &ht_full, hist);
        __syncthreads();
        for (int i = threadIdx.x; i < HT_SIZE; i += TB) {
            const uint32_t c = ht_cnt[i];
            if (c) atomicAdd(&hist[ht_key[i]], c);
        }
        for (int i = threadIdx.x; i < HV_SIZE; i += TB) {
            const uint32_t c = hv_cnt[i];
            if (c) atomicAdd(&hist[hv_key[i]], c);
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

// The rows the traversal noted in lr, entry-parallel over the whole grid: every block takes chunks of LB * LR_U entries
// of each row in turn, checks them (inside [0, n), above their predecessor) and, with DO_HIST, counts them straight
// into the histogram (the entries of one row lie on distinct diagonals: no two atomics of a chunk meet).  An error is
// left in part[0].err, where the host looks for the traversal's errors.  The block that finishes last clears the list
// (unless a conversion wants it: keep).
constexpr int LB = 256, LR_U = 4, LR_BLOCKS = 512;
template <bool DO_HIST>
__global__ __launch_bounds__(LB) void k_long_rows(const int32_t *__restrict__ row_ptr, const int32_t *__restrict__ col_idx, int64_t m,
                                                  int64_t n, int64_t nnz, uint32_t *__restrict__ hist, LongRows *__restrict__ lr,
                                                  RowPart *__restrict__ part, int keep)
{
    const uint32_t cnt_all = lr->count;
    const int cnt = (int)(cnt_all < (uint32_t)LR_CAP ? cnt_all : (uint32_t)LR_CAP);
    bool err = false;
    for (int li = 0; li < cnt; ++li) {
        int64_t row = lr->rows[li];
        row = row < 0 ? 0 : (row > m - 1 ? m - 1 : row);
        int64_t lo = row_ptr[row], hi = row_ptr[row + 1];
        lo = lo < 0 ? 0 : (lo > nnz ? nnz : lo);
        hi = hi < lo ? lo : (hi > nnz ? nnz : hi);
        for (int64_t q0 = lo + (int64_t)blockIdx.x * (LB * LR_U) + threadIdx.x; q0 - threadIdx.x < hi; q0 += (int64_t)gridDim.x * (LB * LR_U)) {
            int64_t c[LR_U], cp[LR_U];
#pragma unroll
            for (int u = 0; u < LR_U; ++u) {
                const int64_t q = q0 + u * LB, qc = q < hi ? q : hi - 1;   // hi > lo here
                c[u] = col_idx[qc];
                cp[u] = qc > lo ? (int64_t)col_idx[qc - 1] : (int64_t)-1;
            }
#pragma unroll
            for (int u = 0; u < LR_U; ++u) {
                if (q0 + u * LB >= hi) continue;
                const bool ok = c[u] >= 0 && c[u] < n && c[u] > cp[u];
                if (!ok) err = true;
                else if (DO_HIST) atomicAdd(&hist[c[u] - row + (m - 1)], 1u);
            }
        }
    }
    if (err) part[0].err = 1ull;   // every writer stores the same value
    __syncthreads();
    if (threadIdx.x == 0) {
        __threadfence();
        if (atomicAdd(&lr->done, 1u) == gridDim.x - 1) { if (!keep) lr->count = 0u; lr->done = 0u; }   // keep: the caller reads the list
    }
}

// The row half of the traversal alone: row lengths (max, min, sum of squares) and the row-pointer half of the CSR
// precondition (row_ptr[0] = 0, row_ptr[m] = nnz, non-decreasing, inside [0, nnz]), for the path that counts the
// diagonals by partition and checks the columns there.  Same block layout and results as k_traverse.
__global__ __launch_bounds__(TB) void k_row_stats(const int32_t *__restrict__ row_ptr, int64_t m, int64_t nnz, int64_t rows_per_block,
                                                   RowPart *__restrict__ part)
{
    unsigned long long mx = 0ull, mn = ~0ull, sq = 0ull;
    bool err = false;
    const int64_t row_begin = (int64_t)blockIdx.x * rows_per_block;
    int64_t row_end = row_begin + rows_per_block;
    row_end = row_end < m ? row_end : m;
    for (int64_t row = row_begin + threadIdx.x; row < row_end; row += TB) {
        const int64_t a = row_ptr[row], b = row_ptr[row + 1];
        if (row == 0 && a != 0) err = true;
        if (row == m - 1 && b != nnz) err = true;
        if (b < a || a < 0 || b > nnz) err = true;
        const unsigned long long l = b > a ? (unsigned long long)(b - a) : 0ull;
        mx = l > mx ? l : mx;
        mn = l < mn ? l : mn;
        sq += l * l;
    }
    mx = wave_max(mx); mn = wave_min(mn); sq = wave_sum(sq);
    __shared__ unsigned long long s_mx[TB / WAVE], s_mn[TB / WAVE], s_sq[TB / WAVE];
    __shared__ int s_err;
    if (threadIdx.x == 0) s_err = 0;
    __syncthreads();
    if (err) s_err = 1;
    if (lane_id() == 0) { s_mx[threadIdx.x / WAVE] = mx; s_mn[threadIdx.x / WAVE] = mn; s_sq[threadIdx.x / WAVE] = sq; }
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
    const int64_t ndiag = a.m + a.n - 1;
    // one allocation: [diagonal counters | row partials | words of the partition's sample | list of very long rows | histogram]
    static_assert(sizeof(LongRows) == 4096, "the list of very long rows owns 4096 bytes");
    static_assert(sizeof(Counters) <= 256, "the counters own the first 256 bytes");
    const size_t off_acc = 256 + (size_t)TRAV_BLOCKS * sizeof(RowPart);
    const size_t off_lr = off_acc + SAMPLE_WORDS * sizeof(uint32_t);
    const size_t head = off_lr + sizeof(LongRows);
    char *base = (char *)scratch.get(head + (want_hist ? (size_t)ndiag * sizeof(uint32_t) : 0));
    if (!base) return MO_E_ALLOC;
    Counters *ctr = (Counters *)base;
    RowPart *part = (RowPart *)(base + 256);
    uint32_t *acc = (uint32_t *)(base + off_acc);
    LongRows *lr = (LongRows *)(base + off_lr);
    uint32_t *hist = want_hist ? (uint32_t *)(base + head) : nullptr;
    // The usual case costs no more launches than it needs: the kernels are enqueued as if the matrix were structured and
    // held no very long rows; what a kernel ahead in the stream finds out (the partition's sample, the traversal's list)
    // makes the kernels behind it return at once, and the host, which reads those findings with the results, then sends
    // what is missing.
    const bool may_defer = a.nnz > VLONG_ROW;             // a row of more than VLONG_ROW entries can exist
    const bool sampled = want_hist && partition_possible(a);
    const int nzero = (int)SAMPLE_WORDS + 2;              // the sample's words and the head of the list (count, done)
    const int64_t mn = a.m < a.n ? a.m : a.n;
    const unsigned long long thr = (unsigned long long)mn * (unsigned long long)p.td_num;
    // two flags in the spare words of the counters' 256 bytes, so that they come back in the same copy
    uint32_t *long_flag = (uint32_t *)(base + 64), *part_flag_dev = (uint32_t *)(base + 68);
    if (want_hist) {
        hipLaunchKernelGGL(k_zero_and_reset, dim3(grid_for(ndiag, FB * 4, 4096)), dim3(FB), 0, s, hist, ndiag, ctr, acc, nzero);
        MO_LAUNCH_CHECK();
        if (sampled) MO_TRY(partition_decide_async(a, acc, part_flag_dev, s));
        hipLaunchKernelGGL(k_traverse<true>, dim3((unsigned)row_blocks), dim3(TB), 0, s, a.row_ptr, a.col_idx, a.m, a.n, a.nnz,
                           rows_per_block, hist, part, sampled ? acc + 3 : (const uint32_t *)nullptr, may_defer ? lr : (LongRows *)nullptr,
                           long_flag);
        MO_LAUNCH_CHECK();
        hipLaunchKernelGGL(k_diag_count, dim3(grid_for(ndiag, FB * 4, 512)), dim3(FB), 0, s, hist, ndiag, thr, (unsigned long long)p.td_den, ctr,
                           sampled ? acc + 3 : (const uint32_t *)nullptr, may_defer ? &lr->count : (const uint32_t *)nullptr);
        MO_LAUNCH_CHECK();
    } else {
        if (may_defer) {   // the counters' block (for its flags) and the head of the list
            hipLaunchKernelGGL(k_zero_and_reset, dim3(1), dim3(64), 0, s, (uint32_t *)nullptr, (int64_t)0, ctr, (uint32_t *)lr, 2);
            MO_LAUNCH_CHECK();
        }
        hipLaunchKernelGGL(k_traverse<false>, dim3((unsigned)row_blocks), dim3(TB), 0, s, a.row_ptr, a.col_idx, a.m, a.n, a.nnz,
                           rows_per_block, hist, part, (const uint32_t *)nullptr, may_defer ? lr : (LongRows *)nullptr, long_flag);
        MO_LAUNCH_CHECK();
    }
    struct { Counters c; char pad[256 - sizeof(Counters)]; RowPart part[TRAV_BLOCKS]; } h;
    static_assert(sizeof(h) == 256 + TRAV_BLOCKS * sizeof(RowPart), "host mirror of the head of the scratch block");
    const size_t bytes = 256 + (size_t)row_blocks * sizeof(RowPart);
    MO_HIP(hipMemcpyAsync(&h, base, bytes, hipMemcpyDeviceToHost, s));
    MO_HIP(hipStreamSynchronize(s));
    static_assert(sizeof(Counters) <= 64, "the flags live at bytes 64 and 68 of the counters' block");
    uint32_t flags[2];
    memcpy(flags, h.pad + (64 - sizeof(Counters)), sizeof(flags));
    const bool by_partition = sampled && flags[1] != 0u;
    uint32_t n_long = 0;
    if (may_defer && flags[0] != 0u) {   // rare: how many rows the list holds
        MO_HIP(hipMemcpyAsync(&n_long, &lr->count, sizeof(n_long), hipMemcpyDeviceToHost, s));
        MO_HIP(hipStreamSynchronize(s));
    }
    if (by_partition) {           // the traversal and the counting kernel returned at once; the list is empty
        void *pbuf = scratch.get(partition_scratch_bytes(a));
        if (!pbuf) return MO_E_ALLOC;
        hipLaunchKernelGGL(k_row_stats, dim3((unsigned)row_blocks), dim3(TB), 0, s, a.row_ptr, a.m, a.nnz, rows_per_block, part);
        MO_LAUNCH_CHECK();
        MO_TRY(partition_counts(a, p, pbuf, hist, nullptr, ctr, &ctr->err, s));
        n_long = 0;
    } else if (n_long > 0) {      // the traversal left rows to k_long_rows, and the counting kernel returned at once
        if (want_hist) {
            hipLaunchKernelGGL(k_long_rows<true>, dim3(LR_BLOCKS), dim3(LB), 0, s, a.row_ptr, a.col_idx, a.m, a.n, a.nnz, hist, lr, part, 1);
            MO_LAUNCH_CHECK();
            hipLaunchKernelGGL(k_diag_count, dim3(grid_for(ndiag, FB * 4, 512)), dim3(FB), 0, s, hist, ndiag, thr, (unsigned long long)p.td_den,
                               ctr, (const uint32_t *)nullptr, (const uint32_t *)nullptr);
            MO_LAUNCH_CHECK();
        } else {
            hipLaunchKernelGGL(k_long_rows<false>, dim3(LR_BLOCKS), dim3(LB), 0, s, a.row_ptr, a.col_idx, a.m, a.n, a.nnz, hist, lr, part, 1);
            MO_LAUNCH_CHECK();
        }
    }
    if (by_partition || n_long > 0) {
        MO_HIP(hipMemcpyAsync(&h, base, bytes, hipMemcpyDeviceToHost, s));
        MO_HIP(hipStreamSynchronize(s));
    }
    unsigned long long mx = 0ull, mnr = ~0ull, sq = 0ull, err = 0ull;
    for (int64_t b = 0; b < row_blocks; ++b) {
        mx = h.part[b].max_row > mx ? h.part[b].max_row : mx;
        mnr = h.part[b].min_row < mnr ? h.part[b].min_row : mnr;
        sq += h.part[b].sum_sq;
        err |= h.part[b].err;
    }
    if (by_partition) err |= h.c.err;   // the columns were checked by the partition's first pass
    if (err) return MO_E_CSR_INVALID;
    out->max_row = (int64_t)mx;
    out->min_row = (int64_t)mnr;
    out->sum_sq = sq;
    out->n_diag = want_hist ? (int64_t)h.c.n_diag : 0;
    out->n_true = want_hist ? (int64_t)h.c.n_true : 0;
    out->hist = hist;
    out->long_rows = n_long > 0 ? lr : nullptr;
    out->n_long = (n_long > 0 && n_long <= (uint32_t)LR_CAP) ? (int)n_long : 0;
    return MO_OK;
}

// ------------------------------------------------------------------ the tuner's hot call
// mo_features is what a deployed tuner pays per matrix, and on small matrices its cost is launches and allocator
// calls, not kernels.  It therefore keeps one scratch block between calls (grown on demand, through the installed
// allocator) and a pinned host block for the results, under these rules:
//   * on entry the histogram part of the block is all zero: the counting kernel clears what it reads, so no fill
//     kernel runs after the first call;
//   * both kernels leave their per-block results (row statistics, diagonal counts) directly in the pinned host block,
//     which the host adds up after the synchronisation: no counters to reset and no copy command after the kernels;
//   * `clean` is dropped before the first launch and set again only after the final synchronisation, so an error on
//     the way makes the next call zero the block again;
//   * one call at a time owns the block (try-lock); a concurrent call, or a failed allocation, takes the ordinary
//     path with per-call scratch.
// mo_set_allocator releases the block through the allocator it came from.
namespace {

constexpr int DIAG_BLOCKS = 2048;

// Counts the non-empty and the true diagonals and clears the counters it reads; every block leaves its two counts in
// dpart[blockIdx.x] (no atomics: the host adds the few hundred partial results).
__global__ __launch_bounds__(FB) void k_diag_count_clear(uint32_t *__restrict__ hist, int64_t nd, unsigned long long thr_rhs,
                                                          unsigned long long td_den, DiagPart *__restrict__ dpart,
                                                          const uint32_t *__restrict__ skip, const uint32_t *__restrict__ skip2)
{
    if ((skip && *skip) || (skip2 && *skip2)) return;
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
        dpart[blockIdx.x] = DiagPart{c_nd, c_td};
    }
}

// results of one call, written by the kernels straight into pinned host memory (no copy command after them)
constexpr size_t HOST_BYTES = (size_t)TRAV_BLOCKS * sizeof(RowPart) + (size_t)DIAG_BLOCKS * sizeof(DiagPart);

struct FeatureCache {
    std::mutex mu;
    uint32_t *dev = nullptr;   // histogram of hist_cap counters
    int64_t hist_cap = 0;
    bool clean = false;
    void *host = nullptr;      // pinned: [RowPart x TRAV_BLOCKS | DiagPart x DIAG_BLOCKS | sample counts of the partition's decision]
    int device = -1;
    void *pbuf = nullptr;      // scratch of the partition path (feat_part.hip)
    size_t pbuf_cap = 0;
};
FeatureCache g_fc;

}  // namespace

void release_feature_cache()
{
    std::lock_guard<std::mutex> lk(g_fc.mu);
    if (g_fc.dev) dev_free(g_fc.dev, nullptr);
    if (g_fc.pbuf) dev_free(g_fc.pbuf, nullptr);
    g_fc.dev = nullptr; g_fc.hist_cap = 0; g_fc.clean = false;
    g_fc.pbuf = nullptr; g_fc.pbuf_cap = 0;
}

mo_status analyse_cached(const mo_csr &a, const mo_params &p, Analysis *out, hipStream_t s)
{
    std::unique_lock<std::mutex> lk(g_fc.mu, std::try_to_lock);
    int dev_now = -1;
    bool usable = lk.owns_lock() && hipGetDevice(&dev_now) == hipSuccess;
    if (usable && !g_fc.host && hipHostMalloc(&g_fc.host, HOST_BYTES + partition_sample_bytes() + 256, hipHostMallocDefault) != hipSuccess) {
        g_fc.host = nullptr;
        usable = false;
    }
    const int64_t ndiag = a.m + a.n - 1;
    if (usable && (g_fc.hist_cap < ndiag || g_fc.device != dev_now)) {
        if (g_fc.dev) dev_free(g_fc.dev, s);
        if (g_fc.pbuf && g_fc.device != dev_now) { dev_free(g_fc.pbuf, s); g_fc.pbuf = nullptr; g_fc.pbuf_cap = 0; }
        g_fc.hist_cap = ndiag + ndiag / 2;
        // + the sample's words + the list of very long rows
        const size_t TAIL = SAMPLE_WORDS + sizeof(LongRows) / sizeof(uint32_t);
        g_fc.hist_cap = (g_fc.hist_cap + 63) / 64 * 64;   // the list starts on a 256-byte boundary
        g_fc.dev = (uint32_t *)dev_alloc(((size_t)g_fc.hist_cap + TAIL) * sizeof(uint32_t), s);
        if (g_fc.dev) {
            hipLaunchKernelGGL(k_fill_u32, dim3(4), dim3(256), 0, s, g_fc.dev + g_fc.hist_cap, (int64_t)TAIL, 0u);
            MO_LAUNCH_CHECK();
        }
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
    RowPart *part = (RowPart *)g_fc.host;
    DiagPart *dpart = (DiagPart *)((char *)g_fc.host + (size_t)TRAV_BLOCKS * sizeof(RowPart));
    uint32_t *hist = g_fc.dev;
    int64_t rows_per_block = (a.m + TRAV_BLOCKS - 1) / TRAV_BLOCKS;
    rows_per_block = ((rows_per_block + TB - 1) / TB) * TB;
    const int64_t row_blocks = (a.m + rows_per_block - 1) / rows_per_block;
    // Scattered columns (decided from a sample): the diagonals are counted by partition, in scratch that is kept
    // like the histogram; the histogram itself is not touched and stays as clean as it was.
    // Matrices that could take the partition path (feat_part.hip) are sampled first, on the device; the traversal
    // kernels behind the sample skip themselves when it decides for the partition, and the host learns the decision
    // with the results, after the one synchronisation every call has.  A structured matrix pays one small kernel; a
    // scattered one pays two empty kernels and a second synchronisation on a call that is several times cheaper.
    const bool sampled = partition_possible(a);
    uint32_t *acc = g_fc.dev + g_fc.hist_cap, *flag_dev = acc + 3;   // the sample's words: counts, decision, bucket counts
    uint32_t *flag_host = (uint32_t *)((char *)g_fc.host + HOST_BYTES);
    uint32_t *col_err = flag_host + 1;
    *flag_host = 0u;   // pinned memory, written before the launches that may set it
    *col_err = 0u;
    if (sampled) MO_TRY(partition_decide_async(a, acc, flag_host, s));
    const bool was_clean = g_fc.clean;
    g_fc.clean = false;
    if (!was_clean) {
        hipLaunchKernelGGL(k_fill_u32, dim3(grid_for(g_fc.hist_cap, FB * 4, 4096)), dim3(FB), 0, s, hist, g_fc.hist_cap, 0u);
        MO_LAUNCH_CHECK();
    }
    // Rows of more than VLONG_ROW entries are noted by the traversal, not walked; the counting kernel then skips itself,
    // and the host, which learns of them with the results, sends k_long_rows and the counting kernel after them.
    LongRows *lr = a.nnz > VLONG_ROW ? (LongRows *)(g_fc.dev + g_fc.hist_cap + SAMPLE_WORDS) : (LongRows *)nullptr;
    uint32_t *long_host = flag_host + 2;
    *long_host = 0u;
    hipLaunchKernelGGL(k_traverse<true>, dim3((unsigned)row_blocks), dim3(TB), 0, s, a.row_ptr, a.col_idx, a.m, a.n, a.nnz,
                       rows_per_block, hist, part, sampled ? flag_dev : (const uint32_t *)nullptr, lr, long_host);
    MO_LAUNCH_CHECK();
    const int64_t mn = a.m < a.n ? a.m : a.n;
    int dblocks = grid_for(ndiag, FB * 16, DIAG_BLOCKS);
    hipLaunchKernelGGL(k_diag_count_clear, dim3(dblocks), dim3(FB), 0, s, hist, ndiag,
                       (unsigned long long)mn * (unsigned long long)p.td_num, (unsigned long long)p.td_den, dpart,
                       sampled ? flag_dev : (const uint32_t *)nullptr, lr ? &lr->count : (const uint32_t *)nullptr);
    MO_LAUNCH_CHECK();
    MO_HIP(hipStreamSynchronize(s));   // the kernels' stores to the pinned block are visible after this
    if (lr && *long_host != 0u) {
        hipLaunchKernelGGL(k_long_rows<true>, dim3(LR_BLOCKS), dim3(LB), 0, s, a.row_ptr, a.col_idx, a.m, a.n, a.nnz, hist, lr, part, 0);
        MO_LAUNCH_CHECK();
        hipLaunchKernelGGL(k_diag_count_clear, dim3(dblocks), dim3(FB), 0, s, hist, ndiag,
                           (unsigned long long)mn * (unsigned long long)p.td_num, (unsigned long long)p.td_den, dpart,
                           (const uint32_t *)nullptr, (const uint32_t *)nullptr);
        MO_LAUNCH_CHECK();
        MO_HIP(hipStreamSynchronize(s));
    }
    g_fc.clean = true;                 // skipped or not, the kernels leave the histogram all zero
    const bool by_partition = sampled && *flag_host != 0u;
    if (by_partition) {
        const size_t need = partition_scratch_bytes(a);
        if (g_fc.pbuf_cap < need) {
            if (g_fc.pbuf) dev_free(g_fc.pbuf, s);
            g_fc.pbuf = dev_alloc(need + need / 4, s);
            g_fc.pbuf_cap = g_fc.pbuf ? need + need / 4 : 0;
        }
        if (!g_fc.pbuf) return MO_E_ALLOC;
        hipLaunchKernelGGL(k_row_stats, dim3((unsigned)row_blocks), dim3(TB), 0, s, a.row_ptr, a.m, a.nnz, rows_per_block, part);
        MO_LAUNCH_CHECK();
        MO_TRY(partition_counts(a, p, g_fc.pbuf, nullptr, dpart, nullptr, col_err, s));
        dblocks = partition_buckets(a);
        MO_HIP(hipStreamSynchronize(s));
    }
    const RowPart *hp = part;
    unsigned long long mx = 0ull, mnr = ~0ull, sq = 0ull, err = 0ull;
    for (int64_t b = 0; b < row_blocks; ++b) {
        mx = hp[b].max_row > mx ? hp[b].max_row : mx;
        mnr = hp[b].min_row < mnr ? hp[b].min_row : mnr;
        sq += hp[b].sum_sq;
        err |= hp[b].err;
    }
    if (by_partition) err |= *col_err;
    unsigned long long n_diag = 0ull, n_true = 0ull;
    for (int b = 0; b < dblocks; ++b) { n_diag += dpart[b].n_diag; n_true += dpart[b].n_true; }
    if (err) return MO_E_CSR_INVALID;
    out->max_row = (int64_t)mx;
    out->min_row = (int64_t)mnr;
    out->sum_sq = sq;
    out->n_diag = (int64_t)n_diag;
    out->n_true = (int64_t)n_true;
    out->hist = nullptr;
    return MO_OK;
}

// ------------------------------------------------------------------ the call that allocates nothing
// For callers that cannot allocate (stream capture, tight serving loops): the same two kernels as above, with the
// diagonal histogram and the per-block partial results in a file-scope device array instead of allocator memory, and
// a last one-block kernel that adds the partial results up on the device and writes the integers where the caller
// wants them.  Every GPU holds its own copy of the array at its own address; the address is looked up once per device.
namespace {

constexpr int64_t STATIC_MAX_DIAGS = (int64_t)MO_STATIC_MAX_DIAGS;
struct StaticScratch {
    LongRows lr;               // zero when the module is loaded, cleared again by the kernel that reads it
    uint32_t hist[STATIC_MAX_DIAGS];
    RowPart part[TRAV_BLOCKS];
    DiagPart dpart[DIAG_BLOCKS];
};
static __device__ __align__(256) unsigned char scratch[sizeof(StaticScratch)];

constexpr int MAX_DEVICES = 64;
std::mutex g_static_mu;
StaticScratch *g_static_ptr[MAX_DEVICES] = {};

// One block: adds up the partial results of the two kernels before it, in index order.
__global__ __launch_bounds__(FB) void k_static_finish(const RowPart *__restrict__ part, int row_blocks, const DiagPart *__restrict__ dpart,
                                                       int dblocks, int64_t m, int64_t n, int64_t nnz, mo_feature_result *__restrict__ out)
{
    unsigned long long mx = 0ull, mn = ~0ull, sq = 0ull, err = 0ull, nd = 0ull, nt = 0ull;
    for (int b = threadIdx.x; b < row_blocks; b += FB) {
        const RowPart p = part[b];
        mx = p.max_row > mx ? p.max_row : mx;
        mn = p.min_row < mn ? p.min_row : mn;
        sq += p.sum_sq;
        err |= p.err;
    }
    for (int b = threadIdx.x; b < dblocks; b += FB) { nd += dpart[b].n_diag; nt += dpart[b].n_true; }
    mx = wave_max(mx); mn = wave_min(mn); sq = wave_sum(sq); err = wave_max(err); nd = wave_sum(nd); nt = wave_sum(nt);
    __shared__ unsigned long long s[6][FB / WAVE];
    const int w = threadIdx.x / WAVE;
    if (lane_id() == 0) { s[0][w] = mx; s[1][w] = mn; s[2][w] = sq; s[3][w] = err; s[4][w] = nd; s[5][w] = nt; }
    __syncthreads();
    if (threadIdx.x == 0) {
        for (int q = 1; q < FB / WAVE; ++q) {
            mx = s[0][q] > mx ? s[0][q] : mx;
            mn = s[1][q] < mn ? s[1][q] : mn;
            sq += s[2][q]; err |= s[3][q]; nd += s[4][q]; nt += s[5][q];
        }
        out->ints.m = m; out->ints.n = n; out->ints.nnz = nnz;
        out->ints.max_row = (int64_t)mx; out->ints.min_row = (int64_t)mn;
        out->ints.n_diag = (int64_t)nd; out->ints.n_true_diag = (int64_t)nt;
        out->ints.sum_sq_row = sq;
        out->status = err ? (int32_t)MO_E_CSR_INVALID : (int32_t)MO_OK;
        out->pad = 0;
    }
}

}  // namespace

mo_status features_static(const mo_csr &a, const mo_params &p, mo_feature_result *out_dev, hipStream_t s)
{
    const int64_t ndiag = a.m + a.n - 1;
    if (ndiag > STATIC_MAX_DIAGS) return MO_E_SHAPE;
    int dev = -1;
    MO_HIP(hipGetDevice(&dev));
    if (dev < 0 || dev >= MAX_DEVICES) return MO_E_DEVICE;
    StaticScratch *sc = nullptr;
    {
        std::lock_guard<std::mutex> lk(g_static_mu);
        if (!g_static_ptr[dev]) {
            void *ptr = nullptr;
            MO_HIP(hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)));
            g_static_ptr[dev] = (StaticScratch *)ptr;
        }
        sc = g_static_ptr[dev];
    }
    if (!sc) return MO_E_DEVICE;
    // the array keeps whatever the last call left (possibly one that was cut short): the counters start from zero
    hipLaunchKernelGGL(k_fill_u32, dim3(grid_for(ndiag, FB * 4, 4096)), dim3(FB), 0, s, sc->hist, ndiag, 0u);
    MO_LAUNCH_CHECK();
    int64_t rows_per_block = (a.m + TRAV_BLOCKS - 1) / TRAV_BLOCKS;
    rows_per_block = ((rows_per_block + TB - 1) / TB) * TB;
    const int64_t row_blocks = (a.m + rows_per_block - 1) / rows_per_block;
    hipLaunchKernelGGL(k_traverse<true>, dim3((unsigned)row_blocks), dim3(TB), 0, s, a.row_ptr, a.col_idx, a.m, a.n, a.nnz,
                       rows_per_block, sc->hist, sc->part, (const uint32_t *)nullptr, a.nnz > VLONG_ROW ? &sc->lr : (LongRows *)nullptr,
                       (uint32_t *)nullptr);
    MO_LAUNCH_CHECK();
    if (a.nnz > VLONG_ROW) {   // no host in between here: the kernel for very long rows always runs (usually over an empty list)
        hipLaunchKernelGGL(k_long_rows<true>, dim3(LR_BLOCKS), dim3(LB), 0, s, a.row_ptr, a.col_idx, a.m, a.n, a.nnz, sc->hist, &sc->lr,
                           sc->part, 0);
        MO_LAUNCH_CHECK();
    }
    const int64_t mn = a.m < a.n ? a.m : a.n;
    const int dblocks = grid_for(ndiag, FB * 16, DIAG_BLOCKS);
    hipLaunchKernelGGL(k_diag_count_clear, dim3(dblocks), dim3(FB), 0, s, sc->hist, ndiag,
                       (unsigned long long)mn * (unsigned long long)p.td_num, (unsigned long long)p.td_den, sc->dpart, (const uint32_t *)nullptr,
                       (const uint32_t *)nullptr);
    MO_LAUNCH_CHECK();
    hipLaunchKernelGGL(k_static_finish, dim3(1), dim3(FB), 0, s, sc->part, (int)row_blocks, sc->dpart, dblocks, a.m, a.n, a.nnz, out_dev);
    MO_LAUNCH_CHECK();
    return MO_OK;
}

}  // namespace mo

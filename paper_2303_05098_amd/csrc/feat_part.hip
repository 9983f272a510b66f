// Entries per diagonal (the histogram behind N_D and N_TD of Table I; Sections IV-A and VI-C) for matrices whose
// entries share no diagonals from one row to the next: by partition instead of by atomics.
//
// The traversal kernel of features.hip merges counts in registers and LDS before they reach memory, which is what a
// banded or stencil matrix needs.  A matrix with scattered columns gives it nothing to merge: every entry becomes one
// global atomic on its own address, and the chip serves about 27 G of those per second (17 M entries: 0.63 ms).
// Here the diagonal numbers d = col - row + (m - 1) are instead cut into buckets of PB_KEYS consecutive diagonals:
//   1. k_part_count: every block counts the entries of its share of the matrix per bucket (LDS);
//   2. an exclusive scan over the counts, bucket-major, gives every (bucket, block) the place of its entries;
//   3. k_part_scatter: the same blocks sort their entries by bucket in LDS, tile by tile, and append each bucket's run
//      of 16-bit diagonal numbers (relative to the bucket) to the bucket's part of one array;
//   4. k_part_hist: one block per bucket counts its bucket's entries per diagonal in an LDS table, counts the
//      non-empty and the true diagonals, and (when a conversion needs it) writes its stretch of the histogram.
// Everything is streamed: 4 bytes read twice, 2 bytes written and read once per entry, no global atomics.
// The kernels clamp what they read (rows by search in row_ptr, diagonal numbers into [0, m + n - 1)), so that arrays
// that violate the CSR precondition, which the validation kernel reports in the same call, cannot make them index
// outside their buffers; the counts are then meaningless and the call returns the error.  The first pass also checks
// the columns (inside [0, n), ascending inside a row), so that the traversal kernel is not needed at all on this path:
// the row pointers and the row statistics take a kernel that reads row_ptr only (k_row_stats in features.hip).
//
// Which matrices take this path is decided from a sample (partition_wanted): groups of adjacent rows whose sampled
// entries repeat no diagonal within the group.
#include "dev_common.hpp"
#include "feat_common.hpp"
#include "mo_internal.hpp"


namespace mo {

namespace {

constexpr int PB_BITS = 13;
constexpr int PB_KEYS = 1 << PB_BITS;     // diagonals per bucket: a table of 32 KB in LDS
constexpr int PB_MAX = 1024;              // buckets at most (m + n - 1 <= 8 388 608)
constexpr int PT = 512;                   // threads per block of the count and scatter kernels
constexpr int PE = 8;                     // consecutive entries per thread and tile
constexpr int PH = 1024;                  // threads per block of the histogram kernel (one block per bucket)
constexpr int PSUB = PT * PE;             // entries per tile
constexpr int P_MAX_BLOCKS = 1024;        // blocks of the count and scatter kernels at most
constexpr int P_MAX_TILES = 512;          // tiles per block at most: 2^31 entries / P_MAX_BLOCKS / PSUB
constexpr int64_t PART_MIN_NNZ = (int64_t)1 << 21;   // below: the traversal kernel (the extra launches would cost more)

constexpr int SG = 128, SR = 8, SE = 32;  // sample: SG groups of SR adjacent rows, SE entries of each row

// The diagonal numbers of a tile's entries, PE consecutive entries per thread.  The rows that intersect the tile are
// found by two searches in row_ptr; their slice of row_ptr is staged in LDS when it is short enough (a tile that
// spans many empty rows searches row_ptr itself).  key[k] = -1 past the end of the tile.
typedef int int4u __attribute__((ext_vector_type(4), aligned(4)));

struct TileRows {
    int64_t r0;
    int nr;
    bool staged;
};

// The first and the last row of every tile of a block's share: 2 * tiles searches for the largest row r with
// row_ptr[r] <= p.  A binary search is some twenty dependent loads, which cost more than the tile's own work, so the
// block searches with all its threads instead, in three steps of independent loads: PT rows spread over the whole
// matrix, then 32 rows inside the interval each search fell into, then 64 inside the next, and a few binary steps on
// what is left (none for matrices of up to a million rows).  scr: PSUB ints of LDS (the tile stage, not in use yet);
// shares of more than 32 tiles (more than 2^27 entries in the matrix) search one boundary per thread the plain way.
// tile_rows (global, or nullptr): the block's results are also written there (2 ints per tile, at tile_base) for
// the scatter pass, which walks the same tiles.  Indices stay inside [0, m) whatever row_ptr holds.
constexpr int FT_MAX = 32;   // tiles per block up to which the cooperative search is used
__device__ __forceinline__ int last_not_above(const int32_t *v, int cnt, int64_t p)
{
    int lo = 0, hi = cnt - 1;   // largest j with v[j] <= p, 0 when there is none
    while (lo < hi) {
        const int mid = (lo + hi + 1) >> 1;
        if ((int64_t)v[mid] <= p) lo = mid; else hi = mid - 1;
    }
    return lo;
}

__device__ __forceinline__ void find_tile_rows(const int32_t *__restrict__ row_ptr, int64_t m, int64_t b0, int64_t b1, int32_t *s_first,
                                               int32_t *s_last, int32_t *scr, int32_t *__restrict__ tile_rows, int64_t tile_base)
{
    const int nt = (int)((b1 - b0 + PSUB - 1) / PSUB);
    auto target = [&](int q) {
        const int64_t t0 = b0 + (int64_t)(q >> 1) * PSUB, t1 = t0 + PSUB < b1 ? t0 + PSUB : b1;
        return (q & 1) ? t1 - 1 : t0;
    };
    auto publish = [&](int q, int64_t r) {
        if (q & 1) s_last[q >> 1] = (int32_t)r; else s_first[q >> 1] = (int32_t)r;
        if (tile_rows) tile_rows[2 * tile_base + q] = (int32_t)r;
    };
    if (nt > FT_MAX) {
        for (int q = threadIdx.x; q < 2 * nt; q += PT) publish(q, row_of_entry(row_ptr, 0, m - 1, target(q)));
        __syncthreads();
        return;
    }
    __shared__ int32_t s_lo[2 * FT_MAX], s_hi[2 * FT_MAX];
    const int nq = 2 * nt;
    const int64_t l1 = (m + PT - 1) / PT;   // rows between the probes of the first step
    {
        const int64_t r = (int64_t)threadIdx.x * l1;
        scr[threadIdx.x] = row_ptr[r < m ? r : m - 1];
    }
    __syncthreads();
    if ((int)threadIdx.x < nq) {
        const int j = last_not_above(scr, PT, target(threadIdx.x));
        const int64_t lo = (int64_t)j * l1 < m ? (int64_t)j * l1 : m - 1, hi = lo + l1 < m ? lo + l1 : m - 1;
        s_lo[threadIdx.x] = (int32_t)lo; s_hi[threadIdx.x] = (int32_t)hi;
    }
    __syncthreads();
    int64_t len = l1;
    for (int probes = 32; probes <= 64; probes *= 2) {   // second and third step
        const int64_t step = (len + probes - 1) / probes;
        for (int i = threadIdx.x; i < nq * probes; i += PT) {
            const int q = i / probes, j = i % probes;
            const int64_t r = (int64_t)s_lo[q] + j * step;
            scr[i] = row_ptr[r < s_hi[q] ? r : s_hi[q]];
        }
        __syncthreads();
        if ((int)threadIdx.x < nq) {
            const int q = threadIdx.x;
            const int j = last_not_above(scr + q * probes, probes, target(q));
            int64_t lo = (int64_t)s_lo[q] + j * step;
            lo = lo < s_hi[q] ? lo : s_hi[q];
            const int64_t hi = lo + step < s_hi[q] ? lo + step : s_hi[q];
            s_lo[q] = (int32_t)lo; s_hi[q] = (int32_t)hi;
        }
        __syncthreads();
        len = step;
    }
    if ((int)threadIdx.x < nq) publish(threadIdx.x, row_of_entry(row_ptr, s_lo[threadIdx.x], s_hi[threadIdx.x], target(threadIdx.x)));
    __syncthreads();
}

__device__ __forceinline__ TileRows stage_tile_rows(const int32_t *__restrict__ row_ptr, int64_t first, int64_t last, int32_t *rps)
{
    __syncthreads();   // the previous tile's readers of rps are done
    TileRows tr;
    tr.r0 = first;
    const int64_t nr = last - first + 1;
    tr.staged = nr >= 1 && nr <= PSUB + 1;
    tr.nr = tr.staged ? (int)nr : 0;
    if (tr.staged)
        for (int i = threadIdx.x; i < tr.nr; i += PT) rps[i] = row_ptr[tr.r0 + i];
    __syncthreads();
    return tr;
}

// CHECK: also the column half of the CSR precondition (columns inside [0, n), ascending inside a row), given row
// pointers that hold theirs (which the caller checks elsewhere: with those, the row found for an entry is its row);
// returns false when an entry of this thread violates it.
template <bool CHECK>
__device__ __forceinline__ bool tile_keys(const int32_t *__restrict__ row_ptr, const int32_t *__restrict__ col_idx, int64_t m, int64_t n,
                                          int64_t ndiag, int64_t t0, int64_t t1, const TileRows &tr, const int32_t *rps, int (&key)[PE])
{
    const int64_t p0 = t0 + (int64_t)threadIdx.x * PE;
    bool good = true;
    int32_t before = -1;   // the column of the entry before this thread's first one (used when both lie in one row)
    if (CHECK && p0 < t1 && p0 > 0) before = col_idx[p0 - 1];
    int32_t c[PE];
    if (p0 + PE <= t1) {   // 64 bytes per lane as four 16-byte loads (any alignment the caller's array has)
#pragma unroll
        for (int q = 0; q < PE / 4; ++q) {
            const int4u w = __builtin_nontemporal_load(reinterpret_cast<const int4u *>(col_idx + p0) + q);
            c[4 * q] = w.x; c[4 * q + 1] = w.y; c[4 * q + 2] = w.z; c[4 * q + 3] = w.w;
        }
    } else {
#pragma unroll
        for (int k = 0; k < PE; ++k) {   // the ragged end of the share: position clamped into the tile
            const int64_t p = p0 + k;
            c[k] = p0 < t1 ? ld_stream(col_idx + (p < t1 ? p : t1 - 1)) : 0;
        }
    }
    int64_t r = tr.r0;
    int lo = 0;
    if (p0 < t1) {
        if (tr.staged) {
            int hi = tr.nr - 1;
            while (lo < hi) {
                const int mid = (lo + hi + 1) >> 1;
                if ((int64_t)rps[mid] <= p0) lo = mid; else hi = mid - 1;
            }
        } else {
            r = row_of_entry(row_ptr, 0, m - 1, p0);
        }
    }
#pragma unroll
    for (int k = 0; k < PE; ++k) {
        const int64_t p = p0 + k;
        if (p < t1) {
            if (tr.staged) {
                while (lo + 1 < tr.nr && (int64_t)rps[lo + 1] <= p) ++lo;
                r = tr.r0 + lo;
            } else {
                while (r + 1 < m && (int64_t)row_ptr[r + 1] <= p) ++r;
            }
            if (CHECK) {
                const int64_t row_start = tr.staged ? (int64_t)rps[lo] : (int64_t)row_ptr[r];
                const int32_t prev = k > 0 ? c[k - 1] : before;
                good = good && (uint32_t)c[k] < (uint64_t)n && (p <= row_start || c[k] > prev);
            }
            int64_t d = (int64_t)c[k] - r + (m - 1);
            d = d < 0 ? 0 : (d >= ndiag ? ndiag - 1 : d);
            key[k] = (int)d;
        } else {
            key[k] = -1;
        }
    }
    return good;
}

// counts[b * gridDim.x + blockIdx.x] = entries of this block's share [blockIdx.x * share, ...) in bucket b.
// err: set to 1 when an entry of the share violates the column half of the CSR precondition.
__global__ __launch_bounds__(PT) void k_part_count(const int32_t *__restrict__ row_ptr, const int32_t *__restrict__ col_idx, int64_t m,
                                                   int64_t n, int64_t nnz, int64_t ndiag, int64_t share, int nb,
                                                   int32_t *__restrict__ counts, uint32_t *__restrict__ err,
                                                   int32_t *__restrict__ tile_rows)
{
    __shared__ int32_t rps[PSUB + 2];
    __shared__ int32_t s_first[P_MAX_TILES], s_last[P_MAX_TILES];
    __shared__ int32_t s_cnt[PB_MAX];
    for (int i = threadIdx.x; i < nb; i += PT) s_cnt[i] = 0;
    const int64_t b0 = (int64_t)blockIdx.x * share;
    const int64_t b1 = b0 + share < nnz ? b0 + share : nnz;
    find_tile_rows(row_ptr, m, b0, b1, s_first, s_last, rps, tile_rows, (int64_t)blockIdx.x * (share / PSUB));
    int t = 0;
    bool bad = false;
    for (int64_t t0 = b0; t0 < b1; t0 += PSUB, ++t) {   // uniform trip count across the block
        const int64_t t1 = t0 + PSUB < b1 ? t0 + PSUB : b1;
        const TileRows tr = stage_tile_rows(row_ptr, s_first[t], s_last[t], rps);
        int key[PE];
        bad = !tile_keys<true>(row_ptr, col_idx, m, n, ndiag, t0, t1, tr, rps, key) || bad;
#pragma unroll
        for (int k = 0; k < PE; ++k)
            if (key[k] >= 0) atomicAdd(&s_cnt[key[k] >> PB_BITS], 1);
    }
    if (bad) *err = 1u;   // every writer stores the same value
    __syncthreads();
    for (int i = threadIdx.x; i < nb; i += PT) counts[(int64_t)i * gridDim.x + blockIdx.x] = s_cnt[i];
}

// Exclusive scan of s_in[0, nb) into s_out[0, nb), nb <= PB_MAX (PB_MAX / PT counters per thread); s_wave: PT / WAVE ints.
__device__ __forceinline__ void block_scan(const int32_t *s_in, int32_t *s_out, int nb, int32_t *s_wave)
{
    constexpr int PER = PB_MAX / PT;
    const int lane = lane_id(), w = threadIdx.x / WAVE;
    int v[PER], sum = 0;
#pragma unroll
    for (int q = 0; q < PER; ++q) {
        const int i = threadIdx.x * PER + q;
        v[q] = i < nb ? s_in[i] : 0;
        sum += v[q];
    }
    int incl = sum;
    for (int o = 1; o < WAVE; o <<= 1) {
        const int t = __shfl_up(incl, o, WAVE);
        if (lane >= o) incl += t;
    }
    if (lane == WAVE - 1) s_wave[w] = incl;
    __syncthreads();
    int base = incl - sum;
    for (int q = 0; q < w; ++q) base += s_wave[q];
#pragma unroll
    for (int q = 0; q < PER; ++q) {
        const int i = threadIdx.x * PER + q;
        if (i < nb) s_out[i] = base;
        base += v[q];
    }
    __syncthreads();
}

// offs: the exclusive scan of counts (same layout).  keys16[offs[b][block] ...] receives this block's entries of
// bucket b, as diagonal numbers relative to the bucket.
__global__ __launch_bounds__(PT) void k_part_scatter(const int32_t *__restrict__ row_ptr, const int32_t *__restrict__ col_idx, int64_t m,
                                                     int64_t nnz, int64_t ndiag, int64_t share, int nb, const int32_t *__restrict__ offs,
                                                     const int32_t *__restrict__ tile_rows, uint16_t *__restrict__ keys16)
{
    __shared__ int32_t rps[PSUB + 2];
    __shared__ int32_t s_first[P_MAX_TILES], s_last[P_MAX_TILES];
    __shared__ int32_t s_cnt[PB_MAX], s_start[PB_MAX], s_goff[PB_MAX], s_wave[PT / WAVE];
    __shared__ uint16_t s_key[PSUB], s_bkt[PSUB];
    for (int i = threadIdx.x; i < nb; i += PT) s_goff[i] = offs[(int64_t)i * gridDim.x + blockIdx.x];
    const int64_t b0 = (int64_t)blockIdx.x * share;
    const int64_t b1 = b0 + share < nnz ? b0 + share : nnz;
    {   // the rows of the tiles, as the count pass found them (clamped: they index row_ptr)
        const int nt = (int)((b1 - b0 + PSUB - 1) / PSUB);
        const int64_t tile_base = (int64_t)blockIdx.x * (share / PSUB);
        for (int q = threadIdx.x; q < 2 * nt; q += PT) {
            int64_t r = tile_rows[2 * tile_base + q];
            r = r < 0 ? 0 : (r > m - 1 ? m - 1 : r);
            if (q & 1) s_last[q >> 1] = (int32_t)r; else s_first[q >> 1] = (int32_t)r;
        }
        __syncthreads();
    }
    int t = 0;
    for (int64_t t0 = b0; t0 < b1; t0 += PSUB, ++t) {   // uniform trip count across the block
        const int64_t t1 = t0 + PSUB < b1 ? t0 + PSUB : b1;
        const int cnt_tile = (int)(t1 - t0);
        for (int i = threadIdx.x; i < nb; i += PT) s_cnt[i] = 0;
        const TileRows tr = stage_tile_rows(row_ptr, s_first[t], s_last[t], rps);
        int key[PE], rank[PE];
        tile_keys<false>(row_ptr, col_idx, m, 0, ndiag, t0, t1, tr, rps, key);
#pragma unroll
        for (int k = 0; k < PE; ++k) rank[k] = key[k] >= 0 ? atomicAdd(&s_cnt[key[k] >> PB_BITS], 1) : 0;
        __syncthreads();
        block_scan(s_cnt, s_start, nb, s_wave);
#pragma unroll
        for (int k = 0; k < PE; ++k) {
            if (key[k] >= 0) {
                const int b = key[k] >> PB_BITS, pos = s_start[b] + rank[k];   // < cnt_tile
                s_key[pos] = (uint16_t)(key[k] & (PB_KEYS - 1));
                s_bkt[pos] = (uint16_t)b;
            }
        }
        __syncthreads();
        for (int pos = threadIdx.x; pos < cnt_tile; pos += PT) {   // runs of one bucket go to consecutive addresses
            const int b = s_bkt[pos];
            const int64_t dst = (int64_t)s_goff[b] + (pos - s_start[b]);
            if (dst >= 0 && dst < nnz) keys16[dst] = s_key[pos];
        }
        __syncthreads();
        for (int i = threadIdx.x; i < nb; i += PT) s_goff[i] += s_cnt[i];
        __syncthreads();
    }
}

// Block b owns bucket b: entries [offs[b * nblk], offs[(b + 1) * nblk]) of keys16 (the last bucket ends at nnz).
// hist (or nullptr): receives the bucket's stretch of the full histogram.  dpart (or nullptr): receives the block's
// two counts; otherwise they are added to ctr.
__global__ __launch_bounds__(PH) void k_part_hist(const uint16_t *__restrict__ keys16, const int32_t *__restrict__ offs, int nblk, int nb,
                                                  int64_t nnz, int64_t ndiag, unsigned long long thr_rhs, unsigned long long td_den,
                                                  uint32_t *__restrict__ hist, DiagPart *__restrict__ dpart, Counters *__restrict__ ctr)
{
    __shared__ uint32_t s_tab[PB_KEYS];
    for (int i = threadIdx.x; i < PB_KEYS; i += PH) s_tab[i] = 0u;
    __syncthreads();
    const int b = blockIdx.x;
    int64_t e0 = offs[(int64_t)b * nblk], e1 = b + 1 < nb ? (int64_t)offs[(int64_t)(b + 1) * nblk] : nnz;
    e0 = e0 < 0 ? 0 : (e0 > nnz ? nnz : e0);
    e1 = e1 < e0 ? e0 : (e1 > nnz ? nnz : e1);
    constexpr int U = 8;
    for (int64_t i0 = e0 + threadIdx.x; i0 < e1; i0 += (int64_t)PH * U) {
        uint16_t k[U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int64_t i = i0 + (int64_t)u * PH;
            k[u] = ld_stream(keys16 + (i < e1 ? i : e1 - 1));
        }
#pragma unroll
        for (int u = 0; u < U; ++u)
            if (i0 + (int64_t)u * PH < e1) atomicAdd(&s_tab[k[u] & (PB_KEYS - 1)], 1u);
    }
    __syncthreads();
    unsigned long long c_nd = 0ull, c_td = 0ull;
    const int64_t g0 = (int64_t)b * PB_KEYS;
    for (int i = threadIdx.x; i < PB_KEYS; i += PH) {
        const int64_t g = g0 + i;
        if (g < ndiag) {
            const unsigned long long c = s_tab[i];
            if (hist) hist[g] = (uint32_t)c;
            if (c >= 1ull) {
                ++c_nd;
                if (c * td_den >= thr_rhs) ++c_td;
            }
        }
    }
    c_nd = wave_sum(c_nd); c_td = wave_sum(c_td);
    __shared__ unsigned long long s_nd[PH / WAVE], s_td[PH / WAVE];
    if (lane_id() == 0) { s_nd[threadIdx.x / WAVE] = c_nd; s_td[threadIdx.x / WAVE] = c_td; }
    __syncthreads();
    if (threadIdx.x == 0) {
        for (int w = 1; w < PH / WAVE; ++w) { c_nd += s_nd[w]; c_td += s_td[w]; }
        if (dpart) dpart[b] = DiagPart{c_nd, c_td};
        else {
            if (c_nd) atomicAdd(&ctr->n_diag, c_nd);
            if (c_td) atomicAdd(&ctr->n_true, c_td);
        }
    }
}

// The rule of the decision: enough sampled entries, fewer than a quarter of them on a diagonal that another row of
// their group of adjacent rows also holds (nothing for the traversal kernel to merge), and no bucket with more than a
// tenth of them (columns scattered inside a narrow band would leave the last pass to one or two blocks).
__host__ __device__ inline bool sample_says_partition(uint64_t total, uint64_t repeated, uint64_t biggest_bucket)
{
    return total >= 2048 && repeated * 4 < total && biggest_bucket * 10 <= total;
}

// Block g samples the SR adjacent rows that start at row floor(g * (m - SR + 1) / SG), SE entries of each (entry
// floor(e * len / SE) of the row, or every entry when the row holds at most SE), and leaves two counts in
// out[2 g], out[2 g + 1]: the sampled entries, and those among them whose diagonal another row of the group also holds.
// acc: device words (8-byte aligned), zero on entry: [0, 1] one 64-bit word that packs the sampled entries, those on a
// diagonal that another row of their group also holds, and the blocks that are done, [2] unused, [3] the decision, [4 .. 4 + nb) sampled entries per bucket.  The block that finishes
// last turns the counts into the decision (1 = partition), stores it in acc[3] and, when given, in *flag_host (pinned),
// and clears the rest for the next call: kernels launched behind this one can read the decision without the host in
// between.
__global__ __launch_bounds__(SR * SE) void k_part_sample(const int32_t *__restrict__ row_ptr, const int32_t *__restrict__ col_idx, int64_t m,
                                                          int64_t nnz, int64_t ndiag, int nb, uint32_t *acc, uint32_t *flag_host)
{
    __shared__ int32_t s_key[SR * SE];
    __shared__ uint32_t s_tot[SR * SE / WAVE], s_rep[SR * SE / WAVE];
    __shared__ uint32_t s_last, s_max;
    __shared__ unsigned long long s_sum;
    static_assert(SG < 256 && SR * SE * SG < (1 << 20), "the packed counters of the sample");
    const int r = threadIdx.x / SE, e = threadIdx.x % SE;
    const int64_t span = m - SR + 1 > 0 ? m - SR + 1 : 1;
    const int64_t row = (int64_t)blockIdx.x * span / SG + r;
    int32_t key = -1;
    if (row < m) {
        int64_t lo = row_ptr[row], hi = row_ptr[row + 1];
        lo = lo < 0 ? 0 : (lo > nnz ? nnz : lo);
        hi = hi < lo ? lo : (hi > nnz ? nnz : hi);
        const int64_t len = hi - lo;
        if (len > 0 && (len > SE || e < len)) {
            const int64_t q = lo + (len > SE ? (int64_t)e * len / SE : (int64_t)e);
            int64_t d = (int64_t)col_idx[q] - row + (m - 1);
            d = d < 0 ? 0 : (d >= ndiag ? ndiag - 1 : d);
            key = (int32_t)d;
        }
    }
    s_key[threadIdx.x] = key;
    if (threadIdx.x == 0) { s_last = 0u; s_max = 0u; }
    // bucket counts of the block first (a structured matrix puts all its samples into a few buckets: one global atomic
    // per sample on those few addresses took 100 us), then one atomic per bucket the block met
    __shared__ uint32_t s_bkt[PB_MAX];
    for (int i = threadIdx.x; i < nb; i += SR * SE) s_bkt[i] = 0u;
    __syncthreads();
    if (key >= 0) atomicAdd(&s_bkt[key >> PB_BITS], 1u);   // key >> PB_BITS < nb <= PB_MAX
    __syncthreads();
    for (int i = threadIdx.x; i < nb; i += SR * SE) {
        const uint32_t c = s_bkt[i];
        if (c) {
            atomicAdd(&acc[4 + i], c);
            __threadfence();   // out before the block reports itself done (few threads get here)
        }
    }
    int hits = 0;   // every lane runs the whole loop: its LDS reads are independent and overlap
#pragma unroll 16
    for (int j = 0; j < SR * SE; ++j) hits += (s_key[j] == key) & (j / SE != r);
    const bool rep = key >= 0 && hits > 0;
    const uint32_t tot_w = (uint32_t)__popcll(ballot64(key >= 0)), rep_w = (uint32_t)__popcll(ballot64(rep));
    if (lane_id() == 0) { s_tot[threadIdx.x / WAVE] = tot_w; s_rep[threadIdx.x / WAVE] = rep_w; }
    __syncthreads();
    if (threadIdx.x == 0) {
        uint32_t t = 0, q = 0;
        for (int w = 0; w < SR * SE / WAVE; ++w) { t += s_tot[w]; q += s_rep[w]; }
        // one atomic for the three: sampled entries in bits 0-19, repeated ones in bits 20-39, blocks done from bit 40 on
        // (same-address atomics are served one after the other, and 128 blocks send theirs at about the same time)
        unsigned long long *word = reinterpret_cast<unsigned long long *>(acc);
        const unsigned long long old = atomicAdd(word, (unsigned long long)t | ((unsigned long long)q << 20) | (1ull << 40));
        if ((old >> 40) == gridDim.x - 1) {   // every other block's counts are in
            s_last = 1u;
            s_sum = old + ((unsigned long long)t | ((unsigned long long)q << 20));
        }
    }
    __syncthreads();
    if (!s_last) return;
    uint32_t mx = 0u;
    for (int i = threadIdx.x; i < nb; i += SR * SE) {   // read and cleared with atomics: they were counted with atomics
        const uint32_t c = atomicExch(&acc[4 + i], 0u);
        mx = c > mx ? c : mx;
    }
    atomicMax(&s_max, mx);
    __syncthreads();
    if (threadIdx.x == 0) {
        const uint32_t total = (uint32_t)(s_sum & 0xfffffull), repeated = (uint32_t)((s_sum >> 20) & 0xfffffull);
        const uint32_t want = sample_says_partition(total, repeated, s_max) ? 1u : 0u;
        acc[3] = want;
        if (flag_host) *flag_host = want;
        atomicExch(reinterpret_cast<unsigned long long *>(acc), 0ull);
    }
}

int part_blocks(int64_t nnz, int64_t *share)
{
    int64_t sh = (nnz + P_MAX_BLOCKS - 1) / P_MAX_BLOCKS;
    sh = (sh + PSUB - 1) / PSUB * PSUB;
    if (sh < PSUB) sh = PSUB;
    *share = sh;
    return (int)((nnz + sh - 1) / sh);
}

}  // namespace

bool partition_possible(const mo_csr &a)
{
    const int64_t ndiag = a.m + a.n - 1;
    return a.nnz >= PART_MIN_NNZ && a.m >= SR && ndiag <= (int64_t)PB_MAX * PB_KEYS;
}

int partition_buckets(const mo_csr &a) { return (int)((a.m + a.n - 1 + PB_KEYS - 1) / PB_KEYS); }

size_t partition_sample_bytes() { return (size_t)(4 + PB_MAX) * sizeof(uint32_t); }

// Enqueues the sample, whose last block leaves the decision in acc[3] (for the kernels enqueued behind it) and in
// *flag_host (pinned, or nullptr).  acc: partition_sample_bytes() of device memory that is zero between calls (the
// kernel leaves it so, acc[3] aside).
mo_status partition_decide_async(const mo_csr &a, uint32_t *acc, uint32_t *flag_host, hipStream_t s)
{
    const int64_t ndiag = a.m + a.n - 1;
    hipLaunchKernelGGL(k_part_sample, dim3(SG), dim3(SR * SE), 0, s, a.row_ptr, a.col_idx, a.m, a.nnz, ndiag, partition_buckets(a), acc,
                       flag_host);
    MO_LAUNCH_CHECK();
    return MO_OK;
}

// The same decision for a caller that waits for it.  acc as above.  Synchronises the stream.
mo_status partition_wanted(const mo_csr &a, uint32_t *acc, bool *wanted, hipStream_t s)
{
    *wanted = false;
    if (!partition_possible(a)) return MO_OK;
    MO_TRY(partition_decide_async(a, acc, nullptr, s));
    uint32_t flag = 0;
    MO_HIP(hipMemcpyAsync(&flag, acc + 3, sizeof(flag), hipMemcpyDeviceToHost, s));
    MO_HIP(hipStreamSynchronize(s));
    *wanted = flag != 0u;
    return MO_OK;
}

// Device memory the partition needs besides the histogram: [counts | offsets | scan temporary | tile rows | keys16].
size_t partition_scratch_bytes(const mo_csr &a)
{
    int64_t share = 0;
    const int nblk = part_blocks(a.nnz, &share);
    const size_t cells = (size_t)partition_buckets(a) * (size_t)nblk;
    const size_t ints = ((cells + 1) * 4 + 255) / 256 * 256;   // the scan also writes the total behind its last prefix
    const size_t tmp = (scan_tmp_bytes((int64_t)cells) + 255) / 256 * 256;
    const size_t trows = ((size_t)nblk * (size_t)(share / PSUB) * 2 * 4 + 255) / 256 * 256;
    return 2 * ints + tmp + trows + (size_t)a.nnz * sizeof(uint16_t) + 256;
}

// The diagonal counts by partition.  buf: partition_scratch_bytes(a) of device memory.  hist (or nullptr): receives all
// m + n - 1 counters.  dpart (or nullptr): receives one pair of counts per bucket (partition_buckets(a) of them);
// otherwise the counts are added to ctr, which the caller has reset.  err: a word the caller has cleared, set to 1 when
// a column lies outside [0, n) or does not ascend inside its row (meaningful for row pointers that are in order, which
// the caller checks with k_row_stats).  Enqueues only.
mo_status partition_counts(const mo_csr &a, const mo_params &p, void *buf, uint32_t *hist, DiagPart *dpart, Counters *ctr, uint32_t *err,
                           hipStream_t s)
{
    const int64_t ndiag = a.m + a.n - 1;
    int64_t share = 0;
    const int nblk = part_blocks(a.nnz, &share);
    const int nb = partition_buckets(a);
    const size_t cells = (size_t)nb * (size_t)nblk;
    const size_t ints = ((cells + 1) * 4 + 255) / 256 * 256;   // the scan also writes the total behind its last prefix
    const size_t tmp = (scan_tmp_bytes((int64_t)cells) + 255) / 256 * 256;
    int32_t *counts = (int32_t *)buf;
    int32_t *offs = (int32_t *)((char *)buf + ints);
    void *scan_tmp = (char *)buf + 2 * ints;
    const size_t trows = ((size_t)nblk * (size_t)(share / PSUB) * 2 * 4 + 255) / 256 * 256;
    int32_t *tile_rows = (int32_t *)((char *)buf + 2 * ints + tmp);
    uint16_t *keys16 = (uint16_t *)((char *)buf + 2 * ints + tmp + trows);
    hipLaunchKernelGGL(k_part_count, dim3((unsigned)nblk), dim3(PT), 0, s, a.row_ptr, a.col_idx, a.m, a.n, a.nnz, ndiag, share, nb, counts, err, tile_rows);
    MO_LAUNCH_CHECK();
    MO_TRY(exclusive_scan_i32(counts, offs, (int64_t)cells, scan_tmp, s));
    hipLaunchKernelGGL(k_part_scatter, dim3((unsigned)nblk), dim3(PT), 0, s, a.row_ptr, a.col_idx, a.m, a.nnz, ndiag, share, nb, offs, tile_rows, keys16);
    MO_LAUNCH_CHECK();
    const int64_t mn = a.m < a.n ? a.m : a.n;
    hipLaunchKernelGGL(k_part_hist, dim3((unsigned)nb), dim3(PH), 0, s, keys16, offs, nblk, nb, a.nnz, ndiag,
                       (unsigned long long)mn * (unsigned long long)p.td_num, (unsigned long long)p.td_den, hist, dpart, ctr);
    MO_LAUNCH_CHECK();
    return MO_OK;
}

}  // namespace mo

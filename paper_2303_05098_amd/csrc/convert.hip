// CSR -> {COO, DIA, ELL, HYB, HDC} on the device (formats: Section II-B).
//
// Every conversion is integer bookkeeping plus copies of the stored values, so the produced arrays are fully
// determined by the input: offsets ascending, row entries in ascending column order, padding col = -1 / val = +0.
// Rows are mapped one per lane, which makes the writes into the slot-major ELL slabs and the diagonal-major DIA
// slabs coalesced; a row longer than SHORT_ROW entries is handled by the whole wave.
#include "dev_common.hpp"
#include "feat_common.hpp"
#include "mo_internal.hpp"

#include <algorithm>
#include <cmath>
#include <new>

namespace mo {

constexpr int CB = 256;
// SHORT_ROW (feat_common.hpp): entries of a row handled lane-per-row; the rest is walked by the whole wave

// ------------------------------------------------------------------ row walker
// Calls f(row, p, s, col, val, own) for every stored entry p of the rows owned by this wave (one row per lane), s =
// position of the entry inside its row.
// The entries of the wave's rows (one contiguous run of the CSR arrays) are first streamed into
// the wave's own LDS region with coalesced loads, WCAP entries at a time, and the lanes then pick their rows' entries
// out of LDS.  Lane-per-row reads straight from global memory touch one cache line per lane
// and step; this way every line is read once.  Rows longer than SHORT_ROW are left to the cooperative loop, which
// reads global memory with consecutive lanes anyway.  No block barrier: a wave's LDS accesses execute in order.
constexpr int WCAP = 1024;
constexpr int WALK_U = 4;

template <typename T, class F>
__device__ __forceinline__ void walk_rows_lds(bool rv, int64_t row, int64_t lo64, int64_t hi64, const int32_t *__restrict__ col_idx,
                                              const T *__restrict__ val, int32_t *s_col, T *s_val, int skip_len, F f)
{
    const int lane = lane_id();
    const int lo = (int)lo64, hi = (int)hi64;   // positions fit 32 bits: nnz < 2^31
    const int len = hi - lo;
    const bool is_short = rv && len <= SHORT_ROW;
    // The valid rows of a wave are a prefix of its lanes and row_ptr is non-decreasing (conversions run on a CSR that
    // has passed validation), so the wave's run starts at the first lane's lo and ends at the last valid lane's hi.
    const int nvalid = __popcll(ballot64(rv));
    const int wb = __builtin_amdgcn_readfirstlane(lo);
    const int we = nvalid ? __builtin_amdgcn_readlane(hi, nvalid - 1) : 0;
    for (int c0 = wb; c0 < we; c0 += WCAP) {
        const int c1 = we - c0 > WCAP ? c0 + WCAP : we;
        if (ballot64(is_short && hi > c0 && lo < c1) == 0ull) continue;   // a stretch inside one long row: nothing to stage
        stage_pair_to_lds(col_idx + c0, val + c0, s_col, s_val, c1 - c0, lane);
        const int a = lo > c0 ? lo : c0, b = hi < c1 ? hi : c1;
        const int cnt = (is_short && b > a) ? b - a : 0;
        const int off = cnt ? a - c0 : 0;
        // WALK_U entries per lane and step: their LDS reads are issued together (clamped inside the lane's run, so
        // unconditional), then handed to f one by one
        for (int k = 0; ballot64(k < cnt) != 0ull; k += WALK_U) {
            int32_t cc[WALK_U];
            T vv[WALK_U];
#pragma unroll
            for (int u = 0; u < WALK_U; ++u) {
                const int kk = k + u < cnt ? k + u : (cnt > 0 ? cnt - 1 : 0);
                cc[u] = s_col[off + kk];
                vv[u] = s_val[off + kk];
            }
#pragma unroll
            for (int u = 0; u < WALK_U; ++u)
                if (k + u < cnt) f(row, (int64_t)a + k + u, (int64_t)(a + k + u - lo), cc[u], vv[u], true);
        }
    }
    // skip_len > 0: rows longer than that are left to a kernel that spreads their entries over the whole chip
    uint64_t longmask = ballot64(rv && len > SHORT_ROW && !(skip_len > 0 && len > skip_len));
    while (longmask) {
        const int l = __ffsll((unsigned long long)longmask) - 1;
        longmask &= longmask - 1;
        const int64_t r = row - lane + l;
        const int rlo = __builtin_amdgcn_readlane(lo, l), rhi = __builtin_amdgcn_readlane(hi, l);
        for (int q = rlo + lane; q < rhi; q += WAVE) f(r, (int64_t)q, (int64_t)(q - rlo), col_idx[q], val[q], false);
    }
}

__global__ void k_fill_i32(int32_t *p, int64_t n, int32_t v)
{
    int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    for (; i < n; i += stride) p[i] = v;
}

// ------------------------------------------------------------------ COO
// Entry-parallel: a block copies a tile of COO_CT consecutive entries with coalesced loads and stores and attaches
// the row index to each.  The rows that intersect the tile are found by two binary searches in row_ptr; their
// row_ptr slice is staged in LDS and every entry searches that slice (global row_ptr when the slice is too long,
// i.e. when the tile spans many empty rows).
constexpr int COO_CT = 2048;

template <typename T>
__global__ __launch_bounds__(CB) void k_csr_to_coo(const int32_t *__restrict__ row_ptr, const int32_t *__restrict__ col_idx,
                                                    const T *__restrict__ val, int64_t m, int64_t nnz, int32_t *__restrict__ orow,
                                                    int32_t *__restrict__ ocol, T *__restrict__ oval)
{
    __shared__ int32_t rps[COO_CT + 2];
    __shared__ int64_t s_r[2];
    const int64_t t0 = (int64_t)blockIdx.x * COO_CT;
    const int64_t t1 = t0 + COO_CT < nnz ? t0 + COO_CT : nnz;
    if (threadIdx.x == 0) s_r[0] = row_of_entry(row_ptr, 0, m - 1, t0);
    if (threadIdx.x == WAVE) s_r[1] = row_of_entry(row_ptr, 0, m - 1, t1 - 1);
    __syncthreads();
    const int64_t r0 = s_r[0], r1 = s_r[1];
    const int64_t nr = r1 - r0 + 1;
    const bool staged = nr <= COO_CT + 1;
    if (staged) {
        for (int i = threadIdx.x; i < (int)nr; i += CB) rps[i] = row_ptr[r0 + i];
        __syncthreads();
    }
    for (int64_t p = t0 + threadIdx.x; p < t1; p += CB) {
        int64_t r;
        if (staged) {
            int lo = 0, hi = (int)nr - 1;
            while (lo < hi) {
                const int mid = (lo + hi + 1) >> 1;
                if ((int64_t)rps[mid] <= p) lo = mid; else hi = mid - 1;
            }
            r = r0 + lo;
        } else {
            r = row_of_entry(row_ptr, r0, r1, p);
        }
        orow[p] = (int32_t)r;
        ocol[p] = ld_stream(col_idx + p);
        oval[p] = ld_stream(val + p);
    }
}

// ------------------------------------------------------------------ diagonal selection
// Appends the offset of every diagonal kept by the DIA part - all non-empty ones (DIA) or the true ones (HDC) - to
// off_out, in any order: there are few of them (at most max_fill times the mean row length), so the host sorts the
// list, which it needs anyway for the launch plan of the SpMV kernel, and sends it back.
__global__ __launch_bounds__(CB) void k_collect_diag(const uint32_t *__restrict__ hist, int64_t ndiag, int all_nonempty,
                                                      unsigned long long thr_rhs, unsigned long long td_den, int64_t m,
                                                      int32_t *__restrict__ count, int32_t *__restrict__ off_out, int32_t cap)
{
    const int64_t stride = (int64_t)gridDim.x * CB;
    for (int64_t i = (int64_t)blockIdx.x * CB + threadIdx.x; i < ndiag; i += stride) {
        const unsigned long long c = hist[i];
        if (c >= 1ull && (all_nonempty || c * td_den >= thr_rhs)) {
            const int32_t p = atomicAdd(count, 1);
            if (p < cap) off_out[p] = (int32_t)(i - (m - 1));
        }
    }
}

// Index of offset `off` in the ascending list dia_off[0, nd), or -1.
__device__ __forceinline__ int find_slot(const int32_t *__restrict__ dia_off, int nd, int32_t off)
{
    int lo = 0, hi = nd;
    while (lo < hi) {
        const int mid = (lo + hi) >> 1;
        if (dia_off[mid] < off) lo = mid + 1; else hi = mid;
    }
    return (lo < nd && dia_off[lo] == off) ? lo : -1;
}

// DIA part of DIA / HDC.  A wave owns rw consecutive rows and stages their run of entries in LDS once.  Columns ascend
// inside a row (CSR precondition) and so do the kept offsets, so a row is merged against the offset list: the loop
// runs over the kept diagonals, the same for every lane, and each lane either consumes its next entry (when that
// entry lies on the diagonal) or contributes a zero.  Every slot of the slab is therefore written exactly once, by
// stores that cover rw consecutive rows of one diagonal; no zero-fill pass and no per-entry slot lookup are needed.
// Entries that fall between kept diagonals (HDC) are skipped and counted into rest_cnt[row].
// Rows that do not fit the staged window are merged straight from global memory; rows longer than SHORT_ROW are
// handled by the whole wave, each entry finding its slot by binary search in the offset list (zero the row's slots,
// wait for those stores, then scatter).
template <typename T, class ColAt, class ValAt>
__device__ __forceinline__ int dia_merge_row(bool act, bool store, int cnt, int64_t row, const int32_t *__restrict__ dia_off, int nd,
                                             int64_t ld, T *__restrict__ dval, ColAt col_at, ValAt val_at)
{
    constexpr int32_t NONE = 0x7fffffff;        // no entry left: larger than any offset (m + n <= 2^31 - 1)
    int e = 0, matched = 0;
    int32_t cur = (act && cnt > 0) ? (int32_t)((int64_t)col_at(0) - row) : NONE;
    for (int d = 0; d < nd; ++d) {
        const int32_t target = dia_off[d];
        while (cur < target) {                   // entries on diagonals that are not kept
            ++e;
            cur = e < cnt ? (int32_t)((int64_t)col_at(e) - row) : NONE;
        }
        T out = (T)0;
        if (cur == target) {
            out = val_at(e);
            ++e;
            ++matched;
            cur = e < cnt ? (int32_t)((int64_t)col_at(e) - row) : NONE;
        }
        if (store) dval[(int64_t)d * ld + row] = out;
    }
    return matched;
}

template <typename T>
__global__ __launch_bounds__(CB) void k_fill_dia(const int32_t *__restrict__ row_ptr, const int32_t *__restrict__ col_idx,
                                                  const T *__restrict__ val, int64_t m,
                                                  const int32_t *__restrict__ dia_off, int nd, int64_t ld, T *__restrict__ dval,
                                                  int32_t *__restrict__ rest_cnt, int rw, int skip_len)
{
    __shared__ int32_t s_col[(CB / WAVE) * WCAP];
    __shared__ T s_val[(CB / WAVE) * WCAP];
    const int lane = lane_id();
    int32_t *sc = s_col + (threadIdx.x / WAVE) * WCAP;
    T *sv = s_val + (threadIdx.x / WAVE) * WCAP;
    const int64_t row = (xcd_block(blockIdx.x, gridDim.x) * (CB / WAVE) + threadIdx.x / WAVE) * rw + lane;
    const bool rv = lane < rw && row < m;
    const bool pad = lane < rw && row >= m && row < ld;      // rows of the slab beyond the matrix hold zeros
    const int lo = row_ptr[row < m ? row : m], hi = row_ptr[row + 1 < m ? row + 1 : m];   // empty run past the last row
    const int len = hi - lo;
    const int nvalid = __popcll(ballot64(rv));   // the valid rows of a wave are a prefix of its lanes
    const int wb = __builtin_amdgcn_readfirstlane(lo);
    const int we = nvalid ? __builtin_amdgcn_readlane(hi, nvalid - 1) : wb;
    const int staged = we - wb < WCAP ? we - wb : WCAP;
    if (staged > 0) stage_pair_to_lds(col_idx + wb, val + wb, sc, sv, staged, lane);
    const bool is_short = rv && len <= SHORT_ROW;
    const bool in_lds = is_short && hi - wb <= staged;
    const int off = in_lds ? lo - wb : 0;
    int matched = dia_merge_row<T>(in_lds, in_lds || pad, in_lds ? len : 0, row, dia_off, nd, ld, dval,
                                   [&](int e) { return sc[off + e]; }, [&](int e) { return sv[off + e]; });
    // Longer rows whose entries mostly lie on kept diagonals (a wide band: at most two entries per kept diagonal) are
    // merged by their own lane as well, straight from global memory: the stores stay coalesced across the rows of the
    // wave and no slot is zeroed first (a 100 000-row band of 300 diagonals: 6.0 -> 1.7 ms, 400 000 rows of 64: 14.8 -> 1.1 ms; row by row with the whole
    // wave, every store hits a line of its own).
    const bool merged_long = rv && !is_short && (int64_t)len <= 2 * (int64_t)nd;
    const bool direct = (is_short && !in_lds) || merged_long;
    if (ballot64(direct) != 0ull)
        matched += dia_merge_row<T>(direct, direct, direct ? len : 0, row, dia_off, nd, ld, dval,
                                    [&](int e) { return col_idx[lo + e]; }, [&](int e) { return val[lo + e]; });
    if (rest_cnt && (is_short || merged_long)) rest_cnt[row] = len - matched;
    uint64_t longmask = ballot64(rv && len > SHORT_ROW && !merged_long);
    while (longmask) {
        const int l = __ffsll((unsigned long long)longmask) - 1;
        longmask &= longmask - 1;
        const int64_t r = row - lane + l;
        const int rlo = __builtin_amdgcn_readlane(lo, l), rhi = __builtin_amdgcn_readlane(hi, l);
        for (int d = lane; d < nd; d += WAVE) dval[(int64_t)d * ld + r] = (T)0;
        if (skip_len > 0 && rhi - rlo > skip_len) {   // its entries are left to k_fill_dia_long, launched behind this kernel
            if (rest_cnt && lane == 0) rest_cnt[r] = 0;
            continue;
        }
        __threadfence();                         // the zeros are in place before other lanes store values of this row
        int rest = 0;
        for (int q0 = rlo; q0 < rhi; q0 += WAVE) {
            const int q = q0 + lane;
            int k = 0;
            if (q < rhi) {
                k = find_slot(dia_off, nd, (int32_t)((int64_t)col_idx[q] - r));
                if (k >= 0) dval[(int64_t)k * ld + r] = val[q];
            }
            rest += (int)__popcll(ballot64(k < 0));
        }
        if (rest_cnt && lane == 0) rest_cnt[r] = rest;
    }
}

// ------------------------------------------------------------------ rows too long for one wave (DIA / HDC)
// The rows that k_fill_dia and k_hdc_rest skipped (longer than VLONG_ROW and not merged lane per row; listed by the
// analysis), entry-parallel over the whole grid in chunks of RL_CHUNK entries, RL_U consecutive entries per thread.
constexpr int RL_B = 256, RL_U = 4, RL_CHUNK = RL_B * RL_U, RL_BLOCKS = 512;

__device__ __forceinline__ int rl_block_sum(int v, int *s_w)
{
    v = wave_sum(v);
    if (lane_id() == 0) s_w[threadIdx.x / WAVE] = v;
    __syncthreads();
    int t = 0;
    for (int w = 0; w < RL_B / WAVE; ++w) t += s_w[w];
    __syncthreads();
    return t;
}

// s_base[li] = chunks of the listed rows before row li (s_base[nrows] = all chunks); rows that the main kernels did
// not skip (merged lane per row: at most two entries per kept diagonal) count no chunks.
__device__ __forceinline__ void rl_chunk_bases(const LongRows *__restrict__ lr, int nrows, const int32_t *__restrict__ row_ptr, int64_t m,
                                               int nd, int *s_base)
{
    for (int li = threadIdx.x; li < nrows; li += RL_B) {
        const int64_t r = lr->rows[li];
        int64_t len = (r >= 0 && r < m) ? (int64_t)row_ptr[r + 1] - row_ptr[r] : 0;
        if (len <= 2 * (int64_t)nd || len <= VLONG_ROW) len = 0;
        s_base[li + 1] = (int)((len + RL_CHUNK - 1) / RL_CHUNK);
    }
    if (threadIdx.x == 0) s_base[0] = 0;
    __syncthreads();
    if (threadIdx.x == 0)
        for (int li = 0; li < nrows; ++li) s_base[li + 1] += s_base[li];
    __syncthreads();
}

// Row of the list that chunk g belongs to: the largest li with s_base[li] <= g.
__device__ __forceinline__ int rl_row_of_chunk(const int *s_base, int nrows, int g)
{
    int lo = 0, hi = nrows - 1;
    while (lo < hi) {
        const int mid = (lo + hi + 1) >> 1;
        if (s_base[mid] <= g) lo = mid; else hi = mid - 1;
    }
    return lo;
}

// DIA part: every entry finds its slot (the main kernel has zeroed the row's slots); entries off the kept diagonals
// are counted into rest_cnt[row] (HDC; set to 0 by the main kernel).
template <typename T>
__global__ __launch_bounds__(RL_B) void k_fill_dia_long(const LongRows *__restrict__ lr, int nrows, const int32_t *__restrict__ row_ptr,
                                                        const int32_t *__restrict__ col_idx, const T *__restrict__ val, int64_t m,
                                                        const int32_t *__restrict__ dia_off, int nd, int64_t ld, T *__restrict__ dval,
                                                        int32_t *__restrict__ rest_cnt)
{
    __shared__ int s_base[LR_CAP + 2];
    __shared__ int s_w[RL_B / WAVE];
    rl_chunk_bases(lr, nrows, row_ptr, m, nd, s_base);
    const int total = s_base[nrows];
    for (int g = blockIdx.x; g < total; g += gridDim.x) {   // uniform across the block
        const int li = rl_row_of_chunk(s_base, nrows, g);
        const int64_t r = lr->rows[li];
        const int64_t lo = row_ptr[r], hi = row_ptr[r + 1];
        const int64_t q0 = lo + (int64_t)(g - s_base[li]) * RL_CHUNK + (int64_t)threadIdx.x * RL_U;
        int rest = 0;
#pragma unroll
        for (int u = 0; u < RL_U; ++u) {
            const int64_t q = q0 + u;
            if (q < hi) {
                const int k = find_slot(dia_off, nd, (int32_t)((int64_t)col_idx[q] - r));
                if (k >= 0) dval[(int64_t)k * ld + r] = val[q];
                else ++rest;
            }
        }
        if (rest_cnt) {   // uniform
            const int t = rl_block_sum(rest, s_w);
            if (threadIdx.x == 0 && t) atomicAdd(&rest_cnt[r], t);
        }
    }
}

// CSR remainder of HDC, first pass: chunk_cnt[g] = entries of chunk g that lie off the kept diagonals.
__global__ __launch_bounds__(RL_B) void k_hdc_rest_long_count(const LongRows *__restrict__ lr, int nrows, const int32_t *__restrict__ row_ptr,
                                                              const int32_t *__restrict__ col_idx, int64_t m,
                                                              const int32_t *__restrict__ dia_off, int nd, int32_t *__restrict__ chunk_cnt)
{
    __shared__ int s_base[LR_CAP + 2];
    __shared__ int s_w[RL_B / WAVE];
    rl_chunk_bases(lr, nrows, row_ptr, m, nd, s_base);
    const int total = s_base[nrows];
    for (int g = blockIdx.x; g < total; g += gridDim.x) {
        const int li = rl_row_of_chunk(s_base, nrows, g);
        const int64_t r = lr->rows[li];
        const int64_t lo = row_ptr[r], hi = row_ptr[r + 1];
        const int64_t q0 = lo + (int64_t)(g - s_base[li]) * RL_CHUNK + (int64_t)threadIdx.x * RL_U;
        int rest = 0;
#pragma unroll
        for (int u = 0; u < RL_U; ++u) {
            const int64_t q = q0 + u;
            if (q < hi && find_slot(dia_off, nd, (int32_t)((int64_t)col_idx[q] - r)) < 0) ++rest;
        }
        const int t = rl_block_sum(rest, s_w);
        if (threadIdx.x == 0) chunk_cnt[g] = t;
    }
}

// Second pass: the remainder entries of chunk g go to rest_ptr[row] + (remainder entries in the row's chunks before
// g) + (those before them inside the chunk), in the order of the row.
template <typename T>
__global__ __launch_bounds__(RL_B) void k_hdc_rest_long_write(const LongRows *__restrict__ lr, int nrows, const int32_t *__restrict__ row_ptr,
                                                              const int32_t *__restrict__ col_idx, const T *__restrict__ val, int64_t m,
                                                              const int32_t *__restrict__ dia_off, int nd,
                                                              const int32_t *__restrict__ chunk_cnt, const int32_t *__restrict__ rest_ptr,
                                                              int32_t *__restrict__ rcol, T *__restrict__ rval)
{
    __shared__ int s_base[LR_CAP + 2];
    __shared__ int s_w[RL_B / WAVE];
    __shared__ int s_scan[RL_B / WAVE];
    rl_chunk_bases(lr, nrows, row_ptr, m, nd, s_base);
    const int total = s_base[nrows];
    for (int g = blockIdx.x; g < total; g += gridDim.x) {
        const int li = rl_row_of_chunk(s_base, nrows, g);
        const int64_t r = lr->rows[li];
        const int64_t lo = row_ptr[r], hi = row_ptr[r + 1];
        int before = 0;
        for (int c = s_base[li] + threadIdx.x; c < g; c += RL_B) before += chunk_cnt[c];
        before = rl_block_sum(before, s_w);
        const int64_t q0 = lo + (int64_t)(g - s_base[li]) * RL_CHUNK + (int64_t)threadIdx.x * RL_U;
        int32_t cc[RL_U];
        bool rest[RL_U];
        int mine = 0;
#pragma unroll
        for (int u = 0; u < RL_U; ++u) {
            const int64_t q = q0 + u;
            cc[u] = q < hi ? col_idx[q] : 0;
            rest[u] = q < hi && find_slot(dia_off, nd, (int32_t)((int64_t)cc[u] - r)) < 0;
            mine += rest[u] ? 1 : 0;
        }
        // exclusive scan of `mine` over the block, in thread order
        int incl = mine;
        for (int o = 1; o < WAVE; o <<= 1) {
            const int t = __shfl_up(incl, o, WAVE);
            if (lane_id() >= o) incl += t;
        }
        if (lane_id() == WAVE - 1) s_scan[threadIdx.x / WAVE] = incl;
        __syncthreads();
        int pos = incl - mine;
        for (int w = 0; w < (int)threadIdx.x / WAVE; ++w) pos += s_scan[w];
        __syncthreads();
        int64_t out = (int64_t)rest_ptr[r] + before + pos;
#pragma unroll
        for (int u = 0; u < RL_U; ++u) {
            if (rest[u]) {
                rcol[out] = cc[u];
                rval[out] = val[q0 + u];
                ++out;
            }
        }
    }
}

// ------------------------------------------------------------------ ELL (and the ELL part of HYB)
// Entries at position s < K go to slot s; entries at s >= K (HYB only) go to the COO part at
// coo_ptr[row] + (s - K).  Slots s in [len, K) receive the padding markers.
template <typename T>
__global__ __launch_bounds__(CB) void k_fill_ell(const int32_t *__restrict__ row_ptr, const int32_t *__restrict__ col_idx,
                                                  const T *__restrict__ val, int64_t m, int64_t K, int64_t ld,
                                                  int32_t *__restrict__ ecol, T *__restrict__ eval,
                                                  const int32_t *__restrict__ coo_ptr, int32_t *__restrict__ crow,
                                                  int32_t *__restrict__ ccol, T *__restrict__ cval, int rw, int skip_len)
{
    const int64_t row = (xcd_block(blockIdx.x, gridDim.x) * (CB / WAVE) + threadIdx.x / WAVE) * rw + lane_id();
    const bool rv = lane_id() < rw && row < m;
    const int64_t lo = row_ptr[row < m ? row : m], hi = row_ptr[row + 1 < m ? row + 1 : m];   // empty run past the last row
    if (lane_id() < rw && row < ld) {
        for (int64_t s = (hi - lo); s < K; ++s) {
            ecol[s * ld + row] = -1;
            eval[s * ld + row] = (T)0;
        }
    }
    __shared__ int32_t s_col[(CB / WAVE) * WCAP];
    __shared__ T s_val[(CB / WAVE) * WCAP];
    const int w = threadIdx.x / WAVE;
    walk_rows_lds<T>(rv, row, lo, hi, col_idx, val, s_col + w * WCAP, s_val + w * WCAP, skip_len,
                     [&](int64_t r, int64_t, int64_t s, int32_t c, T v, bool) {
        if (s < K) {
            ecol[s * ld + r] = c;
            eval[s * ld + r] = v;
        } else {
            const int64_t q = (int64_t)coo_ptr[r] + (s - K);
            crow[q] = (int32_t)r;
            ccol[q] = c;
            cval[q] = v;
        }
    });
}

// The rows that k_fill_ell skipped (longer than VLONG_ROW; listed by the analysis), entry-parallel over the whole grid:
// the same stores, FL_B * FL_U entries of a row per block and step.  One wave alone walks 64 entries per step, which
// for a row of a million entries took 5 ms.
constexpr int FL_B = 256, FL_U = 4, FL_BLOCKS = 512;
template <typename T>
__global__ __launch_bounds__(FL_B) void k_fill_ell_long(const LongRows *__restrict__ lr, int nrows, const int32_t *__restrict__ row_ptr,
                                                        const int32_t *__restrict__ col_idx, const T *__restrict__ val, int64_t m,
                                                        int64_t K, int64_t ld, int32_t *__restrict__ ecol, T *__restrict__ eval,
                                                        const int32_t *__restrict__ coo_ptr, int32_t *__restrict__ crow,
                                                        int32_t *__restrict__ ccol, T *__restrict__ cval)
{
    for (int li = 0; li < nrows; ++li) {
        const int64_t r = lr->rows[li];
        if (r < 0 || r >= m) continue;   // the list was written for this matrix: never taken
        const int64_t lo = row_ptr[r], hi = row_ptr[r + 1];
        for (int64_t q0 = lo + (int64_t)blockIdx.x * (FL_B * FL_U) + threadIdx.x; q0 - threadIdx.x < hi; q0 += (int64_t)gridDim.x * (FL_B * FL_U)) {
            int32_t cc[FL_U];
            T vv[FL_U];
#pragma unroll
            for (int u = 0; u < FL_U; ++u) {
                const int64_t q = q0 + u * FL_B, qc = q < hi ? q : hi - 1;
                cc[u] = ld_stream(col_idx + qc);
                vv[u] = ld_stream(val + qc);
            }
#pragma unroll
            for (int u = 0; u < FL_U; ++u) {
                const int64_t q = q0 + u * FL_B;
                if (q >= hi) continue;
                const int64_t s = q - lo;
                if (s < K) {
                    ecol[s * ld + r] = cc[u];
                    eval[s * ld + r] = vv[u];
                } else {
                    const int64_t p = (int64_t)coo_ptr[r] + (s - K);
                    crow[p] = (int32_t)r;
                    ccol[p] = cc[u];
                    cval[p] = vv[u];
                }
            }
        }
    }
}

// Histogram of row lengths.  Regular matrices put every row on the same counter, and same-address atomics serialise
// in L2, so counts are merged inside the wave (ballot), then inside the block (LDS histogram for lengths below
// LEN_LDS, flushed once per block); a block owns a contiguous run of rows.
constexpr int LEN_LDS = 2048;

// Lengths above cap are counted as cap (the caller needs them only as "at least cap").
__global__ __launch_bounds__(CB) void k_len_hist(const int32_t *__restrict__ row_ptr, int64_t m, int64_t rows_per_block, int cap,
                                                  uint32_t *__restrict__ lhist)
{
    __shared__ uint32_t sh[LEN_LDS];
    for (int i = threadIdx.x; i < LEN_LDS; i += CB) sh[i] = 0u;
    __syncthreads();
    const int lane = lane_id();
    const int64_t row_begin = (int64_t)blockIdx.x * rows_per_block;
    int64_t row_end = row_begin + rows_per_block;
    row_end = row_end < m ? row_end : m;
    for (int64_t base = row_begin; base < row_end; base += CB) {
        const int64_t row = base + threadIdx.x;
        const bool rv = row < row_end;
        int key = rv ? (row_ptr[row + 1] - row_ptr[row]) : -1;
        key = key > cap ? cap : key;
        uint64_t todo = ballot64(rv);
        while (todo) {
            const int leader = __ffsll((unsigned long long)todo) - 1;
            const int lkey = __shfl(key, leader, WAVE);
            const uint64_t same = ballot64(rv && key == lkey) & todo;
            if (lane == leader) {
                if (lkey < LEN_LDS) atomicAdd(&sh[lkey], (uint32_t)__popcll(same));
                else atomicAdd(&lhist[lkey], (uint32_t)__popcll(same));
            }
            todo &= ~same;
        }
    }
    __syncthreads();
    for (int i = threadIdx.x; i < LEN_LDS; i += CB)
        if (sh[i]) atomicAdd(&lhist[i], sh[i]);
}

__global__ __launch_bounds__(CB) void k_surplus(const int32_t *__restrict__ row_ptr, int64_t m, int64_t K, int32_t *__restrict__ cnt)
{
    const int64_t row = (int64_t)blockIdx.x * CB + threadIdx.x;
    if (row >= m) return;
    const int64_t len = row_ptr[row + 1] - row_ptr[row];
    cnt[row] = (int32_t)(len > K ? len - K : 0);
}

// Row pointers of the HDC remainder relative to the first entry of the row's block of `rows` rows (see mo_matrix::hdc_rp16).
__global__ __launch_bounds__(CB) void k_hdc_rp16(const int32_t *__restrict__ rest_ptr, int64_t m, int rows, int32_t *__restrict__ blk,
                                                 uint16_t *__restrict__ rp16)
{
    const int64_t row = (int64_t)blockIdx.x * CB + threadIdx.x;
    if (row > m) return;
    if (row == m) { blk[(m + rows - 1) / rows] = rest_ptr[m]; return; }
    const int64_t b = row / rows;
    const int32_t base = rest_ptr[b * rows];
    if (row == b * rows) blk[b] = base;
    rp16[row] = (uint16_t)(rest_ptr[row] - base);
}

// ------------------------------------------------------------------ HDC remainder
// The entries of a row that are on no kept diagonal are written, in row order, to the CSR part starting at
// rest_ptr[row] (their number per row was counted while the DIA part was filled).  Same staging and the same merge
// against the ascending offset list as the DIA fill, except that here the entries the merge steps over are the
// output; rows without remainder take no part.  A long row is compacted by the whole wave, 64 entries at a time,
// with a ballot prefix so that the order inside the row is kept.
template <typename T, class ColAt, class ValAt>
__device__ __forceinline__ void hdc_rest_row(bool act, int cnt, int need, int64_t row, int64_t base, const int32_t *__restrict__ dia_off,
                                             int nd, int32_t *__restrict__ rcol, T *__restrict__ rval, ColAt col_at, ValAt val_at)
{
    constexpr int32_t NONE = 0x7fffffff;
    int e = 0, done = 0;
    if (!act) need = 0;
    int32_t c = (need > 0 && cnt > 0) ? col_at(0) : 0;
    int32_t cur = (need > 0 && cnt > 0) ? (int32_t)((int64_t)c - row) : NONE;
    for (int d = 0; d < nd; ++d) {
        if (ballot64(done < need) == 0ull) return;            // every row of the wave has its remainder
        const int32_t target = dia_off[d];
        while (done < need && cur <= target) {
            if (cur < target) {
                rcol[base + done] = c;
                rval[base + done] = val_at(e);
                ++done;
            }
            ++e;
            c = e < cnt ? col_at(e) : 0;
            cur = e < cnt ? (int32_t)((int64_t)c - row) : NONE;
        }
    }
    while (done < need) {                                     // entries beyond the last kept diagonal
        rcol[base + done] = c;
        rval[base + done] = val_at(e);
        ++done;
        ++e;
        c = e < cnt ? col_at(e) : 0;
    }
}

// SPARSE: the remainder is a small share of the entries, so only the columns are staged and the few values that leave
// are fetched one by one (staging every value would double the bytes this pass reads).
template <typename T, bool SPARSE>
__global__ __launch_bounds__(CB) void k_hdc_rest(const int32_t *__restrict__ row_ptr, const int32_t *__restrict__ col_idx,
                                                  const T *__restrict__ val, int64_t m,
                                                  const int32_t *__restrict__ dia_off, int nd, const int32_t *__restrict__ rest_ptr,
                                                  int32_t *__restrict__ rcol, T *__restrict__ rval, int rw, int skip_len)
{
    __shared__ int32_t s_col[(CB / WAVE) * WCAP];
    __shared__ T s_val[SPARSE ? 1 : (CB / WAVE) * WCAP];
    const int lane = lane_id();
    int32_t *sc = s_col + (threadIdx.x / WAVE) * WCAP;
    T *sv = s_val + (SPARSE ? 0 : (threadIdx.x / WAVE) * WCAP);
    const int64_t row = (xcd_block(blockIdx.x, gridDim.x) * (CB / WAVE) + threadIdx.x / WAVE) * rw + lane;
    const bool rv = lane < rw && row < m;
    const int lo = row_ptr[row < m ? row : m], hi = row_ptr[row + 1 < m ? row + 1 : m];   // empty run past the last row
    const int len = hi - lo;
    const int64_t base = rest_ptr[row < m ? row : m];
    const int need = rv ? rest_ptr[row + 1 < m ? row + 1 : m] - (int32_t)base : 0;
    if (ballot64(need > 0) == 0ull) return;                   // no remainder in these rows
    const int nvalid = __popcll(ballot64(rv));                // the valid rows of a wave are a prefix of its lanes
    const int wb = __builtin_amdgcn_readfirstlane(lo);
    const int we = nvalid ? __builtin_amdgcn_readlane(hi, nvalid - 1) : wb;
    const int staged = we - wb < WCAP ? we - wb : WCAP;
    if (staged > 0) {
        if constexpr (SPARSE) stage_to_lds(col_idx + wb, sc, staged, lane);
        else stage_pair_to_lds(col_idx + wb, val + wb, sc, sv, staged, lane);
    }
    const bool is_short = rv && len <= SHORT_ROW;
    const bool in_lds = is_short && hi - wb <= staged;
    const int off = in_lds ? lo - wb : 0;
    hdc_rest_row<T>(in_lds, len, need, row, base, dia_off, nd, rcol, rval,
                    [&](int e) { return sc[off + e]; }, [&](int e) { return SPARSE ? val[lo + e] : sv[off + e]; });
    const bool direct = is_short && !in_lds;
    if (ballot64(direct && need > 0) != 0ull)
        hdc_rest_row<T>(direct, len, need, row, base, dia_off, nd, rcol, rval,
                        [&](int e) { return col_idx[lo + e]; }, [&](int e) { return val[lo + e]; });
    // skip_len > 0: rows longer than that (and not merged lane per row by the fill kernel) are left to the chip-wide kernels
    uint64_t longmask = ballot64(rv && len > SHORT_ROW && need > 0 && !(skip_len > 0 && len > skip_len && (int64_t)len > 2 * (int64_t)nd));
    const uint64_t below = (lane == 0) ? 0ull : (~0ull >> (WAVE - lane));
    while (longmask) {
        const int l = __ffsll((unsigned long long)longmask) - 1;
        longmask &= longmask - 1;
        const int64_t r = row - lane + l;
        const int rlo = __builtin_amdgcn_readlane(lo, l), rhi = __builtin_amdgcn_readlane(hi, l);
        const int64_t rbase = __shfl(base, l, WAVE);
        int64_t run = 0;
        for (int q0 = rlo; q0 < rhi; q0 += WAVE) {
            const int q = q0 + lane;
            bool rest = false;
            int32_t c = 0;
            if (q < rhi) {
                c = col_idx[q];
                rest = find_slot(dia_off, nd, (int32_t)((int64_t)c - r)) < 0;
            }
            const uint64_t mask = ballot64(rest);
            if (rest) {
                const int64_t pos = rbase + run + __popcll(mask & below);
                rcol[pos] = c;
                rval[pos] = val[q];
            }
            run += __popcll(mask);
        }
    }
}

// ------------------------------------------------------------------ host side
static unsigned blocks_for(int64_t n) { return (unsigned)((n + CB - 1) / CB > 0 ? (n + CB - 1) / CB : 1); }
// Rows per wave of the fill kernels: as many (64, 32, 16 or 8) as keep the wave's run of entries within one LDS stage
// at the mean row length.  A second stage in the same wave would have to wait until the stores of the first have
// drained (loads and stores share one in-order counter), which cost a third of the bandwidth on the 27-point stencil.
static int rows_per_wave(int64_t m, int64_t nnz)
{
    const double avg = m > 0 ? (double)nnz / (double)m : 0.0;
    int rw = WAVE;
    while (rw > 8 && avg * rw > 0.9 * WCAP) rw >>= 1;
    return rw;
}
static unsigned wave_blocks_for(int64_t rows, int rw)
{
    const int64_t per_block = (int64_t)rw * (CB / WAVE);
    const int64_t g = (rows + per_block - 1) / per_block;
    return (unsigned)(g > 0 ? g : 1);
}
static unsigned fill_grid(int64_t n)
{
    int64_t g = (n + (int64_t)CB * 8 - 1) / ((int64_t)CB * 8);
    if (g < 1) g = 1;
    if (g > 8192) g = 8192;
    return (unsigned)g;
}

mo_status check_csr_args(const mo_csr *a)
{
    if (!a) return MO_E_NULL;
    if (a->dtype != MO_F32 && a->dtype != MO_F64) return MO_E_DTYPE;
    if (a->m < 1 || a->n < 1 || a->nnz < 0) return MO_E_SHAPE;
    if (a->nnz > 2147483647LL || a->m + a->n > 2147483647LL) return MO_E_SHAPE;
    if (!a->row_ptr) return MO_E_NULL;
    if (a->nnz > 0 && (!a->col_idx || !a->val)) return MO_E_NULL;
    return MO_OK;
}

mo_status check_params(const mo_params *in, mo_params *out)
{
    mo_default_params(out);
    if (in) *out = *in;
    if (out->td_den <= 0 || out->hyb_den <= 0 || out->td_num < 0 || out->hyb_num < 0 || out->max_fill < 0 || out->max_slots < 0)
        return MO_E_PARAM;
    return MO_OK;
}

bool slab_feasible(int64_t width, int64_t m, int64_t nnz, const mo_params &p)
{
    const __int128 slots = (__int128)width * (__int128)m;
    if (slots > (__int128)p.max_fill * (__int128)nnz) return false;
    if (slots > (__int128)p.max_slots) return false;
    return true;
}

namespace {

struct Builder {
    mo_matrix *h;
    hipStream_t s;
    bool failed = false;
    std::vector<std::vector<int32_t>> keep;   // host arrays that asynchronous uploads still read: alive until the end
    Builder(hipStream_t st) : h(new (std::nothrow) mo_matrix()), s(st) { if (h) h->home = st; }
    ~Builder()
    {
        if (!keep.empty()) (void)hipStreamSynchronize(s);   // a no-op after the conversion's final synchronisation
        if (h) release();
    }
    void *own(size_t bytes)
    {
        void *p = dev_alloc(bytes, s);
        if (!p) { failed = true; return nullptr; }
        h->owned.push_back(p);
        return p;
    }
    void release()
    {
        for (mo_matrix *part : h->csr_slices) mo_matrix_free(part);
        for (void *p : h->owned) dev_free(p, s);
        delete h;
        h = nullptr;
    }
    mo_matrix *take() { mo_matrix *r = h; h = nullptr; return r; }
};

// Launch plan of a CSR part (MO_CSR itself, or the remainder of HDC).
mo_status plan_csr(Builder &b, const int32_t *row_ptr, int64_t m, int64_t nnz, int64_t max_row)
{
    mo_matrix *h = b.h;
    h->csr_max_row = max_row;
    const double avg = m > 0 ? (double)nnz / (double)m : 0.0;
    // Large tiles amortise what a block pays once (header, barrier, the wait for its y stores) over more entries, as long
    // as several blocks still fit a CU's LDS: measured on the 27-point stencil (fp64, 27 per row) 128 us with 4096-entry
    // tiles against 135 us with 2048, on the band matrix (9 per row) 106 against 108 us in fp64 and 76 against 74 us in fp32.
    int tile = nnz < CSR_SMALL_NNZ ? CSR_TILE_SMALL : CSR_TILE;
    if (tile == CSR_TILE && max_row <= CSR_MAX_ROW && (dtype_size(h->dtype) == 4 || avg >= 16.0)) tile = CSR_TILE_LARGE;
    h->csr_tile = tile;
    // lanes per row: the rows of one tile (about tile / avg) should fit one pass of 256 / g rows
    int g = 1;
    while (g < 16 && avg > (10.0 * tile / CSR_TILE) * g) g <<= 1;
    h->csr_group = g;
    h->csr_tiles = csr_tile_count(nnz, tile);
    h->csr_split = max_row > CSR_MAX_ROW ? 1 : 0;
    // Rows per cache line of y (16 in fp64, 32 in fp32): tiles of the row-owning kernel begin on such a row when the
    // rows this adds to a tile cannot overflow its slack.  Tiles that cut rows (csr_split) are defined by entry
    // positions alone.
    int row_align = 1;
    if (!h->csr_split) {
        const int64_t line_rows = 128 / (int64_t)dtype_size(h->dtype);
        while (row_align < line_rows && (int64_t)row_align * 2 * (max_row > 0 ? max_row : 1) <= CSR_TILE_SLACK) row_align <<= 1;
    }
    {
        h->csr_tile_rp = (int32_t *)b.own((size_t)(h->csr_tiles + 1) * 8);
        if (h->csr_split) {
            h->csr_carry_row = (int32_t *)b.own((size_t)h->csr_tiles * 4);
            h->csr_carry_val = b.own((size_t)h->csr_tiles * dtype_size(h->dtype));
        }
        if (b.failed) return MO_E_ALLOC;
        MO_TRY(csr_build_tiles(row_ptr, m, nnz, h->csr_tiles, tile, row_align, h->csr_tile_rp, b.s));
    }
    return MO_OK;
}

// ------------------------------------------------------------------ column slices of a CSR matrix
// Columns ascend inside a row and rows follow each other, so the entries with lo <= col < hi, taken in storage order,
// are the CSR arrays of that column slice of the matrix: a stable selection from the entry array.  Per slice: flag ->
// exclusive scan -> scatter; the row pointers of the slice are the scanned flags read at the row starts.
__global__ __launch_bounds__(CB) void k_slice_flags(const int32_t *__restrict__ col_idx, int64_t nnz, int32_t lo, int32_t hi, int32_t *__restrict__ flag)
{
    const int64_t stride = (int64_t)gridDim.x * CB;
    for (int64_t p = (int64_t)blockIdx.x * CB + threadIdx.x; p < nnz; p += stride) {
        const int32_t c = ld_stream(col_idx + p);
        flag[p] = (c >= lo && c < hi) ? 1 : 0;
    }
}

template <typename T>
__global__ __launch_bounds__(CB) void k_slice_scatter(const int32_t *__restrict__ col_idx, const T *__restrict__ val, int64_t nnz, int32_t lo,
                                                       int32_t hi, const int32_t *__restrict__ before, int32_t *__restrict__ col_s,
                                                       T *__restrict__ val_s)
{
    const int64_t stride = (int64_t)gridDim.x * CB;
    for (int64_t p = (int64_t)blockIdx.x * CB + threadIdx.x; p < nnz; p += stride) {
        const int32_t c = ld_stream(col_idx + p);
        if (c >= lo && c < hi) {
            const int32_t d = before[p];
            col_s[d] = c;
            val_s[d] = ld_stream(val + p);
        }
    }
}

__global__ __launch_bounds__(CB) void k_slice_row_ptr(const int32_t *__restrict__ row_ptr, int64_t m, const int32_t *__restrict__ before,
                                                       int32_t *__restrict__ rp_s)
{
    const int64_t r = (int64_t)blockIdx.x * CB + threadIdx.x;
    if (r > m) return;
    rp_s[r] = before[row_ptr[r]];   // `before` has nnz + 1 entries
}

mo_status plan_csr(Builder &b, const int32_t *row_ptr, int64_t m, int64_t nnz, int64_t max_row);

template <typename T>
mo_status build_csr_slices(const mo_csr &a, int nslices, int64_t max_row, Builder &parent, Scratch &scr)
{
    hipStream_t s = parent.s;
    int32_t *flag = (int32_t *)scr.get((size_t)a.nnz * 4);
    int32_t *before = (int32_t *)scr.get((size_t)(a.nnz + 1) * 4);
    void *tmp = scr.get(scan_tmp_bytes(a.nnz));
    if (!flag || !before || !tmp) return MO_E_ALLOC;
    const unsigned g = fill_grid(a.nnz);
    const int64_t width = (a.n + nslices - 1) / nslices;
    for (int q = 0; q < nslices; ++q) {
        const int32_t lo = (int32_t)(q * width), hi = (int32_t)((q + 1) * width < a.n ? (q + 1) * width : a.n);
        hipLaunchKernelGGL(k_slice_flags, dim3(g), dim3(CB), 0, s, a.col_idx, a.nnz, lo, hi, flag);
        MO_LAUNCH_CHECK();
        MO_TRY(exclusive_scan_i32(flag, before, a.nnz, tmp, s));
        int32_t cnt = 0;
        MO_HIP(hipMemcpyAsync(&cnt, before + a.nnz, 4, hipMemcpyDeviceToHost, s));
        MO_HIP(hipStreamSynchronize(s));
        Builder part(s);
        if (!part.h) return MO_E_ALLOC;
        mo_matrix *h = part.h;
        h->fmt = MO_CSR; h->dtype = a.dtype; h->m = a.m; h->n = a.n; h->nnz = cnt; h->nnz_csr = cnt;
        h->ld = (a.m + 63) & ~(int64_t)63;
        int32_t *rp = (int32_t *)part.own((size_t)(a.m + 1) * 4);
        int32_t *col = (int32_t *)part.own((size_t)(cnt > 0 ? cnt : 1) * 4);
        T *val = (T *)part.own((size_t)(cnt > 0 ? cnt : 1) * sizeof(T));
        if (part.failed) return MO_E_ALLOC;
        h->csr_row_ptr = rp; h->csr_col = col; h->csr_val = val;
        hipLaunchKernelGGL(k_slice_scatter<T>, dim3(g), dim3(CB), 0, s, a.col_idx, (const T *)a.val, a.nnz, lo, hi, before, col, val);
        MO_LAUNCH_CHECK();
        hipLaunchKernelGGL(k_slice_row_ptr, dim3(blocks_for(a.m + 1)), dim3(CB), 0, s, a.row_ptr, a.m, before, rp);
        MO_LAUNCH_CHECK();
        MO_TRY(plan_csr(part, rp, a.m, cnt, max_row));
        MO_HIP(hipStreamSynchronize(s));   // `flag` and `before` are rewritten for the next slice
        parent.h->csr_slices.push_back(part.take());
    }
    return MO_OK;
}

// DIA part: the kept offsets, ascending, into h->dia_off; the slab filled; the launch plan of the SpMV kernel.
template <typename T>
mo_status build_dia_part(const mo_csr &a, const mo_params &p, const Analysis &an, bool all_nonempty, int64_t nd,
                         Builder &b, Scratch &scr, int32_t *rest_cnt = nullptr)
{
    hipStream_t s = b.s;
    const int64_t ndiag = a.m + a.n - 1;
    mo_matrix *h = b.h;
    h->nd = nd;
    h->dia_off = (int32_t *)b.own((size_t)(nd > 0 ? nd : 1) * 4);
    h->dia_val = b.own((size_t)(nd > 0 ? nd : 1) * (size_t)h->ld * sizeof(T));
    if (b.failed) return MO_E_ALLOC;
    if (nd > 0) {
        int32_t *count = (int32_t *)scr.get(256);
        if (!count) return MO_E_ALLOC;
        hipLaunchKernelGGL(k_fill_i32, dim3(1), dim3(CB), 0, s, count, (int64_t)1, 0);
        MO_LAUNCH_CHECK();
        const int64_t mn = a.m < a.n ? a.m : a.n;
        hipLaunchKernelGGL(k_collect_diag, dim3(fill_grid(ndiag)), dim3(CB), 0, s, an.hist, ndiag, all_nonempty ? 1 : 0,
                           (unsigned long long)mn * (unsigned long long)p.td_num, (unsigned long long)p.td_den, a.m, count,
                           h->dia_off, (int32_t)nd);
        MO_LAUNCH_CHECK();
        b.keep.emplace_back((size_t)nd);
        std::vector<int32_t> &hoff = b.keep.back();   // stays alive until the conversion's final synchronisation
        MO_HIP(hipMemcpyAsync(hoff.data(), h->dia_off, (size_t)nd * 4, hipMemcpyDeviceToHost, s));
        MO_HIP(hipStreamSynchronize(s));
        std::sort(hoff.begin(), hoff.end());
        MO_HIP(hipMemcpyAsync(h->dia_off, hoff.data(), (size_t)nd * 4, hipMemcpyHostToDevice, s));
        const int rw = rows_per_wave(a.m, a.nnz);
        hipLaunchKernelGGL(k_fill_dia<T>, dim3(wave_blocks_for(h->ld, rw)), dim3(CB), 0, s, a.row_ptr, a.col_idx, (const T *)a.val, a.m,
                           h->dia_off, (int)nd, h->ld, (T *)h->dia_val, rest_cnt, rw, an.n_long > 0 ? (int)VLONG_ROW : 0);
        MO_LAUNCH_CHECK();
        if (an.n_long > 0) {   // rows too long for one wave: their entries, chip-wide
            hipLaunchKernelGGL(k_fill_dia_long<T>, dim3(RL_BLOCKS), dim3(RL_B), 0, s, an.long_rows, an.n_long, a.row_ptr, a.col_idx,
                               (const T *)a.val, a.m, h->dia_off, (int)nd, h->ld, (T *)h->dia_val, rest_cnt);
            MO_LAUNCH_CHECK();
        }
    } else if (rest_cnt) {   // no diagonal is kept: every entry is remainder
        hipLaunchKernelGGL(k_surplus, dim3(blocks_for(a.m)), dim3(CB), 0, s, a.row_ptr, a.m, (int64_t)0, rest_cnt);
        MO_LAUNCH_CHECK();
    }
    // launch plans for the LDS-staged kernels, from the offsets the host already holds; the four arrays go to the device
    // as one block with one copy
    if (nd > 0) {
        const std::vector<int32_t> hoff = b.keep.back();
        // SpMV: 512 threads per block, one row per lane in fp64 and two in fp32 (8 bytes per lane and load either way):
        // measured best of {256, 512} x {1, 2} on the stencil and band configurations.  Matrices of fewer than 2^17
        // rows get 256-thread blocks: twice as many, shorter blocks on a chip they cannot fill anyway.
        const int block = a.m < 131072 ? 256 : 512, rows = DIA_ROWS_PER_LANE<T>;
        std::vector<int32_t> xpos, cl, mxpos, mcl, mmap;
        int64_t elems = 0, melems = 0;
        const bool have_v = plan_dia_clusters(hoff, block * rows, DIA_LDS_BYTES / (int64_t)sizeof(T), &xpos, &cl, &elems);
        // the multi-vector product: blocks of SPMM_ROWS rows; kept when a 16-byte piece per row of X fits
        const bool have_m = plan_dia_clusters(hoff, SPMM_ROWS, SPMM_WIN_BYTES / 16, &mxpos, &mcl, &melems);
        if (have_m) {
            // Every window is at least SPMM_ROWS long, so a run of SPMM_ROWS staged rows lies in at most two windows.
            const int64_t nrun = (melems + SPMM_ROWS - 1) / SPMM_ROWS;
            mmap.resize((size_t)nrun * 3);
            for (int64_t u = 0; u < nrun; ++u) {
                size_t q = 0;   // window that holds staged row u * SPMM_ROWS
                while (q + 5 < mcl.size() && (int64_t)mcl[q + 5] <= u * SPMM_ROWS) q += 3;
                const bool more = q + 5 < mcl.size();
                mmap[3 * u] = more ? mcl[q + 5] : (int32_t)melems;
                mmap[3 * u + 1] = mcl[q] - mcl[q + 2];
                mmap[3 * u + 2] = more ? mcl[q + 3] - mcl[q + 5] : 0;
            }
        }
        if (have_v || have_m) {
            b.keep.emplace_back();
            std::vector<int32_t> &all = b.keep.back();   // alive until the conversion's final synchronisation
            const size_t o_xpos = 0, o_cl = o_xpos + (have_v ? xpos.size() : 0), o_mx = o_cl + (have_v ? cl.size() : 0),
                         o_map = o_mx + (have_m ? mxpos.size() : 0), total = o_map + (have_m ? mmap.size() : 0);
            all.reserve(total);
            if (have_v) { all.insert(all.end(), xpos.begin(), xpos.end()); all.insert(all.end(), cl.begin(), cl.end()); }
            if (have_m) { all.insert(all.end(), mxpos.begin(), mxpos.end()); all.insert(all.end(), mmap.begin(), mmap.end()); }
            int32_t *dev = (int32_t *)b.own(total * 4);
            if (b.failed) return MO_E_ALLOC;
            MO_HIP(hipMemcpyAsync(dev, all.data(), total * 4, hipMemcpyHostToDevice, s));
            if (have_v) {
                h->dia_xpos = dev + o_xpos;
                h->dia_clusters = dev + o_cl;
                h->dia_block = block;
                h->dia_rows = rows;
                h->dia_ncl = (int32_t)(cl.size() / 3);
                h->dia_lds_elems = elems;
                // large matrices with few diagonals: the batched kernel, whose plan travels in the kernel arguments
                if (a.m >= DIA_BATCH_MIN_ROWS && block == DIA_BATCH_BLOCK && nd <= DIA_PRE && elems <= (int64_t)DIA_MAX_RUNS * block) {
                    DiaPlan &pl = h->dia_plan;
                    std::vector<int32_t> wlo, wlen;
                    for (size_t q = 0; q < cl.size(); q += 3) { wlo.push_back(cl[q]); wlen.push_back(cl[q + 1]); }
                    if (plan_window_runs(wlo.data(), wlen.data(), (int)wlo.size(), block, &pl.win)) {
                        for (size_t k = 0; k < xpos.size(); ++k) pl.xpos[k] = xpos[k];
                        h->dia_batch = true;
                    }
                }
            }
            if (have_m) {
                h->mm_xpos = dev + o_mx;
                h->mm_map = dev + o_map;
                h->mm_lds_elems = melems;
            }
        }
    }
    return MO_OK;
}

void setup_coo_tiles(Builder &b, size_t sv)
{
    mo_matrix *h = b.h;
    // Entries per thread: 8 for large parts (2048-entry tiles: 157 against 163 us on the 27-point stencil, 129 against
    // 132 us on the band matrix), 4 below COO_SMALL_NNZ entries (more blocks for a chip that a small part cannot fill), 2
    // for the small scattered COO part of a HYB matrix, whose SpMV read-modify-writes y (measured 148 vs 165 us on the
    // banded+scatter matrix).
    h->coo_strip = h->nnz_coo >= COO_SMALL_NNZ ? 8 : (h->fmt == MO_HYB ? 2 : 4);
    const int64_t tile = (int64_t)COO_B_THREADS * h->coo_strip;
    h->coo_tiles = (h->nnz_coo + tile - 1) / tile;
    const int64_t t = h->coo_tiles > 0 ? h->coo_tiles : 1;
    h->coo_carry_row = (int32_t *)b.own((size_t)t * 4);
    h->coo_carry_val = b.own((size_t)t * sv);
}

// Leading dimension of the DIA / ELL slabs: M rounded up to whole groups of 64 rows; when that makes consecutive slabs
// lie a multiple of 64 KB apart (a matrix whose row count is a power of two, say), 576 rows more.  A row block reads
// the same rows of every slab at once, and with slabs a large power of two apart those reads fall on the same memory
// channels: measured with 2^21 rows x 27 diagonals 77.5 us as it is and 75.8 us with the extra rows, with 2^22 rows x 9
// diagonals 75.0 / 73.4 us (fp32 47.1 / 46.0 us); 128 .. 2368 extra rows all help, 576 most evenly.
static int64_t slab_ld(int64_t m, size_t sv)
{
    int64_t ld = (m + 63) & ~(int64_t)63;
    if (ld > 0 && (ld * (int64_t)sv) % 65536 == 0) ld += 576;
    return ld;
}

template <typename T>
mo_status convert_typed(const mo_csr &a, mo_format fmt, const mo_params &p, const Analysis &an, mo_matrix **out, hipStream_t s)
{
    Builder b(s);
    if (!b.h) return MO_E_ALLOC;
    mo_matrix *h = b.h;
    Scratch scr(s);
    h->fmt = fmt; h->dtype = a.dtype; h->m = a.m; h->n = a.n; h->nnz = a.nnz;
    h->ld = slab_ld(a.m, sizeof(T));
    const T *aval = (const T *)a.val;
    const unsigned row_blocks = blocks_for(a.m);

    switch (fmt) {
    case MO_CSR: {
        h->csr_row_ptr = a.row_ptr; h->csr_col = a.col_idx; h->csr_val = a.val; h->nnz_csr = a.nnz;
        MO_TRY(plan_csr(b, a.row_ptr, a.m, a.nnz, an.max_row));
        MO_TRY(plan_x_windows(a.row_ptr, a.col_idx, a.m, a.nnz, &h->xplan, s));
        // Scattered columns (no populated diagonals) and an x that one XCD's L2 cannot hold: the gathers of such a
        // matrix miss L2 most of the time and every miss moves a 128-byte line.  Passes over column slices of at most
        // 5 MB keep each pass's part of x in L2.  Measured (separate launches per slice): lognormal configuration, x =
        // 8 MB: 185 us in one pass, 135 in two, 147 in four, 171 in eight (the per-pass row pointers and y traffic
        // grow); 3.8 M rows, 106 M entries, x = 31 MB: 1725 us in one pass, 1082 in four, 819 in eight, 982 in
        // sixteen; 1.6 M rows of 54 entries, x = 12.5 MB: 1071 us in one pass, 553 in four, 580 in eight.
        {
            const int64_t xb = a.n * (int64_t)sizeof(T);
            // every pass re-reads the row pointers and y: worth it only when the rows are long enough for the size of
            // x (over the sweep's 189 scattered matrices above 5 MB of x the passes win from about 64 MB x entries per
            // row on, by up to 2.3x, and lose up to 13 % below)
            const bool long_rows = (__int128)a.nnz * (__int128)xb >= (__int128)CSR_SLICE_MIN_WORK * (__int128)a.m;
            if (h->xplan.ncl == 0 && xb >= CSR_SLICE_MIN_X_BYTES && a.nnz >= CSR_SLICE_MIN_NNZ && long_rows) {
                int nslices = 2;
                while (nslices < CSR_MAX_SLICES && xb > (int64_t)nslices * CSR_SLICE_X_BYTES) nslices <<= 1;
                MO_TRY(build_csr_slices<T>(a, nslices, an.max_row, b, scr));
            }
        }
        break;
    }
    case MO_COO: {
        h->nnz_coo = a.nnz;
        const size_t e = (size_t)(a.nnz > 0 ? a.nnz : 1);
        h->coo_row = (int32_t *)b.own(e * 4);
        h->coo_col = (int32_t *)b.own(e * 4);
        h->coo_val = b.own(e * sizeof(T));
        int32_t *rp_copy = (int32_t *)b.own((size_t)(a.m + 1) * 4);
        setup_coo_tiles(b, sizeof(T));
        h->coo_every_row = an.min_row >= 1;
        if (b.failed) return MO_E_ALLOC;
        MO_HIP(hipMemcpyAsync(rp_copy, a.row_ptr, (size_t)(a.m + 1) * 4, hipMemcpyDeviceToDevice, s));
        h->coo_rp = rp_copy;
        if (a.nnz > 0) {
            hipLaunchKernelGGL(k_csr_to_coo<T>, dim3((unsigned)((a.nnz + COO_CT - 1) / COO_CT)), dim3(CB), 0, s, a.row_ptr, a.col_idx, aval,
                               a.m, a.nnz, h->coo_row, h->coo_col, (T *)h->coo_val);
            MO_LAUNCH_CHECK();
        }
        break;
    }
    case MO_DIA: {
        if (!slab_feasible(an.n_diag, a.m, a.nnz, p)) return MO_E_FILL;
        MO_TRY(build_dia_part<T>(a, p, an, true, an.n_diag, b, scr));
        break;
    }
    case MO_ELL:
    case MO_HYB: {
        int64_t K = an.max_row;
        int32_t *coo_ptr = nullptr;
        if (fmt == MO_ELL) {
            if (!slab_feasible(K, a.m, a.nnz, p)) return MO_E_FILL;
        } else {
            // K_H from the histogram of row lengths: largest k with #{len >= k} * den >= m * num.  Since #{len >= k} * k
            // <= nnz, no k above nnz * den / (m * num) qualifies, so longer rows share the last counter: a matrix with one
            // row of a million entries does not send a million counters to the host.
            int64_t cap = an.max_row;
            if (p.hyb_num > 0) {
                const __int128 bound = (__int128)a.nnz * (__int128)p.hyb_den / ((__int128)a.m * (__int128)p.hyb_num) + 1;
                if (bound < (__int128)cap) cap = (int64_t)bound;
            }
            const int64_t nh = cap + 1;
            uint32_t *lhist = (uint32_t *)scr.get((size_t)nh * 4);
            if (!lhist) return MO_E_ALLOC;
            hipLaunchKernelGGL(k_fill_i32, dim3(fill_grid(nh)), dim3(CB), 0, s, (int32_t *)lhist, nh, 0);
            MO_LAUNCH_CHECK();
            int64_t rpb = (a.m + 1023) / 1024;                 // at most 1024 blocks, each a multiple of the block size
            rpb = ((rpb + CB - 1) / CB) * CB;
            hipLaunchKernelGGL(k_len_hist, dim3((unsigned)((a.m + rpb - 1) / rpb)), dim3(CB), 0, s, a.row_ptr, a.m, rpb, (int)cap, lhist);
            MO_LAUNCH_CHECK();
            std::vector<uint32_t> hh((size_t)nh);
            MO_HIP(hipMemcpyAsync(hh.data(), lhist, (size_t)nh * 4, hipMemcpyDeviceToHost, s));
            MO_HIP(hipStreamSynchronize(s));
            const __int128 need = (__int128)a.m * (__int128)p.hyb_num;
            int64_t rows_ge = 0;   // rows with len >= k, walking k downwards
            K = 0;
            for (int64_t k = cap; k >= 1; --k) {
                rows_ge += hh[(size_t)k];
                if ((__int128)rows_ge * (__int128)p.hyb_den >= need) { K = k; break; }
            }
            // entries beyond slot K: all entries minus min(len, K) per row (rows counted at cap are longer than K, or
            // cap is the longest row)
            int64_t kept = 0;
            for (int64_t len = 1; len <= cap; ++len) kept += (int64_t)hh[(size_t)len] * (len < K ? len : K);
            const int64_t surplus = a.nnz - kept;
            h->nnz_coo = surplus;
            h->hyb_max_surplus = an.max_row > K ? an.max_row - K : 0;
            const size_t e = (size_t)(surplus > 0 ? surplus : 1);
            h->coo_row = (int32_t *)b.own(e * 4);
            h->coo_col = (int32_t *)b.own(e * 4);
            h->coo_val = b.own(e * sizeof(T));
            setup_coo_tiles(b, sizeof(T));
            int32_t *cnt = (int32_t *)scr.get((size_t)a.m * 4);
            coo_ptr = (int32_t *)b.own((size_t)(a.m + 1) * 4);   // kept: start of each row's run in the COO part
            h->coo_rp = coo_ptr;
            void *tmp = scr.get(scan_tmp_bytes(a.m));
            if (b.failed || !cnt || !coo_ptr || !tmp) return MO_E_ALLOC;
            hipLaunchKernelGGL(k_surplus, dim3(row_blocks), dim3(CB), 0, s, a.row_ptr, a.m, K, cnt);
            MO_LAUNCH_CHECK();
            MO_TRY(exclusive_scan_i32(cnt, coo_ptr, a.m, tmp, s));
        }
        h->k = K;
        const size_t slots = (size_t)(K > 0 ? K : 1) * (size_t)h->ld;
        h->ell_col = (int32_t *)b.own(slots * 4);
        h->ell_val = b.own(slots * sizeof(T));
        if (b.failed) return MO_E_ALLOC;
        const int rw = rows_per_wave(a.m, a.nnz);
        hipLaunchKernelGGL(k_fill_ell<T>, dim3(wave_blocks_for(h->ld, rw)), dim3(CB), 0, s, a.row_ptr, a.col_idx, aval, a.m, K, h->ld,
                           h->ell_col, (T *)h->ell_val, coo_ptr, h->coo_row, h->coo_col, (T *)h->coo_val, rw,
                           an.n_long > 0 ? (int)VLONG_ROW : 0);
        MO_LAUNCH_CHECK();
        if (an.n_long > 0) {
            hipLaunchKernelGGL(k_fill_ell_long<T>, dim3(FL_BLOCKS), dim3(FL_B), 0, s, an.long_rows, an.n_long, a.row_ptr, a.col_idx, aval, a.m,
                               K, h->ld, h->ell_col, (T *)h->ell_val, coo_ptr, h->coo_row, h->coo_col, (T *)h->coo_val);
            MO_LAUNCH_CHECK();
        }
        MO_TRY(plan_x_windows(a.row_ptr, a.col_idx, a.m, a.nnz, &h->xplan, s));
        break;
    }
    case MO_HDC: {
        int32_t *cnt = (int32_t *)scr.get((size_t)a.m * 4);
        int32_t *rest_ptr = (int32_t *)b.own((size_t)(a.m + 1) * 4);
        void *tmp = scr.get(scan_tmp_bytes(a.m));
        if (b.failed || !cnt || !tmp) return MO_E_ALLOC;
        MO_TRY(build_dia_part<T>(a, p, an, false, an.n_true, b, scr, cnt));   // also counts the remainder per row
        MO_TRY(exclusive_scan_i32(cnt, rest_ptr, a.m, tmp, s));
        int32_t total = 0;
        MO_HIP(hipMemcpyAsync(&total, rest_ptr + a.m, 4, hipMemcpyDeviceToHost, s));
        MO_HIP(hipStreamSynchronize(s));
        h->nnz_csr = total;
        const size_t e = (size_t)(total > 0 ? total : 1);
        int32_t *rcol = (int32_t *)b.own(e * 4);
        T *rval = (T *)b.own(e * sizeof(T));
        if (b.failed) return MO_E_ALLOC;
        if (total > 0 && h->nd == 0) {   // no diagonal is kept: the remainder is the matrix itself
            MO_HIP(hipMemcpyAsync(rcol, a.col_idx, (size_t)total * 4, hipMemcpyDeviceToDevice, s));
            MO_HIP(hipMemcpyAsync(rval, aval, (size_t)total * sizeof(T), hipMemcpyDeviceToDevice, s));
        } else if (total > 0) {
            const int rw = rows_per_wave(a.m, a.nnz);
            const int skip_len = an.n_long > 0 ? (int)VLONG_ROW : 0;
            if ((int64_t)total * 4 < a.nnz)
                hipLaunchKernelGGL((k_hdc_rest<T, true>), dim3(wave_blocks_for(a.m, rw)), dim3(CB), 0, s, a.row_ptr, a.col_idx, aval, a.m,
                               h->dia_off, (int)h->nd, rest_ptr, rcol, rval, rw, skip_len);
            else
                hipLaunchKernelGGL((k_hdc_rest<T, false>), dim3(wave_blocks_for(a.m, rw)), dim3(CB), 0, s, a.row_ptr, a.col_idx, aval, a.m,
                               h->dia_off, (int)h->nd, rest_ptr, rcol, rval, rw, skip_len);
            MO_LAUNCH_CHECK();
            if (an.n_long > 0) {   // rows too long for one wave: count per chunk, then write in the order of the row
                int32_t *chunk_cnt = (int32_t *)scr.get((size_t)(a.nnz / RL_CHUNK + an.n_long + 1) * 4);
                if (!chunk_cnt) return MO_E_ALLOC;
                hipLaunchKernelGGL(k_hdc_rest_long_count, dim3(RL_BLOCKS), dim3(RL_B), 0, s, an.long_rows, an.n_long, a.row_ptr, a.col_idx,
                                   a.m, h->dia_off, (int)h->nd, chunk_cnt);
                MO_LAUNCH_CHECK();
                hipLaunchKernelGGL(k_hdc_rest_long_write<T>, dim3(RL_BLOCKS), dim3(RL_B), 0, s, an.long_rows, an.n_long, a.row_ptr, a.col_idx,
                                   aval, a.m, h->dia_off, (int)h->nd, chunk_cnt, rest_ptr, rcol, rval);
                MO_LAUNCH_CHECK();
            }
        }
        h->csr_row_ptr = rest_ptr; h->csr_col = rcol; h->csr_val = rval;
        MO_TRY(plan_csr(b, rest_ptr, a.m, total, an.max_row));
        if (total > 0 && h->dia_batch && an.max_row <= HDC_FUSED_MAX_ROW) {
            // a block of the fused kernel holds at most 1024 rows of at most 64 entries: offsets inside it fit 16 bits
            static_assert(1023 * HDC_FUSED_MAX_ROW <= 65535, "remainder offsets inside a row block");
            const int rows = h->dia_block * h->dia_rows;
            h->hdc_blk = (int32_t *)b.own((size_t)((a.m + rows - 1) / rows + 1) * 4);
            h->hdc_rp16 = (uint16_t *)b.own((size_t)a.m * 2);
            if (b.failed) return MO_E_ALLOC;
            hipLaunchKernelGGL(k_hdc_rp16, dim3(blocks_for(a.m + 1)), dim3(CB), 0, s, rest_ptr, a.m, rows, h->hdc_blk, h->hdc_rp16);
            MO_LAUNCH_CHECK();
        }
        break;
    }
    default:
        return MO_E_FORMAT;
    }
    // scratch is released after the kernels that use it: the allocator contract is stream-ordered
    MO_HIP(hipStreamSynchronize(s));
    *out = b.take();
    return MO_OK;
}

}  // namespace

mo_status convert_impl(const mo_csr &a, mo_format fmt, const mo_params &p, const Analysis &an, mo_matrix **out, hipStream_t s)
{
    if (a.dtype == MO_F32) return convert_typed<float>(a, fmt, p, an, out, s);
    return convert_typed<double>(a, fmt, p, an, out, s);
}

}  // namespace mo

// Pieces shared by the feature kernels over CSR (features.hip) and over the other formats (switch.hip): the
// counter block read back by the host, the block-level LDS hash table that merges diagonal counts before they reach
// global memory, and the final count of non-empty / true diagonals.
#pragma once

#include "dev_common.hpp"

namespace mo {

struct Counters {
    unsigned long long max_row, min_row, sum_sq, n_diag, n_true;
    unsigned int err;
    unsigned int pad;
};

// Non-empty and true diagonals one block counted (no atomics: whoever reads the results adds them up).
struct DiagPart {
    unsigned long long n_diag, n_true;
};

// Rows that are too long for one wave (one row of a million entries, walked 64 entries at a time, costs a hundred
// SpMVs) are not walked where they are met: the traversal notes them here and a kernel of its own spreads their
// entries over the whole chip (k_long_rows in features.hip).  count may exceed LR_CAP (rows beyond it are walked in
// place after all); count and done are zero between calls (the kernel's last block clears them).
constexpr int VLONG_ROW = 8192;
constexpr int LR_CAP = 1022;
struct LongRows {
    uint32_t count, done;
    int32_t rows[LR_CAP];
};

constexpr int FB = 256;        // threads per block
constexpr int SHORT_ROW = 32;  // entries of a row handled lane-per-row; the rest is walked by the whole wave

static __global__ void k_init_counters(Counters *c)
{
    if (threadIdx.x == 0 && blockIdx.x == 0) {
        c->max_row = 0ull; c->min_row = ~0ull; c->sum_sq = 0ull; c->n_diag = 0ull; c->n_true = 0ull; c->err = 0u; c->pad = 0u;
    }
}

static __global__ void k_fill_u32(uint32_t *p, int64_t n, uint32_t v)
{
    int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    for (; i < n; i += stride) p[i] = v;
}

// p[0, n) = 0, q[0, nq) = 0 (q may be nullptr) and the counter block reset (the counters and the rest of the 256 bytes
// they own, which callers use for flags that come back with them), in one launch of at least 64 threads.
static __global__ void k_zero_and_reset(uint32_t *p, int64_t n, Counters *c, uint32_t *q, int nq)
{
    int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    if (i == 0) { c->max_row = 0ull; c->min_row = ~0ull; c->sum_sq = 0ull; c->n_diag = 0ull; c->n_true = 0ull; c->err = 0u; c->pad = 0u; }
    if (i >= (int64_t)(sizeof(Counters) / 4) && i < 64) reinterpret_cast<uint32_t *>(c)[i] = 0u;   // the rest of the counters' 256 bytes
    if (q)
        for (int64_t j = i; j < nq; j += stride) q[j] = 0u;
    for (; i < n; i += stride) p[i] = 0u;
}

constexpr int HT_SIZE = 2048;     // LDS table slots (power of two)
constexpr int HT_PROBES = 4;
constexpr int MERGE_ROUNDS = 4;
constexpr int FCAP = 1024;        // entries a wave stages in LDS at a time

__device__ __forceinline__ void count_key(int key, uint32_t n, int *ht_key, uint32_t *ht_cnt, int *ht_full, uint32_t *__restrict__ hist)
{
    const uint32_t h = ((uint32_t)key * 2654435761u) >> 21;   // 11 bits
    // once the table has overflowed, single counts of keys it does not hold skip it: they are almost surely keys
    // that do not repeat.  Keys it holds still go to LDS: a frequent diagonal must not turn into a stream of
    // same-address global atomics.
    if (n == 1u && *ht_full) {
        for (int p = 0; p < HT_PROBES; ++p) {
            const int s = (int)((h + p) & (HT_SIZE - 1));
            if (ht_key[s] == key) { atomicAdd(&ht_cnt[s], 1u); return; }
        }
        atomicAdd(&hist[key], 1u);
        return;
    }
    for (int p = 0; p < HT_PROBES; ++p) {
        const int s = (int)((h + p) & (HT_SIZE - 1));
        const int old = atomicCAS(&ht_key[s], -1, key);
        if (old == -1 || old == key) { atomicAdd(&ht_cnt[s], n); return; }
    }
    *ht_full = 1;
    atomicAdd(&hist[key], n);
}

// N_D = diagonals with at least one entry; N_TD = non-empty diagonals with cnt * td_den >= min(m, n) * td_num.
// skip, skip2 (or nullptr): device words that a kernel ahead in the stream may have set; when either is non-zero this
// kernel does nothing (its caller then counts in another way, or once more later).
static __global__ __launch_bounds__(FB) void k_diag_count(const uint32_t *__restrict__ hist, int64_t nd, unsigned long long thr_rhs,
                                                    unsigned long long td_den, Counters *ctr, const uint32_t *__restrict__ skip,
                                                    const uint32_t *__restrict__ skip2)
{
    if ((skip && *skip) || (skip2 && *skip2)) return;
    unsigned long long c_nd = 0, c_td = 0;
    const int64_t stride = (int64_t)gridDim.x * FB;
    for (int64_t i = (int64_t)blockIdx.x * FB + threadIdx.x; i < nd; i += stride) {
        const unsigned long long c = hist[i];
        if (c >= 1ull) {
            ++c_nd;
            if (c * td_den >= thr_rhs) ++c_td;
        }
    }
    c_nd = wave_sum(c_nd); c_td = wave_sum(c_td);
    __shared__ unsigned long long s_nd[FB / WAVE], s_td[FB / WAVE];
    if (lane_id() == 0) { s_nd[threadIdx.x / WAVE] = c_nd; s_td[threadIdx.x / WAVE] = c_td; }
    __syncthreads();
    if (threadIdx.x == 0) {   // one pair of atomics per block: same-address atomics serialise
        for (int w = 1; w < FB / WAVE; ++w) { c_nd += s_nd[w]; c_td += s_td[w]; }
        if (c_nd) atomicAdd(&ctr->n_diag, c_nd);
        if (c_td) atomicAdd(&ctr->n_true, c_td);
    }
}

static int grid_for(int64_t n, int per_block, int cap)
{
    int64_t g = (n + per_block - 1) / per_block;
    if (g < 1) g = 1;
    if (g > cap) g = cap;
    return (int)g;
}

}  // namespace mo

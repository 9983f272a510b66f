// Device-side helpers for gfx950 (64-lane wavefronts, 8 XCDs).
#pragma once

#include <hip/hip_runtime.h>

#include <cstdint>

namespace mo {

constexpr int WAVE = 64;
constexpr int NUM_XCD = 8;

// Workgroups are handed to the 8 XCDs round-robin by their linear id.  Each XCD has its own L2, so neighbouring
// row blocks should land on the same XCD: this maps the hardware block id to a logical block id such that XCD x
// owns one contiguous run of logical blocks.  A bijection on [0, nb) for any nb.
__device__ __forceinline__ int64_t xcd_block(int64_t bid, int64_t nb)
{
    const int64_t q = nb / NUM_XCD, r = nb % NUM_XCD;
    const int64_t x = bid % NUM_XCD, j = bid / NUM_XCD;
    return x * q + (x < r ? x : r) + j;
}

__device__ __forceinline__ int lane_id() { return (int)(threadIdx.x & (WAVE - 1)); }

// Sum over aligned groups of `width` lanes (power of two, <= 64); every lane of the group gets lane-0-valid sum.
template <typename T>
__device__ __forceinline__ T group_sum_down(T v, int width)
{
    for (int off = width >> 1; off > 0; off >>= 1) v += __shfl_down(v, off, width);
    return v;
}

template <typename T>
__device__ __forceinline__ T wave_max(T v)
{
    for (int off = WAVE / 2; off > 0; off >>= 1) {
        T o = __shfl_xor(v, off, WAVE);
        v = o > v ? o : v;
    }
    return v;
}

template <typename T>
__device__ __forceinline__ T wave_min(T v)
{
    for (int off = WAVE / 2; off > 0; off >>= 1) {
        T o = __shfl_xor(v, off, WAVE);
        v = o < v ? o : v;
    }
    return v;
}

template <typename T>
__device__ __forceinline__ T wave_sum(T v)
{
    for (int off = WAVE / 2; off > 0; off >>= 1) v += __shfl_xor(v, off, WAVE);
    return v;
}

__device__ __forceinline__ uint64_t ballot64(bool p) { return __builtin_amdgcn_ballot_w64(p); }

// Streaming accesses for data that is touched once per SpMV (matrix values, indices, y): marked non-temporal so
// that they do not displace x from the caches.  Measured on MI355X: a plain read stream sustains about 6.4 TB/s,
// the same stream with non-temporal loads about 7.1 TB/s.
template <typename T>
__device__ __forceinline__ T ld_stream(const T *p) { return __builtin_nontemporal_load(p); }
template <typename T>
__device__ __forceinline__ void st_stream(T *p, T v) { __builtin_nontemporal_store(v, p); }

// Copy `count` >= 1 consecutive elements from global memory into a wave's LDS region.  The loads of a batch are all
// issued before the first one is consumed (registers in between), so a wave keeps STAGE_BATCH cache lines per lane
// group in flight instead of paying one memory latency per 64 elements.
constexpr int STAGE_BATCH = 8;
template <typename T, int BATCH = STAGE_BATCH>
__device__ __forceinline__ void stage_to_lds(const T *__restrict__ g, T *s, int count, int lane)
{
    for (int i0 = 0; i0 < count; i0 += WAVE * BATCH) {
        T r[BATCH];
#pragma unroll
        for (int u = 0; u < BATCH; ++u) {   // unconditional loads (index clamped into the run) so that none waits for another
            const int i = i0 + u * WAVE + lane;
            r[u] = ld_stream(g + (i < count ? i : count - 1));
        }
#pragma unroll
        for (int u = 0; u < BATCH; ++u) {
            const int i = i0 + u * WAVE + lane;
            if (i < count) s[i] = r[u];
        }
    }
}

// The same for two arrays that are indexed alike (column indices and values of one run of entries): the loads of
// both arrays, PAIR_BATCH per lane and array, are in flight together, so a run of up to 64 * PAIR_BATCH entries costs
// one memory latency instead of one per array and batch.
constexpr int PAIR_BATCH = 16;
template <typename A, typename B>
__device__ __forceinline__ void stage_pair_to_lds(const A *__restrict__ ga, const B *__restrict__ gb, A *sa, B *sb, int count, int lane)
{
    for (int i0 = 0; i0 < count; i0 += WAVE * PAIR_BATCH) {
        A ra[PAIR_BATCH];
        B rb[PAIR_BATCH];
#pragma unroll
        for (int u = 0; u < PAIR_BATCH; ++u) {
            const int i = i0 + u * WAVE + lane;
            ra[u] = ld_stream(ga + (i < count ? i : count - 1));
        }
#pragma unroll
        for (int u = 0; u < PAIR_BATCH; ++u) {
            const int i = i0 + u * WAVE + lane;
            rb[u] = ld_stream(gb + (i < count ? i : count - 1));
        }
#pragma unroll
        for (int u = 0; u < PAIR_BATCH; ++u) {
            const int i = i0 + u * WAVE + lane;
            if (i < count) { sa[i] = ra[u]; sb[i] = rb[u]; }
        }
    }
}

// Windows of x staged in LDS, B positions ("a run") at a time, after a plan of type WinRuns<NR> (mo_internal.hpp)
// that the kernel receives as an argument, so all of it sits in scalar registers.
// Requests x for the positions tid + u * B, u = u0 .. u0 + WB - 1, of a block's windows (clamped into x; bit u of
// *in tells whether the position lies inside [0, n): outside, the window holds 0).  The loads stand alone behind
// conditions that are the same for every thread, and nothing here waits for them: a caller issues its other loads
// next and calls window_stores after that, so a block pays one memory latency for all of them.
template <typename T, int B, int WB, typename PL>
__device__ __forceinline__ void window_loads(const PL &pl, int u0, int tid, int64_t row0, int64_t n, const T *__restrict__ x,
                                             T (&w)[WB], uint32_t *in)
{
    int64_t jj[WB];
    uint32_t bits = 0;
#pragma unroll
    for (int u = 0; u < WB; ++u) {
        constexpr int NR = (int)(sizeof(pl.bnd) / sizeof(pl.bnd[0]));
        const int r = u0 + u < NR ? u0 + u : NR - 1;
        const int64_t s0 = row0 + (int64_t)r * B + pl.d0[r], s1 = row0 + (int64_t)r * B + pl.d1[r];   // scalar
        const int64_t j = (tid + r * B < pl.bnd[r] ? s0 : s1) + tid;
        const bool ok = (uint64_t)j < (uint64_t)n;
        jj[u] = ok ? j : 0;
        bits |= ok ? 1u << u : 0u;
    }
#pragma unroll
    for (int u = 0; u < WB; ++u)
        if (u0 + u == 0 || (u0 + u) * B < pl.elems) w[u] = x[jj[u]];   // run 0 always exists: a window is at least B long
    *in = bits;
}

template <typename T, int B, int WB, typename PL>
__device__ __forceinline__ void window_stores(const PL &pl, int u0, int tid, const T (&w)[WB], uint32_t in, T *xs)
{
#pragma unroll
    for (int u = 0; u < WB; ++u) {
        const int i = tid + (u0 + u) * B;
        if (i < pl.elems) xs[i] = (in >> u & 1u) ? w[u] : (T)0;
    }
}

// The row that holds entry p of a CSR matrix: the largest r in [lo, hi] with row_ptr[r] <= p (row_ptr[lo] <= p is
// given).  Terminates with a result in [lo, hi] whatever row_ptr holds.
__device__ __forceinline__ int64_t row_of_entry(const int32_t *__restrict__ row_ptr, int64_t lo, int64_t hi, int64_t p)
{
    while (lo < hi) {
        const int64_t mid = (lo + hi + 1) >> 1;
        if ((int64_t)row_ptr[mid] <= p) lo = mid; else hi = mid - 1;
    }
    return lo;
}

typedef int int4v __attribute__((ext_vector_type(4)));
typedef int int2v __attribute__((ext_vector_type(2)));
typedef double dbl2v __attribute__((ext_vector_type(2)));
typedef float flt2v __attribute__((ext_vector_type(2)));
typedef float flt4v __attribute__((ext_vector_type(4)));

}  // namespace mo

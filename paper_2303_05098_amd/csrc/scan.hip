// Exclusive prefix sum over int32 (reduce / spine / apply), used by the conversions to turn per-row or
// per-diagonal counts into output positions.  Integer only, so the result is independent of scheduling.
#include "dev_common.hpp"
#include "mo_internal.hpp"

namespace mo {

constexpr int SB = 256;             // threads per block
constexpr int SI = 8;               // items per thread
constexpr int SCHUNK = SB * SI;     // items per block

// Exclusive scan of one value per thread across the block; returns the exclusive prefix, *total = block sum.
__device__ __forceinline__ int block_exclusive_scan(int v, int *total, int *s_wave /* SB / WAVE + 1 ints */)
{
    const int lane = lane_id(), w = threadIdx.x / WAVE;
    int inc = v;
    for (int off = 1; off < WAVE; off <<= 1) {
        const int o = __shfl_up(inc, off, WAVE);
        if (lane >= off) inc += o;
    }
    if (lane == WAVE - 1) s_wave[w] = inc;
    __syncthreads();
    if (threadIdx.x == 0) {
        int run = 0;
        for (int i = 0; i < SB / WAVE; ++i) { const int t = s_wave[i]; s_wave[i] = run; run += t; }
        s_wave[SB / WAVE] = run;
    }
    __syncthreads();
    *total = s_wave[SB / WAVE];
    const int res = s_wave[w] + inc - v;
    __syncthreads();
    return res;
}

__global__ __launch_bounds__(SB) void k_scan_reduce(const int32_t *__restrict__ in, int64_t n, int32_t *__restrict__ partial)
{
    const int64_t base = (int64_t)blockIdx.x * SCHUNK;
    int sum = 0;
    for (int k = 0; k < SI; ++k) {
        const int64_t i = base + (int64_t)k * SB + threadIdx.x;
        if (i < n) sum += in[i];
    }
    sum = wave_sum(sum);
    __shared__ int s[SB / WAVE];
    if (lane_id() == 0) s[threadIdx.x / WAVE] = sum;
    __syncthreads();
    if (threadIdx.x == 0) {
        int t = 0;
        for (int i = 0; i < SB / WAVE; ++i) t += s[i];
        partial[blockIdx.x] = t;
    }
}

// One block turns the per-block sums into exclusive prefixes in place.
__global__ __launch_bounds__(SB) void k_scan_spine(int32_t *__restrict__ partial, int64_t nb)
{
    __shared__ int s_wave[SB / WAVE + 1];
    int carry = 0;
    for (int64_t base = 0; base < nb; base += SB) {
        const int64_t i = base + threadIdx.x;
        const int v = i < nb ? partial[i] : 0;
        int total;
        const int ex = block_exclusive_scan(v, &total, s_wave);
        if (i < nb) partial[i] = carry + ex;
        carry += total;
    }
}

__global__ __launch_bounds__(SB) void k_scan_apply(const int32_t *__restrict__ in, int32_t *__restrict__ out, int64_t n,
                                                    const int32_t *__restrict__ partial)
{
    __shared__ int s_wave[SB / WAVE + 1];
    const int64_t base = (int64_t)blockIdx.x * SCHUNK + (int64_t)threadIdx.x * SI;   // SI consecutive items per thread
    int v[SI];
    int sum = 0;
    for (int k = 0; k < SI; ++k) {
        v[k] = (base + k < n) ? in[base + k] : 0;
        sum += v[k];
    }
    int total;
    int run = block_exclusive_scan(sum, &total, s_wave) + partial[blockIdx.x];
    for (int k = 0; k < SI; ++k) {
        if (base + k < n) out[base + k] = run;
        run += v[k];
        if (base + k == n - 1) out[n] = run;
    }
}

__global__ void k_scan_empty(int32_t *out) { if (threadIdx.x == 0 && blockIdx.x == 0) out[0] = 0; }

size_t scan_tmp_bytes(int64_t n)
{
    const int64_t nb = (n + SCHUNK - 1) / SCHUNK;
    return (size_t)(nb > 0 ? nb : 1) * sizeof(int32_t);
}

mo_status exclusive_scan_i32(const int32_t *in, int32_t *out, int64_t n, void *tmp, hipStream_t s)
{
    if (n <= 0) {
        hipLaunchKernelGGL(k_scan_empty, dim3(1), dim3(64), 0, s, out);
        MO_LAUNCH_CHECK();
        return MO_OK;
    }
    const int64_t nb = (n + SCHUNK - 1) / SCHUNK;
    int32_t *partial = (int32_t *)tmp;
    hipLaunchKernelGGL(k_scan_reduce, dim3((unsigned)nb), dim3(SB), 0, s, in, n, partial);
    MO_LAUNCH_CHECK();
    hipLaunchKernelGGL(k_scan_spine, dim3(1), dim3(SB), 0, s, partial, nb);
    MO_LAUNCH_CHECK();
    hipLaunchKernelGGL(k_scan_apply, dim3((unsigned)nb), dim3(SB), 0, s, in, out, n, partial);
    MO_LAUNCH_CHECK();
    return MO_OK;
}

}  // namespace mo

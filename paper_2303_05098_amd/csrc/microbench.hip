// Stand-alone measurements of what the memory system of one MI355X gives the access patterns of the SpMV and feature
// kernels: the ceilings their design notes refer to.  Not part of libmo.so; built as its own program (mo_microbench).
//
//   1. sequential reads of 1 GiB: plain and non-temporal loads, and a device copy (the stream ceilings);
//   2. the CSR tile kernel taken apart on the access pattern of a 27-point stencil (2 097 152 rows of 27 entries):
//      entry stream alone, + x gathers, + products through LDS and row sums, + y written, with the tile's entry stream
//      and its rows of y starting on cache-line boundaries or not;
//   3. random 8-byte gathers from tables of 2, 8 and 32 MB (indices streamed): the rate that bounds matrices with
//      scattered columns, in and out of one XCD's 4 MB L2;
//   4. random 4-byte atomic adds on distinct addresses of a 16 MB table: the rate that bounds the diagonal histogram of
//      a matrix without diagonal structure;
//   5. the HDC traffic of the banded + scatter configuration in its simplest form: nine slabs of 4 194 304 doubles (or
//      floats) streamed one row per lane with x taken from the row's own neighbourhood, y written, and 1 167 106
//      random gathers of x (one per row for 28 % of the rows), with and without the gathers: what the scattered
//      remainder costs any kernel on this memory system, each gather moving a 128-byte line.
//   6. the rate at which cache-resident data reaches registers, by bytes per lane and load (4, 8, 16) and by where the
//      data sits (a 2 KB region per block: the CU's L1; 31 regions of 64 KB shared by all blocks, a CU's blocks on
//      different ones: the XCD's L2): what bounds a kernel that fetches a row of a dense operand per matrix entry (the multi-vector
//      product) once the matrix stream itself is no longer the limit.
// Every kernel is timed with events over 20 launches after 3 warm-ups; sizes are printed with the results.
#include <hip/hip_runtime.h>

#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <vector>

#define CK(x)                                                                         \
    do {                                                                              \
        hipError_t e_ = (x);                                                          \
        if (e_ != hipSuccess) {                                                       \
            std::printf("HIP error %s at line %d\n", hipGetErrorString(e_), __LINE__); \
            std::exit(1);                                                             \
        }                                                                             \
    } while (0)

template <class F>
static float time_ms(F f, int reps = 20)
{
    hipEvent_t a, b;
    CK(hipEventCreate(&a));
    CK(hipEventCreate(&b));
    for (int i = 0; i < 3; ++i) f();
    CK(hipEventRecord(a));
    for (int i = 0; i < reps; ++i) f();
    CK(hipEventRecord(b));
    CK(hipEventSynchronize(b));
    float ms = 0.f;
    CK(hipEventElapsedTime(&ms, a, b));
    CK(hipEventDestroy(a));
    CK(hipEventDestroy(b));
    return ms / reps;
}

// ------------------------------------------------------------------ 1. sequential streams
template <int U, bool NT>
__global__ __launch_bounds__(256) void k_read(const double *__restrict__ p, size_t n, double *out)
{
    const size_t stride = (size_t)gridDim.x * 256 * U;
    double s = 0;
    for (size_t i = (size_t)blockIdx.x * 256 * U + threadIdx.x; i + 256 * (U - 1) < n; i += stride) {
        double v[U];
#pragma unroll
        for (int u = 0; u < U; ++u) v[u] = NT ? __builtin_nontemporal_load(p + i + 256 * u) : p[i + 256 * u];
#pragma unroll
        for (int u = 0; u < U; ++u) s += v[u];
    }
    if (s == 1.2345) out[0] = s;   // never true for the zero-filled input: keeps the loads alive
}

__global__ __launch_bounds__(256) void k_copy(const double2 *__restrict__ a, double2 *__restrict__ b, size_t n)
{
    const size_t stride = (size_t)gridDim.x * 256;
    for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n; i += stride) b[i] = a[i];
}

// ------------------------------------------------------------------ 2. the CSR tile kernel, step by step
__global__ void k_stencil_pattern(int *col, double *val, int *rp, long nnz, long m)
{
    const int off[27] = {-16513, -16512, -16511, -16385, -16384, -16383, -16257, -16256, -16255, -129, -128, -127, -1, 0,
                         1,      127,    128,    129,    16255,  16256,  16257,  16383,  16384,  16385,  16511, 16512, 16513};
    for (long e = (long)blockIdx.x * blockDim.x + threadIdx.x; e < nnz; e += (long)gridDim.x * blockDim.x) {
        const long r = e / 27;
        long c = r + off[e % 27];
        c = c < 0 ? 0 : (c >= m ? m - 1 : c);
        col[e] = (int)c;
        val[e] = 1.0 + (double)(e & 7);
        if (e <= m) rp[e] = (int)(e * 27);
    }
}

// STEP 0: entry stream only.  1: + x gathers.  2: + products to LDS, barrier, row sums (4 lanes per row), nothing stored.
// 3: + y stored.  A tile is TILE consecutive entries and ROWS rows of y (ROWS * 27 need not equal TILE: the pattern of
// the accesses is what is measured, not a product).  E loads of 256 entries each per tile.
template <int STEP, int TILE, int E, int ROWS>
__global__ __launch_bounds__(256) void k_tile(const int *__restrict__ col, const double *__restrict__ val, const int *__restrict__ rp,
                                              const double *__restrict__ x, double *__restrict__ y, double *__restrict__ out, long nnz,
                                              long m)
{
    constexpr int G = 4, RPB = 256 / G;
    __shared__ double ps[E * 256];
    const long tile = blockIdx.x, p0 = tile * TILE, ra = tile * ROWS;
    const int cnt = (int)((nnz - p0) < (long)E * 256 ? (nnz - p0) : (long)E * 256), last = cnt - 1;
    int c[E];
    double v[E];
#pragma unroll
    for (int j = 0; j < E; ++j) {
        const int i = threadIdx.x + j * 256;
        c[j] = __builtin_nontemporal_load(col + p0 + (i < cnt ? i : last));
    }
#pragma unroll
    for (int j = 0; j < E; ++j) {
        const int i = threadIdx.x + j * 256;
        v[j] = __builtin_nontemporal_load(val + p0 + (i < cnt ? i : last));
    }
    int r0a = 0, r0b = 0, r1a = 0, r1b = 0;
    if (STEP >= 2) {
        const long r0 = ra + threadIdx.x / G, r1 = r0 + RPB;
        r0a = rp[r0 < m ? r0 : m]; r0b = rp[r0 + 1 < m ? r0 + 1 : m];
        r1a = rp[r1 < m ? r1 : m]; r1b = rp[r1 + 1 < m ? r1 + 1 : m];
    }
    double xv[E];
#pragma unroll
    for (int j = 0; j < E; ++j) xv[j] = STEP >= 1 ? x[c[j]] : (double)c[j];
    if (STEP <= 1) {
        double s = 0;
#pragma unroll
        for (int j = 0; j < E; ++j) s += v[j] * xv[j];
        if (s == 12345.678) out[blockIdx.x] = s;
        return;
    }
#pragma unroll
    for (int j = 0; j < E; ++j) {
        const int i = threadIdx.x + j * 256;
        if (i < cnt) ps[i] = v[j] * xv[j];
    }
    __syncthreads();
    const int sub = threadIdx.x % G;
    for (int base = 0; base < ROWS; base += RPB) {
        const int q = base + threadIdx.x / G;
        // rows of 27 entries laid over the tile from its start; the row pointers are loaded as the kernel would load
        // them and take part in a comparison that never holds (they are multiples of 27, never negative)
        int lo = q * 27, hi = q * 27 + 27;
        if ((base == 0 ? r0a + r0b : r1a + r1b) < 0) lo = hi;
        lo = lo > cnt ? cnt : lo;
        hi = hi > cnt ? cnt : hi;
        if (q >= ROWS || ra + q >= m) lo = hi = 0;
        double sum = 0;
        for (int e = lo + sub; e < hi; e += G) sum += ps[e];
        for (int o = G >> 1; o > 0; o >>= 1) sum += __shfl_down(sum, o, G);
        if (STEP == 2) { if (sum == 12345.678) out[blockIdx.x] = sum; }
        else if (sub == 0 && q < ROWS && ra + q < m) __builtin_nontemporal_store(sum, y + ra + q);
    }
}

// ------------------------------------------------------------------ 3. random gathers, 4. random atomics
__global__ __launch_bounds__(256) void k_gather(const int32_t *__restrict__ idx, const double *__restrict__ x, int64_t cnt, double *out)
{
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    double s = 0;
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < cnt; i += stride) s += x[__builtin_nontemporal_load(idx + i)];
    if (s == 1.2345e300) out[0] = s;
}

__global__ __launch_bounds__(256) void k_atomic(const int32_t *__restrict__ idx, uint32_t *table, int64_t cnt)
{
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < cnt; i += stride)
        atomicAdd(table + __builtin_nontemporal_load(idx + i), 1u);
}

// ------------------------------------------------------------------ 5. nine slabs + scattered gathers
template <typename T, bool GATHER>
__global__ __launch_bounds__(512) void k_slabs(const T *__restrict__ val, long m, long ld, const T *__restrict__ x,
                                               const int32_t *__restrict__ gcol, T *__restrict__ y)
{
    const long row = (long)blockIdx.x * 512 + threadIdx.x;
    if (row >= m) return;
    T s = (T)0;
#pragma unroll
    for (int k = 0; k < 9; ++k) s += __builtin_nontemporal_load(val + k * ld + row) * x[row];
    if (GATHER) {
        const int32_t c = __builtin_nontemporal_load(gcol + row);   // -1: this row has no scattered entry
        if (c >= 0) s += x[c];
    }
    __builtin_nontemporal_store(s, y + row);
}

// skew: rows between the end of one slab and the start of the next.  With 0 the slabs lie 2^22 elements apart and the
// nine loads of a row fall on the same memory channels; the library's conversions add 576 rows in that case.
template <typename T>
static void run_slabs(const char *name, long skew)
{
    const long m = 4194304, scattered = 1167106, ld = m + skew;
    T *val, *x, *y;
    int32_t *gcol;
    CK(hipMalloc(&val, 9 * ld * sizeof(T))); CK(hipMalloc(&x, m * sizeof(T))); CK(hipMalloc(&y, m * sizeof(T))); CK(hipMalloc(&gcol, m * 4));
    CK(hipMemset(val, 0, 9 * ld * sizeof(T))); CK(hipMemset(x, 0, m * sizeof(T)));
    std::vector<int32_t> h((size_t)m, -1);
    uint64_t z = 777;
    for (long i = 0; i < scattered; ++i) {   // rows i * m / scattered carry one gather each, to a random column
        z = z * 6364136223846793005ull + 1442695040888963407ull;
        h[(size_t)(i * m / scattered)] = (int32_t)((z >> 33) % (uint64_t)m);
    }
    CK(hipMemcpy(gcol, h.data(), m * 4, hipMemcpyHostToDevice));
    const double bytes = (9.0 + 2.0) * m * sizeof(T) + m * 4.0;
    float ms = time_ms([&] { k_slabs<T, false><<<(unsigned)(m / 512), 512>>>(val, m, ld, x, gcol, y); });
    std::printf("5 %s, slabs %4ld rows apart: nine slabs, x, y                       : %7.1f us  %7.1f GB/s\n", name, skew, ms * 1e3,
                (bytes - m * 4.0) / ms / 1e6);
    ms = time_ms([&] { k_slabs<T, true><<<(unsigned)(m / 512), 512>>>(val, m, ld, x, gcol, y); });
    std::printf("5 %s, slabs %4ld rows apart: + gather flags and %ld random gathers : %7.1f us  %7.1f GB/s (without the lines the gathers move)\n",
                name, skew, scattered, ms * 1e3, bytes / ms / 1e6);
    CK(hipFree(val)); CK(hipFree(x)); CK(hipFree(y)); CK(hipFree(gcol));
}

// ------------------------------------------------------------------ 6. cache-resident data into registers
// Block b reads `region` elements starting at region number (b / 8) mod nregion, 256 consecutive elements per step, round
// and round.  Blocks b .. b + 7 go to the 8 XCDs, so every XCD sees every region (nregion regions have to fit its L2),
// and nregion is odd so that the blocks that share a CU (b / 8 apart by multiples of the CUs per XCD) read different ones.
template <typename VT>
__global__ __launch_bounds__(256) void k_fill_regs(const VT *__restrict__ p, unsigned region, unsigned nregion, int steps, double *out)
{
    const VT *base = p + (size_t)((blockIdx.x / 8) % nregion) * region;
    float s = 0.f;
    for (int it = 0; it < steps; it += 8) {
        VT v[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) v[u] = base[(unsigned)((it + u) * 256 + threadIdx.x) & (region - 1)];
#pragma unroll
        for (int u = 0; u < 8; ++u)
            for (unsigned w = 0; w < sizeof(VT) / 4; ++w) s += reinterpret_cast<const float *>(&v[u])[w];   // every loaded word is used
    }
    if (s == 1.2345f) out[0] = s;   // never true for the zero-filled input: keeps the loads alive
}

template <typename VT>
static void run_fill_regs(const char *what, const void *table, double *out)
{
    const unsigned grid = 256 * 8 * 4;
    const int steps = 512;
    const double bytes = (double)grid * steps * 256 * sizeof(VT);
    float ms = time_ms([&] { k_fill_regs<VT><<<grid, 256>>>((const VT *)table, 2048 / sizeof(VT), grid / 8, steps, out); }, 5);
    std::printf("6 %s per lane, 2 KB per block (L1)                    : %8.1f us  %7.1f GB/s\n", what, ms * 1e3, bytes / ms / 1e6);
    ms = time_ms([&] { k_fill_regs<VT><<<grid, 256>>>((const VT *)table, 65536 / sizeof(VT), 31, steps, out); }, 5);
    std::printf("6 %s per lane, 64 KB per block, 31 such regions (L2): %8.1f us  %7.1f GB/s\n", what, ms * 1e3, bytes / ms / 1e6);
}

int main()
{
    double *out;
    CK(hipMalloc(&out, 1 << 24));
    {
        const size_t n = (size_t)1 << 27;   // 1 GiB of doubles
        double *p, *q;
        CK(hipMalloc(&p, n * 8));
        CK(hipMalloc(&q, n * 8));
        CK(hipMemset(p, 0, n * 8));
        CK(hipMemset(q, 0, n * 8));
        float ms = time_ms([&] { k_read<8, false><<<4096, 256>>>(p, n, out); });
        std::printf("1 read 1 GiB, plain loads         : %8.1f us  %7.1f GB/s\n", ms * 1e3, n * 8.0 / ms / 1e6);
        ms = time_ms([&] { k_read<8, true><<<4096, 256>>>(p, n, out); });
        std::printf("1 read 1 GiB, non-temporal loads  : %8.1f us  %7.1f GB/s\n", ms * 1e3, n * 8.0 / ms / 1e6);
        ms = time_ms([&] { k_copy<<<8192, 256>>>((const double2 *)p, (double2 *)q, n / 2); });
        std::printf("1 copy 1 GiB -> 1 GiB             : %8.1f us  %7.1f GB/s (read + written)\n", ms * 1e3, 2.0 * n * 8.0 / ms / 1e6);
        CK(hipFree(p));
        CK(hipFree(q));
    }
    {
        const long m = 2097152, nnz = m * 27;
        int *col, *rp;
        double *val, *x, *y;
        CK(hipMalloc(&col, nnz * 4)); CK(hipMalloc(&val, nnz * 8)); CK(hipMalloc(&rp, (m + 1) * 4));
        CK(hipMalloc(&x, m * 8)); CK(hipMalloc(&y, m * 8));
        k_stencil_pattern<<<4096, 256>>>(col, val, rp, nnz, m);
        CK(hipMemset(x, 0, m * 8));
        CK(hipDeviceSynchronize());
        const double bytes = nnz * 12.0 + (m + 1) * 4.0 + 2.0 * m * 8.0;
        std::printf("2 CSR tile steps, 27-point pattern, %ld rows, %ld entries, %.1f MB per pass (all of a CSR SpMV)\n", m, nnz, bytes / 1e6);
#define RUN(STEP, TILE, E, ROWS, what)                                                                                              \
        {                                                                                                                               \
            const long nt = (nnz + TILE - 1) / TILE;                                                                                    \
            const float ms = time_ms([&] { k_tile<STEP, TILE, E, ROWS><<<nt, 256>>>(col, val, rp, x, y, out, nnz, m); });            \
            std::printf("2 %-66s: %7.1f us  %7.1f GB/s\n", what, ms * 1e3, bytes / ms / 1e6);                                          \
        }
        RUN(0, 2048, 8, 76, "entry stream, tiles of 2048 entries on line boundaries")
        RUN(1, 2048, 8, 76, "+ x gathers")
        RUN(2, 2048, 8, 76, "+ products through LDS, row sums (nothing stored)")
        RUN(3, 2048, 8, 64, "+ y stored, 64 rows per tile (whole lines of y)")
        RUN(3, 2048, 8, 76, "+ y stored, 76 rows per tile (tiles share lines of y)")
        RUN(1, 2052, 9, 76, "stream + gathers, tiles of 2052 entries (76 whole rows, off line boundaries)")
        RUN(3, 2052, 9, 76, "all steps, tiles of 2052 entries, 76 rows")
        RUN(3, 4096, 16, 128, "all steps, tiles of 4096 entries, 128 rows (whole lines of y)")
#undef RUN
        CK(hipFree(col)); CK(hipFree(val)); CK(hipFree(rp)); CK(hipFree(x)); CK(hipFree(y));
    }
    {
        const int64_t cnt = 16777216;
        std::vector<int32_t> h((size_t)cnt);
        int32_t *idx;
        CK(hipMalloc(&idx, cnt * 4));
        for (int64_t n : {(int64_t)1 << 18, (int64_t)1 << 20, (int64_t)1 << 22}) {
            uint64_t z = 12345;
            for (int64_t i = 0; i < cnt; ++i) {
                z = z * 6364136223846793005ull + 1442695040888963407ull;
                h[(size_t)i] = (int32_t)((z >> 33) % (uint64_t)n);
            }
            CK(hipMemcpy(idx, h.data(), cnt * 4, hipMemcpyHostToDevice));
            double *x;
            CK(hipMalloc(&x, n * 8));
            CK(hipMemset(x, 0, n * 8));
            const float ms = time_ms([&] { k_gather<<<4096, 256>>>(idx, x, cnt, out); }, 10);
            std::printf("3 %lld random 8-byte gathers from a %lld MB table: %7.1f us  %6.1f G gathers/s\n", (long long)cnt,
                        (long long)(n * 8 >> 20), ms * 1e3, cnt / ms / 1e6);
            CK(hipFree(x));
        }
        uint32_t *table;
        CK(hipMalloc(&table, (size_t)(1 << 22) * 4));
        CK(hipMemset(table, 0, (size_t)(1 << 22) * 4));
        const float ms = time_ms([&] { k_atomic<<<4096, 256>>>(idx, table, cnt); }, 10);
        std::printf("4 %lld random 4-byte atomic adds on a 16 MB table  : %7.1f us  %6.1f G atomics/s\n", (long long)cnt, ms * 1e3, cnt / ms / 1e6);
        CK(hipFree(table));
        CK(hipFree(idx));
    }
    run_slabs<double>("fp64", 0);
    run_slabs<double>("fp64", 576);
    run_slabs<float>("fp32", 0);
    run_slabs<float>("fp32", 576);
    {
        void *table;
        CK(hipMalloc(&table, (size_t)4 << 20));   // 1024 regions of 2 KB or 31 of 64 KB
        CK(hipMemset(table, 0, (size_t)4 << 20));
        run_fill_regs<float>(" 4 bytes", table, out);
        run_fill_regs<float2>(" 8 bytes", table, out);
        run_fill_regs<float4>("16 bytes", table, out);
        CK(hipFree(table));
    }
    CK(hipFree(out));
    return 0;
}

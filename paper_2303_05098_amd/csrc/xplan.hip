// Launch data for the SpMV kernels that gather x by column index (CSR, COO, ELL, HYB): where x is read from.
//
// A banded or stencil matrix keeps most of its entries on a few diagonals, so the columns a block of consecutive rows
// touches fall into a few short windows of x: rows [ra, rb) and a group of diagonals with offsets [lo, lo + span)
// only read x[ra + lo, rb - 1 + lo + span).  A kernel that knows those groups can fetch the windows once, coalesced,
// into LDS and serve its entries from there; the entries that fall outside every window are still gathered from
// global memory, so the plan changes how fast a kernel runs and never what it computes.
//
// The diagonals that matter are found by sampling (Section IV-A characterises a matrix by its populated diagonals;
// here only a cheap estimate is needed): XP_SAMPLES rows spread evenly over the matrix, the offsets col - row of
// their first XP_PER_ROW entries each; an offset met in at least a quarter of the sampled non-empty rows is "hot".
// Hot offsets closer than XP_GAP are grouped; more than XP_MAX_CL groups are merged by widening the gap.
#include "dev_common.hpp"
#include "mo_internal.hpp"

#include <algorithm>
#include <map>

namespace mo {

constexpr int XP_SAMPLES = 256;
constexpr int XP_PER_ROW = 64;
constexpr int XP_GAP = 256;
constexpr int64_t XP_MAX_SPAN = 4096;   // offsets one group may cover (wider groups cannot fit any kernel's LDS windows)

// Block s samples row floor(s * m / nsamp): out[s * (XP_PER_ROW + 1)] = entries recorded, then their offsets.
__global__ __launch_bounds__(XP_PER_ROW) void k_sample_rows(const int32_t *__restrict__ row_ptr, const int32_t *__restrict__ col_idx, int64_t m,
                                                             int nsamp, int32_t *__restrict__ out)
{
    const int64_t row = (int64_t)blockIdx.x * m / nsamp;
    const int64_t lo = row_ptr[row], hi = row_ptr[row + 1];
    const int cnt = (int)(hi - lo < XP_PER_ROW ? hi - lo : XP_PER_ROW);
    int32_t *o = out + (int64_t)blockIdx.x * (XP_PER_ROW + 1);
    if (threadIdx.x == 0) o[0] = cnt;
    if ((int)threadIdx.x < cnt) o[1 + threadIdx.x] = (int32_t)((int64_t)col_idx[lo + threadIdx.x] - row);
}

mo_status plan_x_windows(const int32_t *row_ptr, const int32_t *col_idx, int64_t m, int64_t nnz, XPlan *out, hipStream_t s)
{
    out->ncl = 0;
    if (m < 1 || nnz < 1) return MO_OK;
    const int nsamp = (int)(m < XP_SAMPLES ? m : XP_SAMPLES);
    const size_t count = (size_t)nsamp * (XP_PER_ROW + 1);
    Scratch scr(s);
    int32_t *dev = (int32_t *)scr.get(count * 4);
    if (!dev) return MO_E_ALLOC;
    hipLaunchKernelGGL(k_sample_rows, dim3(nsamp), dim3(XP_PER_ROW), 0, s, row_ptr, col_idx, m, nsamp, dev);
    MO_LAUNCH_CHECK();
    std::vector<int32_t> host(count);
    MO_HIP(hipMemcpyAsync(host.data(), dev, count * 4, hipMemcpyDeviceToHost, s));
    MO_HIP(hipStreamSynchronize(s));
    std::map<int32_t, int> freq;
    int nonempty = 0;
    for (int q = 0; q < nsamp; ++q) {
        const int32_t *o = host.data() + (size_t)q * (XP_PER_ROW + 1);
        const int cnt = o[0] < 0 ? 0 : (o[0] > XP_PER_ROW ? XP_PER_ROW : o[0]);
        if (cnt > 0) ++nonempty;
        for (int j = 0; j < cnt; ++j) ++freq[o[1 + j]];
    }
    std::vector<int32_t> hot;   // ascending: std::map iterates in key order
    for (const auto &kv : freq)
        if (kv.second * 4 >= nonempty) hot.push_back(kv.first);
    if (hot.empty() || hot.size() > 256) return MO_OK;
    for (int64_t gap = XP_GAP; gap <= XP_MAX_SPAN; gap *= 2) {
        XPlan p;
        p.ncl = 0;
        bool ok = true;
        size_t k = 0;
        while (k < hot.size() && ok) {
            size_t e = k;
            while (e + 1 < hot.size() && (int64_t)hot[e + 1] - (int64_t)hot[e] < gap) ++e;
            const int64_t span = (int64_t)hot[e] - (int64_t)hot[k] + 1;
            if (p.ncl == XP_MAX_CL || span > XP_MAX_SPAN) { ok = false; break; }
            p.lo[p.ncl] = hot[k];
            p.span[p.ncl] = (int32_t)span;
            ++p.ncl;
            k = e + 1;
        }
        if (ok) { *out = p; return MO_OK; }
    }
    return MO_OK;
}

}  // namespace mo

// Internal declarations shared by the library's translation units (host side).
#pragma once

#include <hip/hip_runtime.h>

#include <climits>
#include <cstdint>
#include <new>
#include <vector>

#include "mo.h"

namespace mo {

// ---------------------------------------------------------------- errors
void set_hip_error(hipError_t e);

#define MO_HIP(call)                                        \
    do {                                                    \
        hipError_t mo_e_ = (call);                          \
        if (mo_e_ != hipSuccess) {                          \
            ::mo::set_hip_error(mo_e_);                     \
            return MO_E_DEVICE;                             \
        }                                                   \
    } while (0)

#define MO_TRY(call)                                        \
    do {                                                    \
        mo_status mo_s_ = (call);                           \
        if (mo_s_ != MO_OK) return mo_s_;                   \
    } while (0)

// Nothing may leave an extern "C" function by exception: host containers that fail to grow become MO_E_ALLOC.
template <typename F>
inline mo_status no_throw(F &&body)
{
    try {
        return body();
    } catch (const std::bad_alloc &) {
        return MO_E_ALLOC;
    } catch (...) {
        return MO_E_ALLOC;
    }
}

// Launch check: catches bad launch configurations right away.
#define MO_LAUNCH_CHECK() MO_HIP(hipGetLastError())

// ---------------------------------------------------------------- device memory
void *dev_alloc(size_t bytes, hipStream_t s);   // never returns NULL for bytes == 0 (allocates 256 B)
void dev_free(void *p, hipStream_t s);

// Scoped scratch: everything allocated through it is released when it goes out of scope.
struct Scratch {
    hipStream_t s;
    std::vector<void *> ptrs;
    explicit Scratch(hipStream_t st) : s(st) {}
    ~Scratch() { for (void *p : ptrs) dev_free(p, s); }
    void *get(size_t bytes) {
        void *p = dev_alloc(bytes, s);
        if (p) ptrs.push_back(p);
        return p;
    }
    Scratch(const Scratch &) = delete;
    Scratch &operator=(const Scratch &) = delete;
};

// ---------------------------------------------------------------- handle
constexpr int CSR_TILE = 2048;        // entries per CSR work tile
constexpr int CSR_TILE_LARGE = 4096;  // ... of the row-owning kernel in fp32, or when rows average 16 entries or more
constexpr int CSR_TILE_SMALL = 512;   // ... for parts of fewer than CSR_SMALL_NNZ entries, which 2048-entry tiles would
constexpr int64_t CSR_SMALL_NNZ = 1 << 20;   // spread over too few blocks (measured cross-over: 1 - 2 M entries)
constexpr int CSR_MAX_ROW = 256;      // longest row the row-owning tiled CSR kernel accepts
constexpr int CSR_TILE_SLACK = 512;   // entries a tile may hold beyond its nominal size: the rows it owns run to the end of
                                      // the last of them, and its first row is rounded up to a multiple of row_align rows
constexpr int CSR_HEAD = 32;          // a tile's stream starts on a multiple of this many entries (a 128-byte line of columns)
constexpr int COO_B_THREADS = 256;    // threads per COO block; a tile is COO_B_THREADS * coo_strip entries
constexpr int64_t COO_SMALL_NNZ = 4 * 1024 * 1024;   // from this many entries on a COO part uses 8-entry strips (below: 4, or 2 inside HYB)


// Windows of x that cover the matrix's heavily populated diagonals (launch data, see xplan.hip): group c covers the
// offsets col - row in [lo[c], lo[c] + span[c]).  ncl = 0: no such structure was found, x is gathered.
constexpr int XP_MAX_CL = 8;
struct XPlan {
    int32_t ncl = 0;
    int32_t lo[XP_MAX_CL] = {};
    int32_t span[XP_MAX_CL] = {};
};

}  // namespace mo

namespace mo {
// Windows of x staged in LDS, B positions ("a run") at a time.  The windows of a block lie one after the other in
// LDS, elems positions in all, and every window is at least B long, so run u (positions u * B .. u * B + B - 1) lies
// in at most two windows: position i of it holds x[row0 + i + (i < bnd[u] ? d0[u] : d1[u])], row0 being the block's
// first row.  The plan is a kernel argument, so all of this sits in scalar registers.
template <int NR>
struct WinRuns {
    int32_t elems = 0;
    int32_t bnd[NR] = {};
    int32_t d0[NR] = {};
    int32_t d1[NR] = {};
};


// Host side: the runs of B positions for windows given as (first offset, length) in LDS order.
template <int NR>
inline bool plan_window_runs(const int32_t *lo, const int32_t *len, int nwin, int B, WinRuns<NR> *out)
{
    int64_t total = 0;
    for (int q = 0; q < nwin; ++q) {
        if (len[q] < B) return false;
        total += len[q];
    }
    if (total > (int64_t)NR * B) return false;
    out->elems = (int32_t)total;
    int q = 0;
    int64_t base = 0;   // LDS position of window q
    for (int u = 0; (int64_t)u * B < total; ++u) {
        while (q + 1 < nwin && base + len[q] <= (int64_t)u * B) { base += len[q]; ++q; }
        const bool more = q + 1 < nwin;
        out->bnd[u] = more ? (int32_t)(base + len[q]) : INT32_MAX;
        out->d0[u] = (int32_t)(lo[q] - base);
        out->d1[u] = more ? (int32_t)(lo[q + 1] - (base + len[q])) : 0;
    }
    return true;
}

// Launch plan of the batched DIA / HDC kernel (large matrices with at most DIA_PRE diagonals), passed by value in the
// kernel arguments (scalar registers: no load to wait for): the x windows of a block as runs of DIA_BATCH_BLOCK LDS
// positions (WinRuns), and xpos[k], the position of x[row0 + off_k] for the block's first row row0.
constexpr int DIA_MAX_RUNS = 16;
constexpr int DIA_PRE = 12;                        // diagonals the batched kernel takes at most: all loaded as one batch
constexpr int DIA_BATCH_BLOCK = 512;               // its threads per block
constexpr int64_t DIA_BATCH_MIN_ROWS = 1 << 19;    // below, the streaming kernel is as fast or faster (measured)
struct DiaPlan {
    WinRuns<DIA_MAX_RUNS> win;
    int32_t xpos[DIA_PRE] = {};
};
}  // namespace mo

struct mo_matrix {
    mo_format fmt = MO_CSR;
    mo_dtype dtype = MO_F64;
    int64_t m = 0, n = 0, nnz = 0, ld = 0;
    // DIA part
    int64_t nd = 0;
    int32_t *dia_off = nullptr;
    void *dia_val = nullptr;
    // x windows the DIA kernels stage in LDS (launch data, derived from dia_off at conversion time)
    int32_t dia_block = 0;            // threads per block of the LDS kernel; 0 = direct kernel
    int32_t dia_rows = 1;             // rows per thread of the LDS kernel
    int32_t dia_ncl = 0;
    int64_t dia_lds_elems = 0;
    int32_t *dia_xpos = nullptr, *dia_clusters = nullptr;
    bool dia_batch = false;           // the batched kernel runs (large matrix, few diagonals), with this plan:
    mo::DiaPlan dia_plan;
    // HDC run by the batched kernel: the remainder's row pointers in the form that kernel reads (launch data; the
    // exported csr_row_ptr stays as it is).  hdc_blk[b] = first remainder entry of row block b (blocks of dia_block *
    // dia_rows rows; one entry more than blocks), hdc_rp16[row] = csr_row_ptr[row] - hdc_blk[block of row]: 2 bytes per
    // row streamed instead of 4.  Null when that kernel is not the one that runs.
    int32_t *hdc_blk = nullptr;
    uint16_t *hdc_rp16 = nullptr;
    // the same kind of plan for blocks of SPMM_ROWS rows: windows of X for the multi-vector product
    int64_t mm_lds_elems = 0;         // staged rows of X per block; 0 = no plan (windows too large), direct kernel
    int32_t *mm_xpos = nullptr;       // per diagonal: staged row that the block's first matrix row reads
    int32_t *mm_map = nullptr;        // per run of SPMM_ROWS staged rows: (first staged row of the next window, row of X minus
                                      // staged row in the run's first window, the same in the next), rows of X relative to the
                                      // block's first matrix row
    // ELL part
    int64_t k = 0;
    int32_t *ell_col = nullptr;
    void *ell_val = nullptr;
    // COO part
    int64_t nnz_coo = 0;
    int32_t *coo_row = nullptr, *coo_col = nullptr;
    void *coo_val = nullptr;
    // CSR part (borrowed for MO_CSR, owned for MO_HDC)
    int64_t nnz_csr = 0;
    const int32_t *csr_row_ptr = nullptr, *csr_col = nullptr;
    const void *csr_val = nullptr;
    // launch data derived at conversion time (not part of the format)
    int64_t csr_max_row = 0;
    int64_t csr_tiles = 0;            // tiles of csr_tile entries; csr_group lanes per row in the LDS reduction
    bool coo_every_row = false;       // MO_COO: every row holds an entry, so the SpMV writes all of y and needs no zero pass
    int32_t csr_tile = mo::CSR_TILE;  // CSR_TILE, CSR_TILE_LARGE or CSR_TILE_SMALL
    int32_t csr_group = 1;
    int32_t csr_split = 0;            // 1: tiles cut rows (any row length), carries in csr_carry_*
    int32_t *csr_carry_row = nullptr;
    void *csr_carry_val = nullptr;
    int32_t *csr_tile_rp = nullptr;   // (first row, its row_ptr) per tile, tiles + 1 pairs
    const int32_t *coo_rp = nullptr;  // m + 1 positions: where each row's run starts in the sorted COO part (launch data
                                      // of the multi-vector product; not part of the format)
    int64_t hyb_max_surplus = 0;      // HYB: longest row minus the ELL width (entries of one row in the COO part)
    int64_t coo_tiles = 0;
    int32_t coo_strip = 4;            // entries per thread of the COO kernel (8, 4 or 2)
    int32_t *coo_carry_row = nullptr; // one per COO tile
    void *coo_carry_val = nullptr;
    // MO_CSR on a matrix with scattered columns whose x exceeds one XCD's L2: the entries again, regrouped into 2, 4 or 8
    // column slices (each a CSR matrix of its own over all rows: launch data, not part of the format).  y = A_0 x, then
    // y += A_s x for the others: each pass gathers from one slice of x, which stays in L2.
    std::vector<mo_matrix *> csr_slices;
    mo::XPlan xplan;                  // x windows for the kernels that gather x by column index
    // everything this handle owns
    std::vector<void *> owned;
    hipStream_t home = nullptr;
};

namespace mo {

// ---------------------------------------------------------------- analysis (features.hip)
struct Analysis {
    int64_t max_row = 0, min_row = 0;
    uint64_t sum_sq = 0;
    int64_t n_diag = 0, n_true = 0;
    uint32_t *hist = nullptr;  // device, m + n - 1 counters (only when requested); owned by the Scratch passed in
    // rows of more than VLONG_ROW entries, which one wave should not walk alone (device list, owned by the Scratch passed
    // in; n_long = how many it holds, 0 also when there were more than it can hold)
    struct LongRows *long_rows = nullptr;
    int n_long = 0;
};

// Validates the CSR arrays and gathers the row statistics; with want_hist also the per-diagonal counts and the
// two diagonal features.  Synchronises the stream.
mo_status analyse(const mo_csr &a, const mo_params &p, bool want_hist, Analysis *out, Scratch &scratch, hipStream_t s);
// The same numbers (histogram included in the counts, not handed out) with scratch that is kept between calls.
mo_status analyse_cached(const mo_csr &a, const mo_params &p, Analysis *out, hipStream_t s);
void release_feature_cache();
// The diagonal counts by partition into buckets of diagonals (feat_part.hip), for matrices with scattered columns.
struct DiagPart;
struct Counters;
struct LongRows;
bool partition_possible(const mo_csr &a);
int partition_buckets(const mo_csr &a);
size_t partition_sample_bytes();
size_t partition_scratch_bytes(const mo_csr &a);
mo_status partition_wanted(const mo_csr &a, uint32_t *acc, bool *wanted, hipStream_t s);
mo_status partition_decide_async(const mo_csr &a, uint32_t *acc, uint32_t *flag_host, hipStream_t s);
mo_status partition_counts(const mo_csr &a, const mo_params &p, void *buf, uint32_t *hist, DiagPart *dpart, Counters *ctr, uint32_t *err,
                           hipStream_t s);
// The no-allocation variant: integers and status into caller memory, asynchronous.
mo_status features_static(const mo_csr &a, const mo_params &p, mo_feature_result *out_dev, hipStream_t s);

// ---------------------------------------------------------------- conversions (convert.hip)
mo_status convert_impl(const mo_csr &a, mo_format fmt, const mo_params &p, const Analysis &an, mo_matrix **out, hipStream_t s);
mo_status check_csr_args(const mo_csr *a);
mo_status check_params(const mo_params *in, mo_params *out);
// exact integer feasibility of a DIA / ELL slab
bool slab_feasible(int64_t width, int64_t m, int64_t nnz, const mo_params &p);

// ---------------------------------------------------------------- x window plan (xplan.hip)
// Samples the (validated) CSR arrays and groups the heavily populated diagonals.  Synchronises the stream.
mo_status plan_x_windows(const int32_t *row_ptr, const int32_t *col_idx, int64_t m, int64_t nnz, XPlan *out, hipStream_t s);

// ---------------------------------------------------------------- scans (scan.hip)
// out[i] = sum_{j<i} in[j] for i in [0, n]; out has n + 1 entries (out[n] = total).  tmp: >= scan_tmp_bytes(n).
size_t scan_tmp_bytes(int64_t n);
mo_status exclusive_scan_i32(const int32_t *in, int32_t *out, int64_t n, void *tmp, hipStream_t s);

// ---------------------------------------------------------------- SpMV launchers (spmv_*.hip)
mo_status spmv_csr(const mo_matrix &a, const void *x, void *y, bool accumulate, hipStream_t s);
mo_status spmv_coo(const mo_matrix &a, const void *x, void *y, bool accumulate, hipStream_t s);
mo_status spmv_dia(const mo_matrix &a, const void *x, void *y, hipStream_t s);
mo_status spmv_ell(const mo_matrix &a, const void *x, void *y, hipStream_t s);
mo_status spmv_hyb_fused(const mo_matrix &a, const void *x, void *y, hipStream_t s);
bool ell_uses_windows(const mo_matrix &a);   // one-row-per-lane ELL / fused HYB kernel with x served from LDS windows
// The slot-split ELL kernel pays off while one-row-per-lane blocks cannot fill the chip (measured: faster up to about
// 260 000 rows at K = 27, slower beyond; no gain for K < 16).
constexpr int64_t ELL_SPLIT_MAX_ROWS = 300000;
constexpr int64_t ELL_SPLIT_MIN_K = 16;
constexpr int64_t HYB_FUSED_MAX_SURPLUS = 16;   // longer COO runs per row go through the COO kernel
mo_status spmv_hdc_fused(const mo_matrix &a, const void *x, void *y, hipStream_t s);
bool plan_dia_clusters(const std::vector<int32_t> &off, int block, int64_t max_elems, std::vector<int32_t> *xpos,
                       std::vector<int32_t> *clusters, int64_t *total_elems);
constexpr int64_t DIA_LDS_BYTES = 48 * 1024;  // LDS budget for staged x windows per block
// rows per lane of the LDS-staged DIA kernel: a lane moves 8 bytes per slab load in either precision
template <typename T> constexpr int DIA_ROWS_PER_LANE = sizeof(T) == 4 ? 2 : 1;
constexpr int SPMM_ROWS = 64;                 // matrix rows per block of the DIA multi-vector kernel with staged windows of X
constexpr int64_t SPMM_WIN_BYTES = 64 * 1024; // its LDS budget per block (two blocks per CU at least; four below 40 KB)
// column slices of a CSR handle: from an x of this size on (one XCD's L2 is 4 MB), so many that a slice is at most
// CSR_SLICE_X_BYTES, at most CSR_MAX_SLICES; only for matrices of at least CSR_SLICE_MIN_NNZ entries whose rows are
// long enough (CSR_SLICE_MIN_WORK)
constexpr int64_t CSR_SLICE_MIN_X_BYTES = 5 * 1024 * 1024, CSR_SLICE_X_BYTES = 5 * 1024 * 1024;
constexpr int CSR_MAX_SLICES = 8;
constexpr int64_t CSR_SLICE_MIN_NNZ = 1 << 22;
constexpr int64_t CSR_SLICE_MIN_WORK = (int64_t)64 << 20;   // mean entries per row x bytes of x
constexpr int64_t HDC_FUSED_MAX_ROW = 64;   // longest row for which HDC runs as one fused kernel
mo_status fill_zero(void *p, int64_t n_elems, mo_dtype dt, hipStream_t s);

// ---------------------------------------------------------------- multi-vector product (spmm.hip)
mo_status spmm(const mo_matrix &a, const void *x, void *y, int k, hipStream_t s);
int64_t csr_tile_count(int64_t nnz, int tile_size);
// y[row] += carries of every chain of consecutive tiles with the same carry row (shared by the COO and CSR kernels)
mo_status carry_fixup(const int32_t *carry_row, const void *carry_val, int64_t tiles, void *y, mo_dtype dt, hipStream_t s);
mo_status csr_build_tiles(const int32_t *row_ptr, int64_t m, int64_t nnz, int64_t ntiles, int tile_size, int row_align, int32_t *tile_rp,
                          hipStream_t s);

inline size_t dtype_size(mo_dtype d) { return d == MO_F32 ? 4 : 8; }

}  // namespace mo

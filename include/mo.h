/*
 * mo — sparse-format SpMV engine and format auto-tuner for AMD MI355X (gfx950).
 *
 * C ABI of the data-parallel path behind the paper's format auto-tuner
 * (Stylianou & Weiland, "Optimizing Sparse Linear Algebra Through Automatic
 * Format Selection and Machine Learning"): SpMV y = A x in six storage formats,
 * CSR -> format conversion on the device, extraction of the ten sparsity
 * features, the run-first tuner and evaluation of a decision tree / forest.
 *
 * Conventions
 *   - One GPU, one process.  Every `stream` argument is a hipStream_t passed
 *     as void* (NULL = the default stream).  All kernels of a call are
 *     enqueued on that stream.
 *   - Pointers inside mo_csr, and the x / y arguments, are DEVICE pointers
 *     owned by the caller.  They are only read (y only written) and must stay
 *     valid until the work enqueued on `stream` has finished.
 *   - Indices are int32, sizes int64.  Requirements: m >= 1, n >= 1,
 *     0 <= nnz <= 2^31 - 1, m + n <= 2^31 - 1.
 *   - CSR precondition (checked on the device by mo_features / mo_convert /
 *     mo_tune, violation -> MO_E_CSR_INVALID): row_ptr[0] = 0, row_ptr
 *     non-decreasing, row_ptr[m] = nnz, 0 <= col < n, columns strictly
 *     ascending inside a row.  Stored zeros are ordinary entries.
 *   - Every function returns a status and never throws or aborts.  On error
 *     output handles are NULL and nothing is leaked.
 *   - Format ids follow the order in which the paper lists the formats
 *     (Section II-B and Eq. 1): COO, CSR, DIA, ELL, HYB, HDC.
 */
#ifndef MO_H
#define MO_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum { MO_COO = 0, MO_CSR = 1, MO_DIA = 2, MO_ELL = 3, MO_HYB = 4, MO_HDC = 5 } mo_format;
#define MO_NUM_FORMATS 6
#define MO_NUM_FEATURES 10

typedef enum { MO_F32 = 0, MO_F64 = 1 } mo_dtype;

typedef enum {
    MO_OK = 0,
    MO_E_NULL = 1,        /* a required pointer is NULL */
    MO_E_SHAPE = 2,       /* m, n, nnz outside the supported range */
    MO_E_CSR_INVALID = 3, /* the CSR precondition does not hold */
    MO_E_FORMAT = 4,      /* unknown format id */
    MO_E_DTYPE = 5,       /* unknown value type */
    MO_E_FILL = 6,        /* DIA / ELL would need more padding than mo_params allows */
    MO_E_ALLOC = 7,       /* the device allocator returned NULL */
    MO_E_DEVICE = 8,      /* a HIP call failed; see mo_last_hip_error() */
    MO_E_MODEL = 9,       /* model file unreadable, malformed or inconsistent */
    MO_E_PARAM = 10,      /* a parameter struct holds a non-positive denominator or negative value */
    MO_E_IO = 11          /* a matrix file is unreadable, malformed or of an unsupported kind */
} mo_status;

/* Borrowed view of a CSR matrix in device memory (Section II-B: values, column
 * indices and a row-pointer array marking row boundaries). */
typedef struct {
    int64_t m, n, nnz;
    const int32_t *row_ptr;  /* device, m + 1 entries */
    const int32_t *col_idx;  /* device, nnz entries   */
    const void *val;         /* device, nnz entries of `dtype` */
    mo_dtype dtype;
} mo_csr;

/* Format parameters the paper names but does not fix (Section II-B: K_H for
 * HYB, the true-diagonal threshold for HDC), as exact integer fractions.
 *   true diagonal  : non-empty and  cnt * td_den  >= min(m, n) * td_num      (default 1/2)
 *   HYB ELL width  : largest k >= 0 with #{rows with len >= k} * hyb_den >= m * hyb_num  (default 1/3)
 *   DIA / ELL are refused (MO_E_FILL) when slots > max_fill * nnz or slots > max_slots,
 *   slots = (#diagonals or max row length) * m.                              (defaults 16, 2^62)
 * Pass NULL for the defaults. */
typedef struct {
    int32_t td_num, td_den;
    int32_t hyb_num, hyb_den;
    int32_t max_fill;
    int64_t max_slots;
} mo_params;

/* The integer statistics behind the features (Table I).  sum_sq_row is the sum
 * over rows of (row length)^2, from which both the variance and the standard
 * deviation reading of sigma_NNZ follow. */
typedef struct {
    int64_t m, n, nnz, max_row, min_row, n_diag, n_true_diag;
    uint64_t sum_sq_row;
} mo_feature_ints;

typedef struct mo_matrix mo_matrix; /* a matrix held in one format; library-owned */
typedef struct mo_model mo_model;   /* a loaded tree / forest; library-owned, host memory */

typedef struct { int32_t warmups, reps; } mo_tune_opts; /* NULL -> 5 warm-ups, 50 timed repetitions */

/* Device pointers and dimensions of every array a handle holds; arrays a format
 * does not use are NULL / 0.  Borrowed from the handle.
 *   DIA part (DIA, HDC): dia_off[nd] ascending offsets d = col - row; dia_val[k*ld + i] = A(i, i + dia_off[k]) or +0.
 *   ELL part (ELL, HYB): width k, slot-major: ell_col[s*ld + i], ell_val[s*ld + i]; row entries in ascending
 *                        column order from slot 0; padding col = -1, val = +0.
 *   COO part (COO, HYB): coo_row / coo_col / coo_val [nnz_coo], sorted by (row, col).
 *   CSR part (CSR, HDC): csr_row_ptr[m+1], csr_col / csr_val [nnz_csr].
 * ld >= m is the common leading dimension of the DIA and ELL slabs; positions i in [m, ld) are unspecified. */
typedef struct {
    mo_format fmt;
    mo_dtype dtype;
    int64_t m, n, nnz, ld, nd, k, nnz_coo, nnz_csr;
    const int32_t *dia_off, *ell_col, *coo_row, *coo_col, *csr_row_ptr, *csr_col;
    const void *dia_val, *ell_val, *coo_val, *csr_val;
} mo_matrix_view;

/* Defaults for mo_params (1/2, 1/3, 16, 2^62). */
void mo_default_params(mo_params *out);

/* The ten features of Table I in table order: M, N, NNZ, NNZ/M, NNZ/(M*N), max, min and standard deviation
 * of the number of entries per row, number of non-empty diagonals, number of true diagonals (Section IV-A).
 * The integer counts come from device kernels over the CSR arrays; the four derived doubles are formed on the
 * host from those integers (std = sqrt((M*sum_sq_row - NNZ^2) / M^2), correctly rounded operations only).
 * out: host array of 10 doubles.  ints_opt: optional host struct.  Synchronises `stream`.  This is the call a deployed
 * tuner pays per matrix, so it keeps its device scratch (about 6*(m+n) bytes, and about 2*nnz more once a matrix of
 * at least 2^21 entries with scattered columns has been seen: its diagonals are counted by partition instead of by
 * atomics; grown on demand through the installed allocator) and a small pinned host block between calls;
 * mo_set_allocator releases the device blocks.  Calls from several threads are safe: one of them uses the kept
 * blocks, the others allocate and free per call. */
mo_status mo_features(const mo_csr *a, const mo_params *params, double out[MO_NUM_FEATURES],
                      mo_feature_ints *ints_opt, void *stream);

/* The host half of mo_features on its own (Table I): the ten doubles from the integer statistics, with the same
 * correctly rounded operations, so that the result equals mo_features' bit for bit.  Pure host. */
mo_status mo_features_finalize(const mo_feature_ints *ints, double out[MO_NUM_FEATURES]);

/* mo_features for callers that cannot allocate or wait: code under HIP stream capture, tight serving loops, harnesses
 * that forbid hipMalloc.  Same kernels and same integers as mo_features, but the diagonal histogram and the per-block
 * partial results live in a device array inside the library (one copy per GPU, about 16 MiB, held until the process
 * ends) and the call neither allocates, frees nor synchronises: it enqueues four kernels (five for matrices of more
 * than 8192 entries, which may hold rows too long for one wavefront) on `stream` and returns.
 *   out_dev : DEVICE-accessible memory owned by the caller (device memory or pinned host memory); when the enqueued
 *             work has finished it holds the integer statistics and status = MO_OK or MO_E_CSR_INVALID (then the
 *             integers mean nothing).  mo_features_finalize turns ints into the ten doubles.
 *   limit   : m + n - 1 <= MO_STATIC_MAX_DIAGS, else MO_E_SHAPE and nothing is enqueued.
 * All calls on one GPU share that GPU's array: calls that overlap in time on one GPU (different streams or threads)
 * race and give wrong counts; calls in stream order are fine, each starts by clearing what it uses.  The first call
 * on a device looks the array's address up (no allocation); make that call once outside any capture. */
#define MO_STATIC_MAX_DIAGS 4194304
typedef struct {
    mo_feature_ints ints;
    int32_t status; /* mo_status */
    int32_t pad;
} mo_feature_result;
mo_status mo_features_static(const mo_csr *a, const mo_params *params, mo_feature_result *out_dev, void *stream);

/* Build a handle holding `a` in format `fmt` (Section II-B).  The handle owns its arrays (installed allocator)
 * and does not alias the input, with one exception: an MO_CSR handle BORROWS row_ptr / col_idx / val, so those
 * must outlive it.  Validates the CSR precondition.  Synchronises `stream` (sizes are read back).
 * MO_E_FILL for DIA / ELL beyond the padding limits; HYB and HDC are always feasible; either part of a hybrid
 * may be empty. */
mo_status mo_convert(const mo_csr *a, mo_format fmt, const mo_params *params, mo_matrix **out, void *stream);

/* y = A x, overwriting y (device, m entries of the handle's dtype); x: device, n entries.  Asynchronous:
 * enqueues one to three kernels on `stream`, never allocates, never synchronises.  x and y must not overlap.
 * Results are bit-identical from run to run (no floating-point atomics).  A handle may carry small scratch
 * used by its kernels, so two mo_spmv calls on the SAME handle must not run concurrently on different streams. */
mo_status mo_spmv(const mo_matrix *a, const void *x, void *y, void *stream);

/* Infrastructure, not in the paper: the names of the kernels mo_spmv enqueues for this handle, joined by '+', as a
 * NUL-terminated string in buf (host, cap bytes; MO_E_PARAM when it does not fit).  For benchmark and profile reports. */
mo_status mo_spmv_kernels(const mo_matrix *a, char *buf, size_t cap);

/* Run-first tuner (Section VI-A): for every format that is feasible, convert, run `warmups` untimed and `reps`
 * timed SpMVs back to back between two events, free; best = format with the smallest time per repetition
 * (Section VII-A), ties to the lowest id.  ms_per_rep[f] is NaN for an infeasible format.  convert_ms[f]
 * (optional) is the wall time of the conversion, reported beside the choice and not part of it.
 * Allocates x and y scratch through the installed allocator.  Synchronises `stream`. */
mo_status mo_tune(const mo_csr *a, const mo_params *params, const mo_tune_opts *opts, mo_format *best,
                  double ms_per_rep[MO_NUM_FORMATS], double convert_ms[MO_NUM_FORMATS], void *stream);

/* A second operation under the same interface (Section VI-B leaves the tuning interface open to further operations):
 * Y = A X for k right-hand sides, 1 <= k <= MO_MAX_RHS.  X: device, n x k, row-major (the k values of one row of X are
 * contiguous); Y: device, m x k, row-major, overwritten.  Same rules as mo_spmv: asynchronous on `stream`, no
 * allocation, no synchronisation, X and Y must not overlap, bit-identical reruns.  mo_tune_spmm is mo_tune with this
 * operation timed in place of SpMV. */
#define MO_MAX_RHS 64
mo_status mo_spmm(const mo_matrix *a, const void *x, void *y, int32_t k, void *stream);
mo_status mo_tune_spmm(const mo_csr *a, int32_t k, const mo_params *params, const mo_tune_opts *opts, mo_format *best,
                       double ms_per_rep[MO_NUM_FORMATS], double convert_ms[MO_NUM_FORMATS], void *stream);

/* Pure host: the rule by which the run-first tuner and the training labels name the best format (Section VII-A: the
 * format with the minimum runtime): index of the smallest non-NaN entry, ties to the lowest id; MO_E_PARAM if all are NaN. */
mo_status mo_pick(const double ms[MO_NUM_FORMATS], mo_format *best);

/* Model file -> forest (Section III-B: the model is loaded from a file named at run time).  Binary,
 * little-endian: char magic[8] = "MOMDL1\0\0"; int32 version = 1, n_features = 10, n_classes = 6, n_trees >= 1;
 * then per tree: int32 n_nodes >= 1, int32 feature[n_nodes] (-1 = leaf), double threshold[n_nodes],
 * int32 left[n_nodes], int32 right[n_nodes], int32 klass[n_nodes].  Node 0 is the root; children must have a
 * larger index than their parent (so walks terminate); leaves carry a class in [0, 6). */
mo_status mo_model_load(const char *path, mo_model **out);
void mo_model_free(mo_model *model);
/* Infrastructure, not in the paper: number of trees and total number of nodes of a loaded model. */
mo_status mo_model_info(const mo_model *model, int32_t *n_trees, int32_t *n_nodes_total);

/* Pure host (Section VI-A): walk every tree from its root (left iff features[f] <= threshold), one vote per
 * tree for the class at the leaf reached, result = class with most votes, ties to the lowest id.  A single
 * tree is a forest of one. */
mo_status mo_select(const mo_model *model, const double features[MO_NUM_FEATURES], mo_format *out);

/* Offline training stage on the host (Section V; hyper-parameters of Table III).  A tree is grown greedily: at every
 * node the admissible cut (between two distinct neighbouring values of one feature, at least min_samples_leaf rows on
 * each side) with the lowest weighted impurity is taken, rows with value <= threshold go left; a node is a leaf at
 * max_depth (< 0: no limit), when it holds one class, fewer than min_samples_split or fewer than 2*min_samples_leaf
 * rows, or no admissible cut.  With max_features < 10 the features of a node are tried in a seeded random order until
 * max_features were tried and a cut is known.  bootstrap: every tree trains on n rows drawn with replacement.  Equal
 * costs resolve to the lower feature index, then the lower threshold; a leaf predicts its most frequent class, ties to
 * the lowest id.  The result is a pure function of the data and the options (seed included). */
typedef enum { MO_GINI = 0, MO_ENTROPY = 1 } mo_criterion;
typedef struct {
    int32_t n_estimators;      /* >= 1; 1 with bootstrap = 0 and max_features = 10 is a plain decision tree */
    int32_t bootstrap;         /* 0 or 1 */
    int32_t max_depth;         /* < 0: unlimited */
    int32_t min_samples_leaf;  /* >= 1 */
    int32_t min_samples_split; /* >= 2 */
    int32_t max_features;      /* 1 .. 10 */
    int32_t criterion;         /* mo_criterion */
    uint64_t seed;
} mo_fit_opts;
/* The baseline column of Table III: 100 estimators, bootstrap, no depth limit, leaf 1, split 2, 10 features, gini; seed 0. */
void mo_default_fit_opts(mo_fit_opts *out);
/* features: host, n rows of 10 doubles (row-major, no NaN); labels: host, n format ids in [0, 6); 1 <= n <= 2^20.
 * NULL opts = the defaults.  The model is owned by the caller (mo_model_free). */
mo_status mo_model_fit(const double *features, const int32_t *labels, int64_t n, const mo_fit_opts *opts, mo_model **out);
/* Writes the model in the file format mo_model_load reads.  MO_E_MODEL when the file cannot be written. */
mo_status mo_model_save(const mo_model *model, const char *path);
/* mo_select for n feature rows at once (host, n rows of 10 doubles -> n format ids). */
mo_status mo_predict(const mo_model *model, const double *features, int64_t n, int32_t *out);

/* Run-time switching between any two formats (Section II-C): rebuilds CSR from whatever `a` holds (row lengths ->
 * exclusive scan -> rows written in ascending column order) and converts that to `fmt`.  A handle produced with
 * fmt = MO_CSR OWNS its arrays.  A DIA slab cannot tell a stored zero from padding, so positions holding exactly 0
 * are not entries on the way back; every other format keeps stored zeros.  Same errors and synchronisation as
 * mo_convert.  `a` is not modified and may be freed afterwards. */
mo_status mo_switch(const mo_matrix *a, mo_format fmt, const mo_params *params, mo_matrix **out, void *stream);

/* The ten features of Table I for a matrix in whatever format it is held, gathered from that format's own arrays
 * without converting back (Section VI-C).  Equal, bit for bit, to mo_features of the CSR the handle was built from
 * (for DIA / HDC: as long as no stored entry of a kept diagonal is exactly 0).  Synchronises `stream`; allocates
 * and frees 4*(2m + n) bytes of scratch. */
mo_status mo_matrix_features(const mo_matrix *a, const mo_params *params, double out[MO_NUM_FEATURES],
                             mo_feature_ints *ints_opt, void *stream);

/* Host: read a Matrix Market file (the format of the SuiteSparse collection the paper profiles, Section VII "Setup")
 * into CSR.  Coordinate format; field real, integer or pattern (entries mean 1); symmetry general, symmetric or
 * skew-symmetric (the stored triangle is mirrored).  Indices in the file are 1-based.  Entries naming the same
 * position are summed (the file's entries in file order, then the mirrored ones); explicit zeros stay entries; columns
 * come out ascending inside each row.  The three arrays are host memory owned by the caller: release each with
 * mo_host_free.  MO_E_IO for an unreadable, malformed or unsupported (array format, complex, hermitian) file,
 * MO_E_SHAPE when sizes exceed the limits stated at the top of this header.  An empty matrix (L = 0) is valid. */
mo_status mo_mtx_read(const char *path, int64_t *m, int64_t *n, int64_t *nnz, int32_t **row_ptr, int32_t **col_idx,
                      double **val);
void mo_host_free(void *p);

/* Infrastructure, not in the paper: the arrays a handle holds, laid out as Section II-B defines each format (see
 * mo_matrix_view), so that tests can compare them element by element; and the release of a handle. */
mo_status mo_matrix_export(const mo_matrix *a, mo_matrix_view *out);
void mo_matrix_free(mo_matrix *a);

/* Infrastructure, not in the paper.  Install the device allocator used for handles and scratch.  alloc returns a device pointer aligned to at
 * least 256 bytes or NULL; free_ releases it.  Both receive the stream of the calling entry point.  NULL, NULL
 * restores the default (hipMalloc / hipFree).  Not thread-safe against concurrent library calls. */
mo_status mo_set_allocator(void *(*alloc)(size_t bytes, void *stream, void *user),
                           void (*free_)(void *ptr, void *stream, void *user), void *user);

const char *mo_strerror(mo_status s);
/* The hipError_t (as int) of the last failed HIP call in this thread, 0 if none. */
int mo_last_hip_error(void);

#ifdef __cplusplus
}
#endif
#endif /* MO_H */

/*
 * CPU oracle for the sparse-format engine.  TEST INFRASTRUCTURE ONLY.
 *
 * This file is the slow, plain statement of what the GPU library must compute,
 * written from the paper's definitions.  It shares no code with the HIP path
 * and must never be called from it; only the tests, the smoke check and the
 * benchmark's cpu_baseline leg may load it.
 *
 * The matrix is always a list of triplets (i, j, a_ij) in fp64 (Section II-B,
 * COO: one value with its row and column index per stored entry, no ordering
 * promised).  Stored zeros are entries like any other.
 *
 * What is a definition and what is a procedure:
 *   - SpMV, its multi-vector form Y = A X, the five conversions, the way back
 *     from each format to triplets and to CSR, and the ten features are
 *     definitions: the code below writes each one out directly (Section II-B
 *     for the formats, Table I and Section IV-A for the features).  A DIA slab
 *     cannot tell a stored zero from padding: on the way back positions
 *     holding exactly 0 are not entries.
 *   - The HYB width K_H, the true-diagonal test, tree/forest evaluation
 *     (Section VI-A: traverse each tree, majority vote) and the run-first pick
 *     (Section VII-A: the format with the minimum runtime) are procedures and
 *     follow the stated steps.
 *
 * Readings taken where the paper leaves a choice open (all are inputs here,
 * never constants shared with the GPU side):
 *   - sigma_NNZ is the population standard deviation (Table I names it "std";
 *     the printed formula lacks the root);
 *   - a diagonal d = j - i is "true" iff it is non-empty and
 *     cnt_d * td_den >= min(M,N) * td_num;
 *   - K_H = largest k >= 0 with #{rows of length >= k} * hyb_den >= M * hyb_num;
 *   - DIA: offsets ascending, slot (k, i) holds a_{i, i+off_k} or +0.0;
 *   - ELL: row entries in ascending column order from slot 0, padding
 *     col = -1, val = +0.0;
 *   - COO output order: (row, col) ascending.
 *
 * Accumulation is in long double (x87 80-bit on x86-64), rounded once to fp64.
 *
 * Pins (tests, CPU only): dense matvec on tiny matrices, closed forms for the
 * 2-D 5-point and 3-D 27-point stencils, scipy.sparse cross-checks, brute
 * force on small random inputs, round trips of every conversion, hand-built
 * trees and scikit-learn tree arrays, and a mutation run that plants mistakes
 * in copies of this file and requires the pins to catch each.  Run-first timings are hardware
 * measurements: parity unpinned for those (only argmin bookkeeping is pinned).
 */
#include <math.h>
#include <pthread.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#define ORC_OK 0
#define ORC_E_ARG 1
#define ORC_E_MEM 2

/* ------------------------------------------------------------------ SpMV */

/* y = A x  (Section I: SpMV).  acc_i = sum a_ij x_j, mag_i = sum |a_ij||x_j|,
 * both over the triplets of row i, in extended precision. */
int orc_spmv(int64_t m, int64_t n, int64_t nnz, const int32_t *ti, const int32_t *tj, const double *ta,
             const double *x, double *y, double *mag)
{
    if (m < 0 || n < 0 || nnz < 0) return ORC_E_ARG;
    long double *acc = (long double *)calloc((size_t)(m > 0 ? m : 1), sizeof(long double));
    long double *mg = (long double *)calloc((size_t)(m > 0 ? m : 1), sizeof(long double));
    if (!acc || !mg) { free(acc); free(mg); return ORC_E_MEM; }
    for (int64_t t = 0; t < nnz; ++t) {
        int64_t i = ti[t], j = tj[t];
        if (i < 0 || i >= m || j < 0 || j >= n) { free(acc); free(mg); return ORC_E_ARG; }
        long double a = (long double)ta[t], xv = (long double)x[j];
        acc[i] += a * xv;
        mg[i] += fabsl(a) * fabsl(xv);
    }
    for (int64_t i = 0; i < m; ++i) {
        y[i] = (double)acc[i];
        if (mag) mag[i] = (double)mg[i];
    }
    free(acc); free(mg);
    return ORC_OK;
}

/* Y = A X for k right-hand sides at once: the operation of Section I applied to every column of X (the paper's tuning
 * interface, Section VI-B, is meant for further operations of this kind).  X is n x k and Y is m x k, both row-major.
 * acc_iv = sum_j a_ij x_jv and mag_iv = sum_j |a_ij||x_jv| over the triplets of row i, in extended precision. */
int orc_spmm(int64_t m, int64_t n, int64_t nnz, const int32_t *ti, const int32_t *tj, const double *ta, int64_t k,
             const double *x, double *y, double *mag)
{
    if (m < 0 || n < 0 || nnz < 0 || k < 1) return ORC_E_ARG;
    size_t cells = (size_t)(m > 0 ? m : 1) * (size_t)k;
    long double *sum = (long double *)calloc(cells, sizeof(long double));
    long double *abs_sum = (long double *)calloc(cells, sizeof(long double));
    if (!sum || !abs_sum) { free(sum); free(abs_sum); return ORC_E_MEM; }
    for (int64_t e = 0; e < nnz; ++e) {
        int64_t row = ti[e], col = tj[e];
        if (row < 0 || row >= m || col < 0 || col >= n) { free(sum); free(abs_sum); return ORC_E_ARG; }
        long double a = (long double)ta[e];
        for (int64_t v = 0; v < k; ++v) {
            long double xv = (long double)x[col * k + v];
            sum[row * k + v] += a * xv;
            abs_sum[row * k + v] += fabsl(a) * fabsl(xv);
        }
    }
    for (int64_t c = 0; c < m * k; ++c) {
        y[c] = (double)sum[c];
        if (mag) mag[c] = (double)abs_sum[c];
    }
    free(sum); free(abs_sum);
    return ORC_OK;
}

/* The same loop split over row ranges, for the benchmark's host baseline.
 * Needs row-sorted triplets so that ranges never share a row. */
typedef struct {
    int64_t t0, t1;
    const int32_t *ti, *tj;
    const double *ta, *x;
    double *y;
} orc_span;

static void *orc_span_run(void *p)
{
    orc_span *s = (orc_span *)p;
    int64_t t = s->t0;
    while (t < s->t1) {
        int32_t i = s->ti[t];
        long double acc = 0.0L;
        while (t < s->t1 && s->ti[t] == i) {
            acc += (long double)s->ta[t] * (long double)s->x[s->tj[t]];
            ++t;
        }
        s->y[i] = (double)acc;
    }
    return NULL;
}

int orc_spmv_rowsorted_mt(int64_t m, int64_t nnz, const int32_t *ti, const int32_t *tj, const double *ta,
                          const double *x, double *y, int nthreads)
{
    if (nthreads < 1) nthreads = 1;
    if (nthreads > 256) nthreads = 256;
    for (int64_t t = 1; t < nnz; ++t)
        if (ti[t] < ti[t - 1]) return ORC_E_ARG;
    memset(y, 0, (size_t)m * sizeof(double));
    orc_span sp[256];
    pthread_t th[256];
    int64_t prev = 0;
    int used = 0;
    for (int k = 0; k < nthreads; ++k) {
        int64_t cut = (k == nthreads - 1) ? nnz : (nnz * (k + 1)) / nthreads;
        if (cut < prev) cut = prev;
        while (cut > prev && cut < nnz && ti[cut] == ti[cut - 1]) ++cut;   /* move to a row boundary */
        sp[used].t0 = prev; sp[used].t1 = cut;
        sp[used].ti = ti; sp[used].tj = tj; sp[used].ta = ta; sp[used].x = x; sp[used].y = y;
        prev = cut;
        ++used;
    }
    for (int k = 1; k < used; ++k) pthread_create(&th[k], NULL, orc_span_run, &sp[k]);
    orc_span_run(&sp[0]);
    for (int k = 1; k < used; ++k) pthread_join(th[k], NULL);
    return ORC_OK;
}

/* ------------------------------------------------------- counts per row/diag */

static int64_t *orc_row_len(int64_t m, int64_t nnz, const int32_t *ti)
{
    int64_t *len = (int64_t *)calloc((size_t)(m > 0 ? m : 1), sizeof(int64_t));
    if (!len) return NULL;
    for (int64_t t = 0; t < nnz; ++t) len[ti[t]]++;
    return len;
}

/* cnt[d + (m-1)] = number of triplets with j - i = d, d in [-(m-1), n-1]. */
static int64_t *orc_diag_cnt(int64_t m, int64_t n, int64_t nnz, const int32_t *ti, const int32_t *tj)
{
    int64_t nd = m + n - 1;
    int64_t *cnt = (int64_t *)calloc((size_t)(nd > 0 ? nd : 1), sizeof(int64_t));
    if (!cnt) return NULL;
    for (int64_t t = 0; t < nnz; ++t) cnt[(int64_t)tj[t] - (int64_t)ti[t] + (m - 1)]++;
    return cnt;
}

static int orc_is_true_diag(int64_t cnt, int64_t m, int64_t n, int64_t td_num, int64_t td_den)
{
    int64_t mn = m < n ? m : n;
    return cnt >= 1 && (__int128)cnt * td_den >= (__int128)mn * td_num;
}

/* ---------------------------------------------------------------- features */

/* The ten features of Table I in table order:
 * M, N, NNZ, NNZ/M, NNZ/(M*N), max_i NNZ_i, min_i NNZ_i, std_i NNZ_i, N_D, N_TD.
 * ints (optional, 8 entries): m, n, nnz, max, min, N_D, N_TD, sum of NNZ_i^2. */
int orc_features(int64_t m, int64_t n, int64_t nnz, const int32_t *ti, const int32_t *tj,
                 int64_t td_num, int64_t td_den, double *out, int64_t *ints)
{
    if (m <= 0 || n <= 0 || nnz < 0) return ORC_E_ARG;
    int64_t *len = orc_row_len(m, nnz, ti);
    int64_t *cnt = orc_diag_cnt(m, n, nnz, ti, tj);
    if (!len || !cnt) { free(len); free(cnt); return ORC_E_MEM; }
    int64_t mx = len[0], mn = len[0];
    unsigned __int128 sumsq = 0;
    for (int64_t i = 0; i < m; ++i) {
        if (len[i] > mx) mx = len[i];
        if (len[i] < mn) mn = len[i];
        sumsq += (unsigned __int128)len[i] * (unsigned __int128)len[i];
    }
    int64_t n_d = 0, n_td = 0;
    for (int64_t d = 0; d < m + n - 1; ++d) {
        if (cnt[d] >= 1) n_d++;
        if (orc_is_true_diag(cnt[d], m, n, td_num, td_den)) n_td++;
    }
    /* M * sum(len^2) - NNZ^2 = M^2 * (mean of squared deviations): an exact integer */
    unsigned __int128 num = (unsigned __int128)m * sumsq - (unsigned __int128)nnz * (unsigned __int128)nnz;
    double var = (double)num / ((double)m * (double)m);
    out[0] = (double)m;
    out[1] = (double)n;
    out[2] = (double)nnz;
    out[3] = (double)nnz / (double)m;
    out[4] = (double)nnz / ((double)m * (double)n);
    out[5] = (double)mx;
    out[6] = (double)mn;
    out[7] = sqrt(var);
    out[8] = (double)n_d;
    out[9] = (double)n_td;
    if (ints) {
        ints[0] = m; ints[1] = n; ints[2] = nnz; ints[3] = mx; ints[4] = mn;
        ints[5] = n_d; ints[6] = n_td; ints[7] = (int64_t)sumsq;
    }
    free(len); free(cnt);
    return ORC_OK;
}

/* ------------------------------------------------------------- conversions */

typedef struct { int32_t i, j; double a; } orc_trip;

static int orc_trip_cmp(const void *pa, const void *pb)
{
    const orc_trip *a = (const orc_trip *)pa, *b = (const orc_trip *)pb;
    if (a->i != b->i) return a->i < b->i ? -1 : 1;
    if (a->j != b->j) return a->j < b->j ? -1 : 1;
    return 0;
}

static orc_trip *orc_sorted(int64_t nnz, const int32_t *ti, const int32_t *tj, const double *ta)
{
    orc_trip *t = (orc_trip *)malloc((size_t)(nnz > 0 ? nnz : 1) * sizeof(orc_trip));
    if (!t) return NULL;
    for (int64_t k = 0; k < nnz; ++k) { t[k].i = ti[k]; t[k].j = tj[k]; t[k].a = ta[k]; }
    qsort(t, (size_t)nnz, sizeof(orc_trip), orc_trip_cmp);
    return t;
}

/* COO: the triplets ordered by (row, col). */
int orc_to_coo(int64_t nnz, const int32_t *ti, const int32_t *tj, const double *ta,
               int32_t *row, int32_t *col, double *val)
{
    orc_trip *t = orc_sorted(nnz, ti, tj, ta);
    if (!t) return ORC_E_MEM;
    for (int64_t k = 0; k < nnz; ++k) { row[k] = t[k].i; col[k] = t[k].j; val[k] = t[k].a; }
    free(t);
    return ORC_OK;
}

/* Offsets of the diagonals kept by a DIA part, ascending.  all_nonempty != 0:
 * every non-empty diagonal (plain DIA); otherwise only true diagonals (HDC).
 * off may be NULL to ask for the count alone. */
int64_t orc_dia_offsets(int64_t m, int64_t n, int64_t nnz, const int32_t *ti, const int32_t *tj,
                        int all_nonempty, int64_t td_num, int64_t td_den, int32_t *off)
{
    int64_t *cnt = orc_diag_cnt(m, n, nnz, ti, tj);
    if (!cnt) return -1;
    int64_t k = 0;
    for (int64_t d = 0; d < m + n - 1; ++d) {
        int keep = all_nonempty ? (cnt[d] >= 1) : orc_is_true_diag(cnt[d], m, n, td_num, td_den);
        if (keep) { if (off) off[k] = (int32_t)(d - (m - 1)); k++; }
    }
    free(cnt);
    return k;
}

/* DIA values for a given ascending offset list: val[k*m + i] = a_{i, i+off[k]}
 * when that triplet exists, +0.0 otherwise.  taken[t] (optional) is set to 1 for
 * every triplet that landed in the DIA part. */
int orc_fill_dia(int64_t m, int64_t n, int64_t nnz, const int32_t *ti, const int32_t *tj, const double *ta,
                 int64_t nd, const int32_t *off, double *val, uint8_t *taken)
{
    (void)n;
    for (int64_t s = 0; s < nd * m; ++s) val[s] = 0.0;
    for (int64_t t = 0; t < nnz; ++t) {
        int64_t d = (int64_t)tj[t] - (int64_t)ti[t];
        int64_t k = -1;
        for (int64_t q = 0; q < nd; ++q) if (off[q] == d) { k = q; break; }
        if (k >= 0) { val[k * m + ti[t]] = ta[t]; if (taken) taken[t] = 1; }
        else if (taken) taken[t] = 0;
    }
    return ORC_OK;
}

/* ELL of width k: the first min(len_i, k) entries of row i (ascending column)
 * sit in slots 0.., slot-major: col[s*m + i], val[s*m + i]; padding -1 / +0.0.
 * The entries that did not fit are returned as (row, col)-sorted COO in
 * rrow/rcol/rval (each sized for nnz; may be NULL when nothing can overflow). */
int orc_to_ell(int64_t m, int64_t nnz, const int32_t *ti, const int32_t *tj, const double *ta,
               int64_t k, int32_t *col, double *val, int64_t *n_rest, int32_t *rrow, int32_t *rcol, double *rval)
{
    orc_trip *t = orc_sorted(nnz, ti, tj, ta);
    if (!t) return ORC_E_MEM;
    for (int64_t s = 0; s < k * m; ++s) { col[s] = -1; val[s] = 0.0; }
    int64_t rest = 0, pos = 0;
    for (int64_t q = 0; q < nnz; ++q) {
        if (q > 0 && t[q].i != t[q - 1].i) pos = 0;
        if (pos < k) {
            col[pos * m + t[q].i] = t[q].j;
            val[pos * m + t[q].i] = t[q].a;
        } else {
            if (!rrow) { free(t); return ORC_E_ARG; }
            rrow[rest] = t[q].i; rcol[rest] = t[q].j; rval[rest] = t[q].a;
            rest++;
        }
        pos++;
    }
    if (n_rest) *n_rest = rest;
    free(t);
    return ORC_OK;
}

int64_t orc_max_row(int64_t m, int64_t nnz, const int32_t *ti)
{
    int64_t *len = orc_row_len(m, nnz, ti);
    if (!len) return -1;
    int64_t mx = 0;
    for (int64_t i = 0; i < m; ++i) if (len[i] > mx) mx = len[i];
    free(len);
    return mx;
}

/* K_H for HYB (Section II-B: rows longer than K_H spill into COO).
 * Largest k >= 0 such that (#rows with len >= k) * den >= M * num. */
int64_t orc_hyb_k(int64_t m, int64_t nnz, const int32_t *ti, int64_t hyb_num, int64_t hyb_den)
{
    int64_t *len = orc_row_len(m, nnz, ti);
    if (!len) return -1;
    int64_t mx = 0;
    for (int64_t i = 0; i < m; ++i) if (len[i] > mx) mx = len[i];
    int64_t best = 0;
    for (int64_t k = 0; k <= mx; ++k) {
        int64_t rows = 0;
        for (int64_t i = 0; i < m; ++i) if (len[i] >= k) rows++;
        if ((__int128)rows * hyb_den >= (__int128)m * hyb_num) best = k;
    }
    free(len);
    return best;
}

/* HDC remainder: the triplets with taken[t] == 0 as CSR (columns ascending). */
int orc_rest_to_csr(int64_t m, int64_t nnz, const int32_t *ti, const int32_t *tj, const double *ta,
                    const uint8_t *taken, int32_t *row_ptr, int32_t *col, double *val)
{
    int64_t keep = 0;
    for (int64_t t = 0; t < nnz; ++t) if (!taken[t]) keep++;
    int32_t *ri = (int32_t *)malloc((size_t)(keep > 0 ? keep : 1) * sizeof(int32_t));
    int32_t *rj = (int32_t *)malloc((size_t)(keep > 0 ? keep : 1) * sizeof(int32_t));
    double *ra = (double *)malloc((size_t)(keep > 0 ? keep : 1) * sizeof(double));
    if (!ri || !rj || !ra) { free(ri); free(rj); free(ra); return ORC_E_MEM; }
    int64_t q = 0;
    for (int64_t t = 0; t < nnz; ++t) if (!taken[t]) { ri[q] = ti[t]; rj[q] = tj[t]; ra[q] = ta[t]; q++; }
    orc_trip *s = orc_sorted(keep, ri, rj, ra);
    free(ri); free(rj); free(ra);
    if (!s) return ORC_E_MEM;
    for (int64_t i = 0; i <= m; ++i) row_ptr[i] = 0;
    for (int64_t t = 0; t < keep; ++t) row_ptr[s[t].i + 1]++;
    for (int64_t i = 0; i < m; ++i) row_ptr[i + 1] += row_ptr[i];
    for (int64_t t = 0; t < keep; ++t) { col[t] = s[t].j; val[t] = s[t].a; }
    free(s);
    return ORC_OK;
}

/* DIA and ELL are refused when padding is excessive (Section II-B notes both
 * can suffer from it): slots > max_fill * nnz or slots > max_slots. */
int orc_feasible(int64_t slots, int64_t nnz, int64_t max_fill, int64_t max_slots)
{
    if ((__int128)slots > (__int128)max_fill * nnz) return 0;
    if (slots > max_slots) return 0;
    return 1;
}

/* ------------------------------------------------------------------ tuners */

/* Forest evaluation (Section VI-A).  Tree t owns nodes [tree_off[t], tree_off[t+1]);
 * child indices are relative to the tree's first node; feature < 0 marks a leaf.
 * Walk: left iff x[feature] <= threshold.  Votes per class, winner = most votes,
 * ties to the lowest class id.  Returns the class, or -1 on a malformed model. */
int orc_select(int32_t n_trees, const int32_t *tree_off, const int32_t *feature, const double *threshold,
               const int32_t *left, const int32_t *right, const int32_t *klass, int32_t n_classes,
               const double *x)
{
    int64_t votes[64];
    if (n_classes < 1 || n_classes > 64 || n_trees < 1) return -1;
    for (int c = 0; c < n_classes; ++c) votes[c] = 0;
    for (int32_t t = 0; t < n_trees; ++t) {
        int32_t base = tree_off[t], cnt = tree_off[t + 1] - tree_off[t];
        int32_t node = 0, steps = 0;
        if (cnt < 1) return -1;
        while (feature[base + node] >= 0) {
            int32_t f = feature[base + node];
            int32_t nxt = (x[f] <= threshold[base + node]) ? left[base + node] : right[base + node];
            if (nxt < 0 || nxt >= cnt || ++steps > cnt) return -1;
            node = nxt;
        }
        int32_t c = klass[base + node];
        if (c < 0 || c >= n_classes) return -1;
        votes[c]++;
    }
    int best = 0;
    for (int c = 1; c < n_classes; ++c) if (votes[c] > votes[best]) best = c;
    return best;
}

/* Run-first pick (Section VII-A): index of the smallest time; NaN entries are
 * formats that were not run; ties to the lowest index; -1 if all are NaN. */
int orc_pick(int32_t n, const double *ms)
{
    int best = -1;
    for (int32_t k = 0; k < n; ++k) {
        if (isnan(ms[k])) continue;
        if (best < 0 || ms[k] < ms[best]) best = k;
    }
    return best;
}

/* ------------------------------------------------- back from a format to triplets */

/* Section II-C: the formats can be switched at run time in any direction.  Going back to triplets is the
 * definition of each format read backwards.  Each function returns the number of triplets and fills ti/tj/ta
 * (sized by the caller for the worst case) unless they are NULL (count only).
 *
 * DIA cannot tell a stored zero from padding, so exactly-zero positions are not entries; positions whose column
 * falls outside [0, n) are never entries. */
int64_t orc_from_dia(int64_t m, int64_t n, int64_t nd, const int32_t *off, const double *val,
                     int32_t *ti, int32_t *tj, double *ta)
{
    int64_t c = 0;
    for (int64_t k = 0; k < nd; ++k)
        for (int64_t i = 0; i < m; ++i) {
            int64_t j = i + off[k];
            if (j < 0 || j >= n) continue;
            if (val[k * m + i] == 0.0) continue;
            if (ti) { ti[c] = (int32_t)i; tj[c] = (int32_t)j; ta[c] = val[k * m + i]; }
            c++;
        }
    return c;
}

/* ELL: every slot whose column is not the padding marker is an entry (stored zeros included). */
int64_t orc_from_ell(int64_t m, int64_t k, const int32_t *col, const double *val, int32_t *ti, int32_t *tj, double *ta)
{
    int64_t c = 0;
    for (int64_t s = 0; s < k; ++s)
        for (int64_t i = 0; i < m; ++i) {
            if (col[s * m + i] < 0) continue;
            if (ti) { ti[c] = (int32_t)i; tj[c] = col[s * m + i]; ta[c] = val[s * m + i]; }
            c++;
        }
    return c;
}

/* CSR: expand the row pointer. */
int64_t orc_from_csr(int64_t m, const int32_t *row_ptr, const int32_t *col, const double *val, int32_t *ti, int32_t *tj, double *ta)
{
    int64_t c = 0;
    for (int64_t i = 0; i < m; ++i)
        for (int64_t p = row_ptr[i]; p < row_ptr[i + 1]; ++p) {
            if (ti) { ti[c] = (int32_t)i; tj[c] = col[p]; ta[c] = val[p]; }
            c++;
        }
    return c;
}

/* Triplets -> CSR with ascending columns (the inverse conversions all end here). */
int orc_to_csr(int64_t m, int64_t nnz, const int32_t *ti, const int32_t *tj, const double *ta,
               int32_t *row_ptr, int32_t *col, double *val)
{
    orc_trip *s = orc_sorted(nnz, ti, tj, ta);
    if (!s) return ORC_E_MEM;
    for (int64_t i = 0; i <= m; ++i) row_ptr[i] = 0;
    for (int64_t t = 0; t < nnz; ++t) row_ptr[s[t].i + 1]++;
    for (int64_t i = 0; i < m; ++i) row_ptr[i + 1] += row_ptr[i];
    for (int64_t t = 0; t < nnz; ++t) { col[t] = s[t].j; val[t] = s[t].a; }
    free(s);
    return ORC_OK;
}

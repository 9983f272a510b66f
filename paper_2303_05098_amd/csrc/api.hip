// C-ABI entry points: argument checks, allocator, feature finalisation, run-first tuner, handle lifetime.
#include "mo_internal.hpp"

#include <chrono>
#include <cmath>
#include <cstring>
#include <limits>
#include <string>

namespace mo {

static thread_local int g_last_hip_error = 0;
void set_hip_error(hipError_t e) { g_last_hip_error = (int)e; }

static void *(*g_alloc)(size_t, void *, void *) = nullptr;
static void (*g_free)(void *, void *, void *) = nullptr;
static void *g_user = nullptr;

void *dev_alloc(size_t bytes, hipStream_t s)
{
    if (bytes == 0) bytes = 256;
    if (g_alloc) return g_alloc(bytes, (void *)s, g_user);
    void *p = nullptr;
    hipError_t e = hipMalloc(&p, bytes);
    if (e != hipSuccess) { set_hip_error(e); return nullptr; }
    return p;
}

void dev_free(void *p, hipStream_t s)
{
    if (!p) return;
    if (g_free) { g_free(p, (void *)s, g_user); return; }
    (void)hipFree(p);
}

// x[i] = a fixed pseudo-random value in [-1, 1) (integer hash of i).
template <typename T>
__global__ void k_fill_operand(T *__restrict__ p, int64_t n)
{
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += stride) {
        uint64_t z = ((uint64_t)i + 1u) * 0x9E3779B97F4A7C15ull;
        z ^= z >> 31; z *= 0xBF58476D1CE4E5B9ull; z ^= z >> 29;
        p[i] = (T)((double)(z >> 11) * (2.0 / 9007199254740992.0) - 1.0);
    }
}

}  // namespace mo

using namespace mo;

extern "C" {

void mo_default_params(mo_params *out)
{
    if (!out) return;
    out->td_num = 1; out->td_den = 2;
    out->hyb_num = 1; out->hyb_den = 3;
    out->max_fill = 16;
    out->max_slots = (int64_t)1 << 62;
}

mo_status mo_set_allocator(void *(*alloc)(size_t, void *, void *), void (*free_)(void *, void *, void *), void *user)
{
    if ((alloc == nullptr) != (free_ == nullptr)) return MO_E_NULL;
    release_feature_cache();   // through the allocator it came from
    g_alloc = alloc; g_free = free_; g_user = user;
    return MO_OK;
}

const char *mo_strerror(mo_status s)
{
    switch (s) {
    case MO_OK: return "ok";
    case MO_E_NULL: return "null pointer argument";
    case MO_E_SHAPE: return "matrix dimensions out of range";
    case MO_E_CSR_INVALID: return "CSR arrays violate the precondition";
    case MO_E_FORMAT: return "unknown format id";
    case MO_E_DTYPE: return "unknown value type";
    case MO_E_FILL: return "format needs more padding than the parameters allow";
    case MO_E_ALLOC: return "device allocation failed";
    case MO_E_DEVICE: return "HIP call failed";
    case MO_E_MODEL: return "model file unreadable or malformed";
    case MO_E_PARAM: return "invalid parameter";
    case MO_E_IO: return "matrix file unreadable, malformed or unsupported";
    }
    return "unknown status";
}

int mo_last_hip_error(void) { return g_last_hip_error; }

mo_status mo_features(const mo_csr *a, const mo_params *params, double out[MO_NUM_FEATURES], mo_feature_ints *ints_opt, void *stream)
{
    if (!out) return MO_E_NULL;
    MO_TRY(check_csr_args(a));
    mo_params p;
    MO_TRY(check_params(params, &p));
    hipStream_t s = (hipStream_t)stream;
    Analysis an;
    MO_TRY(analyse_cached(*a, p, &an, s));
    mo_feature_ints ints;
    ints.m = a->m; ints.n = a->n; ints.nnz = a->nnz;
    ints.max_row = an.max_row; ints.min_row = an.min_row;
    ints.n_diag = an.n_diag; ints.n_true_diag = an.n_true;
    ints.sum_sq_row = an.sum_sq;
    if (ints_opt) *ints_opt = ints;
    return mo_features_finalize(&ints, out);
}

mo_status mo_features_finalize(const mo_feature_ints *ints, double out[MO_NUM_FEATURES])
{
    if (!ints || !out) return MO_E_NULL;
    if (ints->m < 1 || ints->n < 1 || ints->nnz < 0) return MO_E_SHAPE;
    // Table I, from exact integers.  M * sum(len^2) - NNZ^2 equals M^2 times the mean squared deviation of the row
    // lengths; every floating-point operation below is a single correctly rounded IEEE operation.
    const unsigned __int128 num = (unsigned __int128)ints->m * (unsigned __int128)ints->sum_sq_row -
                                  (unsigned __int128)ints->nnz * (unsigned __int128)ints->nnz;
    const double md = (double)ints->m, nd = (double)ints->n, zd = (double)ints->nnz;
    const double mm = md * md;
    const double var = (double)num / mm;
    out[0] = md;
    out[1] = nd;
    out[2] = zd;
    out[3] = zd / md;
    const double mn = md * nd;
    out[4] = zd / mn;
    out[5] = (double)ints->max_row;
    out[6] = (double)ints->min_row;
    out[7] = std::sqrt(var);
    out[8] = (double)ints->n_diag;
    out[9] = (double)ints->n_true_diag;
    return MO_OK;
}

mo_status mo_features_static(const mo_csr *a, const mo_params *params, mo_feature_result *out_dev, void *stream)
{
    if (!out_dev) return MO_E_NULL;
    MO_TRY(check_csr_args(a));
    mo_params p;
    MO_TRY(check_params(params, &p));
    return features_static(*a, p, out_dev, (hipStream_t)stream);
}

mo_status mo_convert(const mo_csr *a, mo_format fmt, const mo_params *params, mo_matrix **out, void *stream)
{
    if (!out) return MO_E_NULL;
    *out = nullptr;
    MO_TRY(check_csr_args(a));
    if ((int)fmt < 0 || (int)fmt >= MO_NUM_FORMATS) return MO_E_FORMAT;
    mo_params p;
    MO_TRY(check_params(params, &p));
    hipStream_t s = (hipStream_t)stream;
    const mo_status rc = no_throw([&]() -> mo_status {
        Scratch scr(s);
        Analysis an;
        const bool want_hist = (fmt == MO_DIA || fmt == MO_HDC);
        MO_TRY(analyse(*a, p, want_hist, &an, scr, s));
        return convert_impl(*a, fmt, p, an, out, s);
    });
    if (rc != MO_OK) *out = nullptr;
    return rc;
}

mo_status mo_spmv(const mo_matrix *a, const void *x, void *y, void *stream)
{
    if (!a || !x || !y) return MO_E_NULL;
    hipStream_t s = (hipStream_t)stream;
    switch (a->fmt) {
    case MO_COO: return spmv_coo(*a, x, y, false, s);
    case MO_CSR:
        if (!a->csr_slices.empty()) {
            for (size_t q = 0; q < a->csr_slices.size(); ++q) MO_TRY(spmv_csr(*a->csr_slices[q], x, y, q > 0, s));
            return MO_OK;
        }
        return spmv_csr(*a, x, y, false, s);
    case MO_DIA: return spmv_dia(*a, x, y, s);
    case MO_ELL: return spmv_ell(*a, x, y, s);
    case MO_HYB:
        if (a->nnz_coo > 0 && a->hyb_max_surplus <= HYB_FUSED_MAX_SURPLUS && a->coo_rp) return spmv_hyb_fused(*a, x, y, s);
        MO_TRY(spmv_ell(*a, x, y, s));
        return a->nnz_coo > 0 ? spmv_coo(*a, x, y, true, s) : MO_OK;
    case MO_HDC:
        if (a->nd == 0) return spmv_csr(*a, x, y, false, s);
        if (a->csr_max_row <= HDC_FUSED_MAX_ROW) return spmv_hdc_fused(*a, x, y, s);
        MO_TRY(spmv_dia(*a, x, y, s));
        return a->nnz_csr > 0 ? spmv_csr(*a, x, y, true, s) : MO_OK;
    }
    return MO_E_FORMAT;
}

// The kernels mo_spmv enqueues for a handle, by the same conditions as the dispatch above and in the launchers.
static const char *csr_kernel(const mo_matrix &a) { return a.csr_split ? "k_csr_split+k_coo_fixup" : "k_csr_tiled"; }
static const char *ell_kernel(const mo_matrix &a)
{
    if (a.m <= ELL_SPLIT_MAX_ROWS && a.k >= ELL_SPLIT_MIN_K) return "k_ell_split";
    return ell_uses_windows(a) ? "k_ell_win" : "k_ell";
}
static const char *dia_kernel(const mo_matrix &a, bool hdc)
{
    if (a.dia_batch) return "k_dia_batch";
    return a.dia_block ? "k_dia_lds" : (hdc ? "k_hdc_fused" : "k_dia");
}

mo_status mo_spmv_kernels(const mo_matrix *a, char *buf, size_t cap)
{
    if (!a || !buf || cap == 0) return MO_E_NULL;
    std::string s;
    switch (a->fmt) {
    case MO_COO:
        if (!a->coo_every_row) s += "k_zero+";
        s += a->coo_tiles > 1 ? "k_coo_tile+k_coo_fixup" : "k_coo_tile";
        break;
    case MO_CSR:
        if (!a->csr_slices.empty()) {
            s = std::to_string(a->csr_slices.size()) + " column slices x (" + csr_kernel(*a->csr_slices[0]) + ")";
            break;
        }
        s = csr_kernel(*a);
        break;
    case MO_DIA: s = dia_kernel(*a, false); break;
    case MO_ELL: s = ell_kernel(*a); break;
    case MO_HYB:
        if (a->nnz_coo > 0 && a->hyb_max_surplus <= HYB_FUSED_MAX_SURPLUS && a->coo_rp) s = ell_uses_windows(*a) ? "k_ell_win(hyb)" : "k_ell_hyb";
        else {
            s = ell_kernel(*a);
            if (a->nnz_coo > 0) s += a->coo_tiles > 1 ? "+k_coo_tile+k_coo_fixup" : "+k_coo_tile";
        }
        break;
    case MO_HDC:
        if (a->nd == 0) s = csr_kernel(*a);
        else if (a->csr_max_row <= HDC_FUSED_MAX_ROW) s = dia_kernel(*a, true);
        else { s = dia_kernel(*a, false); if (a->nnz_csr > 0) { s += "+"; s += csr_kernel(*a); } }
        break;
    default: return MO_E_FORMAT;
    }
    if (s.size() + 1 > cap) return MO_E_PARAM;
    std::memcpy(buf, s.c_str(), s.size() + 1);
    return MO_OK;
}

mo_status mo_pick(const double ms[MO_NUM_FORMATS], mo_format *best)
{
    if (!ms || !best) return MO_E_NULL;
    int b = -1;
    for (int f = 0; f < MO_NUM_FORMATS; ++f) {
        if (std::isnan(ms[f])) continue;
        if (b < 0 || ms[f] < ms[b]) b = f;
    }
    if (b < 0) return MO_E_PARAM;
    *best = (mo_format)b;
    return MO_OK;
}

mo_status mo_spmm(const mo_matrix *a, const void *x, void *y, int32_t k, void *stream)
{
    if (!a || !x || !y) return MO_E_NULL;
    if (k < 1 || k > MO_MAX_RHS) return MO_E_PARAM;
    if (k == 1) return mo_spmv(a, x, y, stream);   // an n x 1 matrix is a vector
    return spmm(*a, x, y, (int)k, (hipStream_t)stream);
}

// The run-first tuner for either operation: k = 0 times mo_spmv, k >= 1 times mo_spmm with k right-hand sides.
static mo_status tune_impl(const mo_csr *a, int k, const mo_params *params, const mo_tune_opts *opts, mo_format *best,
                           double ms_per_rep[MO_NUM_FORMATS], double convert_ms[MO_NUM_FORMATS], void *stream)
{
    if (!best || !ms_per_rep) return MO_E_NULL;
    MO_TRY(check_csr_args(a));
    mo_params p;
    MO_TRY(check_params(params, &p));
    int warm = 5, reps = 50;
    if (opts) { warm = opts->warmups; reps = opts->reps; }
    if (warm < 0 || reps < 1) return MO_E_PARAM;
    hipStream_t s = (hipStream_t)stream;
    for (int f = 0; f < MO_NUM_FORMATS; ++f) {
        ms_per_rep[f] = std::numeric_limits<double>::quiet_NaN();
        if (convert_ms) convert_ms[f] = std::numeric_limits<double>::quiet_NaN();
    }
    Scratch scr(s);
    Analysis an;
    MO_TRY(analyse(*a, p, true, &an, scr, s));
    const size_t sv = dtype_size(a->dtype);
    const int64_t width = k > 0 ? k : 1;
    void *x = scr.get((size_t)(a->n * width) * sv);
    void *y = scr.get((size_t)(a->m * width) * sv);
    if (!x || !y) return MO_E_ALLOC;
    // a dense, sign-mixed operand of ordinary magnitude, the same on every call: the timed kernels then toggle the data
    // paths and multipliers as they do on real vectors
    if (a->dtype == MO_F32) hipLaunchKernelGGL(k_fill_operand<float>, dim3(1024), dim3(256), 0, s, (float *)x, a->n * width);
    else hipLaunchKernelGGL(k_fill_operand<double>, dim3(1024), dim3(256), 0, s, (double *)x, a->n * width);
    MO_LAUNCH_CHECK();
    hipEvent_t e0, e1;
    MO_HIP(hipEventCreate(&e0));
    if (hipEventCreate(&e1) != hipSuccess) { (void)hipEventDestroy(e0); return MO_E_DEVICE; }
    mo_status rc = MO_OK;
    for (int f = 0; f < MO_NUM_FORMATS && rc == MO_OK; ++f) {
        mo_matrix *h = nullptr;
        const auto t0 = std::chrono::steady_clock::now();
        mo_status c = convert_impl(*a, (mo_format)f, p, an, &h, s);
        if (c == MO_E_FILL) continue;
        if (c != MO_OK) { rc = c; break; }
        const auto t1 = std::chrono::steady_clock::now();
        if (convert_ms) convert_ms[f] = std::chrono::duration<double, std::milli>(t1 - t0).count();
        for (int i = 0; i < warm && rc == MO_OK; ++i) rc = k > 1 ? spmm(*h, x, y, k, s) : mo_spmv(h, x, y, s);
        if (rc == MO_OK && hipEventRecord(e0, s) != hipSuccess) rc = MO_E_DEVICE;
        for (int i = 0; i < reps && rc == MO_OK; ++i) rc = k > 1 ? spmm(*h, x, y, k, s) : mo_spmv(h, x, y, s);
        if (rc == MO_OK && hipEventRecord(e1, s) != hipSuccess) rc = MO_E_DEVICE;
        if (rc == MO_OK && hipEventSynchronize(e1) != hipSuccess) rc = MO_E_DEVICE;
        float ms = 0.f;
        if (rc == MO_OK && hipEventElapsedTime(&ms, e0, e1) != hipSuccess) rc = MO_E_DEVICE;
        if (rc == MO_OK) ms_per_rep[f] = (double)ms / (double)reps;
        (void)hipStreamSynchronize(s);
        mo_matrix_free(h);
    }
    (void)hipEventDestroy(e0);
    (void)hipEventDestroy(e1);
    if (rc != MO_OK) return rc;
    return mo_pick(ms_per_rep, best);
}

mo_status mo_tune(const mo_csr *a, const mo_params *params, const mo_tune_opts *opts, mo_format *best,
                  double ms_per_rep[MO_NUM_FORMATS], double convert_ms[MO_NUM_FORMATS], void *stream)
{
    return no_throw([&] { return tune_impl(a, 0, params, opts, best, ms_per_rep, convert_ms, stream); });
}

mo_status mo_tune_spmm(const mo_csr *a, int32_t k, const mo_params *params, const mo_tune_opts *opts, mo_format *best,
                       double ms_per_rep[MO_NUM_FORMATS], double convert_ms[MO_NUM_FORMATS], void *stream)
{
    if (k < 1 || k > MO_MAX_RHS) return MO_E_PARAM;
    return no_throw([&] { return tune_impl(a, (int)k, params, opts, best, ms_per_rep, convert_ms, stream); });
}

mo_status mo_matrix_export(const mo_matrix *a, mo_matrix_view *out)
{
    if (!a || !out) return MO_E_NULL;
    out->fmt = a->fmt; out->dtype = a->dtype;
    out->m = a->m; out->n = a->n; out->nnz = a->nnz; out->ld = a->ld;
    out->nd = a->nd; out->k = a->k; out->nnz_coo = a->nnz_coo; out->nnz_csr = a->nnz_csr;
    const bool dia = a->fmt == MO_DIA || a->fmt == MO_HDC;
    const bool ell = a->fmt == MO_ELL || a->fmt == MO_HYB;
    const bool coo = a->fmt == MO_COO || a->fmt == MO_HYB;
    const bool csr = a->fmt == MO_CSR || a->fmt == MO_HDC;
    out->dia_off = dia ? a->dia_off : nullptr; out->dia_val = dia ? a->dia_val : nullptr;
    out->ell_col = ell ? a->ell_col : nullptr; out->ell_val = ell ? a->ell_val : nullptr;
    out->coo_row = coo ? a->coo_row : nullptr; out->coo_col = coo ? a->coo_col : nullptr; out->coo_val = coo ? a->coo_val : nullptr;
    out->csr_row_ptr = csr ? a->csr_row_ptr : nullptr; out->csr_col = csr ? a->csr_col : nullptr; out->csr_val = csr ? a->csr_val : nullptr;
    return MO_OK;
}

void mo_matrix_free(mo_matrix *a)
{
    if (!a) return;
    for (mo_matrix *part : a->csr_slices) mo_matrix_free(part);
    for (void *p : a->owned) dev_free(p, a->home);
    delete a;
}

}  // extern "C"

// Matrix Market reader on the host (the paper's data set, Section VII "Setup", is distributed in this format).
//
// Coordinate format only, as published in "The Matrix Market Exchange Formats: Initial Design" (NISTIR 5935):
// banner "%%MatrixMarket matrix coordinate <real|integer|pattern> <general|symmetric|skew-symmetric>", comment lines
// starting with '%', a size line "M N L", then L entries "i j [value]" with 1-based indices.  Symmetric files store
// one triangle: an off-diagonal entry also stands for its mirror image (negated for skew-symmetric, where diagonal
// entries are not allowed).  Pattern entries mean 1.  Entries naming the same position are summed, first the file's
// own entries in file order, then the mirrored ones; explicit zeros stay entries.  The result is CSR with columns
// ascending inside each row, which is what every other call of this library expects.
#include <algorithm>
#include <cctype>
#include <cerrno>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <new>
#include <string>
#include <vector>

#include "mo.h"

namespace {

struct Entry {
    int32_t row, col;
    double val;
};

inline bool is_space(char c) { return c == ' ' || c == '\t' || c == '\r' || c == '\f' || c == '\v'; }

// Splits one line into whitespace-separated tokens (views into the buffer).
struct Tokens {
    const char *begin[8];
    size_t len[8];
    int count = 0;   // 9 = more than 8
};

Tokens split(const char *p, const char *end)
{
    Tokens t;
    while (p < end) {
        while (p < end && is_space(*p)) ++p;
        if (p >= end) break;
        const char *q = p;
        while (q < end && !is_space(*q)) ++q;
        if (t.count == 8) { t.count = 9; return t; }
        t.begin[t.count] = p; t.len[t.count] = (size_t)(q - p); ++t.count;
        p = q;
    }
    return t;
}

bool ieq(const char *p, size_t n, const char *lit)
{
    if (std::strlen(lit) != n) return false;
    for (size_t i = 0; i < n; ++i)
        if (std::tolower((unsigned char)p[i]) != lit[i]) return false;
    return true;
}

bool parse_int(const char *p, size_t n, int64_t *out)
{
    if (n == 0 || n > 20) return false;
    char buf[24];
    std::memcpy(buf, p, n); buf[n] = 0;
    char *e = nullptr;
    errno = 0;
    const long long v = std::strtoll(buf, &e, 10);
    if (errno || e != buf + n) return false;
    *out = v;
    return true;
}

bool parse_real(const char *p, size_t n, double *out)
{
    if (n == 0 || n > 62) return false;
    char buf[64];
    std::memcpy(buf, p, n); buf[n] = 0;
    if (buf[0] == '0' && (buf[1] == 'x' || buf[1] == 'X')) return false;   // no hexadecimal floats in this format
    char *e = nullptr;
    const double v = std::strtod(buf, &e);
    if (e != buf + n) return false;
    *out = v;
    return true;
}

}  // namespace

extern "C" {

void mo_host_free(void *p) { std::free(p); }

mo_status mo_mtx_read(const char *path, int64_t *m_out, int64_t *n_out, int64_t *nnz_out, int32_t **row_ptr_out,
                      int32_t **col_idx_out, double **val_out)
{
    if (!path || !m_out || !n_out || !nnz_out || !row_ptr_out || !col_idx_out || !val_out) return MO_E_NULL;
    *row_ptr_out = nullptr; *col_idx_out = nullptr; *val_out = nullptr;
    *m_out = *n_out = *nnz_out = 0;
    try {
        std::string text;
        {
            FILE *f = std::fopen(path, "rb");
            if (!f) return MO_E_IO;
            char chunk[1 << 16];
            size_t got;
            while ((got = std::fread(chunk, 1, sizeof(chunk), f)) > 0) text.append(chunk, got);
            const bool bad = std::ferror(f) != 0;
            std::fclose(f);
            if (bad) return MO_E_IO;
        }
        const char *p = text.data(), *end = p + text.size();
        auto next_line = [&](const char *&lb, const char *&le) -> bool {   // false at end of file
            if (p >= end) return false;
            lb = p;
            const char *nl = (const char *)std::memchr(p, '\n', (size_t)(end - p));
            le = nl ? nl : end;
            p = nl ? nl + 1 : end;
            return true;
        };
        const char *lb, *le;
        if (!next_line(lb, le) || le - lb < 14 || std::memcmp(lb, "%%MatrixMarket", 14) != 0) return MO_E_IO;
        Tokens b = split(lb, le);
        if (b.count != 5 || !ieq(b.begin[1], b.len[1], "matrix") || !ieq(b.begin[2], b.len[2], "coordinate")) return MO_E_IO;
        const bool pattern = ieq(b.begin[3], b.len[3], "pattern");
        if (!pattern && !ieq(b.begin[3], b.len[3], "real") && !ieq(b.begin[3], b.len[3], "integer")) return MO_E_IO;
        const bool symmetric = ieq(b.begin[4], b.len[4], "symmetric"), skew = ieq(b.begin[4], b.len[4], "skew-symmetric");
        if (!symmetric && !skew && !ieq(b.begin[4], b.len[4], "general")) return MO_E_IO;
        // comments and blank lines, then the size line
        Tokens t;
        for (;;) {
            if (!next_line(lb, le)) return MO_E_IO;
            t = split(lb, le);
            if (t.count == 0 || t.begin[0][0] == '%') continue;
            break;
        }
        int64_t m, n, count;
        if (t.count != 3 || !parse_int(t.begin[0], t.len[0], &m) || !parse_int(t.begin[1], t.len[1], &n) ||
            !parse_int(t.begin[2], t.len[2], &count))
            return MO_E_IO;
        if (m < 1 || n < 1 || count < 0) return MO_E_IO;
        if ((symmetric || skew) && m != n) return MO_E_IO;
        if (m + n > 2147483647ll || count > 2147483647ll) return MO_E_SHAPE;
        std::vector<Entry> direct, mirrored;
        direct.reserve((size_t)count);
        for (int64_t k = 0; k < count; ++k) {
            do {
                if (!next_line(lb, le)) return MO_E_IO;   // fewer entries than announced
                t = split(lb, le);
            } while (t.count == 0);
            int64_t i, j;
            double v = 1.0;
            if (t.count != (pattern ? 2 : 3) || !parse_int(t.begin[0], t.len[0], &i) || !parse_int(t.begin[1], t.len[1], &j)) return MO_E_IO;
            if (!pattern && !parse_real(t.begin[2], t.len[2], &v)) return MO_E_IO;
            if (i < 1 || i > m || j < 1 || j > n) return MO_E_IO;
            if (skew && i == j) return MO_E_IO;
            direct.push_back({(int32_t)(i - 1), (int32_t)(j - 1), v});
            if ((symmetric || skew) && i != j) mirrored.push_back({(int32_t)(j - 1), (int32_t)(i - 1), skew ? -v : v});
        }
        while (next_line(lb, le))
            if (split(lb, le).count != 0) return MO_E_IO;   // more entries than announced
        if (direct.size() + mirrored.size() > 2147483647ull) return MO_E_SHAPE;
        direct.insert(direct.end(), mirrored.begin(), mirrored.end());
        std::vector<Entry>().swap(mirrored);
        // stable: entries of one position keep their order, so sums run in the order stated above
        std::stable_sort(direct.begin(), direct.end(), [](const Entry &a, const Entry &b) {
            return a.row != b.row ? a.row < b.row : a.col < b.col;
        });
        size_t distinct = 0;
        for (size_t k = 0; k < direct.size(); ++k)
            if (k == 0 || direct[k].row != direct[k - 1].row || direct[k].col != direct[k - 1].col) ++distinct;
        int32_t *rp = (int32_t *)std::calloc((size_t)m + 1, sizeof(int32_t));
        int32_t *ci = (int32_t *)std::malloc((distinct ? distinct : 1) * sizeof(int32_t));
        double *va = (double *)std::malloc((distinct ? distinct : 1) * sizeof(double));
        if (!rp || !ci || !va) { std::free(rp); std::free(ci); std::free(va); return MO_E_ALLOC; }
        size_t w = 0;
        for (size_t k = 0; k < direct.size(); ++k) {
            if (k > 0 && direct[k].row == direct[k - 1].row && direct[k].col == direct[k - 1].col) {
                va[w - 1] += direct[k].val;
            } else {
                ci[w] = direct[k].col; va[w] = direct[k].val; ++w;
                rp[direct[k].row + 1]++;
            }
        }
        for (int64_t r = 0; r < m; ++r) rp[r + 1] += rp[r];
        *m_out = m; *n_out = n; *nnz_out = (int64_t)distinct;
        *row_ptr_out = rp; *col_idx_out = ci; *val_out = va;
        return MO_OK;
    } catch (const std::bad_alloc &) {
        return MO_E_ALLOC;
    }
}

}  // extern "C"

// Tree / forest models on the host: file loader and evaluation (Sections III-B and VI-A).
#include <cstdio>
#include <cstring>
#include <new>
#include <vector>

#include "mo.h"
#include "model.hpp"

namespace {

bool read_exact(FILE *f, void *dst, size_t bytes) { return bytes == 0 || std::fread(dst, 1, bytes, f) == bytes; }

constexpr int32_t kMaxTrees = 1 << 16;
constexpr int32_t kMaxNodes = 1 << 24;

}  // namespace

extern "C" {

mo_status mo_model_load(const char *path, mo_model **out)
{
    if (!out) return MO_E_NULL;
    *out = nullptr;
    if (!path) return MO_E_NULL;
    FILE *f = std::fopen(path, "rb");
    if (!f) return MO_E_MODEL;
    mo_model *m = new (std::nothrow) mo_model();
    if (!m) { std::fclose(f); return MO_E_ALLOC; }
    mo_status rc = MO_E_MODEL;
    // what the file can still deliver bounds every allocation made on the say-so of a header field
    long file_bytes = -1;
    if (std::fseek(f, 0, SEEK_END) == 0) { file_bytes = std::ftell(f); std::rewind(f); }
    try {
    do {
        if (file_bytes < 0) break;
        char magic[8];
        int32_t hdr[4];
        if (!read_exact(f, magic, 8) || std::memcmp(magic, "MOMDL1\0\0", 8) != 0) break;
        if (!read_exact(f, hdr, sizeof(hdr))) break;
        if (hdr[0] != 1 || hdr[1] != MO_NUM_FEATURES || hdr[2] != MO_NUM_FORMATS) break;
        if (hdr[3] < 1 || hdr[3] > kMaxTrees) break;
        m->n_trees = hdr[3];
        m->tree_off.push_back(0);
        bool ok = true;
        int64_t total = 0;
        for (int32_t t = 0; t < m->n_trees && ok; ++t) {
            int32_t nn = 0;
            if (!read_exact(f, &nn, 4) || nn < 1 || nn > kMaxNodes || total + nn > kMaxNodes) { ok = false; break; }
            const long here = std::ftell(f);
            if (here < 0 || (int64_t)nn * 24 > (int64_t)file_bytes - here) { ok = false; break; }   // truncated or lying header
            const size_t base = m->feature.size();
            m->feature.resize(base + nn); m->threshold.resize(base + nn);
            m->left.resize(base + nn); m->right.resize(base + nn); m->klass.resize(base + nn);
            ok = read_exact(f, &m->feature[base], (size_t)nn * 4) && read_exact(f, &m->threshold[base], (size_t)nn * 8) &&
                 read_exact(f, &m->left[base], (size_t)nn * 4) && read_exact(f, &m->right[base], (size_t)nn * 4) &&
                 read_exact(f, &m->klass[base], (size_t)nn * 4);
            for (int32_t i = 0; i < nn && ok; ++i) {
                const int32_t ft = m->feature[base + i];
                if (ft < 0) {
                    if (ft != -1 || m->klass[base + i] < 0 || m->klass[base + i] >= MO_NUM_FORMATS) ok = false;
                } else {
                    // children strictly after the parent: every walk ends, no cycles
                    const int32_t l = m->left[base + i], r = m->right[base + i];
                    if (ft >= MO_NUM_FEATURES || l <= i || l >= nn || r <= i || r >= nn) ok = false;
                    if (m->threshold[base + i] != m->threshold[base + i]) ok = false;   // NaN threshold
                }
            }
            total += nn;
            m->tree_off.push_back((int32_t)total);
        }
        if (!ok) break;
        char extra;
        if (std::fread(&extra, 1, 1, f) != 0) break;   // trailing bytes
        rc = MO_OK;
    } while (false);
    } catch (const std::bad_alloc &) {
        rc = MO_E_ALLOC;
    }
    std::fclose(f);
    if (rc != MO_OK) { delete m; return rc; }
    *out = m;
    return MO_OK;
}

void mo_model_free(mo_model *model) { delete model; }

mo_status mo_model_info(const mo_model *model, int32_t *n_trees, int32_t *n_nodes_total)
{
    if (!model) return MO_E_NULL;
    if (n_trees) *n_trees = model->n_trees;
    if (n_nodes_total) *n_nodes_total = model->tree_off.back();
    return MO_OK;
}

mo_status mo_model_save(const mo_model *model, const char *path)
{
    if (!model || !path) return MO_E_NULL;
    FILE *f = std::fopen(path, "wb");
    if (!f) return MO_E_MODEL;
    const int32_t hdr[4] = {1, MO_NUM_FEATURES, MO_NUM_FORMATS, model->n_trees};
    bool ok = std::fwrite("MOMDL1\0\0", 1, 8, f) == 8 && std::fwrite(hdr, 4, 4, f) == 4;
    for (int32_t t = 0; t < model->n_trees && ok; ++t) {
        const int32_t base = model->tree_off[t], nn = model->tree_off[t + 1] - base;
        const size_t k = (size_t)nn;
        ok = std::fwrite(&nn, 4, 1, f) == 1 && std::fwrite(&model->feature[base], 4, k, f) == k &&
             std::fwrite(&model->threshold[base], 8, k, f) == k && std::fwrite(&model->left[base], 4, k, f) == k &&
             std::fwrite(&model->right[base], 4, k, f) == k && std::fwrite(&model->klass[base], 4, k, f) == k;
    }
    if (std::fclose(f) != 0) ok = false;
    return ok ? MO_OK : MO_E_MODEL;
}

static int vote(const mo_model *model, const double *features)
{
    int64_t votes[MO_NUM_FORMATS] = {0, 0, 0, 0, 0, 0};
    for (int32_t t = 0; t < model->n_trees; ++t) {
        const int32_t base = model->tree_off[t];
        int32_t node = 0;
        while (model->feature[base + node] >= 0) {
            const int32_t f = model->feature[base + node];
            node = (features[f] <= model->threshold[base + node]) ? model->left[base + node] : model->right[base + node];
        }
        votes[model->klass[base + node]]++;
    }
    int best = 0;
    for (int c = 1; c < MO_NUM_FORMATS; ++c)
        if (votes[c] > votes[best]) best = c;
    return best;
}

mo_status mo_select(const mo_model *model, const double features[MO_NUM_FEATURES], mo_format *out)
{
    if (!model || !features || !out) return MO_E_NULL;
    *out = (mo_format)vote(model, features);
    return MO_OK;
}

mo_status mo_predict(const mo_model *model, const double *features, int64_t n, int32_t *out)
{
    if (!model || (n > 0 && (!features || !out))) return MO_E_NULL;
    if (n < 0) return MO_E_SHAPE;
    for (int64_t i = 0; i < n; ++i) out[i] = vote(model, features + i * MO_NUM_FEATURES);
    return MO_OK;
}

}  // extern "C"

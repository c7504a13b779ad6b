// C ABI of the SwiftPrune layer path (see include/swiftprune.h): argument
// checks, path selection (16-byte vector loads vs element-wise) and launches.
#include "../../include/swiftprune.h"

#include "kernels.hpp"

#include <math.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

namespace sp {

Tuning read_tuning() {
    Tuning t = {0, 0, false, 0, false, 0, 0};
    if (const char* e = getenv("SWIFTPRUNE_STATS_PLAN")) {
        int rows = 0, groups = 0;
        if (sscanf(e, "%d,%d", &rows, &groups) == 2 && (rows == 4 || rows == 8 || rows == 16) && groups >= 1 &&
            groups <= 4096) {
            t.stats_rows = rows;
            t.stats_groups = groups;
            t.stats_plain = strstr(e, ",plain") != nullptr;
        }
    }
    if (const char* e = getenv("SWIFTPRUNE_SELECT_TEAM")) {
        const int v = atoi(e);
        if (v == 1 || v == 2 || v == 4) t.team = v;
        t.select_direct = strstr(e, ",direct") != nullptr;
    }
    if (const char* e = getenv("SWIFTPRUNE_BAND_GROUPS")) {
        int a = 0, b = 0;
        if (sscanf(e, "%d,%d", &a, &b) == 2 && a >= 1 && a <= 4096 && b >= 1 && b <= 4096) {
            t.apply_groups = a;
            t.select_groups = b;
        }
    }
    return t;
}

}  // namespace sp

namespace {

inline bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }
inline int64_t elem_size(int dt) { return dt == SP_F32 ? 4 : 2; }
inline bool dtype_ok(int dt) { return dt == SP_F32 || dt == SP_BF16 || dt == SP_F16; }

// the 16-byte-vector path of the statistics kernel
inline bool stats_vec_ok(const void* X, int64_t in, int64_t ldx, int dt) {
    const int64_t epu = 16 / elem_size(dt);
    return aligned16(X) && in % epu == 0 && ldx % epu == 0;
}

// the 16-byte-vector path of the per-weight kernels (8 columns per lane)
inline bool weight_vec_ok(const void* W, int64_t in, int64_t ldw, int dt, const float* hr,
                          const float* scores) {
    const int64_t epu = 16 / elem_size(dt);
    return aligned16(W) && in % 8 == 0 && ldw % epu == 0 && (hr == nullptr || aligned16(hr)) &&
           (scores == nullptr || aligned16(scores));
}

// the fast selection kernels number the rows of a launch with 32 bits (and add a grid stride to them)
constexpr int64_t kMaxFastRows = (int64_t)1 << 30;

const float kTableRatio[5] = {0.5f, 0.6f, 0.7f, 0.8f, 0.9f};
const float kTableLa[5] = {0.5f, 0.2f, -0.2f, -0.9f, -1.5f};

}  // namespace

extern "C" {

const char* swiftprune_version(void) { return "0.1.0"; }

const char* swiftprune_strerror(int code) {
    switch (code) {
        case SP_OK: return "success";
        case SP_EINVAL: return "invalid argument";
        case SP_ENOSPC: return "workspace too small";
        case SP_EHIP: return "HIP runtime error (see hipGetLastError)";
        case SP_ERANGE: return "target not reachable within tolerance; closest value returned";
        default: return "unknown status";
    }
}

int swiftprune_la_for_sparsity(float sparsity, float* la) {
    if (la == nullptr || !(sparsity >= 0.5f && sparsity <= 0.9f)) return SP_EINVAL;
    for (int i = 0; i < 5; ++i) {
        if (fabsf(sparsity - kTableRatio[i]) < 1e-6f) {
            *la = kTableLa[i];
            return SP_OK;
        }
    }
    for (int i = 0; i < 4; ++i) {
        if (sparsity > kTableRatio[i] && sparsity < kTableRatio[i + 1]) {
            const float t = (sparsity - kTableRatio[i]) / (kTableRatio[i + 1] - kTableRatio[i]);
            *la = kTableLa[i] + t * (kTableLa[i + 1] - kTableLa[i]);
            return SP_OK;
        }
    }
    return SP_EINVAL;
}

size_t swiftprune_stats_workspace_bytes(int64_t tokens, int64_t in) {
    if (tokens <= 0 || in <= 0) return 0;
    size_t bytes = 0;
    for (int dt = 0; dt < 3; ++dt)
        for (int vec = 0; vec < 2; ++vec) {
            const size_t b = sp::stats_workspace_bytes(sp::make_stats_plan(tokens, in, dt, vec != 0));
            if (b > bytes) bytes = b;
        }
    return bytes;
}

int swiftprune_layer_stats(const void* X, int64_t tokens, int64_t in, int64_t ldx, sp_dtype dt,
                           float* xsq, float* S, float* hr, int accumulate, int finalize,
                           void* workspace, size_t workspace_bytes, void* hip_stream) {
    if (X == nullptr || xsq == nullptr || workspace == nullptr) return SP_EINVAL;
    if (tokens <= 0 || in <= 0 || ldx < in || !dtype_ok((int)dt)) return SP_EINVAL;
    if (S == nullptr || (finalize && hr == nullptr)) return SP_EINVAL;
    if (reinterpret_cast<uintptr_t>(X) % elem_size((int)dt) != 0) return SP_EINVAL;
    if (reinterpret_cast<uintptr_t>(workspace) % 256 != 0) return SP_EINVAL;
    if (workspace_bytes < swiftprune_stats_workspace_bytes(tokens, in)) return SP_ENOSPC;
    const bool vec = stats_vec_ok(X, in, ldx, (int)dt);
    const hipError_t e = sp::launch_layer_stats(X, tokens, in, ldx, (int)dt, vec, xsq, S, hr, accumulate,
                                                finalize, workspace, static_cast<hipStream_t>(hip_stream));
    return e == hipSuccess ? SP_OK : SP_EHIP;
}

int swiftprune_channel_factor(const float* xsq, const float* S, int64_t in, float* hr, void* hip_stream) {
    if (xsq == nullptr || S == nullptr || hr == nullptr || in <= 0) return SP_EINVAL;
    if (in > (int64_t)0x7fffffff * 256) return SP_EINVAL;
    if (reinterpret_cast<uintptr_t>(xsq) % 4 != 0 || reinterpret_cast<uintptr_t>(S) % 4 != 0 ||
        reinterpret_cast<uintptr_t>(hr) % 4 != 0)
        return SP_EINVAL;
    const hipError_t e = sp::launch_channel_factor(xsq, S, in, hr, static_cast<hipStream_t>(hip_stream));
    return e == hipSuccess ? SP_OK : SP_EHIP;
}

int swiftprune_layer_stats_from_partials(const float* partials, int64_t parts, int64_t in, int64_t ld, float* xsq,
                                         float* S, float* hr, int accumulate, int finalize, void* hip_stream) {
    if (partials == nullptr || xsq == nullptr || S == nullptr || (finalize && hr == nullptr)) return SP_EINVAL;
    if (parts <= 0 || in <= 0 || ld < in) return SP_EINVAL;
    if (parts > ((int64_t)1 << 24) || in > (int64_t)0x7fffffff * 64) return SP_EINVAL;
    if (reinterpret_cast<uintptr_t>(partials) % 4 != 0 || reinterpret_cast<uintptr_t>(xsq) % 4 != 0 ||
        reinterpret_cast<uintptr_t>(S) % 4 != 0 || (hr != nullptr && reinterpret_cast<uintptr_t>(hr) % 4 != 0))
        return SP_EINVAL;
    const hipError_t e = sp::launch_stats_from_pieces(partials, parts, in, ld, xsq, S, hr, accumulate, finalize,
                                                      static_cast<hipStream_t>(hip_stream));
    return e == hipSuccess ? SP_OK : SP_EHIP;
}

int swiftprune_score_select(const void* W, int64_t out, int64_t in, int64_t ldw, sp_dtype dt,
                            const float* hr, float sparsity, const sp_ewma_params* params,
                            uint32_t* keep_mask, int32_t* row_pruned, float* scores,
                            uint32_t flags, void* hip_stream) {
    if (W == nullptr || hr == nullptr || keep_mask == nullptr) return SP_EINVAL;
    if (out <= 0 || in <= 0 || ldw < in || !dtype_ok((int)dt)) return SP_EINVAL;
    if (flags & ~(SP_SEQUENTIAL_ORDER | SP_APPLY_INPLACE)) return SP_EINVAL;
    if (reinterpret_cast<uintptr_t>(W) % elem_size((int)dt) != 0) return SP_EINVAL;
    sp_ewma_params p = {0.125f, 0.125f, NAN};
    if (params != nullptr) p = *params;
    if (isnan(p.la)) {
        if (swiftprune_la_for_sparsity(sparsity, &p.la) != SP_OK) return SP_EINVAL;
    }
    if (!(p.alpha > 0.0f && p.alpha <= 1.0f) || !(p.beta > 0.0f && p.beta <= 1.0f) || isinf(p.la))
        return SP_EINVAL;
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    const bool apply = (flags & SP_APPLY_INPLACE) != 0;
    hipError_t e;
    if (flags & SP_SEQUENTIAL_ORDER) {
        e = sp::launch_ewma_sequential(W, out, in, ldw, (int)dt, hr, p.alpha, p.beta, p.la, keep_mask,
                                       row_pruned, scores, apply, stream);
    } else {
        const bool vec = out <= kMaxFastRows && weight_vec_ok(W, in, ldw, (int)dt, hr, scores);
        const sp::EwmaConsts c = sp::make_ewma_consts(p.alpha, p.beta, p.la);
        e = sp::launch_ewma_scan(W, out, in, ldw, (int)dt, vec, hr, c, keep_mask, row_pruned, scores,
                                 apply, stream);
    }
    return e == hipSuccess ? SP_OK : SP_EHIP;
}

static bool group_ok(const sp_matrix* mats, int n_mats, int64_t in, int dt) {
    if (mats == nullptr || n_mats < 1 || n_mats > SP_MAX_GROUP || in <= 0 || !dtype_ok(dt)) return false;
    int64_t rows = 0;
    for (int j = 0; j < n_mats; ++j) {
        const sp_matrix& m = mats[j];
        if (m.W == nullptr || m.keep_mask == nullptr || m.out <= 0 || m.ldw < in) return false;
        if (reinterpret_cast<uintptr_t>(m.W) % elem_size(dt) != 0) return false;
        rows += m.out;
        if (rows > kMaxFastRows) return false;
    }
    return true;
}

static sp::RowGroups make_groups(const sp_matrix* mats, int n_mats) {
    sp::RowGroups g;
    g.n = n_mats;
    int64_t end = 0;
    for (int j = 0; j < sp::kMaxGroup; ++j) {
        const sp_matrix& m = mats[j < n_mats ? j : n_mats - 1];
        if (j < n_mats) end += m.out;
        g.row_end[j] = (int32_t)end;
        g.W[j] = m.W;
        g.ldw[j] = m.ldw;
        g.keep_mask[j] = m.keep_mask;
        g.row_pruned[j] = m.row_pruned;
    }
    return g;
}

int swiftprune_score_select_group(const sp_matrix* mats, int n_mats, int64_t in, sp_dtype dt,
                                  const float* hr, float sparsity, const sp_ewma_params* params,
                                  uint32_t flags, void* hip_stream) {
    static_assert(SP_MAX_GROUP == sp::kMaxGroup, "group size of the header and of the kernels");
    if (hr == nullptr || !group_ok(mats, n_mats, in, (int)dt)) return SP_EINVAL;
    if (flags & ~(SP_SEQUENTIAL_ORDER | SP_APPLY_INPLACE)) return SP_EINVAL;
    sp_ewma_params p = {0.125f, 0.125f, NAN};
    if (params != nullptr) p = *params;
    if (isnan(p.la) && swiftprune_la_for_sparsity(sparsity, &p.la) != SP_OK) return SP_EINVAL;
    if (!(p.alpha > 0.0f && p.alpha <= 1.0f) || !(p.beta > 0.0f && p.beta <= 1.0f) || isinf(p.la))
        return SP_EINVAL;
    bool fast = !(flags & SP_SEQUENTIAL_ORDER) && p.alpha < 1.0f;
    for (int j = 0; j < n_mats && fast; ++j) fast = weight_vec_ok(mats[j].W, in, mats[j].ldw, (int)dt, hr, nullptr);
    if (fast) {
        const sp::EwmaConsts c = sp::make_ewma_consts(p.alpha, p.beta, p.la);
        const hipError_t e = sp::launch_ewma_team(make_groups(mats, n_mats), in, (int)dt, hr, c,
                                                  (flags & SP_APPLY_INPLACE) != 0, 0,
                                                  static_cast<hipStream_t>(hip_stream));
        return e == hipSuccess ? SP_OK : SP_EHIP;
    }
    for (int j = 0; j < n_mats; ++j) {
        const int rc = swiftprune_score_select(mats[j].W, mats[j].out, in, mats[j].ldw, dt, hr, sparsity, &p,
                                               mats[j].keep_mask, mats[j].row_pruned, nullptr, flags, hip_stream);
        if (rc != SP_OK) return rc;
    }
    return SP_OK;
}

int swiftprune_nm_select_group(const sp_matrix* mats, int n_mats, int64_t in, sp_dtype dt, const float* hr,
                               int n_keep, int m_group, uint32_t flags, void* hip_stream) {
    if (hr == nullptr || !group_ok(mats, n_mats, in, (int)dt)) return SP_EINVAL;
    if (m_group != 4 && m_group != 8 && m_group != 16) return SP_EINVAL;
    if (n_keep <= 0 || n_keep >= m_group || in % m_group != 0) return SP_EINVAL;
    if (flags & ~SP_APPLY_INPLACE) return SP_EINVAL;
    bool fast = true;
    for (int j = 0; j < n_mats && fast; ++j) fast = weight_vec_ok(mats[j].W, in, mats[j].ldw, (int)dt, hr, nullptr);
    if (fast) {
        const hipError_t e = sp::launch_nm_select_group(make_groups(mats, n_mats), in, (int)dt, hr, n_keep, m_group,
                                                        nullptr, (flags & SP_APPLY_INPLACE) != 0,
                                                        static_cast<hipStream_t>(hip_stream));
        return e == hipSuccess ? SP_OK : SP_EHIP;
    }
    for (int j = 0; j < n_mats; ++j) {
        const int rc = swiftprune_nm_select(mats[j].W, mats[j].out, in, mats[j].ldw, dt, hr, n_keep, m_group,
                                            mats[j].keep_mask, nullptr, flags, hip_stream);
        if (rc != SP_OK) return rc;
    }
    return SP_OK;
}

int swiftprune_ewma_trace(const void* W, int64_t out, int64_t in, int64_t ldw, sp_dtype dt,
                          const float* hr, float alpha, float beta, float* est, float* dev,
                          void* hip_stream) {
    if (W == nullptr || hr == nullptr || (est == nullptr && dev == nullptr)) return SP_EINVAL;
    if (out <= 0 || in <= 0 || ldw < in || !dtype_ok((int)dt)) return SP_EINVAL;
    if (!(alpha > 0.0f && alpha <= 1.0f) || !(beta > 0.0f && beta <= 1.0f)) return SP_EINVAL;
    if (reinterpret_cast<uintptr_t>(W) % elem_size((int)dt) != 0) return SP_EINVAL;
    if (reinterpret_cast<uintptr_t>(est) % 4 != 0 || reinterpret_cast<uintptr_t>(dev) % 4 != 0) return SP_EINVAL;
    const bool vec = weight_vec_ok(W, in, ldw, (int)dt, hr, est) && (dev == nullptr || aligned16(dev));
    const sp::EwmaConsts c = sp::make_ewma_consts(alpha, beta, 0.0f);
    const hipError_t e = sp::launch_ewma_trace(W, out, in, ldw, (int)dt, vec, hr, c, est, dev,
                                               static_cast<hipStream_t>(hip_stream));
    return e == hipSuccess ? SP_OK : SP_EHIP;
}

int swiftprune_count_pruned(const void* W, int64_t out, int64_t in, int64_t ldw, sp_dtype dt,
                            const float* hr, float alpha, float beta, const float* la, int n_la,
                            unsigned long long* counts, void* hip_stream) {
    if (W == nullptr || hr == nullptr || la == nullptr || counts == nullptr) return SP_EINVAL;
    if (out <= 0 || in <= 0 || ldw < in || !dtype_ok((int)dt)) return SP_EINVAL;
    if (n_la < 1 || n_la > 16) return SP_EINVAL;
    if (!(alpha > 0.0f && alpha <= 1.0f) || !(beta > 0.0f && beta <= 1.0f)) return SP_EINVAL;
    for (int i = 0; i < n_la; ++i)
        if (isnan(la[i]) || isinf(la[i])) return SP_EINVAL;
    if (reinterpret_cast<uintptr_t>(W) % elem_size((int)dt) != 0) return SP_EINVAL;
    if (reinterpret_cast<uintptr_t>(counts) % 8 != 0) return SP_EINVAL;
    const bool vec = weight_vec_ok(W, in, ldw, (int)dt, hr, nullptr);
    const sp::EwmaConsts c = sp::make_ewma_consts(alpha, beta, 0.0f);
    const hipError_t e = sp::launch_count_pruned(W, out, in, ldw, (int)dt, vec, hr, c, la, n_la, counts,
                                                 static_cast<hipStream_t>(hip_stream));
    return e == hipSuccess ? SP_OK : SP_EHIP;
}

int swiftprune_calibrate_la(const void* W, int64_t out, int64_t in, int64_t ldw, sp_dtype dt,
                            const float* hr, float alpha, float beta, float target_sparsity,
                            float tolerance, float la_lo, float la_hi, unsigned long long* counts_ws,
                            float* la, float* achieved, void* hip_stream) {
    if (W == nullptr || hr == nullptr || counts_ws == nullptr || la == nullptr || achieved == nullptr)
        return SP_EINVAL;
    if (out <= 0 || in <= 0 || ldw < in || !dtype_ok((int)dt)) return SP_EINVAL;
    if (!(alpha > 0.0f && alpha <= 1.0f) || !(beta > 0.0f && beta <= 1.0f)) return SP_EINVAL;
    if (!(target_sparsity > 0.0f && target_sparsity < 1.0f) || !(tolerance > 0.0f)) return SP_EINVAL;
    if (!(la_lo < la_hi) || isinf(la_lo) || isinf(la_hi)) return SP_EINVAL;
    if (reinterpret_cast<uintptr_t>(W) % elem_size((int)dt) != 0) return SP_EINVAL;
    if (reinterpret_cast<uintptr_t>(counts_ws) % 8 != 0) return SP_EINVAL;
    const bool vec = weight_vec_ok(W, in, ldw, (int)dt, hr, nullptr);
    const sp::EwmaConsts c = sp::make_ewma_consts(alpha, beta, 0.0f);
    int status = 1;
    const hipError_t e = sp::run_calibrate_la(W, out, in, ldw, (int)dt, vec, hr, c, target_sparsity, tolerance,
                                              la_lo, la_hi, counts_ws, la, achieved, &status,
                                              static_cast<hipStream_t>(hip_stream));
    if (e != hipSuccess) return SP_EHIP;
    return status == 0 ? SP_OK : SP_ERANGE;
}

size_t swiftprune_la_workspace_bytes(void) { return sp::la_workspace_bytes(); }

int swiftprune_calibrate_la_device(const void* W, int64_t out, int64_t in, int64_t ldw, sp_dtype dt,
                                   const float* hr, float alpha, float beta, float target_sparsity,
                                   void* workspace, size_t workspace_bytes, float* la_device,
                                   unsigned long long* pruned_device, int* status_device, void* hip_stream) {
    if (W == nullptr || hr == nullptr || workspace == nullptr || la_device == nullptr) return SP_EINVAL;
    if (out <= 0 || in <= 0 || ldw < in || !dtype_ok((int)dt)) return SP_EINVAL;
    if (!(alpha > 0.0f && alpha <= 1.0f) || !(beta > 0.0f && beta <= 1.0f)) return SP_EINVAL;
    if (!(target_sparsity > 0.0f && target_sparsity < 1.0f)) return SP_EINVAL;
    if (reinterpret_cast<uintptr_t>(W) % elem_size((int)dt) != 0) return SP_EINVAL;
    if (reinterpret_cast<uintptr_t>(workspace) % 256 != 0 || reinterpret_cast<uintptr_t>(la_device) % 4 != 0 ||
        reinterpret_cast<uintptr_t>(pruned_device) % 8 != 0 || reinterpret_cast<uintptr_t>(status_device) % 4 != 0)
        return SP_EINVAL;
    if (workspace_bytes < sp::la_workspace_bytes()) return SP_ENOSPC;
    const double total = (double)out * (double)in;
    double k = floor((double)target_sparsity * total + 0.5);
    if (k > total - 1.0) k = total - 1.0;
    const bool vec = weight_vec_ok(W, in, ldw, (int)dt, hr, nullptr);
    const sp::EwmaConsts c = sp::make_ewma_consts(alpha, beta, 0.0f);
    const hipError_t e = sp::launch_calibrate_la_device(W, out, in, ldw, (int)dt, vec, hr, c, (unsigned long long)k,
                                                        workspace, la_device, pruned_device, status_device,
                                                        static_cast<hipStream_t>(hip_stream));
    return e == hipSuccess ? SP_OK : SP_EHIP;
}

int swiftprune_score_select_la(const void* W, int64_t out, int64_t in, int64_t ldw, sp_dtype dt, const float* hr,
                               float alpha, float beta, const float* la_device, uint32_t* keep_mask,
                               int32_t* row_pruned, uint32_t flags, void* hip_stream) {
    if (W == nullptr || hr == nullptr || keep_mask == nullptr || la_device == nullptr) return SP_EINVAL;
    if (out <= 0 || in <= 0 || ldw < in || !dtype_ok((int)dt)) return SP_EINVAL;
    if (flags & ~SP_APPLY_INPLACE) return SP_EINVAL;
    if (!(alpha > 0.0f && alpha <= 1.0f) || !(beta > 0.0f && beta <= 1.0f)) return SP_EINVAL;
    if (reinterpret_cast<uintptr_t>(W) % elem_size((int)dt) != 0 || reinterpret_cast<uintptr_t>(la_device) % 4 != 0)
        return SP_EINVAL;
    const bool vec = out <= kMaxFastRows && weight_vec_ok(W, in, ldw, (int)dt, hr, nullptr);
    sp::EwmaConsts c = sp::make_ewma_consts(alpha, beta, 0.0f);
    c.la_dev = la_device;
    const hipError_t e = sp::launch_ewma_scan(W, out, in, ldw, (int)dt, vec, hr, c, keep_mask, row_pruned, nullptr,
                                              (flags & SP_APPLY_INPLACE) != 0, static_cast<hipStream_t>(hip_stream));
    return e == hipSuccess ? SP_OK : SP_EHIP;
}

int swiftprune_topk_select(const void* W, int64_t out, int64_t in, int64_t ldw, sp_dtype dt,
                           const float* hr, const int32_t* k_per_row, int64_t k_uniform,
                           uint32_t* keep_mask, uint32_t flags, void* hip_stream) {
    if (W == nullptr || hr == nullptr || keep_mask == nullptr) return SP_EINVAL;
    if (out <= 0 || in <= 0 || ldw < in || !dtype_ok((int)dt)) return SP_EINVAL;
    if (out > 0x7fffffff || in > (int64_t)1 << 30) return SP_EINVAL;
    if (flags & ~SP_APPLY_INPLACE) return SP_EINVAL;
    if (reinterpret_cast<uintptr_t>(W) % elem_size((int)dt) != 0) return SP_EINVAL;
    const hipError_t e = sp::launch_topk_select(W, out, in, ldw, (int)dt, hr, k_per_row, k_uniform, keep_mask,
                                                (flags & SP_APPLY_INPLACE) != 0,
                                                static_cast<hipStream_t>(hip_stream));
    return e == hipSuccess ? SP_OK : SP_EHIP;
}

int swiftprune_nm_select(const void* W, int64_t out, int64_t in, int64_t ldw, sp_dtype dt,
                         const float* hr, int n_keep, int m_group, uint32_t* keep_mask, float* scores,
                         uint32_t flags, void* hip_stream) {
    if (W == nullptr || hr == nullptr || keep_mask == nullptr) return SP_EINVAL;
    if (out <= 0 || in <= 0 || ldw < in || !dtype_ok((int)dt)) return SP_EINVAL;
    if (m_group != 4 && m_group != 8 && m_group != 16) return SP_EINVAL;
    if (n_keep <= 0 || n_keep >= m_group || in % m_group != 0) return SP_EINVAL;
    if (flags & ~SP_APPLY_INPLACE) return SP_EINVAL;
    if (reinterpret_cast<uintptr_t>(W) % elem_size((int)dt) != 0) return SP_EINVAL;
    const bool vec = out <= kMaxFastRows && weight_vec_ok(W, in, ldw, (int)dt, hr, scores);
    const hipError_t e =
        sp::launch_nm_select(W, out, in, ldw, (int)dt, vec, hr, n_keep, m_group, keep_mask, scores,
                             (flags & SP_APPLY_INPLACE) != 0, static_cast<hipStream_t>(hip_stream));
    return e == hipSuccess ? SP_OK : SP_EHIP;
}

static bool nm_pattern_ok(int64_t in, int n_keep, int m_group) {
    if (m_group != 4 && m_group != 8 && m_group != 16) return false;
    return n_keep > 0 && n_keep < m_group && in % m_group == 0;
}

size_t swiftprune_nm_meta_words(int64_t in, int n_keep, int m_group) {
    if (in <= 0 || !nm_pattern_ok(in, n_keep, m_group)) return 0;
    return (size_t)sp::nm_meta_words(in, n_keep, m_group);
}

int swiftprune_compact_nm(const void* W, int64_t out, int64_t in, int64_t ldw, sp_dtype dt,
                          const uint32_t* keep_mask, int n_keep, int m_group, void* values,
                          uint32_t* meta, void* hip_stream) {
    if (W == nullptr || keep_mask == nullptr || values == nullptr || meta == nullptr) return SP_EINVAL;
    if (out <= 0 || in <= 0 || ldw < in || !dtype_ok((int)dt)) return SP_EINVAL;
    if (!nm_pattern_ok(in, n_keep, m_group)) return SP_EINVAL;
    if (reinterpret_cast<uintptr_t>(W) % elem_size((int)dt) != 0 ||
        reinterpret_cast<uintptr_t>(values) % elem_size((int)dt) != 0)
        return SP_EINVAL;
    const hipError_t e = sp::launch_compact_nm(W, out, in, ldw, (int)dt, keep_mask, n_keep, m_group, values,
                                               meta, static_cast<hipStream_t>(hip_stream));
    return e == hipSuccess ? SP_OK : SP_EHIP;
}

int swiftprune_expand_nm(const void* values, const uint32_t* meta, int64_t out, int64_t in, sp_dtype dt,
                         int n_keep, int m_group, void* W_out, int64_t ldw_out, void* hip_stream) {
    if (values == nullptr || meta == nullptr || W_out == nullptr) return SP_EINVAL;
    if (out <= 0 || in <= 0 || ldw_out < in || !dtype_ok((int)dt)) return SP_EINVAL;
    if (!nm_pattern_ok(in, n_keep, m_group)) return SP_EINVAL;
    if (reinterpret_cast<uintptr_t>(W_out) % elem_size((int)dt) != 0 ||
        reinterpret_cast<uintptr_t>(values) % elem_size((int)dt) != 0)
        return SP_EINVAL;
    const hipError_t e = sp::launch_expand_nm(values, meta, out, in, (int)dt, n_keep, m_group, W_out, ldw_out,
                                              static_cast<hipStream_t>(hip_stream));
    return e == hipSuccess ? SP_OK : SP_EHIP;
}

int swiftprune_apply(void* W, int64_t out, int64_t in, int64_t ldw, sp_dtype dt,
                     const uint32_t* keep_mask, void* hip_stream) {
    if (W == nullptr || keep_mask == nullptr) return SP_EINVAL;
    if (out <= 0 || in <= 0 || ldw < in || !dtype_ok((int)dt)) return SP_EINVAL;
    if (reinterpret_cast<uintptr_t>(W) % elem_size((int)dt) != 0) return SP_EINVAL;
    const bool vec = weight_vec_ok(W, in, ldw, (int)dt, nullptr, nullptr);
    const hipError_t e = sp::launch_apply(W, out, in, ldw, (int)dt, vec, keep_mask,
                                          static_cast<hipStream_t>(hip_stream));
    return e == hipSuccess ? SP_OK : SP_EHIP;
}

}  // extern "C"

// Host-side launchers of the SwiftPrune kernels (internal to the library).
#pragma once

#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

namespace sp {

// ---- step 1: calibration statistics ----
// Launch geometry of the statistics pass, a pure function of the shape so the
// workspace size can be computed without a device.
struct StatsPlan {
    int epu;                 // elements per 16-byte unit a lane loads (8 bf16 / 4 fp32), 1 = element-wise path
    int64_t units;           // ceil(in / epu)
    int strip_units;         // units per column strip (<= 256, one per lane of a workgroup)
    int nstrips;             // column strips
    int splits;              // workgroups per strip; row batches are dealt to them round-robin
    int unroll;              // rows per batch (4, 8 or 16)
    int64_t rows_per_split;  // upper bound of the tokens one workgroup sees
    int combine_groups;      // workgroups of the combine kernel (64 columns each)
    size_t partial_floats;   // splits * units * epu
    bool plain_loads;        // experiment: ordinary instead of non-temporal loads
};

// Launch-shape overrides for measurements, read from the environment at every call (unset = the built-in
// choices, which were swept on MI355X):
//   SWIFTPRUNE_STATS_PLAN   = "<rows in flight: 4|8|16>,<workgroups>[,plain]"   statistics kernel
//   SWIFTPRUNE_SELECT_TEAM  = "<0|1|2|4>[,direct]"                               wavefronts per row, EWMA kernel (0 = built-in);
//                                                                               direct = no LDS staging, no request ahead
//   SWIFTPRUNE_BAND_GROUPS  = "<apply>,<N:M select>"                            workgroups of the band kernels
struct Tuning {
    int stats_rows, stats_groups;  // 0 = default
    bool stats_plain;
    int team;                      // 0 = default
    bool select_direct;
    int apply_groups, select_groups;
};
Tuning read_tuning();
constexpr size_t kStatsHeaderBytes = 256;  // counters at the start of the workspace
StatsPlan make_stats_plan(int64_t tokens, int64_t in, int dt, bool vec);
size_t stats_workspace_bytes(const StatsPlan& p);  // header + per-workgroup S sums + partial rows

hipError_t launch_layer_stats(const void* X, int64_t tokens, int64_t in, int64_t ldx, int dt, bool vec,
                              float* xsq, float* S, float* hr, int accumulate, int finalize,
                              void* workspace, hipStream_t stream);

// ---- several weight matrices that share one layer input (same columns, same channel factor), pruned by
// one launch: the rows of all matrices are numbered consecutively, matrix j owning [row_end[j-1], row_end[j]) ----
constexpr int kMaxGroup = 8;
struct RowGroups {
    int n;                          // matrices in use (1 .. kMaxGroup)
    int32_t row_end[kMaxGroup];     // running totals of the row counts (all rows together < 2^31); unused entries repeat the last total
    void* W[kMaxGroup];
    int64_t ldw[kMaxGroup];
    uint32_t* keep_mask[kMaxGroup];
    int32_t* row_pruned[kMaxGroup];  // nullable per matrix
    __host__ __device__ int32_t total() const { return row_end[kMaxGroup - 1]; }
};

// ---- steps 2+3: EWMA selection ----
struct EwmaConsts {
    float alpha, beta, la;
    float inv_alpha;    // 1 / alpha
    float thr_scale;    // (1-alpha) * la * beta: prune iff alpha*x_k - L_k > thr_scale * y_{k-1}
    float A_pow[9];     // (1-alpha)^k, k = 0..8
    float B_pow[9];     // (1-beta)^k
    float A8_pow[65];   // ((1-alpha)^8)^k, k = 0..64: the weight of a state k lanes (8 k columns) to the left
    float B8_pow[65];
    const float* la_dev;  // nullable: when set, la is read from device memory by the kernel (la, thr_scale unused)
};
EwmaConsts make_ewma_consts(float alpha, float beta, float la);

hipError_t launch_ewma_scan(const void* W, int64_t out, int64_t in, int64_t ldw, int dt, bool vec,
                            const float* hr, const EwmaConsts& c, uint32_t* keep_mask,
                            int32_t* row_pruned, float* scores, bool apply, hipStream_t stream);
// fast path for the 16-byte-vector layout and alpha < 1; team = wavefronts per row (1, 2, 4; 0 = by row count)
hipError_t launch_ewma_team(const RowGroups& g, int64_t in, int dt, const float* hr, const EwmaConsts& c,
                            bool apply, int team, hipStream_t stream);
RowGroups single_matrix(const void* W, int64_t out, int64_t ldw, uint32_t* keep_mask, int32_t* row_pruned);
hipError_t launch_ewma_sequential(const void* W, int64_t out, int64_t in, int64_t ldw, int dt,
                                  const float* hr, float alpha, float beta, float la,
                                  uint32_t* keep_mask, int32_t* row_pruned, float* scores, bool apply,
                                  hipStream_t stream);

hipError_t launch_channel_factor(const float* xsq, const float* S, int64_t in, float* hr, hipStream_t stream);
// statistics from per-piece sums of squares formed by the producer of X (stats_partials.hip)
hipError_t launch_stats_from_pieces(const float* P, int64_t parts, int64_t in, int64_t ld, float* xsq, float* S,
                                    float* hr, int accumulate, int finalize, hipStream_t stream);

// ---- est / dev sequences written out (diagnostic) ----
hipError_t launch_ewma_trace(const void* W, int64_t out, int64_t in, int64_t ldw, int dt, bool vec,
                             const float* hr, const EwmaConsts& c, float* est, float* dev,
                             hipStream_t stream);

// ---- threshold calibration (count the pruned weights for up to 16 candidate la in one pass) ----
hipError_t launch_count_pruned(const void* W, int64_t out, int64_t in, int64_t ldw, int dt, bool vec,
                               const float* hr, const EwmaConsts& c, const float* la, int n_la,
                               unsigned long long* counts, hipStream_t stream);
size_t la_workspace_bytes();
hipError_t launch_calibrate_la_device(const void* W, int64_t out, int64_t in, int64_t ldw, int dt, bool vec,
                                      const float* hr, const EwmaConsts& c, unsigned long long target_count,
                                      void* workspace, float* la_dev, unsigned long long* pruned_dev,
                                      int* status_dev, hipStream_t stream);
hipError_t run_calibrate_la(const void* W, int64_t out, int64_t in, int64_t ldw, int dt, bool vec,
                            const float* hr, const EwmaConsts& c, float target, float tolerance,
                            float la_lo, float la_hi, unsigned long long* counts_dev, float* la_out,
                            float* achieved_out, int* status, hipStream_t stream);

// ---- exact per-row top-k comparator ----
hipError_t launch_topk_select(const void* W, int64_t out, int64_t in, int64_t ldw, int dt,
                              const float* hr, const int32_t* k_per_row, int64_t k_uniform,
                              uint32_t* keep_mask, bool apply, hipStream_t stream);

// ---- compact N:M storage ----
int64_t nm_meta_words(int64_t in, int n_keep, int m_group);
hipError_t launch_compact_nm(const void* W, int64_t out, int64_t in, int64_t ldw, int dt,
                             const uint32_t* keep_mask, int n_keep, int m_group, void* values,
                             uint32_t* meta, hipStream_t stream);
hipError_t launch_expand_nm(const void* values, const uint32_t* meta, int64_t out, int64_t in, int dt,
                            int n_keep, int m_group, void* W_out, int64_t ldw, hipStream_t stream);

// ---- steps 2+3 structured, step 4 ----
hipError_t launch_nm_select(const void* W, int64_t out, int64_t in, int64_t ldw, int dt, bool vec,
                            const float* hr, int n_keep, int m_group, uint32_t* keep_mask,
                            float* scores, bool apply, hipStream_t stream);
// N:M selection of a group of matrices in one launch (16-byte-vector layout only)
hipError_t launch_nm_select_group(const RowGroups& g, int64_t in, int dt, const float* hr, int n_keep,
                                  int m_group, float* scores, bool apply, hipStream_t stream);
hipError_t launch_apply(void* W, int64_t out, int64_t in, int64_t ldw, int dt, bool vec,
                        const uint32_t* keep_mask, hipStream_t stream);

}  // namespace sp

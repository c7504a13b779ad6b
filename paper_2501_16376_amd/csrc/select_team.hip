// Steps 2+3 of the SwiftPrune layer path, unstructured, fast path (Sec. 3.1 score
// equation; Sec. 3.2; Algorithm 1 loop; state-update table of Sec. 3.1; S held fixed).
//
// The two recurrences of a row
//     x_q = A x_{q-1} + L_q            (x = est / alpha,  A = 1 - alpha,  x_{-1} = L_0 / alpha)
//     y_q = B y_{q-1} + |alpha x_q - L_q|   (y = dev / beta, B = 1 - beta,  y_{-1} = 0)
// are linear once the sum S is fixed, so a row can be cut into pieces that are
// evaluated from a zero state and stitched together afterwards.  Three levels:
//   lane      8 consecutive columns, sequential
//   wavefront 64 lanes = one segment of 512 columns: weighted DPP scan of the
//             lanes' end values (scan_common.hpp); a wavefront chains kSegs
//             consecutive segments by itself
//   team      NW wavefronts of a workgroup share a row: wavefront p owns the
//             p-th run of kSegs segments of every span of NW * kSegs segments,
//             publishes the end value of its run (zero entry state) in LDS, and
//             after one barrier every wavefront folds the runs before its own
//             into its entry state:  in_p = P in_{p-1} + end_{p-1},  P = A^(512 kSegs).
// The y recurrence needs the final x (through the absolute value), so a span
// takes two such exchanges.  The lanes' entry states are only then turned into
// per-element values, so the stitching costs no extra work per weight.
// NW = 4 puts a whole 4096-column row in flight at once (short matrices: four
// times the wavefronts, a quarter of the serial work per row); NW = 1 is one
// wavefront per row with no LDS traffic and no barriers (tall matrices).
//
// Decisions:  L_q < est_{q-1} - la dev_{q-1}.  The est update gives
// est_q - L_q = A (est_{q-1} - L_q), hence  prune  <=>  alpha x_q - L_q > (A la beta) y_{q-1}.
// The scan reorders additions of non-negative terms: est/dev differ from the
// sequential fp32 walk by a few ulp.
#include "scan_common.hpp"

#include <math.h>

namespace sp {

constexpr int kTeamThreads = 256;
constexpr int kSegs = 2;  // consecutive 512-column segments a wavefront handles per span

// Inclusive weighted scans over the 64 lanes of two independent values at once:
//     r_j = sum_{i <= j} m^(j-i) v_i        (m = c.m1 per lane step)
// as row_shr 1/2/4/8, row_bcast 15, row_bcast 31 steps with per-lane powers.  One step is a single
// v_fmac_f32 with a DPP source operand (the compiler spends three instructions on it); the two chains
// alternate so that each fills one of the two wait states the other needs between writing a register
// and reading it through DPP (the assembler does not see that hazard inside inline assembly, hence the
// explicit s_nop).  In-place use is safe: row_shr reads stay inside the 16-lane row being written, and
// the row_bcast steps read lanes 15/47 and 31, whose rows are masked off for writing.
__device__ __forceinline__ void team_scan2(float& r0, float& r1, const ScanLaneConsts& c) {
#define SP_STEP(mul, ctrl)                                     \
    "s_nop 0\n\t"                                              \
    "v_fmac_f32_dpp %0, %0, " mul " " ctrl " bank_mask:0xf\n\t" \
    "v_fmac_f32_dpp %1, %1, " mul " " ctrl " bank_mask:0xf\n\t"
    // one statement, so that nothing is scheduled into it and the wait states are exactly these; the
    // extra s_nop in front covers r0 / r1 having been written by the instruction just before, the one at
    // the end a DPP read of r1 right behind
    asm volatile("s_nop 0\n\t"
                 SP_STEP("%2", "row_shr:1 row_mask:0xf")
                 SP_STEP("%3", "row_shr:2 row_mask:0xf")
                 SP_STEP("%4", "row_shr:4 row_mask:0xf")
                 SP_STEP("%5", "row_shr:8 row_mask:0xf")
                 SP_STEP("%6", "row_bcast:15 row_mask:0xa")
                 SP_STEP("%7", "row_bcast:31 row_mask:0xc")
                 "s_nop 1"
                 : "+v"(r0), "+v"(r1)
                 : "v"(c.m1), "v"(c.m2), "v"(c.m4), "v"(c.m8), "v"(c.cross15), "v"(c.cross31));
#undef SP_STEP
}

// workgroup barrier that orders LDS traffic only: outstanding global loads and stores keep flying
__device__ __forceinline__ void team_barrier() {
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup", "local");
    __builtin_amdgcn_s_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup", "local");
}

// grid = ceil(rows of all matrices / (4 / NW)), block = 256 (4 wavefronts).  Requires the 16-byte-vector layout
// (W and hr 16-byte aligned, in % 8 == 0, ldw a multiple of 16 bytes) and alpha < 1.
template <int DT, int NW>
__global__ __launch_bounds__(kTeamThreads) void ewma_team_kernel(
    const RowGroups g, int64_t in, const float* __restrict__ hr, const EwmaConsts c, int apply) {
    constexpr int kRowsPerGroup = 4 / NW;
    __shared__ float lds_x[kRowsPerGroup][NW];
    __shared__ float lds_y[kRowsPerGroup][NW];
    __shared__ float lds_first[kRowsPerGroup];
    __shared__ int lds_count[kRowsPerGroup][NW];

    const int lane = threadIdx.x & (kWave - 1);
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);  // uniform: the row lookup below stays scalar
    const int slot = wave / NW;  // which row of the workgroup
    const int part = wave % NW;  // which run of the row's spans
    const int32_t global_row = (int32_t)(blockIdx.x * kRowsPerGroup + slot);   // the launcher keeps the row total below 2^31
    const bool has_row = global_row < g.total();
    // a wavefront without a row (past the last one) still walks the loop and meets the barriers, with all
    // its lanes switched off
    const RowOwner<RowGroups> own(g, has_row ? global_row : 0);
    void* const W = own.W;
    uint32_t* const keep_mask = own.keep_mask;
    int32_t* const row_pruned = own.row_pruned;
    const int64_t row = own.row;
    const int64_t cols = has_row ? in : 0;
    const int64_t row_off = row * own.ldw;
    const int64_t mask_words = (in + 31) >> 5;
    const int64_t span_cols = (int64_t)NW * kSegs * 512;
    const int64_t nspans = (in + span_cols - 1) / span_cols;

    const ScanLaneConsts ce = make_lane_consts(c.A8_pow, lane);
    const ScanLaneConsts cd = make_lane_consts(c.B8_pow, lane);
    const float A = c.A_pow[1], B = c.B_pow[1];
    const float thr_scale = ewma_thr_scale(c);
    const float A512 = c.A8_pow[64], B512 = c.B8_pow[64];
    // entry weight of a run's s-th segment at this lane, and of a whole run
    float shift_x[kSegs], shift_y[kSegs];
    shift_x[0] = ce.shift;
    shift_y[0] = cd.shift;
#pragma unroll
    for (int s = 1; s < kSegs; ++s) {
        shift_x[s] = shift_x[s - 1] * A512;
        shift_y[s] = shift_y[s - 1] * B512;
    }
    float run_x = 1.f, run_y = 1.f;
#pragma unroll
    for (int s = 0; s < kSegs; ++s) {
        run_x *= A512;
        run_y *= B512;
    }

    static_assert(kSegs == 2, "the scans below run two segments side by side");
    float span_x = 0.f, span_y = 0.f;  // state entering the current span (uniform)
    int pruned = 0;
    // lanes past the end of the row (and wavefronts without a row) read valid memory and compute on it, but
    // store nothing: whatever they compute can only reach columns to their right, which do not exist either
    const int64_t row_off_ld = row_off;

    for (int64_t span = 0; span < nspans; ++span) {
        const int64_t q_run = span * span_cols + (int64_t)part * (kSegs * 512) + (int64_t)lane * 8;

        // ---- scores and the x recurrence of this run, from a zero entry state
        Unpacked8<DT> w[kSegs];
        float L[kSegs][8], x[kSegs][8], x_in[kSegs];
        Factor8 f[kSegs];
#pragma unroll
        for (int s = 0; s < kSegs; ++s) {
            const int64_t q0 = q_run + (int64_t)s * 512;
            const int64_t q_ld = q0 < cols ? q0 : 0;
            Chunk8<DT> raw;
            raw.load_vec(W, row_off_ld + q_ld);
            f[s].load_vec(hr, q_ld);
            w[s].unpack(raw);
        }
#pragma unroll
        for (int s = 0; s < kSegs; ++s) {
#pragma unroll
            for (int k = 0; k < 8; ++k) L[s][k] = score_of(w[s].w[k], f[s].v[k]);
            x[s][0] = L[s][0];
#pragma unroll
            for (int k = 1; k < 8; ++k) x[s][k] = fmaf(A, x[s][k - 1], L[s][k]);
        }
        float end0, end1;
        {
            float r0 = x[0][7], r1 = x[1][7];
            team_scan2(r0, r1, ce);
            end0 = readlane_f(r0, kWave - 1);
            end1 = readlane_f(r1, kWave - 1);
            x_in[0] = dpp_f<kWaveShr1>(r0);                            // lane 0: nothing to its left
            x_in[1] = fmaf(ce.shift, end0, dpp_f<kWaveShr1>(r1));     // + what segment 0 leaves behind
        }
        float chain = fmaf(A512, end0, end1);                         // end of the run from a zero entry state
        float enter_x;
        if (NW > 1) {
            if (lane == 0) {
                lds_x[slot][part] = chain;
                if (part == 0 && span == 0) lds_first[slot] = L[0][0] * c.inv_alpha;
            }
            team_barrier();
            enter_x = span == 0 ? lds_first[slot] : span_x;
            float t = enter_x;
#pragma unroll
            for (int v = 0; v < NW; ++v) {
                if (v == part) enter_x = t;
                t = fmaf(run_x, t, lds_x[slot][v]);
            }
            span_x = t;
        } else {
            enter_x = span == 0 ? readlane_f(L[0][0], 0) * c.inv_alpha : span_x;
            span_x = fmaf(run_x, enter_x, chain);
        }

        // ---- final x, gaps, and the y recurrence from a zero entry state
        float y[kSegs][8], y_in[kSegs];
#pragma unroll
        for (int s = 0; s < kSegs; ++s) {
            const float xin = fmaf(shift_x[s], enter_x, x_in[s]);
#pragma unroll
            for (int k = 0; k < 8; ++k) x[s][k] = fmaf(c.alpha, fmaf(c.A_pow[k + 1], xin, x[s][k]), -L[s][k]);  // now the gap
            y[s][0] = fabsf(x[s][0]);
#pragma unroll
            for (int k = 1; k < 8; ++k) y[s][k] = fmaf(B, y[s][k - 1], fabsf(x[s][k]));
        }
        {
            float r0 = y[0][7], r1 = y[1][7];
            team_scan2(r0, r1, cd);
            end0 = readlane_f(r0, kWave - 1);
            end1 = readlane_f(r1, kWave - 1);
            y_in[0] = dpp_f<kWaveShr1>(r0);
            y_in[1] = fmaf(cd.shift, end0, dpp_f<kWaveShr1>(r1));
        }
        chain = fmaf(B512, end0, end1);
        float enter_y;
        if (NW > 1) {
            if (lane == 0) lds_y[slot][part] = chain;
            team_barrier();
            float t = span_y;
            enter_y = t;
#pragma unroll
            for (int v = 0; v < NW; ++v) {
                if (v == part) enter_y = t;
                t = fmaf(run_y, t, lds_y[slot][v]);
            }
            span_y = t;
        } else {
            enter_y = span_y;
            span_y = fmaf(run_y, enter_y, chain);
        }

        // ---- decisions, mask words, in-place zeroing
#pragma unroll
        for (int s = 0; s < kSegs; ++s) {
            const int64_t q0 = q_run + (int64_t)s * 512;
            const bool on = q0 < cols;
            const float yin = fmaf(shift_y[s], enter_y, y_in[s]);
            bool prune[8];
            // the row's first weight is never pruned (est starts at its score, dev at 0); in scaled form
            // that equality is only approximate, so it is stated
            prune[0] = (x[s][0] > thr_scale * yin) && q0 != 0;
#pragma unroll
            for (int k = 1; k < 8; ++k)
                prune[k] = x[s][k] > thr_scale * fmaf(c.B_pow[k], yin, y[s][k - 1]);
            const uint32_t gone = pack_bits8(prune);  // bit k = prune[k]
            const uint32_t keep = on ? (gone ^ 0xffu) : 0u;
            pruned += on ? __popc(gone) : 0;
            const uint32_t word = quad_gather_bytes(keep, lane);
            if ((lane & 3) == 0 && on) keep_mask[row * mask_words + (q0 >> 5)] = word;
            if (apply && on) w[s].store_pruned(W, row_off + q0, prune);
        }
    }

    // counts: unconditional, so that every wavefront of the workgroup meets the barrier
    {
#pragma unroll
        for (int off = 32; off > 0; off >>= 1) pruned += __shfl_xor(pruned, off, kWave);
        if (NW > 1) {
            if (lane == 0) lds_count[slot][part] = pruned;
            team_barrier();
            if (lane == 0 && part == 0 && has_row && row_pruned != nullptr) {
                int total = 0;
#pragma unroll
                for (int v = 0; v < NW; ++v) total += lds_count[slot][v];
                row_pruned[row] = total;
            }
        } else if (lane == 0 && has_row && row_pruned != nullptr) {
            row_pruned[row] = pruned;
        }
    }
}

template <int DT, int NW>
static hipError_t launch_team_t(const RowGroups& g, int64_t in, const float* hr, const EwmaConsts& c, bool apply,
                                hipStream_t stream) {
    constexpr int rows = 4 / NW;
    const int64_t groups = ((int64_t)g.total() + rows - 1) / rows;
    hipLaunchKernelGGL((ewma_team_kernel<DT, NW>), dim3((unsigned)groups), dim3(kTeamThreads), 0, stream, g, in, hr, c,
                       apply ? 1 : 0);
    return hipGetLastError();
}

RowGroups single_matrix(const void* W, int64_t out, int64_t ldw, uint32_t* keep_mask, int32_t* row_pruned) {
    RowGroups g;
    g.n = 1;
    for (int j = 0; j < kMaxGroup; ++j) {
        g.row_end[j] = (int32_t)out;
        g.W[j] = const_cast<void*>(W);
        g.ldw[j] = ldw;
        g.keep_mask[j] = keep_mask;
        g.row_pruned[j] = row_pruned;
    }
    return g;
}

// team size: `team` = 1, 2 or 4 wavefronts per row; 0 picks by the number of rows
hipError_t launch_ewma_team(const RowGroups& g, int64_t in, int dt, const float* hr, const EwmaConsts& c,
                            bool apply, int team, hipStream_t stream) {
    // at least four wavefronts per SIMD (1024 SIMDs) before a row gets a wavefront to itself
    const int64_t out = g.total();
    if (team == 0) team = read_tuning().team;  // measurement override
    if (team == 0) team = out <= 1024 ? 4 : (out <= 2048 ? 2 : 1);
    return with_dtype(dt, [&](auto tag) {
        constexpr int DT = decltype(tag)::value;
        switch (team) {
            case 4: return launch_team_t<DT, 4>(g, in, hr, c, apply, stream);
            case 2: return launch_team_t<DT, 2>(g, in, hr, c, apply, stream);
            default: return launch_team_t<DT, 1>(g, in, hr, c, apply, stream);
        }
    });
}

}  // namespace sp

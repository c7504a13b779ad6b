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
// wavefront per row with no exchange between wavefronts (tall matrices).
//
// Decisions:  L_q < est_{q-1} - la dev_{q-1}.  The est update gives
// est_q - L_q = A (est_{q-1} - L_q), hence  prune  <=>  alpha x_q - L_q > (A la beta) y_{q-1}.
// The scan reorders additions of non-negative terms: est/dev differ from the
// sequential fp32 walk by a few ulp.
#include "scan_common.hpp"

#include <math.h>

#include <type_traits>

namespace sp {

constexpr int kTeamThreads = 256;
constexpr int kSegs = 2;  // consecutive 512-column segments a wavefront handles per span
constexpr int64_t kStagedCols = 4096;  // channel factors staged in LDS at a time (16 KB a workgroup)

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

// Where the factor of column q (relative to the staged chunk, a multiple of 4) sits in LDS: per 512-column
// segment first the lanes' factors 0..3, then their factors 4..7.  A lane reads its eight factors with two
// 16-byte reads; in this layout neighbouring lanes' reads are 16 bytes apart (in column order they would be
// 32 bytes apart and collide two by two on the LDS banks).
__device__ __forceinline__ int staged_slot(int q) {
    return (q & ~511) | ((q & 4) << 6) | (((q & 511) >> 3) << 2);
}

// workgroup barrier that orders LDS traffic only: outstanding global loads and stores keep flying
__device__ __forceinline__ void team_barrier() {
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup", "local");
    __builtin_amdgcn_s_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup", "local");
}

// grid = ceil(rows of all matrices / (4 / NW)), block = 256 (4 wavefronts).  Requires the 16-byte-vector layout
// (W and hr 16-byte aligned, in % 8 == 0, ldw a multiple of 16 bytes) and alpha < 1.
//
// STAGED (the built-in choice): the channel factors of kStagedCols columns at a time are copied into LDS by the
// workgroup (dynamic shared memory: kStagedCols floats), and the weights of the next span are requested while
// the current one is worked on, so that a span starts with nothing to wait for but LDS.  The wavefronts of a
// launch that fits the device at once move in lock step - all wait for their loads, then all compute - so
// without this the memory system idles while the vector units work and the other way round.  The other
// version (each span loads its weights and factors from global memory and waits) is kept for comparison.
//
// A span that lies inside the row (FULL) stores without any predicate: every store is then issued on every
// path, the number of memory operations behind the requested loads is fixed, and the wait for those loads
// does not have to include the stores that follow them (vmcnt counts loads and stores in one order).
template <int DT, int NW, bool STAGED, bool APPLY>
__global__ __launch_bounds__(kTeamThreads) void ewma_team_kernel(
    const RowGroups g, int64_t in, const float* __restrict__ hr, const EwmaConsts c) {
    constexpr int kRowsPerGroup = 4 / NW;
    extern __shared__ __align__(16) float lds_hr[];
    __shared__ float lds_x[kRowsPerGroup][NW];
    __shared__ float lds_y[kRowsPerGroup][NW];
    __shared__ float lds_first[kRowsPerGroup];
    __shared__ int lds_count[kRowsPerGroup][NW];

    const int lane = threadIdx.x & (kWave - 1);
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);  // uniform: the row lookup below stays scalar
    const int slot = wave / NW;  // which row of the workgroup
    const int part = wave % NW;  // which run of the row's spans
    const int32_t global_row = (int32_t)(blockIdx.x * kRowsPerGroup + slot);   // the launcher keeps the row total below 2^31
    const bool has_row = __builtin_amdgcn_readfirstlane((int)(global_row < g.total())) != 0;  // uniform, and known to be
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
    const int nspans = (int)((in + span_cols - 1) / span_cols);  // 32-bit: the scalar unit compares no wider

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
    const int64_t lane_col = (int64_t)part * (kSegs * 512) + (int64_t)lane * 8;

    Chunk8<DT> ahead[kSegs];  // STAGED: the weights of the span to come
    auto request = [&](int span) {
#pragma unroll
        for (int s = 0; s < kSegs; ++s) {
            const int64_t q0 = (int64_t)span * span_cols + lane_col + (int64_t)s * 512;
            ahead[s].load_vec(W, row_off + (q0 < cols ? q0 : 0));
        }
    };
    // STAGED: kStagedCols factors at a time sit in LDS; a chunk is replaced every kStageSpans spans, by all
    // wavefronts of the workgroup together (they walk the same columns, of one row or of several)
    constexpr int kStageSpans = (int)(kStagedCols / ((int64_t)NW * kSegs * 512));
    auto stage = [&](int span) {
        if (span != 0) team_barrier();  // nobody reads the chunk before any more
        const int64_t base = (int64_t)span * span_cols;
        const int64_t n = in - base < kStagedCols ? in - base : kStagedCols;
        // all loads first, then all LDS writes: one memory latency per chunk, not one per pass
        constexpr int kPasses = (int)(kStagedCols / (kTeamThreads * 4));
        u32x4 v[kPasses];  // a native vector type: an array of HIP's float4 ends up in private memory
#pragma unroll
        for (int j = 0; j < kPasses; ++j) {
            const int64_t q = (int64_t)threadIdx.x * 4 + (int64_t)j * kTeamThreads * 4;
            v[j] = *reinterpret_cast<const u32x4*>(hr + base + (q < n ? q : 0));
        }
#pragma unroll
        for (int j = 0; j < kPasses; ++j) {
            const int64_t q = (int64_t)threadIdx.x * 4 + (int64_t)j * kTeamThreads * 4;
            *reinterpret_cast<u32x4*>(lds_hr + staged_slot((int)q)) = v[j];  // past the row end: a copy of the chunk's start, never read
        }
        team_barrier();
    };
    if (STAGED) {
        request(0);
        stage(0);
        // The first request is taken as complete here (the copy above has waited for later loads anyway).
        // Entering the loop with it still pending would make the compiler wait, at the top of every
        // iteration, as if the newest memory operations were loads to be waited for - and there they are
        // the stores of the span before.
#pragma unroll
        for (int s = 0; s < kSegs; ++s)
#pragma unroll
            for (int j = 0; j < (int)(sizeof(ahead[s].raw) / sizeof(ahead[s].raw[0])); ++j)
                asm volatile("" : "+v"(ahead[s].raw[j]));
    }

    auto work = [&](int span, auto full_tag, auto more_tag) {
        constexpr bool FULL = decltype(full_tag)::value;
        constexpr bool MORE = decltype(more_tag)::value;  // a span is known to follow (otherwise: looked up)
        const int64_t q_run = (int64_t)span * span_cols + lane_col;
        const int64_t chunk_base = (int64_t)(span - span % kStageSpans) * span_cols;  // first column of the staged chunk
        if (STAGED && span != 0 && span % kStageSpans == 0) stage(span);

        // ---- scores and the x recurrence of this run, from a zero entry state
        Unpacked8<DT> w[kSegs];
        float L[kSegs][8], x[kSegs][8], x_in[kSegs];
        Factor8 f[kSegs];
#pragma unroll
        for (int s = 0; s < kSegs; ++s) {
            const int64_t q0 = q_run + (int64_t)s * 512;
            const int64_t q_ld = (FULL || q0 < cols) ? q0 : 0;
            if (STAGED) {
                const int at = staged_slot((FULL || q0 < cols) ? (int)(q0 - chunk_base) : 0);
                const float4 lo = *reinterpret_cast<const float4*>(lds_hr + at);
                const float4 hi = *reinterpret_cast<const float4*>(lds_hr + at + 256);
                f[s].v[0] = lo.x; f[s].v[1] = lo.y; f[s].v[2] = lo.z; f[s].v[3] = lo.w;
                f[s].v[4] = hi.x; f[s].v[5] = hi.y; f[s].v[6] = hi.z; f[s].v[7] = hi.w;
                w[s].unpack(ahead[s]);
            } else {
                Chunk8<DT> raw;
                raw.load_vec(W, row_off + q_ld);
                f[s].load_vec(hr, q_ld);
                w[s].unpack(raw);
            }
        }
        if (STAGED && (MORE || span + 1 < nspans)) request(span + 1);
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
            const bool on = FULL || q0 < cols;
            const float yin = fmaf(shift_y[s], enter_y, y_in[s]);
            // decisions as lane masks: they feed the bit packing and the zeroing from scalar registers
            uint64_t prune[8];
            // the row's first weight is never pruned (est starts at its score, dev at 0); in scaled form
            // that equality is only approximate, so it is stated
            prune[0] = __builtin_amdgcn_ballot_w64((x[s][0] > thr_scale * yin) && q0 != 0);
#pragma unroll
            for (int k = 1; k < 8; ++k)
                prune[k] = __builtin_amdgcn_ballot_w64(x[s][k] > thr_scale * fmaf(c.B_pow[k], yin, y[s][k - 1]));
            const uint32_t gone = pack_masks8(prune);  // bit k = decision k of this lane
            const uint32_t keep = on ? (gone ^ 0xffu) : 0u;
            pruned += on ? __popc(gone) : 0;
            const uint32_t word = quad_gather_bytes(keep, lane);
            // the four lanes of a quad hold the same word; in a FULL span all of them store it
            if (FULL || ((lane & 3) == 0 && on)) keep_mask[row * mask_words + (q0 >> 5)] = word;
            if (APPLY && on) w[s].store_pruned_masks(W, row_off + q0, prune);
        }
    };
    // spans that end inside the row: only a wavefront that has a row takes the unpredicated code (the choice is
    // uniform per wavefront, and both versions meet the same barriers)
    const int full_spans = has_row ? (int)(in / span_cols) : 0;
    // the full spans that are followed by another span request it without asking (no branch around the loads:
    // the requested registers are then the loop's own, and nothing is copied at its end)
    const int full_with_next = nspans > full_spans ? full_spans : full_spans - 1;
    int span = 0;
    for (; span < full_with_next; ++span) work(span, std::true_type(), std::true_type());
    for (; span < full_spans; ++span) work(span, std::true_type(), std::false_type());
    for (; span < nspans; ++span) work(span, std::false_type(), std::false_type());

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
                                bool staged, hipStream_t stream) {
    constexpr int rows = 4 / NW;
    const int64_t groups = ((int64_t)g.total() + rows - 1) / rows;
    const dim3 grid((unsigned)groups), block(kTeamThreads);
    const size_t lds = staged ? (size_t)kStagedCols * sizeof(float) : 0;
    if (staged && apply)
        hipLaunchKernelGGL((ewma_team_kernel<DT, NW, true, true>), grid, block, lds, stream, g, in, hr, c);
    else if (staged)
        hipLaunchKernelGGL((ewma_team_kernel<DT, NW, true, false>), grid, block, lds, stream, g, in, hr, c);
    else if (apply)
        hipLaunchKernelGGL((ewma_team_kernel<DT, NW, false, true>), grid, block, lds, stream, g, in, hr, c);
    else
        hipLaunchKernelGGL((ewma_team_kernel<DT, NW, false, false>), grid, block, lds, stream, g, in, hr, c);
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
    // at least four wavefronts per SIMD (1024 SIMDs) before a row gets a wavefront to itself; rows more than
    // twice as long as the matrix is tall are shared by two wavefronts (measured 4-9 % faster on the wide
    // projections: half the spans a wavefront walks in sequence, for two barriers per span)
    const int64_t out = g.total();
    const Tuning tune = read_tuning();  // measurement overrides
    if (team == 0) team = tune.team;
    if (team == 0) team = out <= 1024 ? 4 : ((out <= 2048 || in > 2 * out) ? 2 : 1);
    const bool st = !tune.select_direct;
    return with_dtype(dt, [&](auto tag) {
        constexpr int DT = decltype(tag)::value;
        switch (team) {
            case 4: return launch_team_t<DT, 4>(g, in, hr, c, apply, st, stream);
            case 2: return launch_team_t<DT, 2>(g, in, hr, c, apply, st, stream);
            default: return launch_team_t<DT, 1>(g, in, hr, c, apply, st, stream);
        }
    });
}

}  // namespace sp

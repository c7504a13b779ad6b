// Wavefront-wide evaluation of the two EWMA recurrences of SwiftPrune's selection
// rule (Sec. 3.2; Algorithm 1 loop body; state-update table of Sec. 3.1) with the
// sum S held fixed:
//     est_q = A est_{q-1} + alpha L_q                 A = 1 - alpha
//     dev_q = B dev_{q-1} + beta |est_q - L_q|        B = 1 - beta
//     est_{-1} = L_0, dev_{-1} = 0
// One wavefront owns a row and walks it in segments of 512 columns, 8 consecutive
// columns per lane.  Per segment:
//   1. lane-local est recurrence from a zero state
//   2. weighted inclusive scan of the lanes' end values with multiplier A^8
//      (row_shr 1/2/4/8, row_bcast 15, row_bcast 31), shifted one lane to make
//      it exclusive, plus A^(8*lane) times the state carried in from the
//      previous segment -> est entering the lane
//   3. est at every element, |est - L|, lane-local dev recurrence, the same
//      scan with B^8 -> dev at every element.
// The scan reorders additions of non-negative terms, so est/dev differ from a
// sequential fp32 walk by a few ulp.
#pragma once

#include "common.hpp"
#include "kernels.hpp"

namespace sp {

constexpr int kScanWaves = 4;  // rows per workgroup (one wavefront each)
constexpr int kPrefetch = 4;   // row segments (16-byte loads per lane) in flight per wavefront

// la and the scaled threshold factor (1-alpha) la beta, from the launch constants or, when the caller left
// la in device memory (calibrated on the same stream), from there; the product is formed in double and
// rounded once, exactly as the host does it
__device__ __forceinline__ float ewma_la(const EwmaConsts& c) { return c.la_dev != nullptr ? c.la_dev[0] : c.la; }
__device__ __forceinline__ float ewma_thr_scale(const EwmaConsts& c) {
    if (c.la_dev == nullptr) return c.thr_scale;
    return (float)((double)c.A_pow[1] * (double)c.la_dev[0] * (double)c.beta);
}

struct ScanLaneConsts {
    float shift;   // m^lane          : weight of the carried-in state at this lane
    float cross15; // m^((lane&15)+1) : weight of the previous 16-lane row's total
    float cross31; // m^((lane&31)+1) : weight of the lower half-wave's total
    float m1, m2, m4, m8;  // m^1, m^2, m^4, m^8 (uniform)
};

// per-lane scan weights from the host's table pw[k] = m^k, k = 0..64 (m = A^8 or B^8), each rounded once
// from double
__device__ __forceinline__ ScanLaneConsts make_lane_consts(const float* pw, int lane) {
    ScanLaneConsts c;
    c.shift = pw[lane];
    c.cross15 = pw[(lane & 15) + 1];
    c.cross31 = pw[(lane & 31) + 1];
    c.m1 = pw[1];
    c.m2 = pw[2];
    c.m4 = pw[4];
    c.m8 = pw[8];
    return c;
}

// Inclusive scan R_j = sum_{i <= j} m^(j-i) v_i over the 64 lanes, then the
// state entering lane j:  R_{j-1} + m^j * carry.
__device__ __forceinline__ float scan_entering(float v, const ScanLaneConsts& c, float carry) {
    float r = v;
    r = fmaf(c.m1, dpp_f<kRowShr1>(r), r);
    r = fmaf(c.m2, dpp_f<kRowShr2>(r), r);
    r = fmaf(c.m4, dpp_f<kRowShr4>(r), r);
    r = fmaf(c.m8, dpp_f<kRowShr8>(r), r);
    r = fmaf(c.cross15, dpp_f<kRowBcast15, 0xA>(r), r);
    r = fmaf(c.cross31, dpp_f<kRowBcast31, 0xC>(r), r);
    return fmaf(c.shift, carry, dpp_f<kWaveShr1>(r));
}

// Walks row `row` of W segment by segment and hands every segment to `body`:
//   body(seg, q0, valid, chunk, L, e_in, d_in, e, d)
// q0 = first column of this lane, valid = how many of its 8 columns exist,
// chunk = the raw weights, L = scores, (e_in, d_in) = state before the lane's
// first column, e[k] / d[k] = state after column q0 + k.
// All 64 lanes must call it together.  scores (nullable) receives L.
template <int DT, bool VEC, class Body>
__device__ __forceinline__ void ewma_walk_row(const void* W, int64_t row, int64_t in, int64_t ldw,
                                              const float* __restrict__ hr, const EwmaConsts& c, int lane,
                                              float* __restrict__ scores, Body&& body) {
    const ScanLaneConsts ce = make_lane_consts(c.A8_pow, lane);
    const ScanLaneConsts cd = make_lane_consts(c.B8_pow, lane);
    const int64_t nseg = (in + 511) >> 9;
    float carry_e = 0.f, carry_d = 0.f;

    // ring of kPrefetch row segments in flight; the factors are fetched one segment ahead
    auto load_chunk = [&](Chunk8<DT>& ch, int64_t seg) {
        const int64_t q0 = (seg << 9) + (int64_t)lane * 8;
        const int valid = (int)min((int64_t)8, max((int64_t)0, in - q0));
        if (VEC) { if (valid) ch.load_vec(W, row * ldw + q0); else ch.zero(); }
        else ch.load_elems(W, row * ldw + q0, valid);
    };
    auto load_factor = [&](Factor8& f, int64_t seg) {
        const int64_t q0 = (seg << 9) + (int64_t)lane * 8;
        const int valid = (int)min((int64_t)8, max((int64_t)0, in - q0));
        if (VEC) { if (valid) f.load_vec(hr, q0); else f.load_elems(hr, q0, 0); }
        else f.load_elems(hr, q0, valid);
    };
    Chunk8<DT> ring[kPrefetch];
#pragma unroll
    for (int j = 0; j < kPrefetch; ++j) load_chunk(ring[j], j);
    Factor8 f;
    load_factor(f, 0);

    for (int64_t base = 0; base < nseg; base += kPrefetch) {
#pragma unroll
        for (int j = 0; j < kPrefetch; ++j) {
            const int64_t seg = base + j;
            if (seg >= nseg) break;  // uniform over the wavefront
            const int64_t q0 = (seg << 9) + (int64_t)lane * 8;
            const int valid = (int)min((int64_t)8, max((int64_t)0, in - q0));

            Chunk8<DT> cur = ring[j];
            load_chunk(ring[j], seg + kPrefetch);  // reads nothing beyond the row end
            Factor8 fn;
            load_factor(fn, seg + 1);

            float L[8];
#pragma unroll
            for (int k = 0; k < 8; ++k) L[k] = score_of(cur.get(k), f.v[k]);
            f = fn;
            if (scores != nullptr && valid) store8(scores + row * in + q0, L, VEC, valid);

            if (seg == 0) carry_e = readlane_f(L[0], 0);  // est starts at the row's first score

            // 1. lane-local est from a zero state
            float e[8];
            e[0] = c.alpha * L[0];
#pragma unroll
            for (int k = 1; k < 8; ++k) e[k] = fmaf(c.A_pow[1], e[k - 1], c.alpha * L[k]);
            // 2. est entering this lane
            const float e_in = scan_entering(e[7], ce, carry_e);
            // 3. est per element, deviations, lane-local dev, dev entering the lane, dev per element
            float d[8];
#pragma unroll
            for (int k = 0; k < 8; ++k) e[k] = fmaf(c.A_pow[k + 1], e_in, e[k]);
            d[0] = c.beta * fabsf(e[0] - L[0]);
#pragma unroll
            for (int k = 1; k < 8; ++k) d[k] = fmaf(c.B_pow[1], d[k - 1], c.beta * fabsf(e[k] - L[k]));
            const float d_in = scan_entering(d[7], cd, carry_d);
#pragma unroll
            for (int k = 0; k < 8; ++k) d[k] = fmaf(c.B_pow[k + 1], d_in, d[k]);

            carry_e = readlane_f(e[7], kWave - 1);
            carry_d = readlane_f(d[7], kWave - 1);

            body(seg, q0, valid, cur, L, e_in, d_in, e, d);
        }
    }
}

}  // namespace sp

// Steps 2+3 of the SwiftPrune layer path, unstructured: contribution score of
// every weight and the per-row EWMA threshold walk (Sec. 3.1 score equation and
// state-update table; Sec. 3.2; Algorithm 1 loop body), evaluated as
// wavefront-wide linear-recurrence scans.
//
// With the sum S held fixed, both state variables are first-order linear
// recurrences with constant decay and the decisions do not feed back:
//     est_q = A est_{q-1} + alpha L_q                 A = 1 - alpha
//     dev_q = B dev_{q-1} + beta |est_q - L_q|        B = 1 - beta
//     prune_q = L_q < est_{q-1} - la dev_{q-1}        est_{-1} = L_0, dev_{-1} = 0
//
// One wavefront owns a row.  It walks the row in segments of 512 columns; each
// lane holds 8 consecutive columns.  Per segment:
//   1. lane-local est recurrence from a zero state          (8 fma)
//   2. weighted inclusive scan of the lanes' end values with multiplier A^8
//      (row_shr 1/2/4/8, row_bcast 15, row_bcast 31), shifted one lane to make
//      it exclusive, plus A^(8*lane) times the state carried in from the
//      previous segment -> true est entering the lane
//   3. true est at every element, |est - L|, lane-local dev recurrence, the
//      same scan with B^8 -> true dev
//   4. thresholds from the state before each element, compare, pack keep bits.
// The scan reorders the additions, so est/dev differ from a sequential fp32
// walk by a few ulp.
#include "common.hpp"
#include "kernels.hpp"

#include <math.h>

namespace sp {

constexpr int kScanWaves = 4;  // rows per workgroup (one wavefront each)
constexpr int kPrefetch = 4;   // row segments (16-byte loads per lane) in flight per wavefront

struct ScanLaneConsts {
    float shift;   // m^lane          : weight of the carried-in state at this lane
    float cross15; // m^((lane&15)+1) : weight of the previous 16-lane row's total
    float cross31; // m^((lane&31)+1) : weight of the lower half-wave's total
    float m1, m2, m4, m8;  // m^1, m^2, m^4, m^8 (uniform)
};

__device__ __forceinline__ float pow_bits(const double* sq, int e) {
    double p = 1.0;
#pragma unroll
    for (int i = 0; i < 7; ++i)
        if ((e >> i) & 1) p *= sq[i];
    return (float)p;
}

__device__ __forceinline__ ScanLaneConsts make_lane_consts(const double* sq, int lane) {
    ScanLaneConsts c;
    c.shift = pow_bits(sq, lane);
    c.cross15 = pow_bits(sq, (lane & 15) + 1);
    c.cross31 = pow_bits(sq, (lane & 31) + 1);
    c.m1 = (float)sq[0];
    c.m2 = (float)sq[1];
    c.m4 = (float)sq[2];
    c.m8 = (float)sq[3];
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

template <int DT, bool VEC>
__global__ __launch_bounds__(kScanWaves* kWave) void ewma_scan_kernel(
    void* __restrict__ W, int64_t out, int64_t in, int64_t ldw, const float* __restrict__ hr,
    const EwmaConsts c, uint32_t* __restrict__ keep_mask, int32_t* __restrict__ row_pruned,
    float* __restrict__ scores, int apply) {
    const int lane = threadIdx.x & (kWave - 1);
    const int wave = threadIdx.x >> 6;
    const int64_t row = (int64_t)blockIdx.x * kScanWaves + wave;
    if (row >= out) return;  // whole wavefront leaves together

    const ScanLaneConsts ce = make_lane_consts(c.A8_sq, lane);
    const ScanLaneConsts cd = make_lane_consts(c.B8_sq, lane);
    const int64_t mask_words = (in + 31) >> 5;
    const int64_t nseg = (in + 511) >> 9;
    const float neg_la = -c.la;

    float carry_e = 0.f, carry_d = 0.f;
    int pruned = 0;

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
            // 3. true est, deviations, lane-local dev
            float d[8];
#pragma unroll
            for (int k = 0; k < 8; ++k) e[k] = fmaf(c.A_pow[k + 1], e_in, e[k]);
            d[0] = c.beta * fabsf(e[0] - L[0]);
#pragma unroll
            for (int k = 1; k < 8; ++k) d[k] = fmaf(c.B_pow[1], d[k - 1], c.beta * fabsf(e[k] - L[k]));
            const float d_in = scan_entering(d[7], cd, carry_d);
#pragma unroll
            for (int k = 0; k < 8; ++k) d[k] = fmaf(c.B_pow[k + 1], d_in, d[k]);
            // 4. decisions from the state before each element
            uint32_t keep = 0u;
            {
                const float thr = fmaf(neg_la, d_in, e_in);
                keep |= (L[0] < thr) ? 0u : 1u;
            }
#pragma unroll
            for (int k = 1; k < 8; ++k) {
                const float thr = fmaf(neg_la, d[k - 1], e[k - 1]);
                keep |= (L[k] < thr) ? 0u : (1u << k);
            }
            keep &= (valid >= 8) ? 0xffu : ((1u << valid) - 1u);
            pruned += valid - __popc(keep);

            carry_e = readlane_f(e[7], kWave - 1);
            carry_d = readlane_f(d[7], kWave - 1);

            const uint32_t word = quad_gather_bytes(keep, lane);
            const int64_t widx = (seg << 4) + (lane >> 2);
            if ((lane & 3) == 0 && widx < mask_words) keep_mask[row * mask_words + widx] = word;

            if (apply && valid) {
                cur.apply(keep);
                if (VEC) cur.store_vec(W, row * ldw + q0);
                else cur.store_elems(W, row * ldw + q0, valid);
            }
        }
    }

    if (row_pruned != nullptr) {
#pragma unroll
        for (int off = 32; off > 0; off >>= 1) pruned += __shfl_xor(pruned, off, kWave);
        if (lane == 0) row_pruned[row] = pruned;
    }
}

EwmaConsts make_ewma_consts(float alpha, float beta, float la) {
    EwmaConsts c;
    c.alpha = alpha;
    c.beta = beta;
    c.la = la;
    const double A = (double)(1.0f - alpha);  // the decay as the fp32 walk sees it
    const double B = (double)(1.0f - beta);
    for (int k = 0; k <= 8; ++k) {
        c.A_pow[k] = (float)pow(A, k);
        c.B_pow[k] = (float)pow(B, k);
    }
    double a = pow(A, 8), b = pow(B, 8);
    for (int i = 0; i < 7; ++i) {
        c.A8_sq[i] = a;
        c.B8_sq[i] = b;
        a *= a;
        b *= b;
    }
    return c;
}

template <int DT, bool VEC>
static hipError_t launch_scan_t(const void* W, int64_t out, int64_t in, int64_t ldw, const float* hr,
                                const EwmaConsts& c, uint32_t* keep_mask, int32_t* row_pruned,
                                float* scores, bool apply, hipStream_t stream) {
    const unsigned grid = (unsigned)((out + kScanWaves - 1) / kScanWaves);
    hipLaunchKernelGGL((ewma_scan_kernel<DT, VEC>), dim3(grid), dim3(kScanWaves * kWave), 0, stream,
                       const_cast<void*>(W), out, in, ldw, hr, c, keep_mask, row_pruned, scores,
                       apply ? 1 : 0);
    return hipGetLastError();
}

hipError_t launch_ewma_scan(const void* W, int64_t out, int64_t in, int64_t ldw, int dt, bool vec,
                            const float* hr, const EwmaConsts& c, uint32_t* keep_mask,
                            int32_t* row_pruned, float* scores, bool apply, hipStream_t stream) {
    if (dt == kBF16)
        return vec ? launch_scan_t<kBF16, true>(W, out, in, ldw, hr, c, keep_mask, row_pruned, scores, apply, stream)
                   : launch_scan_t<kBF16, false>(W, out, in, ldw, hr, c, keep_mask, row_pruned, scores, apply, stream);
    return vec ? launch_scan_t<kF32, true>(W, out, in, ldw, hr, c, keep_mask, row_pruned, scores, apply, stream)
               : launch_scan_t<kF32, false>(W, out, in, ldw, hr, c, keep_mask, row_pruned, scores, apply, stream);
}

}  // namespace sp

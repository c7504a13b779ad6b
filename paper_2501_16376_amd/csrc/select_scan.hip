// Steps 2+3 of the SwiftPrune layer path, unstructured: contribution score of
// every weight and the per-row EWMA threshold decisions (Sec. 3.1 score equation;
// Sec. 3.2; Algorithm 1 loop body), with est/dev from the wavefront scans of
// scan_common.hpp:   prune_q = L_q < est_{q-1} - la dev_{q-1}.
// Keep bits are packed per lane (8 columns), gathered per quad into one 32-bit
// mask word, and the pruned weights can be zeroed in the same pass.
#include "scan_common.hpp"

#include <math.h>

namespace sp {

template <int DT, bool VEC>
__global__ __launch_bounds__(kScanWaves* kWave) void ewma_scan_kernel(
    void* __restrict__ W, int64_t out, int64_t in, int64_t ldw, const float* __restrict__ hr,
    const EwmaConsts c, uint32_t* __restrict__ keep_mask, int32_t* __restrict__ row_pruned,
    float* __restrict__ scores, int apply) {
    const int lane = threadIdx.x & (kWave - 1);
    const int wave = threadIdx.x >> 6;
    const int64_t row = (int64_t)blockIdx.x * kScanWaves + wave;
    if (row >= out) return;  // whole wavefront leaves together

    const int64_t mask_words = (in + 31) >> 5;
    const float neg_la = -c.la;
    int pruned = 0;

    ewma_walk_row<DT, VEC>(W, row, in, ldw, hr, c, lane, scores,
        [&](int64_t seg, int64_t q0, int valid, Chunk8<DT>& cur, const float (&L)[8], float e_in,
            float d_in, const float (&e)[8], const float (&d)[8]) {
            // decisions from the state before each element
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

            const uint32_t word = quad_gather_bytes(keep, lane);
            const int64_t widx = (seg << 4) + (lane >> 2);
            if ((lane & 3) == 0 && widx < mask_words) keep_mask[row * mask_words + widx] = word;

            if (apply && valid) {
                cur.apply(keep);
                if (VEC) cur.store_vec(W, row * ldw + q0);
                else cur.store_elems(W, row * ldw + q0, valid);
            }
        });

    if (row_pruned != nullptr) {
#pragma unroll
        for (int off = 32; off > 0; off >>= 1) pruned += __shfl_xor(pruned, off, kWave);
        if (lane == 0) row_pruned[row] = pruned;
    }
}

// ---------------------------------------------------------------------------
// Fast variant for the 16-byte-vector path (alpha < 1).  Same mathematics as
// above with three changes that cut the VALU work per weight by about half
// (the kernel is VALU-bound, not HBM-bound):
//  * the recurrences run on x = est/alpha and y = dev/beta, which removes the
//    per-element multiplications by alpha and beta:
//        x_k = A x_{k-1} + L_k ,   diff_k = alpha x_k - L_k ,   y_k = B y_{k-1} + |diff_k|
//  * the decision uses the identity  est_k - L_k = A (est_{k-1} - L_k)  (from the est update), i.e.
//        L_k < est_{k-1} - la dev_{k-1}   <=>   diff_k > (A la beta) y_{k-1}
//    so no threshold has to be formed;
//  * every scan step is a single v_fmac_f32 with a DPP source operand (inline
//    assembly; the compiler emits mov + dpp-mov + fmac for the same thing).
//    In-place use is safe: row_shr reads stay inside the 16-lane row being
//    written, and the row_bcast steps read lanes 15/47 and 31, whose rows are
//    masked off for writing.  "s_nop" covers the VALU-write -> DPP-read hazard,
//    which the assembler does not see inside inline assembly.
// ---------------------------------------------------------------------------
#define SP_DPP_FMAC(ctrl, nops)                                                              \
    asm volatile("s_nop " #nops "\n\tv_fmac_f32_dpp %0, %0, %1 " ctrl : "+v"(r) : "v"(m))

__device__ __forceinline__ float scan_entering_fast(float v, const ScanLaneConsts& c, float carry) {
    float r = v;
    { const float m = c.m1; SP_DPP_FMAC("row_shr:1 row_mask:0xf bank_mask:0xf", 4); }
    { const float m = c.m2; SP_DPP_FMAC("row_shr:2 row_mask:0xf bank_mask:0xf", 1); }
    { const float m = c.m4; SP_DPP_FMAC("row_shr:4 row_mask:0xf bank_mask:0xf", 1); }
    { const float m = c.m8; SP_DPP_FMAC("row_shr:8 row_mask:0xf bank_mask:0xf", 1); }
    { const float m = c.cross15; SP_DPP_FMAC("row_bcast:15 row_mask:0xa bank_mask:0xf", 1); }
    { const float m = c.cross31; SP_DPP_FMAC("row_bcast:31 row_mask:0xc bank_mask:0xf", 1); }
    float e = c.shift * carry;  // lane 0 has no left neighbour and keeps this (shift = 1 there)
    asm volatile("s_nop 1\n\tv_add_f32_dpp %0, %1, %0 wave_shr:1 row_mask:0xf bank_mask:0xf"
                 : "+v"(e)
                 : "v"(r));
    return e;
}
#undef SP_DPP_FMAC

template <int DT>
__global__ __launch_bounds__(kScanWaves* kWave) void ewma_scan_fast_kernel(
    void* __restrict__ W, int64_t out, int64_t in, int64_t ldw, const float* __restrict__ hr,
    const EwmaConsts c, uint32_t* __restrict__ keep_mask, int32_t* __restrict__ row_pruned, int apply) {
    const int lane = threadIdx.x & (kWave - 1);
    const int wave = threadIdx.x >> 6;
    const int64_t row = (int64_t)blockIdx.x * kScanWaves + wave;
    if (row >= out) return;  // whole wavefront leaves together

    const ScanLaneConsts ce = make_lane_consts(c.A8_sq, lane);
    const ScanLaneConsts cd = make_lane_consts(c.B8_sq, lane);
    const int64_t mask_words = (in + 31) >> 5;
    const int64_t nseg = (in + 511) >> 9;
    const int64_t nseg_padded = (nseg + kPrefetch - 1) / kPrefetch * kPrefetch;  // empty segments do nothing
    const int64_t row_off = row * ldw;
    const int64_t lane_col = (int64_t)lane * 8;
    const float A = c.A_pow[1], B = c.B_pow[1];

    float carry_x = 0.f, carry_y = 0.f;
    int pruned = 0;

    Chunk8<DT> ring[kPrefetch];
#pragma unroll
    for (int j = 0; j < kPrefetch; ++j) {
        const int64_t q = ((int64_t)j << 9) + lane_col;
        if (q < in) ring[j].load_vec(W, row_off + q); else ring[j].zero();
    }
    Factor8 f;
    if (lane_col < in) f.load_vec(hr, lane_col); else f.load_elems(hr, 0, 0);

    for (int64_t base = 0; base < nseg_padded; base += kPrefetch) {
#pragma unroll
        for (int j = 0; j < kPrefetch; ++j) {
            const int64_t seg = base + j;
            const int64_t q0 = (seg << 9) + lane_col;
            const bool active = q0 < in;

            Chunk8<DT> cur = ring[j];
            if (q0 + ((int64_t)kPrefetch << 9) < in) ring[j].load_vec(W, row_off + q0 + ((int64_t)kPrefetch << 9));
            else ring[j].zero();
            Factor8 fn;
            if (q0 + 512 < in) fn.load_vec(hr, q0 + 512); else fn.load_elems(hr, 0, 0);

            float L[8];
#pragma unroll
            for (int k = 0; k < 8; ++k) L[k] = score_of(cur.get(k), f.v[k]);
            f = fn;
            if (seg == 0) carry_x = readlane_f(L[0], 0) * c.inv_alpha;  // est starts at the row's first score

            float x[8], y[8], diff[8];
            x[0] = L[0];
#pragma unroll
            for (int k = 1; k < 8; ++k) x[k] = fmaf(A, x[k - 1], L[k]);
            const float x_in = scan_entering_fast(x[7], ce, carry_x);
#pragma unroll
            for (int k = 0; k < 8; ++k) x[k] = fmaf(c.A_pow[k + 1], x_in, x[k]);
#pragma unroll
            for (int k = 0; k < 8; ++k) diff[k] = fmaf(c.alpha, x[k], -L[k]);
            y[0] = fabsf(diff[0]);
#pragma unroll
            for (int k = 1; k < 8; ++k) y[k] = fmaf(B, y[k - 1], fabsf(diff[k]));
            const float y_in = scan_entering_fast(y[7], cd, carry_y);
#pragma unroll
            for (int k = 0; k < 8; ++k) y[k] = fmaf(c.B_pow[k + 1], y_in, y[k]);
            carry_x = readlane_f(x[7], kWave - 1);
            carry_y = readlane_f(y[7], kWave - 1);

            bool prune[8];
            // the row's first weight is never pruned (est starts at its score, dev at 0); in scaled
            // form that exact equality is only approximate, so it is stated explicitly
            prune[0] = (diff[0] > c.thr_scale * y_in) && !(seg == 0 && lane == 0);
#pragma unroll
            for (int k = 1; k < 8; ++k) prune[k] = diff[k] > c.thr_scale * y[k - 1];

            uint32_t keep = 0u;
#pragma unroll
            for (int k = 0; k < 8; ++k) keep |= prune[k] ? 0u : (1u << k);
            if (!active) keep = 0u;
            pruned += active ? 8 - __popc(keep) : 0;

            const uint32_t word = quad_gather_bytes(keep, lane);
            const int64_t widx = (seg << 4) + (lane >> 2);
            if ((lane & 3) == 0 && widx < mask_words) keep_mask[row * mask_words + widx] = word;

            if (apply && active) {
                cur.apply_flags(prune);
                cur.store_vec(W, row_off + q0);
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
    c.inv_alpha = (float)(1.0 / (double)alpha);
    c.thr_scale = (float)(A * (double)la * (double)beta);
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
    return with_dtype(dt, [&](auto tag) {
        constexpr int DT = decltype(tag)::value;
        if (vec && scores == nullptr && c.alpha < 1.0f) {
            const unsigned grid = (unsigned)((out + kScanWaves - 1) / kScanWaves);
            hipLaunchKernelGGL(ewma_scan_fast_kernel<DT>, dim3(grid), dim3(kScanWaves * kWave), 0, stream,
                               const_cast<void*>(W), out, in, ldw, hr, c, keep_mask, row_pruned, apply ? 1 : 0);
            return hipGetLastError();
        }
        return vec ? launch_scan_t<DT, true>(W, out, in, ldw, hr, c, keep_mask, row_pruned, scores, apply, stream)
                   : launch_scan_t<DT, false>(W, out, in, ldw, hr, c, keep_mask, row_pruned, scores, apply, stream);
    });
}

}  // namespace sp

// Steps 2+3 of the SwiftPrune layer path, unstructured: contribution score of
// every weight and the per-row EWMA threshold decisions (Sec. 3.1 score equation;
// Sec. 3.2; Algorithm 1 loop body), with est/dev from the wavefront scans of
// scan_common.hpp:   prune_q = L_q < est_{q-1} - la dev_{q-1}.
// Keep bits are packed per lane (8 columns), gathered per quad into one 32-bit
// mask word, and the pruned weights can be zeroed in the same pass.
// This is the general kernel (element-wise layouts, alpha = 1, the scores
// output); aligned inputs take the kernel of select_team.hip.
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
    const float neg_la = -ewma_la(c);
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

EwmaConsts make_ewma_consts(float alpha, float beta, float la) {
    EwmaConsts c;
    c.alpha = alpha;
    c.beta = beta;
    c.la = la;
    c.la_dev = nullptr;
    const double A = (double)(1.0f - alpha);  // the decay as the fp32 walk sees it
    const double B = (double)(1.0f - beta);
    c.inv_alpha = (float)(1.0 / (double)alpha);
    c.thr_scale = (float)(A * (double)la * (double)beta);
    for (int k = 0; k <= 8; ++k) {
        c.A_pow[k] = (float)pow(A, k);
        c.B_pow[k] = (float)pow(B, k);
    }
    const double a = pow(A, 8), b = pow(B, 8);
    double ak = 1.0, bk = 1.0;  // running products in double: 64 roundings of 2^-53 each, far below fp32's
    for (int k = 0; k <= 64; ++k) {
        c.A8_pow[k] = (float)ak;
        c.B8_pow[k] = (float)bk;
        ak *= a;
        bk *= b;
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
        if (vec && scores == nullptr && c.alpha < 1.0f)   // the fast path (select_team.hip)
            return launch_ewma_team(single_matrix(W, out, ldw, keep_mask, row_pruned), in, DT, hr, c, apply, 0, stream);
        return vec ? launch_scan_t<DT, true>(W, out, in, ldw, hr, c, keep_mask, row_pruned, scores, apply, stream)
                   : launch_scan_t<DT, false>(W, out, in, ldw, hr, c, keep_mask, row_pruned, scores, apply, stream);
    });
}

}  // namespace sp

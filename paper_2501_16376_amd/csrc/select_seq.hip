// Steps 2+3 of the SwiftPrune layer path in strict sequential order: one lane
// walks one row element by element, executing the statements of Algorithm 1's
// loop body in the order they are written, every operation rounded on its own
// (no fused multiply-add).  It exists to reproduce a sequential fp32 evaluation
// bit for bit; the scan kernel is the fast path.
#include "common.hpp"
#include "kernels.hpp"

namespace sp {

template <int DT>
__global__ __launch_bounds__(64) void ewma_sequential_kernel(
    void* __restrict__ W, int64_t out, int64_t in, int64_t ldw, const float* __restrict__ hr,
    float alpha, float beta, float la, uint32_t* __restrict__ keep_mask,
    int32_t* __restrict__ row_pruned, float* __restrict__ scores, int apply) {
    const int64_t row = (int64_t)blockIdx.x * 64 + threadIdx.x;
    if (row >= out) return;
    const int64_t mask_words = (in + 31) >> 5;
    const float A = __fsub_rn(1.0f, alpha);
    const float B = __fsub_rn(1.0f, beta);
    float est = 0.f, dev = 0.f;
    int pruned = 0;
    uint32_t word = 0u;
    for (int64_t q = 0; q < in; ++q) {
        const float w = load_scalar<DT>(W, row * ldw + q);
        const float L = score_of(w, hr[q]);
        if (scores != nullptr) scores[row * in + q] = L;
        if (q == 0) est = L;
        const float t = __fmul_rn(la, dev);
        const float thr = __fsub_rn(est, t);
        const bool prune = L < thr;
        const float a_est = __fmul_rn(A, est);
        const float a_new = __fmul_rn(alpha, L);
        est = __fadd_rn(a_est, a_new);
        const float diff = __fsub_rn(est, L);
        const float b_dev = __fmul_rn(B, dev);
        const float b_new = __fmul_rn(beta, fabsf(diff));
        dev = __fadd_rn(b_dev, b_new);
        if (prune) {
            ++pruned;
            if (apply) store_zero<DT>(W, row * ldw + q);
        } else {
            word |= 1u << (q & 31);
        }
        if ((q & 31) == 31 || q == in - 1) {
            keep_mask[row * mask_words + (q >> 5)] = word;
            word = 0u;
        }
    }
    if (row_pruned != nullptr) row_pruned[row] = pruned;
}

hipError_t launch_ewma_sequential(const void* W, int64_t out, int64_t in, int64_t ldw, int dt,
                                  const float* hr, float alpha, float beta, float la,
                                  uint32_t* keep_mask, int32_t* row_pruned, float* scores, bool apply,
                                  hipStream_t stream) {
    const unsigned grid = (unsigned)((out + 63) / 64);
    return with_dtype(dt, [&](auto tag) {
        constexpr int DT = decltype(tag)::value;
        hipLaunchKernelGGL(ewma_sequential_kernel<DT>, dim3(grid), dim3(64), 0, stream, const_cast<void*>(W), out,
                           in, ldw, hr, alpha, beta, la, keep_mask, row_pruned, scores, apply ? 1 : 0);
        return hipGetLastError();
    });
}

}  // namespace sp

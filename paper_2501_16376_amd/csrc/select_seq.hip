// Steps 2+3 of the SwiftPrune layer path in strict sequential order (Sec. 3.2;
// Algorithm 1 loop; state-update table of Sec. 3.1): one lane owns one row and
// consumes it one 32-column mask word at a time.  For every word it first forms
// the 32 scores (loads hoisted ahead of the dependent chain), then threads the
// (est, dev) state through them with every operation rounded on its own - no
// fused multiply-add, no reassociation - so the result is the sequential fp32
// evaluation bit for bit.  It exists for validation; the scan kernel is the
// fast path.
#include "common.hpp"
#include "kernels.hpp"

namespace sp {

// (est, dev) of one row, in fp32, advanced one score at a time.
struct StrictWalk {
    float est, dev;
    float keep_est, keep_dev;  // 1 - alpha, 1 - beta
    float alpha, beta, la;

    __device__ __forceinline__ StrictWalk(float a, float b, float l)
        : est(0.f), dev(0.f), keep_est(__fsub_rn(1.0f, a)), keep_dev(__fsub_rn(1.0f, b)), alpha(a), beta(b), la(l) {}

    // the test uses the state as it stands before the score is absorbed
    __device__ __forceinline__ bool below_threshold(float score) const {
        return score < __fsub_rn(est, __fmul_rn(la, dev));
    }
    // est first, then dev from the new est
    __device__ __forceinline__ void absorb(float score) {
        est = __fadd_rn(__fmul_rn(keep_est, est), __fmul_rn(alpha, score));
        const float gap = fabsf(__fsub_rn(est, score));
        dev = __fadd_rn(__fmul_rn(keep_dev, dev), __fmul_rn(beta, gap));
    }
};

template <int DT>
__global__ __launch_bounds__(64) void ewma_sequential_kernel(
    void* __restrict__ W, int64_t out, int64_t in, int64_t ldw, const float* __restrict__ hr,
    float alpha, float beta, float la, uint32_t* __restrict__ keep_mask,
    int32_t* __restrict__ row_pruned, float* __restrict__ scores, int apply) {
    const int64_t row = (int64_t)blockIdx.x * 64 + threadIdx.x;
    if (row >= out) return;
    const int64_t words = (in + 31) >> 5;
    const int64_t w_row = row * ldw;
    StrictWalk walk(alpha, beta, la);
    int gone = 0;

    for (int64_t word = 0; word < words; ++word) {
        const int64_t q0 = word << 5;
        const int live = (int)min((int64_t)32, in - q0);
        float score[32];
#pragma unroll
        for (int b = 0; b < 32; ++b)
            score[b] = b < live ? score_of(load_scalar<DT>(W, w_row + q0 + b), hr[q0 + b]) : 0.f;
        if (scores != nullptr)
            for (int b = 0; b < live; ++b) scores[row * in + q0 + b] = score[b];
        if (word == 0) walk.est = score[0];  // the walk starts at the row's first score, dev at 0

        uint32_t drop = 0u;
#pragma unroll
        for (int b = 0; b < 32; ++b) {
            if (b < live) {
                drop |= walk.below_threshold(score[b]) ? (1u << b) : 0u;
                walk.absorb(score[b]);
            }
        }
        const uint32_t live_bits = live == 32 ? 0xffffffffu : ((1u << live) - 1u);
        keep_mask[row * words + word] = ~drop & live_bits;
        gone += __popc(drop);
        if (apply)
            for (uint32_t d = drop; d != 0u; d &= d - 1u) store_zero<DT>(W, w_row + q0 + (__ffs(d) - 1));
    }
    if (row_pruned != nullptr) row_pruned[row] = gone;
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

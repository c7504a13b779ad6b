// Diagnostic: the est / dev sequences of the EWMA walk for every weight of every
// row (Sec. 3.2 and the state-update table of Sec. 3.1; the paper's tracking
// figure plots exactly these two sequences against the running mean and mean
// deviation of the scores).  Same wavefront scans as the selection kernel, with
// the state after each element written out instead of being turned into a mask:
//     est[r,q] = A est[r,q-1] + alpha L[r,q],   dev[r,q] = B dev[r,q-1] + beta |est[r,q] - L[r,q]|.
#include "scan_common.hpp"

namespace sp {

template <int DT, bool VEC>
__global__ __launch_bounds__(kScanWaves* kWave) void ewma_trace_kernel(
    const void* __restrict__ W, int64_t out, int64_t in, int64_t ldw, const float* __restrict__ hr,
    const EwmaConsts c, float* __restrict__ est, float* __restrict__ dev) {
    const int lane = threadIdx.x & (kWave - 1);
    const int wave = threadIdx.x >> 6;
    const int64_t row = (int64_t)blockIdx.x * kScanWaves + wave;
    if (row >= out) return;  // whole wavefront leaves together

    ewma_walk_row<DT, VEC>(W, row, in, ldw, hr, c, lane, nullptr,
        [&](int64_t, int64_t q0, int valid, Chunk8<DT>&, const float (&)[8], float, float,
            const float (&e)[8], const float (&d)[8]) {
            if (!valid) return;
            if (est != nullptr) store8(est + row * in + q0, e, VEC, valid);
            if (dev != nullptr) store8(dev + row * in + q0, d, VEC, valid);
        });
}

template <int DT, bool VEC>
static hipError_t launch_trace_t(const void* W, int64_t out, int64_t in, int64_t ldw, const float* hr,
                                 const EwmaConsts& c, float* est, float* dev, hipStream_t stream) {
    const unsigned grid = (unsigned)((out + kScanWaves - 1) / kScanWaves);
    hipLaunchKernelGGL((ewma_trace_kernel<DT, VEC>), dim3(grid), dim3(kScanWaves * kWave), 0, stream, W, out,
                       in, ldw, hr, c, est, dev);
    return hipGetLastError();
}

hipError_t launch_ewma_trace(const void* W, int64_t out, int64_t in, int64_t ldw, int dt, bool vec,
                             const float* hr, const EwmaConsts& c, float* est, float* dev,
                             hipStream_t stream) {
    return with_dtype(dt, [&](auto tag) {
        constexpr int DT = decltype(tag)::value;
        return vec ? launch_trace_t<DT, true>(W, out, in, ldw, hr, c, est, dev, stream)
                   : launch_trace_t<DT, false>(W, out, in, ldw, hr, c, est, dev, stream);
    });
}

}  // namespace sp

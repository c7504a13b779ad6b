// Threshold calibration for the EWMA selection rule.  Sec. 3.1 lists the multiplier
// la for five pruning ratios (50 % to 90 %) and leaves every other ratio to tuning
// la; the appendix reports ratios of 10-40 % without their la.  With S held fixed
// est and dev do not depend on la, so one pass over W can count the pruned
// weights for many candidate la at once, and the pruned fraction is monotone
// non-increasing in la.  The search below brackets the target ratio with 16
// candidates per pass.
#include "scan_common.hpp"

namespace sp {

constexpr int kMaxCandidates = 16;

struct LaCandidates {
    int n;
    float la[kMaxCandidates];
};

__global__ void zero_counts_kernel(unsigned long long* counts, int n) {
    if ((int)threadIdx.x < n) counts[threadIdx.x] = 0ull;
}

// counts[i] += number of weights with L_q < est_{q-1} - la[i] dev_{q-1}, over the rows of this grid
template <int DT, bool VEC>
__global__ __launch_bounds__(kScanWaves* kWave) void ewma_count_kernel(
    const void* __restrict__ W, int64_t out, int64_t in, int64_t ldw, const float* __restrict__ hr,
    const EwmaConsts c, const LaCandidates cand, unsigned long long* __restrict__ counts) {
    const int lane = threadIdx.x & (kWave - 1);
    const int wave = threadIdx.x >> 6;
    const int64_t row = (int64_t)blockIdx.x * kScanWaves + wave;
    if (row >= out) return;

    int cnt[kMaxCandidates];
#pragma unroll
    for (int i = 0; i < kMaxCandidates; ++i) cnt[i] = 0;

    ewma_walk_row<DT, VEC>(W, row, in, ldw, hr, c, lane, nullptr,
        [&](int64_t, int64_t, int valid, Chunk8<DT>&, const float (&L)[8], float e_in, float d_in,
            const float (&e)[8], const float (&d)[8]) {
#pragma unroll
            for (int i = 0; i < kMaxCandidates; ++i) {  // unused slots repeat candidate 0 and are dropped
                const float neg_la = -cand.la[i];
                int n = (0 < valid && L[0] < fmaf(neg_la, d_in, e_in)) ? 1 : 0;
#pragma unroll
                for (int k = 1; k < 8; ++k)
                    n += (k < valid && L[k] < fmaf(neg_la, d[k - 1], e[k - 1])) ? 1 : 0;
                cnt[i] += n;
            }
        });

#pragma unroll
    for (int i = 0; i < kMaxCandidates; ++i) {
        int v = cnt[i];
#pragma unroll
        for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off, kWave);
        if (lane == 0 && i < cand.n) atomicAdd(&counts[i], (unsigned long long)v);  // integer: order-independent
    }
}

hipError_t launch_count_pruned(const void* W, int64_t out, int64_t in, int64_t ldw, int dt, bool vec,
                               const float* hr, const EwmaConsts& c, const float* la, int n_la,
                               unsigned long long* counts, hipStream_t stream) {
    LaCandidates cand;
    cand.n = n_la;
    for (int i = 0; i < kMaxCandidates; ++i) cand.la[i] = i < n_la ? la[i] : la[0];
    hipLaunchKernelGGL(zero_counts_kernel, dim3(1), dim3(64), 0, stream, counts, n_la);
    const unsigned grid = (unsigned)((out + kScanWaves - 1) / kScanWaves);
    const dim3 block(kScanWaves * kWave);
    return with_dtype(dt, [&](auto tag) {
        constexpr int DT = decltype(tag)::value;
        if (vec) hipLaunchKernelGGL((ewma_count_kernel<DT, true>), dim3(grid), block, 0, stream, W, out, in, ldw, hr, c, cand, counts);
        else hipLaunchKernelGGL((ewma_count_kernel<DT, false>), dim3(grid), block, 0, stream, W, out, in, ldw, hr, c, cand, counts);
        return hipGetLastError();
    });
}

// Host-driven bracketing search.  Each pass: 16 equally spaced candidates over [lo, hi], one counting
// launch, one 128-byte copy to the host.  f(la) = pruned fraction is non-increasing in la.
// Returns hipSuccess and *status = 0 (found within tolerance), 1 (closest achievable returned: the
// target lies outside what [la_lo, la_hi] reaches, or the fraction jumps across it).
hipError_t run_calibrate_la(const void* W, int64_t out, int64_t in, int64_t ldw, int dt, bool vec,
                            const float* hr, const EwmaConsts& c, float target, float tolerance,
                            float la_lo, float la_hi, unsigned long long* counts_dev, float* la_out,
                            float* achieved_out, int* status, hipStream_t stream) {
    const double total = (double)out * (double)in;
    float lo = la_lo, hi = la_hi;
    float best_la = lo;
    double best_f = -1.0;
    *status = 1;
    for (int pass = 0; pass < 8; ++pass) {
        float cand[kMaxCandidates];
        for (int i = 0; i < kMaxCandidates; ++i)
            cand[i] = lo + (hi - lo) * (float)i / (float)(kMaxCandidates - 1);
        hipError_t e = launch_count_pruned(W, out, in, ldw, dt, vec, hr, c, cand, kMaxCandidates, counts_dev, stream);
        if (e != hipSuccess) return e;
        unsigned long long host[kMaxCandidates];
        e = hipMemcpyAsync(host, counts_dev, sizeof host, hipMemcpyDeviceToHost, stream);
        if (e != hipSuccess) return e;
        e = hipStreamSynchronize(stream);
        if (e != hipSuccess) return e;
        double f[kMaxCandidates];
        for (int i = 0; i < kMaxCandidates; ++i) {
            f[i] = (double)host[i] / total;
            if (best_f < 0.0 || fabs(f[i] - target) < fabs(best_f - target)) {
                best_f = f[i];
                best_la = cand[i];
            }
        }
        if (fabs(best_f - target) <= tolerance) {
            *status = 0;
            break;
        }
        // bracket: last candidate still at or above the target, first one below it
        int j = -1;
        for (int i = 0; i < kMaxCandidates; ++i)
            if (f[i] >= target) j = i;
        if (j < 0 || j == kMaxCandidates - 1) break;  // target outside the reachable range
        lo = cand[j];
        hi = cand[j + 1];
        if (!(hi - lo > 1e-6f * fmaxf(1.0f, fabsf(lo)))) break;  // a jump in f straddles the target
    }
    *la_out = best_la;
    *achieved_out = (float)best_f;
    return hipSuccess;
}

}  // namespace sp

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

// ---------------------------------------------------------------------------
// The same calibration without the host in the loop.  With S fixed every weight has a critical
// multiplier: it is pruned exactly when la lies below
//     lambda_q = (est_{q-1} - L_q) / dev_{q-1}          (dev_{q-1} > 0)
// (+inf if dev_{q-1} = 0 and L_q < est_{q-1}: pruned whatever la is; -inf if it can never be pruned,
// which includes every row's first weight).  The number pruned at la is #{lambda > la}, so the la that
// prunes k weights is the (k+1)-th largest lambda of the matrix: a radix select over the order-
// preserving bit patterns of the lambdas, 11 + 11 + 10 bits in three passes over W.  Each pass is the
// scan walk with a workgroup-private histogram in LDS that is flushed with integer atomics (order-
// independent, so the result does not depend on scheduling); a one-workgroup kernel between the passes
// picks the bin that holds the wanted rank.  Everything stays on the stream; nothing returns to the host.
// ---------------------------------------------------------------------------
constexpr int kLaBins = 2048;
constexpr int kLaHistGroups = 512;  // workgroups of a histogram pass (they loop over the rows)

struct LaState {            // lives at the start of the workspace
    unsigned int prefix;    // bits of the wanted key fixed so far (right-aligned)
    unsigned int pad;
    unsigned long long rank;   // 1-based rank, counted from the largest, inside the keys that match the prefix
    unsigned long long above;  // keys strictly greater than every key that matches the prefix
};

__device__ __forceinline__ unsigned int la_key(float lambda) {
    if (lambda != lambda) lambda = -INFINITY;  // cannot happen for finite scores; ranks with "never pruned"
    const unsigned int u = __float_as_uint(lambda);
    return (u & 0x80000000u) ? ~u : (u | 0x80000000u);  // ascending in lambda
}
__device__ __forceinline__ float la_from_key(unsigned int key) {
    return __uint_as_float((key & 0x80000000u) ? (key & 0x7fffffffu) : ~key);
}

__global__ void la_init_kernel(LaState* st, unsigned int* hist, unsigned long long rank) {
    for (int i = threadIdx.x; i < kLaBins; i += blockDim.x) hist[i] = 0u;
    if (threadIdx.x == 0) {
        st->prefix = 0u;
        st->pad = 0u;
        st->rank = rank;
        st->above = 0ull;
    }
}

// pass 0 looks at key bits 31..21, pass 1 at 20..10, pass 2 at 9..0
__host__ __device__ inline int la_shift(int pass) { return pass == 0 ? 21 : (pass == 1 ? 10 : 0); }
__host__ __device__ inline int la_bits(int pass) { return pass == 2 ? 10 : 11; }

template <int DT, bool VEC>
__global__ __launch_bounds__(kScanWaves* kWave) void la_hist_kernel(
    const void* __restrict__ W, int64_t out, int64_t in, int64_t ldw, const float* __restrict__ hr,
    const EwmaConsts c, const LaState* __restrict__ st, unsigned int* __restrict__ hist, int pass) {
    __shared__ unsigned int bins[kLaBins];
    for (int i = threadIdx.x; i < kLaBins; i += kScanWaves * kWave) bins[i] = 0u;
    __syncthreads();

    const int lane = threadIdx.x & (kWave - 1);
    const int wave = threadIdx.x >> 6;
    const int shift = la_shift(pass), nbits = la_bits(pass);
    const unsigned int prefix = st->prefix;
    const unsigned int bin_mask = (1u << nbits) - 1u;

    for (int64_t row = (int64_t)blockIdx.x * kScanWaves + wave; row < out; row += (int64_t)gridDim.x * kScanWaves) {
        ewma_walk_row<DT, VEC>(W, row, in, ldw, hr, c, lane, nullptr,
            [&](int64_t seg, int64_t, int valid, Chunk8<DT>&, const float (&L)[8], float e_in, float d_in,
                const float (&e)[8], const float (&d)[8]) {
#pragma unroll
                for (int k = 0; k < 8; ++k) {
                    const float ep = k == 0 ? e_in : e[k - 1];
                    const float dp = k == 0 ? d_in : d[k - 1];
                    const float gap = ep - L[k];
                    float lambda = dp > 0.0f ? gap / dp : (gap > 0.0f ? INFINITY : -INFINITY);
                    if (seg == 0 && lane == 0 && k == 0) lambda = -INFINITY;  // a row's first weight is never pruned
                    const unsigned int key = la_key(lambda);
                    const bool mine = k < valid && (pass == 0 || (key >> (shift + nbits)) == prefix);
                    if (mine) atomicAdd(&bins[(key >> shift) & bin_mask], 1u);
                }
            });
    }
    __syncthreads();
    for (int i = threadIdx.x; i < kLaBins; i += kScanWaves * kWave)
        if (bins[i] != 0u) atomicAdd(&hist[i], bins[i]);
}

// One workgroup: walks the bins from the top, finds the one that holds the wanted rank, narrows the state,
// clears the histogram for the next pass.  After the last pass it writes la, the number of weights with a
// larger lambda (those la prunes) and a status (0 = exact rank found, 1 = the rank falls among weights that
// are pruned for every la or for none: la is clamped to the nearest finite lambda's side).
__global__ __launch_bounds__(256) void la_pick_kernel(LaState* st, unsigned int* hist, int pass, float* la_out,
                                                      unsigned long long* pruned_out, int* status_out) {
    __shared__ unsigned long long part[256];
    __shared__ int chosen;
    const int nb = 1 << la_bits(pass);
    const int per = nb / 256;  // bins per thread (8 or 4), thread 0 owns the highest bins
    // thread t owns bins [nb - (t+1)*per, nb - t*per)
    unsigned long long mine = 0ull;
    for (int j = 0; j < per; ++j) mine += hist[nb - 1 - (threadIdx.x * per + j)];
    part[threadIdx.x] = mine;
    __syncthreads();
    if (threadIdx.x == 0) {
        unsigned long long rank = st->rank, acc = 0ull;
        int t = 0;
        while (t < 255 && acc + part[t] < rank) acc += part[t++];
        int b = nb - 1 - t * per;
        const int b_last = nb - (t + 1) * per;
        while (b > b_last && acc + hist[b] < rank) acc += hist[b--];
        chosen = b;
        st->above += acc;
        st->rank = rank - acc;           // rank inside the chosen bin (may exceed its count if the rank is out of range)
        st->prefix = (st->prefix << la_bits(pass)) | (unsigned int)b;
        if (pass == 2) {
            float la = la_from_key(st->prefix);
            int status = 0;
            // ranks that land on +inf (pruned for every la) or -inf (never pruned) have no finite answer
            if (!(la < INFINITY)) { la = 3.0e38f; status = 1; }
            if (!(la > -INFINITY)) { la = -3.0e38f; status = 1; }
            la_out[0] = la;
            if (pruned_out != nullptr) pruned_out[0] = st->above;
            if (status_out != nullptr) status_out[0] = status;
        }
    }
    __syncthreads();
    for (int i = threadIdx.x; i < kLaBins; i += 256) hist[i] = 0u;
    (void)chosen;
}

size_t la_workspace_bytes() { return 256 + kLaBins * sizeof(unsigned int); }

hipError_t launch_calibrate_la_device(const void* W, int64_t out, int64_t in, int64_t ldw, int dt, bool vec,
                                      const float* hr, const EwmaConsts& c, unsigned long long target_count,
                                      void* workspace, float* la_dev, unsigned long long* pruned_dev,
                                      int* status_dev, hipStream_t stream) {
    LaState* st = static_cast<LaState*>(workspace);
    unsigned int* hist = reinterpret_cast<unsigned int*>(static_cast<char*>(workspace) + 256);
    // la prunes the weights with lambda > la: the (target_count + 1)-th largest lambda prunes target_count
    hipLaunchKernelGGL(la_init_kernel, dim3(1), dim3(256), 0, stream, st, hist, target_count + 1ull);
    int64_t groups = (out + kScanWaves - 1) / kScanWaves;
    if (groups > kLaHistGroups) groups = kLaHistGroups;
    const dim3 grid((unsigned)groups), block(kScanWaves * kWave);
    for (int pass = 0; pass < 3; ++pass) {
        const hipError_t e = with_dtype(dt, [&](auto tag) {
            constexpr int DT = decltype(tag)::value;
            if (vec) hipLaunchKernelGGL((la_hist_kernel<DT, true>), grid, block, 0, stream, W, out, in, ldw, hr, c, st, hist, pass);
            else hipLaunchKernelGGL((la_hist_kernel<DT, false>), grid, block, 0, stream, W, out, in, ldw, hr, c, st, hist, pass);
            return hipGetLastError();
        });
        if (e != hipSuccess) return e;
        hipLaunchKernelGGL(la_pick_kernel, dim3(1), dim3(256), 0, stream, st, hist, pass, la_dev, pruned_dev, status_dev);
        const hipError_t e2 = hipGetLastError();
        if (e2 != hipSuccess) return e2;
    }
    return hipSuccess;
}

}  // namespace sp

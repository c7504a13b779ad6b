// Exact per-row selection of the k smallest scores - the order-and-drop-the-
// lowest rule of Sec. 3.1 that the EWMA walk replaces - as a
// comparator on the GPU, without a sort: one workgroup per row runs a 4-pass
// radix select (8 bits per pass, LDS histogram) on the order-preserving bit
// pattern of the non-negative fp32 scores, then prunes everything below the
// k-th value and the first `remaining` entries equal to it in index order
// (workgroup-wide exclusive count).  Scores are recomputed from W in every pass
// (a row stays in cache), so no per-row buffer is needed.
#include "common.hpp"
#include "kernels.hpp"

namespace sp {

constexpr int kTopkThreads = 256;

template <int DT>
__device__ __forceinline__ uint32_t score_key(const void* W, int64_t idx, float factor) {
    const float L = score_of(load_scalar<DT>(W, idx), factor);
    // scores are >= +0 (or NaN): the bit pattern orders them.  Every NaN gets the one key above +inf, so
    // that NaNs rank after all numbers and among themselves in index order, whatever their payload
    return L != L ? 0x7fffffffu : (__float_as_uint(L) & 0x7fffffffu);
}

// exclusive prefix sum of one int per thread over 256 threads; also returns the total
__device__ __forceinline__ int block_excl_scan_256(int v, int* total, int* lds /*[5]*/) {
    const int lane = threadIdx.x & (kWave - 1);
    const int wave = threadIdx.x >> 6;
    int incl = v;
#pragma unroll
    for (int off = 1; off < kWave; off <<= 1) {
        const int t = __shfl_up(incl, off, kWave);
        if (lane >= off) incl += t;
    }
    if (lane == kWave - 1) lds[wave] = incl;
    __syncthreads();
    int base = 0;
#pragma unroll
    for (int w = 0; w < 4; ++w)
        if (w < wave) base += lds[w];
    *total = lds[0] + lds[1] + lds[2] + lds[3];
    __syncthreads();
    return base + incl - v;
}

// grid = out, block = 256.  Thread t owns the columns [t*cpt, (t+1)*cpt), cpt a multiple of 32, so it
// owns whole mask words and index order is thread order.
template <int DT>
__global__ __launch_bounds__(kTopkThreads) void topk_select_kernel(
    void* __restrict__ W, int64_t in, int64_t ldw, const float* __restrict__ hr,
    const int32_t* __restrict__ k_per_row, int64_t k_uniform, uint32_t* __restrict__ keep_mask,
    int cpt, int apply) {
    __shared__ int hist[256];
    __shared__ int scan_lds[5];
    __shared__ uint32_t sel_prefix;
    __shared__ int sel_remaining;

    const int64_t row = blockIdx.x;
    const int64_t mask_words = (in + 31) >> 5;
    const int64_t c0 = (int64_t)threadIdx.x * cpt;
    const int64_t c1 = min(in, c0 + cpt);
    const int64_t base = row * ldw;

    int64_t k = k_per_row != nullptr ? (int64_t)k_per_row[row] : k_uniform;
    k = max((int64_t)0, min(k, in));

    uint32_t T = 0u;       // key of the k-th smallest score
    int remaining = 0;     // how many entries equal to T are pruned
    if (k > 0) {
        uint32_t prefix = 0u;
        int rem = (int)k;
        for (int shift = 24; shift >= 0; shift -= 8) {
            hist[threadIdx.x] = 0;
            __syncthreads();
            const uint32_t hi_mask = (shift == 24) ? 0u : (0xffffffffu << (shift + 8));
            for (int64_t q = c0; q < c1; ++q) {
                const uint32_t key = score_key<DT>(W, base + q, hr[q]);
                if ((key & hi_mask) == prefix) atomicAdd(&hist[(key >> shift) & 255u], 1);
            }
            __syncthreads();
            int total;
            const int mine = hist[threadIdx.x];
            const int before = block_excl_scan_256(mine, &total, scan_lds);
            if (before < rem && rem <= before + mine) {  // exactly one digit satisfies this
                sel_prefix = prefix | ((uint32_t)threadIdx.x << shift);
                sel_remaining = rem - before;
            }
            __syncthreads();
            prefix = sel_prefix;
            rem = sel_remaining;
            __syncthreads();
        }
        T = prefix;
        remaining = rem;
    }

    // rank of this thread's first tie among all ties of the row, in index order
    int ties = 0;
    if (k > 0)
        for (int64_t q = c0; q < c1; ++q) ties += (score_key<DT>(W, base + q, hr[q]) == T) ? 1 : 0;
    int total_ties;
    int tie_rank = block_excl_scan_256(ties, &total_ties, scan_lds);

    for (int64_t w0 = c0; w0 < c1; w0 += 32) {
        uint32_t word = 0u;
        const int64_t w1 = min(c1, w0 + 32);
        for (int64_t q = w0; q < w1; ++q) {
            bool prune = false;
            if (k > 0) {
                const uint32_t key = score_key<DT>(W, base + q, hr[q]);
                if (key < T) prune = true;
                else if (key == T) prune = (tie_rank++ < remaining);
            }
            if (!prune) word |= 1u << (q & 31);
            else if (apply) store_zero<DT>(W, base + q);
        }
        keep_mask[row * mask_words + (w0 >> 5)] = word;
    }
}

hipError_t launch_topk_select(const void* W, int64_t out, int64_t in, int64_t ldw, int dt,
                              const float* hr, const int32_t* k_per_row, int64_t k_uniform,
                              uint32_t* keep_mask, bool apply, hipStream_t stream) {
    int64_t cpt = (in + kTopkThreads - 1) / kTopkThreads;
    cpt = (cpt + 31) / 32 * 32;
    void* Wm = const_cast<void*>(W);
    return with_dtype(dt, [&](auto tag) {
        constexpr int DT = decltype(tag)::value;
        hipLaunchKernelGGL(topk_select_kernel<DT>, dim3((unsigned)out), dim3(kTopkThreads), 0, stream, Wm, in, ldw,
                           hr, k_per_row, k_uniform, keep_mask, (int)cpt, apply ? 1 : 0);
        return hipGetLastError();
    });
}

}  // namespace sp

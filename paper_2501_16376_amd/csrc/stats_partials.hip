// Step 1 of the SwiftPrune layer path when the producer of X has already added up the squares of its own
// pieces of the tokens (Algorithm 1, first statement: x_q^2 is a sum over tokens, so it can be cut in pieces
// anywhere; Sec. 3.1: S is the sum of the x_q^2, the factor 1/2 / (1 - x_q^2/S) the score's denominator).
// The caller hands over P[p*ld + q] = sum over the tokens of piece p of X[t,q]^2 (fp32); this file adds the
// pieces per channel in fp64, forms S from the channel sums in fp64, and writes xsq, S and the factors.
// Nothing of X is read: a GEMM or activation kernel that writes X can emit P from its epilogue, and the
// 2 bytes per activation that swiftprune_layer_stats streams are never fetched again.
#include "common.hpp"
#include "kernels.hpp"

namespace sp {

constexpr int kPieceThreads = 256;  // 64 channels x 4 interleaved groups of pieces
constexpr int kTotalThreads = 1024;

// grid = ceil(in / 64), block = 256: thread (c = tid & 63, g = tid >> 6) adds the pieces p = g, g+4, ... of
// channel blockIdx.x*64 + c in fp64; the four groups are added in order through LDS.
__global__ __launch_bounds__(kPieceThreads) void pieces_sum_kernel(const float* __restrict__ P, int64_t parts,
                                                                  int64_t ld, int64_t in, float* __restrict__ xsq,
                                                                  int accumulate) {
    __shared__ double group[4][64];
    const int c = threadIdx.x & 63;
    const int g = threadIdx.x >> 6;
    const int64_t q = (int64_t)blockIdx.x * 64 + c;
    double s = 0.0;
    if (q < in) {
        const float* col = P + q;
        int64_t p = g;
        for (; p + 28 < parts; p += 32) {  // eight loads in flight
            float a[8];
#pragma unroll
            for (int j = 0; j < 8; ++j) a[j] = col[(p + 4 * j) * ld];
#pragma unroll
            for (int j = 0; j < 8; ++j) s += (double)a[j];
        }
        for (; p < parts; p += 4) s += (double)col[p * ld];
    }
    group[g][c] = s;
    __syncthreads();
    if (g == 0 && q < in) {
        double t = ((group[0][c] + group[1][c]) + group[2][c]) + group[3][c];
        if (accumulate) t += (double)xsq[q];
        xsq[q] = (float)t;
    }
}

// grid = 1, block = 1024: S = sum of xsq in fp64 (each thread its strided share in ascending order, then the
// wavefronts' and the block's totals in a fixed order), then the factor of every channel.
__global__ __launch_bounds__(kTotalThreads) void channel_total_kernel(const float* __restrict__ xsq, int64_t in,
                                                                      float* __restrict__ S_out,
                                                                      float* __restrict__ hr, int finalize) {
    __shared__ double waves[kTotalThreads / kWave];
    __shared__ float S_all;
    double s = 0.0;
    for (int64_t q = threadIdx.x; q < in; q += kTotalThreads) s += (double)xsq[q];
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) s += __shfl_down(s, off, kWave);
    if ((threadIdx.x & (kWave - 1)) == 0) waves[threadIdx.x >> 6] = s;
    __syncthreads();
    if (threadIdx.x == 0) {
        double t = 0.0;
        for (int w = 0; w < kTotalThreads / kWave; ++w) t += waves[w];
        S_all = (float)t;
        S_out[0] = (float)t;
    }
    __syncthreads();
    if (!finalize) return;
    const float S = S_all;
    for (int64_t q = threadIdx.x; q < in; q += kTotalThreads) {
        // 1/2 / (1 - xsq/S): three fp32 roundings; S == 0 gives 1/2, a denominator that is not positive
        // becomes FLT_EPSILON (the conventions of swiftprune_layer_stats)
        float f = 0.5f;
        if (S != 0.0f) {
            const float rho = __fdiv_rn(xsq[q], S);
            float den = __fsub_rn(1.0f, rho);
            if (!(den > 0.0f)) den = 1.1920928955078125e-07f;
            f = __fdiv_rn(0.5f, den);
        }
        hr[q] = f;
    }
}

hipError_t launch_stats_from_pieces(const float* P, int64_t parts, int64_t in, int64_t ld, float* xsq, float* S,
                                    float* hr, int accumulate, int finalize, hipStream_t stream) {
    const int64_t groups = (in + 63) / 64;
    hipLaunchKernelGGL(pieces_sum_kernel, dim3((unsigned)groups), dim3(kPieceThreads), 0, stream, P, parts, ld, in,
                       xsq, accumulate);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(channel_total_kernel, dim3(1), dim3(kTotalThreads), 0, stream, xsq, in, S, hr, finalize);
    return hipGetLastError();
}

}  // namespace sp

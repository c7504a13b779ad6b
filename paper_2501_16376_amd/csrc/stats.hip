// Step 1 of the SwiftPrune layer path: per-input-channel sums of squares of the
// calibration activations, their total S, and the per-channel score factor
// (Algorithm 1, first statement; Sec. 3.1, definition of S and the score equation).
//
// X[tokens, in] is streamed once.  A workgroup of kStatsWaves wavefronts owns a
// strip of 64 sixteen-byte units (512 bf16 / 256 fp32 columns) and a range of
// tokens; its wavefronts take interleaved rows, every lane keeps fp32 running
// sums for the columns of its unit, and the wavefronts' sums are combined
// through LDS into one partial row per workgroup.  A second small kernel adds
// the partial rows in fp64 in a fixed order, and its last workgroup to finish
// derives S and the factor.  No floating-point atomics: results are
// independent of scheduling.
#include "common.hpp"
#include "kernels.hpp"

namespace sp {

constexpr int kStatsWaves = 16;          // wavefronts per workgroup (1024 threads)
constexpr int kStatsUnroll = 4;          // rows in flight per wavefront and iteration
constexpr int kStatsTargetGroups = 512;  // 2 workgroups on each of the 256 compute units

template <int DT, int EPU>
struct XUnit;

template <>
struct XUnit<kBF16, 8> {
    uint4 r;
    __device__ __forceinline__ void load(const void* X, int64_t elem) {
        r = *reinterpret_cast<const uint4*>(static_cast<const uint16_t*>(X) + elem);
    }
    __device__ __forceinline__ void zero() { r = make_uint4(0, 0, 0, 0); }
    __device__ __forceinline__ void sq_add(float* a) const {
        float v;
        v = bf16lo(r.x); a[0] = fmaf(v, v, a[0]);
        v = bf16hi(r.x); a[1] = fmaf(v, v, a[1]);
        v = bf16lo(r.y); a[2] = fmaf(v, v, a[2]);
        v = bf16hi(r.y); a[3] = fmaf(v, v, a[3]);
        v = bf16lo(r.z); a[4] = fmaf(v, v, a[4]);
        v = bf16hi(r.z); a[5] = fmaf(v, v, a[5]);
        v = bf16lo(r.w); a[6] = fmaf(v, v, a[6]);
        v = bf16hi(r.w); a[7] = fmaf(v, v, a[7]);
    }
};

template <>
struct XUnit<kF32, 4> {
    float4 r;
    __device__ __forceinline__ void load(const void* X, int64_t elem) {
        r = *reinterpret_cast<const float4*>(static_cast<const float*>(X) + elem);
    }
    __device__ __forceinline__ void zero() { r = make_float4(0.f, 0.f, 0.f, 0.f); }
    __device__ __forceinline__ void sq_add(float* a) const {
        a[0] = fmaf(r.x, r.x, a[0]);
        a[1] = fmaf(r.y, r.y, a[1]);
        a[2] = fmaf(r.z, r.z, a[2]);
        a[3] = fmaf(r.w, r.w, a[3]);
    }
};

template <>
struct XUnit<kBF16, 1> {
    float r;
    __device__ __forceinline__ void load(const void* X, int64_t elem) {
        r = __uint_as_float((uint32_t)static_cast<const uint16_t*>(X)[elem] << 16);
    }
    __device__ __forceinline__ void zero() { r = 0.f; }
    __device__ __forceinline__ void sq_add(float* a) const { a[0] = fmaf(r, r, a[0]); }
};

template <>
struct XUnit<kF32, 1> {
    float r;
    __device__ __forceinline__ void load(const void* X, int64_t elem) {
        r = static_cast<const float*>(X)[elem];
    }
    __device__ __forceinline__ void zero() { r = 0.f; }
    __device__ __forceinline__ void sq_add(float* a) const { a[0] = fmaf(r, r, a[0]); }
};

// grid = (nstrips, splits), block = kStatsWaves * 64.
// partials[(strip * splits + split) * 64*EPU + lane*EPU + k] = sum over the
// workgroup's token range of X[t, (strip*64 + lane)*EPU + k]^2.
template <int DT, int EPU>
__global__ __launch_bounds__(kStatsWaves* kWave) void stats_partial_kernel(
    const void* __restrict__ X, int64_t tokens, int64_t units, int64_t ldx, int64_t rows_per_split,
    float* __restrict__ partials, unsigned int* __restrict__ counters) {
    __shared__ float red[kStatsWaves][kWave * EPU];

    const int lane = threadIdx.x & (kWave - 1);
    const int wave = threadIdx.x >> 6;
    const int strip = blockIdx.x;
    const int split = blockIdx.y;
    const int splits = gridDim.y;

    if (strip == 0 && split == 0 && threadIdx.x == 0) counters[0] = 0u;  // ticket of the combine kernel

    const int64_t u = (int64_t)strip * kWave + lane;
    const bool active = u < units;
    const int64_t col = u * EPU;
    const int64_t r_begin = (int64_t)split * rows_per_split;
    const int64_t r_end = min(tokens, r_begin + rows_per_split);

    float acc0[EPU], acc1[EPU];
#pragma unroll
    for (int k = 0; k < EPU; ++k) acc0[k] = acc1[k] = 0.f;

    if (active) {
        int64_t r = r_begin + wave;
        constexpr int64_t kStep = (int64_t)kStatsWaves * kStatsUnroll;
        // full batches: kStatsUnroll independent loads in flight, two accumulator sets
        for (; r + (kStatsUnroll - 1) * kStatsWaves < r_end; r += kStep) {
            XUnit<DT, EPU> v[kStatsUnroll];
#pragma unroll
            for (int j = 0; j < kStatsUnroll; ++j) v[j].load(X, (r + (int64_t)j * kStatsWaves) * ldx + col);
#pragma unroll
            for (int j = 0; j < kStatsUnroll; ++j) v[j].sq_add((j & 1) ? acc1 : acc0);
        }
        for (; r < r_end; r += kStatsWaves) {
            XUnit<DT, EPU> v;
            v.load(X, r * ldx + col);
            v.sq_add(acc0);
        }
    }

#pragma unroll
    for (int k = 0; k < EPU; ++k) red[wave][lane * EPU + k] = acc0[k] + acc1[k];
    __syncthreads();

    for (int c = threadIdx.x; c < kWave * EPU; c += kStatsWaves * kWave) {
        float s = 0.f;
#pragma unroll
        for (int w = 0; w < kStatsWaves; ++w) s += red[w][c];
        partials[((int64_t)strip * splits + split) * (kWave * EPU) + c] = s;
    }
}

// grid = ceil(in / 64), block = 256: thread (c = tid & 63, g = tid >> 6) adds the
// partial rows s = g, g+4, ... of column blockIdx.x*64 + c in fp64; the four
// groups are then added in order.  The last workgroup to finish computes S and hr.
__global__ __launch_bounds__(256) void stats_combine_kernel(
    const float* __restrict__ partials, int splits, int cols_per_strip, int64_t in,
    float* xsq, int accumulate, int finalize, float* __restrict__ S_out, float* __restrict__ hr,
    unsigned int* __restrict__ counters) {
    __shared__ double part[4][64];
    __shared__ double red[256];
    __shared__ unsigned int ticket;

    const int c = threadIdx.x & 63;
    const int g = threadIdx.x >> 6;
    const int64_t col = (int64_t)blockIdx.x * 64 + c;

    double s = 0.0;
    if (col < in) {
        const int64_t strip = col / cols_per_strip;
        const int64_t within = col - strip * cols_per_strip;
        const float* p = partials + strip * splits * (int64_t)cols_per_strip + within;
        for (int sp = g; sp < splits; sp += 4) s += (double)p[(int64_t)sp * cols_per_strip];
    }
    part[g][c] = s;
    __syncthreads();
    if (g == 0 && col < in) {
        double t = ((part[0][c] + part[1][c]) + part[2][c]) + part[3][c];
        if (accumulate) t += (double)xsq[col];
        xsq[col] = (float)t;
    }
    if (!finalize) return;

    // last-workgroup-done: publish this workgroup's xsq, take a ticket
    __threadfence();
    __syncthreads();
    if (threadIdx.x == 0) ticket = atomicAdd(&counters[0], 1u);
    __syncthreads();
    if (ticket != gridDim.x - 1) return;
    __threadfence();

    const volatile float* xs = xsq;  // written by other workgroups of this launch: bypass stale caches
    double t = 0.0;
    for (int64_t q = threadIdx.x; q < in; q += 256) t += (double)xs[q];
    red[threadIdx.x] = t;
    __syncthreads();
    for (int w = 128; w > 0; w >>= 1) {
        if ((int)threadIdx.x < w) red[threadIdx.x] += red[threadIdx.x + w];
        __syncthreads();
    }
    const float S = (float)red[0];
    if (threadIdx.x == 0) S_out[0] = S;
    for (int64_t q = threadIdx.x; q < in; q += 256) {
        float f = 0.5f;
        if (S != 0.0f) {
            const float rho = __fdiv_rn(xs[q], S);
            float den = __fsub_rn(1.0f, rho);
            if (!(den > 0.0f)) den = 1.1920928955078125e-07f;  // FLT_EPSILON
            f = __fdiv_rn(0.5f, den);
        }
        hr[q] = f;
    }
}

StatsPlan make_stats_plan(int64_t tokens, int64_t in, int dt, bool vec) {
    StatsPlan p;
    p.epu = vec ? (dt == kBF16 ? 8 : 4) : 1;
    p.units = (in + p.epu - 1) / p.epu;
    p.nstrips = (int)((p.units + kWave - 1) / kWave);
    // one round of workgroups: as many token splits as keep the total at or below the target,
    // but no split shorter than one batch of rows per wavefront
    int64_t splits = kStatsTargetGroups / p.nstrips;
    const int64_t min_rows = (int64_t)kStatsWaves * kStatsUnroll;
    const int64_t max_splits = (tokens + min_rows - 1) / min_rows;
    if (splits > max_splits) splits = max_splits;
    if (splits < 1) splits = 1;
    p.splits = (int)splits;
    p.rows_per_split = (tokens + splits - 1) / splits;
    p.partial_floats = (size_t)p.nstrips * (size_t)p.splits * (size_t)(kWave * p.epu);
    return p;
}

template <int DT, int EPU>
static hipError_t launch_partial(const void* X, int64_t tokens, int64_t ldx, const StatsPlan& p,
                                 float* partials, unsigned int* counters, hipStream_t stream) {
    dim3 grid((unsigned)p.nstrips, (unsigned)p.splits);
    hipLaunchKernelGGL((stats_partial_kernel<DT, EPU>), grid, dim3(kStatsWaves * kWave), 0, stream, X,
                       tokens, p.units, ldx, p.rows_per_split, partials, counters);
    return hipGetLastError();
}

hipError_t launch_layer_stats(const void* X, int64_t tokens, int64_t in, int64_t ldx, int dt, bool vec,
                              float* xsq, float* S, float* hr, int accumulate, int finalize,
                              void* workspace, hipStream_t stream) {
    const StatsPlan p = make_stats_plan(tokens, in, dt, vec);
    unsigned int* counters = static_cast<unsigned int*>(workspace);
    float* partials = reinterpret_cast<float*>(static_cast<char*>(workspace) + kStatsHeaderBytes);
    hipError_t e;
    if (dt == kBF16)
        e = vec ? launch_partial<kBF16, 8>(X, tokens, ldx, p, partials, counters, stream)
                : launch_partial<kBF16, 1>(X, tokens, ldx, p, partials, counters, stream);
    else
        e = vec ? launch_partial<kF32, 4>(X, tokens, ldx, p, partials, counters, stream)
                : launch_partial<kF32, 1>(X, tokens, ldx, p, partials, counters, stream);
    if (e != hipSuccess) return e;
    const unsigned nblk = (unsigned)((in + 63) / 64);
    hipLaunchKernelGGL(stats_combine_kernel, dim3(nblk), dim3(256), 0, stream, partials, p.splits,
                       kWave * p.epu, in, xsq, accumulate, finalize, S, hr, counters);
    return hipGetLastError();
}

}  // namespace sp

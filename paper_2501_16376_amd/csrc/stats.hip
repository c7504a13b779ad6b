// Step 1 of the SwiftPrune layer path: per-input-channel sums of squares of the
// calibration activations, their total S, and the per-channel score factor
// (Algorithm 1, first statement; Sec. 3.1, definition of S and the score equation).
//
// X[tokens, in] is streamed exactly once with non-temporal 16-byte loads.  The
// columns are cut into strips of at most 256 sixteen-byte units (one unit per
// lane of a 256-thread workgroup: 2048 bf16 or 1024 fp32 columns, contiguous in
// every row) and the tokens into ranges; strips x ranges is chosen to be about
// one workgroup per compute unit, which measured fastest on MI355X (more
// resident workgroups lower the achieved HBM rate).  Every lane keeps fp32
// running sums for the columns of its unit, eight rows in flight, four
// independent accumulator sets so no serial fp32 chain exceeds a quarter of the
// range.  Each workgroup writes one partial row; a second small kernel adds the
// partial rows in fp64 in a fixed order (LDS-staged), reduces S, and its last
// workgroup to finish derives the factor for every channel.  No floating-point
// atomics: results do not depend on scheduling.
#include "common.hpp"
#include "kernels.hpp"

namespace sp {

constexpr int kStatsThreads = 256;       // one wide strip per workgroup, 4 wavefronts
constexpr int kStatsUnroll = 8;          // rows (independent 16-byte loads) in flight per lane
constexpr int kStatsSets = 4;            // independent accumulator sets per column
constexpr int kStatsTargetGroups = 256;  // one workgroup per compute unit
constexpr int kCombineThreads = 1024;    // 64 columns x 16 groups of partial rows
constexpr int kCombineGroups = kCombineThreads / 64;

template <int DT, int EPU>
struct XUnit;

template <>
struct XUnit<kBF16, 8> {
    u32x4 r;
    __device__ __forceinline__ void load(const void* X, int64_t elem) {
        r = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(static_cast<const uint16_t*>(X) + elem));
    }
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
    f32x4 r;
    __device__ __forceinline__ void load(const void* X, int64_t elem) {
        r = __builtin_nontemporal_load(reinterpret_cast<const f32x4*>(static_cast<const float*>(X) + elem));
    }
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
        r = __uint_as_float((uint32_t)__builtin_nontemporal_load(static_cast<const uint16_t*>(X) + elem) << 16);
    }
    __device__ __forceinline__ void sq_add(float* a) const { a[0] = fmaf(r, r, a[0]); }
};

template <>
struct XUnit<kF32, 1> {
    float r;
    __device__ __forceinline__ void load(const void* X, int64_t elem) {
        r = __builtin_nontemporal_load(static_cast<const float*>(X) + elem);
    }
    __device__ __forceinline__ void sq_add(float* a) const { a[0] = fmaf(r, r, a[0]); }
};

// grid = (nstrips, splits), block = 256.
// partials[split * in_pad + u*EPU + k] = sum over the workgroup's token range of X[t, u*EPU + k]^2
// for the units u of its strip (in_pad = units * EPU).
template <int DT, int EPU>
__global__ __launch_bounds__(kStatsThreads) void stats_partial_kernel(
    const void* __restrict__ X, int64_t tokens, int64_t units, int strip_units, int64_t ldx,
    int64_t rows_per_split, float* __restrict__ partials, unsigned int* __restrict__ counters) {
    const int strip = blockIdx.x;
    const int split = blockIdx.y;
    if (strip == 0 && split == 0 && threadIdx.x == 0) counters[0] = 0u;  // ticket of the combine kernel

    const int64_t u = (int64_t)strip * strip_units + threadIdx.x;
    if ((int)threadIdx.x >= strip_units || u >= units) return;
    const int64_t col = u * EPU;
    const int64_t r_begin = (int64_t)split * rows_per_split;
    const int64_t r_end = min(tokens, r_begin + rows_per_split);

    float acc[kStatsSets][EPU];
#pragma unroll
    for (int s = 0; s < kStatsSets; ++s)
#pragma unroll
        for (int k = 0; k < EPU; ++k) acc[s][k] = 0.f;

    int64_t r = r_begin;
    for (; r + kStatsUnroll <= r_end; r += kStatsUnroll) {
        XUnit<DT, EPU> v[kStatsUnroll];
#pragma unroll
        for (int j = 0; j < kStatsUnroll; ++j) v[j].load(X, (r + j) * ldx + col);
#pragma unroll
        for (int j = 0; j < kStatsUnroll; ++j) v[j].sq_add(acc[j % kStatsSets]);
    }
    for (; r < r_end; ++r) {
        XUnit<DT, EPU> v;
        v.load(X, r * ldx + col);
        v.sq_add(acc[0]);
    }

    float* p = partials + (int64_t)split * (units * EPU) + col;
#pragma unroll
    for (int k = 0; k < EPU; ++k) p[k] = (acc[0][k] + acc[1][k]) + (acc[2][k] + acc[3][k]);
}

// hr = 1/2 / (1 - xsq/S): three fp32 roundings (divide, subtract, divide).
// S == 0 gives 1/2; a denominator that is not positive is replaced by FLT_EPSILON.
__device__ __forceinline__ float channel_factor(float xsq, float S) {
    if (S == 0.0f) return 0.5f;
    const float rho = __fdiv_rn(xsq, S);
    float den = __fsub_rn(1.0f, rho);
    if (!(den > 0.0f)) den = 1.1920928955078125e-07f;
    return __fdiv_rn(0.5f, den);
}

// grid = ceil(in / 64), block = 1024: thread (c = tid & 63, g = tid >> 6) adds the partial rows
// s = g, g+16, ... of column blockIdx.x*64 + c in fp64; the sixteen groups are added in order
// through LDS.  Every workgroup also leaves the fp64 sum of its 64 columns in s_part; the last
// workgroup to finish adds those in order (= S) and writes the factor for all channels.
__global__ __launch_bounds__(kCombineThreads) void stats_combine_kernel(
    const float* __restrict__ partials, int splits, int64_t in_pad, int64_t in, float* xsq,
    int accumulate, int finalize, float* __restrict__ S_out, float* __restrict__ hr,
    unsigned int* __restrict__ counters, double* s_part) {
    __shared__ double part[kCombineGroups][64];
    __shared__ double colsum[64];
    __shared__ double red[kCombineThreads / 64];
    __shared__ unsigned int ticket;
    __shared__ float S_sh;

    const int c = threadIdx.x & 63;
    const int g = threadIdx.x >> 6;
    const int64_t col = (int64_t)blockIdx.x * 64 + c;

    double s = 0.0;
    if (col < in) {
        const float* p = partials + col;
        int sp = g;
        for (; sp + 3 * kCombineGroups < splits; sp += 4 * kCombineGroups) {
            const float a0 = p[(int64_t)sp * in_pad];
            const float a1 = p[(int64_t)(sp + kCombineGroups) * in_pad];
            const float a2 = p[(int64_t)(sp + 2 * kCombineGroups) * in_pad];
            const float a3 = p[(int64_t)(sp + 3 * kCombineGroups) * in_pad];
            s += (double)a0;
            s += (double)a1;
            s += (double)a2;
            s += (double)a3;
        }
        for (; sp < splits; sp += kCombineGroups) s += (double)p[(int64_t)sp * in_pad];
    }
    part[g][c] = s;
    __syncthreads();
    if (g == 0) {
        double t = 0.0;
#pragma unroll
        for (int i = 0; i < kCombineGroups; ++i) t += part[i][c];
        float x = 0.f;
        if (col < in) {
            if (accumulate) t += (double)xsq[col];
            x = (float)t;
            xsq[col] = x;
        }
        colsum[c] = (double)x;  // S is the sum of the rounded per-channel values
    }
    if (!finalize) return;
    __syncthreads();
    if (threadIdx.x == 0) {
        double t = 0.0;
        for (int i = 0; i < 64; ++i) t += colsum[i];
        s_part[blockIdx.x] = t;
        __threadfence();  // publish s_part (and this workgroup's xsq) before taking the ticket
        ticket = atomicAdd(&counters[0], 1u);
    }
    __syncthreads();
    if (ticket != gridDim.x - 1) return;
    __threadfence();

    // last workgroup: S = sum of the per-workgroup sums, in index order
    const volatile double* sp_v = s_part;
    const int nblk = (int)gridDim.x;
    double t = 0.0;
    for (int i = threadIdx.x; i < nblk; i += kCombineThreads) t += sp_v[i];
    // fixed-shape tree: within a wavefront by lane halving, then across wavefronts in order
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) t += __shfl_down(t, off, kWave);
    if (c == 0) red[g] = t;
    __syncthreads();
    if (threadIdx.x == 0) {
        double tot = 0.0;
        for (int i = 0; i < kCombineThreads / 64; ++i) tot += red[i];
        S_sh = (float)tot;
        S_out[0] = S_sh;
    }
    __syncthreads();
    const float S = S_sh;
    const volatile float* xs = xsq;  // written by other workgroups of this launch
    for (int64_t q0 = threadIdx.x; q0 < in; q0 += 4 * kCombineThreads) {
        float x[4];
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int64_t q = q0 + (int64_t)j * kCombineThreads;
            x[j] = (q < in) ? xs[q] : 0.f;
        }
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int64_t q = q0 + (int64_t)j * kCombineThreads;
            if (q < in) hr[q] = channel_factor(x[j], S);
        }
    }
}

static inline int64_t ceil_div(int64_t a, int64_t b) { return (a + b - 1) / b; }

StatsPlan make_stats_plan(int64_t tokens, int64_t in, int dt, bool vec) {
    StatsPlan p;
    p.epu = vec ? (dt == kBF16 ? 8 : 4) : 1;
    p.units = ceil_div(in, p.epu);
    p.nstrips = (int)ceil_div(p.units, kStatsThreads);
    // equal strips, rounded up to 8 units (128 bytes) so that strips start on a cache line
    int64_t su = ceil_div(ceil_div(p.units, p.nstrips), 8) * 8;
    if (su > kStatsThreads) su = kStatsThreads;
    p.strip_units = (int)su;
    p.nstrips = (int)ceil_div(p.units, su);
    // about one workgroup per compute unit, and no range shorter than one batch of rows
    int64_t splits = kStatsTargetGroups / p.nstrips;
    const int64_t max_splits = ceil_div(tokens, kStatsUnroll);
    if (splits > max_splits) splits = max_splits;
    if (splits < 1) splits = 1;
    p.rows_per_split = ceil_div(tokens, splits);
    p.splits = (int)ceil_div(tokens, p.rows_per_split);  // drop ranges that would be empty
    p.combine_groups = (int)ceil_div(in, 64);
    p.partial_floats = (size_t)p.splits * (size_t)(p.units * p.epu);
    return p;
}

size_t stats_workspace_bytes(const StatsPlan& p) {
    return kStatsHeaderBytes + (size_t)ceil_div(p.combine_groups * 8, 256) * 256 +
           p.partial_floats * sizeof(float);
}

template <int DT, int EPU>
static hipError_t launch_partial(const void* X, int64_t tokens, int64_t ldx, const StatsPlan& p,
                                 float* partials, unsigned int* counters, hipStream_t stream) {
    dim3 grid((unsigned)p.nstrips, (unsigned)p.splits);
    hipLaunchKernelGGL((stats_partial_kernel<DT, EPU>), grid, dim3(kStatsThreads), 0, stream, X, tokens,
                       p.units, p.strip_units, ldx, p.rows_per_split, partials, counters);
    return hipGetLastError();
}

hipError_t launch_layer_stats(const void* X, int64_t tokens, int64_t in, int64_t ldx, int dt, bool vec,
                              float* xsq, float* S, float* hr, int accumulate, int finalize,
                              void* workspace, hipStream_t stream) {
    const StatsPlan p = make_stats_plan(tokens, in, dt, vec);
    char* ws = static_cast<char*>(workspace);
    unsigned int* counters = reinterpret_cast<unsigned int*>(ws);
    double* s_part = reinterpret_cast<double*>(ws + kStatsHeaderBytes);
    float* partials =
        reinterpret_cast<float*>(ws + kStatsHeaderBytes + (size_t)ceil_div(p.combine_groups * 8, 256) * 256);
    hipError_t e;
    if (dt == kBF16)
        e = vec ? launch_partial<kBF16, 8>(X, tokens, ldx, p, partials, counters, stream)
                : launch_partial<kBF16, 1>(X, tokens, ldx, p, partials, counters, stream);
    else
        e = vec ? launch_partial<kF32, 4>(X, tokens, ldx, p, partials, counters, stream)
                : launch_partial<kF32, 1>(X, tokens, ldx, p, partials, counters, stream);
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(stats_combine_kernel, dim3((unsigned)p.combine_groups), dim3(kCombineThreads), 0,
                       stream, partials, p.splits, p.units * p.epu, in, xsq, accumulate, finalize, S, hr,
                       counters, s_part);
    return hipGetLastError();
}

}  // namespace sp

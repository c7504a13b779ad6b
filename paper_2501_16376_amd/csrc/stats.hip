// Step 1 of the SwiftPrune layer path: per-input-channel sums of squares of the
// calibration activations, their total S, and the per-channel score factor
// (Algorithm 1, first statement; Sec. 3.1, definition of S and the score equation).
//
// X[tokens, in] is streamed exactly once with non-temporal 16-byte loads.  The
// columns are cut into strips of at most 256 sixteen-byte units (one unit per
// lane of a 256-thread workgroup: 2048 bf16 / fp16 or 1024 fp32 columns, contiguous in
// every row) and the tokens into batches of 4 or 8 consecutive rows that are
// dealt round-robin to `splits` workgroups per strip, so that at any moment the
// whole device reads one moving window of a few MB (measured 1-7 % faster than
// giving every workgroup its own contiguous token range); strips x splits is
// about one workgroup per compute unit (more resident workgroups lower the
// achieved HBM rate).  Every lane keeps fp32 running sums for the columns of
// its unit, a batch of rows in flight, in four independent accumulator sets that
// are folded into fp64 sums every 128 rows, so no serial fp32 chain exceeds 32
// terms.  Each workgroup writes one partial row segment and the fp64 sum of it;
// a second small kernel adds the partial rows of every column in fp64 in a fixed
// order (LDS-staged), adds the per-workgroup sums in index order to get S (every
// workgroup redoes that small sum, so none waits for another) and writes the
// factor.  No atomics, no fences: results do not depend on scheduling.
#include "common.hpp"
#include "kernels.hpp"

namespace sp {

constexpr int kStatsThreads = 256;       // one wide strip per workgroup, 4 wavefronts
constexpr int kStatsSets = 4;            // independent fp32 accumulator sets per column
constexpr int kStatsFlushRows = 128;     // rows between folds of the fp32 sets into the fp64 sums
constexpr int kStatsComputeUnits = 256;   // compute units of an MI355X
constexpr int kCombineThreads = 256;     // 64 columns x 4 groups of partial rows
constexpr int kCombineGroups = kCombineThreads / 64;

template <int DT, int EPU>
struct XUnit;

template <>
struct XUnit<kBF16, 8> {
    u32x4 r;
    __device__ __forceinline__ void load(const void* X, int64_t elem) {
        r = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(static_cast<const uint16_t*>(X) + elem));
    }
    __device__ __forceinline__ void load_plain(const void* X, int64_t elem) {
        r = *reinterpret_cast<const u32x4*>(static_cast<const uint16_t*>(X) + elem);
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
struct XUnit<kF16, 8> {
    u32x4 r;
    __device__ __forceinline__ void load(const void* X, int64_t elem) {
        r = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(static_cast<const uint16_t*>(X) + elem));
    }
    __device__ __forceinline__ void sq_add(float* a) const {
        float v;
        v = f16lo(r.x); a[0] = fmaf(v, v, a[0]);
        v = f16hi(r.x); a[1] = fmaf(v, v, a[1]);
        v = f16lo(r.y); a[2] = fmaf(v, v, a[2]);
        v = f16hi(r.y); a[3] = fmaf(v, v, a[3]);
        v = f16lo(r.z); a[4] = fmaf(v, v, a[4]);
        v = f16hi(r.z); a[5] = fmaf(v, v, a[5]);
        v = f16lo(r.w); a[6] = fmaf(v, v, a[6]);
        v = f16hi(r.w); a[7] = fmaf(v, v, a[7]);
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
struct XUnit<kF16, 1> {
    float r;
    __device__ __forceinline__ void load(const void* X, int64_t elem) {
        r = f16bits(__builtin_nontemporal_load(static_cast<const uint16_t*>(X) + elem));
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

// Sum of a double over the 256 threads of a workgroup, fixed shape: lane tree
// inside each wavefront, then the four wavefront totals in order.  All threads
// must call it; every thread gets the result.
__device__ __forceinline__ double block_sum_256(double v, double* lds4) {
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) v += __shfl_down(v, off, kWave);
    if ((threadIdx.x & (kWave - 1)) == 0) lds4[threadIdx.x >> 6] = v;
    __syncthreads();
    const double t = ((lds4[0] + lds4[1]) + lds4[2]) + lds4[3];
    __syncthreads();
    return t;
}

// grid = (nstrips, splits), block = 256.  Workgroup (strip, split) takes the row batches
// b = split, split + splits, ... (batch b = rows [b*UNROLL, (b+1)*UNROLL)).
// partials[split * in_pad + u*EPU + k] = sum over those rows of X[t, u*EPU + k]^2
// for the units u of its strip (in_pad = units * EPU);
// group_sums[strip * splits + split] = fp64 sum of that partial row segment (its share of S).
template <int DT, int EPU, int UNROLL, bool PLAIN = false>
__global__ __launch_bounds__(kStatsThreads) __attribute__((amdgpu_waves_per_eu(1, 2))) void stats_partial_kernel(
    const void* __restrict__ X, int64_t tokens, int64_t units, int strip_units, int64_t ldx,
    float* __restrict__ partials, double* __restrict__ group_sums) {
    __shared__ double lds4[4];
    const int strip = blockIdx.x;
    const int split = blockIdx.y;
    const int64_t splits = gridDim.y;
    const int64_t u = (int64_t)strip * strip_units + threadIdx.x;
    const bool active = (int)threadIdx.x < strip_units && u < units;
    const int64_t col = u * EPU;

    // two levels: four fp32 accumulator sets per column take at most kStatsFlushRows rows, then they
    // are folded into an fp64 sum and cleared.  A long fp32 chain of squares loses every addend that
    // falls below half an ulp of the running sum (a systematic deficit of several 1e-6 after a few
    // thousand rows); with short chains the result is within one fp32 rounding of the exact sum.
    float acc[kStatsSets][EPU];
    double acc64[EPU];
#pragma unroll
    for (int k = 0; k < EPU; ++k) {
        acc64[k] = 0.0;
#pragma unroll
        for (int s = 0; s < kStatsSets; ++s) acc[s][k] = 0.f;
    }
    auto fold = [&]() {
#pragma unroll
        for (int k = 0; k < EPU; ++k) {
            acc64[k] += (double)((acc[0][k] + acc[1][k]) + (acc[2][k] + acc[3][k]));
#pragma unroll
            for (int s = 0; s < kStatsSets; ++s) acc[s][k] = 0.f;
        }
    };

    double lane_total = 0.0;
    if (active) {
        int64_t r = (int64_t)split * UNROLL;
        const int64_t step = splits * UNROLL;
        constexpr int kFoldEvery = kStatsFlushRows / UNROLL;  // batches between folds
        int since_fold = 0;
        for (; r + UNROLL <= tokens; r += step) {
            XUnit<DT, EPU> v[UNROLL];
#pragma unroll
            for (int j = 0; j < UNROLL; ++j) {
                if constexpr (PLAIN) v[j].load_plain(X, (r + j) * ldx + col);   // measurement variant, bf16 vector path only
                else v[j].load(X, (r + j) * ldx + col);
            }
            if (++since_fold == kFoldEvery) {  // uniform; runs while the loads above are in flight
                fold();
                since_fold = 0;
            }
#pragma unroll
            for (int j = 0; j < UNROLL; ++j) v[j].sq_add(acc[j % kStatsSets]);
        }
        for (; r < tokens; ++r) {  // the one batch that is cut short by the end of X, if it is ours
            XUnit<DT, EPU> v;
            v.load(X, r * ldx + col);
            v.sq_add(acc[0]);
        }
        fold();
        float* p = partials + (int64_t)split * (units * EPU) + col;
#pragma unroll
        for (int k = 0; k < EPU; ++k) {
            p[k] = (float)acc64[k];
            lane_total += acc64[k];
        }
    }
    const double total = block_sum_256(lane_total, lds4);
    if (threadIdx.x == 0) group_sums[(int64_t)strip * gridDim.y + split] = total;
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

// grid = ceil(in / 64), block = 256: thread (c = tid & 63, g = tid >> 6) adds the partial rows
// s = g, g+4, ... of column blockIdx.x*64 + c in fp64; the four groups are added in order through
// LDS.  Every workgroup also adds the streaming kernel's per-workgroup sums in index order, so all
// of them hold the same S without talking to each other, and writes the factor of its 64 columns.
__global__ __launch_bounds__(kCombineThreads) void stats_combine_kernel(
    const float* __restrict__ partials, int splits, int64_t in_pad, int64_t in,
    const double* __restrict__ group_sums, int ngroups, float* __restrict__ xsq, int accumulate,
    int finalize, float* __restrict__ S_io, float* __restrict__ hr) {
    __shared__ double part[kCombineGroups][64];
    __shared__ double lds4[4];

    const int c = threadIdx.x & 63;
    const int g = threadIdx.x >> 6;
    const int64_t col = (int64_t)blockIdx.x * 64 + c;

    // S of this call: the same fixed-order sum in every workgroup
    double gs = 0.0;
    for (int i = threadIdx.x; i < ngroups; i += kCombineThreads) gs += group_sums[i];
    double S_d = block_sum_256(gs, lds4);
    // the running S is read by everybody only when the factors are due; otherwise workgroup 0 alone reads
    // and rewrites it
    if (accumulate && (finalize || blockIdx.x == 0)) S_d += (double)S_io[0];
    const float S = (float)S_d;

    double s = 0.0;
    if (col < in) {
        const float* p = partials + col;
        int sp = g;
        for (; sp + 7 * kCombineGroups < splits; sp += 8 * kCombineGroups) {
            float a[8];
#pragma unroll
            for (int j = 0; j < 8; ++j) a[j] = p[(int64_t)(sp + j * kCombineGroups) * in_pad];
#pragma unroll
            for (int j = 0; j < 8; ++j) s += (double)a[j];
        }
        for (; sp < splits; sp += kCombineGroups) s += (double)p[(int64_t)sp * in_pad];
    }
    part[g][c] = s;
    __syncthreads();
    if (g == 0 && col < in) {
        double t = ((part[0][c] + part[1][c]) + part[2][c]) + part[3][c];
        if (accumulate) t += (double)xsq[col];
        const float x = (float)t;
        xsq[col] = x;
        if (finalize) hr[col] = channel_factor(x, S);
    }
    // when accumulating and finalising, every workgroup reads the old S_io above, so the new value is stored
    // by a separate launch; otherwise nobody but workgroup 0 reads it and workgroup 0 stores it here
    if (!(accumulate && finalize) && blockIdx.x == 0 && threadIdx.x == 0) S_io[0] = S;
}

// S[0] <- (accumulate ? S[0] : 0) + sum of the per-workgroup sums; same order as in the combine kernel
__global__ __launch_bounds__(kCombineThreads) void stats_total_kernel(const double* __restrict__ group_sums,
                                                                     int ngroups, int accumulate,
                                                                     float* __restrict__ S_io) {
    __shared__ double lds4[4];
    double gs = 0.0;
    for (int i = threadIdx.x; i < ngroups; i += kCombineThreads) gs += group_sums[i];
    double S_d = block_sum_256(gs, lds4);
    if (threadIdx.x == 0) {
        if (accumulate) S_d += (double)S_io[0];
        S_io[0] = (float)S_d;
    }
}

// hr[q] from given xsq[q] and S: the last part of the statistics step on its own.
__global__ __launch_bounds__(kCombineThreads) void channel_factor_kernel(const float* __restrict__ xsq,
                                                                        const float* __restrict__ S, int64_t in,
                                                                        float* __restrict__ hr) {
    const int64_t q = (int64_t)blockIdx.x * kCombineThreads + threadIdx.x;
    if (q < in) hr[q] = channel_factor(xsq[q], S[0]);
}

static inline int64_t ceil_div(int64_t a, int64_t b) { return (a + b - 1) / b; }

StatsPlan make_stats_plan(int64_t tokens, int64_t in, int dt, bool vec) {
    StatsPlan p;
    p.epu = vec ? (dt == kF32 ? 4 : 8) : 1;
    p.units = ceil_div(in, p.epu);
    p.nstrips = (int)ceil_div(p.units, kStatsThreads);
    // equal strips, rounded up to 8 units (128 bytes) so that strips start on a cache line
    int64_t su = ceil_div(ceil_div(p.units, p.nstrips), 8) * 8;
    if (su > kStatsThreads) su = kStatsThreads;
    p.strip_units = (int)su;
    p.nstrips = (int)ceil_div(p.units, su);
    // Rows in flight per lane and workgroups, from sweeps over 2560 ... 28672 bf16 columns at 262144 tokens
    // on MI355X (rows in flight 4 / 8 / 16 against 256 / 384 / 512 / 768 workgroups):
    //  * strips much narrower than the workgroup (fewer than 70 % of the lanes used, e.g. 2560 columns =
    //    2 x 160 lanes): every lane keeps 16 rows in flight, or too few bytes are in flight
    //  * strips whose last wavefront is less than half used (5120 columns = 3 x 216 lanes): 4 rows and two
    //    workgroups per compute unit (11008 = 6 x 232 lanes is better off with the rule for full strips)
    //  * full strips: a power-of-two number of strips maps every strip to a fixed subset of the 8 XCDs and
    //    does best with 4 rows and 1.5 workgroups per compute unit; otherwise 8 rows and 1 workgroup
    //  * two full strips (4096 bf16 columns, six of the seven layers of a Llama block): 8 rows and 224
    //    workgroups, a narrow optimum (whole-model time with 200 / 208 / 216 / 224 / 232 / 240 workgroups:
    //    99.2 / 97.8 / 96.7 / 95.9 / 96.4 / 97.5 ms, against 97.3 ms for 4 rows and 384).
    const bool pow2_strips = (p.nstrips & (p.nstrips - 1)) == 0;
    const int fill_pct = (int)(su * 100 / kStatsThreads);
    int64_t target;
    if (fill_pct < 70) {
        p.unroll = 16;
        target = kStatsComputeUnits;
    } else if (fill_pct < 88) {
        p.unroll = 4;
        target = kStatsComputeUnits * 2;
    } else if (p.nstrips == 2) {
        p.unroll = 8;
        target = 224;
    } else if (pow2_strips) {
        p.unroll = 4;
        target = kStatsComputeUnits * 3 / 2;
    } else {
        p.unroll = 8;
        target = kStatsComputeUnits;
    }
    int64_t splits = target / p.nstrips;
    const int64_t batches = ceil_div(tokens, p.unroll);
    if (splits > batches) splits = batches;
    if (splits < 1) splits = 1;
    p.splits = (int)splits;
    p.rows_per_split = ceil_div(batches, splits) * p.unroll;  // upper bound, informational
    p.plain_loads = false;
    const Tuning t = read_tuning();
    if (t.stats_rows != 0) {  // measurement override
        p.unroll = t.stats_rows;
        int64_t s2 = t.stats_groups / p.nstrips;
        const int64_t b2 = ceil_div(tokens, p.unroll);
        if (s2 > b2) s2 = b2;
        if (s2 < 1) s2 = 1;
        p.splits = (int)s2;
        p.rows_per_split = ceil_div(b2, s2) * p.unroll;
        p.plain_loads = t.stats_plain && vec && dt == kBF16;
    }
    p.combine_groups = (int)ceil_div(in, 64);
    p.partial_floats = (size_t)p.splits * (size_t)(p.units * p.epu);
    return p;
}

static inline size_t group_sum_bytes(const StatsPlan& p) {
    return (size_t)ceil_div((int64_t)p.nstrips * p.splits * 8, 256) * 256;
}

size_t stats_workspace_bytes(const StatsPlan& p) {
    return kStatsHeaderBytes + group_sum_bytes(p) + p.partial_floats * sizeof(float);
}

template <int DT, int EPU>
static hipError_t launch_partial(const void* X, int64_t tokens, int64_t ldx, const StatsPlan& p,
                                 float* partials, double* group_sums, hipStream_t stream) {
    dim3 grid((unsigned)p.nstrips, (unsigned)p.splits);
    if constexpr (DT == kBF16 && EPU == 8) {
        if (p.plain_loads) {
            if (p.unroll == 16)
                hipLaunchKernelGGL((stats_partial_kernel<DT, EPU, 16, true>), grid, dim3(kStatsThreads), 0, stream, X, tokens,
                                   p.units, p.strip_units, ldx, partials, group_sums);
            else if (p.unroll == 4)
                hipLaunchKernelGGL((stats_partial_kernel<DT, EPU, 4, true>), grid, dim3(kStatsThreads), 0, stream, X, tokens,
                                   p.units, p.strip_units, ldx, partials, group_sums);
            else
                hipLaunchKernelGGL((stats_partial_kernel<DT, EPU, 8, true>), grid, dim3(kStatsThreads), 0, stream, X, tokens,
                                   p.units, p.strip_units, ldx, partials, group_sums);
            return hipGetLastError();
        }
    }
    if (p.unroll == 16)
        hipLaunchKernelGGL((stats_partial_kernel<DT, EPU, 16>), grid, dim3(kStatsThreads), 0, stream, X, tokens,
                           p.units, p.strip_units, ldx, partials, group_sums);
    else if (p.unroll == 4)
        hipLaunchKernelGGL((stats_partial_kernel<DT, EPU, 4>), grid, dim3(kStatsThreads), 0, stream, X, tokens,
                           p.units, p.strip_units, ldx, partials, group_sums);
    else
        hipLaunchKernelGGL((stats_partial_kernel<DT, EPU, 8>), grid, dim3(kStatsThreads), 0, stream, X, tokens,
                           p.units, p.strip_units, ldx, partials, group_sums);
    return hipGetLastError();
}

hipError_t launch_layer_stats(const void* X, int64_t tokens, int64_t in, int64_t ldx, int dt, bool vec,
                              float* xsq, float* S, float* hr, int accumulate, int finalize,
                              void* workspace, hipStream_t stream) {
    const StatsPlan p = make_stats_plan(tokens, in, dt, vec);
    char* ws = static_cast<char*>(workspace);
    double* group_sums = reinterpret_cast<double*>(ws + kStatsHeaderBytes);
    float* partials = reinterpret_cast<float*>(ws + kStatsHeaderBytes + group_sum_bytes(p));
    hipError_t e;
    if (dt == kBF16)
        e = vec ? launch_partial<kBF16, 8>(X, tokens, ldx, p, partials, group_sums, stream)
                : launch_partial<kBF16, 1>(X, tokens, ldx, p, partials, group_sums, stream);
    else if (dt == kF16)
        e = vec ? launch_partial<kF16, 8>(X, tokens, ldx, p, partials, group_sums, stream)
                : launch_partial<kF16, 1>(X, tokens, ldx, p, partials, group_sums, stream);
    else
        e = vec ? launch_partial<kF32, 4>(X, tokens, ldx, p, partials, group_sums, stream)
                : launch_partial<kF32, 1>(X, tokens, ldx, p, partials, group_sums, stream);
    if (e != hipSuccess) return e;
    const int ngroups = p.nstrips * p.splits;
    hipLaunchKernelGGL(stats_combine_kernel, dim3((unsigned)p.combine_groups), dim3(kCombineThreads), 0,
                       stream, partials, p.splits, p.units * p.epu, in, group_sums, ngroups, xsq,
                       accumulate, finalize, S, hr);
    e = hipGetLastError();
    if (e != hipSuccess || !(accumulate && finalize)) return e;
    hipLaunchKernelGGL(stats_total_kernel, dim3(1), dim3(kCombineThreads), 0, stream, group_sums, ngroups,
                       accumulate, S);
    return hipGetLastError();
}

hipError_t launch_channel_factor(const float* xsq, const float* S, int64_t in, float* hr, hipStream_t stream) {
    hipLaunchKernelGGL(channel_factor_kernel, dim3((unsigned)ceil_div(in, kCombineThreads)), dim3(kCombineThreads),
                       0, stream, xsq, S, in, hr);
    return hipGetLastError();
}

}  // namespace sp

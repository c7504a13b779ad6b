// N:M structured selection (Sec. 3.3) fused with the score (Sec. 3.1), and the
// in-place apply step (Algorithm 1: pruned w_i = 0).
//
// Both are plain streaming kernels.  A lane owns one chunk of 8 consecutive
// columns (one 16-byte load of bf16) and walks several rows with it, so the
// channel factors of its columns are loaded once and several independent loads
// are in flight.  N:M ranks are computed in registers by counting, with ties
// broken towards the lower index: rank_i = #{p : (L_p, p) < (L_i, i)}, and
// entry i is pruned iff rank_i < M - N.  Groups of 4 and 8 live inside one
// lane; a group of 16 spans two neighbouring lanes and exchanges its scores
// with one DPP quad permute per value.
// Two kernel families: tile kernels for element-wise layouts (odd widths,
// unaligned pointers), band kernels for the 16-byte-vector layout.
#include "common.hpp"
#include "kernels.hpp"

namespace sp {

constexpr int kRows = 8;        // rows per lane
constexpr int kColThreads = 256;

// keep bits of the 8 scores of a lane for group size M <= 8.  One comparison per pair serves both of its
// entries: with c(p,i) = [L_p <= L_i] for p < i,
//     rank_i = #{p < i : L_p <= L_i} + #{p > i : L_p < L_i} = sum_{p<i} c(p,i) + (M-1-i) - sum_{p>i} c(i,p).
template <int M>
__device__ __forceinline__ uint32_t nm_keep_bits(const float* L, int n_prune) {
    uint32_t keep = 0u;
#pragma unroll
    for (int g = 0; g < 8; g += M) {
        int rank[M];
#pragma unroll
        for (int i = 0; i < M; ++i) rank[i] = M - 1 - i;
#pragma unroll
        for (int i = 1; i < M; ++i) {
#pragma unroll
            for (int p = 0; p < i; ++p) {
                const int c = (L[g + p] <= L[g + i]) ? 1 : 0;
                rank[i] += c;
                rank[p] -= c;
            }
        }
#pragma unroll
        for (int i = 0; i < M; ++i) keep |= (rank[i] >= n_prune) ? (1u << (g + i)) : 0u;
    }
    return keep;
}

// group of 16 = this lane's 8 scores and its partner lane's (lane ^ 1) 8 scores
__device__ __forceinline__ uint32_t nm_keep_bits16(const float* L, int n_prune, int lane) {
    float other[8];
#pragma unroll
    for (int k = 0; k < 8; ++k) other[k] = dpp_f<kQuadSwap1>(L[k]);
    const bool upper = lane & 1;  // this lane holds group positions 8..15
    uint32_t keep = 0u;
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        int rank = 0;
#pragma unroll
        for (int p = 0; p < 8; ++p) {
            if (p != i) {
                const bool less = (p < i) ? (L[p] <= L[i]) : (L[p] < L[i]);
                rank += less ? 1 : 0;
            }
            // partner entries all precede (upper) or all follow (lower) this lane's entries
            const bool less_o = upper ? (other[p] <= L[i]) : (other[p] < L[i]);
            rank += less_o ? 1 : 0;
        }
        keep |= (rank >= n_prune) ? (1u << i) : 0u;
    }
    return keep;
}

// A wavefront owns a tile of kRows rows x 64 chunks (512 columns); tiles are numbered column-first, so the
// four wavefronts of a workgroup and consecutive workgroups touch consecutive memory, and a row width that
// is not a multiple of 2048 columns wastes at most part of one wavefront.  grid = ceil(tiles / 4), block = 256.
template <int DT, int M>
__global__ __launch_bounds__(kColThreads) void nm_select_kernel(
    void* __restrict__ W, int64_t out, int64_t in, int64_t ldw, const float* __restrict__ hr,
    int n_prune, uint32_t* __restrict__ keep_mask, float* __restrict__ scores, int apply,
    unsigned col_tiles) {
    const int lane = threadIdx.x & (kWave - 1);
    const int64_t tile = (int64_t)blockIdx.x * (kColThreads / kWave) + (threadIdx.x >> 6);
    const int64_t chunk = (tile % col_tiles) * kWave + lane;
    const int64_t q0 = chunk * 8;
    const int valid = (int)min((int64_t)8, max((int64_t)0, in - q0));
    const int64_t row0 = (tile / col_tiles) * kRows;
    const int64_t mask_words = (in + 31) >> 5;
    const int nrows = (int)max((int64_t)0, min((int64_t)kRows, out - row0));  // 0 for a wavefront past the last tile

    Factor8 f;
    f.load_elems(hr, q0, valid);

    Chunk8<DT> w[kRows];
#pragma unroll
    for (int r = 0; r < kRows; ++r) {
        w[r].zero();
        if (r < nrows && valid) {
            w[r].load_elems(W, (row0 + r) * ldw + q0, valid);
        }
    }
#pragma unroll
    for (int r = 0; r < kRows; ++r) {
        if (r >= nrows) break;  // uniform over the wavefront
        float L[8];
#pragma unroll
        for (int k = 0; k < 8; ++k) L[k] = score_of(w[r].get(k), f.v[k]);
        uint32_t keep = (M == 16) ? nm_keep_bits16(L, n_prune, lane) : nm_keep_bits<(M == 16 ? 8 : M)>(L, n_prune);
        keep &= (valid >= 8) ? 0xffu : ((1u << valid) - 1u);
        const int64_t row = row0 + r;
        if (scores != nullptr && valid) store8(scores + row * in + q0, L, false, valid);
        const uint32_t word = quad_gather_bytes(keep, lane);
        const int64_t widx = q0 >> 5;
        if ((lane & 3) == 0 && widx < mask_words) keep_mask[row * mask_words + widx] = word;
        if (apply && valid) {
            w[r].apply(keep);
            w[r].store_elems(W, row * ldw + q0, valid);
        }
    }
}

// grid / block as above
template <int DT>
__global__ __launch_bounds__(kColThreads) void apply_kernel(void* __restrict__ W, int64_t out, int64_t in,
                                                           int64_t ldw,
                                                           const uint32_t* __restrict__ keep_mask,
                                                           unsigned col_tiles) {
    const int64_t tile = (int64_t)blockIdx.x * (kColThreads / kWave) + (threadIdx.x >> 6);
    const int64_t chunk = (tile % col_tiles) * kWave + (threadIdx.x & (kWave - 1));
    const int64_t q0 = chunk * 8;
    const int valid = (int)min((int64_t)8, max((int64_t)0, in - q0));
    if (valid == 0) return;
    const int64_t row0 = (tile / col_tiles) * kRows;
    const int64_t mask_words = (in + 31) >> 5;
    const int nrows = (int)max((int64_t)0, min((int64_t)kRows, out - row0));  // 0 for a wavefront past the last tile
    const int shift = (int)(q0 & 31);

    Chunk8<DT> w[kRows];
    uint32_t keep[kRows];
#pragma unroll
    for (int r = 0; r < kRows; ++r) {
        if (r < nrows) {
            w[r].load_elems(W, (row0 + r) * ldw + q0, valid);
            keep[r] = (keep_mask[(row0 + r) * mask_words + (q0 >> 5)] >> shift) & 0xffu;
        }
    }
#pragma unroll
    for (int r = 0; r < kRows; ++r) {
        if (r < nrows) {
            w[r].apply(keep[r]);
            w[r].store_elems(W, (row0 + r) * ldw + q0, valid);
        }
    }
}

// ---------------------------------------------------------------------------
// Band variants for the 16-byte-vector path.  In-place read-modify-write streams
// run fastest on this part when the whole device walks ONE contiguous window in
// lock step (a few workgroups per compute unit, non-temporal loads and stores)
// instead of every workgroup owning a region of its own.  The columns are cut
// into strips of at most 256 chunks (one chunk of 8 columns per lane, fixed for
// the lifetime of the lane, so its channel factors are loaded once) and the
// rows into batches of U consecutive rows dealt round-robin to the `splits`
// workgroups of a strip: at any moment all workgroups together read, and then
// rewrite, splits*U consecutive rows.  grid = (nstrips, splits), block = 256.
// ---------------------------------------------------------------------------
struct BandPlan {
    int strip_units;  // chunks of 8 columns per strip (multiple of 8, <= 256)
    int nstrips;
    int splits;
    int unroll;       // rows per batch
};

BandPlan make_band_plan(int64_t out, int64_t in, int target_groups, int unroll = 4) {
    BandPlan p;
    const int64_t units = (in + 7) / 8;
    int64_t nstrips = (units + kColThreads - 1) / kColThreads;
    int64_t su = ((units + nstrips - 1) / nstrips + 7) / 8 * 8;
    if (su > kColThreads) su = kColThreads;
    nstrips = (units + su - 1) / su;
    p.strip_units = (int)su;
    p.nstrips = (int)nstrips;
    p.unroll = unroll > 4 ? 4 : unroll;  // 1, 2 or 4 rows per batch
    int64_t splits = target_groups / nstrips;
    // small matrices: fewer rows per batch before fewer workgroups
    while (p.unroll > 1 && (out + p.unroll - 1) / p.unroll < splits) p.unroll >>= 1;
    const int64_t batches = (out + p.unroll - 1) / p.unroll;
    if (splits > batches) splits = batches;
    if (splits < 1) splits = 1;
    p.splits = (int)splits;
    return p;
}

template <int DT, int M, int U, bool GROUPED>
__global__ __launch_bounds__(kColThreads) void nm_select_band_kernel(
    const RowGroups g, int64_t in, const float* __restrict__ hr, int n_prune, float* __restrict__ scores,
    int apply, int strip_units) {
    const int lane = threadIdx.x & (kWave - 1);
    const int64_t unit = (int64_t)blockIdx.x * strip_units + threadIdx.x;
    const int64_t q0 = unit * 8;
    const bool active = (int)threadIdx.x < strip_units && q0 < in;  // in % 8 == 0 on this path
    const int64_t q_ld = active ? q0 : 0;  // lanes without columns read the row's start and store nothing
    const int64_t mask_words = (in + 31) >> 5;
    const int32_t step = (int32_t)(gridDim.y * U);
    const int32_t out = g.total();  // rows of all matrices of the group, numbered consecutively (< 2^31)

    Factor8 f;
    f.load_vec(hr, q_ld);

    auto fetch = [&](Chunk8<DT>* w, int32_t r0) {
        if (r0 >= out) return;  // uniform, like every row test below: the lookups stay on the scalar unit
        RowOwner<RowGroups> own(g, GROUPED ? r0 : 0);
#pragma unroll
        for (int j = 0; j < U; ++j) {
            if (r0 + j < out) {
                if (GROUPED) own.seek(g, r0 + j);
                const int64_t row = GROUPED ? own.row : (int64_t)(r0 + j);
                w[j].load_vec(own.W, row * own.ldw + q_ld);
            }
        }
    };
    auto work = [&](Chunk8<DT>* w, int32_t r0) {
        RowOwner<RowGroups> own(g, GROUPED ? r0 : 0);
#pragma unroll
        for (int j = 0; j < U; ++j) {
            if (r0 + j >= out) break;  // uniform over the workgroup
            if (GROUPED) own.seek(g, r0 + j);
            const int64_t row = GROUPED ? own.row : (int64_t)(r0 + j);
            float L[8];
#pragma unroll
            for (int k = 0; k < 8; ++k) L[k] = score_of(w[j].get(k), f.v[k]);
            if (scores != nullptr && active) store8(scores + (int64_t)(r0 + j) * in + q0, L, true, 8);  // single matrix only
            uint32_t keep = (M == 16) ? nm_keep_bits16(L, n_prune, lane) : nm_keep_bits<(M == 16 ? 8 : M)>(L, n_prune);
            if (apply && active) {
                w[j].apply(keep);
                w[j].store_vec_nt(own.W, row * own.ldw + q0);
            }
            if (!active) keep = 0u;
            const uint32_t word = quad_gather_bytes(keep, lane);
            if ((lane & 3) == 0 && active) own.keep_mask[row * mask_words + (q0 >> 5)] = word;
        }
    };
    // two batches alternate: while one is worked on, the loads of the next are in flight
    // (row numbers stay below 2^31 - step: the launcher refuses larger groups)
    Chunk8<DT> a[U], b[U];
    int32_t r0 = (int32_t)(blockIdx.y * U);
    fetch(a, r0);
    while (r0 < out) {
        fetch(b, r0 + step);
        work(a, r0);
        r0 += step;
        if (r0 >= out) break;
        fetch(a, r0 + step);
        work(b, r0);
        r0 += step;
    }
}

template <int DT, int U>
__global__ __launch_bounds__(kColThreads) void apply_band_kernel(void* __restrict__ W, int64_t out, int64_t in,
                                                                int64_t ldw,
                                                                const uint32_t* __restrict__ keep_mask,
                                                                int strip_units) {
    const int64_t unit = (int64_t)blockIdx.x * strip_units + threadIdx.x;
    const int64_t q0 = unit * 8;
    if ((int)threadIdx.x >= strip_units || q0 >= in) return;
    const int64_t mask_words = (in + 31) >> 5;
    const int64_t step = (int64_t)gridDim.y * U;
    const int shift = (int)(q0 & 31);

    auto fetch = [&](Chunk8<DT>* w, uint32_t* keep, int64_t r0) {
#pragma unroll
        for (int j = 0; j < U; ++j) {
            if (r0 + j < out) {
                w[j].load_vec(W, (r0 + j) * ldw + q0);
                keep[j] = keep_mask[(r0 + j) * mask_words + (q0 >> 5)];
            }
        }
    };
    auto work = [&](Chunk8<DT>* w, uint32_t* keep, int64_t r0) {
#pragma unroll
        for (int j = 0; j < U; ++j) {
            if (r0 + j < out) {
                w[j].apply((keep[j] >> shift) & 0xffu);
                w[j].store_vec_nt(W, (r0 + j) * ldw + q0);
            }
        }
    };
    Chunk8<DT> a[U], b[U];
    uint32_t ka[U], kb[U];
    int64_t r0 = (int64_t)blockIdx.y * U;
    fetch(a, ka, r0);
    while (r0 < out) {
        fetch(b, kb, r0 + step);
        work(a, ka, r0);
        r0 += step;
        if (r0 >= out) break;
        fetch(a, ka, r0 + step);
        work(b, kb, r0);
        r0 += step;
    }
}

// Workgroups of a band launch, from sweeps on MI355X (bf16, 1024 ... 14336 rows x 4096 ... 14336 columns):
// the plain apply stream is best with two workgroups per compute unit, the selection kernels, which do
// ~100 VALU instructions per 16-byte load, need three to hide them.  Four rows per batch, two batches alternating.
constexpr int kApplyBandGroups = 512;
constexpr int kSelectBandGroups = 768;

template <int DT, int M, bool GROUPED>
static hipError_t launch_nm_band_t(const RowGroups& g, int64_t in, const float* hr, int n_prune, float* scores,
                                   int apply, int target_groups, hipStream_t stream, int unroll) {
    const BandPlan p = make_band_plan(g.total(), in, target_groups, unroll);
    const dim3 grid((unsigned)p.nstrips, (unsigned)p.splits), block(kColThreads);
    switch (p.unroll) {
        case 4: hipLaunchKernelGGL((nm_select_band_kernel<DT, M, 4, GROUPED>), grid, block, 0, stream, g, in, hr, n_prune, scores, apply, p.strip_units); break;
        case 2: hipLaunchKernelGGL((nm_select_band_kernel<DT, M, 2, GROUPED>), grid, block, 0, stream, g, in, hr, n_prune, scores, apply, p.strip_units); break;
        default: hipLaunchKernelGGL((nm_select_band_kernel<DT, M, 1, GROUPED>), grid, block, 0, stream, g, in, hr, n_prune, scores, apply, p.strip_units); break;
    }
    return hipGetLastError();
}

template <int DT, int M>
static hipError_t launch_nm_band(const RowGroups& g, int64_t in, const float* hr, int n_prune, float* scores,
                                 int apply, int target_groups, hipStream_t stream, int unroll = 4) {
    return g.n > 1 ? launch_nm_band_t<DT, M, true>(g, in, hr, n_prune, scores, apply, target_groups, stream, unroll)
                   : launch_nm_band_t<DT, M, false>(g, in, hr, n_prune, scores, apply, target_groups, stream, unroll);
}

template <int DT>
static hipError_t launch_apply_band(void* W, int64_t out, int64_t in, int64_t ldw, const uint32_t* keep_mask,
                                    int target_groups, hipStream_t stream, int unroll = 4) {
    const BandPlan p = make_band_plan(out, in, target_groups, unroll);
    const dim3 grid((unsigned)p.nstrips, (unsigned)p.splits), block(kColThreads);
    switch (p.unroll) {
        case 4: hipLaunchKernelGGL((apply_band_kernel<DT, 4>), grid, block, 0, stream, W, out, in, ldw, keep_mask, p.strip_units); break;
        case 2: hipLaunchKernelGGL((apply_band_kernel<DT, 2>), grid, block, 0, stream, W, out, in, ldw, keep_mask, p.strip_units); break;
        default: hipLaunchKernelGGL((apply_band_kernel<DT, 1>), grid, block, 0, stream, W, out, in, ldw, keep_mask, p.strip_units); break;
    }
    return hipGetLastError();
}

template <int DT>
static hipError_t launch_nm_t(const void* W, int64_t out, int64_t in, int64_t ldw, const float* hr,
                              int n_keep, int m_group, uint32_t* keep_mask, float* scores, bool apply,
                              hipStream_t stream) {
    const int64_t chunks = (in + 7) / 8;
    const unsigned col_tiles = (unsigned)((chunks + kWave - 1) / kWave);
    const int64_t tiles = (int64_t)col_tiles * ((out + kRows - 1) / kRows);
    const int64_t groups = (tiles + kColThreads / kWave - 1) / (kColThreads / kWave);
    if (groups > 0x7fffffff) return hipErrorInvalidValue;
    dim3 grid((unsigned)groups);
    void* Wm = const_cast<void*>(W);
    const int n_prune = m_group - n_keep;
    const int ap = apply ? 1 : 0;
    switch (m_group) {
        case 4:
            hipLaunchKernelGGL((nm_select_kernel<DT, 4>), grid, dim3(kColThreads), 0, stream, Wm, out, in,
                               ldw, hr, n_prune, keep_mask, scores, ap, col_tiles);
            break;
        case 8:
            hipLaunchKernelGGL((nm_select_kernel<DT, 8>), grid, dim3(kColThreads), 0, stream, Wm, out, in,
                               ldw, hr, n_prune, keep_mask, scores, ap, col_tiles);
            break;
        case 16:
            hipLaunchKernelGGL((nm_select_kernel<DT, 16>), grid, dim3(kColThreads), 0, stream, Wm, out, in,
                               ldw, hr, n_prune, keep_mask, scores, ap, col_tiles);
            break;
        default:
            return hipErrorInvalidValue;
    }
    return hipGetLastError();
}

hipError_t launch_nm_select(const void* W, int64_t out, int64_t in, int64_t ldw, int dt, bool vec,
                            const float* hr, int n_keep, int m_group, uint32_t* keep_mask,
                            float* scores, bool apply, hipStream_t stream) {
    return with_dtype(dt, [&](auto tag) {
        constexpr int DT = decltype(tag)::value;
        if (vec)
            return launch_nm_select_group(single_matrix(W, out, ldw, keep_mask, nullptr), in, DT, hr, n_keep, m_group,
                                          scores, apply, stream);
        return launch_nm_t<DT>(W, out, in, ldw, hr, n_keep, m_group, keep_mask, scores, apply, stream);
    });
}

hipError_t launch_nm_select_group(const RowGroups& g, int64_t in, int dt, const float* hr, int n_keep,
                                  int m_group, float* scores, bool apply, hipStream_t stream) {
    const int n_prune = m_group - n_keep, ap = apply ? 1 : 0;
    const Tuning t = read_tuning();
    const int groups = t.select_groups != 0 ? t.select_groups : kSelectBandGroups;  // measurement override
    return with_dtype(dt, [&](auto tag) {
        constexpr int DT = decltype(tag)::value;
        switch (m_group) {
            case 4: return launch_nm_band<DT, 4>(g, in, hr, n_prune, scores, ap, groups, stream);
            case 8: return launch_nm_band<DT, 8>(g, in, hr, n_prune, scores, ap, groups, stream);
            case 16: return launch_nm_band<DT, 16>(g, in, hr, n_prune, scores, ap, groups, stream);
            default: return hipErrorInvalidValue;
        }
    });
}

hipError_t launch_apply(void* W, int64_t out, int64_t in, int64_t ldw, int dt, bool vec,
                        const uint32_t* keep_mask, hipStream_t stream) {
    const int64_t chunks = (in + 7) / 8;
    const unsigned col_tiles = (unsigned)((chunks + kWave - 1) / kWave);
    const int64_t tiles = (int64_t)col_tiles * ((out + kRows - 1) / kRows);
    const int64_t groups = (tiles + kColThreads / kWave - 1) / (kColThreads / kWave);
    if (!vec && groups > 0x7fffffff) return hipErrorInvalidValue;
    dim3 grid((unsigned)groups);
    return with_dtype(dt, [&](auto tag) {
        constexpr int DT = decltype(tag)::value;
        if (vec) {
            const Tuning t = read_tuning();  // measurement override
            return launch_apply_band<DT>(W, out, in, ldw, keep_mask, t.apply_groups != 0 ? t.apply_groups : kApplyBandGroups, stream);
        }
        hipLaunchKernelGGL((apply_kernel<DT>), grid, dim3(kColThreads), 0, stream, W, out, in, ldw, keep_mask, col_tiles);
        return hipGetLastError();
    });
}

}  // namespace sp

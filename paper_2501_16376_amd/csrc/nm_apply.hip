// N:M structured selection (Sec. 3.3) fused with the score (Sec. 3.1), and the
// in-place apply step (Algorithm 1: pruned w_i = 0).
//
// Both are plain streaming kernels.  A lane owns one chunk of 8 consecutive
// columns (one 16-byte load of bf16) and walks kRows rows with it, so the
// channel factors of its columns are loaded once and kRows independent loads
// are in flight.  N:M ranks are computed in registers by counting, with ties
// broken towards the lower index: rank_i = #{p : (L_p, p) < (L_i, i)}, and
// entry i is pruned iff rank_i < M - N.  Groups of 4 and 8 live inside one
// lane; a group of 16 spans two neighbouring lanes and exchanges its scores
// with one DPP quad permute per value.
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
template <int DT, bool VEC, int M>
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
    if (VEC) { if (valid) f.load_vec(hr, q0); else f.load_elems(hr, q0, 0); }
    else f.load_elems(hr, q0, valid);

    Chunk8<DT> w[kRows];
#pragma unroll
    for (int r = 0; r < kRows; ++r) {
        w[r].zero();
        if (r < nrows && valid) {
            if (VEC) w[r].load_vec(W, (row0 + r) * ldw + q0);
            else w[r].load_elems(W, (row0 + r) * ldw + q0, valid);
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
        if (scores != nullptr && valid) store8(scores + row * in + q0, L, VEC, valid);
        const uint32_t word = quad_gather_bytes(keep, lane);
        const int64_t widx = q0 >> 5;
        if ((lane & 3) == 0 && widx < mask_words) keep_mask[row * mask_words + widx] = word;
        if (apply && valid) {
            w[r].apply(keep);
            if (VEC) w[r].store_vec_nt(W, row * ldw + q0);
            else w[r].store_elems(W, row * ldw + q0, valid);
        }
    }
}

// grid / block as above
template <int DT, bool VEC>
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
            if (VEC) w[r].load_vec(W, (row0 + r) * ldw + q0);
            else w[r].load_elems(W, (row0 + r) * ldw + q0, valid);
            keep[r] = (keep_mask[(row0 + r) * mask_words + (q0 >> 5)] >> shift) & 0xffu;
        }
    }
#pragma unroll
    for (int r = 0; r < kRows; ++r) {
        if (r < nrows) {
            w[r].apply(keep[r]);
            if (VEC) w[r].store_vec_nt(W, (row0 + r) * ldw + q0);
            else w[r].store_elems(W, (row0 + r) * ldw + q0, valid);
        }
    }
}

template <int DT, bool VEC>
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
            hipLaunchKernelGGL((nm_select_kernel<DT, VEC, 4>), grid, dim3(kColThreads), 0, stream, Wm, out, in,
                               ldw, hr, n_prune, keep_mask, scores, ap, col_tiles);
            break;
        case 8:
            hipLaunchKernelGGL((nm_select_kernel<DT, VEC, 8>), grid, dim3(kColThreads), 0, stream, Wm, out, in,
                               ldw, hr, n_prune, keep_mask, scores, ap, col_tiles);
            break;
        case 16:
            hipLaunchKernelGGL((nm_select_kernel<DT, VEC, 16>), grid, dim3(kColThreads), 0, stream, Wm, out, in,
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
        return vec ? launch_nm_t<DT, true>(W, out, in, ldw, hr, n_keep, m_group, keep_mask, scores, apply, stream)
                   : launch_nm_t<DT, false>(W, out, in, ldw, hr, n_keep, m_group, keep_mask, scores, apply, stream);
    });
}

hipError_t launch_apply(void* W, int64_t out, int64_t in, int64_t ldw, int dt, bool vec,
                        const uint32_t* keep_mask, hipStream_t stream) {
    const int64_t chunks = (in + 7) / 8;
    const unsigned col_tiles = (unsigned)((chunks + kWave - 1) / kWave);
    const int64_t tiles = (int64_t)col_tiles * ((out + kRows - 1) / kRows);
    const int64_t groups = (tiles + kColThreads / kWave - 1) / (kColThreads / kWave);
    if (groups > 0x7fffffff) return hipErrorInvalidValue;
    dim3 grid((unsigned)groups);
    return with_dtype(dt, [&](auto tag) {
        constexpr int DT = decltype(tag)::value;
        if (vec) hipLaunchKernelGGL((apply_kernel<DT, true>), grid, dim3(kColThreads), 0, stream, W, out, in, ldw, keep_mask, col_tiles);
        else hipLaunchKernelGGL((apply_kernel<DT, false>), grid, dim3(kColThreads), 0, stream, W, out, in, ldw, keep_mask, col_tiles);
        return hipGetLastError();
    });
}

}  // namespace sp

// Compact storage of an N:M-pruned matrix and its inverse.  Sec. 3.3 motivates N:M
// sparsity by hardware formats that hold only the kept values and their
// positions; this is an open layout of that kind (not a vendor format):
//   values[r, g*N + j] = j-th kept entry (ascending column) of group g of row r
//   meta               = position (0..M-1) of that entry inside its group, a field
//                        of b bits (b = 2 for M = 4, else 4), field number g*N + j
//                        of the row, packed little-endian into uint32 words.
// One lane handles 32 groups (32*M columns = M mask words) of a row, so the meta
// bits it produces are a whole number of words (32*N*b bits) and no two lanes
// share a word.
#include "common.hpp"
#include "kernels.hpp"

namespace sp {

__host__ __device__ inline int nm_index_bits(int m_group) { return m_group == 4 ? 2 : 4; }

template <int DT>
__device__ __forceinline__ uint32_t load_raw(const void* p, int64_t idx) {
    if (DT != kF32) return static_cast<const uint16_t*>(p)[idx];   // bf16 and fp16: 16-bit storage
    return static_cast<const uint32_t*>(p)[idx];
}
template <int DT>
__device__ __forceinline__ void store_raw(void* p, int64_t idx, uint32_t v) {
    if (DT != kF32) static_cast<uint16_t*>(p)[idx] = (uint16_t)v;
    else static_cast<uint32_t*>(p)[idx] = v;
}

// grid = ceil(chunks / 64) * out (one dimension, chunk block fastest), block = 64; chunk = 32 groups
template <int DT>
__global__ __launch_bounds__(64) void compact_nm_kernel(const void* __restrict__ W, int64_t in, int64_t ldw,
                                                        const uint32_t* __restrict__ keep_mask, int n_keep,
                                                        int m_group, void* __restrict__ values,
                                                        uint32_t* __restrict__ meta, int64_t meta_words,
                                                        unsigned chunk_blocks) {
    const int64_t row = blockIdx.x / chunk_blocks;
    const int64_t chunk = (int64_t)(blockIdx.x % chunk_blocks) * 64 + threadIdx.x;
    const int64_t groups = in / m_group;
    const int64_t g0 = chunk * 32;
    if (g0 >= groups) return;
    const int64_t g1 = min(groups, g0 + 32);
    const int b = nm_index_bits(m_group);
    const int64_t mask_words = (in + 31) >> 5;
    const int64_t per_row = groups * n_keep;

    int64_t f = g0 * n_keep;                 // next field (kept-value slot) of the row
    int64_t cur_word = (f * b) >> 5;         // meta word being assembled
    uint32_t acc = 0u;
    for (int64_t g = g0; g < g1; ++g) {
        int j = 0;
        for (int i = 0; i < m_group; ++i) {
            const int64_t q = g * m_group + i;
            const bool keep = (keep_mask[row * mask_words + (q >> 5)] >> (q & 31)) & 1u;
            if (!keep || j >= n_keep) continue;
            store_raw<DT>(values, row * per_row + f, load_raw<DT>(W, row * ldw + q));
            const int64_t bit = f * b;
            if ((bit >> 5) != cur_word) {
                meta[row * meta_words + cur_word] = acc;
                acc = 0u;
                cur_word = bit >> 5;
            }
            acc |= (uint32_t)i << (bit & 31);
            ++f;
            ++j;
        }
        for (; j < n_keep; ++j) {            // fewer kept entries than N: pad with +0 at position 0
            store_raw<DT>(values, row * per_row + f, 0u);
            const int64_t bit = f * b;
            if ((bit >> 5) != cur_word) {
                meta[row * meta_words + cur_word] = acc;
                acc = 0u;
                cur_word = bit >> 5;
            }
            ++f;
        }
    }
    if (cur_word < meta_words) meta[row * meta_words + cur_word] = acc;
}

// grid / block as above: the lane zero-fills its 32*M dense columns, then places its stored values
template <int DT>
__global__ __launch_bounds__(64) void expand_nm_kernel(const void* __restrict__ values,
                                                       const uint32_t* __restrict__ meta, int64_t in,
                                                       int n_keep, int m_group, int64_t meta_words,
                                                       void* __restrict__ W_out, int64_t ldw,
                                                       unsigned chunk_blocks) {
    const int64_t row = blockIdx.x / chunk_blocks;
    const int64_t chunk = (int64_t)(blockIdx.x % chunk_blocks) * 64 + threadIdx.x;
    const int64_t groups = in / m_group;
    const int64_t g0 = chunk * 32;
    if (g0 >= groups) return;
    const int64_t g1 = min(groups, g0 + 32);
    const int b = nm_index_bits(m_group);
    const int64_t per_row = groups * n_keep;
    for (int64_t q = g0 * m_group; q < g1 * m_group; ++q) store_raw<DT>(W_out, row * ldw + q, 0u);
    for (int64_t f = g0 * n_keep; f < g1 * n_keep; ++f) {
        const uint32_t v = load_raw<DT>(values, row * per_row + f);
        if (v == 0u) continue;               // +0 (stored or padding) is already there
        const int64_t bit = f * b;
        const uint32_t pos = (meta[row * meta_words + (bit >> 5)] >> (bit & 31)) & ((1u << b) - 1u);
        store_raw<DT>(W_out, row * ldw + f / n_keep * m_group + pos, v);
    }
}

int64_t nm_meta_words(int64_t in, int n_keep, int m_group) {
    return (in / m_group * n_keep * nm_index_bits(m_group) + 31) / 32;
}

hipError_t launch_compact_nm(const void* W, int64_t out, int64_t in, int64_t ldw, int dt,
                             const uint32_t* keep_mask, int n_keep, int m_group, void* values,
                             uint32_t* meta, hipStream_t stream) {
    const int64_t chunks = (in / m_group + 31) / 32;
    const unsigned chunk_blocks = (unsigned)((chunks + 63) / 64);
    if ((int64_t)chunk_blocks * out > 0x7fffffff) return hipErrorInvalidValue;
    dim3 grid((unsigned)(chunk_blocks * out));
    const int64_t mw = nm_meta_words(in, n_keep, m_group);
    return with_dtype(dt, [&](auto tag) {
        constexpr int DT = decltype(tag)::value;
        hipLaunchKernelGGL(compact_nm_kernel<DT>, grid, dim3(64), 0, stream, W, in, ldw, keep_mask, n_keep, m_group,
                           values, meta, mw, chunk_blocks);
        return hipGetLastError();
    });
}

hipError_t launch_expand_nm(const void* values, const uint32_t* meta, int64_t out, int64_t in, int dt,
                            int n_keep, int m_group, void* W_out, int64_t ldw, hipStream_t stream) {
    const int64_t chunks = (in / m_group + 31) / 32;
    const unsigned chunk_blocks = (unsigned)((chunks + 63) / 64);
    if ((int64_t)chunk_blocks * out > 0x7fffffff) return hipErrorInvalidValue;
    dim3 grid((unsigned)(chunk_blocks * out));
    const int64_t mw = nm_meta_words(in, n_keep, m_group);
    return with_dtype(dt, [&](auto tag) {
        constexpr int DT = decltype(tag)::value;
        hipLaunchKernelGGL(expand_nm_kernel<DT>, grid, dim3(64), 0, stream, values, meta, in, n_keep, m_group, mw,
                           W_out, ldw, chunk_blocks);
        return hipGetLastError();
    });
}

}  // namespace sp

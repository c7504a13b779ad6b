// Device helpers shared by the SwiftPrune kernels (gfx950, wave64).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include <type_traits>

namespace sp {

typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

constexpr int kWave = 64;
constexpr int kF32 = 0;
constexpr int kBF16 = 1;
constexpr int kF16 = 2;   // IEEE binary16

// ---- bf16 -> fp32 (bf16 is the upper half of an IEEE binary32) ----
__device__ __forceinline__ float bf16lo(uint32_t pair) { return __uint_as_float(pair << 16); }
__device__ __forceinline__ float bf16hi(uint32_t pair) { return __uint_as_float(pair & 0xffff0000u); }
// ---- binary16 -> fp32 (exact; one conversion instruction, subnormals included) ----
__device__ __forceinline__ float f16bits(uint16_t h) { return (float)__builtin_bit_cast(_Float16, h); }
__device__ __forceinline__ float f16lo(uint32_t pair) { return f16bits((uint16_t)(pair & 0xffffu)); }
__device__ __forceinline__ float f16hi(uint32_t pair) { return f16bits((uint16_t)(pair >> 16)); }

// Host side: calls f(std::integral_constant<int, DT>{}) with the storage type as a compile-time constant.
template <class F>
inline hipError_t with_dtype(int dt, F&& f) {
    switch (dt) {
        case kF32: return f(std::integral_constant<int, kF32>{});
        case kBF16: return f(std::integral_constant<int, kBF16>{});
        case kF16: return f(std::integral_constant<int, kF16>{});
        default: return hipErrorInvalidValue;
    }
}

// One stored element as fp32 / set to +0 (element-wise paths).
template <int DT>
__device__ __forceinline__ float load_scalar(const void* p, int64_t idx) {
    if (DT == kBF16) return __uint_as_float((uint32_t)static_cast<const uint16_t*>(p)[idx] << 16);
    if (DT == kF16) return f16bits(static_cast<const uint16_t*>(p)[idx]);
    return static_cast<const float*>(p)[idx];
}
template <int DT>
__device__ __forceinline__ void store_zero(void* p, int64_t idx) {
    if (DT == kF32) static_cast<float*>(p)[idx] = 0.0f;
    else static_cast<uint16_t*>(p)[idx] = 0;
}

// ---- DPP moves; lanes without a valid source (or masked off) receive 0 ----
template <int CTRL, int ROW_MASK = 0xf>
__device__ __forceinline__ float dpp_f(float v) {
    return __int_as_float(
        __builtin_amdgcn_update_dpp(0, __float_as_int(v), CTRL, ROW_MASK, 0xf, false));
}
template <int CTRL>
__device__ __forceinline__ uint32_t dpp_u(uint32_t v) {
    return (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, CTRL, 0xf, 0xf, false);
}
constexpr int kRowShr1 = 0x111, kRowShr2 = 0x112, kRowShr4 = 0x114, kRowShr8 = 0x118;
constexpr int kWaveShr1 = 0x138;
constexpr int kRowBcast15 = 0x142, kRowBcast31 = 0x143;
constexpr int kQuadSwap1 = 0xB1;  // quad_perm [1,0,3,2]
constexpr int kQuadSwap2 = 0x4E;  // quad_perm [2,3,0,1]

__device__ __forceinline__ float readlane_f(float v, int lane) {
    return __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), lane));
}

// OR the per-lane bytes of the four lanes of a quad into one word:
// lane (4k + j) contributes bits [8j, 8j+8).  Every lane of the quad gets the word.
__device__ __forceinline__ uint32_t quad_gather_bytes(uint32_t byte, int lane) {
    uint32_t v = byte << (8 * (lane & 3));
    v |= dpp_u<kQuadSwap1>(v);
    v |= dpp_u<kQuadSwap2>(v);
    return v;
}

// Eight consecutive elements of a row as fp32 plus their raw storage.
template <int DT>
struct Chunk8;

// storage side of the two 16-bit types: four 32-bit words holding eight elements
struct Chunk8Halves {
    uint32_t raw[4];
    // 16-byte aligned vector load; weights are streamed once, so the load is non-temporal
    __device__ __forceinline__ void load_vec(const void* base, int64_t elem_off) {
        const u32x4 v = __builtin_nontemporal_load(
            reinterpret_cast<const u32x4*>(static_cast<const uint16_t*>(base) + elem_off));
        raw[0] = v.x; raw[1] = v.y; raw[2] = v.z; raw[3] = v.w;
    }
    // element-wise load of the first `valid` elements, the rest read as +0
    __device__ __forceinline__ void load_elems(const void* base, int64_t elem_off, int valid) {
        const uint16_t* p = static_cast<const uint16_t*>(base) + elem_off;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            uint32_t lo = (2 * j < valid) ? p[2 * j] : 0u;
            uint32_t hi = (2 * j + 1 < valid) ? p[2 * j + 1] : 0u;
            raw[j] = lo | (hi << 16);
        }
    }
    __device__ __forceinline__ void zero() { raw[0] = raw[1] = raw[2] = raw[3] = 0u; }
    // zero the elements whose keep bit is 0
    __device__ __forceinline__ void apply(uint32_t keep_byte) {
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            uint32_t m = ((keep_byte >> (2 * j)) & 1u ? 0x0000ffffu : 0u) |
                         ((keep_byte >> (2 * j + 1)) & 1u ? 0xffff0000u : 0u);
            raw[j] &= m;
        }
    }
    // zero the elements whose flag is set (two selects per 32-bit pair)
    __device__ __forceinline__ void apply_flags(const bool* prune) {
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const uint32_t lo_gone = prune[2 * j] ? (raw[j] & 0xffff0000u) : raw[j];
            raw[j] = prune[2 * j + 1] ? (lo_gone & 0x0000ffffu) : lo_gone;
        }
    }
    __device__ __forceinline__ void store_vec(void* base, int64_t elem_off) const {
        *reinterpret_cast<uint4*>(static_cast<uint16_t*>(base) + elem_off) =
            make_uint4(raw[0], raw[1], raw[2], raw[3]);
    }
    // non-temporal variant: measured 3-7 % faster in the pure streaming kernels (apply, N:M), not in the scan
    __device__ __forceinline__ void store_vec_nt(void* base, int64_t elem_off) const {
        u32x4 v;
        v.x = raw[0]; v.y = raw[1]; v.z = raw[2]; v.w = raw[3];
        __builtin_nontemporal_store(v, reinterpret_cast<u32x4*>(static_cast<uint16_t*>(base) + elem_off));
    }
    __device__ __forceinline__ void store_elems(void* base, int64_t elem_off, int valid) const {
        uint16_t* p = static_cast<uint16_t*>(base) + elem_off;
#pragma unroll
        for (int k = 0; k < 8; ++k)
            if (k < valid) p[k] = (uint16_t)((k & 1) ? (raw[k >> 1] >> 16) : (raw[k >> 1] & 0xffffu));
    }
};

template <>
struct Chunk8<kBF16> : Chunk8Halves {
    __device__ __forceinline__ float get(int k) const {
        return (k & 1) ? bf16hi(raw[k >> 1]) : bf16lo(raw[k >> 1]);
    }
};

template <>
struct Chunk8<kF16> : Chunk8Halves {
    __device__ __forceinline__ float get(int k) const {
        return (k & 1) ? f16hi(raw[k >> 1]) : f16lo(raw[k >> 1]);
    }
};

template <>
struct Chunk8<kF32> {
    uint32_t raw[8];
    __device__ __forceinline__ void load_vec(const void* base, int64_t elem_off) {
        const u32x4* p = reinterpret_cast<const u32x4*>(static_cast<const float*>(base) + elem_off);
        const u32x4 a = __builtin_nontemporal_load(p), b = __builtin_nontemporal_load(p + 1);
        raw[0] = a.x; raw[1] = a.y; raw[2] = a.z; raw[3] = a.w;
        raw[4] = b.x; raw[5] = b.y; raw[6] = b.z; raw[7] = b.w;
    }
    __device__ __forceinline__ void load_elems(const void* base, int64_t elem_off, int valid) {
        const uint32_t* p = static_cast<const uint32_t*>(base) + elem_off;
#pragma unroll
        for (int k = 0; k < 8; ++k) raw[k] = (k < valid) ? p[k] : 0u;
    }
    __device__ __forceinline__ void zero() {
#pragma unroll
        for (int k = 0; k < 8; ++k) raw[k] = 0u;
    }
    __device__ __forceinline__ float get(int k) const { return __uint_as_float(raw[k]); }
    __device__ __forceinline__ void apply(uint32_t keep_byte) {
#pragma unroll
        for (int k = 0; k < 8; ++k)
            if (!((keep_byte >> k) & 1u)) raw[k] = 0u;
    }
    __device__ __forceinline__ void apply_flags(const bool* prune) {
#pragma unroll
        for (int k = 0; k < 8; ++k) raw[k] = prune[k] ? 0u : raw[k];
    }
    __device__ __forceinline__ void store_vec(void* base, int64_t elem_off) const {
        uint4* p = reinterpret_cast<uint4*>(static_cast<float*>(base) + elem_off);
        p[0] = make_uint4(raw[0], raw[1], raw[2], raw[3]);
        p[1] = make_uint4(raw[4], raw[5], raw[6], raw[7]);
    }
    __device__ __forceinline__ void store_vec_nt(void* base, int64_t elem_off) const {
        u32x4* p = reinterpret_cast<u32x4*>(static_cast<float*>(base) + elem_off);
        u32x4 a, b;
        a.x = raw[0]; a.y = raw[1]; a.z = raw[2]; a.w = raw[3];
        b.x = raw[4]; b.y = raw[5]; b.z = raw[6]; b.w = raw[7];
        __builtin_nontemporal_store(a, p);
        __builtin_nontemporal_store(b, p + 1);
    }
    __device__ __forceinline__ void store_elems(void* base, int64_t elem_off, int valid) const {
        uint32_t* p = static_cast<uint32_t*>(base) + elem_off;
#pragma unroll
        for (int k = 0; k < 8; ++k)
            if (k < valid) p[k] = raw[k];
    }
};

// Eight consecutive per-channel factors.
struct Factor8 {
    float v[8];
    __device__ __forceinline__ void load_vec(const float* hr, int64_t q) {
        const float4 a = *reinterpret_cast<const float4*>(hr + q);
        const float4 b = *reinterpret_cast<const float4*>(hr + q + 4);
        v[0] = a.x; v[1] = a.y; v[2] = a.z; v[3] = a.w;
        v[4] = b.x; v[5] = b.y; v[6] = b.z; v[7] = b.w;
    }
    __device__ __forceinline__ void load_elems(const float* hr, int64_t q, int valid) {
#pragma unroll
        for (int k = 0; k < 8; ++k) v[k] = (k < valid) ? hr[q + k] : 0.0f;
    }
};

// Contribution score of a weight: (w*w) rounded, times the channel factor, rounded.
// Written as two separate multiplications so that no contraction can change it.
__device__ __forceinline__ float score_of(float w, float factor) {
    const float w2 = __fmul_rn(w, w);
    return __fmul_rn(w2, factor);
}

// Packs eight per-lane decisions, given as lane masks (bit `lane` of m[k] = decision k of that lane), into
// bits 0..7 of every lane (bit k = decision k) with one add-with-carry each: acc <- 2 acc + decision k,
// k = 7 .. 0, the lane mask entering as the carry.
__device__ __forceinline__ uint32_t pack_masks8(const uint64_t* m) {
    uint32_t acc = 0u;
    const uint64_t b0 = m[0], b1 = m[1], b2 = m[2], b3 = m[3], b4 = m[4], b5 = m[5], b6 = m[6], b7 = m[7];
    asm("v_addc_co_u32 %0, vcc, %0, %0, %8\n\t"
        "v_addc_co_u32 %0, vcc, %0, %0, %7\n\t"
        "v_addc_co_u32 %0, vcc, %0, %0, %6\n\t"
        "v_addc_co_u32 %0, vcc, %0, %0, %5\n\t"
        "v_addc_co_u32 %0, vcc, %0, %0, %4\n\t"
        "v_addc_co_u32 %0, vcc, %0, %0, %3\n\t"
        "v_addc_co_u32 %0, vcc, %0, %0, %2\n\t"
        "v_addc_co_u32 %0, vcc, %0, %0, %1"
        : "+v"(acc)
        : "s"(b0), "s"(b1), "s"(b2), "s"(b3), "s"(b4), "s"(b5), "s"(b6), "s"(b7)
        : "vcc");
    return acc;
}

// eight weights of a lane as fp32, kept unpacked until they are stored again
template <int DT>
struct Unpacked8 {
    float w[8];
    __device__ __forceinline__ void unpack(const Chunk8<DT>& c) {
#pragma unroll
        for (int k = 0; k < 8; ++k) w[k] = c.get(k);
    }
    // pruned entries (decisions given as lane masks) become +0: one select per weight that reads the mask from
    // scalar registers, with no second comparison; bf16 / fp16 pairs are re-packed with one byte permute each
    __device__ __forceinline__ void store_pruned_masks(void* W, int64_t elem, const uint64_t* gone) const {
        uint32_t z[8];
#pragma unroll
        for (int k = 0; k < 8; ++k)
            asm("v_cndmask_b32_e64 %0, %1, 0, %2" : "=v"(z[k]) : "v"(w[k]), "s"(gone[k]));
        store_words(W, elem, z);
    }
    __device__ __forceinline__ void store_words(void* W, int64_t elem, const uint32_t* z) const {
        if (DT == kF32) {
            u32x4* p = reinterpret_cast<u32x4*>(static_cast<float*>(W) + elem);
            u32x4 a, b;
            a.x = z[0]; a.y = z[1]; a.z = z[2]; a.w = z[3];
            b.x = z[4]; b.y = z[5]; b.z = z[6]; b.w = z[7];
            __builtin_nontemporal_store(a, p);
            __builtin_nontemporal_store(b, p + 1);
        } else {
            uint32_t pk[4];
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                if (DT == kBF16) {
                    // high halves of the two fp32 patterns: bytes 2,3 of z[2j] below bytes 2,3 of z[2j+1]
                    pk[j] = __builtin_amdgcn_perm(z[2 * j + 1], z[2 * j], 0x07060302u);
                } else {
                    const _Float16 lo = (_Float16)__uint_as_float(z[2 * j]);   // exact: the value came from binary16
                    const _Float16 hi = (_Float16)__uint_as_float(z[2 * j + 1]);
                    pk[j] = (uint32_t)__builtin_bit_cast(uint16_t, lo) | ((uint32_t)__builtin_bit_cast(uint16_t, hi) << 16);
                }
            }
            u32x4 v;
            v.x = pk[0]; v.y = pk[1]; v.z = pk[2]; v.w = pk[3];
            __builtin_nontemporal_store(v, reinterpret_cast<u32x4*>(static_cast<uint16_t*>(W) + elem));
        }
    }
};

// Which matrix of a group a consecutively numbered row belongs to, and its row number inside that matrix.
// The group description is a kernel argument, i.e. it sits in memory: the matrix index is found with a few
// compares and its entries are fetched by index (scalar loads when the row is wave-uniform).  Unused entries
// of row_end repeat the total, so a valid row never compares above them.  Row numbers are 32-bit: the scalar
// unit has no 64-bit ordered compare.
template <class Groups>
struct RowOwner {
    void* W;
    int64_t ldw, row;
    uint32_t* keep_mask;
    int32_t* row_pruned;
    int item;
    int32_t first, end;  // global numbers of the matrix's first row and of the row behind its last
    __device__ __forceinline__ RowOwner(const Groups& g, int32_t global_row) {
        item = 0;
#pragma unroll
        for (int j = 1; j < (int)(sizeof(g.row_end) / sizeof(g.row_end[0])); ++j)
            item += global_row >= g.row_end[j - 1] ? 1 : 0;
        first = item > 0 ? g.row_end[item - 1] : 0;
        bind(g, global_row);
    }
    // moves on to a later row (never back): one compare unless the row belongs to a later matrix
    __device__ __forceinline__ void seek(const Groups& g, int32_t global_row) {
        if (global_row >= end) {
            while (global_row >= g.row_end[item]) ++item;
            first = g.row_end[item - 1];
            bind(g, global_row);
        } else {
            row = (int64_t)(global_row - first);
        }
    }

  private:
    __device__ __forceinline__ void bind(const Groups& g, int32_t global_row) {
        end = g.row_end[item];
        W = g.W[item];
        ldw = g.ldw[item];
        keep_mask = g.keep_mask[item];
        row_pruned = g.row_pruned[item];
        row = (int64_t)(global_row - first);
    }
};

__device__ __forceinline__ void store8(float* dst, const float* v, bool vec, int valid) {
    if (vec) {
        reinterpret_cast<float4*>(dst)[0] = make_float4(v[0], v[1], v[2], v[3]);
        reinterpret_cast<float4*>(dst)[1] = make_float4(v[4], v[5], v[6], v[7]);
    } else {
#pragma unroll
        for (int k = 0; k < 8; ++k)
            if (k < valid) dst[k] = v[k];
    }
}

}  // namespace sp

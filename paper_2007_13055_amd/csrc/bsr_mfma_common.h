// Device-side building blocks shared by the matrix-core kernels: element and vector types, a
// lane's contiguous operand run (Frag), the MFMA step for every supported element type and tile
// edge, and the 4-wide store of a lane's results.
#pragma once

#include <type_traits>

#include "bsr_internal.h"

namespace bsr_dev {

typedef _Float16 f16_t;
typedef __bf16 bf16_t;
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef _Float16 f16x4 __attribute__((ext_vector_type(4)));
typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef short i16x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

template <typename O> __device__ __forceinline__ O from_f32(float v);
template <> __device__ __forceinline__ f16_t from_f32<f16_t>(float v) { return (f16_t)v; }     // nearest-even
template <> __device__ __forceinline__ bf16_t from_f32<bf16_t>(float v) { return (bf16_t)v; }   // nearest-even

// The lanes of one wavefront pass data to each other through LDS without a workgroup barrier: a wavefront's
// LDS operations complete in order, so no instruction is needed.  The compiler has to be told, though: it
// reasons about one lane, and may otherwise keep an operand it read before ("this lane stored nothing since")
// or move a read in front of the lane's own write to another address.  No instruction is emitted.
__device__ __forceinline__ void wave_lds_fence() { asm volatile("" ::: "memory"); }

// A lane's operand: CH contiguous elements of type T, kept as 32-bit words.
template <typename T, int CH>
struct Frag {
    static constexpr int BYTES = CH * (int)sizeof(T);
    static constexpr int WORDS = BYTES / 4;
    static_assert(BYTES % 8 == 0, "a lane's run must be a multiple of 8 bytes");
    uint32_t w[WORDS];

    __device__ __forceinline__ void load(const T* __restrict__ p)
    {
        if constexpr (BYTES % 16 == 0) {
            const u32x4* q = reinterpret_cast<const u32x4*>(p);
#pragma unroll
            for (int i = 0; i < BYTES / 16; ++i) {
                const u32x4 v = q[i];
                w[4 * i] = v.x; w[4 * i + 1] = v.y; w[4 * i + 2] = v.z; w[4 * i + 3] = v.w;
            }
        } else {
            const u32x2* q = reinterpret_cast<const u32x2*>(p);
#pragma unroll
            for (int i = 0; i < BYTES / 8; ++i) {
                const u32x2 v = q[i];
                w[2 * i] = v.x; w[2 * i + 1] = v.y;
            }
        }
    }
};

template <int MM> struct AccT { typedef f32x16 type; };
template <> struct AccT<16> { typedef f32x4 type; };

// acc += Wfrag (rows) x Xfrag (columns), all of the lane's CH elements.
template <typename T, int MM, int CH>
__device__ __forceinline__ void mfma_frag(typename AccT<MM>::type& acc, const Frag<T, CH>& a, const Frag<T, CH>& b)
{
    if constexpr (std::is_same<T, float>::value) {
#pragma unroll
        for (int s = 0; s < CH; ++s) {
            const float av = __builtin_bit_cast(float, a.w[s]);
            const float bv = __builtin_bit_cast(float, b.w[s]);
            if constexpr (MM == 32) acc = __builtin_amdgcn_mfma_f32_32x32x2f32(av, bv, acc, 0, 0, 0);
            else                    acc = __builtin_amdgcn_mfma_f32_16x16x4f32(av, bv, acc, 0, 0, 0);
        }
    } else if constexpr (CH % 8 == 0) {
#pragma unroll
        for (int s = 0; s < CH / 8; ++s) {
            const u32x4 ar = {a.w[4 * s], a.w[4 * s + 1], a.w[4 * s + 2], a.w[4 * s + 3]};
            const u32x4 br = {b.w[4 * s], b.w[4 * s + 1], b.w[4 * s + 2], b.w[4 * s + 3]};
            if constexpr (std::is_same<T, f16_t>::value) {
                const f16x8 av = __builtin_bit_cast(f16x8, ar), bv = __builtin_bit_cast(f16x8, br);
                if constexpr (MM == 32) acc = __builtin_amdgcn_mfma_f32_32x32x16_f16(av, bv, acc, 0, 0, 0);
                else                    acc = __builtin_amdgcn_mfma_f32_16x16x32_f16(av, bv, acc, 0, 0, 0);
            } else {
                const bf16x8 av = __builtin_bit_cast(bf16x8, ar), bv = __builtin_bit_cast(bf16x8, br);
                if constexpr (MM == 32) acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(av, bv, acc, 0, 0, 0);
                else                    acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(av, bv, acc, 0, 0, 0);
            }
        }
    } else {
        static_assert(std::is_same<T, float>::value || CH % 4 == 0, "16-bit runs come in multiples of 4");
#pragma unroll
        for (int s = 0; s < CH / 4; ++s) {
            const u32x2 ar = {a.w[2 * s], a.w[2 * s + 1]};
            const u32x2 br = {b.w[2 * s], b.w[2 * s + 1]};
            if constexpr (std::is_same<T, f16_t>::value) {
                const f16x4 av = __builtin_bit_cast(f16x4, ar), bv = __builtin_bit_cast(f16x4, br);
                if constexpr (MM == 32) acc = __builtin_amdgcn_mfma_f32_32x32x8f16(av, bv, acc, 0, 0, 0);
                else                    acc = __builtin_amdgcn_mfma_f32_16x16x16f16(av, bv, acc, 0, 0, 0);
            } else {
                const i16x4 av = __builtin_bit_cast(i16x4, ar), bv = __builtin_bit_cast(i16x4, br);
                if constexpr (MM == 32) acc = __builtin_amdgcn_mfma_f32_32x32x8bf16_1k(av, bv, acc, 0, 0, 0);
                else                    acc = __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(av, bv, acc, 0, 0, 0);
            }
        }
    }
}

// Store 4 consecutive columns of one row of Y (the 4 accumulator values a lane holds for 4
// consecutive rows of the MFMA result).
template <typename O>
__device__ __forceinline__ void store4(O* __restrict__ dst, float v0, float v1, float v2, float v3)
{
    if constexpr (std::is_same<O, float>::value) {
        const f32x4 v = {v0, v1, v2, v3};
        *reinterpret_cast<f32x4*>(dst) = v;
    } else {
        typedef O o4 __attribute__((ext_vector_type(4)));
        const o4 v = {from_f32<O>(v0), from_f32<O>(v1), from_f32<O>(v2), from_f32<O>(v3)};
        *reinterpret_cast<o4*>(dst) = v;
    }
}

// As store4, with the non-temporal hint: the line is not kept in L2 for re-use (Y is written once
// and never read by the kernel, so it should not push re-used X tiles out of the cache).
template <typename O>
__device__ __forceinline__ void store4_nt(O* __restrict__ dst, float v0, float v1, float v2, float v3)
{
    if constexpr (std::is_same<O, float>::value) {
        const f32x4 v = {v0, v1, v2, v3};
        __builtin_nontemporal_store(v, reinterpret_cast<f32x4*>(dst));
    } else {
        typedef O o4 __attribute__((ext_vector_type(4)));
        const o4 v = {from_f32<O>(v0), from_f32<O>(v1), from_f32<O>(v2), from_f32<O>(v3)};
        __builtin_nontemporal_store(v, reinterpret_cast<o4*>(dst));
    }
}

}  // namespace bsr_dev

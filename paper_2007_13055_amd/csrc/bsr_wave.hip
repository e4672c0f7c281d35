// Wavefront-reduction kernels for Y = X * W^T, W in BSR.
//
// Descendant of the paper's "parallelize within blocks" schedule (Section 4.4.2) and its
// cross-thread aggregation (Section 4.4.3): the lanes of one 64-wide wavefront split the
// reduction that produces an output element -- they stride through the consecutive elements of
// each stored block of the block-row, so the loads of W coalesce -- and the partial sums are
// added across lanes at the end.  Where the paper uses a shared-memory tree (or __shfl_down for
// 32 threads), a wave64 sums through DPP row operations and one ds_swizzle, without touching
// LDS memory.
#include "bsr_internal.h"

namespace {

typedef _Float16 f16_t;
typedef __bf16 bf16_t;

__device__ __forceinline__ float to_f32(float v) { return v; }
__device__ __forceinline__ float to_f32(f16_t v) { return (float)v; }
__device__ __forceinline__ float to_f32(bf16_t v) { return (float)v; }

template <typename O> __device__ __forceinline__ O from_f32(float v);
template <> __device__ __forceinline__ float from_f32<float>(float v) { return v; }
template <> __device__ __forceinline__ f16_t from_f32<f16_t>(float v) { return (f16_t)v; }     // nearest-even
template <> __device__ __forceinline__ bf16_t from_f32<bf16_t>(float v) { return (bf16_t)v; }   // nearest-even

template <int CTRL>
__device__ __forceinline__ float dpp_f32(float v)
{
    return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), CTRL, 0xF, 0xF, false));
}

// Sum of v over the 64 lanes; every lane returns the total.
// Steps 1-4 stay inside a DPP row of 16 lanes (quad swaps, half-row mirror, row mirror), step 5
// swaps the 16-lane halves of each 32 lanes through ds_swizzle, step 6 adds the two 32-lane
// halves through scalar lane reads.
__device__ __forceinline__ float wave_sum(float v)
{
    v += dpp_f32<0xB1>(v);    // quad_perm [1,0,3,2]
    v += dpp_f32<0x4E>(v);    // quad_perm [2,3,0,1]
    v += dpp_f32<0x141>(v);   // row_half_mirror
    v += dpp_f32<0x140>(v);   // row_mirror
    v += __builtin_bit_cast(float, __builtin_amdgcn_ds_swizzle(__builtin_bit_cast(int, v), 0x401F));  // lane ^ 16
    const float lo = __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, v), 0));
    const float hi = __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, v), 32));
    return lo + hi;
}

// One wavefront per output column j and per group of TM rows of X.
//   column j = r*bs_r + a; the lanes stride over e = (p - p0)*bs_c + c, i.e. over row a of every
//   stored block of block-row r in storage order; each lane keeps TM partial sums.
// Any block shape, any m.  A block-row without stored blocks leaves the partial sums at zero.
template <typename T, typename O, int TM>
__global__ __launch_bounds__(256) void bsr_wave_generic(const T* __restrict__ X, const T* __restrict__ data,
                                                        const int32_t* __restrict__ indices,
                                                        const int32_t* __restrict__ indptr, O* __restrict__ Y,
                                                        int m, int k, int n, int bs_r, int bs_c, int col_groups)
{
    const int lane = threadIdx.x & 63;
    const int wave = threadIdx.x >> 6;
    const int j = (int)(blockIdx.x % (unsigned)col_groups) * 4 + wave;
    const int i0 = (int)(blockIdx.x / (unsigned)col_groups) * TM;
    if (j >= n) return;                              // whole wave leaves together; no barrier in this kernel
    const int r = j / bs_r, a = j - r * bs_r;
    const int p0 = indptr[r], p1 = indptr[r + 1];
    const int len = (p1 - p0) * bs_c;

    const T* xrow[TM];
#pragma unroll
    for (int t = 0; t < TM; ++t) xrow[t] = X + (size_t)min(i0 + t, m - 1) * (size_t)k;   // clamp, masked at the store

    float acc[TM];
#pragma unroll
    for (int t = 0; t < TM; ++t) acc[t] = 0.f;

    for (int e = lane; e < len; e += 64) {
        const int q = e / bs_c, c = e - q * bs_c;
        const int p = p0 + q;
        const float w = to_f32(data[((size_t)p * bs_r + a) * bs_c + c]);
        const int col = indices[p] * bs_c + c;
#pragma unroll
        for (int t = 0; t < TM; ++t) acc[t] = fmaf(to_f32(xrow[t][col]), w, acc[t]);
    }
#pragma unroll
    for (int t = 0; t < TM; ++t) {
        const float s = wave_sum(acc[t]);
        if (lane == 0 && i0 + t < m) Y[(size_t)(i0 + t) * n + j] = from_f32<O>(s);
    }
}

template <typename T, typename O>
bsr_status launch_generic(const spmm_args& a)
{
    const bsr_matrix* W = a.W;
    const int m = (int)a.m, n = (int)W->n, k = (int)W->k;
    const int col_groups = (n + 3) / 4;
    auto go = [&](auto tm_tag) -> bsr_status {
        constexpr int TM = decltype(tm_tag)::value;
        const int64_t row_groups = (m + TM - 1) / TM;
        const int64_t blocks = row_groups * col_groups;
        if (blocks >= ((int64_t)1 << 31) || blocks * 256 >= ((int64_t)1 << 32)) return BSR_ERR_SHAPE;
        hipLaunchKernelGGL((bsr_wave_generic<T, O, TM>), dim3((unsigned)blocks), dim3(256), 0, a.stream,
                           (const T*)a.X, (const T*)W->data, W->indices, W->indptr, (O*)a.Y, m, k, n,
                           (int)W->bs_r, (int)W->bs_c, col_groups);
        return hipGetLastError() == hipSuccess ? BSR_OK : BSR_ERR_HIP;
    };
    if (m >= 8) return go(std::integral_constant<int, 8>{});
    if (m >= 4) return go(std::integral_constant<int, 4>{});
    if (m >= 2) return go(std::integral_constant<int, 2>{});
    return go(std::integral_constant<int, 1>{});
}

}  // namespace

bsr_status launch_wave(const spmm_args& a)
{
    const bsr_dtype in = a.W->dtype, out = a.y_dtype;
    if (in == BSR_F32) return launch_generic<float, float>(a);
    if (in == BSR_F16) return out == BSR_F32 ? launch_generic<f16_t, float>(a) : launch_generic<f16_t, f16_t>(a);
    if (in == BSR_BF16) return out == BSR_F32 ? launch_generic<bf16_t, float>(a) : launch_generic<bf16_t, bf16_t>(a);
    return BSR_ERR_DTYPE;
}

// Wavefront-reduction kernels for Y = X * W^T, W in BSR.
//
// Descendant of the paper's "parallelize within blocks" schedule (Section 4.4.2) and its
// cross-thread aggregation (Section 4.4.3): the lanes of one 64-wide wavefront split the
// reduction that produces an output element -- they stride through the consecutive elements of
// each stored block of the block-row, so the loads of W coalesce -- and the partial sums are
// added across lanes at the end.  Where the paper uses a shared-memory tree (or __shfl_down for
// 32 threads), a wave64 sums through DPP row operations and one ds_swizzle, without touching
// LDS memory.
#include <type_traits>

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

// One wavefront per output column and per group of TM rows of X.
//   The wavefront takes row a of the block-row in plan slot s (longest block-rows first): output
//   column j = r*bs_r + a.  The lanes stride over the elements (p - p0)*bs_c + c of row a of every
//   stored block of block-row r, in storage order and VEC consecutive elements at a time (one
//   16-byte load per lane for W and for each row of X when bs_c allows, else single elements); each
//   lane keeps TM partial sums.
//   The slot's row descriptor holds the block-row, its first block, its count and its first
//   block-columns, so the block-column of a lane's elements comes from the same 128 bytes as the
//   row bounds; longer block-rows read block_indices for the rest.
// Any block shape, any m.  A block-row without stored blocks leaves the partial sums at zero.
template <typename T, typename O, int TM, int VEC>
__global__ __launch_bounds__(256) void bsr_wave_generic(const T* __restrict__ X, const T* __restrict__ data,
                                                        const int32_t* __restrict__ indices,
                                                        const int32_t* __restrict__ row_desc, O* __restrict__ Y,
                                                        int m, int k, int n, int bs_r, int bs_c, int col_groups)
{
    struct alignas(sizeof(T) * VEC) vec_t { T v[VEC]; };
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int js = (int)(blockIdx.x % (unsigned)col_groups) * 4 + wave;     // slot*bs_r + a
    const int i0 = (int)(blockIdx.x / (unsigned)col_groups) * TM;
    if (js >= n) return;                             // whole wave leaves together; no barrier in this kernel
    const int slot = js / bs_r, a = js - slot * bs_r;
    const int32_t* __restrict__ desc = row_desc + (size_t)slot * kRowDescWords;
    const int r = desc[0], p0 = desc[1];
    const int vpr = bs_c / VEC;                      // VEC-element pieces per block row
    const int len = desc[2] * vpr;
    const int j = r * bs_r + a;

    const T* xrow[TM];
#pragma unroll
    for (int t = 0; t < TM; ++t) xrow[t] = X + (size_t)min(i0 + t, m - 1) * (size_t)k;   // clamp, masked at the store

    float acc[TM];
#pragma unroll
    for (int t = 0; t < TM; ++t) acc[t] = 0.f;

    for (int e = lane; e < len; e += 64) {
        const int q = e / vpr, c = (e - q * vpr) * VEC;
        const int p = p0 + q;
        const vec_t w = *reinterpret_cast<const vec_t*>(data + ((size_t)p * bs_r + a) * bs_c + c);
        const int col = (q < kRowDescCols ? desc[kRowDescColsAt + q] : indices[p]) * bs_c + c;
        vec_t x[TM];
#pragma unroll
        for (int t = 0; t < TM; ++t) x[t] = *reinterpret_cast<const vec_t*>(xrow[t] + col);
#pragma unroll
        for (int t = 0; t < TM; ++t)
#pragma unroll
            for (int v = 0; v < VEC; ++v) acc[t] = fmaf(to_f32(x[t].v[v]), to_f32(w.v[v]), acc[t]);
    }
#pragma unroll
    for (int t = 0; t < TM; ++t) {
        const float s = wave_sum(acc[t]);
        if (lane == 0 && i0 + t < m) Y[(size_t)(i0 + t) * n + j] = from_f32<O>(s);
    }
}

template <typename T, typename O>
bsr_status launch_generic(const spmm_args& a, const tune_opts& tune)
{
    const bsr_matrix* W = a.W;
    const int m = (int)a.m, n = (int)W->n, k = (int)W->k;
    const int col_groups = (n + 3) / 4;
    auto go = [&](auto tm_tag, auto vec_tag) -> bsr_status {
        constexpr int TM = decltype(tm_tag)::value, VEC = decltype(vec_tag)::value;
        const int64_t row_groups = (m + TM - 1) / TM;
        const int64_t blocks = row_groups * col_groups;
        if (blocks >= ((int64_t)1 << 31) || blocks * 256 >= ((int64_t)1 << 32)) return BSR_ERR_SHAPE;
        hipLaunchKernelGGL((bsr_wave_generic<T, O, TM, VEC>), dim3((unsigned)blocks), dim3(256), 0, a.stream,
                           (const T*)a.X, (const T*)W->data, W->indices, W->row_desc, (O*)a.Y, m, k, n,
                           (int)W->bs_r, (int)W->bs_c, col_groups);
        return hipGetLastError() == hipSuccess ? BSR_OK : BSR_ERR_HIP;
    };
    // 16-byte pieces when a block row is made of them (k is a multiple of bs_c and X, W are 16-byte
    // aligned, so every piece is aligned), single elements otherwise
    constexpr int V16 = 16 / (int)sizeof(T);
    // rows of X per wavefront: 8 amortise the reads of W best when there are many rows; up to m = 8
    // the wavefronts are few and short, and 4 rows each (twice the wavefronts) finish sooner
    const int rows = tune.mt > 0 ? tune.mt : (m > 8 ? 8 : (m >= 4 ? 4 : m));
    auto with_tm = [&](auto vec_tag) -> bsr_status {
        if (rows >= 8) return go(std::integral_constant<int, 8>{}, vec_tag);
        if (rows >= 4) return go(std::integral_constant<int, 4>{}, vec_tag);
        if (rows >= 2) return go(std::integral_constant<int, 2>{}, vec_tag);
        return go(std::integral_constant<int, 1>{}, vec_tag);
    };
    if (W->bs_c % V16 == 0) return with_tm(std::integral_constant<int, V16>{});
    return with_tm(std::integral_constant<int, 1>{});
}

}  // namespace

bsr_status launch_wave(const spmm_args& a, const tune_opts& t)
{
    const bsr_dtype in = a.W->dtype, out = a.y_dtype;
    if (in == BSR_F32) return launch_generic<float, float>(a, t);
    if (in == BSR_F16) return out == BSR_F32 ? launch_generic<f16_t, float>(a, t) : launch_generic<f16_t, f16_t>(a, t);
    if (in == BSR_BF16) return out == BSR_F32 ? launch_generic<bf16_t, float>(a, t) : launch_generic<bf16_t, bf16_t>(a, t);
    return BSR_ERR_DTYPE;
}

// Matrix-core (MFMA) kernels for Y = X * W^T, W in BSR, gfx950.
//
// Work unit: a wavefront owns a tile of Y that is one block-row of W wide (bs_r columns) and
// MT*MM rows of X tall, and walks the stored blocks of that block-row (Background: index_pointer
// gives the range, block_indices the block-column of each stored block).  This is the
// tile-per-thread-block design of the paper's "Utilizing shared memory" section, which the
// paper could not build because its compiler needed the cached extents at compile time; here
// the indices are read at run time and only the X columns of stored blocks are fetched.
//
// MFMA operand roles: the W block supplies the rows of the MFMA result (index a, the n side),
// the X tile supplies its columns (index i, the m side), so one lane ends up holding 4
// consecutive columns of Y for one row i, which are stored as one vector.  Both operands are
// read straight from their row-major storage: in both, the reduction index c is the contiguous
// one, so a lane's operand is a contiguous run of CH elements of a block row / an X row.  The
// lane groups split the bs_c columns of a block into 64/MM contiguous runs; W and X use the same
// split, so the sum over c is complete whatever order the instruction takes its k in.
#include <type_traits>

#include "bsr_internal.h"

namespace {

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

// Direct kernel: operands go from global memory (L1/L2) straight into registers.
//   MM   MFMA tile edge: 32 when bs_r >= 32, else 16          NA = BS_R / MM   result tiles along n
//   MT   result tiles along m per wavefront                    CH = BS_C / (64/MM) contiguous run per lane
// grid: blockIdx.x = slot + R * (m-tile); slot s works on block-row row_order[s] (longest first).
// No LDS and no barrier: wavefronts whose rows lie beyond m leave at once.
template <typename T, typename O, int BS_R, int BS_C, int MT>
__global__ __launch_bounds__(256) void bsr_mfma_direct(const T* __restrict__ X, const T* __restrict__ data,
                                                       const int32_t* __restrict__ indices,
                                                       const int32_t* __restrict__ indptr,
                                                       const int32_t* __restrict__ row_order, O* __restrict__ Y,
                                                       int m, int k, int n, int R)
{
    constexpr int MM = BS_R >= 32 ? 32 : 16;
    constexpr int NA = BS_R / MM;
    constexpr int G = 64 / MM;
    constexpr int CH = BS_C / G;
    typedef typename AccT<MM>::type acc_t;

    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, waves = blockDim.x >> 6;
    const int li = lane % MM, h = lane / MM;
    const int slot = (int)(blockIdx.x % (unsigned)R);
    const int tile = (int)(blockIdx.x / (unsigned)R);
    const int i_base = (tile * waves + wave) * (MT * MM);
    if (i_base >= m) return;
    const int r = row_order[slot];
    const int p0 = indptr[r], p1 = indptr[r + 1];

    acc_t acc[NA][MT];
#pragma unroll
    for (int u = 0; u < NA; ++u)
#pragma unroll
        for (int t = 0; t < MT; ++t)
#pragma unroll
            for (int e = 0; e < (MM == 32 ? 16 : 4); ++e) acc[u][t][e] = 0.f;

    // per-lane bases: X rows (clamped to m-1; the surplus rows are never stored) and the lane's run
    const T* xbase[MT];
#pragma unroll
    for (int t = 0; t < MT; ++t)
        xbase[t] = X + (size_t)min(i_base + t * MM + li, m - 1) * (size_t)k + h * CH;
    const T* wbase = data + (size_t)li * BS_C + h * CH;

    Frag<T, CH> wf[2][NA], xf[2][MT];
    auto fetch = [&](int buf, int p) {
        const int c = indices[p];
        const T* wp = wbase + (size_t)p * (BS_R * BS_C);
#pragma unroll
        for (int u = 0; u < NA; ++u) wf[buf][u].load(wp + u * (MM * BS_C));
#pragma unroll
        for (int t = 0; t < MT; ++t) xf[buf][t].load(xbase[t] + (size_t)c * BS_C);
    };
    auto compute = [&](int buf) {
#pragma unroll
        for (int u = 0; u < NA; ++u)
#pragma unroll
            for (int t = 0; t < MT; ++t) mfma_frag<T, MM, CH>(acc[u][t], wf[buf][u], xf[buf][t]);
    };

    // two-stage software pipeline over the stored blocks of the block-row
    int p = p0;
    if (p < p1) fetch(0, p);
    while (p < p1) {
        if (p + 1 < p1) fetch(1, p + 1);
        compute(0);
        ++p;
        if (p >= p1) break;
        if (p + 1 < p1) fetch(0, p + 1);
        compute(1);
        ++p;
    }

    // store: lane holds, for row i, columns r*BS_R + u*MM + (MM==32 ? 8*g + 4*h : 4*h) + 0..3
    O* yrow_base = Y + (size_t)r * BS_R;
#pragma unroll
    for (int t = 0; t < MT; ++t) {
        const int i = i_base + t * MM + li;
        if (i < m) {
            O* yrow = yrow_base + (size_t)i * (size_t)n;
#pragma unroll
            for (int u = 0; u < NA; ++u) {
                if constexpr (MM == 32) {
#pragma unroll
                    for (int g = 0; g < 4; ++g)
                        store4<O>(yrow + u * 32 + 8 * g + 4 * h, acc[u][t][4 * g], acc[u][t][4 * g + 1],
                                  acc[u][t][4 * g + 2], acc[u][t][4 * g + 3]);
                } else {
                    store4<O>(yrow + u * 16 + 4 * h, acc[u][t][0], acc[u][t][1], acc[u][t][2], acc[u][t][3]);
                }
            }
        }
    }
}

template <typename T, typename O, int BS_R, int BS_C>
bsr_status launch_shape(const spmm_args& a)
{
    const bsr_matrix* W = a.W;
    const int m = (int)a.m, n = (int)W->n, k = (int)W->k, R = W->R;
    constexpr int MM = BS_R >= 32 ? 32 : 16;
    auto go = [&](auto mt_tag, int waves) -> bsr_status {
        constexpr int MT = decltype(mt_tag)::value;
        const int rows_per_wg = waves * MT * MM;
        const int64_t tiles = (m + rows_per_wg - 1) / rows_per_wg;
        const int64_t blocks = tiles * R;
        if (blocks >= ((int64_t)1 << 31) || blocks * 64 * waves >= ((int64_t)1 << 32)) return BSR_ERR_SHAPE;
        hipLaunchKernelGGL((bsr_mfma_direct<T, O, BS_R, BS_C, MT>), dim3((unsigned)blocks), dim3(64 * waves), 0,
                           a.stream, (const T*)a.X, (const T*)W->data, W->indices, W->indptr, W->row_order,
                           (O*)a.Y, m, k, n, R);
        return hipGetLastError() == hipSuccess ? BSR_OK : BSR_ERR_HIP;
    };
    // Tile height: enough workgroups to fill 256 CUs several times over when m allows it, taller
    // wavefront tiles (more reuse of each W block) when m is large.
    const int sub = (m + MM - 1) / MM;                 // MFMA tiles along m
    if (sub >= 64) return go(std::integral_constant<int, 2>{}, 4);
    if (sub >= 8) return go(std::integral_constant<int, 1>{}, 4);
    return go(std::integral_constant<int, 1>{}, 1);
}

template <typename T, typename O>
bsr_status launch_dtype(const spmm_args& a)
{
    const int br = a.W->bs_r, bc = a.W->bs_c;
#define BSR_CASE(BR, BC) if (br == BR && bc == BC) return launch_shape<T, O, BR, BC>(a)
    BSR_CASE(16, 16); BSR_CASE(16, 32); BSR_CASE(16, 64);
    BSR_CASE(32, 16); BSR_CASE(32, 32); BSR_CASE(32, 64);
    BSR_CASE(64, 16); BSR_CASE(64, 32); BSR_CASE(64, 64);
#undef BSR_CASE
    return BSR_ERR_UNSUPPORTED;
}

}  // namespace

bool mfma_supports(const bsr_matrix* W)
{
    const int br = W->bs_r, bc = W->bs_c;
    const bool r_ok = br == 16 || br == 32 || br == 64;
    const bool c_ok = bc == 16 || bc == 32 || bc == 64;
    return r_ok && c_ok && W->R > 0;
}

bsr_status launch_mfma(const spmm_args& a)
{
    const bsr_dtype in = a.W->dtype, out = a.y_dtype;
    if (in == BSR_F32) return launch_dtype<float, float>(a);
    if (in == BSR_F16) return out == BSR_F32 ? launch_dtype<f16_t, float>(a) : launch_dtype<f16_t, f16_t>(a);
    if (in == BSR_BF16) return out == BSR_F32 ? launch_dtype<bf16_t, float>(a) : launch_dtype<bf16_t, bf16_t>(a);
    return BSR_ERR_DTYPE;
}

// Matrix-core kernel for blocks smaller than an MFMA tile: bs_r, bs_c in {8, 16}, not both 16.
//
// The paper's own shape grid includes 8x8 blocks, below the 16x16 minimum of the matrix cores.  The
// plan groups the stored blocks into 16x16 TILES of W (2x2, 2x1 or 1x2 blocks; a position without a
// stored block is empty) and lists, per tile-row, its tiles by tile-column: an entry holds the byte
// offsets of the tile's blocks in block_data.  The kernel is the k-split kernel's scheme on those
// tiles: a workgroup owns 16 rows of X x one tile-row, its wavefronts share out the tile-row's
// entries, each assembles a W tile in its own LDS area -- lane l fetches 16 bytes of one of the
// tile's blocks with a buffer load, an empty position reads as zeros -- next to the X tile, reads
// both back in MFMA operand order, and the fp32 partial tiles are summed through LDS in fixed order.
// The values are read from block_data at every product: nothing is repacked, so they may change
// between products as with every other kernel.
#include <algorithm>

#include "bsr_mfma_common.h"

using namespace bsr_dev;

namespace {

constexpr unsigned kDead = 0x80000000u;               // byte offset no buffer reaches: reads as zero

typedef int i32x4 __attribute__((ext_vector_type(4)));

#ifndef BSR_PLAIN_LOADS
typedef i32x4 rsrc_t;
__device__ __forceinline__ rsrc_t make_rsrc(const void* base, int bytes)
{
    const unsigned long long a = reinterpret_cast<unsigned long long>(base);
    i32x4 r;
    r.x = __builtin_amdgcn_readfirstlane((int)(unsigned)a);
    r.y = __builtin_amdgcn_readfirstlane((int)(unsigned)(a >> 32) & 0xFFFF);
    r.z = __builtin_amdgcn_readfirstlane(bytes);
    r.w = 0x00020000;
    return r;
}

// 16-byte buffer load with hand-placed waits (see bsr_mfma_ksplit.hip for why).
__device__ __forceinline__ void load_b128(u32x4& dst, const rsrc_t& rsrc, unsigned offset)
{
    asm volatile("buffer_load_dwordx4 %0, %1, %2, 0 offen" : "=v"(dst) : "v"(offset), "s"(rsrc));
}
template <int N> __device__ __forceinline__ void wait_loads() { asm volatile("s_waitcnt vmcnt(%0)" ::"n"(N)); }
__device__ __forceinline__ void arrived(u32x4& v) { asm volatile("" : "+v"(v)); }
#else
// the same loads with compiler-placed waits (see bsr_mfma_ksplit.hip): the checking build
typedef __amdgpu_buffer_rsrc_t rsrc_t;
__device__ __forceinline__ rsrc_t make_rsrc(const void* base, int bytes)
{
    const unsigned long long a = reinterpret_cast<unsigned long long>(base);
    const unsigned long long u = (unsigned long long)(unsigned)__builtin_amdgcn_readfirstlane((int)(unsigned)a) |
                                 ((unsigned long long)(unsigned)__builtin_amdgcn_readfirstlane((int)(unsigned)(a >> 32)) << 32);
    return __builtin_amdgcn_make_buffer_rsrc(reinterpret_cast<void*>(u), 0, __builtin_amdgcn_readfirstlane(bytes), 0x00020000);
}
__device__ __forceinline__ void load_b128(u32x4& dst, const rsrc_t& rsrc, unsigned offset)
{
    dst = __builtin_bit_cast(u32x4, __builtin_amdgcn_raw_buffer_load_b128(rsrc, (int)offset, 0, 0));
}
template <int N> __device__ __forceinline__ void wait_loads() {}
__device__ __forceinline__ void arrived(u32x4&) {}
#endif

template <typename T>
struct small_geom {
    static constexpr int S = (int)sizeof(T);
    static constexpr int RBS = 16 * S;                 // bytes of a tile row
    static constexpr int P = RBS + 16;                 // padded LDS row
    static constexpr int LD = 16 + 4;                  // padded row of the fp32 partial-sum tile
    static constexpr int STAGE = 32 * P;               // W tile + X tile, 16 rows each
    static constexpr int PART = 16 * LD * 4;
    static constexpr int REGION = ((STAGE > PART ? STAGE : PART) + 15) & ~15;
};

template <typename T, typename O, int BS_R, int BS_C>
__global__ __launch_bounds__(512) void bsr_mfma_small(const T* __restrict__ X, const T* __restrict__ data, int w_bytes,
                                                      const int32_t* __restrict__ sb_desc,
                                                      const i32x4* __restrict__ sb_entries,
                                                      const int32_t* __restrict__ sb_cols, O* __restrict__ Y,
                                                      int m, int k, int n, int sb_rows, int per)
{
    typedef small_geom<T> geo;
    constexpr int S = geo::S, RBS = geo::RBS, P = geo::P, LD = geo::LD;
    constexpr int SC = 16 / BS_C;                      // blocks across a tile
    constexpr int NSUB = (16 / BS_R) * SC;             // blocks of a tile
    constexpr int SUBB = BS_R * BS_C * S;              // bytes of a block
    constexpr int LPS = SUBB / 16;                     // lanes that fetch one block
    constexpr int LPR = RBS / 16, RPI = 64 / LPR;      // X tile: lanes per row, rows per load
    constexpr int CH = 4;                              // a lane's run of the tile's 16 columns (4 lane groups)
    static_assert(NSUB * LPS <= 64 && 16 <= RPI, "a tile of W and a tile of X are one load each");
    extern __shared__ __attribute__((aligned(16))) unsigned char lds[];   // [wavefronts][REGION]

    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int nw_max = blockDim.x >> 6;
    const int li = lane & 15, h = lane >> 4;
    // workgroup b: tile-row slot b mod sb_rows (longest first), m-tile b div sb_rows; the descriptor is
    // read a word per lane: {tile-row, first entry, entries, -, first tile-columns}
    const int32_t* __restrict__ desc = sb_desc + (size_t)(blockIdx.x % (unsigned)sb_rows) * kRowDescWords;
    const int dword = lane < kRowDescWords ? desc[lane] : 0;
    const int tr = __builtin_amdgcn_readlane(dword, 0);
    const int e0 = __builtin_amdgcn_readlane(dword, 1), cnt = __builtin_amdgcn_readlane(dword, 2);
    const int i_base = (int)(blockIdx.x / (unsigned)sb_rows) * 16;
    const int nw = max(1, min(nw_max, (cnt + per - 1) / per));

    f32x4 acc = {0.f, 0.f, 0.f, 0.f};
    unsigned char* wl = lds + (size_t)wave * geo::REGION;      // this wavefront's W tile, [16][P]
    unsigned char* xl = wl + 16 * P;                           // and X tile, [16][P]

    if (wave < nw && wave < cnt) {
        const rsrc_t wrsrc = make_rsrc(data, w_bytes);
        const rsrc_t xrsrc = make_rsrc(X + (size_t)i_base * (size_t)k, min(16, m - i_base) * k * S);
        // lane's piece of the W tile: 16 bytes of block q = lane / LPS of the tile (dead past the last)
        const int q = lane / LPS;
        const unsigned within = (unsigned)(lane % LPS) * 16;
        const unsigned w_l = ((unsigned)(q / SC) * BS_R + within / (BS_C * S)) * P + (unsigned)(q % SC) * (BS_C * S) + within % (BS_C * S);
        // and of the X tile: 16 bytes of row lane / LPR
        const unsigned xrow = (unsigned)(lane / LPR), xpiece = (unsigned)(lane % LPR);
        const unsigned x_g = xrow < 16u ? xrow * (unsigned)(k * S) + xpiece * 16 : kDead;
        const unsigned x_l = xrow * P + xpiece * 16;
        const unsigned char* wop = wl + li * P + h * (CH * S);
        const unsigned char* xop = xl + li * P + h * (CH * S);

        u32x4 gw[2], gx[2];
        auto issue = [&](int s, int j) {               // entry j of the tile-row
            const i32x4 e = sb_entries[e0 + j];        // uniform: a scalar read
            const int c = j < kRowDescCols ? __builtin_amdgcn_readlane(dword, kRowDescColsAt + j) : sb_cols[e0 + j];
            const int off = q == 0 ? e.x : (q == 1 ? e.y : (q == 2 ? e.z : e.w));
            load_b128(gw[s], wrsrc, q < NSUB ? (unsigned)off + within : kDead);   // an empty position has off = 2^31
            load_b128(gx[s], xrsrc, x_g + (unsigned)c * RBS);
        };
        auto consume = [&](int s, bool behind) {
            if (behind) wait_loads<2>(); else wait_loads<0>();   // uniform
            arrived(gw[s]);
            arrived(gx[s]);
            wave_lds_fence();                          // the other lanes have read the previous tile's operands
            if (NSUB * LPS == 64 || lane < NSUB * LPS) *reinterpret_cast<u32x4*>(wl + w_l) = gw[s];
            if (RPI == 16 || xrow < 16u) *reinterpret_cast<u32x4*>(xl + x_l) = gx[s];
            wave_lds_fence();                          // operands are what the other lanes just wrote
            Frag<T, CH> wf, xf;
            wf.load(reinterpret_cast<const T*>(wop));
            xf.load(reinterpret_cast<const T*>(xop));
            mfma_frag<T, 16, CH>(acc, wf, xf);
        };
        // every load issued is waited for before the wavefront ends
        issue(0, wave);
        bool odd = wave + nw < cnt;
        if (odd) issue(1, wave + nw);
        for (int j = wave; j < cnt; j += 2 * nw) {
            consume(0, odd);
            const bool next = j + 2 * nw < cnt;
            if (next) issue(0, j + 2 * nw);
            if (odd) {
                consume(1, next);
                odd = j + 3 * nw < cnt;
                if (odd) issue(1, j + 3 * nw);
            }
        }
        wait_loads<0>();
    }
    const int used = min(nw, cnt);
    if (wave < used) {
        float* mine = reinterpret_cast<float*>(wl) + (size_t)li * LD;
        *reinterpret_cast<f32x4*>(mine + 4 * h) = acc;
    }
    __syncthreads();

    // fixed-order sum over the partial tiles: thread t < 64 owns 4 consecutive columns of one row
    for (int t = threadIdx.x; t < 16 * 4; t += blockDim.x) {
        const int i = t / 4, c4 = t - i * 4;
        f32x4 s = {0.f, 0.f, 0.f, 0.f};
        for (int w = 0; w < used; ++w)
            s += *reinterpret_cast<const f32x4*>(lds + (size_t)w * geo::REGION + ((size_t)i * LD + 4 * c4) * 4);
        if (i_base + i < m)
            store4<O>(Y + (size_t)(i_base + i) * (size_t)n + (size_t)tr * 16 + 4 * c4, s.x, s.y, s.z, s.w);
    }
}

template <typename T, typename O, int BS_R, int BS_C>
bsr_status launch_small_shape(const spmm_args& a, const tune_opts& tune)
{
    typedef small_geom<T> geo;
    const bsr_matrix* W = a.W;
    const int m = (int)a.m, n = (int)W->n, k = (int)W->k;
    if ((int64_t)16 * k * geo::S >= ((int64_t)1 << 31)) return BSR_ERR_UNSUPPORTED;
    const int64_t tiles = (m + 15) / 16;
    const int64_t blocks = tiles * W->sb_rows;
    if (blocks >= ((int64_t)1 << 31)) return BSR_ERR_SHAPE;
    int per = tune.a > 0 ? tune.a : 2;
    int nw = (W->sb_max_entries + per - 1) / per;
    const int nw_cap = blocks > 1024 ? 2 : (blocks > 256 ? 4 : 8);
    nw = nw < 1 ? 1 : (nw > nw_cap ? nw_cap : nw);
    if (tune.nw >= 1 && tune.nw <= 8) nw = tune.nw;
    const size_t lds = (size_t)nw * geo::REGION;
    hipLaunchKernelGGL((bsr_mfma_small<T, O, BS_R, BS_C>), dim3((unsigned)blocks), dim3(64 * nw), lds, a.stream,
                       (const T*)a.X, (const T*)W->data, (int)(W->nnzb * W->bs_r * W->bs_c * geo::S), W->sb_desc,
                       reinterpret_cast<const i32x4*>(W->sb_entries), W->sb_cols, (O*)a.Y, m, k, n, W->sb_rows, per);
    return hipGetLastError() == hipSuccess ? BSR_OK : BSR_ERR_HIP;
}

template <typename T, typename O>
bsr_status launch_small_types(const spmm_args& a, const tune_opts& t)
{
    const int br = a.W->bs_r, bc = a.W->bs_c;
    if (br == 8 && bc == 8) return launch_small_shape<T, O, 8, 8>(a, t);
    if (br == 8 && bc == 16) return launch_small_shape<T, O, 8, 16>(a, t);
    if (br == 16 && bc == 8) return launch_small_shape<T, O, 16, 8>(a, t);
    return BSR_ERR_UNSUPPORTED;
}

}  // namespace

bool mfma_small_supports(const bsr_matrix* W)
{
    const bool shape = (W->bs_r == 8 || W->bs_r == 16) && (W->bs_c == 8 || W->bs_c == 16) && !(W->bs_r == 16 && W->bs_c == 16);
    return shape && W->sb_desc != nullptr && W->sb_rows > 0;
}

bsr_status launch_mfma_small(const spmm_args& a, const tune_opts& t)
{
    const bsr_matrix* W = a.W;
    if (!mfma_small_supports(W)) return BSR_ERR_UNSUPPORTED;
    if (W->dtype == BSR_F32) return launch_small_types<float, float>(a, t);
    if (W->dtype == BSR_F16) return a.y_dtype == BSR_F32 ? launch_small_types<_Float16, float>(a, t)
                                                         : launch_small_types<_Float16, _Float16>(a, t);
    if (W->dtype == BSR_BF16) return a.y_dtype == BSR_F32 ? launch_small_types<__bf16, float>(a, t)
                                                          : launch_small_types<__bf16, __bf16>(a, t);
    return BSR_ERR_UNSUPPORTED;
}

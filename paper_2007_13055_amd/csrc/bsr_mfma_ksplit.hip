// Matrix-core kernel for products with few rows of X (few MFMA tiles along m).
//
// One workgroup owns an (MM rows of X) x (one block-row of W) tile of Y.  Its wavefronts share
// out the stored blocks of the block-row -- wavefront w takes blocks p0+w, p0+w+NW, ... -- so a
// block-row's reduction runs NW-wide instead of serially; each wavefront keeps a full-tile fp32
// partial sum, and the partial sums are added through LDS in a fixed order (wavefront 0, 1, ...),
// which keeps the result deterministic.  This is the paper's concurrent reduction (Section 4.4:
// several threads share one output's reduction, partial results aggregated at the end) moved from
// single output elements to MFMA tiles.
//
// Operands reach the matrix cores through LDS.  An MFMA operand wants lane l to hold a run of ROW
// l mod MM, so neighbouring lanes would read addresses a whole row apart, and the memory pipeline
// serves such 16-byte pieces one per cycle (measured: 16 B/clk per CU against 58 B/clk when
// neighbouring lanes read neighbouring pieces).  So a wavefront reads its W block and its X tile
// with lane l taking piece l of the contiguous data, writes them to its own LDS area (rows padded
// by 16 bytes) and reads them back in operand order.  The area belongs to one wavefront, whose LDS
// operations complete in order: no barrier.  Loads are buffer loads: a block the wavefront does
// not have and rows of X past m read as zeros without touching memory, which keeps a wavefront's
// loads unconditional and their number in flight fixed (two blocks ahead).
#include "bsr_mfma_common.h"

using namespace bsr_dev;

namespace {

constexpr unsigned kDead = 0x80000000u;               // byte offset no buffer reaches: reads as zero

typedef int i32x4 __attribute__((ext_vector_type(4)));

#ifndef BSR_PLAIN_LOADS
// Buffer resource over [base, base + bytes): raw 32-bit data, no swizzle.
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

// 16-byte buffer load the compiler neither moves nor waits for: the caller places s_waitcnt itself
// (the compiler would otherwise sink the loads of a wavefront's second block behind the
// arithmetic of its first).
__device__ __forceinline__ void load_b128(u32x4& dst, const rsrc_t& rsrc, unsigned offset)
{
    asm volatile("buffer_load_dwordx4 %0, %1, %2, 0 offen" : "=v"(dst) : "v"(offset), "s"(rsrc));
}
template <int N> __device__ __forceinline__ void wait_loads() { asm volatile("s_waitcnt vmcnt(%0)" ::"n"(N)); }
__device__ __forceinline__ void arrived(u32x4& v) { asm volatile("" : "+v"(v)); }   // use v only below this point
#else
// The same loads through the compiler's buffer-load builtin, which places the waits itself (slower: it
// waits for every load before the first use).  A second library is built this way; a test holds the two
// builds' results against each other bit for bit, so a compiler that mishandled a register of a
// hand-placed load (copied it before the data arrived) would show.
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

template <typename T, int BS_R, int BS_C, int MM_>
struct ksplit_geom {
    static constexpr int MM = MM_;                     // rows of X per workgroup = MFMA tile edge
    static constexpr int S = (int)sizeof(T);
    static constexpr int RBS = BS_C * S;               // bytes of a block's row (and of an X tile's row)
    static constexpr int P = RBS + 16;                 // padded LDS row
    static constexpr int BLK = BS_R * RBS;             // bytes of a stored block
    static constexpr int NLW = (BLK + 1023) / 1024;    // 1 KiB load instructions per block
    static constexpr int LPR = RBS / 16;               // X tile: lanes per row
    static constexpr int RPI = 64 / LPR;               //         rows per load instruction
    static constexpr int NLX = (MM + RPI - 1) / RPI;   //         load instructions
    static constexpr int LD = BS_R + 4;                // padded row of the fp32 partial-sum tile
    static constexpr int STAGE = (BS_R + MM) * P;      // W block + X tile
    static constexpr int PART = MM * LD * 4;           // partial-sum tile (reuses the staging area)
    static constexpr int REGION = ((STAGE > PART ? STAGE : PART) + 15) & ~15;   // LDS bytes per wavefront
};

template <typename T, typename O, int BS_R, int BS_C, int MM_>
__global__ __launch_bounds__(512) void bsr_mfma_ksplit(const T* __restrict__ X, const T* __restrict__ data,
                                                       const int32_t* __restrict__ indices,
                                                       const int32_t* __restrict__ row_desc, O* __restrict__ Y,
                                                       int m, int k, int n, int R, int per, int items)
{
    typedef ksplit_geom<T, BS_R, BS_C, MM_> geo;
    constexpr int MM = geo::MM, S = geo::S, RBS = geo::RBS, P = geo::P, BLK = geo::BLK;
    constexpr int NLW = geo::NLW, LPR = geo::LPR, RPI = geo::RPI, NLX = geo::NLX, LD = geo::LD;
    constexpr int NA = BS_R / MM;
    constexpr int G = 64 / MM;
    constexpr int CH = BS_C / G;
    constexpr int NE = MM == 32 ? 16 : 4;             // accumulator values per lane and tile
    typedef typename AccT<MM>::type acc_t;
    extern __shared__ __attribute__((aligned(16))) unsigned char lds[];   // [wavefronts][REGION]

    const int lane = threadIdx.x & 63;
    const int hw_wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int nw_max = blockDim.x >> 6;
    const int li = lane % MM, h = lane / MM;
    // One read of the workgroup's descriptor, a word per lane: block-row, first stored block, count,
    // m-tile, first block-columns.  With a work-item table (items = the number of CUs it was laid out
    // for, else 0) workgroup b takes entry b --
    // the table is laid out so that the workgroups sharing a CU carry about equal work -- and an
    // entry with block-row -1 is a filler; without one, workgroup b takes slot b mod R of m-tile b div R.
    const int32_t* __restrict__ desc =
        row_desc + (size_t)(items ? blockIdx.x : blockIdx.x % (unsigned)R) * kRowDescWords;
    const int dword = lane < kRowDescWords ? desc[lane] : 0;
    const int r = __builtin_amdgcn_readlane(dword, 0);
    if (r < 0) return;                                // whole workgroup leaves together
    const int p0 = __builtin_amdgcn_readlane(dword, 1), cnt = __builtin_amdgcn_readlane(dword, 2);
    const int i_base = (items ? __builtin_amdgcn_readlane(dword, 3) : (int)(blockIdx.x / (unsigned)R)) * MM;
    // wavefronts that take part: about `per` stored blocks each, at most all of the workgroup's;
    // the others go straight to the barrier
    const int nw = max(1, min(nw_max, (cnt + per - 1) / per));
    // Wavefront w of a workgroup runs on SIMD w mod 4 and the low-numbered wavefronts get a block-row's
    // odd blocks.  The workgroups stacked on one CU (table entries b, b + #CUs, ...) therefore number
    // their wavefronts from different starts: `wave` is the number used for sharing out blocks and
    // for the order of the final sum; wavefronts nw and up take no part.
    const int wave = hw_wave < nw ? (hw_wave + (items ? (int)(blockIdx.x / (unsigned)items) : 0)) % nw : hw_wave;

    acc_t acc[NA];
#pragma unroll
    for (int u = 0; u < NA; ++u)
#pragma unroll
        for (int e = 0; e < NE; ++e) acc[u][e] = 0.f;

    unsigned char* wl = lds + (size_t)wave * geo::REGION;      // this wavefront's W block, [BS_R][P]
    unsigned char* xl = wl + BS_R * P;                         // and X tile, [MM][P]

    if (wave < nw && wave < cnt) {                     // this wavefront has at least one block
        // W of this block-row and the X rows of this m-tile as buffers: offsets past their ends read zero
        const rsrc_t wrsrc = make_rsrc(data + (size_t)p0 * (BS_R * BS_C), cnt * BLK);
        const rsrc_t xrsrc = make_rsrc(X + (size_t)i_base * (size_t)k, min(MM, m - i_base) * k * S);
        // lane's pieces: W piece t is bytes t*1024 + lane*16 of the block; X piece t is 16 bytes of
        // row t*RPI + lane/LPR of the tile
        unsigned w_g[NLW], w_l[NLW], x_g[NLX], x_l[NLX];
#pragma unroll
        for (int t = 0; t < NLW; ++t) {
            const unsigned b = (unsigned)(t * 1024 + lane * 16);
            w_g[t] = b < (unsigned)BLK ? b : kDead;
            w_l[t] = (b / RBS) * P + (b % RBS);
        }
#pragma unroll
        for (int t = 0; t < NLX; ++t) {
            const unsigned row = (unsigned)(t * RPI + lane / LPR), piece = (unsigned)(lane % LPR);
            x_g[t] = row < (unsigned)MM ? row * (unsigned)(k * S) + piece * 16 : kDead;
            x_l[t] = row * P + piece * 16;
        }
        const unsigned char* wop = wl + li * P + h * (CH * S);       // lane's operand runs
        const unsigned char* xop = xl + li * P + h * (CH * S);

        // The wavefront's blocks are j = wave, wave + nw, ...; two register sets alternate, so the
        // loads of the next two blocks are in flight while one is multiplied.
        u32x4 gw[2][NLW], gx[2][NLX];
        auto issue = [&](int s, int j) {
            const int c = j < kRowDescCols ? __builtin_amdgcn_readlane(dword, kRowDescColsAt + j) : indices[p0 + j];
#pragma unroll
            for (int t = 0; t < NLW; ++t) load_b128(gw[s][t], wrsrc, w_g[t] + (unsigned)j * BLK);
#pragma unroll
            for (int t = 0; t < NLX; ++t) load_b128(gx[s][t], xrsrc, x_g[t] + (unsigned)c * RBS);
        };
        // `behind`: another block's loads were issued after this one's (loads return in issue order)
        auto consume = [&](int s, bool behind) {
            if (behind) wait_loads<NLW + NLX>(); else wait_loads<0>();   // uniform
#pragma unroll
            for (int t = 0; t < NLW; ++t) arrived(gw[s][t]);
#pragma unroll
            for (int t = 0; t < NLX; ++t) arrived(gx[s][t]);
            wave_lds_fence();                          // the other lanes have read the previous block's operands
#pragma unroll
            for (int t = 0; t < NLW; ++t)
                if (BLK % 1024 == 0 || t * 1024 + lane * 16 < BLK) *reinterpret_cast<u32x4*>(wl + w_l[t]) = gw[s][t];
#pragma unroll
            for (int t = 0; t < NLX; ++t)
                if (MM % RPI == 0 || t * RPI + lane / LPR < MM) *reinterpret_cast<u32x4*>(xl + x_l[t]) = gx[s][t];
            wave_lds_fence();                          // operands are what the other lanes just wrote
            Frag<T, CH> wf[NA], xf;
#pragma unroll
            for (int u = 0; u < NA; ++u) wf[u].load(reinterpret_cast<const T*>(wop + u * (MM * P)));
            xf.load(reinterpret_cast<const T*>(xop));
#pragma unroll
            for (int u = 0; u < NA; ++u) mfma_frag<T, MM, CH>(acc[u], wf[u], xf);
        };
        // every load issued below is waited for before the wavefront ends: none is left in flight.
        // Two register sets only where both fit the register file: the loads are written in
        // assembly, so a spill of a register a load has not filled yet would store garbage.
        constexpr bool kTwoSets = NLW + NLX <= 12;
        if constexpr (kTwoSets) {
            issue(0, wave);
            bool odd = wave + nw < cnt;                         // set 1 holds a block (all uniform)
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
        } else {
            for (int j = wave; j < cnt; j += nw) {
                issue(0, j);
                consume(0, false);
            }
        }
        wait_loads<0>();
    }
    // partial sums of the wavefronts that had at least one block -> LDS (over the wavefront's own
    // staging area, whose contents it has already consumed)
    const int used = min(nw, cnt);
    wave_lds_fence();
    if (wave < used) {
        float* mine = reinterpret_cast<float*>(wl) + (size_t)li * LD;
#pragma unroll
        for (int u = 0; u < NA; ++u) {
            if constexpr (MM == 32) {
#pragma unroll
                for (int g = 0; g < 4; ++g) {
                    const f32x4 v = {acc[u][4 * g], acc[u][4 * g + 1], acc[u][4 * g + 2], acc[u][4 * g + 3]};
                    *reinterpret_cast<f32x4*>(mine + u * 32 + 8 * g + 4 * h) = v;
                }
            } else {
                const f32x4 v = {acc[u][0], acc[u][1], acc[u][2], acc[u][3]};
                *reinterpret_cast<f32x4*>(mine + u * 16 + 4 * h) = v;
            }
        }
    }
    __syncthreads();

    // fixed-order sum over the partial tiles; each thread owns 4 consecutive columns of one row
    constexpr int QUADS = BS_R / 4;
    for (int t = threadIdx.x; t < MM * QUADS; t += blockDim.x) {
        const int i = t / QUADS, q = t - i * QUADS;
        f32x4 s = {0.f, 0.f, 0.f, 0.f};
        for (int w = 0; w < used; ++w)
            s += *reinterpret_cast<const f32x4*>(lds + (size_t)w * geo::REGION + ((size_t)i * LD + 4 * q) * 4);
        if (i_base + i < m)
            store4<O>(Y + (size_t)(i_base + i) * (size_t)n + (size_t)r * BS_R + 4 * q, s.x, s.y, s.z, s.w);
    }
}

template <typename T, typename O, int BS_R, int BS_C, int MM>
bsr_status launch_ksplit_tile(const spmm_args& a, const tune_opts& tune)
{
    typedef ksplit_geom<T, BS_R, BS_C, MM> geo;
    const bsr_matrix* W = a.W;
    const int m = (int)a.m, n = (int)W->n, k = (int)W->k, R = W->R;
    // 32-bit byte offsets inside a block-row's blocks and inside an m-tile's rows of X
    if ((int64_t)W->max_row_blocks * geo::BLK >= ((int64_t)1 << 31) || (int64_t)MM * k * geo::S >= ((int64_t)1 << 31))
        return BSR_ERR_UNSUPPORTED;
    // wavefronts per workgroup: about `per` stored blocks each for the longest block-row; at most 8
    // when every workgroup has a CU to itself, at most 4 up to four workgroups per CU and 2 beyond
    // (starting wavefronts costs time too, about 11 cycles each per XCD, and with many workgroups the
    // CUs are busy anyway), and no more than LDS has room for
    const int64_t tiles = (m + MM - 1) / MM;
    int64_t blocks = tiles * R;
    int per = tune.a > 0 ? tune.a : 2;
    int nw = (W->max_row_blocks + per - 1) / per;
    const int nw_cap = blocks > 1024 ? 2 : (blocks > 256 ? 4 : 8);
    nw = nw < 1 ? 1 : (nw > nw_cap ? nw_cap : nw);
    if (tune.nw >= 1 && tune.nw <= 8) nw = tune.nw;
    nw = std::min(nw, 160 * 1024 / geo::REGION);
    if (blocks >= ((int64_t)1 << 31) || blocks * 64 * nw >= ((int64_t)1 << 32)) return BSR_ERR_SHAPE;
    // CU-balanced work-item table when there are more items than CUs (else every item has a CU to itself)
    const int32_t* table = W->row_desc;
    int items = 0;
    if (tune.b != 1 && blocks > 256 && blocks <= kMaxKsplitItems) {
        const int32_t* item_table = nullptr;
        const int grid = ksplit_items(W, (int)tiles, a.stream, &item_table);
        if (grid > 0) { table = item_table; items = W->n_cu; blocks = grid; }
    }
    const size_t lds = (size_t)nw * geo::REGION;
    static const hipError_t attr =
        hipFuncSetAttribute(reinterpret_cast<const void*>(&bsr_mfma_ksplit<T, O, BS_R, BS_C, MM>),
                            hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
    if (attr != hipSuccess) return BSR_ERR_HIP;
    hipLaunchKernelGGL((bsr_mfma_ksplit<T, O, BS_R, BS_C, MM>), dim3((unsigned)blocks), dim3(64 * nw), lds, a.stream,
                       (const T*)a.X, (const T*)W->data, W->indices, table, (O*)a.Y, m, k, n, R, per, items);
    return hipGetLastError() == hipSuccess ? BSR_OK : BSR_ERR_HIP;
}

// Rows of X per workgroup: 32 (the larger MFMA tile: every W block is fetched half as often) when
// that still leaves at least three workgroups per CU to even out block-rows of different length,
// else 16.  16-bit blocks narrower than 32 columns stay at 32 rows where they can: their 16-row
// MFMA would run at half rate.
template <typename T, typename O, int BS_R, int BS_C>
bsr_status launch_ksplit_shape(const spmm_args& a, const tune_opts& tune)
{
    if constexpr (BS_R >= 32) {
        const int64_t items32 = (a.m + 31) / 32 * a.W->R;
        const bool slow16 = sizeof(T) == 2 && BS_C < 32;
        bool tall = items32 >= 768 || slow16;
        if (tune.mt == 1) tall = false;
        if (tune.mt == 2) tall = true;
        if (tall) return launch_ksplit_tile<T, O, BS_R, BS_C, 32>(a, tune);
    }
    return launch_ksplit_tile<T, O, BS_R, BS_C, 16>(a, tune);
}

}  // namespace

bsr_status launch_mfma_ksplit(const spmm_args& a, const tune_opts& t)
{
    BSR_MFMA_DISPATCH(launch_ksplit_shape, a.W, a.y_dtype, a, t);
    return BSR_ERR_UNSUPPORTED;
}

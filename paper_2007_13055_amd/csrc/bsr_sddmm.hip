// The sampled sibling: D[p] = G[:, block-row of p]^T * X[:, block-column of p] for every stored
// block p -- the gradient of the block values when Y = X * W^T is a layer's forward pass (Y is
// linear in block_data[p][a][c] with coefficient X[i][col*bs_c + c] in Y[i][r*bs_r + a]).
//
// One workgroup (4 wavefronts) per run of up to NB stored blocks of one block-row (the plan cuts
// every block-row into runs of about equal length): the blocks of a run share the piece of G.  The
// reduction runs over the rows i of G and X, which is the slow axis of both, so the operands cannot
// be read in MFMA order from memory.  A wavefront takes every fourth chunk of 32 rows: it copies the
// 32 x bs_r piece of G and the run's 32 x bs_c pieces of X into its own LDS area with contiguous
// 16-byte reads (the next chunk's loads are in flight while this one is multiplied), and reads the
// operands back transposed -- 16-bit types with the LDS transpose read (ds_read_b64_tr_b16: each
// lane receives, for its row of the MFMA operand, 4 consecutive values of the reduction index),
// fp32 one value per lane and MFMA step.  Every wavefront accumulates the run's whole blocks over
// its chunks; the four partial blocks are added through LDS in fixed order and stored as one
// contiguous block each.
// Other block shapes: one thread per element of the block, a plain loop over i.
#include <algorithm>

#include "bsr_mfma_common.h"

using namespace bsr_dev;

namespace {

constexpr int kChunk = 32;                            // rows of G and X per step of a wavefront

typedef short s16x4 __attribute__((ext_vector_type(4)));

template <typename T, int BS_R, int BS_C, int NB_>
struct sddmm_geom {
    static constexpr int S = (int)sizeof(T);
    static constexpr int NB = NB_;                                     // blocks per run
    static constexpr int MM = (BS_R >= 32 && BS_C >= 32) ? 32 : 16;   // MFMA tile edge
    static constexpr int NA = BS_R / MM, NC = BS_C / MM;
    static constexpr int RBG = BS_R * S, RBC = BS_C * S;               // bytes of a row of the G / X piece
    static constexpr int PG = RBG + 16, PC = RBC + 16;                 // padded LDS rows
    static constexpr int NLG = kChunk * RBG / 1024, NLX = kChunk * RBC / 1024;   // 1 KiB loads per chunk
    static constexpr int LDP = BS_C + 4;                               // padded row of the fp32 partial block
    static constexpr int STAGE = kChunk * (PG + NB * PC);
    static constexpr int PART = BS_R * LDP * 4;
    static constexpr int REGION = ((STAGE > PART ? STAGE : PART) + 15) & ~15;
};

// The lane's 8 consecutive reduction-index values of operand row `row0 + lane's row`, 16-bit types.
//   tile   [kChunk][pitch] bytes, row-major pieces of G or X as they lie in memory
//   MM=32: lane l = 32*kappa + 16*beta + lambda feeds MFMA row 16*beta + lambda, values i0 + 8*kappa .. +7
//   MM=16: lane l = 16*g + lambda feeds MFMA row lambda, values i0 + 8*g .. +7
// ds_read_b64_tr_b16 works on groups of 16 lanes: lane mu supplies the address of 4 consecutive
// 16-bit values, and lane lambda receives value (lambda mod 4) of the lanes lambda/4 + 4j, j = 0..3.
// With lane mu pointing at row (mu div 4) and columns 4*(mu mod 4) .. +3 of a 4 x 16 piece, lane
// lambda therefore receives column lambda of its 4 rows: the transpose an MFMA operand needs.
template <typename T, int MM>
__device__ __forceinline__ u32x4 read_operand16(const unsigned char* tile, int pitch, int i0, int col0, int lane)
{
    const int lambda = lane & 15;
    int irow, ccol;
    if constexpr (MM == 32) {
        irow = i0 + 8 * (lane >> 5) + (lambda >> 2);
        ccol = col0 + 16 * ((lane >> 4) & 1) + 4 * (lambda & 3);
    } else {
        irow = i0 + 8 * (lane >> 4) + (lambda >> 2);
        ccol = col0 + 4 * (lambda & 3);
    }
    typedef __attribute__((address_space(3))) s16x4 lds_s16x4;
    const unsigned char* p0 = tile + irow * pitch + ccol * 2;
    const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4*)(p0));
    const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4*)(p0 + 4 * pitch));
    const u32x2 a = __builtin_bit_cast(u32x2, lo), b = __builtin_bit_cast(u32x2, hi);
    return u32x4{a.x, a.y, b.x, b.y};
}

template <typename T, typename O, int BS_R, int BS_C, int NB_>
__global__ __launch_bounds__(256) void bsr_sddmm_mfma(const T* __restrict__ G, const T* __restrict__ X,
                                                      const int32_t* __restrict__ block_row,
                                                      const int32_t* __restrict__ indices,
                                                      const int32_t* __restrict__ runs, O* __restrict__ D,
                                                      int m, int k, int n, int n_runs)
{
    typedef sddmm_geom<T, BS_R, BS_C, NB_> geo;
    constexpr int S = geo::S, MM = geo::MM, NA = geo::NA, NC = geo::NC, NB = NB_;
    constexpr int RBG = geo::RBG, RBC = geo::RBC, PG = geo::PG, PC = geo::PC, NLG = geo::NLG, NLX = geo::NLX;
    constexpr int LDP = geo::LDP;
    static_assert(NLG >= 1 && NLX >= 1, "a chunk of either piece is at least one load per lane");
    typedef typename AccT<MM>::type acc_t;
    constexpr int NE = MM == 32 ? 16 : 4;
    extern __shared__ __attribute__((aligned(16))) unsigned char lds[];   // [4 wavefronts][REGION]

    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    // workgroup b runs on XCD b mod 8: XCD x takes the x-th eighth of the runs, so that the pieces of G
    // one XCD's L2 holds are those of consecutive block-rows
    const int per_xcd = (int)gridDim.x / 8;
    const int run = (int)(blockIdx.x % 8u) * per_xcd + (int)(blockIdx.x / 8u);
    if (run >= n_runs) return;                        // whole workgroup: the grid is rounded up to 8
    // uniform: scalar reads; 1 <= cnt <= NB.  Without a run table every stored block is its own run.
    const int p0 = runs ? runs[2 * run] : run, cnt = runs ? runs[2 * run + 1] : 1;
    const int r = block_row[p0];
    unsigned char* gt = lds + (size_t)wave * geo::REGION;     // G piece [kChunk][PG]
    unsigned char* xt = gt + kChunk * PG;                     // X pieces [NB][kChunk][PC]

    acc_t acc[NB][NA][NC];
#pragma unroll
    for (int j = 0; j < NB; ++j)
#pragma unroll
        for (int ua = 0; ua < NA; ++ua)
#pragma unroll
            for (int uc = 0; uc < NC; ++uc)
#pragma unroll
                for (int e = 0; e < NE; ++e) acc[j][ua][uc][e] = 0.f;

    // lane's pieces of a chunk: piece t*64 + lane is 16 bytes of row (piece div pieces-per-row)
    const unsigned char* gbase = reinterpret_cast<const unsigned char*>(G + (size_t)r * BS_R);
    const unsigned char* xbase[NB];
#pragma unroll
    for (int j = 0; j < NB; ++j)
        xbase[j] = reinterpret_cast<const unsigned char*>(X + (size_t)indices[p0 + min(j, cnt - 1)] * BS_C);
    const size_t grow = (size_t)n * S, xrow = (size_t)k * S;
    int g_row[NLG], g_cb[NLG], x_row[NLX], x_cb[NLX];
#pragma unroll
    for (int t = 0; t < NLG; ++t) { const int q = t * 64 + lane; g_row[t] = q / (RBG / 16); g_cb[t] = (q % (RBG / 16)) * 16; }
#pragma unroll
    for (int t = 0; t < NLX; ++t) { const int q = t * 64 + lane; x_row[t] = q / (RBC / 16); x_cb[t] = (q % (RBC / 16)) * 16; }

    // the branches on j < cnt are uniform over the workgroup
    u32x4 gg[NLG], gx[NB][NLX];
    auto fetch = [&](int i0) {                        // rows past m repeat row m-1 and are zeroed when staged
#pragma unroll
        for (int t = 0; t < NLG; ++t)
            gg[t] = *reinterpret_cast<const u32x4*>(gbase + (size_t)min(i0 + g_row[t], m - 1) * grow + g_cb[t]);
#pragma unroll
        for (int j = 0; j < NB; ++j)
            if (j < cnt) {
#pragma unroll
                for (int t = 0; t < NLX; ++t)
                    gx[j][t] = *reinterpret_cast<const u32x4*>(xbase[j] + (size_t)min(i0 + x_row[t], m - 1) * xrow + x_cb[t]);
            }
    };
    auto stage = [&](int i0) {
        const bool tail = i0 + kChunk > m;            // uniform
        wave_lds_fence();                             // the other lanes have read the previous chunk
#pragma unroll
        for (int t = 0; t < NLG; ++t) {
            u32x4 v = gg[t];
            if (tail && i0 + g_row[t] >= m) v = u32x4{0u, 0u, 0u, 0u};
            *reinterpret_cast<u32x4*>(gt + g_row[t] * PG + g_cb[t]) = v;
        }
#pragma unroll
        for (int j = 0; j < NB; ++j)
            if (j < cnt) {
#pragma unroll
                for (int t = 0; t < NLX; ++t) {
                    u32x4 v = gx[j][t];
                    if (tail && i0 + x_row[t] >= m) v = u32x4{0u, 0u, 0u, 0u};
                    *reinterpret_cast<u32x4*>(xt + j * (kChunk * PC) + x_row[t] * PC + x_cb[t]) = v;
                }
            }
        wave_lds_fence();                             // what is read next is what the other lanes just wrote
    };
    auto compute = [&]() {
        if constexpr (std::is_same<T, float>::value) {
            constexpr int KS = MM == 32 ? 2 : 4;      // reduction steps per MFMA
            const int irow = lane / MM, col = lane % MM;
#pragma unroll
            for (int s = 0; s < kChunk / KS; ++s) {
                float av[NA];
#pragma unroll
                for (int ua = 0; ua < NA; ++ua) av[ua] = *reinterpret_cast<const float*>(gt + (s * KS + irow) * PG + (ua * MM + col) * 4);
#pragma unroll
                for (int j = 0; j < NB; ++j)
                    if (j < cnt) {
                        float bv[NC];
#pragma unroll
                        for (int uc = 0; uc < NC; ++uc)
                            bv[uc] = *reinterpret_cast<const float*>(xt + j * (kChunk * PC) + (s * KS + irow) * PC + (uc * MM + col) * 4);
#pragma unroll
                        for (int ua = 0; ua < NA; ++ua)
#pragma unroll
                            for (int uc = 0; uc < NC; ++uc) {
                                if constexpr (MM == 32) acc[j][ua][uc] = __builtin_amdgcn_mfma_f32_32x32x2f32(av[ua], bv[uc], acc[j][ua][uc], 0, 0, 0);
                                else                    acc[j][ua][uc] = __builtin_amdgcn_mfma_f32_16x16x4f32(av[ua], bv[uc], acc[j][ua][uc], 0, 0, 0);
                            }
                    }
            }
        } else {
            constexpr int KI = MM == 32 ? 16 : 32;    // rows of the chunk one MFMA reduces over
#pragma unroll
            for (int s = 0; s < kChunk / KI; ++s) {
                Frag<T, 8> af[NA];
#pragma unroll
                for (int ua = 0; ua < NA; ++ua) {
                    const u32x4 v = read_operand16<T, MM>(gt, PG, s * KI, ua * MM, lane);
                    af[ua].w[0] = v.x; af[ua].w[1] = v.y; af[ua].w[2] = v.z; af[ua].w[3] = v.w;
                }
#pragma unroll
                for (int j = 0; j < NB; ++j)
                    if (j < cnt) {
                        Frag<T, 8> bf[NC];
#pragma unroll
                        for (int uc = 0; uc < NC; ++uc) {
                            const u32x4 v = read_operand16<T, MM>(xt + j * (kChunk * PC), PC, s * KI, uc * MM, lane);
                            bf[uc].w[0] = v.x; bf[uc].w[1] = v.y; bf[uc].w[2] = v.z; bf[uc].w[3] = v.w;
                        }
#pragma unroll
                        for (int ua = 0; ua < NA; ++ua)
#pragma unroll
                            for (int uc = 0; uc < NC; ++uc) mfma_frag<T, MM, 8>(acc[j][ua][uc], af[ua], bf[uc]);
                    }
            }
        }
    };

    // chunks wave, wave + 4, ...: the next chunk's loads are issued once this one's registers are in LDS
    const int n_chunks = (m + kChunk - 1) / kChunk;
    if (wave < n_chunks) fetch(wave * kChunk);
    for (int q = wave; q < n_chunks; q += 4) {
        stage(q * kChunk);
        if (q + 4 < n_chunks) fetch((q + 4) * kChunk);
        compute();
    }

    // One block of the run at a time: the wavefront's partial block -> its LDS area as [bs_r][LDP] fp32
    // (the staged pieces are consumed: a wavefront's own LDS operations complete in order), then the
    // fixed-order sum of the four partial blocks, 4 consecutive columns per thread, contiguous store.
    float* part = reinterpret_cast<float*>(gt);
    wave_lds_fence();
#pragma unroll
    for (int j = 0; j < NB; ++j) {
        if (j >= cnt) break;
        if (j > 0) __syncthreads();                   // the sums of block j-1 are read
#pragma unroll
        for (int ua = 0; ua < NA; ++ua)
#pragma unroll
            for (int uc = 0; uc < NC; ++uc)
#pragma unroll
                for (int e = 0; e < NE; ++e) {
                    int a, cc;
                    if constexpr (MM == 32) { a = ua * 32 + 8 * (e / 4) + 4 * (lane / 32) + e % 4; cc = uc * 32 + lane % 32; }
                    else                    { a = ua * 16 + 4 * (lane / 16) + e;                    cc = uc * 16 + lane % 16; }
                    part[a * LDP + cc] = acc[j][ua][uc][e];
                }
        __syncthreads();
        O* dst = D + (size_t)(p0 + j) * (BS_R * BS_C);
        for (int e4 = threadIdx.x; e4 < BS_R * BS_C / 4; e4 += 256) {
            const int a = (e4 * 4) / BS_C, cc = (e4 * 4) % BS_C;
            f32x4 s = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int w = 0; w < 4; ++w)
                s += *reinterpret_cast<const f32x4*>(lds + (size_t)w * geo::REGION + ((size_t)a * LDP + cc) * 4);
            store4<O>(dst + e4 * 4, s.x, s.y, s.z, s.w);
        }
    }
}

// Blocks whose pieces of G or X are narrower than a 128-byte line (16- and 32-wide blocks): a
// workgroup per *tile* of SR adjacent block-rows x LC adjacent block-columns (SR*bs_r and LC*bs_c
// elements fill a line), so every line that comes from L2 is used whole.  The plan lists the tiles
// that hold a stored block: {super-row, column group, first entry of its block list, bit mask of the
// SR*LC positions}; the block list holds the stored-block numbers of the set bits in position order.
//
// Moving a chunk global -> registers -> LDS -> registers costs three trips through the CU's memory
// data path, which is what bounds this kernel; the loads therefore write LDS directly
// (global_load_lds_dwordx4: lane l's 16 bytes land at the instruction's LDS base + 16*l, so a chunk
// lies in LDS as rows without padding).  Which 16-byte piece of its row a lane fetches is free: the
// pieces of row r are stored XOR-swizzled by sigma(r), which spreads the 4 rows a group of 16 lanes
// reads together (and the rows of the neighbouring group) over different banks.  One buffer per
// wavefront: wait for the chunk, read all its operands into registers, start the next chunk's
// loads, multiply.  A position without a stored block is skipped (uniform branch on the mask).
// Rows past m repeat row m-1 and are overwritten with zeros in LDS (last chunk only); columns past
// n or k (a last, partial tile) are read from the tile's first column: absent positions only.
template <typename T, int BS_R, int BS_C>
struct sddmm_tile_geom {
    static constexpr int S = (int)sizeof(T);
    static constexpr int MM = (BS_R >= 32 && BS_C >= 32) ? 32 : 16;
    static constexpr int NA = BS_R / MM, NC = BS_C / MM;
    static constexpr int SR = BS_R * S >= 128 ? 1 : 128 / (BS_R * S);   // sddmm_tile_dims()
    static constexpr int LC = BS_C * S >= 128 ? 1 : 128 / (BS_C * S);
    static constexpr int NPOS = SR * LC;
    static constexpr int RBG = SR * BS_R * S, RBC = LC * BS_C * S;      // bytes of a row of the G / X piece: 128 or 256
    static constexpr int NLG = kChunk * RBG / 1024, NLX = kChunk * RBC / 1024;   // 1 KiB loads per chunk
    static constexpr int LDP = BS_C + 4;
    static constexpr int STAGE = kChunk * (RBG + RBC);
    static constexpr int PART = BS_R * LDP * 4;                         // one partial block
    static constexpr int PR = STAGE / PART >= 1 ? (STAGE / PART > NPOS ? NPOS : STAGE / PART) : 1;   // partial blocks per round
    static constexpr int REGION = ((STAGE > PR * PART ? STAGE : PR * PART) + 1023) & ~1023;
    static_assert(RBG == 128 || RBG == 256, "rows of the G piece");
    static_assert(RBC == 128 || RBC == 256, "rows of the X piece");
};

// Byte offset of byte `cb` of row r in a chunk whose rows are RB bytes: 16-byte pieces XOR-swizzled.
template <int RB>
__device__ __forceinline__ int swz(int r, int cb)
{
    const int sigma = RB == 128 ? ((((r >> 1) & 1) << 1) | (((r >> 3) & 1) << 2))
                                : (((r & 3) << 1) | (((r >> 3) & 1) << 3));
    return r * RB + ((((cb >> 4) ^ sigma)) << 4) + (cb & 15);
}

// read_operand16 on a swizzled chunk (rows i0 .. of the chunk, element columns col0 ..).
template <typename T, int MM, int RB>
__device__ __forceinline__ u32x4 read_operand16_swz(const unsigned char* tile, int i0, int col0, int lane)
{
    const int lambda = lane & 15;
    int irow, ccol;
    if constexpr (MM == 32) {
        irow = i0 + 8 * (lane >> 5) + (lambda >> 2);
        ccol = col0 + 16 * ((lane >> 4) & 1) + 4 * (lambda & 3);
    } else {
        irow = i0 + 8 * (lane >> 4) + (lambda >> 2);
        ccol = col0 + 4 * (lambda & 3);
    }
    typedef __attribute__((address_space(3))) s16x4 lds_s16x4;
    const unsigned char* p0 = tile + swz<RB>(irow, ccol * 2);       // row irow + 4 has the same sigma
    const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4*)(p0));
    const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4*)(p0 + 4 * RB));
    const u32x2 a = __builtin_bit_cast(u32x2, lo), b = __builtin_bit_cast(u32x2, hi);
    return u32x4{a.x, a.y, b.x, b.y};
}

template <typename T, typename O, int BS_R, int BS_C>
__global__ __launch_bounds__(256, sizeof(T) == 4 ? 3 : 4) void bsr_sddmm_tiles(const T* __restrict__ G, const T* __restrict__ X,
                                                       const int32_t* __restrict__ tiles,
                                                       const int32_t* __restrict__ plist, O* __restrict__ D,
                                                       int m, int k, int n, int n_tiles)
{
    typedef sddmm_tile_geom<T, BS_R, BS_C> geo;
    constexpr int S = geo::S, MM = geo::MM, NA = geo::NA, NC = geo::NC, SR = geo::SR, LC = geo::LC, NPOS = geo::NPOS;
    constexpr int RBG = geo::RBG, RBC = geo::RBC, NLG = geo::NLG, NLX = geo::NLX;
    constexpr int LDP = geo::LDP, PR = geo::PR;
    typedef typename AccT<MM>::type acc_t;
    constexpr int NE = MM == 32 ? 16 : 4;
    typedef __attribute__((address_space(3))) void lds_void;
    typedef __attribute__((address_space(1))) const void glob_void;
    extern __shared__ __attribute__((aligned(1024))) unsigned char lds[];   // [4 wavefronts][REGION]

    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int per_xcd = (int)gridDim.x / 8;           // XCD x takes the x-th eighth of the tiles
    const int tile = (int)(blockIdx.x % 8u) * per_xcd + (int)(blockIdx.x / 8u);
    if (tile >= n_tiles) return;                      // whole workgroup: the grid is rounded up to 8
    const int sr = tiles[4 * tile], cg = tiles[4 * tile + 1], first = tiles[4 * tile + 2];   // uniform
    const unsigned mask = (unsigned)tiles[4 * tile + 3];
    unsigned char* gt = lds + (size_t)wave * geo::REGION;     // G piece [kChunk][RBG], swizzled
    unsigned char* xt = gt + kChunk * RBG;                    // X piece [kChunk][RBC], swizzled

    acc_t acc[NPOS][NA][NC];
#pragma unroll
    for (int q = 0; q < NPOS; ++q)
#pragma unroll
        for (int ua = 0; ua < NA; ++ua)
#pragma unroll
            for (int uc = 0; uc < NC; ++uc)
#pragma unroll
                for (int e = 0; e < NE; ++e) acc[q][ua][uc][e] = 0.f;

    // load t of a piece fills LDS bytes [1024 t, 1024 t + 1024): lane l's slot is row (64 t + l) / (RB/16),
    // stored piece (64 t + l) mod (RB/16), which holds the row's piece (stored piece ^ sigma(row))
    const int gcol0 = sr * (SR * BS_R), xcol0 = cg * (LC * BS_C);   // first column of the pieces
    const unsigned char* gbase = reinterpret_cast<const unsigned char*>(G + gcol0);
    const unsigned char* xbase = reinterpret_cast<const unsigned char*>(X + xcol0);
    const size_t grow = (size_t)n * S, xrow = (size_t)k * S;
    int g_row[NLG], g_src[NLG], x_row[NLX], x_src[NLX];
#pragma unroll
    for (int t = 0; t < NLG; ++t) {
        const int q = t * 64 + lane;
        g_row[t] = q / (RBG / 16);
        const int cb = (swz<RBG>(g_row[t], (q % (RBG / 16)) * 16) - g_row[t] * RBG);   // the piece this slot holds
        g_src[t] = gcol0 + cb / S < n ? cb : 0;
    }
#pragma unroll
    for (int t = 0; t < NLX; ++t) {
        const int q = t * 64 + lane;
        x_row[t] = q / (RBC / 16);
        const int cb = (swz<RBC>(x_row[t], (q % (RBC / 16)) * 16) - x_row[t] * RBC);
        x_src[t] = xcol0 + cb / S < k ? cb : 0;
    }

    auto fetch = [&](int i0) {                        // the wavefront's buffer must have been read out
#pragma unroll
        for (int t = 0; t < NLG; ++t)
            __builtin_amdgcn_global_load_lds((glob_void*)(gbase + (size_t)min(i0 + g_row[t], m - 1) * grow + g_src[t]),
                                             (lds_void*)(gt + 1024 * t), 16, 0, 0);
#pragma unroll
        for (int t = 0; t < NLX; ++t)
            __builtin_amdgcn_global_load_lds((glob_void*)(xbase + (size_t)min(i0 + x_row[t], m - 1) * xrow + x_src[t]),
                                             (lds_void*)(xt + 1024 * t), 16, 0, 0);
    };
    auto zero_tail = [&](int i0) {                    // rows past m of the last chunk: zeros in the lane's own slots
#pragma unroll
        for (int t = 0; t < NLG; ++t)
            if (i0 + g_row[t] >= m) *reinterpret_cast<u32x4*>(gt + 1024 * t + 16 * lane) = u32x4{0u, 0u, 0u, 0u};
#pragma unroll
        for (int t = 0; t < NLX; ++t)
            if (i0 + x_row[t] >= m) *reinterpret_cast<u32x4*>(xt + 1024 * t + 16 * lane) = u32x4{0u, 0u, 0u, 0u};
    };

    const int n_chunks = (m + kChunk - 1) / kChunk;
    if (wave < n_chunks) fetch(wave * kChunk);
    for (int q = wave; q < n_chunks; q += 4) {
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");          // the chunk is in LDS
        if ((q + 1) * kChunk > m) zero_tail(q * kChunk);          // uniform
        const bool more = q + 4 < n_chunks;                        // uniform
        if constexpr (std::is_same<T, float>::value) {
            // fp32: one value per lane and MFMA step; the operands of half a chunk at a time, the next
            // chunk's loads start once the second half is in registers
            constexpr int KS = MM == 32 ? 2 : 4;      // reduction steps per MFMA
            constexpr int STEPS = kChunk / KS, HALF = STEPS / 2;
            const int irow = lane / MM, col = lane % MM;
#pragma unroll
            for (int h = 0; h < 2; ++h) {
                float av[HALF][SR][NA], bv[HALF][LC][NC];
#pragma unroll
                for (int s = 0; s < HALF; ++s) {
                    const int r = (h * HALF + s) * KS + irow;
#pragma unroll
                    for (int a = 0; a < SR; ++a)
#pragma unroll
                        for (int ua = 0; ua < NA; ++ua)
                            av[s][a][ua] = *reinterpret_cast<const float*>(gt + swz<RBG>(r, (a * BS_R + ua * MM + col) * 4));
#pragma unroll
                    for (int l = 0; l < LC; ++l)
#pragma unroll
                        for (int uc = 0; uc < NC; ++uc)
                            bv[s][l][uc] = *reinterpret_cast<const float*>(xt + swz<RBC>(r, (l * BS_C + uc * MM + col) * 4));
                }
                if (h == 1) {
                    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");   // every read of the buffer has returned
                    if (more) fetch((q + 4) * kChunk);
                }
#pragma unroll
                for (int s = 0; s < HALF; ++s)
#pragma unroll
                    for (int pq = 0; pq < NPOS; ++pq)
                        if ((mask >> pq) & 1u) {
#pragma unroll
                            for (int ua = 0; ua < NA; ++ua)
#pragma unroll
                                for (int uc = 0; uc < NC; ++uc) {
                                    if constexpr (MM == 32) acc[pq][ua][uc] = __builtin_amdgcn_mfma_f32_32x32x2f32(av[s][pq / LC][ua], bv[s][pq % LC][uc], acc[pq][ua][uc], 0, 0, 0);
                                    else                    acc[pq][ua][uc] = __builtin_amdgcn_mfma_f32_16x16x4f32(av[s][pq / LC][ua], bv[s][pq % LC][uc], acc[pq][ua][uc], 0, 0, 0);
                                }
                        }
            }
        } else {
            constexpr int KI = MM == 32 ? 16 : 32;    // rows of the chunk one MFMA reduces over
            constexpr int STEPS = kChunk / KI;
            Frag<T, 8> af[STEPS][SR][NA], bf[STEPS][LC][NC];
#pragma unroll
            for (int s = 0; s < STEPS; ++s) {
#pragma unroll
                for (int a = 0; a < SR; ++a)
#pragma unroll
                    for (int ua = 0; ua < NA; ++ua) {
                        const u32x4 v = read_operand16_swz<T, MM, RBG>(gt, s * KI, a * BS_R + ua * MM, lane);
                        af[s][a][ua].w[0] = v.x; af[s][a][ua].w[1] = v.y; af[s][a][ua].w[2] = v.z; af[s][a][ua].w[3] = v.w;
                    }
#pragma unroll
                for (int l = 0; l < LC; ++l)
#pragma unroll
                    for (int uc = 0; uc < NC; ++uc) {
                        const u32x4 v = read_operand16_swz<T, MM, RBC>(xt, s * KI, l * BS_C + uc * MM, lane);
                        bf[s][l][uc].w[0] = v.x; bf[s][l][uc].w[1] = v.y; bf[s][l][uc].w[2] = v.z; bf[s][l][uc].w[3] = v.w;
                    }
            }
            asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");       // every read of the buffer has returned
            if (more) fetch((q + 4) * kChunk);
#pragma unroll
            for (int s = 0; s < STEPS; ++s)
#pragma unroll
                for (int pq = 0; pq < NPOS; ++pq)
                    if ((mask >> pq) & 1u) {
#pragma unroll
                        for (int ua = 0; ua < NA; ++ua)
#pragma unroll
                            for (int uc = 0; uc < NC; ++uc) mfma_frag<T, MM, 8>(acc[pq][ua][uc], af[s][pq / LC][ua], bf[s][pq % LC][uc]);
                    }
        }
    }
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");              // nothing in flight into the buffer

    // PR positions a round: partial blocks of the present ones -> the wavefront's LDS area, then the
    // fixed-order sum over the four wavefronts and one contiguous store per block
    float* part = reinterpret_cast<float*>(gt);
    bool wrote = false;                               // uniform
#pragma unroll
    for (int q0 = 0; q0 < NPOS; q0 += PR) {
        const unsigned round_mask = (mask >> q0) & ((1u << PR) - 1u);
        if (round_mask == 0u) continue;
        if (wrote) __syncthreads();                   // the sums of the round before are read
        wrote = true;
#pragma unroll
        for (int j = 0; j < PR; ++j) {
            if (q0 + j >= NPOS || !((round_mask >> j) & 1u)) continue;
#pragma unroll
            for (int ua = 0; ua < NA; ++ua)
#pragma unroll
                for (int uc = 0; uc < NC; ++uc)
#pragma unroll
                    for (int e = 0; e < NE; ++e) {
                        int a, cc;
                        if constexpr (MM == 32) { a = ua * 32 + 8 * (e / 4) + 4 * (lane / 32) + e % 4; cc = uc * 32 + lane % 32; }
                        else                    { a = ua * 16 + 4 * (lane / 16) + e;                    cc = uc * 16 + lane % 16; }
                        part[j * (BS_R * LDP) + a * LDP + cc] = acc[q0 + j < NPOS ? q0 + j : 0][ua][uc][e];
                    }
        }
        __syncthreads();
#pragma unroll
        for (int j = 0; j < PR; ++j) {
            if (q0 + j >= NPOS || !((round_mask >> j) & 1u)) continue;
            const int p = plist[first + __builtin_popcount(mask & ((1u << (q0 + j)) - 1u))];
            O* dst = D + (size_t)p * (BS_R * BS_C);
            for (int e4 = threadIdx.x; e4 < BS_R * BS_C / 4; e4 += 256) {
                const int a = (e4 * 4) / BS_C, cc = (e4 * 4) % BS_C;
                f32x4 sum = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
                for (int w = 0; w < 4; ++w)
                    sum += *reinterpret_cast<const f32x4*>(lds + (size_t)w * geo::REGION + ((size_t)j * (BS_R * LDP) + (size_t)a * LDP + cc) * 4);
                store4<O>(dst + e4 * 4, sum.x, sum.y, sum.z, sum.w);
            }
        }
    }
}

// Blocks below the MFMA tile with BS_R in {1, 2, 4, 8, 16} rows (any bs_c): a lane owns one column
// of one stored block and keeps its BS_R sums.
//   Workgroup (r, t): block-row r, lane slots 64t .. 64t+63 of its cnt*bs_c (block, column) pairs in
//   storage order.  Its four wavefronts take the same slots and a quarter of the rows i each: per row
//   a lane reads its one element of X (the slots of a block are adjacent elements), and the BS_R
//   elements of G -- the same for the whole wavefront -- come through scalar registers.  The four
//   partial sums are added through LDS in fixed order.
// The reads of X are what bounds it: a wavefront instruction gathers 64 different columns of one row.
template <typename T, typename O, int BS_R>
__global__ __launch_bounds__(256) void bsr_sddmm_lanes(const T* __restrict__ G, const T* __restrict__ X,
                                                       const int32_t* __restrict__ indptr,
                                                       const int32_t* __restrict__ indices, O* __restrict__ D,
                                                       int m, int k, int n, int bs_c)
{
    constexpr int kUnroll = 8;
    __shared__ float part[4][BS_R][64];
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int r = blockIdx.x;
    const int first = indptr[r], cnt = indptr[r + 1] - first;
    const int slot0 = (int)blockIdx.y * 64;
    if (slot0 >= cnt * bs_c) return;                  // whole workgroup
    const int slot = slot0 + lane;
    const bool live = slot < cnt * bs_c;
    const int j = live ? slot / bs_c : 0, cc = live ? slot - j * bs_c : 0;
    const int p = first + j;
    const T* __restrict__ xcol = X + (size_t)indices[p] * bs_c + cc;
    const T* __restrict__ gpiece = G + (size_t)r * BS_R;

    float acc[BS_R];
#pragma unroll
    for (int a = 0; a < BS_R; ++a) acc[a] = 0.f;

    const int per_wave = (m + 3) / 4;
    const int i_begin = min(wave * per_wave, m), i_end = min(i_begin + per_wave, m);
    int i = i_begin;
    for (; i + kUnroll <= i_end; i += kUnroll) {
        float xv[kUnroll];
#pragma unroll
        for (int u = 0; u < kUnroll; ++u) xv[u] = (float)xcol[(size_t)(i + u) * k];
#pragma unroll
        for (int u = 0; u < kUnroll; ++u) {
            const T* __restrict__ g = gpiece + (size_t)(i + u) * n;   // uniform address
#pragma unroll
            for (int a = 0; a < BS_R; ++a) acc[a] = fmaf((float)g[a], xv[u], acc[a]);
        }
    }
    for (; i < i_end; ++i) {
        const float x = (float)xcol[(size_t)i * k];
        const T* __restrict__ g = gpiece + (size_t)i * n;
#pragma unroll
        for (int a = 0; a < BS_R; ++a) acc[a] = fmaf((float)g[a], x, acc[a]);
    }
#pragma unroll
    for (int a = 0; a < BS_R; ++a) part[wave][a][lane] = acc[a];
    __syncthreads();
    if (!live) return;
    for (int a = wave; a < BS_R; a += 4) {
        const float sum = ((part[0][a][lane] + part[1][a][lane]) + part[2][a][lane]) + part[3][a][lane];
        D[((size_t)p * BS_R + a) * bs_c + cc] = (O)sum;
    }
}

// Thin blocks (16 x 1, fp32) with a transposed copy XT (k x m) of X in the caller's scratch: a column of X
// is then a contiguous row, and a block-row is a small dense product
//     D[p0 .. p1)[a] = sum_i G[i][16 r + a] * XT[block column of p][i]
// that the matrix cores take 16 stored blocks at a time: MFMA 16x16x4 with M = a, N = block, K = i.
//   Workgroup (r, t): block-row r, its stored blocks 64 t .. 64 t + 63; wavefront w the 16 blocks from
//   64 t + 16 w.  The rows i go by in pieces of 256: the workgroup copies that piece of G's 16 columns
//   into LDS (64 contiguous bytes per row), every wavefront reads its 64 A operands from there (pitch
//   20 words: the four row groups of a read fall on different banks), and then walks the piece 16 rows
//   at a time: one 16-byte read of XT per lane (4 consecutive i of its block's column) feeds 4 MFMAs.
//   MFMA u of a 16-row step reduces over i = I + 4 g + u for k-group g, on both operands.
// Rows past m: G is read from row m-1 and replaced by zero, XT is read as it lies (the scratch is padded)
// and replaced by zero; lanes past the block-row's last block repeat it and store nothing.
__global__ __launch_bounds__(256, 4) void bsr_sddmm_thin16(const float* __restrict__ G, const float* __restrict__ XT,
                                                        const int32_t* __restrict__ indptr,
                                                        const int32_t* __restrict__ indices, float* __restrict__ D,
                                                        int m, int n, int mp)
{
    constexpr int kPiece = 256, kPitch = 20;
    __shared__ float gs[kPiece * kPitch];
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int r = blockIdx.x;
    const int first = indptr[r], cnt = indptr[r + 1] - first;
    const int j0 = ((int)blockIdx.y * 4 + wave) * 16;             // first block of this wavefront's 16
    if ((int)blockIdx.y * 64 >= cnt) return;                      // whole workgroup
    const bool active = j0 < cnt;                                 // uniform over the wavefront
    const int j = lane & 15, g = lane >> 4;
    const int p = first + min(j0 + j, cnt - 1);
    // XT is read with 4 consecutive lanes on the 64 contiguous bytes of one block's column (lane l: block
    // l / 4, k-group l mod 4) and moved to the MFMA's lane order (block l mod 16, k-group l / 16) by lane
    // permutes: four lanes of a quad on four different lines would quarter the load rate
    const int jl = lane >> 2, gl = lane & 3;
    const float* __restrict__ xrow = XT + (size_t)indices[first + min(j0 + jl, cnt - 1)] * mp + 4 * gl;
    const int from = (4 * j + g) * 4;                             // byte address of the source lane for ds_bpermute
    const float* __restrict__ gcols = G + (size_t)r * 16;

    f32x4 acc = {0.f, 0.f, 0.f, 0.f}, acc2 = {0.f, 0.f, 0.f, 0.f};   // two chains: even and odd steps
    for (int i0 = 0; i0 < m; i0 += kPiece) {
        if (i0 > 0) __syncthreads();                              // the piece before is read
        // rows i0 .. i0+255 of G's 16 columns -> LDS; thread t: rows t/4 + 64 q, 16 bytes at column 4 (t mod 4)
#pragma unroll
        for (int q = 0; q < kPiece / 64; ++q) {
            const int row = (tid >> 2) + 64 * q;
            const int i = i0 + row;
            f32x4 v = *reinterpret_cast<const f32x4*>(gcols + (size_t)min(i, m - 1) * n + 4 * (tid & 3));
            if (i >= m) v = f32x4{0.f, 0.f, 0.f, 0.f};
            *reinterpret_cast<f32x4*>(gs + row * kPitch + 4 * (tid & 3)) = v;
        }
        __syncthreads();
        if (!active) continue;
        float A[kPiece / 16][4];
#pragma unroll
        for (int b = 0; b < kPiece / 16; ++b)
#pragma unroll
            for (int u = 0; u < 4; ++u) A[b][u] = gs[(16 * b + 4 * g + u) * kPitch + j];
        // the reads of XT of half a piece (8 steps) are issued before the first is used; a step past m
        // repeats the last step's address and is not multiplied
        const int last_step = ((m - 1) / 16) * 16;
#pragma unroll
        for (int h = 0; h < 2; ++h) {
            u32x4 xl[8];
#pragma unroll
            for (int b = 0; b < 8; ++b) xl[b] = *reinterpret_cast<const u32x4*>(xrow + min(i0 + 16 * (8 * h + b), last_step));
#pragma unroll
            for (int b = 0; b < 8; ++b) {
                const int I = i0 + 16 * (8 * h + b);
                if (I < m) {                                      // uniform
                    f32x4 x;
                    x.x = __builtin_bit_cast(float, __builtin_amdgcn_ds_bpermute(from, (int)xl[b].x));
                    x.y = __builtin_bit_cast(float, __builtin_amdgcn_ds_bpermute(from, (int)xl[b].y));
                    x.z = __builtin_bit_cast(float, __builtin_amdgcn_ds_bpermute(from, (int)xl[b].z));
                    x.w = __builtin_bit_cast(float, __builtin_amdgcn_ds_bpermute(from, (int)xl[b].w));
                    if (I + 16 > m) {                             // uniform: the last, partial step
                        if (I + 4 * g + 0 >= m) x.x = 0.f;
                        if (I + 4 * g + 1 >= m) x.y = 0.f;
                        if (I + 4 * g + 2 >= m) x.z = 0.f;
                        if (I + 4 * g + 3 >= m) x.w = 0.f;
                    }
                    f32x4& c = (b & 1) ? acc2 : acc;
                    c = __builtin_amdgcn_mfma_f32_16x16x4f32(A[8 * h + b][0], x.x, c, 0, 0, 0);
                    c = __builtin_amdgcn_mfma_f32_16x16x4f32(A[8 * h + b][1], x.y, c, 0, 0, 0);
                    c = __builtin_amdgcn_mfma_f32_16x16x4f32(A[8 * h + b][2], x.z, c, 0, 0, 0);
                    c = __builtin_amdgcn_mfma_f32_16x16x4f32(A[8 * h + b][3], x.w, c, 0, 0, 0);
                }
            }
        }
    }
    // lane (block j, group g) holds D[p][4 g .. 4 g + 3]
    if (active && j0 + j < cnt) *reinterpret_cast<f32x4*>(D + (size_t)p * 16 + 4 * g) = acc + acc2;
}

// Any other block shape: thread e of the workgroup owns elements e, e + 256, ... of the block.
template <typename T, typename O>
__global__ __launch_bounds__(256) void bsr_sddmm_generic(const T* __restrict__ G, const T* __restrict__ X,
                                                         const int32_t* __restrict__ block_row,
                                                         const int32_t* __restrict__ indices, O* __restrict__ D,
                                                         int m, int k, int n, int bs_r, int bs_c)
{
    const int p = blockIdx.x;
    const int r = block_row[p], c = indices[p];
    for (int e = threadIdx.x; e < bs_r * bs_c; e += 256) {
        const int a = e / bs_c, cc = e - a * bs_c;
        const T* g = G + (size_t)r * bs_r + a;
        const T* x = X + (size_t)c * bs_c + cc;
        float acc = 0.f;
        for (int i = 0; i < m; ++i) acc = fmaf((float)g[(size_t)i * n], (float)x[(size_t)i * k], acc);
        D[(size_t)p * bs_r * bs_c + e] = (O)acc;
    }
}

template <typename T, typename O, int BS_R, int BS_C, int NB>
bsr_status launch_sddmm_runs(const bsr_matrix* W, int m, const void* G, const void* X, void* D, const int32_t* runs,
                             int n_runs, hipStream_t stream)
{
    typedef sddmm_geom<T, BS_R, BS_C, NB> geo;
    const size_t lds = 4 * (size_t)geo::REGION;
    static const hipError_t attr =
        hipFuncSetAttribute(reinterpret_cast<const void*>(&bsr_sddmm_mfma<T, O, BS_R, BS_C, NB>),
                            hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
    if (attr != hipSuccess) return BSR_ERR_HIP;
    hipLaunchKernelGGL((bsr_sddmm_mfma<T, O, BS_R, BS_C, NB>), dim3((unsigned)((n_runs + 7) / 8 * 8)), dim3(256), lds,
                       stream, (const T*)G, (const T*)X, W->block_row, W->indices, runs, (O*)D, m, (int)W->k,
                       (int)W->n, n_runs);
    return hipGetLastError() == hipSuccess ? BSR_OK : BSR_ERR_HIP;
}

template <typename T, typename O, int BS_R, int BS_C>
bsr_status launch_sddmm_tiles(const bsr_matrix* W, int m, const void* G, const void* X, void* D, hipStream_t stream)
{
    typedef sddmm_tile_geom<T, BS_R, BS_C> geo;
    const size_t lds = 4 * (size_t)geo::REGION;
    static const hipError_t attr =
        hipFuncSetAttribute(reinterpret_cast<const void*>(&bsr_sddmm_tiles<T, O, BS_R, BS_C>),
                            hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
    if (attr != hipSuccess) return BSR_ERR_HIP;
    hipLaunchKernelGGL((bsr_sddmm_tiles<T, O, BS_R, BS_C>), dim3((unsigned)((W->sd_n_tiles + 7) / 8 * 8)), dim3(256), lds,
                       stream, (const T*)G, (const T*)X, W->sd_tiles, W->sd_plist, (O*)D, m, (int)W->k, (int)W->n,
                       (int)W->sd_n_tiles);
    return hipGetLastError() == hipSuccess ? BSR_OK : BSR_ERR_HIP;
}

template <typename T, typename O, int BS_R, int BS_C>
bsr_status launch_sddmm_shape(const bsr_matrix* W, int m, const void* G, const void* X, void* D, hipStream_t stream)
{
    // pieces narrower than a line, many rows, and enough tiles to fill the chip: line-wide tiles
    if constexpr (sddmm_tile_geom<T, BS_R, BS_C>::NPOS > 1) {
        int sr = 0, lc = 0;
        sddmm_tile_dims(BS_R, BS_C, W->dtype, &sr, &lc);
        if (m >= 512 && W->sd_n_tiles >= 256 && W->sd_tiles && sr == sddmm_tile_geom<T, BS_R, BS_C>::SR &&
            lc == sddmm_tile_geom<T, BS_R, BS_C>::LC)
            return launch_sddmm_tiles<T, O, BS_R, BS_C>(W, m, G, X, D, stream);
    }
    constexpr int NB = BS_R * BS_C * (int)sizeof(T) <= 2048 ? 4 : 2;   // sddmm_run_blocks()
    // Sharing the piece of G pays when the rows are many; a short product finishes sooner spread over
    // more workgroups, one per stored block.
    if (m >= 512 && W->sd_n_runs >= 256 && W->sd_runs && NB == sddmm_run_blocks(BS_R, BS_C, W->dtype))
        return launch_sddmm_runs<T, O, BS_R, BS_C, NB>(W, m, G, X, D, W->sd_runs, W->sd_n_runs, stream);
    return launch_sddmm_runs<T, O, BS_R, BS_C, 1>(W, m, G, X, D, nullptr, (int)W->nnzb, stream);
}

template <typename T, typename O>
bsr_status launch_sddmm_types(const bsr_matrix* W, int m, const void* G, const void* X, void* D, hipStream_t stream)
{
    const int br = W->bs_r, bc = W->bs_c;
    BSR_MFMA_SHAPES(launch_sddmm_shape, T, O, br, bc, W, m, G, X, D, stream);
    if constexpr (std::is_same<T, float>::value && std::is_same<O, float>::value) {
        // thin blocks with the caller's scratch lent: transposed copy of X, then the matrix-core kernel
        if (mfma_thin_supports(W) && m >= 32 && W->scratch && W->scratch_bytes >= mfma_thin_scratch_bytes(W, m) &&
            ((int64_t)m + 3) * W->k < ((int64_t)1 << 30)) {
            float* XT = static_cast<float*>(W->scratch);
            const bsr_status st = launch_transpose_f32((const float*)X, XT, m, (int)W->k, stream);
            if (st != BSR_OK) return st;
            const int64_t groups = ((int64_t)W->max_row_blocks + 63) / 64;
            if (groups > 65535) return BSR_ERR_SHAPE;
            hipLaunchKernelGGL(bsr_sddmm_thin16, dim3((unsigned)W->R, (unsigned)groups), dim3(256), 0, stream,
                               (const float*)G, (const float*)XT, W->indptr, W->indices, (float*)D, m, (int)W->n,
                               (m + 3) & ~3);
            return hipGetLastError() == hipSuccess ? BSR_OK : BSR_ERR_HIP;
        }
    }
    auto lanes = [&](auto rows_tag) -> bsr_status {
        constexpr int BS_R = decltype(rows_tag)::value;
        const int64_t tiles = ((int64_t)W->max_row_blocks * bc + 63) / 64;
        if (tiles > 65535 || W->R > 0x7fffffff) return BSR_ERR_SHAPE;
        hipLaunchKernelGGL((bsr_sddmm_lanes<T, O, BS_R>), dim3((unsigned)W->R, (unsigned)tiles), dim3(256), 0, stream,
                           (const T*)G, (const T*)X, W->indptr, W->indices, (O*)D, m, (int)W->k, (int)W->n, bc);
        return hipGetLastError() == hipSuccess ? BSR_OK : BSR_ERR_HIP;
    };
    if (br == 16) return lanes(std::integral_constant<int, 16>{});
    if (br == 8) return lanes(std::integral_constant<int, 8>{});
    if (br == 4) return lanes(std::integral_constant<int, 4>{});
    if (br == 2) return lanes(std::integral_constant<int, 2>{});
    if (br == 1) return lanes(std::integral_constant<int, 1>{});
    hipLaunchKernelGGL((bsr_sddmm_generic<T, O>), dim3((unsigned)W->nnzb), dim3(256), 0, stream,
                       (const T*)G, (const T*)X, W->block_row, W->indices, (O*)D, m, (int)W->k, (int)W->n, br, bc);
    return hipGetLastError() == hipSuccess ? BSR_OK : BSR_ERR_HIP;
}

}  // namespace

extern "C" bsr_status bsr_sddmm(const bsr_matrix* W, int64_t m, const void* G_dev, const void* X_dev, void* D_dev,
                                bsr_dtype d_dtype, void* hip_stream)
{
    if (!W) return BSR_ERR_NULL;
    if (m < 0) return BSR_ERR_SHAPE;
    if (d_dtype != W->dtype && d_dtype != BSR_F32) return BSR_ERR_DTYPE;
    if (W->nnzb == 0) return BSR_OK;
    if (!D_dev || (m > 0 && (!G_dev || !X_dev))) return BSR_ERR_NULL;
    if (m * std::max<int64_t>(W->k, W->n) >= ((int64_t)1 << 31)) return BSR_ERR_SHAPE;
    if (((uintptr_t)G_dev | (uintptr_t)X_dev | (uintptr_t)D_dev) & 15u) return BSR_ERR_ALIGN;
    hipStream_t stream = (hipStream_t)hip_stream;
    order_after_upload(stream, W->plan_uploaded, W->plan_landed);
    if (W->debug) {
        const bsr_status dbg = debug_check_device_arrays(W, stream);
        if (dbg != BSR_OK) return dbg;
    }
    // m == 0 needs no special case: the kernels then read nothing and store zeros (an empty sum)
    const int mi = (int)m;
    if (W->dtype == BSR_F32) return launch_sddmm_types<float, float>(W, mi, G_dev, X_dev, D_dev, stream);
    if (W->dtype == BSR_F16) return d_dtype == BSR_F32 ? launch_sddmm_types<_Float16, float>(W, mi, G_dev, X_dev, D_dev, stream)
                                                       : launch_sddmm_types<_Float16, _Float16>(W, mi, G_dev, X_dev, D_dev, stream);
    return d_dtype == BSR_F32 ? launch_sddmm_types<__bf16, float>(W, mi, G_dev, X_dev, D_dev, stream)
                              : launch_sddmm_types<__bf16, __bf16>(W, mi, G_dev, X_dev, D_dev, stream);
}

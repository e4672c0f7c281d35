// Matrix-core kernel for products with many rows of X: LDS-staged tiles.
//
// One workgroup (4 wavefronts) owns a TM x bs_r tile of Y (TM = 4*MT*32 rows of X, one block-row
// of W) and walks the stored blocks of the block-row.  For each stored block the workgroup stages
// the W block (bs_r x bs_c) and the matching X tile (TM x bs_c, the columns block_indices[p]
// selects) in LDS with fully coalesced reads -- 8 consecutive lanes fetch one 128-byte row
// segment -- and every wavefront then reads its MFMA operands from LDS.  The W block is shared by
// the 4 wavefronts, which is the "cache the needed part of X and block_data per thread block"
// design of the paper's "Utilizing shared memory" section, here with run-time indices.
//
// Launch order: workgroups are numbered so that the 8 XCDs (which take workgroups round-robin and
// have private L2 caches) each work through their own m-tiles one after the other; inside an
// m-tile the block-rows come longest first.  Workgroups that run at the same time on one XCD then
// share an X stripe of TM rows in that XCD's L2.  The few block-rows that are much longer than the
// rest (the plan's long_rows) are started first for all m-tiles.
#include <algorithm>

#include "bsr_mfma_common.h"

using namespace bsr_dev;

namespace {

constexpr int kXcds = 8;
constexpr int kMaxGroups = 8;

// Loads whose waits the kernel places itself (why: at their use below).  Built with BSR_PLAIN_LOADS they
// are ordinary loads with compiler-placed waits: the checking build (see bsr_mfma_ksplit.hip).
#ifndef BSR_PLAIN_LOADS
__device__ __forceinline__ void load16(u32x4& dst, const unsigned char* src) { asm volatile("global_load_dwordx4 %0, %1, off" : "=v"(dst) : "v"(src)); }
__device__ __forceinline__ void load4(int& dst, const int32_t* src) { asm volatile("global_load_dword %0, %1, off" : "=v"(dst) : "v"(src)); }
#else
__device__ __forceinline__ void load16(u32x4& dst, const unsigned char* src) { dst = *reinterpret_cast<const u32x4*>(src); }
__device__ __forceinline__ void load4(int& dst, const int32_t* src) { dst = *src; }
#endif

// Slot ranges [start[g], start[g+1]) of the launch-order groups (passed by value as a kernel argument).
struct slot_groups {
    int n;
    int start[kMaxGroups + 1];
};

template <typename T, typename O, int BS_R, int BS_C, int MT, int D>
__global__ __launch_bounds__(256) void bsr_mfma_tile(const T* __restrict__ X, const T* __restrict__ data,
                                                     const int32_t* __restrict__ indices,
                                                     const int32_t* __restrict__ row_desc, O* __restrict__ Y,
                                                     int m, int k, int n, int R, int n_tiles, slot_groups groups)
{
    constexpr int MM = 32;                            // MFMA tile edge (bs_r >= 32 only)
    constexpr int NA = BS_R / MM;
    constexpr int CH = BS_C / 2;                      // a lane's contiguous run of the block's columns
    constexpr int TM = 4 * MT * MM;                   // rows of X per workgroup
    constexpr int RB = BS_C * (int)sizeof(T);         // bytes of one tile row
    constexpr int RS = RB + 16;                       // padded LDS row stride: rows shift by 4 banks
    constexpr int CPR = RB / 16;                      // 16-byte chunks per row
    constexpr int XCHUNKS = TM * CPR, WCHUNKS = BS_R * CPR;
    static_assert(RB % 16 == 0 && CH * sizeof(T) % 16 == 0, "rows and lane runs are whole 16-byte chunks");

    extern __shared__ __attribute__((aligned(16))) unsigned char lds[];   // [TM + BS_R][RS]

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int li = lane & 31, h = lane >> 5;

    // Workgroup -> (slot, m-tile).  XCD x owns m-tiles x, x+8, ...  The slots (block-rows, longest
    // first) are cut into groups; the XCD works through group after group, and inside a group
    // through its m-tiles one after the other.  Group 0 holds the few very long block-rows: they
    // run longest, so they start first for all m-tiles (otherwise the last m-tile's long rows
    // would run on alone at the end).  The other groups are sized so that a group's W blocks stay
    // in the XCD's L2 while its m-tiles pass: W is then fetched from memory once per group and
    // XCD instead of once per m-tile, at the price of re-reading the X stripe once per group.
    const int xcd = (int)(blockIdx.x % kXcds), local = (int)(blockIdx.x / kXcds);
    const int tiles_here = (n_tiles + kXcds - 1) / kXcds;   // m-tiles per XCD (the last may not exist)
    int slot = 0, tile_local = 0, rest = local;
#pragma unroll
    for (int g = 0; g < kMaxGroups; ++g) {
        const int rows_g = groups.start[g + 1] - groups.start[g];
        const int size_g = rows_g * tiles_here;
        if (g < groups.n && rest >= 0 && rest < size_g) {
            tile_local = rest / rows_g;
            slot = groups.start[g] + rest - tile_local * rows_g;
            rest = -1;
        } else if (g < groups.n && rest >= 0) {
            rest -= size_g;
        }
    }
    const int tile = tile_local * kXcds + xcd;
    if (tile >= n_tiles) return;                      // whole workgroup leaves together
    const int i_base = tile * TM;

    const int32_t* __restrict__ desc = row_desc + (size_t)slot * kRowDescWords;
    const int r = desc[0];
    const int p0 = desc[1], p1 = p0 + desc[2];

    typedef f32x16 acc_t;
    acc_t acc[NA][MT];
#pragma unroll
    for (int u = 0; u < NA; ++u)
#pragma unroll
        for (int t = 0; t < MT; ++t)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[u][t][e] = 0.f;

    // staging map: thread tid moves 16-byte chunk tid + 256*j.  The first NLX chunks per thread
    // are X rows, the next NLW the W block (NLX, NLW known at compile time, so every trip issues
    // the same loads and the oldest block in flight can be waited for alone).  A W chunk index
    // past the block is clamped to the last chunk: those threads copy that chunk a second time
    // (same bytes to the same LDS address), which keeps the staging code free of branches.
    constexpr int NLX = XCHUNKS / 256, NLW = (WCHUNKS + 255) / 256;
    static_assert(XCHUNKS % 256 == 0, "X tile is a whole number of 256-chunk passes");
    const unsigned char* xsrc[NLX];
    int xdst[NLX];
#pragma unroll
    for (int j = 0; j < NLX; ++j) {
        const int q = tid + 256 * j;
        const int row = q / CPR, cc = q - row * CPR;
        xdst[j] = row * RS + cc * 16;
        xsrc[j] = reinterpret_cast<const unsigned char*>(X + (size_t)min(i_base + row, m - 1) * (size_t)k) + cc * 16;
    }
    int wsrc[NLW], wdst[NLW];
#pragma unroll
    for (int j = 0; j < NLW; ++j) {
        const int qc = min(tid + 256 * j, WCHUNKS - 1);
        const int row = qc / CPR, cc = qc - row * CPR;
        wdst[j] = (TM + row) * RS + cc * 16;
        wsrc[j] = qc * 16;
    }
    const unsigned char* wdata = reinterpret_cast<const unsigned char*>(data);

    // D blocks are in flight from memory to registers at any time (stage d holds block p0+d,
    // p0+d+D, ...).  Past the end of the block-row the last block is fetched again.
    //
    // The loads are issued as explicit global_load instructions and waited for with an explicit
    // vmcnt: loads return in issue order, so "at most (D-1)*NL still outstanding" means the oldest
    // stage has landed while the younger ones stay in flight.  (Left to itself the compiler drains
    // every outstanding load at the loop head, which serialises memory latency and arithmetic.)
    // After the wait each staged register passes through an empty asm that redefines it, so no
    // use of the register can be scheduled ahead of the wait.
    // Each step also loads, the same way, the block-column of the block that the same stage will
    // fetch D steps later (cidx[d]); it lands together with the stage's data.
    constexpr int NL = NLX + NLW + 1;
    static_assert((D - 1) * NL <= 63, "vmcnt is a 6-bit counter");
    u32x4 xstage[D][NLX], wstage[D][NLW];
    int cidx[D];
    auto fetch = [&](int d, int p, int c) {            // data of block p (block-column c), then column of block p+D
        // past the end of the block-row every lane reads the same 16 bytes (start of block_data):
        // the count of loads in flight stays fixed, the traffic is one cache line
        const bool real = p < p1;
        p = min(p, p1 - 1);
        const unsigned char* wblk = wdata + (size_t)p * (BS_R * RB);
#pragma unroll
        for (int j = 0; j < NLW; ++j) {
            const unsigned char* src = real ? wblk + wsrc[j] : wdata;
            load16(wstage[d][j], src);
        }
#pragma unroll
        for (int j = 0; j < NLX; ++j) {
            const unsigned char* src = real ? xsrc[j] + (size_t)c * RB : wdata;
            load16(xstage[d][j], src);
        }
        const int32_t* nxt = indices + min(p + D, p1 - 1);
        load4(cidx[d], nxt);
    };
    auto stash = [&](int d) {
        asm volatile("s_waitcnt vmcnt(%0)" ::"n"((D - 1) * NL));
#pragma unroll
        for (int j = 0; j < NLW; ++j) asm volatile("" : "+v"(wstage[d][j]));
#pragma unroll
        for (int j = 0; j < NLX; ++j) asm volatile("" : "+v"(xstage[d][j]));
        asm volatile("" : "+v"(cidx[d]));
#pragma unroll
        for (int j = 0; j < NLW; ++j) *reinterpret_cast<u32x4*>(lds + wdst[j]) = wstage[d][j];
#pragma unroll
        for (int j = 0; j < NLX; ++j) *reinterpret_cast<u32x4*>(lds + xdst[j]) = xstage[d][j];
    };

    const unsigned char* xl = lds + (size_t)(wave * MT * MM + li) * RS + h * (CH * (int)sizeof(T));
    const unsigned char* wl = lds + (size_t)(TM + li) * RS + h * (CH * (int)sizeof(T));
    auto compute = [&]() {
        Frag<T, CH> wf[NA], xf[MT];
#pragma unroll
        for (int u = 0; u < NA; ++u) wf[u].load(reinterpret_cast<const T*>(wl + (size_t)u * MM * RS));
#pragma unroll
        for (int t = 0; t < MT; ++t) xf[t].load(reinterpret_cast<const T*>(xl + (size_t)t * MM * RS));
#pragma unroll
        for (int u = 0; u < NA; ++u)
#pragma unroll
            for (int t = 0; t < MT; ++t) mfma_frag<T, MM, CH>(acc[u][t], wf[u], xf[t]);
    };

    // blocks p+1 .. p+D travel from memory into registers while block p is multiplied out of LDS
    if (p0 < p1) {
#pragma unroll
        for (int d = 0; d < D; ++d) {                 // the first D block-columns come from the descriptor
            const int j0 = min(d, p1 - 1 - p0);
            fetch(d, p0 + d, j0 < kRowDescCols ? desc[kRowDescColsAt + j0] : indices[p0 + j0]);
        }
        for (int p = p0; p < p1; p += D) {
#pragma unroll
            for (int d = 0; d < D; ++d) {
                // every trip does all D steps (a step past the end re-stages the last block and
                // skips the arithmetic), so the loads in flight are the same on every path
                stash(d);
                __syncthreads();                      // tile of block p+d visible
                fetch(d, p + d + D, __builtin_amdgcn_readfirstlane(cidx[d]));
                if (p + d < p1) compute();            // uniform over the workgroup
                __syncthreads();                      // everyone done reading before the next stash
            }
        }
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");   // the re-fetched tail blocks
    }

    // Epilogue.  A lane holds 4 consecutive columns of one row of Y per accumulator group; stored
    // directly that is 8..16 bytes per lane and row.  Instead every wavefront transposes its
    // MT*32 x bs_r result through its own slice of LDS (the staging area is free after the loop's
    // last barrier) and stores whole rows of the tile: OC consecutive lanes write one row's bs_r
    // outputs as 16-byte pieces, i.e. full 128-byte lines for a 64-wide fp16 tile.
    constexpr int OB = BS_R * (int)sizeof(O);         // bytes of one output row of the tile
    constexpr int OS = OB + 16;                       // padded LDS stride
    constexpr int OC = OB / 16;                       // 16-byte pieces per output row
    constexpr int RPP = 64 / OC;                      // rows one wavefront stores per pass
    static_assert(OB % 16 == 0 && 64 % OC == 0 && (MT * MM) % RPP == 0, "output tile splits into 16-byte pieces");
    unsigned char* ol = lds + (size_t)wave * (MT * MM) * OS;
#pragma unroll
    for (int t = 0; t < MT; ++t)
#pragma unroll
        for (int u = 0; u < NA; ++u)
#pragma unroll
            for (int g = 0; g < 4; ++g)
                store4<O>(reinterpret_cast<O*>(ol + (size_t)(t * MM + li) * OS) + u * 32 + 8 * g + 4 * h,
                          acc[u][t][4 * g], acc[u][t][4 * g + 1], acc[u][t][4 * g + 2], acc[u][t][4 * g + 3]);
    // same wavefront wrote and now reads: its LDS operations complete in order, no barrier needed
    wave_lds_fence();
    unsigned char* ybytes = reinterpret_cast<unsigned char*>(Y + (size_t)r * BS_R);
    const int orow = lane / OC, opiece = lane - orow * OC;
#pragma unroll
    for (int pass = 0; pass < MT * MM / RPP; ++pass) {
        const int row = pass * RPP + orow;
        const u32x4 v = *reinterpret_cast<const u32x4*>(ol + (size_t)row * OS + opiece * 16);
        const int i = i_base + wave * (MT * MM) + row;
        if (i < m) __builtin_nontemporal_store(v, reinterpret_cast<u32x4*>(ybytes + (size_t)i * (size_t)n * sizeof(O) + opiece * 16));
    }
}

template <typename T, typename O, int BS_R, int BS_C>
bsr_status launch_tile_shape(const spmm_args& a, const tune_opts& tune)
{
    if constexpr (BS_R < 32) {
        return BSR_ERR_UNSUPPORTED;
    } else {
        const bsr_matrix* W = a.W;
        const int m = (int)a.m, n = (int)W->n, k = (int)W->k, R = W->R;
        auto go = [&](auto mt_tag, auto d_tag) -> bsr_status {
            constexpr int MT = decltype(mt_tag)::value;
            constexpr int D = decltype(d_tag)::value;
            constexpr int TM = 4 * MT * 32;
            const int n_tiles = (m + TM - 1) / TM;
            // groups: the long rows, then runs of slots holding about `target` stored blocks each
            // (a group's W: target * block bytes, chosen near 1.5 MB of the 4 MB L2)
            // (slots before a.first_slot are left out: another kernel multiplies those block-rows)
            slot_groups groups{};
            const int first = std::min(std::max(a.first_slot, 0), R);
            if (first >= R) return BSR_OK;
            {
                const int n_long = std::max(W->long_rows, first);
                const size_t block_bytes = (size_t)BS_R * BS_C * sizeof(T);
                int64_t target = tune.b > 0 ? tune.b : (int64_t)((3u << 19) / block_bytes);
                if (target < 1) target = 1;
                int g = 0;
                groups.start[0] = first;
                if (n_long > first) groups.start[++g] = n_long;
                int64_t acc_blocks = 0;
                for (int s = n_long; s < R; ++s) {
                    acc_blocks += W->slot_blocks[(size_t)s];
                    if (acc_blocks >= target && g < kMaxGroups - 1 && s + 1 < R) { groups.start[++g] = s + 1; acc_blocks = 0; }
                }
                groups.start[++g] = R;
                groups.n = g;
                for (int q = g + 1; q <= kMaxGroups; ++q) groups.start[q] = R;
            }
            const int64_t blocks = (int64_t)((n_tiles + kXcds - 1) / kXcds) * kXcds * (R - first);
            if (blocks >= ((int64_t)1 << 31) || blocks * 256 >= ((int64_t)1 << 32)) return BSR_ERR_SHAPE;
            const size_t lds_stage = (size_t)(TM + BS_R) * (BS_C * sizeof(T) + 16);
            const size_t lds_out = (size_t)TM * (BS_R * sizeof(O) + 16);
            const size_t lds = lds_stage > lds_out ? lds_stage : lds_out;
            if (lds > 48 * 1024) {                    // above the default dynamic-LDS limit: raise it once
                static const hipError_t attr = hipFuncSetAttribute(
                    reinterpret_cast<const void*>(&bsr_mfma_tile<T, O, BS_R, BS_C, MT, D>),
                    hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
                if (attr != hipSuccess) return BSR_ERR_HIP;
            }
            hipLaunchKernelGGL((bsr_mfma_tile<T, O, BS_R, BS_C, MT, D>), dim3((unsigned)blocks), dim3(256), lds, a.stream,
                               (const T*)a.X, (const T*)W->data, W->indices, W->row_desc, (O*)a.Y, m, k, n, R, n_tiles,
                               groups);
            return hipGetLastError() == hipSuccess ? BSR_OK : BSR_ERR_HIP;
        };
        const int depth = tune.a > 0 ? tune.a : 2;
        if (tune.mt == 1) {
            if (depth == 1) return go(std::integral_constant<int, 1>{}, std::integral_constant<int, 1>{});
            if (depth == 2) return go(std::integral_constant<int, 1>{}, std::integral_constant<int, 2>{});
            if (depth == 3) return go(std::integral_constant<int, 1>{}, std::integral_constant<int, 3>{});
            return go(std::integral_constant<int, 1>{}, std::integral_constant<int, 4>{});
        }
        // two tiles along m: at most two blocks in flight -- a third does not fit the register file for
        // the largest fp32 blocks, and the loads are written in assembly, so a spilled register that a
        // load has not filled yet would store garbage
        if (depth == 1) return go(std::integral_constant<int, 2>{}, std::integral_constant<int, 1>{});
        return go(std::integral_constant<int, 2>{}, std::integral_constant<int, 2>{});
    }
}

}  // namespace

bsr_status launch_mfma_tile(const spmm_args& a, const tune_opts& t)
{
    BSR_MFMA_DISPATCH(launch_tile_shape, a.W, a.y_dtype, a, t);
    return BSR_ERR_UNSUPPORTED;
}

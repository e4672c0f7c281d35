// Matrix-core kernel for the few very long block-rows of a matrix with 64x64 blocks of a 16-bit type.
//
// The paper's "Utilizing shared memory" design gives a thread block a tile of Y and caches the parts
// of X and of block_data that tile needs; its Discussion names block-rows of very different length
// as what hurts most.  A handful of block-rows that hold most of the stored blocks also share most
// of their block-columns, so here they are multiplied together: a workgroup owns 64 rows of X times
// a GROUP of up to 8 such block-rows and walks the union of the group's block-columns in ascending
// order.  The 64x64 tile of X of a block-column is staged in LDS once and multiplied with the stored
// block of every row of the group that has one there: X is fetched once per group instead of once
// per stored block.  The other block-rows stay with the tile kernel (bsr_mfma_tile.hip), which is
// launched for the slots behind the grouped ones.
//
// Plan (bsr_create).  The grouped rows are the leading slots of the longest-first order that store
// at least kHeavyMin blocks, at most 8 per group and kMaxGroups groups, dealt out so that the groups
// hold about equal numbers of blocks; inside a group the rows come longest first.  A group's work is a
// stream of 8 KiB tiles -- the X tile of a block-column, then the stored blocks of that column -- cut
// into WINDOWS of at most kWin tiles: whole columns, except that a column with more blocks than fit is
// continued in the next window with its X tile staged again.  One 16-word record per window:
//   word 0   stored blocks per row of the group in this window, 4 bits each (row j at bits 4j..4j+3)
//   word 1   tiles in the window (bits 0-3), X tiles among them (bits 4-7)
//   word 2   for the window's i-th stored block, 4 bits each: which of the window's X tiles it multiplies
//   word 4.. the tiles: first the X tiles (0x80000000 | block-column), then the stored blocks
//            (stored-block number) sorted by row of the group
//
// Workgroup: 12 wavefronts, three per SIMD.  Wavefront j < 8 multiplies the group's row j; wavefronts
// 8-11 only move tiles.  (A wavefront that issues loads waits for the memory pipeline to take them,
// about 130 cycles per 1 KiB load while a window streams in; one that multiplied as well would be the
// last at every barrier.)
//
// Data movement.  Tiles go from global memory straight into LDS (global_load_lds_dwordx4: no staging
// registers).  The ring holds three windows of kWin slots, window w in the slots (w mod 3) * kWin ..;
// each of the four moving wavefronts takes a quarter (16 rows) of every tile.  Loads complete in issue
// order: before window w is multiplied a moving wavefront waits until only its loads of window w+1 are
// outstanding, then the workgroup meets at a barrier -- which also says that everybody is done with
// window w-1 -- and the loads of window w+2 are issued into the slots of window w-1.  A 16-byte piece
// q of row i of a tile lies at piece position q ^ (i mod 8) of its 128-byte LDS row, which makes the
// operand reads of 16 consecutive rows at one k offset conflict-free without padding.  The window
// records travel the same way, 64 at a time, into an 8 KiB record area in front of the ring, and are
// read from there one word per lane (scalar loads from global memory cost a cache miss per window on
// the critical path).
//
// Arithmetic.  A wavefront multiplies whole 64x64 blocks of its row: v_mfma_f32_16x16x32 on 4x4 tiles, 16
// independent accumulators (64 registers per lane), the accumulator a block adds to known at compile
// time.  It holds the operands of one k half of a block at a time (4 tiles of the block, 4 of X) in each
// of two register sets; while one half is multiplied (16 MFMAs) the eight LDS reads of the half after
// the next are interleaved with the first eight of them.  Every stored block costs 16 KiB of LDS reads
// (quadrants shared by four wavefronts cost 32 KiB and twice the instructions per flop).
//
// Measured on the 8192^3 power-law workload (16 grouped rows = 573 of 819 blocks): this kernel fetches
// 221 MB from beyond L2 where the tile kernel fetches 601 MB for the same rows, and takes about 65 us
// for them against 105 us; with the tile kernel for the other rows the product takes 117 us instead of
// 135 us and fetches 405 instead of 825 MB.  What bounds it: a workgroup streams 3.3 MB of tiles per 64
// rows of X, and a CU takes in about 30 bytes per clock while its LDS also serves the operand reads.
#include <algorithm>
#include <numeric>

#include "bsr_mfma_common.h"

using namespace bsr_dev;

namespace {

constexpr int kXcds = 8;
constexpr int kG = 8;                                 // block-rows per group
constexpr int kSub = 64;                              // rows of X per workgroup
constexpr int kTileBytes = 8192;                      // a staged tile: 64 rows x 128 bytes
constexpr int kSlots = 19;                            // ring slots: 3 windows of kWin, and one that is only ever read
#ifndef GRP_KWIN
#define GRP_KWIN 6
#define GRP_RING 3
#endif
constexpr int kWin = GRP_KWIN;                        // tiles per window at most
constexpr int kRingWin = GRP_RING;                    // windows the ring holds: one in use, the others on their way
constexpr int kRecLds = 128;                          // window records kept in LDS: two halves of 64, refilled in turn
constexpr int kRec = 16;                              // words per window record
constexpr int kRecTilesAt = 4;
constexpr int kDescWords = 16;                        // group descriptor: 8 rows, first record, windows, 0...
constexpr int kRecBytes = kRecLds * kRec * 4;         // 8 KiB
constexpr int kLdsBytes = kRecBytes + kSlots * kTileBytes;
constexpr int kHeavyMin = 8;                          // a grouped block-row stores at least this many blocks
constexpr int kMaxGroups = 2;
static_assert(kRingWin * kWin <= kSlots && (kRingWin == 2 || kRingWin == 3) && kWin <= 9, "the windows fit the ring; a record lists at most 9 tiles");

template <int N>
__device__ __forceinline__ void wait_vm()
{
    asm volatile("s_waitcnt vmcnt(%0)" ::"n"(N) : "memory");
}

// Returns when at most the loads of `tiles` tiles (two per tile and moving wavefront, the youngest) are still in flight.
__device__ __forceinline__ void wait_all_but_tiles(int tiles)
{
    switch (tiles) {
        case 0: wait_vm<0>(); break;
        case 1: wait_vm<2>(); break;
        case 2: wait_vm<4>(); break;
        case 3: wait_vm<6>(); break;
        case 4: wait_vm<8>(); break;
        case 5: wait_vm<10>(); break;
        default: wait_vm<12>(); break;
    }
}

// Workgroup barrier that neither the compiler nor the scheduler moves memory operations across.
__device__ __forceinline__ void barrier() { asm volatile("s_barrier" ::: "memory"); }

template <typename T>
__device__ __forceinline__ f32x4 mfma16(const u32x4& a, const u32x4& b, const f32x4& c)
{
    if constexpr (std::is_same<T, f16_t>::value)
        return __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(f16x8, a), __builtin_bit_cast(f16x8, b), c, 0, 0, 0);
    else
        return __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, a), __builtin_bit_cast(bf16x8, b), c, 0, 0, 0);
}

// A wavefront's operand of one staged tile: 2 tiles of 16 rows x 2 k-steps, 16 bytes each.
struct frag4 {
    u32x4 v[2][2];
    __device__ __forceinline__ void load(const unsigned char* tile, unsigned off)
    {
#pragma unroll
        for (int u = 0; u < 2; ++u)
#pragma unroll
            for (int ks = 0; ks < 2; ++ks) v[u][ks] = *reinterpret_cast<const u32x4*>(tile + ((off + u * 2048u) ^ (ks * 64u)));
    }
};

template <typename O>
struct out_geom {
    static constexpr int OB = 64 * (int)sizeof(O);    // bytes of one output row of a block-row
    static constexpr int OS = OB + 16;                // padded LDS stride
    static constexpr int OUT = 64 * OS;               // one block-row's staging buffer
    static_assert(kG * OUT <= kSlots * kTileBytes, "the group's results fit the ring");
};

template <typename T, typename O>
__global__ __launch_bounds__(768) void bsr_mfma_group(const T* __restrict__ X, const T* __restrict__ data,
                                                      const int32_t* __restrict__ recs,
                                                      const int32_t* __restrict__ gdesc, O* __restrict__ Y,
                                                      int m, int k, int n, int n_groups, int n_sub)
{
    typedef out_geom<O> geo;
    typedef __attribute__((address_space(3))) void lds_void;
    typedef __attribute__((address_space(1))) const void glob_void;
    extern __shared__ __attribute__((aligned(1024))) unsigned char lds[];
    unsigned char* const ring = lds + kRecBytes;      // records first, then the ring of tiles

    // 12 wavefronts, three per SIMD.  Wavefront j < 8 multiplies the group's row j (the rows come longest
    // first); wavefronts 8-11 only move tiles, each a quarter (16 rows) of every tile: a wavefront that
    // issues loads waits for the memory pipeline to take them (about 100 cycles per 1 KiB load while a
    // window streams in), and a wavefront that multiplied as well would be the last at every barrier.
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const bool producer = wave >= kG;
    const int pq = wave & 3;

    // workgroup -> (64-row sub-tile of X, group): XCD x (which receives the workgroups b = x mod 8) takes the
    // sub-tiles x, x+8, ..., and the groups of a sub-tile follow each other on that XCD, so the second
    // group finds the X tiles the first one fetched in the XCD's L2
    const int xcd = (int)(blockIdx.x % kXcds), local = (int)(blockIdx.x / kXcds);
    const int sub = (local / n_groups) * kXcds + xcd, g = local % n_groups;
    if (sub >= n_sub) return;                         // whole workgroup: the grid is padded to whole rounds of XCDs
    const int32_t* __restrict__ gd = gdesc + (size_t)g * kDescWords;   // uniform
    int rows[kG];
#pragma unroll
    for (int j = 0; j < kG; ++j) rows[j] = gd[j];
    const int n_win = gd[9];
    const int32_t* __restrict__ rec = recs + (size_t)gd[8] * kRec;

    // ---- moving tiles: wavefront 4+q takes rows 16q .. 16q+15 of every tile, two 1 KiB loads ----
    // load i covers rows 16q + 8i .. +7: lane l moves the 16 bytes at piece position l mod 8 of row
    // 16q + 8i + l div 8, which hold the row's piece (position ^ row mod 8)
    const unsigned char* Xb = reinterpret_cast<const unsigned char*>(X);
    const unsigned char* Wb = reinterpret_cast<const unsigned char*>(data);
    const int lrow = lane >> 3;
    const unsigned piece = (unsigned)((lane & 7) ^ lrow) * 16u;
    const unsigned row_bytes = (unsigned)k * (unsigned)sizeof(T);
    // byte offsets of the lane's two pieces (m*k*2 < 2^32); rows past m repeat row m-1, their results are never stored
    const int prow0 = 16 * pq + lrow, prow1 = prow0 + 8;
    const unsigned x_off0 = (unsigned)min(sub * kSub + prow0, m - 1) * row_bytes + piece;
    const unsigned x_off1 = (unsigned)min(sub * kSub + prow1, m - 1) * row_bytes + piece;
    const unsigned w_off0 = (unsigned)prow0 * 128u + piece, w_off1 = (unsigned)prow1 * 128u + piece;
    // Window w lives in the kWin slots starting at slot (w mod 3) * kWin, tile i in the i-th of them.
    // A window's record is read from LDS one word per lane (rv: lanes 16q .. 16q+15 hold record w+q) and
    // its words are taken out with lane reads; `at` = lane of the record's word 0.
    auto issue = [&](int rv, int at, int w3) __attribute__((always_inline)) {   // the tiles of one window
        const int nt = __builtin_amdgcn_readlane(rv, at + 1) & 15;
        unsigned char* dst = ring + w3 * (kWin * kTileBytes) + pq * 2048;
        for (int i = 0; i < nt; ++i, dst += kTileBytes) {
            const int code = __builtin_amdgcn_readlane(rv, at + kRecTilesAt + i);
            if (code < 0) {                           // X tile of a block-column
                const unsigned char* base = Xb + (size_t)(code & 0x7fffffff) * 128u;
                __builtin_amdgcn_global_load_lds((glob_void*)(base + x_off0), (lds_void*)dst, 16, 0, 0);
                __builtin_amdgcn_global_load_lds((glob_void*)(base + x_off1), (lds_void*)(dst + 1024), 16, 0, 0);
            } else {                                  // a stored block
                const unsigned char* base = Wb + (size_t)code * (size_t)kTileBytes;
                __builtin_amdgcn_global_load_lds((glob_void*)(base + w_off0), (lds_void*)dst, 16, 0, 0);
                __builtin_amdgcn_global_load_lds((glob_void*)(base + w_off1), (lds_void*)(dst + 1024), 16, 0, 0);
            }
        }
    };
    // 64 records (4 KiB) into their half of the record area, 1 KiB per moving wavefront; pieces past the
    // group's last record repeat its last piece (never used)
    const int last_piece = n_win * (kRec / 4) - 1;
    auto load_records = [&](int chunk) __attribute__((always_inline)) {
        const int pc = min(chunk * 256 + pq * 64 + lane, last_piece);
        __builtin_amdgcn_global_load_lds((glob_void*)(reinterpret_cast<const unsigned char*>(rec) + (size_t)pc * 16),
                                         (lds_void*)(lds + (chunk & 1) * (kRecBytes / 2) + pq * 1024), 16, 0, 0);
    };
    auto read_records = [&](int w) -> int {           // lane l: word l mod 16 of record w + l div 16
        const int q = (w + (lane >> 4)) & (kRecLds - 1);
        return *reinterpret_cast<const int*>(lds + q * (kRec * 4) + (lane & 15) * 4);
    };

    // ---- multiplying: a whole 64x64 block per wavefront ----
    // operand of a 16x16x32 MFMA: lane l supplies row (l mod 16) of its 16-row tile, k elements
    // 32*ks + 8*(l div 16) .. +7 = piece 4*ks + l div 16 of the row; ks = 1 differs by XOR 64 bytes.
    // A wavefront keeps the operands of one k half of a block at a time (4 tiles of the block, 4 of X):
    // while one half is multiplied (16 MFMAs on 16 accumulators) the same half of the next block is read.
    const int fr = lane & 15, fq = lane >> 4;
    const unsigned f_off = (unsigned)fr * 128u + (unsigned)((fq ^ (fr & 7)) * 16);
    struct half_frag {
        u32x4 w[4], x[4];
        __device__ __forceinline__ void load(const unsigned char* wt, const unsigned char* xt, unsigned off)
        {
#pragma unroll
            for (int t = 0; t < 4; ++t) w[t] = *reinterpret_cast<const u32x4*>(wt + off + t * 2048u);
#pragma unroll
            for (int t = 0; t < 4; ++t) x[t] = *reinterpret_cast<const u32x4*>(xt + off + t * 2048u);
        }
    };
    f32x4 acc[4][4];                                  // [16 rows of the block][16 rows of X]
#pragma unroll
    for (int ct = 0; ct < 4; ++ct)
#pragma unroll
        for (int rt = 0; rt < 4; ++rt) acc[ct][rt] = f32x4{0.f, 0.f, 0.f, 0.f};
    auto multiply = [&](const half_frag& f) __attribute__((always_inline)) {
#pragma unroll
        for (int ct = 0; ct < 4; ++ct)
#pragma unroll
            for (int rt = 0; rt < 4; ++rt) acc[ct][rt] = mfma16<T>(f.w[ct], f.x[rt], acc[ct][rt]);
    };

    // the first 128 records, then windows 0 and 1, are on their way before the loop
    if (producer) {
        load_records(0);
        if (n_win > 64) load_records(1);
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    }
    barrier();
    int rv = read_records(0);
    if (producer) {
        issue(rv, 0, 0);
        if (kRingWin == 3 && n_win > 1) issue(rv, 16, 1);
    }

    int w3 = 0;                                       // w mod 3
    for (int w = 0; w < n_win; ++w) {
        if (producer) {
            const int next_tiles = kRingWin == 3 && w + 1 < n_win ? (__builtin_amdgcn_readlane(rv, 17) & 15) : 0;
            wait_all_but_tiles(next_tiles);           // this wavefront's share of window w has landed
        }
        barrier();                                    // ... everybody's has, and everybody is done with window w-1
        const int rv_next = read_records(w + 1);      // used in the next trip
        if (producer) {
            // every 64 windows the half of the record area that was used up takes the records 64 .. 127 ahead
            // (loads complete in order, so they have landed, for everybody, many windows before they are read)
            if ((w & 63) == 0 && w > 0 && w + 64 < n_win) load_records((w >> 6) + 1);
            // the window kRingWin - 1 ahead takes the slots of window w-1
            if (w + kRingWin - 1 < n_win) issue(rv, 16 * (kRingWin - 1), w3 == 0 ? kRingWin - 1 : w3 - 1);
        }
        const unsigned all_counts = (unsigned)__builtin_amdgcn_readlane(rv, 0);
        const int info = __builtin_amdgcn_readlane(rv, 1);
        const unsigned xis = (unsigned)__builtin_amdgcn_readlane(rv, 2);
        const int nx = (info >> 4) & 15;
        // this wavefront's row: its count, and the blocks of the rows before it (the window's blocks are sorted by row)
        const int c = producer ? 0 : (int)((all_counts >> (4 * (wave & 7))) & 15u);
        const unsigned below = all_counts & ((1u << (4 * (wave & 7))) - 1u);
        const unsigned pairs = (below & 0x0f0f0f0fu) + ((below >> 4) & 0x0f0f0f0fu);
        const int before = (int)((pairs * 0x01010101u) >> 24);
        if (c > 0) {                                  // uniform
            const unsigned char* wb = ring + w3 * (kWin * kTileBytes);
            const unsigned char* wt = wb + (nx + before) * kTileBytes;       // the row's first block in this window
            unsigned xsel = xis >> (4 * before);      // which X tile each of its blocks multiplies, 4 bits each
            // fa / fb: k elements 0-31 / 32-63 of the block in turn.  While one half is multiplied the other
            // half's operands are read: 8 LDS reads interleaved with the first 8 of the 16 MFMAs.
            half_frag fa, fb;
            fa.load(wt, wb + (xsel & 15u) * kTileBytes, f_off);
            for (int i = 0; i < c; ++i) {
                // behind the row's last block of the window the reads repeat that block's and are dropped
                const bool more = i + 1 < c;
                const unsigned char* wn = more ? wt + kTileBytes : wt;
                const unsigned xnext = more ? xsel >> 4 : xsel;
                __builtin_amdgcn_sched_barrier(0);
                fb.load(wt, wb + (xsel & 15u) * kTileBytes, f_off ^ 64u);
                multiply(fa);
#pragma unroll
                for (int q = 0; q < 8; ++q) {
                    __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);   // one MFMA
                    __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);   // one LDS read
                }
                __builtin_amdgcn_sched_group_barrier(0x008, 8, 0);
                __builtin_amdgcn_sched_barrier(0);
                fa.load(wn, wb + (xnext & 15u) * kTileBytes, f_off);
                multiply(fb);
#pragma unroll
                for (int q = 0; q < 8; ++q) {
                    __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
                    __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
                }
                __builtin_amdgcn_sched_group_barrier(0x008, 8, 0);
                __builtin_amdgcn_sched_barrier(0);
                wt = wn;
                xsel = xnext;
            }
        }
        w3 = w3 == kRingWin - 1 ? 0 : w3 + 1;
        rv = rv_next;
    }

    // ---- epilogue: the group's block-rows through LDS (the ring is free: no load is outstanding), whole rows to Y ----
    // result of a 16x16 tile: lane l holds X row (l mod 16), 4 consecutive columns 4*(l div 16) ..
    asm volatile("s_waitcnt vmcnt(0) lgkmcnt(0)" ::: "memory");
    barrier();
    {
        // wavefront j holds row j's 64x64 result: tile (ct, rt) = columns 16ct.. of the block-row, rows 16rt.. of X
        int my_row = -1;
#pragma unroll
        for (int j = 0; j < kG; ++j) my_row = wave == j ? rows[j] : my_row;
        if (my_row >= 0) {                            // uniform
            unsigned char* ob = ring + wave * geo::OUT;
#pragma unroll
            for (int ct = 0; ct < 4; ++ct)
#pragma unroll
                for (int rt = 0; rt < 4; ++rt) {
                    const int orow = 16 * rt + fr, ocol = 16 * ct + 4 * fq;
                    store4<O>(reinterpret_cast<O*>(ob + orow * geo::OS) + ocol, acc[ct][rt][0], acc[ct][rt][1],
                              acc[ct][rt][2], acc[ct][rt][3]);
                }
        }
    }
    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
    barrier();
    const int i0 = sub * kSub;
    constexpr int PPR = geo::OB / 16;                 // 16-byte pieces per output row
    constexpr int RPP = 512 / PPR;                    // rows per pass of the first 512 threads (the moving wavefronts are done)
    if (tid >= 512) return;
#pragma unroll
    for (int j = 0; j < kG; ++j) {
        if (rows[j] >= 0) {
            const unsigned char* ob = ring + j * geo::OUT;
            unsigned char* yb = reinterpret_cast<unsigned char*>(Y + (size_t)rows[j] * 64);
#pragma unroll
            for (int pass = 0; pass < 64 / RPP; ++pass) {
                const int row = pass * RPP + tid / PPR, pc = tid % PPR;
                const u32x4 v = *reinterpret_cast<const u32x4*>(ob + row * geo::OS + pc * 16);
                if (i0 + row < m)
                    __builtin_nontemporal_store(v, reinterpret_cast<u32x4*>(yb + (size_t)(i0 + row) * (size_t)n * sizeof(O) + pc * 16));
            }
        }
    }
}

}  // namespace

size_t group_plan_words(int64_t R, int32_t bs_r, int32_t bs_c, int64_t nnzb)
{
    if (bs_r != 64 || bs_c != 64) return 0;
    (void)R;
    // a window holds at least one stored block, so there are at most nnzb records
    return (size_t)kRec * (size_t)nnzb + (size_t)kMaxGroups * kDescWords + 256;
}

bool mfma_group_supports(const bsr_matrix* W) { return W->grp_n > 0; }

void build_group_plan(bsr_matrix* W, const int32_t* ptr, const int32_t* idx, size_t* words)
{
    W->grp_n = 0;
    W->grp_slots = 0;
    W->grp_blocks = 0;
    W->grp_host.clear();
    if (W->bs_r != 64 || W->bs_c != 64 || (W->dtype != BSR_F16 && W->dtype != BSR_BF16) || W->R <= 0 || W->nnzb <= 0) return;
    const int R = W->R;
    const int32_t* order = W->staging.data();         // block-rows by stored-block count, longest first: the plan's slot order
    auto count = [&](int r) { return ptr[r + 1] - ptr[r]; };
    const int min_count = W->env_tune.variant == 5 && W->env_tune.b > 0 ? W->env_tune.b : kHeavyMin;
    int max_groups = W->env_tune.variant == 5 && W->env_tune.nw > 0 ? W->env_tune.nw : kMaxGroups;
    max_groups = std::min(max_groups, kMaxGroups);
    int H = 0;
    while (H < R && H < kG * max_groups && count(order[H]) >= min_count) ++H;
    if (H == 0) return;
    const int n_groups = (H + kG - 1) / kG;
    // deal the rows out longest first, each to the group with the fewest blocks that still has room
    std::vector<std::vector<int>> members((size_t)n_groups);
    std::vector<int64_t> load((size_t)n_groups, 0);
    for (int s = 0; s < H; ++s) {
        int best = -1;
        for (int q = 0; q < n_groups; ++q)
            if ((int)members[(size_t)q].size() < kG && (best < 0 || load[(size_t)q] < load[(size_t)best])) best = q;
        members[(size_t)best].push_back(order[s]);
        load[(size_t)best] += count(order[s]);
        W->grp_blocks += count(order[s]);
    }
    std::vector<int32_t> desc((size_t)n_groups * kDescWords, 0), recs;
    for (int q = 0; q < n_groups; ++q) {
        // rows of the group longest first (the members were dealt out in that order): wavefront j takes row j
        std::vector<int32_t> rows(kG, -1);
        for (size_t j = 0; j < members[(size_t)q].size(); ++j) rows[j] = members[(size_t)q][j];
        int32_t* d = desc.data() + (size_t)q * kDescWords;
        for (int j = 0; j < kG; ++j) d[j] = rows[(size_t)j];
        d[8] = (int32_t)(recs.size() / kRec);
        // the group's stored blocks as (block-column, row of the group, stored-block number), by column
        // (storage order inside a block-row is free, and a row may store a column twice)
        struct entry { int32_t col, j, p; };
        std::vector<entry> all;
        for (size_t j = 0; j < rows.size(); ++j)
            for (int32_t p = rows[j] < 0 ? 0 : ptr[rows[j]]; rows[j] >= 0 && p < ptr[rows[j] + 1]; ++p) all.push_back({idx[p], (int32_t)j, p});
        std::stable_sort(all.begin(), all.end(), [](const entry& a, const entry& b) { return a.col < b.col; });
        // windows: X tile of a column, then its blocks; a column that does not fit what is left of the
        // window opens the next one, and a column with more than kWin-1 blocks continues there
        struct wblock { int32_t j, p, xi; };
        std::vector<int32_t> xcols;
        std::vector<wblock> wb;
        auto close = [&]() {
            if (wb.empty()) return;
            std::stable_sort(wb.begin(), wb.end(), [](const wblock& a, const wblock& b) { return a.j < b.j; });
            int32_t rc[kRec] = {0};
            for (size_t i = 0; i < wb.size(); ++i) {
                rc[0] += 1 << (4 * wb[i].j);
                rc[2] |= wb[i].xi << (4 * (int)i);
            }
            rc[1] = (int32_t)(xcols.size() + wb.size()) | ((int32_t)xcols.size() << 4);
            int t = kRecTilesAt;
            for (int32_t c : xcols) rc[t++] = (int32_t)(0x80000000u | (uint32_t)c);
            for (const auto& b : wb) rc[t++] = b.p;
            recs.insert(recs.end(), rc, rc + kRec);
            xcols.clear();
            wb.clear();
        };
        size_t at = 0;
        while (at < all.size()) {
            size_t end = at;
            while (end < all.size() && all[end].col == all[at].col) ++end;
            while (at < end) {
                const int room = kWin - (int)(xcols.size() + wb.size());
                const int want = (int)std::min<size_t>(end - at, (size_t)(kWin - 1));
                if (room < 1 + want) { close(); continue; }
                xcols.push_back(all[at].col);
                for (int i = 0; i < want; ++i, ++at) wb.push_back({all[at].j, all[at].p, (int32_t)xcols.size() - 1});
            }
        }
        close();
        d[9] = (int32_t)(recs.size() / kRec) - d[8];
    }
    const size_t desc_at = *words, recs_at = (desc_at + desc.size() + 63) & ~(size_t)63;
    const size_t end = (recs_at + recs.size() + 63) & ~(size_t)63;
    W->staging.resize(end + 64, 0);
    std::copy(desc.begin(), desc.end(), W->staging.begin() + (ptrdiff_t)desc_at);
    std::copy(recs.begin(), recs.end(), W->staging.begin() + (ptrdiff_t)recs_at);
    W->grp_desc = W->row_order + desc_at;
    W->grp_recs = W->row_order + recs_at;
    W->grp_n = n_groups;
    W->grp_slots = H;
    W->grp_host.assign(W->staging.begin() + (ptrdiff_t)desc_at, W->staging.begin() + (ptrdiff_t)end);
    W->grp_host_recs_at = recs_at - desc_at;
    *words = end;
}

namespace {

template <typename T, typename O>
bsr_status launch_group_types(const spmm_args& a)
{
    const bsr_matrix* W = a.W;
    const int m = (int)a.m, n = (int)W->n, k = (int)W->k;
    if ((int64_t)m * k * (int64_t)sizeof(T) >= ((int64_t)1 << 32)) return BSR_ERR_UNSUPPORTED;   // 32-bit byte offsets into X
    const int n_sub = (m + kSub - 1) / kSub;
    const int64_t grid = (int64_t)((n_sub + kXcds - 1) / kXcds) * kXcds * W->grp_n;
    if (grid <= 0 || grid >= ((int64_t)1 << 31)) return BSR_ERR_UNSUPPORTED;
    static const hipError_t attr = hipFuncSetAttribute(reinterpret_cast<const void*>(&bsr_mfma_group<T, O>),
                                                       hipFuncAttributeMaxDynamicSharedMemorySize, kLdsBytes);
    if (attr != hipSuccess) return BSR_ERR_HIP;
    hipLaunchKernelGGL((bsr_mfma_group<T, O>), dim3((unsigned)grid), dim3(768), kLdsBytes, a.stream, (const T*)a.X,
                       (const T*)W->data, W->grp_recs, W->grp_desc, (O*)a.Y, m, k, n, W->grp_n, n_sub);
    return hipGetLastError() == hipSuccess ? BSR_OK : BSR_ERR_HIP;
}

}  // namespace

// The grouped block-rows of W (slots 0 .. W->grp_slots-1); the caller multiplies the other slots.
bsr_status launch_mfma_group(const spmm_args& a, const tune_opts&)
{
    const bsr_matrix* W = a.W;
    if (!mfma_group_supports(W)) return BSR_ERR_UNSUPPORTED;
    if (W->dtype == BSR_F16) return a.y_dtype == BSR_F32 ? launch_group_types<f16_t, float>(a) : launch_group_types<f16_t, f16_t>(a);
    if (W->dtype == BSR_BF16) return a.y_dtype == BSR_F32 ? launch_group_types<bf16_t, float>(a) : launch_group_types<bf16_t, bf16_t>(a);
    return BSR_ERR_UNSUPPORTED;
}

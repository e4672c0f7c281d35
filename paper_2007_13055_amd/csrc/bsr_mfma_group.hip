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
// hold about equal numbers of blocks.  A group has 8 multiplying wavefronts: each row gets one, and
// wavefronts that are left over go to the rows with the most blocks per wavefront, which are cut into
// SHARES (the row's blocks in column order, dealt round); the order of the rows over the wavefronts is
// the one that leaves the busiest SIMD the fewest blocks.  A group's work is a stream of 8 KiB tiles --
// the X tile of a block-column, then the stored blocks of that column -- cut into WINDOWS of at most
// kWin tiles: whole columns (a column with more blocks than fit is cut, each part with the X tile),
// starting with the first column not yet placed and filled up with the best-fitting of the next
// kLookAhead ones, so that nearly every window is full and the groups still pass over the
// block-columns at about the same time.  One 16-word record per window:
//   word 0   stored blocks per wavefront of the group in this window, 4 bits each (wavefront j at bits 4j..4j+3)
//   word 1   tiles in the window (bits 0-3), X tiles among them (bits 4-7)
//   word 2   for the window's i-th stored block, 4 bits each: which of the window's X tiles it multiplies
//   word 4.. the tiles by byte offset: first the X tiles (block-column * 128, into a row of X), then the
//            stored blocks (stored-block number * 8192, into block_data) sorted by wavefront
// Group descriptor (16 words): the block-row of each of the 8 wavefronts (-1: none; the wavefronts of
// a row follow each other), the group's first record, its number of windows.
//
// Workgroup: 12 wavefronts, three per SIMD.  Wavefront j < 8 multiplies the blocks counted for it;
// wavefronts 8-11 only move tiles.  (A wavefront that issues loads waits for the memory pipeline to
// take them, about 130 cycles per 1 KiB load while a window streams in; one that multiplied as well
// would be the last at every barrier.)
//
// Data movement.  Tiles go from global memory straight into LDS (global_load_lds_dwordx4: no staging
// registers).  The ring holds three windows of kWin slots, window w in the slots (w mod 3) * kWin ..;
// each of the four moving wavefronts takes a quarter (16 rows, two 1 KiB loads) of every tile (built with
// GRP_G = 6: six wavefronts multiply, six move tiles, each one half of every third tile).  Loads
// complete in issue order: before window w is multiplied a moving wavefront waits until only its loads
// of window w+1 are outstanding, then the workgroup meets at a barrier -- which also says that
// everybody is done with window w-1 -- and the loads of window w+2 are issued into the slots of window
// w-1.  A 16-byte piece q of row i of a tile lies at piece position q ^ (i mod 8) of its 128-byte LDS
// row, which makes the operand reads of 16 consecutive rows at one k offset conflict-free without
// padding.  The window records travel the same way, 64 at a time, into an 8 KiB record area in front
// of the ring, and are read from there one word per lane (scalar loads from global memory cost a cache
// miss per window on the critical path).
//
// Arithmetic.  A wavefront multiplies whole 64x64 blocks of its row: v_mfma_f32_16x16x32 on 4x4 tiles, 16
// independent accumulators (64 registers per lane), the accumulator a block adds to known at compile
// time.  It holds the operands of one k half of a block at a time (4 tiles of the block, 4 of X) in each
// of two register sets; while one half is multiplied (16 MFMAs) the eight LDS reads of the half after
// the next are interleaved with the first eight of them.  Every stored block costs 16 KiB of LDS reads
// (quadrants shared by four wavefronts cost 32 KiB and twice the instructions per flop).
//
// Results.  Every multiplying wavefront writes its 64x64 fp32 result into LDS; the shares of a row are
// added there in wavefront order, rounded once to the type of Y, and whole rows are stored.
//
// Measured on the 8192^3 power-law workload (16 grouped rows = 573 of 819 blocks, 75 and 73 windows):
// this kernel fetches about 220 MB from beyond L2 where the tile kernel fetches 601 MB for the same
// rows, and takes about 65 us for them against 105 us; with the tile kernel for the other rows the
// product takes 111-116 us instead of 135 us.  What bounds it: a workgroup streams 3.3 MB of tiles
// per 64 rows of X; with the multiplying switched off the kernel takes 50 us (a CU takes in about
// 30 bytes per clock), with the loads switched off 51-55 us (per window the busiest SIMD multiplies
// two blocks while the average is one), and the two overlap only partly behind one barrier per window.
#include <algorithm>
#include <numeric>

#include "bsr_mfma_common.h"

using namespace bsr_dev;

namespace {

constexpr int kXcds = 8;
#ifndef GRP_G
#define GRP_G 8
#endif
constexpr int kG = GRP_G;                             // block-rows per group: wavefronts that multiply
constexpr int kLoaders = 12 - kG;                     // wavefronts that only move tiles
constexpr int kSplit = kLoaders == 6 ? 2 : 4;         // a tile moves as kSplit units of 8 / kSplit loads (1 KiB, 8 rows each)
constexpr int kLpu = 8 / kSplit;                      // loads per unit
constexpr int kTileStep = kLoaders / kSplit;          // a moving wavefront takes every kTileStep-th tile of a window
static_assert(kG >= 1 && kG <= 8 && kLoaders >= 4 && kLoaders % kSplit == 0 && (kLpu == 2 || kLpu == 4), "a record counts 8 rows; four wavefronts move the records");
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
#ifndef GRP_LOOK
#define GRP_LOOK 8
#endif
constexpr int kLookAhead = GRP_LOOK;                  // how far behind a window's first block-column the plan looks for more to fill it
static_assert(kRingWin * kWin <= kSlots && (kRingWin == 2 || kRingWin == 3) && kWin <= 9, "the windows fit the ring; a record lists at most 9 tiles");

template <int N>
__device__ __forceinline__ void wait_vm()
{
    asm volatile("s_waitcnt vmcnt(%0)" ::"n"(N) : "memory");
}

// Returns when at most the `loads` youngest loads of this wavefront are still in flight.
__device__ __forceinline__ void wait_all_but(int loads)
{
    switch (loads) {
        case 0: wait_vm<0>(); break;
        case 1: wait_vm<1>(); break;
        case 2: wait_vm<2>(); break;
        case 3: wait_vm<3>(); break;
        case 4: wait_vm<4>(); break;
        case 5: wait_vm<5>(); break;
        case 6: wait_vm<6>(); break;
        case 7: wait_vm<7>(); break;
        case 8: wait_vm<8>(); break;
        case 9: wait_vm<9>(); break;
        case 10: wait_vm<10>(); break;
        case 11: wait_vm<11>(); break;
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

// Results leave a wavefront as fp32 through LDS: one 64x64 staging buffer per multiplying wavefront.
constexpr int kStageStride = 64 * 4 + 16;             // bytes of a staged row, padded
constexpr int kStage = 64 * kStageStride;
static_assert(kG * kStage <= kSlots * kTileBytes, "the group's results fit the ring");

template <typename T, typename O>
__global__ __launch_bounds__(768) void bsr_mfma_group(const T* __restrict__ X, const T* __restrict__ data,
                                                      const int32_t* __restrict__ recs,
                                                      const int32_t* __restrict__ gdesc, O* __restrict__ Y,
                                                      int m, int k, int n, int n_groups, int n_sub)
{
    typedef __attribute__((address_space(3))) void lds_void;
    typedef __attribute__((address_space(1))) const void glob_void;
    extern __shared__ __attribute__((aligned(1024))) unsigned char lds[];
    unsigned char* const ring = lds + kRecBytes;      // records first, then the ring of tiles

    // 12 wavefronts, three per SIMD.  Wavefront j < kG multiplies the blocks the records count for it (a
    // block-row of the group, or a share of one); the others only move tiles: a wavefront that issues
    // loads waits for the memory pipeline to take them (about 130 cycles per 1 KiB load while a window
    // streams in), and a wavefront that multiplied as well would be the last at every barrier.
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const bool producer = wave >= kG;
    const int pq = wave - kG;                         // which of the moving wavefronts (negative: none)

    // workgroup -> (64-row sub-tile of X, group): XCD x (which receives the workgroups b = x mod 8) takes the
    // sub-tiles x, x+8, ..., and the groups of a sub-tile follow each other on that XCD, so the second
    // group finds the X tiles the first one fetched in the XCD's L2
    const int xcd = (int)(blockIdx.x % kXcds), local = (int)(blockIdx.x / kXcds);
    const int sub = (local / n_groups) * kXcds + xcd, g = local % n_groups;
    if (sub >= n_sub) return;                         // whole workgroup: the grid is padded to whole rounds of XCDs
    const int32_t* __restrict__ gd = gdesc + (size_t)g * kDescWords;   // uniform
    const int n_win = gd[9];
    if (n_win <= 0) return;                           // whole workgroup (a plan has no such group)
    const int32_t* __restrict__ rec = recs + (size_t)gd[8] * kRec;

    // ---- moving tiles: 1 KiB loads, each 8 rows of a tile ----
    // lane l moves the 16 bytes at piece position l mod 8 of the load's row l div 8, which hold the row's
    // piece (position ^ row mod 8)
    const unsigned char* Xb = reinterpret_cast<const unsigned char*>(X);
    const unsigned char* Wb = reinterpret_cast<const unsigned char*>(data);
    const int lrow = lane >> 3;
    const unsigned piece = (unsigned)((lane & 7) ^ lrow) * 16u;
    const unsigned row_bytes = (unsigned)k * (unsigned)sizeof(T);
    // Moving wavefront q takes the same part (q mod kSplit: 64 / kSplit rows) of the tiles q div kSplit,
    // q div kSplit + kTileStep, ... of every window: kLpu loads each.  A record names a tile by its byte
    // offset: block-column * 128 into a row of X, stored block * 8192 into the blocks; the window's first nx
    // tiles are X tiles.  Byte offsets into X fit 32 bits (m*k*2 < 2^32); rows past m repeat row m-1, their
    // results are never stored.
    const int part = pq & (kSplit - 1), t0 = pq / kSplit;
    const unsigned char* xa[kLpu];                    // the lane's address in block-column 0 of X, per load
#pragma unroll
    for (int i = 0; i < kLpu; ++i)
        xa[i] = Xb + ((unsigned)min(sub * kSub + part * (kSub / kSplit) + 8 * i + lrow, m - 1) * row_bytes + piece);
    const unsigned char* const wa = Wb + ((unsigned)(part * (kSub / kSplit) + lrow) * 128u + piece);
    auto loads_of = [&](int nt) { return nt > t0 ? kLpu * ((nt - t0 + kTileStep - 1) / kTileStep) : 0; };
    // Window w lives in the kWin slots starting at slot (w mod 3) * kWin, tile i in the i-th of them.
    // A window's record is read from LDS one word per lane (rv: lanes 16q .. 16q+15 hold record w+q) and
    // its words are taken out with lane reads; `at` = lane of the record's word 0.
    auto issue = [&](int rv, int at, int w3) __attribute__((always_inline)) {   // the tiles of one window
        const int info = __builtin_amdgcn_readlane(rv, at + 1);
        const int nt = info & 15, nx = (info >> 4) & 15;
        unsigned char* dst = ring + w3 * (kWin * kTileBytes) + t0 * kTileBytes + part * (kTileBytes / kSplit);
#pragma unroll
        for (int j = 0; j < (kWin + kTileStep - 1) / kTileStep; ++j, dst += kTileStep * kTileBytes) {
            const int t = t0 + j * kTileStep;
            if (t >= nt) break;
            const unsigned code = (unsigned)__builtin_amdgcn_readlane(rv, at + kRecTilesAt + t);
            if (t < nx) {                             // X tile of a block-column: the rows are k elements apart
#pragma unroll
                for (int i = 0; i < kLpu; ++i)
                    __builtin_amdgcn_global_load_lds((glob_void*)(xa[i] + code), (lds_void*)(dst + i * 1024), 16, 0, 0);
            } else {                                  // a stored block: 8 KiB in one piece
                const unsigned char* src = wa + code;
                __builtin_amdgcn_global_load_lds((glob_void*)src, (lds_void*)dst, 16, 0, 0);
                __builtin_amdgcn_global_load_lds((glob_void*)src, (lds_void*)dst, 16, 1024, 0);
                if constexpr (kLpu == 4) {
                    __builtin_amdgcn_global_load_lds((glob_void*)src, (lds_void*)dst, 16, 2048, 0);
                    __builtin_amdgcn_global_load_lds((glob_void*)src, (lds_void*)dst, 16, 3072, 0);
                }
            }
        }
    };
    // 64 records (4 KiB) into their half of the record area, 1 KiB per moving wavefront; pieces past the
    // group's last record repeat its last piece (never used)
    const int last_piece = n_win * (kRec / 4) - 1;
    auto load_records = [&](int chunk) __attribute__((always_inline)) {
        if (pq >= 4) return;
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

    // The two kinds of wavefront run loops of their own and meet at one barrier per window.
    if (producer) {
        int w3 = 0;                                   // w mod 3
        for (int w = 0; w < n_win; ++w) {
            const int next_tiles = kRingWin == 3 && w + 1 < n_win ? (__builtin_amdgcn_readlane(rv, 17) & 15) : 0;
            wait_all_but(loads_of(next_tiles));       // this wavefront's share of window w has landed
            barrier();                                // ... everybody's has, and everybody is done with window w-1
            const int rv_next = read_records(w + 1);  // used in the next trip
            // every 64 windows the half of the record area that was used up takes the records 64 .. 127 ahead
            // (loads complete in order, so they have landed, for everybody, many windows before they are read)
            if ((w & 63) == 0 && w > 0 && w + 64 < n_win) load_records((w >> 6) + 1);
            // the window kRingWin - 1 ahead takes the slots of window w-1
            if (w + kRingWin - 1 < n_win) issue(rv, 16 * (kRingWin - 1), w3 == 0 ? kRingWin - 1 : w3 - 1);
            w3 = w3 == kRingWin - 1 ? 0 : w3 + 1;
            rv = rv_next;
        }
    } else {
        int w3 = 0;
        for (int w = 0; w < n_win; ++w) {
            barrier();                                // window w has landed
            const int rv_next = read_records(w + 1);
            const unsigned all_counts = (unsigned)__builtin_amdgcn_readlane(rv, 0);
            const int info = __builtin_amdgcn_readlane(rv, 1);
            const unsigned xis = (unsigned)__builtin_amdgcn_readlane(rv, 2);
            const int nx = (info >> 4) & 15;
            // this wavefront's blocks: how many, and how many belong to the wavefronts before it (the window's blocks are sorted by wavefront)
            const int c = (int)((all_counts >> (4 * wave)) & 15u);
            const unsigned below = all_counts & ((1u << (4 * wave)) - 1u);
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
    }

    // ---- epilogue: every wavefront's 64x64 fp32 result through LDS (the ring is free: no load is outstanding);
    // a block-row is the sum of its wavefronts' results, in wavefront order, then whole rows go to Y ----
    // result of a 16x16 tile: lane l holds X row (l mod 16), 4 consecutive columns 4*(l div 16) ..
    asm volatile("s_waitcnt vmcnt(0) lgkmcnt(0)" ::: "memory");
    barrier();
    if (!producer && gd[wave] >= 0) {                 // uniform
        unsigned char* ob = ring + wave * kStage;
#pragma unroll
        for (int ct = 0; ct < 4; ++ct)
#pragma unroll
            for (int rt = 0; rt < 4; ++rt)
                *reinterpret_cast<f32x4*>(ob + (16 * rt + fr) * kStageStride + (16 * ct + 4 * fq) * 4) = acc[ct][rt];
    }
    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
    barrier();
    const int i0 = sub * kSub;
    constexpr int EPP = 16 / (int)sizeof(O);          // elements of Y per 16-byte piece
    constexpr int PPR = 64 / EPP;                     // pieces per output row of a block-row
    constexpr int RPP = 512 / PPR;                    // rows per pass of the first 512 threads
    if (tid >= 512) return;
    for (int j = 0; j < kG;) {                        // uniform: the wavefronts of a block-row follow each other
        const int r = gd[j];
        int shares = 1;
        while (j + shares < kG && gd[j + shares] == r) ++shares;
        if (r >= 0) {
            unsigned char* yb = reinterpret_cast<unsigned char*>(Y + (size_t)r * 64);
#pragma unroll
            for (int pass = 0; pass < 64 / RPP; ++pass) {
                const int row = pass * RPP + tid / PPR, pc = tid % PPR;
                const unsigned char* src = ring + j * kStage + row * kStageStride + pc * (EPP * 4);
                float v[EPP];
#pragma unroll
                for (int e = 0; e < EPP; e += 4) {
                    const f32x4 t = *reinterpret_cast<const f32x4*>(src + e * 4);
                    v[e] = t[0]; v[e + 1] = t[1]; v[e + 2] = t[2]; v[e + 3] = t[3];
                }
                for (int sh = 1; sh < shares; ++sh) {
#pragma unroll
                    for (int e = 0; e < EPP; e += 4) {
                        const f32x4 t = *reinterpret_cast<const f32x4*>(src + sh * kStage + e * 4);
                        v[e] += t[0]; v[e + 1] += t[1]; v[e + 2] += t[2]; v[e + 3] += t[3];
                    }
                }
                u32x4 out;
                if constexpr (std::is_same<O, float>::value) {
                    out = __builtin_bit_cast(u32x4, f32x4{v[0], v[1], v[2], v[3]});
                } else {
                    typedef O o8 __attribute__((ext_vector_type(8)));
                    const o8 h = {from_f32<O>(v[0]), from_f32<O>(v[1]), from_f32<O>(v[2]), from_f32<O>(v[3]),
                                  from_f32<O>(v[4]), from_f32<O>(v[5]), from_f32<O>(v[6]), from_f32<O>(v[7])};
                    out = __builtin_bit_cast(u32x4, h);
                }
                if (i0 + row < m)
                    __builtin_nontemporal_store(out, reinterpret_cast<u32x4*>(yb + (size_t)(i0 + row) * (size_t)n * sizeof(O) + pc * 16));
            }
        }
        j += shares;
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
    if (W->nnzb >= ((int64_t)1 << 19) || W->C >= (1 << 24)) return;   // a record holds 32-bit byte offsets of tiles
    const int R = W->R;
    const int32_t* order = W->staging.data();         // block-rows by stored-block count, longest first: the plan's slot order
    auto count = [&](int r) { return ptr[r + 1] - ptr[r]; };
    const int min_count = W->env_tune.variant == 5 && W->env_tune.b > 0 ? W->env_tune.b : kHeavyMin;
    int max_groups = W->env_tune.variant == 5 && W->env_tune.nw > 0 ? W->env_tune.nw : kMaxGroups;
    max_groups = std::min(max_groups, kMaxGroups);
    int cand = 0;
    while (cand < R && cand < kG * max_groups && count(order[cand]) >= min_count) ++cand;
    if (cand == 0) return;
    const int n_groups = std::min(max_groups, (cand + kG - 1) / kG);
    // A wavefront multiplies one block-row, or a share of one: wavefronts that no row needs go, one at a time,
    // to the row with the most blocks per wavefront (while that is more than one block), and the kernel adds
    // up the results of a row's wavefronts.
    const int H = std::min(cand, kG * n_groups);
    std::vector<int> shares((size_t)H, 1);
    for (int spare = kG * n_groups - H; spare > 0; --spare) {
        int best = -1;
        for (int s = 0; s < H; ++s)
            if (shares[(size_t)s] < kG && count(order[s]) > shares[(size_t)s] &&
                (best < 0 || (int64_t)count(order[s]) * shares[(size_t)best] > (int64_t)count(order[best]) * shares[(size_t)s]))
                best = s;
        if (best < 0) break;
        ++shares[(size_t)best];
    }
    // deal the rows out longest first, each to the group with the fewest blocks that has wavefronts left for
    // its shares (for fewer shares, if no group has that many left)
    struct member { int row, shares; };
    std::vector<std::vector<member>> members((size_t)n_groups);
    std::vector<int64_t> load((size_t)n_groups, 0);
    std::vector<int> room((size_t)n_groups, kG);
    for (int s = 0; s < H; ++s) {
        int want = shares[(size_t)s];
        want = std::min(want, *std::max_element(room.begin(), room.end()));
        int best = -1;
        for (int q = 0; q < n_groups; ++q)
            if (room[(size_t)q] >= want && (best < 0 || load[(size_t)q] < load[(size_t)best])) best = q;
        members[(size_t)best].push_back({order[s], want});
        room[(size_t)best] -= want;
        load[(size_t)best] += count(order[s]);
        W->grp_blocks += count(order[s]);
    }
    std::vector<int32_t> desc((size_t)n_groups * kDescWords, 0), recs;
    for (int q = 0; q < n_groups; ++q) {
        // Order of the group's rows over its wavefronts (the shares of a row next to each other): wavefront j
        // runs on SIMD j mod 4; of all orders, the first that leaves the busiest SIMD the fewest blocks.
        std::vector<member>& mem = members[(size_t)q];
        std::vector<int> perm(mem.size()), best_perm;
        std::iota(perm.begin(), perm.end(), 0);
        int64_t best_cost = -1;
        do {
            int64_t simd[4] = {0, 0, 0, 0};
            int j = 0;
            for (int i : perm)
                for (int sh = 0; sh < mem[(size_t)i].shares; ++sh, ++j) {
                    const int c = count(mem[(size_t)i].row), n = mem[(size_t)i].shares;
                    simd[j & 3] += c / n + (sh < c % n ? 1 : 0);
                }
            const int64_t cost = *std::max_element(simd, simd + 4);
            if (best_cost < 0 || cost < best_cost) { best_cost = cost; best_perm = perm; }
        } while (std::next_permutation(perm.begin(), perm.end()));
        // rows[j] = block-row of wavefront j; first[i], n[i] = the wavefronts of the i-th row in this order
        std::vector<int32_t> rows(8, -1);
        struct span { int row, first, n; };
        std::vector<span> spans;
        {
            int j = 0;
            for (int i : best_perm) {
                spans.push_back({mem[(size_t)i].row, j, mem[(size_t)i].shares});
                for (int sh = 0; sh < mem[(size_t)i].shares; ++sh) rows[(size_t)j++] = mem[(size_t)i].row;
            }
        }
        int32_t* d = desc.data() + (size_t)q * kDescWords;
        for (int j = 0; j < 8; ++j) d[j] = rows[(size_t)j];
        d[8] = (int32_t)(recs.size() / kRec);
        // the group's stored blocks as (block-column, wavefront, stored-block number), by column (storage
        // order inside a block-row is free, and a row may store a column twice); the blocks of a row go to
        // its wavefronts in turn, in column order
        struct entry { int32_t col, j, p; };
        std::vector<entry> all;
        for (const span& sp : spans) {
            std::vector<entry> mine;
            for (int32_t p = ptr[sp.row]; p < ptr[sp.row + 1]; ++p) mine.push_back({idx[p], 0, p});
            std::stable_sort(mine.begin(), mine.end(), [](const entry& a, const entry& b) { return a.col < b.col; });
            for (size_t o = 0; o < mine.size(); ++o) mine[o].j = sp.first + (int32_t)(o % (size_t)sp.n);
            all.insert(all.end(), mine.begin(), mine.end());
        }
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
            for (int32_t c : xcols) rc[t++] = (int32_t)((uint32_t)c * 128u);
            for (const auto& b : wb) rc[t++] = (int32_t)((uint32_t)b.p * (uint32_t)kTileBytes);
            recs.insert(recs.end(), rc, rc + kRec);
            xcols.clear();
            wb.clear();
        };
        // columns as runs of `all`, a column with more than kWin-1 blocks cut into several (each stages X again)
        struct run { size_t at; int n; };
        std::vector<run> runs;
        for (size_t at = 0; at < all.size();) {
            size_t end = at;
            while (end < all.size() && all[end].col == all[at].col) ++end;
            for (; at < end; at += (size_t)std::min<size_t>(end - at, (size_t)(kWin - 1)))
                runs.push_back({at, (int)std::min<size_t>(end - at, (size_t)(kWin - 1))});
        }
        // a window takes the first run not yet placed, then, from the kLookAhead runs behind it, whatever
        // fills it best (the largest that fits, the earliest among equals): full windows mean fewer barriers
        // and more bytes on their way, and the groups still walk the block-columns at about the same pace
        std::vector<char> placed(runs.size(), 0);
        for (size_t first = 0; first < runs.size(); ++first) {
            if (placed[first]) continue;
            auto take = [&](size_t r) {
                placed[r] = 1;
                xcols.push_back(all[runs[r].at].col);
                for (int i = 0; i < runs[r].n; ++i) wb.push_back({all[runs[r].at + (size_t)i].j, all[runs[r].at + (size_t)i].p, (int32_t)xcols.size() - 1});
            };
            take(first);
            for (;;) {
                const int room = kWin - (int)(xcols.size() + wb.size());
                size_t best = runs.size();
                for (size_t r = first + 1; r < runs.size() && r <= first + (size_t)kLookAhead; ++r)
                    if (!placed[r] && 1 + runs[r].n <= room && (best == runs.size() || runs[r].n > runs[best].n)) best = r;
                if (best == runs.size()) break;
                take(best);
            }
            close();
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

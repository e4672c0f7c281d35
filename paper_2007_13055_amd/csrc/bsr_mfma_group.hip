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
// hold about equal numbers of blocks.  A group's work is a stream of 8 KiB tiles -- the X tile of a
// block-column, then the stored blocks of that column -- cut into WINDOWS of at most kWin tiles:
// whole columns, except that a column with more blocks than fit is continued in the next window
// with its X tile staged again.  One 16-word record per window:
//   word 0   stored blocks per row of the group in this window, 4 bits each (row j at bits 4j..4j+3)
//   word 1   tiles in the window (bits 0-3), X tiles among them (bits 4-7)
//   word 2   for the window's i-th stored block, 4 bits each: which of the window's X tiles it multiplies
//   word 4.. the tiles: first the X tiles (0x80000000 | block-column), then the stored blocks
//            (stored-block number) sorted by row of the group
//
// Data movement.  Tiles go from global memory straight into LDS (global_load_lds_dwordx4: no staging
// registers).  The ring holds three windows of kWin slots, window w in the slots (w mod 3) * kWin ..;
// every wavefront moves an eighth (8 rows) of every tile, so all wavefronts issue the same number of
// loads per tile.  Loads complete in issue order: before window w is multiplied a wavefront waits
// until only its loads of window w+1 are outstanding, then the workgroup meets at a barrier -- which
// also says that everybody is done with window w-1 -- and the loads of window w+2 are issued into the
// slots of window w-1.  A 16-byte piece q of row i of a tile lies at piece position q ^ (i mod 8) of
// its 128-byte LDS row, which makes the operand reads of 16 consecutive rows at one k offset
// conflict-free without padding.  The window records travel the same way, 64 at a time, into an 8 KiB
// record area in front of the ring, and are read from there one word per lane (scalar loads from
// global memory cost a cache miss per window on the critical path).
//
// Arithmetic.  8 wavefronts, two per SIMD: wavefronts 0-3 take the group's rows 0-3, wavefronts 4-7 its
// rows 4-7 (the plan balances the two halves), each a quadrant (32 rows of X x 32 rows of the block) of
// every block product of its rows: v_mfma_f32_16x16x32 on 2x2 tiles, 4 independent accumulators per
// block-row, 64 accumulator registers per lane.  Inside a window the stored blocks are taken row of the
// group by row of the group, so the accumulator a block adds to is known at compile time; the operands
// of the next block are read from LDS while the current one is multiplied.
//
// Measured on the 8192^3 power-law workload (16 grouped rows = 573 of 819 blocks): the group kernel
// fetches 196 MB from beyond L2 where the tile kernel fetches 522 MB for the same rows, but takes
// 105 us against 107 us: a workgroup streams 3.3 MB of tiles per 64 rows of X and one CU takes in
// 35-40 bytes per clock at best, and the LDS writes of the arriving tiles and the operand reads share
// the LDS.  It is therefore not the default (BSR_SPMM_TUNE variant=5 selects it).
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
constexpr int kWin = 6;                               // tiles per window at most (3 windows fit the ring)
constexpr int kRecLds = 128;                          // window records kept in LDS: two halves of 64, refilled in turn
constexpr int kRec = 16;                              // words per window record
constexpr int kRecTilesAt = 4;
constexpr int kDescWords = 16;                        // group descriptor: 8 rows, first record, windows, 0...
constexpr int kRecBytes = kRecLds * kRec * 4;         // 8 KiB
constexpr int kLdsBytes = kRecBytes + kSlots * kTileBytes;
constexpr int kHeavyMin = 8;                          // a grouped block-row stores at least this many blocks
constexpr int kMaxGroups = 2;
static_assert(3 * kWin + 1 <= kSlots, "three windows and the slot behind them");

template <int N>
__device__ __forceinline__ void wait_vm()
{
    asm volatile("s_waitcnt vmcnt(%0)" ::"n"(N) : "memory");
}

// Returns when at most the loads of `tiles` tiles (one per tile and wavefront, the youngest) are still in flight.
__device__ __forceinline__ void wait_all_but_tiles(int tiles)
{
    switch (tiles) {
        case 0: wait_vm<0>(); break;
        case 1: wait_vm<1>(); break;
        case 2: wait_vm<2>(); break;
        case 3: wait_vm<3>(); break;
        case 4: wait_vm<4>(); break;
        case 5: wait_vm<5>(); break;
        default: wait_vm<6>(); break;
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
__global__ __launch_bounds__(512) void bsr_mfma_group(const T* __restrict__ X, const T* __restrict__ data,
                                                      const int32_t* __restrict__ recs,
                                                      const int32_t* __restrict__ gdesc, O* __restrict__ Y,
                                                      int m, int k, int n, int n_groups, int n_sub)
{
    typedef out_geom<O> geo;
    typedef __attribute__((address_space(3))) void lds_void;
    typedef __attribute__((address_space(1))) const void glob_void;
    extern __shared__ __attribute__((aligned(1024))) unsigned char lds[];
    unsigned char* const ring = lds + kRecBytes;      // records first, then the ring of tiles

    // 8 wavefronts, two per SIMD (one wavefront alone issues an instruction every 4 cycles at best, and the
    // bookkeeping of the tile stream is some 20 instructions per tile): wavefronts 0-3 take the group's
    // rows 0-3, wavefronts 4-7 its rows 4-7, each a quadrant of every block product of its rows; all
    // eight move an eighth (8 rows) of every tile.
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int half = wave >> 2, cw = wave & 3;
    const int wm = cw >> 1, wn = cw & 1;              // the wavefront's quadrant: rows of X, rows of the block

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

    // ---- moving tiles: wavefront q takes rows 8q .. 8q+7 of every tile, one 1 KiB load ----
    // lane l moves the 16 bytes at piece position l mod 8 of row 8q + l div 8, which hold the row's
    // piece (position ^ row mod 8)
    const unsigned char* Xb = reinterpret_cast<const unsigned char*>(X);
    const unsigned char* Wb = reinterpret_cast<const unsigned char*>(data);
    const int lrow = lane >> 3;
    const unsigned piece = (unsigned)((lane & 7) ^ lrow) * 16u;
    const unsigned row_bytes = (unsigned)k * (unsigned)sizeof(T);
    // byte offset of the lane's piece (m*k*2 < 2^32); rows past m repeat row m-1, their results are never stored
    const int prow = 8 * wave + lrow;
    const unsigned x_off = (unsigned)min(sub * kSub + prow, m - 1) * row_bytes + piece;
    const unsigned w_off = (unsigned)prow * 128u + piece;
    // Window w lives in the kWin slots starting at slot (w mod 3) * kWin, tile i in the i-th of them.
    // A window's record is read from LDS one word per lane (rv: lanes 16q .. 16q+15 hold record w+q) and
    // its words are taken out with lane reads; `at` = lane of the record's word 0.
    auto issue = [&](int rv, int at, int w3) __attribute__((always_inline)) {   // the tiles of one window
        const int nt = __builtin_amdgcn_readlane(rv, at + 1) & 15;
        unsigned char* dst = ring + w3 * (kWin * kTileBytes) + wave * 1024;
        for (int i = 0; i < nt; ++i, dst += kTileBytes) {
            const int code = __builtin_amdgcn_readlane(rv, at + kRecTilesAt + i);
            if (code < 0)                             // X tile of a block-column
                __builtin_amdgcn_global_load_lds((glob_void*)(Xb + (size_t)(code & 0x7fffffff) * 128u + x_off), (lds_void*)dst, 16, 0, 0);
            else                                      // a stored block
                __builtin_amdgcn_global_load_lds((glob_void*)(Wb + (size_t)code * (size_t)kTileBytes + w_off), (lds_void*)dst, 16, 0, 0);
        }
    };
    // 64 records (4 KiB) into their half of the record area, 1 KiB per wavefront of the first four; pieces
    // past the group's last record repeat its last piece (never used)
    const int last_piece = n_win * (kRec / 4) - 1;
    auto load_records = [&](int chunk) __attribute__((always_inline)) {
        if (half == 0) {
            const int pc = min(chunk * 256 + cw * 64 + lane, last_piece);
            __builtin_amdgcn_global_load_lds((glob_void*)(reinterpret_cast<const unsigned char*>(rec) + (size_t)pc * 16),
                                             (lds_void*)(lds + (chunk & 1) * (kRecBytes / 2) + cw * 1024), 16, 0, 0);
        }
    };
    auto read_records = [&](int w) -> int {           // lane l: word l mod 16 of record w + l div 16
        const int q = (w + (lane >> 4)) & (kRecLds - 1);
        return *reinterpret_cast<const int*>(lds + q * (kRec * 4) + (lane & 15) * 4);
    };

    // ---- multiplying wavefronts ----
    // operand of a 16x16x32 MFMA: lane l supplies row (l mod 16) of its 16-row tile, k elements
    // 32*ks + 8*(l div 16) .. +7 = piece 4*ks + l div 16 of the row; ks = 1 differs by XOR 64 bytes
    const int fr = lane & 15, fq = lane >> 4;
    const unsigned f_off = (unsigned)fr * 128u + (unsigned)((fq ^ (fr & 7)) * 16);
    const unsigned xf_off = (unsigned)(32 * wm) * 128u + f_off;
    const unsigned wf_off = (unsigned)(32 * wn) * 128u + f_off;

    constexpr int kHalfRows = kG / 2;
    f32x4 acc[kHalfRows][2][2];
#pragma unroll
    for (int j = 0; j < kHalfRows; ++j)
#pragma unroll
        for (int ct = 0; ct < 2; ++ct)
#pragma unroll
            for (int rt = 0; rt < 2; ++rt) acc[j][ct][rt] = f32x4{0.f, 0.f, 0.f, 0.f};

    // the first 128 records, then windows 0 and 1, are on their way before the loop
    load_records(0);
    if (n_win > 64) load_records(1);
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    barrier();
    int rv = read_records(0);
    issue(rv, 0, 0);
    if (n_win > 1) issue(rv, 16, 1);

    int w3 = 0;                                       // w mod 3
    for (int w = 0; w < n_win; ++w) {
        const int next_tiles = w + 1 < n_win ? (__builtin_amdgcn_readlane(rv, 17) & 15) : 0;
        wait_all_but_tiles(next_tiles);               // this wavefront's share of window w has landed
        barrier();                                    // ... everybody's has, and everybody is done with window w-1
        const int rv_next = read_records(w + 1);      // used in the next trip
        // every 64 windows the half of the record area that was used up takes the records 64 .. 127 ahead
        // (loads complete in order, so they have landed, for everybody, many windows before they are read)
        if ((w & 63) == 0 && w > 0 && w + 64 < n_win) load_records((w >> 6) + 1);
        // window w+2 takes the slots of window w-1.  Wavefronts 0-3 issue its loads before they multiply,
        // wavefronts 4-7 afterwards: while one half waits for the memory pipeline to take its loads the
        // other half multiplies.
        if (half == 0 && w + 2 < n_win) issue(rv, 32, w3 == 0 ? 2 : w3 - 1);

        const int all_counts = __builtin_amdgcn_readlane(rv, 0), info = __builtin_amdgcn_readlane(rv, 1);
        int xis = __builtin_amdgcn_readlane(rv, 2);
        const int nx = (info >> 4) & 15;
        // this wavefront's rows: the low or the high 16 bits of the counts; the blocks of the rows before
        // them (the window's blocks are sorted by row) are skipped
        const int lo = all_counts & 0xffff;
        const int before = half == 0 ? 0 : (lo & 15) + ((lo >> 4) & 15) + ((lo >> 8) & 15) + (lo >> 12);
        const int counts = half == 0 ? lo : (int)((unsigned)all_counts >> 16);
        xis = (int)((unsigned)xis >> (4 * before));
        // The operands of the next stored block are read from LDS while the current one is multiplied;
        // behind the last block that reads a slot nobody waits for, and drops it (the slot behind the
        // ring's last window exists for this).
        const unsigned char* wb = ring + w3 * (kWin * kTileBytes);
        const unsigned char* wt = wb + (nx + before) * kTileBytes;   // tile of the block being read ahead
        frag4 xn, wn4;
        xn.load(wb + (xis & 15) * kTileBytes, xf_off);
        wn4.load(wt, wf_off);
#pragma unroll
        for (int j = 0; j < kHalfRows; ++j) {
            int c = (counts >> (4 * j)) & 15;         // uniform
            while (c > 0) {
                const frag4 xc = xn, wc = wn4;
                xis = (int)((unsigned)xis >> 4);
                wt += kTileBytes;
                xn.load(wb + (xis & 15) * kTileBytes, xf_off);
                wn4.load(wt, wf_off);
                __builtin_amdgcn_sched_barrier(0);    // the reads are issued before the multiplications, not after them
#pragma unroll
                for (int ks = 0; ks < 2; ++ks)
#pragma unroll
                    for (int ct = 0; ct < 2; ++ct)
#pragma unroll
                        for (int rt = 0; rt < 2; ++rt)
                            acc[j][ct][rt] = mfma16<T>(wc.v[ct][ks], xc.v[rt][ks], acc[j][ct][rt]);
                __builtin_amdgcn_sched_barrier(0);
                --c;
            }
        }
        if (half == 1 && w + 2 < n_win) issue(rv, 32, w3 == 0 ? 2 : w3 - 1);
        w3 = w3 == 2 ? 0 : w3 + 1;
        rv = rv_next;
    }

    // ---- epilogue: the group's block-rows through LDS (the ring is free: no load is outstanding), whole rows to Y ----
    // result of a 16x16 tile: lane l holds X row (l mod 16), 4 consecutive columns 4*(l div 16) ..
    asm volatile("s_waitcnt vmcnt(0) lgkmcnt(0)" ::: "memory");
    barrier();
#pragma unroll
    for (int jj = 0; jj < kHalfRows; ++jj) {
        const int j = half * kHalfRows + jj;
        if ((half == 0 ? rows[jj] : rows[kHalfRows + jj]) >= 0) {   // uniform; rows fill a group from the front
            unsigned char* ob = ring + j * geo::OUT;
#pragma unroll
            for (int ct = 0; ct < 2; ++ct)
#pragma unroll
                for (int rt = 0; rt < 2; ++rt) {
                    const int orow = 32 * wm + 16 * rt + fr, ocol = 32 * wn + 16 * ct + 4 * fq;
                    store4<O>(reinterpret_cast<O*>(ob + orow * geo::OS) + ocol, acc[jj][ct][rt][0], acc[jj][ct][rt][1],
                              acc[jj][ct][rt][2], acc[jj][ct][rt][3]);
                }
        }
    }
    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
    barrier();
    const int i0 = sub * kSub;
    constexpr int PPR = geo::OB / 16;                 // 16-byte pieces per output row
    constexpr int RPP = 512 / PPR;                    // rows per pass of the 512 threads
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
        // the group's rows 0-3 and 4-7 go to different wavefronts: deal the members (longest first) to the
        // half with fewer blocks; positions without a row hold -1
        std::vector<int32_t> rows(kG, -1);
        {
            int fill[2] = {0, 0};
            int64_t blocks[2] = {0, 0};
            for (int r : members[(size_t)q]) {
                const int h = fill[0] >= kG / 2 ? 1 : fill[1] >= kG / 2 ? 0 : (blocks[1] < blocks[0] ? 1 : 0);
                rows[(size_t)(h * (kG / 2) + fill[h]++)] = r;
                blocks[h] += count(r);
            }
        }
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
    hipLaunchKernelGGL((bsr_mfma_group<T, O>), dim3((unsigned)grid), dim3(512), kLdsBytes, a.stream, (const T*)a.X,
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

// Matrix-core kernel for large products with 64x64 blocks of a 16-bit type: row groups.
//
// The paper's "Utilizing shared memory" design gives a thread block a tile of Y and caches the parts
// of X and of block_data that tile needs; its Discussion names block-rows of very different length
// as what hurts most.  Here a workgroup owns 64 rows of X times a GROUP of up to 8 block-rows and
// walks the union of the group's block-columns in ascending order.  One step = one block-column:
// its 64x64 tile of X is staged in LDS once and multiplied with the stored block of every row of
// the group that has one there, so an X tile is fetched once per group instead of once per stored
// block, and the few very long block-rows, which share most of their columns, form one group whose
// X traffic is that of a single block-row.
//
// Plan (bsr_create): block-rows whose estimated work is at least half a CU's fair share are grouped
// eight at a time, longest first; the rest are spread over as many groups as balance their work
// (each row to the least loaded group that still has room).  Per m a table assigns workgroups:
// XCD x (which receives the workgroups b = x mod 8) owns a contiguous eighth of the 64-row
// sub-tiles of X, every group gets a number of workgroups per XCD in proportion to its work, each
// taking a contiguous run of the XCD's sub-tiles; heavy workgroups come first.  With about one
// workgroup per CU the groups of one XCD pass over the same rows of X at about the same time, so
// that stripe of X is fetched into the XCD's L2 once.
//
// Data movement.  Everything a step needs -- the X tile and the W blocks, 8 KiB each -- goes from
// global memory straight into a ring of LDS slots (global_load_lds_dwordx4: no staging registers),
// issued up to a ring's worth of tiles ahead of the arithmetic, across steps and sub-tiles.  A
// 16-byte piece q of row i of a tile lies at piece position q ^ (i mod 8) of its 128-byte LDS row,
// which makes the operand reads of 16 consecutive rows at one k offset conflict-free without padding.
// Loads complete in issue order, so "all but the youngest N loads have landed" is what the vmcnt
// counter says; the wait before a step allows exactly the tiles issued beyond that step to remain
// in flight.  Stores of Y (which also count in vmcnt) only make that wait stricter.
//
// Arithmetic.  The 4 wavefronts split every 64x64 block product into quadrants (32 rows of X x 32
// columns of the block-row): v_mfma_f32_16x16x32 on 2x2 tiles, 4 independent accumulators per
// block-row and wavefront, 8 block-rows = 128 accumulator registers per lane.
#include <algorithm>
#include <cmath>
#include <numeric>

#include "bsr_mfma_common.h"

using namespace bsr_dev;

namespace {

constexpr int kXcds = 8;
constexpr int kGroupRows = 8;                         // block-rows per group
constexpr int kSub = 64;                              // rows of X per sub-tile
constexpr int kTileBytes = 8192;                      // a staged tile: 64 rows x 128 bytes
constexpr int kStepBlocks = 6;                        // blocks per step: a block-column that more rows of a group store takes two steps
constexpr int kBatchTiles = 1 + kStepBlocks;          // whole steps are taken in batches of at most this many tiles
constexpr int kMaxSteps = 512, kMaxTiles = 1536;      // a group's lists must fit their LDS area
constexpr int kStepsAt = 0, kTilesAt = kMaxSteps * 4; // byte offsets of the two lists in LDS
constexpr int kListBytes = (kMaxSteps + kMaxTiles) * 4;
constexpr int kEntryWords = 16;                       // workgroup table entry: 8 rows, steps_off, n_steps, tiles_off, n_tiles, sub0, n_sub, 0, 0
// step word: bits 0-7 the rows of the group that store a block in the step's column, bits 8-11 their number,
// bit 16 set on the first step of a batch, bits 20-23 the tiles of that batch
constexpr int kStepFirst = 1 << 16, kStepBatchShift = 20;
constexpr int kLdsBytes = 160 * 1024;
constexpr int kRowShift = 28;                         // tile code of a W block: stored-block number | (row of the group << 28); X tile: 2^31 | block-column

template <typename O>
struct group_geom {
    static constexpr int OB = 64 * (int)sizeof(O);    // bytes of one output row of a block-row
    static constexpr int OS = OB + 16;                // padded LDS stride
    static constexpr int OUT = (64 * OS + 1023) & ~1023;   // one output staging buffer
    static constexpr int NBUF = sizeof(O) == 2 ? 4 : 2;    // staging buffers: block-rows stored per barrier
    static constexpr int RING_AT = kListBytes + NBUF * OUT;
    static constexpr int NS = (kLdsBytes - RING_AT) / kTileBytes;   // ring slots
    static constexpr int LDS = RING_AT + NS * kTileBytes;
    // while a batch is multiplied the next one must already be on its way (its tiles are waited for before
    // any slot is handed back), so two batches must fit the ring; and a wavefront's share of the ring in
    // flight, 8 loads a tile, must fit the 6-bit vmcnt
    static_assert(NS >= 2 * kBatchTiles && NS <= 16, "ring size");
};

template <int N>
__device__ __forceinline__ void wait_vm()
{
    asm volatile("s_waitcnt vmcnt(%0)" ::"n"(N) : "memory");
}

// Returns when at most `tiles` of the tiles this wavefront has issued (8 loads each, oldest first) are
// still in flight.
__device__ __forceinline__ void wait_own_tiles_in_flight(int tiles)
{
    switch (tiles) {
        case 0: wait_vm<0>(); break;
        case 1: wait_vm<8>(); break;
        case 2: wait_vm<16>(); break;
        case 3: wait_vm<24>(); break;
        default: wait_vm<32>(); break;                // a wavefront owns at most 4 of the ring's tiles
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

template <typename T, typename O>
__global__ __launch_bounds__(256, 1) void bsr_mfma_group(const T* __restrict__ X, const T* __restrict__ data,
                                                         const int32_t* __restrict__ steps,
                                                         const int32_t* __restrict__ tiles,
                                                         const int32_t* __restrict__ wg_table, O* __restrict__ Y,
                                                         int m, int k, int n)
{
    typedef group_geom<O> geo;
    constexpr int NS = geo::NS;
    typedef __attribute__((address_space(3))) void lds_void;
    typedef __attribute__((address_space(1))) const void glob_void;
    extern __shared__ __attribute__((aligned(1024))) unsigned char lds[];

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm = wave >> 1, wn = wave & 1;          // the wavefront's quadrant: rows of X, columns of the block-row

    const int32_t* __restrict__ e = wg_table + (size_t)blockIdx.x * kEntryWords;   // uniform
    const int n_sub = e[13];
    if (n_sub <= 0) return;                           // whole workgroup: the grid is padded to whole rounds of XCDs
    int rows[kGroupRows];
#pragma unroll
    for (int j = 0; j < kGroupRows; ++j) rows[j] = e[j];
    const int steps_off = e[8], n_steps = e[9], tiles_off = e[10], n_tiles = e[11], sub0 = e[12];

    // the group's lists -> LDS (read once per sub-tile)
    int32_t* lsteps = reinterpret_cast<int32_t*>(lds + kStepsAt);
    int32_t* ltiles = reinterpret_cast<int32_t*>(lds + kTilesAt);
    for (int i = tid; i < n_steps; i += 256) lsteps[i] = steps[steps_off + i];
    for (int i = tid; i < n_tiles; i += 256) ltiles[i] = tiles[tiles_off + i];
    asm volatile("s_waitcnt vmcnt(0) lgkmcnt(0)" ::: "memory");
    barrier();

    unsigned char* ring = lds + geo::RING_AT;

    // ---- producer: the tile stream (the list, sub-tile after sub-tile) goes into consecutive ring
    //      slots; wavefront w issues the tiles t = w mod 4, eight 1 KiB loads each ----
    // load i of a tile covers its rows 8i .. 8i+7: lane l moves the 16 bytes at piece position l mod 8
    // of row 8i + l div 8, which hold the row's piece (position ^ row mod 8)
    const unsigned char* Xb = reinterpret_cast<const unsigned char*>(X);
    const unsigned char* Wb = reinterpret_cast<const unsigned char*>(data);
    const int lrow = lane >> 3;
    const unsigned piece = (unsigned)((lane & 7) ^ lrow) * 16u;
    const unsigned w_off = (unsigned)lrow * 128u + piece;
    const unsigned row_bytes = (unsigned)k * (unsigned)sizeof(T);
    unsigned x_off[8];                                // byte offsets of the lane's 8 rows of the producer's sub-tile (m*k*2 < 2^32)
    const int total = n_sub * n_tiles;
    int p_idx = wave, p_slot = wave % NS, p_t = wave, p_sub = sub0, own_issued = 0;
    auto set_sub = [&](int sub) {
        const int i0 = sub * kSub;
#pragma unroll
        for (int i = 0; i < 8; ++i)                   // rows past m repeat row m-1; their results are never stored
            x_off[i] = (unsigned)min(i0 + 8 * i + lrow, m - 1) * row_bytes + piece;
    };
    auto normalise = [&]() {                          // p_t back into the list, p_sub and the row offsets with it
        bool moved = false;
        while (n_tiles > 0 && p_t >= n_tiles) { p_t -= n_tiles; ++p_sub; moved = true; }
        if (moved) set_sub(p_sub);
    };
    set_sub(p_sub);
    normalise();
    int next_code = total > 0 ? ltiles[min(p_t, n_tiles - 1)] : 0;     // code of the wavefront's next tile, read ahead
    auto produce = [&](int limit) {                   // issue the wavefront's tiles below index `limit`
        while (p_idx < limit) {
            const int code = __builtin_amdgcn_readfirstlane(next_code);
            unsigned char* dst = ring + p_slot * kTileBytes;
            if (code < 0) {                           // X tile of a block-column
                const unsigned char* base = Xb + (size_t)(code & 0x7fffffff) * 128u;
#pragma unroll
                for (int i = 0; i < 8; ++i)
                    __builtin_amdgcn_global_load_lds((glob_void*)(base + x_off[i]), (lds_void*)(dst + i * 1024), 16, 0, 0);
            } else {                                  // a stored block
                const unsigned char* base = Wb + (size_t)(code & ((1 << kRowShift) - 1)) * (size_t)kTileBytes + w_off;
#pragma unroll
                for (int i = 0; i < 8; ++i)
                    __builtin_amdgcn_global_load_lds((glob_void*)(base + i * 1024), (lds_void*)(dst + i * 1024), 16, 0, 0);
            }
            ++own_issued;
            p_idx += 4;
            p_slot = (p_slot + 4) % NS;
            p_t += 4;
            normalise();
            next_code = ltiles[min(p_t, n_tiles - 1)];
        }
    };

    // ---- consumer ----
    // operand of a 16x16x32 MFMA: lane l supplies row (l mod 16) of its 16-row tile, k elements
    // 32*ks + 8*(l div 16) .. +7 = piece 4*ks + l div 16 of the row; ks = 1 differs by XOR 64 bytes
    const int fr = lane & 15, fq = lane >> 4;
    const unsigned f_off = (unsigned)fr * 128u + (unsigned)((fq ^ (fr & 7)) * 16);
    const unsigned xf_off = (unsigned)(32 * wm) * 128u + f_off;
    const unsigned wf_off = (unsigned)(32 * wn) * 128u + f_off;

    f32x4 acc[kGroupRows][2][2];
#pragma unroll
    for (int j = 0; j < kGroupRows; ++j)
#pragma unroll
        for (int ct = 0; ct < 2; ++ct)
#pragma unroll
            for (int rt = 0; rt < 2; ++rt) acc[j][ct][rt] = f32x4{0.f, 0.f, 0.f, 0.f};

    int c_tile = 0, c_slot = 0;                       // first tile of the batch to come, and its slot
    produce(min(NS, total));

    // Operands of the step being multiplied: xc (its X tile) and wc (the block in turn).  While a step
    // runs, the next step's X tile and first block are read ahead into xn and w1n, and inside a step
    // with several blocks the following block into wnx; the values move into xc / wc afterwards.
    // There is ONE multiply site per block-row (the loop over j below, unrolled), so every accumulator
    // lives in fixed registers: with several sites the compiler copied all of them at every join.
    frag4 xc, wc, xn, w1n, wnx;
    auto step_body = [&](int word) {
        if (word & kStepFirst) {                      // a batch begins: its tiles must have landed, for every wavefront
            const int need = c_tile + ((word >> kStepBatchShift) & 15);
            wait_own_tiles_in_flight(own_issued - ((need - wave + 3) >> 2));
            barrier();                                // ... and all wavefronts are done with the previous batch's slots
            produce(min(c_tile + NS, total));
            xc.load(ring + c_slot * kTileBytes, xf_off);
            wc.load(ring + (c_slot + 1 == NS ? 0 : c_slot + 1) * kTileBytes, wf_off);
        }
        const unsigned mask = (unsigned)word & 0xffu;
        const int nb = (word >> 8) & 15;
        int ws = c_slot + 1 == NS ? 0 : c_slot + 1;   // slot of the step's first block
        int xs = c_slot + 1 + nb;                     // slot of the next step's X tile
        xs = xs >= NS ? xs - NS : xs;
        // read ahead (inside a batch these tiles have landed; across batches the values are replaced
        // by the reads at the next batch's start, and what is read here is never used)
        xn.load(ring + xs * kTileBytes, xf_off);
        w1n.load(ring + (xs + 1 == NS ? 0 : xs + 1) * kTileBytes, wf_off);
        int left = nb;
#pragma unroll
        for (int j = 0; j < kGroupRows; ++j)
            if ((mask >> j) & 1u) {                   // uniform
                --left;
                if (left > 0) {                       // (the empty asm keeps this a branch, not 16 lane selects)
                    asm volatile("" ::: "memory");
                    ws = ws + 1 == NS ? 0 : ws + 1;
                    wnx.load(ring + ws * kTileBytes, wf_off);
                }
#pragma unroll
                for (int ks = 0; ks < 2; ++ks)
#pragma unroll
                    for (int ct = 0; ct < 2; ++ct)
#pragma unroll
                        for (int rt = 0; rt < 2; ++rt)
                            acc[j][ct][rt] = mfma16<T>(wc.v[ct][ks], xc.v[rt][ks], acc[j][ct][rt]);
                if (left > 0) {
                    asm volatile("" ::: "memory");
                    wc = wnx;
                }
            }
        xc = xn;
        wc = w1n;
        c_tile += 1 + nb;
        c_slot = xs;
    };

    for (int sub = sub0; sub < sub0 + n_sub; ++sub) {
        int words = 0;                                // 64 step words at a time, one per lane
        for (int s = 0; s < n_steps; ++s) {
            if ((s & 63) == 0) words = lsteps[min(s + lane, n_steps - 1)];
            step_body(__builtin_amdgcn_readlane(words, s & 63));
        }

        // ---- epilogue of the sub-tile: the block-rows of the group through LDS, NBUF at a time, whole rows to Y ----
        // result of a 16x16 tile: lane l holds X row (l mod 16), 4 consecutive columns 4*(l div 16) ..
        const int i0 = sub * kSub;
        constexpr int PPR = geo::OB / 16;             // 16-byte pieces per output row
        constexpr int RPP = 256 / PPR;                // rows per pass of the 256 threads
#pragma unroll
        for (int j0 = 0; j0 < kGroupRows; j0 += geo::NBUF) {
            if (rows[j0] >= 0) {                      // uniform; rows fill a group from the front
                asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
                barrier();                            // earlier reads of the staging buffers are over
#pragma unroll
                for (int jb = 0; jb < geo::NBUF; ++jb) {
                    const int j = j0 + jb;
                    if (rows[j] >= 0) {
                        unsigned char* ob = lds + kListBytes + jb * geo::OUT;
#pragma unroll
                        for (int ct = 0; ct < 2; ++ct)
#pragma unroll
                            for (int rt = 0; rt < 2; ++rt) {
                                const int orow = 32 * wm + 16 * rt + fr, ocol = 32 * wn + 16 * ct + 4 * fq;
                                store4<O>(reinterpret_cast<O*>(ob + orow * geo::OS) + ocol, acc[j][ct][rt][0], acc[j][ct][rt][1],
                                          acc[j][ct][rt][2], acc[j][ct][rt][3]);
                                acc[j][ct][rt] = f32x4{0.f, 0.f, 0.f, 0.f};
                            }
                    }
                }
                asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
                barrier();
#pragma unroll
                for (int jb = 0; jb < geo::NBUF; ++jb) {
                    const int j = j0 + jb;
                    if (rows[j] >= 0) {
                        const unsigned char* ob = lds + kListBytes + jb * geo::OUT;
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
        }
    }
}

// Estimated work of one step of a group with `blocks` stored blocks in it (an X tile, then per
// block a W tile and a quadrant product), and of storing one block-row of a sub-tile.
inline double step_cost(int blocks) { return 1.0 + 2.0 * blocks; }
constexpr double kRowStoreCost = 2.0;

}  // namespace

size_t group_plan_words(int64_t R, int32_t bs_r, int32_t bs_c, int64_t nnzb)
{
    if (bs_r != 64 || bs_c != 64) return 0;
    (void)R;
    return (size_t)3 * (size_t)nnzb + 256;            // steps (<= nnzb) + tiles (<= 2 nnzb) + alignment
}

size_t group_table_words(int64_t R, int32_t bs_r, int32_t bs_c)
{
    if (bs_r != 64 || bs_c != 64) return 0;
    // per XCD: every group at least once, plus at most one further workgroup per CU's share of the work
    return (size_t)kXcds * ((size_t)R + 96) * kEntryWords;
}

bool mfma_group_supports(const bsr_matrix* W) { return !W->groups.empty(); }

void build_group_plan(bsr_matrix* W, const int32_t* ptr, const int32_t* idx, size_t* words)
{
    W->groups.clear();
    if (W->bs_r != 64 || W->bs_c != 64 || (W->dtype != BSR_F16 && W->dtype != BSR_BF16) || W->R <= 0 || W->nnzb <= 0 ||
        W->nnzb >= ((int64_t)1 << kRowShift)) return;
    const int R = W->R;
    // block-rows by stored-block count, longest first: the plan's slot order
    const int32_t* order = W->staging.data();
    auto count = [&](int r) { return ptr[r + 1] - ptr[r]; };
    auto row_cost = [&](int r) { return 3.0 * count(r) + kRowStoreCost; };
    double total = 0.0;
    for (int r = 0; r < R; ++r) total += row_cost(r);
    const double share = total / 32.0;                // a CU's fair share of an XCD's work (32 CUs)
    std::vector<std::vector<int>> members;
    int s = 0;
    while (s < R && row_cost(order[s]) >= 0.5 * share && count(order[s]) > 1) {   // heavy rows, eight at a time
        if (members.empty() || (int)members.back().size() == kGroupRows) members.emplace_back();
        members.back().push_back(order[s++]);
    }
    const size_t n_heavy = members.size();
    if (s < R) {                                      // the rest: balanced over as many groups as their work asks for
        double rest = 0.0;
        for (int q = s; q < R; ++q) rest += row_cost(order[q]);
        const int n_rest = R - s;
        const int n_groups = std::max((n_rest + kGroupRows - 1) / kGroupRows, (int)std::lround(rest / std::max(share, 1.0)));
        std::vector<double> load((size_t)n_groups, 0.0);
        members.resize(n_heavy + (size_t)n_groups);
        for (int q = s; q < R; ++q) {
            int best = -1;
            for (int g = 0; g < n_groups; ++g)
                if ((int)members[n_heavy + (size_t)g].size() < kGroupRows && (best < 0 || load[(size_t)g] < load[(size_t)best])) best = g;
            members[n_heavy + (size_t)best].push_back(order[q]);
            load[(size_t)best] += row_cost(order[q]);
        }
    }
    std::vector<int32_t> steps, tiles;
    for (const auto& rows : members) {
        if (rows.empty()) continue;
        bsr_matrix::row_group g{};
        for (int j = 0; j < kGroupRows; ++j) g.row[j] = j < (int)rows.size() ? rows[(size_t)j] : -1;
        g.steps_off = (int32_t)steps.size();
        g.tiles_off = (int32_t)tiles.size();
        g.cost = kRowStoreCost * (double)rows.size();
        // merge the rows' block lists by block-column (a row's blocks sorted by column first: storage
        // order inside a row is free); a column a row stores twice takes two steps
        std::vector<std::vector<std::pair<int32_t, int32_t>>> lists(rows.size());
        std::vector<size_t> head(rows.size(), 0);
        for (size_t j = 0; j < rows.size(); ++j) {
            for (int32_t p = ptr[rows[j]]; p < ptr[rows[j] + 1]; ++p) lists[j].push_back({idx[p], p});
            std::stable_sort(lists[j].begin(), lists[j].end(), [](const auto& a, const auto& b) { return a.first < b.first; });
        }
        int in_batch = 0;                             // tiles of the batch being filled
        size_t batch_first = 0;                       // its first step word
        auto close_batch = [&]() {
            if (in_batch > 0) steps[batch_first] |= kStepFirst | (in_batch << kStepBatchShift);
            in_batch = 0;
        };
        for (;;) {
            int32_t col = INT32_MAX;
            for (size_t j = 0; j < rows.size(); ++j)
                if (head[j] < lists[j].size()) col = std::min(col, lists[j][head[j]].first);
            if (col == INT32_MAX) break;
            int nb = 0;
            for (size_t j = 0; j < rows.size(); ++j)
                if (head[j] < lists[j].size() && lists[j][head[j]].first == col) ++nb;
            if (nb > kStepBlocks) nb = (nb + 1) / 2;  // the rest of the column's blocks: the next step, same column
            if (in_batch > 0 && in_batch + 1 + nb > kBatchTiles) close_batch();
            if (in_batch == 0) batch_first = steps.size();
            tiles.push_back((int32_t)(0x80000000u | (uint32_t)col));
            int taken = 0;
            uint32_t mask = 0;
            for (size_t j = 0; j < rows.size() && taken < nb; ++j)
                if (head[j] < lists[j].size() && lists[j][head[j]].first == col) {
                    tiles.push_back(lists[j][head[j]].second | (int32_t)(j << kRowShift));
                    mask |= 1u << j;
                    ++head[j];
                    ++taken;
                }
            steps.push_back((int32_t)(mask | ((uint32_t)nb << 8)));
            in_batch += 1 + nb;
            g.cost += step_cost(nb);
        }
        close_batch();
        g.n_steps = (int32_t)steps.size() - g.steps_off;
        g.n_tiles = (int32_t)tiles.size() - g.tiles_off;
        if (g.n_steps > kMaxSteps || g.n_tiles > kMaxTiles) { W->groups.clear(); return; }   // lists beyond their LDS area
        W->groups.push_back(g);
    }
    const size_t steps_at = *words, tiles_at = (steps_at + steps.size() + 63) & ~(size_t)63;
    const size_t end = (tiles_at + tiles.size() + 63) & ~(size_t)63;
    W->staging.resize(end + 64, 0);
    std::copy(steps.begin(), steps.end(), W->staging.begin() + (ptrdiff_t)steps_at);
    std::copy(tiles.begin(), tiles.end(), W->staging.begin() + (ptrdiff_t)tiles_at);
    W->grp_steps = W->row_order + steps_at;
    W->grp_tiles = W->row_order + tiles_at;
    *words = end;
}

// Workgroup table for n_sub sub-tiles of X (see the file comment): kEntryWords words per workgroup,
// workgroup b belongs to XCD b mod 8.  Returns the number of workgroups, 0 if the table does not fit.
int build_group_table(const bsr_matrix* W, int n_sub, int cus_per_xcd, std::vector<int32_t>& host)
{
    const int per_xcd = (n_sub + kXcds - 1) / kXcds;              // sub-tiles per XCD (the last XCDs may have fewer)
    double total = 0.0;
    for (const auto& g : W->groups) total += g.cost * per_xcd;
    const double share = std::max(total / std::max(cus_per_xcd, 1), 1e-9);
    struct item { int g, sub0, n_sub; double cost; };
    std::vector<std::vector<item>> lists(kXcds);
    size_t longest = 0;
    for (int x = 0; x < kXcds; ++x) {
        const int first = std::min(x * per_xcd, n_sub), here = std::min((x + 1) * per_xcd, n_sub) - first;
        if (here <= 0) continue;
        for (size_t gi = 0; gi < W->groups.size(); ++gi) {
            const auto& g = W->groups[gi];
            int parts = (int)std::lround(g.cost * per_xcd / share);
            parts = std::max(1, std::min(parts, here));
            for (int q = 0, at = first; q < parts; ++q) {
                const int len = here / parts + (q < here % parts ? 1 : 0);
                lists[(size_t)x].push_back(item{(int)gi, at, len, g.cost * len});
                at += len;
            }
        }
        std::stable_sort(lists[(size_t)x].begin(), lists[(size_t)x].end(), [](const item& a, const item& b) { return a.cost > b.cost; });
        longest = std::max(longest, lists[(size_t)x].size());
    }
    const size_t grid = longest * kXcds;
    if (grid == 0 || grid > W->grp_capacity) return 0;
    host.assign(grid * kEntryWords, 0);
    for (size_t b = 0; b < grid; ++b) {
        const auto& l = lists[b % kXcds];
        const size_t level = b / kXcds;
        if (level >= l.size()) continue;              // n_sub = 0: the workgroup exits
        const auto& g = W->groups[(size_t)l[level].g];
        int32_t* d = host.data() + b * kEntryWords;
        for (int j = 0; j < kGroupRows; ++j) d[j] = g.row[j];
        d[8] = g.steps_off; d[9] = g.n_steps; d[10] = g.tiles_off; d[11] = g.n_tiles;
        d[12] = l[level].sub0; d[13] = l[level].n_sub;
    }
    return (int)grid;
}

namespace {

int group_items(const bsr_matrix* W, int n_sub, hipStream_t stream, int cus_per_xcd, const int32_t** table_out)
{
    auto build = [&](std::vector<int32_t>& host) -> int { return build_group_table(W, n_sub, cus_per_xcd, host); };
    // one table per (sub-tiles, CUs assumed): the key folds both
    return cached_table(W, W->grp_tables, n_sub * 64 + (cus_per_xcd & 63), stream, W->grp_desc, W->grp_capacity * kEntryWords, build, table_out);
}

template <typename T, typename O>
bsr_status launch_group_types(const spmm_args& a, const tune_opts& tune)
{
    typedef group_geom<O> geo;
    const bsr_matrix* W = a.W;
    const int m = (int)a.m, n = (int)W->n, k = (int)W->k;
    if ((int64_t)m * k * (int64_t)sizeof(T) >= ((int64_t)1 << 32)) return BSR_ERR_UNSUPPORTED;   // 32-bit byte offsets into X
    const int n_sub = (m + kSub - 1) / kSub;
    if (n_sub >= (1 << 24)) return BSR_ERR_UNSUPPORTED;
    const int cus = tune.a > 0 && tune.a < 64 ? tune.a : std::max(W->n_cu / kXcds, 1);
    const int32_t* table = nullptr;
    const int grid = group_items(W, n_sub, a.stream, cus, &table);
    if (grid <= 0) return BSR_ERR_UNSUPPORTED;
    static const hipError_t attr = hipFuncSetAttribute(reinterpret_cast<const void*>(&bsr_mfma_group<T, O>),
                                                       hipFuncAttributeMaxDynamicSharedMemorySize, kLdsBytes);
    if (attr != hipSuccess) return BSR_ERR_HIP;
    hipLaunchKernelGGL((bsr_mfma_group<T, O>), dim3((unsigned)grid), dim3(256), geo::LDS, a.stream, (const T*)a.X,
                       (const T*)W->data, W->grp_steps, W->grp_tiles, table, (O*)a.Y, m, k, n);
    return hipGetLastError() == hipSuccess ? BSR_OK : BSR_ERR_HIP;
}

}  // namespace

bsr_status launch_mfma_group(const spmm_args& a, const tune_opts& t)
{
    const bsr_matrix* W = a.W;
    if (!mfma_group_supports(W)) return BSR_ERR_UNSUPPORTED;
    if (W->dtype == BSR_F16) return a.y_dtype == BSR_F32 ? launch_group_types<f16_t, float>(a, t) : launch_group_types<f16_t, f16_t>(a, t);
    if (W->dtype == BSR_BF16) return a.y_dtype == BSR_F32 ? launch_group_types<bf16_t, float>(a, t) : launch_group_types<bf16_t, bf16_t>(a, t);
    return BSR_ERR_UNSUPPORTED;
}

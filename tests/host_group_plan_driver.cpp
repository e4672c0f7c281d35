// Host-side check of the row-group kernel's plan (test infrastructure; no GPU).  For random and adversarial
// patterns it builds the groups, the step and tile lists and the per-m workgroup tables with the library's
// own host code and verifies what the kernel relies on:
//   - every block-row belongs to exactly one group; every stored block appears exactly once in the tile
//     lists, in a step of its own block-column, under the bit of its own block-row;
//   - a step holds 1..6 blocks, its tile run is "X tile of the column, then the blocks in row order", every
//     W code carries its row of the group; batches are whole steps, 2..7 tiles, two in a row fit the ring;
//   - list sizes stay within the kernel's LDS area; table entries repeat their group's fields, and the
//     (group, sub-tile) pairs of a table cover every pair exactly once, XCD x holding the x-th eighth;
//   - the plan fits the words bsr_workspace_size() promises for it.
// Build: hipcc --offload-arch=gfx950 -O1 -std=c++17 -I include -I paper_2007_13055_amd/csrc \
//        tests/host_group_plan_driver.cpp paper_2007_13055_amd/csrc/bsr_mfma_group.hip -o driver
#include <cstdio>
#include <cstdlib>
#include <algorithm>
#include <numeric>
#include <set>
#include <vector>
#include "bsr_internal.h"

// the two host functions of bsr_host.hip that bsr_mfma_group.hip refers to, not needed here
int cached_table(const bsr_matrix*, bsr_matrix::item_table*, int, hipStream_t, int32_t*, size_t,
                 const std::function<int(std::vector<int32_t>&)>&, const int32_t**) { return 0; }
void order_after_upload(hipStream_t, hipEvent_t, std::atomic<bool>&) {}

#define CHECK(c) do { if (!(c)) { std::printf("FAILED %s (line %d) trial %d\n", #c, __LINE__, trial); return 1; } } while (0)

int main()
{
    std::srand(11);
    int plans = 0, tables = 0;
    for (int trial = 0; trial < 400; ++trial) {
        const int R = 1 + std::rand() % 150, C = 1 + std::rand() % 140;
        std::vector<int32_t> ptr(R + 1, 0), idx;
        const int style = trial % 6;
        for (int r = 0; r < R; ++r) {
            int c;
            if (style == 0) c = std::rand() % (C + 1);
            else if (style == 1) c = (r == 3 % R) ? C : (std::rand() % 3);
            else if (style == 2) c = std::max(0, (int)(C / (1.0 + r)));              // power law
            else if (style == 3) c = 1;
            else if (style == 4) c = (std::rand() % 4 == 0) ? 0 : 1 + std::rand() % 8;
            else c = std::min(3 * C, 2 * (std::rand() % (C + 1)));                   // duplicates
            for (int j = 0; j < c; ++j) idx.push_back(style == 5 || trial % 7 == 0 ? std::rand() % C : (j * 7 + r) % C);
            ptr[r + 1] = ptr[r] + c;
        }
        const int64_t nnzb = ptr[R];
        bsr_matrix W;
        W.n = (int64_t)R * 64; W.k = (int64_t)C * 64; W.nnzb = nnzb; W.bs_r = 64; W.bs_c = 64; W.R = R; W.C = C;
        W.dtype = trial % 2 ? BSR_F16 : BSR_BF16;
        const size_t order_words = (size_t)((R + 63) & ~63);
        W.staging.assign(order_words, 0);
        std::iota(W.staging.begin(), W.staging.begin() + R, 0);
        std::stable_sort(W.staging.begin(), W.staging.begin() + R,
                         [&](int32_t a, int32_t b) { return ptr[a + 1] - ptr[a] > ptr[b + 1] - ptr[b]; });
        std::vector<int32_t> fake_ws(16);
        W.row_order = fake_ws.data();                    // only used to form device addresses, never read
        size_t words = order_words;
        build_group_plan(&W, ptr.data(), idx.data(), &words);
        if (nnzb == 0) { CHECK(W.groups.empty()); continue; }
        if (W.groups.empty()) {                          // refused: a list beyond its LDS area
            bool big = false;
            for (int r = 0; r < R; ++r) big |= ptr[r + 1] - ptr[r] > 60;
            CHECK(big || R > 512 / 8);
            continue;
        }
        ++plans;
        CHECK(words - order_words <= group_plan_words(R, 64, 64, nnzb));
        const int32_t* steps = W.staging.data() + (W.grp_steps - W.row_order);
        const int32_t* tiles = W.staging.data() + (W.grp_tiles - W.row_order);
        std::vector<int> row_seen((size_t)R, 0), blk_seen((size_t)nnzb, 0);
        for (const auto& g : W.groups) {
            CHECK(g.n_steps >= 0 && g.n_steps <= 512 && g.n_tiles >= 0 && g.n_tiles <= 1536);
            for (int j = 0; j < 8; ++j) {
                if (g.row[j] < 0) continue;
                CHECK(g.row[j] < R);
                ++row_seen[(size_t)g.row[j]];
            }
            int t = g.tiles_off, prev_col = -1, prev_nt = 0, left_in_batch = 0;
            for (int q = 0; q < g.n_steps; ++q) {          // step words; batches are whole steps, two in a row fit the 14-slot ring
                const uint32_t word = (uint32_t)steps[g.steps_off + q], mask = word & 0xffu;
                const int nb = (int)((word >> 8) & 15u);
                if (left_in_batch == 0) {
                    CHECK(word & (1u << 16));
                    const int nt = (int)((word >> 20) & 15u);
                    CHECK(nt >= 2 && nt <= 7 && prev_nt + nt <= 14);
                    prev_nt = nt;
                    left_in_batch = nt;
                } else {
                    CHECK(!(word & (1u << 16)));
                }
                CHECK(nb >= 1 && nb <= 6 && nb == __builtin_popcount(mask) && 1 + nb <= left_in_batch);
                left_in_batch -= 1 + nb;
                CHECK(t + 1 + nb <= g.tiles_off + g.n_tiles);
                CHECK(tiles[t] < 0);                       // a step starts with the X tile of its block-column
                const int col = tiles[t] & 0x7fffffff;
                CHECK(col >= 0 && col < C && col >= prev_col);
                prev_col = col;
                ++t;
                for (int j = 0; j < 8; ++j)
                    if ((mask >> j) & 1u) {                // then its blocks in row order, each code carrying its row
                        CHECK(tiles[t] >= 0 && (tiles[t] >> 28) == j);
                        const int p = tiles[t] & ((1 << 28) - 1), r = g.row[j];
                        CHECK(r >= 0 && p >= ptr[r] && p < ptr[r + 1] && idx[p] == col);
                        ++blk_seen[(size_t)p];
                        ++t;
                    }
            }
            CHECK(left_in_batch == 0);
            CHECK(t == g.tiles_off + g.n_tiles);
        }
        for (int r = 0; r < R; ++r) CHECK(row_seen[(size_t)r] == 1);
        for (int64_t p = 0; p < nnzb; ++p) CHECK(blk_seen[(size_t)p] == 1);
        // workgroup tables
        W.grp_capacity = group_table_words(R, 64, 64) / 16;
        for (int n_sub : {1, 3, 8, 9, 64, 128, 1000}) {
            for (int cus : {1, 32, 63}) {
                std::vector<int32_t> host;
                const int grid = build_group_table(&W, n_sub, cus, host);
                CHECK(grid > 0 && grid % 8 == 0 && (size_t)grid <= W.grp_capacity && host.size() == (size_t)grid * 16);
                const int per_xcd = (n_sub + 7) / 8;
                std::vector<std::vector<int>> covered(W.groups.size(), std::vector<int>((size_t)n_sub, 0));
                for (int b = 0; b < grid; ++b) {
                    const int32_t* d = host.data() + (size_t)b * 16;
                    if (d[13] == 0) continue;
                    size_t gi = W.groups.size();
                    for (size_t q = 0; q < W.groups.size(); ++q)
                        if (W.groups[q].steps_off == d[8] && W.groups[q].tiles_off == d[10] && W.groups[q].row[0] == d[0]) gi = q;
                    CHECK(gi < W.groups.size());
                    const auto& g = W.groups[gi];
                    for (int j = 0; j < 8; ++j) CHECK(d[j] == g.row[j]);
                    CHECK(d[9] == g.n_steps && d[11] == g.n_tiles && d[13] > 0 && d[12] >= 0 && d[12] + d[13] <= n_sub);
                    CHECK(d[12] >= (b % 8) * per_xcd && d[12] + d[13] <= std::min((b % 8 + 1) * per_xcd, n_sub));
                    for (int q = d[12]; q < d[12] + d[13]; ++q) ++covered[gi][(size_t)q];
                }
                for (const auto& c : covered)
                    for (int v : c) CHECK(v == 1);
                ++tables;
            }
        }
    }
    std::printf("row-group plans checked: %d, workgroup tables: %d, all consistent\n", plans, tables);
    return 0;
}

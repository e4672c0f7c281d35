// Host-side check of the row-group kernel's plan (test infrastructure; no GPU).  For random and adversarial
// patterns it builds the groups and their window records with the library's own host code and verifies what
// the kernel relies on:
//   - the grouped block-rows are exactly the leading grp_slots slots of the longest-first order, each in one
//     group, on one wavefront or on several that follow each other (a long row is cut into shares); every one
//     stores at least the minimum number of blocks, and every such row up to 16 is grouped; no
//     group is empty, none has more than 8 wavefronts;
//   - every stored block of a grouped row appears exactly once in the records, counted under a wavefront of
//     its own row, pointing at an X tile of the same window whose block-column is the block's; the shares of
//     a row differ by at most one block;
//   - a window holds 2..6 tiles, X tiles first, then the stored blocks sorted by wavefront; its counts add
//     up; three windows in a row fit the 19-slot ring; tiles are named by byte offset;
//   - the plan fits the words bsr_workspace_size() promises for it.
// Build: hipcc --offload-arch=gfx950 -O1 -std=c++17 -I include -I paper_2007_13055_amd/csrc \
//        tests/host_group_plan_driver.cpp paper_2007_13055_amd/csrc/bsr_mfma_group.hip -o driver
#include <cstdio>
#include <cstdlib>
#include <algorithm>
#include <numeric>
#include <vector>
#include "bsr_internal.h"

#define CHECK(c) do { if (!(c)) { std::printf("FAILED %s (line %d) trial %d\n", #c, __LINE__, trial); return 1; } } while (0)

int main()
{
    std::srand(11);
    int plans = 0;
    long windows = 0;
    for (int trial = 0; trial < 600; ++trial) {
        const int R = 1 + std::rand() % 150, C = 1 + std::rand() % 140;
        std::vector<int32_t> ptr(R + 1, 0), idx;
        const int style = trial % 6;
        for (int r = 0; r < R; ++r) {
            int c;
            if (style == 0) c = std::rand() % (C + 1);
            else if (style == 1) c = (r == 3 % R) ? C : (std::rand() % 3);
            else if (style == 2) c = std::max(0, (int)(C / (1.0 + r)));              // power law
            else if (style == 3) c = 1;
            else if (style == 4) c = (std::rand() % 4 == 0) ? 0 : 1 + std::rand() % 12;
            else c = std::min(3 * C, 2 * (std::rand() % (C + 1)));                   // duplicates
            for (int j = 0; j < c; ++j) idx.push_back(style == 5 || trial % 7 == 0 ? std::rand() % C : (j * 7 + r) % C);
            ptr[r + 1] = ptr[r] + c;
        }
        const int64_t nnzb = ptr[R];
        bsr_matrix W;
        W.n = (int64_t)R * 64; W.k = (int64_t)C * 64; W.nnzb = nnzb; W.bs_r = 64; W.bs_c = 64; W.R = R; W.C = C;
        W.dtype = trial % 2 ? BSR_F16 : BSR_BF16;
        int min_count = 8;
        if (trial % 3 == 1) { W.env_tune.variant = 5; W.env_tune.b = min_count = 1 + trial % 5; W.env_tune.nw = 1 + trial % 2; }
        const int max_rows = (trial % 3 == 1 && W.env_tune.nw == 1) ? 8 : 16;
        const size_t order_words = (size_t)((R + 63) & ~63);
        W.staging.assign(order_words, 0);
        std::iota(W.staging.begin(), W.staging.begin() + R, 0);
        std::stable_sort(W.staging.begin(), W.staging.begin() + R,
                         [&](int32_t a, int32_t b) { return ptr[a + 1] - ptr[a] > ptr[b + 1] - ptr[b]; });
        const std::vector<int32_t> order(W.staging.begin(), W.staging.begin() + R);
        std::vector<int32_t> fake_ws(16);
        W.row_order = fake_ws.data();                    // only used to form device addresses, never read
        size_t words = order_words;
        build_group_plan(&W, ptr.data(), idx.data(), &words);
        int cand = 0;
        while (cand < R && cand < max_rows && ptr[order[cand] + 1] - ptr[order[cand]] >= min_count) ++cand;
        const int expect = W.grp_slots;
        CHECK(expect == cand);
        if (expect == 0) { CHECK(W.grp_n == 0 && words == order_words); continue; }
        ++plans;
        CHECK(W.grp_n >= 1 && W.grp_n <= (max_rows + 7) / 8 && W.grp_n <= expect);
        CHECK(words - order_words <= group_plan_words(R, 64, 64, nnzb));
        const int32_t* desc = W.grp_host.data();
        const int32_t* recs = W.grp_host.data() + W.grp_host_recs_at;
        CHECK(W.staging.size() >= words);
        CHECK(std::equal(W.grp_host.begin(), W.grp_host.end(), W.staging.begin() + (W.grp_desc - W.row_order)));
        CHECK((size_t)(W.grp_recs - W.grp_desc) == W.grp_host_recs_at);
        std::vector<int> row_seen((size_t)R, 0), blk_seen((size_t)nnzb, 0);
        int64_t blocks = 0;
        int next_rec = 0;
        for (int g = 0; g < W.grp_n; ++g) {
            const int32_t* d = desc + (size_t)g * 16;
            bool ended = false;
            std::vector<int> share_blocks(8, 0);
            for (int j = 0; j < 8; ++j) {
                if (d[j] < 0) { ended = true; continue; }
                CHECK(!ended && d[j] < R);                 // the wavefronts fill a group from the front
                if (j == 0 || d[j - 1] != d[j]) {
                    for (int i = 0; i < j; ++i) CHECK(d[i] != d[j]);   // a row's wavefronts follow each other
                    ++row_seen[(size_t)d[j]];
                }
            }
            CHECK(d[0] >= 0);
            CHECK(d[8] == next_rec && d[9] >= 1);
            next_rec += d[9];
            int prev = 0, prev2 = 0;
            for (int w = 0; w < d[9]; ++w, ++windows) {
                const int32_t* rc = recs + (size_t)(d[8] + w) * 16;
                const int nt = rc[1] & 15, nx = (rc[1] >> 4) & 15, nb = nt - nx;
                CHECK((rc[1] >> 8) == 0 && nt >= 2 && nt <= 6 && nx >= 1 && nb >= 1);
                CHECK(prev2 + prev + nt <= 19);
                prev2 = prev; prev = nt;
                int sum = 0, at = 0;
                for (int i = 0; i < nx; ++i) CHECK(rc[4 + i] >= 0 && rc[4 + i] % 128 == 0 && rc[4 + i] / 128 < C);   // byte offset into a row of X
                for (int j = 0; j < 8; ++j) {
                    const int c = (rc[0] >> (4 * j)) & 15;
                    sum += c;
                    for (int q = 0; q < c; ++q, ++at) {    // the window's stored blocks come sorted by row of the group
                        CHECK(at < nb);
                        const uint32_t code = (uint32_t)rc[4 + nx + at];      // byte offset into block_data
                        CHECK(code % 8192u == 0);
                        const int p = (int)(code / 8192u), xi = (rc[2] >> (4 * at)) & 15, r = d[j];
                        ++share_blocks[(size_t)j];
                        CHECK(r >= 0 && p >= ptr[r] && p < ptr[r + 1] && xi < nx);
                        CHECK(rc[4 + xi] / 128 == idx[p]);
                        ++blk_seen[(size_t)p];
                        ++blocks;
                    }
                }
                CHECK(sum == nb);
                for (int i = nb; i < 8; ++i) CHECK(((rc[2] >> (4 * i)) & 15) == 0);
                for (int i = nt; i < 12; ++i) CHECK(rc[4 + i] == 0);
            }
            for (int j = 0; j < 8; ++j)                    // shares of a row: equal up to one block, all the row's blocks
                if (d[j] >= 0 && (j == 0 || d[j - 1] != d[j])) {
                    int lo = 1 << 30, hi = 0, sum = 0;
                    for (int i = j; i < 8 && d[i] == d[j]; ++i) { lo = std::min(lo, share_blocks[(size_t)i]); hi = std::max(hi, share_blocks[(size_t)i]); sum += share_blocks[(size_t)i]; }
                    CHECK(hi - lo <= 1 && sum == ptr[d[j] + 1] - ptr[d[j]]);
                }
        }
        CHECK(blocks == W.grp_blocks);
        for (int s = 0; s < R; ++s) {
            const int r = order[s];
            CHECK(row_seen[(size_t)r] == (s < expect ? 1 : 0));
            for (int p = ptr[r]; p < ptr[r + 1]; ++p) CHECK(blk_seen[(size_t)p] == (s < expect ? 1 : 0));
        }
    }
    std::printf("%d plans, %ld windows: all consistent\n", plans, windows);
    return plans > 100 ? 0 : 1;
}

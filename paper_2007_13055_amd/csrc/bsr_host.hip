// Host side of libbsr_spmm: structural validation, the block-row plan, handle life cycle and
// kernel-family dispatch.  Nothing here allocates device memory.
#include <algorithm>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <string>
#include <new>
#include <numeric>
#include <utility>

#include "bsr_internal.h"

namespace {

constexpr int64_t kInt32Limit = (int64_t)1 << 31;

bsr_status check_shape(int64_t n, int64_t k, int32_t bs_r, int32_t bs_c, int64_t nnzb)
{
    if (n < 0 || k < 0 || nnzb < 0 || bs_r <= 0 || bs_c <= 0) return BSR_ERR_SHAPE;
    if (n % bs_r != 0 || k % bs_c != 0) return BSR_ERR_SHAPE;        // b_r | n, b_c | k
    if (n >= kInt32Limit || k >= kInt32Limit || nnzb >= kInt32Limit) return BSR_ERR_SHAPE;
    if (nnzb * (int64_t)bs_r * bs_c >= kInt32Limit) return BSR_ERR_SHAPE;   // element offsets are int32
    if (nnzb > 0 && (n == 0 || k == 0)) return BSR_ERR_SHAPE;
    return BSR_OK;
}

size_t item_table_bytes(int64_t R)
{
    // the table never holds more than 2*kMaxKsplitItems + 256 descriptors, and a W with R block-rows
    // has at most kMaxKsplitItems items when the kernel is used at all
    const size_t items = (size_t)std::min<int64_t>(std::max<int64_t>(R, 1) * 256, 2 * kMaxKsplitItems + 256);
    return items * kRowDescWords * sizeof(int32_t);   // one table; the workspace holds kItemSlots of them
}

size_t plan_bytes(int64_t R, int64_t nnzb, int32_t bs_r, int32_t bs_c, int64_t k)
{
    // row order (4R bytes) + row descriptors + pair pointers (4R) + pair entries (16 bytes each, at
    // most nnzb/2 + kStripeChunkPairs per block-row), each part padded to 256 bytes, + the k-split
    // kernel's work-item table (up to 2*kMaxKsplitItems + 256 descriptors)
    // small blocks instead: tile-row descriptors (at most one per block-row) and 20 bytes per tile entry
    // (at most one per stored block)
    const size_t per_row = 4 + 8 * (size_t)kRowDescWords + 4 + 16 * (size_t)kStripeChunkPairs + 16;
    // + 32 bytes per stored block for the sampled product: its block-row (4), runs (8), tiles (16 + 4)
    size_t b = per_row * (size_t)R + 52 * (size_t)nnzb + 4096 + kItemSlots * item_table_bytes(R);
    // row-group kernel (64x64 blocks): its group descriptors and window records
    b += sizeof(int32_t) * group_plan_words(R, bs_r, bs_c, nnzb);
    // thin blocks: the phase positions of every block-row
    b += sizeof(int32_t) * thinrow_plan_words(R, k, bs_r, bs_c);
    // blocks of one row: the pairs by block-column and their range positions
    b += sizeof(int32_t) * wide_plan_words(R, k, nnzb, bs_r, bs_c);
    b += 256;                                         // debug mode's result words
    return (b + 255) & ~(size_t)255;
}

bool aligned16(const void* p) { return ((uintptr_t)p & 15u) == 0; }

}  // namespace

tune_opts read_tune_env()
{
    tune_opts t;
    const char* e = std::getenv("BSR_SPMM_TUNE");
    if (!e) return t;
    t.from_env = true;
    std::string s(e);
    size_t pos = 0;
    while (pos < s.size()) {
        size_t end = s.find(',', pos);
        if (end == std::string::npos) end = s.size();
        const std::string kv = s.substr(pos, end - pos);
        const size_t eq = kv.find('=');
        if (eq != std::string::npos) {
            const std::string key = kv.substr(0, eq);
            const int val = std::atoi(kv.c_str() + eq + 1);
            if (key == "variant") t.variant = val;
            else if (key == "nw") t.nw = val;
            else if (key == "mt") t.mt = val;
            else if (key == "a") t.a = val;
            else if (key == "b") t.b = val;
        }
        pos = end + 1;
    }
    return t;
}

// Work-item table of the k-split kernel.
//
// The hardware hands workgroup b to XCD b mod 8 and, inside an XCD, round-robin to its CUs, so with
// every workgroup resident at once workgroup b runs on CU (b mod #CUs) (measured on MI355X).  The
// (block-row, m-tile) items differ in their number of stored blocks; this places them longest
// first on the least loaded CU -- all m-tiles of a block-row on one XCD, so the block-row's W
// blocks are fetched into one L2 only -- and writes the table level by level: entry c + #CUs*level
// is the level-th item of CU c, or an empty descriptor (block-row -1) that makes the workgroup exit.
void order_after_upload(hipStream_t stream, hipEvent_t ev, std::atomic<bool>& landed)
{
    if (!ev || landed.load(std::memory_order_acquire)) return;
    hipStreamCaptureStatus cs = hipStreamCaptureStatusNone;
    if (hipStreamIsCapturing(stream, &cs) != hipSuccess) { (void)hipGetLastError(); return; }
    if (cs != hipStreamCaptureStatusNone) return;
    if (hipEventQuery(ev) == hipSuccess) { landed.store(true, std::memory_order_release); return; }
    (void)hipGetLastError();                          // hipErrorNotReady is not an error of the product
    (void)hipStreamWaitEvent(stream, ev, 0);
    (void)hipGetLastError();
}

int cached_table(const bsr_matrix* W, bsr_matrix::item_table* tables, int key, hipStream_t stream, int32_t* dev_base,
                 size_t capacity_words, const std::function<int(std::vector<int32_t>&)>& build, const int32_t** table_out)
{
    std::lock_guard<std::mutex> lock(W->item_mu);
    bsr_matrix::item_table* slot = nullptr;
    for (int i = 0; i < kItemSlots; ++i)
        if (tables[i].tiles == key) slot = &tables[i];
    if (slot) {
        slot->last_use = ++W->item_clock;
        *table_out = dev_base + (size_t)(slot - tables) * capacity_words;
        order_after_upload(stream, slot->uploaded, slot->landed);
        return slot->grid;
    }
    for (int i = 0; i < kItemSlots && !slot; ++i)      // an unused table, else the least recently used one
        if (tables[i].tiles < 0) slot = &tables[i];
    if (!slot) {
        slot = &tables[0];
        for (int i = 1; i < kItemSlots; ++i)
            if (tables[i].last_use < slot->last_use) slot = &tables[i];
    }
    // a replaced table's upload may still be reading its host copy: wait for it before rewriting the
    // buffer (an event that was only captured into a graph cannot be waited for; its upload ran at
    // capture's warm-up or will read the buffer at replay, which a caller changing m must order itself)
    if (slot->uploaded && !slot->landed.load(std::memory_order_acquire)) (void)hipEventSynchronize(slot->uploaded);
    (void)hipGetLastError();
    slot->tiles = -1;
    const int grid = build(slot->host);
    if (grid <= 0 || slot->host.size() > capacity_words) return 0;
    int32_t* dev = dev_base + (size_t)(slot - tables) * capacity_words;
    if (hipMemcpyAsync(dev, slot->host.data(), slot->host.size() * sizeof(int32_t), hipMemcpyHostToDevice, stream) != hipSuccess)
        return 0;
    slot->landed.store(false, std::memory_order_release);
    if (!slot->uploaded && hipEventCreateWithFlags(&slot->uploaded, hipEventDisableTiming) != hipSuccess)
        slot->uploaded = nullptr;
    if (slot->uploaded) (void)hipEventRecord(slot->uploaded, stream);
    (void)hipGetLastError();                          // a refused record (stream capture) is not an error of the product
    slot->tiles = key;
    slot->grid = grid;
    slot->last_use = ++W->item_clock;
    *table_out = dev;
    return grid;
}

int ksplit_items(const bsr_matrix* W, int tiles, hipStream_t stream, const int32_t** table_out)
{
    const int n_cu = W->n_cu;
    constexpr int kXcds = 8;
    if (n_cu <= 0 || n_cu % kXcds != 0) return 0;
    auto build = [&](std::vector<int32_t>& host) -> int {
        const int R = W->R;
        std::vector<int64_t> cu_load((size_t)n_cu, 0), xcd_load(kXcds, 0);
        std::vector<std::vector<int64_t>> lists((size_t)n_cu);       // (slot << 20 | tile) per CU, in placement order
        for (int s = 0; s < R; ++s) {
            const int64_t w = std::max<int32_t>(W->slot_blocks[(size_t)s], 1);
            const int x = (int)(std::min_element(xcd_load.begin(), xcd_load.end()) - xcd_load.begin());
            for (int t = 0; t < tiles; ++t) {
                int best = x;
                for (int c = x; c < n_cu; c += kXcds)
                    if (cu_load[(size_t)c] < cu_load[(size_t)best]) best = c;
                cu_load[(size_t)best] += w;
                lists[(size_t)best].push_back(((int64_t)s << 20) | t);
            }
            xcd_load[(size_t)x] += w * tiles;
        }
        size_t levels = 0;
        for (const auto& l : lists) levels = std::max(levels, l.size());
        const size_t grid = levels * (size_t)n_cu;
        if (grid == 0 || grid > W->item_capacity) return 0;
        const int32_t* base = W->staging.data() + (W->row_desc - W->row_order);   // host copy of the row descriptors
        host.assign(grid * kRowDescWords, 0);
        for (size_t b = 0; b < grid; ++b) {
            int32_t* d = host.data() + b * kRowDescWords;
            const auto& l = lists[b % (size_t)n_cu];
            const size_t level = b / (size_t)n_cu;
            if (level >= l.size()) { d[0] = -1; continue; }
            const int s = (int)(l[level] >> 20), t = (int)(l[level] & 0xFFFFF);
            std::memcpy(d, base + (size_t)s * kRowDescWords, sizeof(int32_t) * kRowDescWords);
            d[3] = t;
        }
        return (int)grid;
    };
    return cached_table(W, W->item_tables, tiles, stream, W->item_desc, W->item_capacity * kRowDescWords, build, table_out);
}

extern "C" {

bsr_status bsr_validate(int64_t n, int64_t k, int32_t bs_r, int32_t bs_c, int64_t nnzb,
                        const int32_t* indptr, const int32_t* indices)
{
    if (!indptr) return BSR_ERR_NULL;
    if (nnzb > 0 && !indices) return BSR_ERR_NULL;
    bsr_status st = check_shape(n, k, bs_r, bs_c, nnzb);
    if (st != BSR_OK) return st;
    const int64_t R = n / bs_r, C = k / bs_c;
    if (indptr[0] != 0) return BSR_ERR_INDPTR;
    for (int64_t r = 0; r < R; ++r)
        if (indptr[r + 1] < indptr[r]) return BSR_ERR_INDPTR;
    if (indptr[R] != nnzb) return BSR_ERR_INDPTR;
    for (int64_t p = 0; p < nnzb; ++p)
        if (indices[p] < 0 || indices[p] >= C) return BSR_ERR_INDEX;
    return BSR_OK;
}

bsr_status bsr_workspace_size(int64_t n, int64_t k, int32_t bs_r, int32_t bs_c, int64_t nnzb,
                              size_t* bytes)
{
    if (!bytes) return BSR_ERR_NULL;
    *bytes = 0;
    bsr_status st = check_shape(n, k, bs_r, bs_c, nnzb);
    if (st != BSR_OK) return st;
    *bytes = plan_bytes(n / bs_r, nnzb, bs_r, bs_c, k);
    return BSR_OK;
}

bsr_status bsr_create(bsr_matrix** out, int64_t n, int64_t k, int32_t bs_r, int32_t bs_c, int64_t nnzb,
                      bsr_dtype dtype, const void* block_data_dev,
                      const int32_t* block_indices_dev, const int32_t* index_pointer_dev,
                      const int32_t* block_indices_host, const int32_t* index_pointer_host,
                      void* workspace_dev, size_t workspace_bytes, void* hip_stream)
{
    if (!out) return BSR_ERR_NULL;
    *out = nullptr;
    if (!index_pointer_dev || !index_pointer_host || !workspace_dev) return BSR_ERR_NULL;
    if (nnzb > 0 && (!block_data_dev || !block_indices_dev || !block_indices_host)) return BSR_ERR_NULL;
    if (dtype != BSR_F32 && dtype != BSR_F16 && dtype != BSR_BF16) return BSR_ERR_DTYPE;
    bsr_status st = bsr_validate(n, k, bs_r, bs_c, nnzb, index_pointer_host, block_indices_host);
    if (st != BSR_OK) return st;
    if (!aligned16(block_data_dev) || !aligned16(workspace_dev) ||
        ((uintptr_t)block_indices_dev & 3u) || ((uintptr_t)index_pointer_dev & 3u))
        return BSR_ERR_ALIGN;
    const int64_t R = n / bs_r;
    if (workspace_bytes < plan_bytes(R, nnzb, bs_r, bs_c, k)) return BSR_ERR_WORKSPACE;

    bsr_matrix* W = new (std::nothrow) bsr_matrix();
    if (!W) return BSR_ERR_HIP;
    W->n = n; W->k = k; W->nnzb = nnzb; W->bs_r = bs_r; W->bs_c = bs_c;
    W->R = (int32_t)R; W->C = (int32_t)(k / bs_c);
    W->dtype = dtype;
    W->data = block_data_dev; W->indices = block_indices_dev; W->indptr = index_pointer_dev;
    W->env_tune = read_tune_env();                    // the development knob is read once per handle
    if (hipGetDevice(&W->device) != hipSuccess) W->device = 0;
    if (hipDeviceGetAttribute(&W->n_cu, hipDeviceAttributeMultiprocessorCount, W->device) != hipSuccess || W->n_cu <= 0)
        W->n_cu = 256;
    (void)hipGetLastError();

    // ---- plan: block-rows by stored-block count, longest first (stable, so equal rows keep
    //      their natural order and neighbouring rows stay neighbours in the launch, unless said otherwise below) ----
    std::vector<int32_t> cnt((size_t)R);
    for (int64_t r = 0; r < R; ++r) cnt[(size_t)r] = index_pointer_host[r + 1] - index_pointer_host[r];
    const size_t order_words = (((size_t)R * 4 + 255) & ~(size_t)255) / 4;   // row_order, padded to 256 B
    W->staging.assign(order_words + (size_t)R * kRowDescWords + 64, 0);
    std::iota(W->staging.begin(), W->staging.begin() + R, 0);
    // Block-rows whose outputs fill whole 128-byte lines of Y by themselves have nothing to gain from their
    // neighbours in the launch; among equally long ones they go by their first block-column instead, so that
    // rows that read the same tiles of X run at about the same time and find them in their XCD's L2.
    const bool by_column = (size_t)bs_r * (dtype == BSR_F32 ? 4 : 2) >= 128;
    std::stable_sort(W->staging.begin(), W->staging.begin() + R, [&](int32_t a, int32_t b) {
        if (cnt[(size_t)a] != cnt[(size_t)b]) return cnt[(size_t)a] > cnt[(size_t)b];
        if (!by_column || cnt[(size_t)a] == 0) return false;
        return block_indices_host[index_pointer_host[a]] < block_indices_host[index_pointer_host[b]];
    });
    // Row descriptors, in slot order: everything a workgroup needs to start on its block-row in
    // ONE read (block-row, first stored block, block count, the first block-columns), instead of
    // the dependent chain row_order -> index_pointer -> block_indices.
    for (int64_t s = 0; s < R; ++s) {
        const int32_t r = W->staging[(size_t)s];
        int32_t* d = W->staging.data() + order_words + (size_t)s * kRowDescWords;
        d[0] = r;
        d[1] = index_pointer_host[r];
        d[2] = cnt[(size_t)r];
        d[3] = 0;
        for (int j = 0; j < kRowDescCols && j < cnt[(size_t)r]; ++j) d[kRowDescColsAt + j] = block_indices_host[d[1] + j];
    }
    W->max_row_blocks = R ? *std::max_element(cnt.begin(), cnt.end()) : 0;
    W->empty_rows = (int32_t)std::count(cnt.begin(), cnt.end(), 0);
    W->mean_row_blocks = R ? (double)nnzb / (double)R : 0.0;
    // bins (paper, Discussion: a few rows with many blocks beside many sparse rows): empty rows,
    // ordinary rows, and "long" rows -- more than 4x the mean and more than 8 blocks -- which the
    // tiled kernel starts ahead of everything else.  Slots are sorted, so the long rows lead.
    W->long_rows = 0;
    for (int64_t s = 0; s < R && s < R - 1; ++s) {
        const int32_t c = cnt[(size_t)W->staging[(size_t)s]];
        if (c > 8 && (double)c > 4.0 * W->mean_row_blocks) ++W->long_rows; else break;
    }
    W->row_order = static_cast<const int32_t*>(workspace_dev);
    W->row_desc = W->row_order + order_words;
    W->slot_blocks.resize((size_t)R);
    for (int64_t s = 0; s < R; ++s) W->slot_blocks[(size_t)s] = cnt[(size_t)W->staging[(size_t)s]];

    // Pair table (16x16 blocks only; the stripe kernel multiplies two stored blocks of a block-row per
    // MFMA).  Per block-row, in natural order, its stored blocks two by two, and the row's list
    // filled up to a whole number of chunks of kStripeChunkPairs entries (an empty row has none).
    // An entry is {byte offset of the first block in block_data, byte offset of the second, first
    // block-column, second block-column}; a slot with no block ("dead") has offset 2^31 -- past the
    // end of W, read as zeros -- and block-column C, the kernel's all-zero panel.  pair_ptr[r] is
    // the first entry of block-row r.  Left out when W has 2 GiB of blocks or more.
    size_t words = order_words + (size_t)R * kRowDescWords;
    words = (words + 63) & ~(size_t)63;
    if (bs_r == 16 && bs_c == 16 && nnzb * 512 < ((int64_t)1 << 31)) {
        const size_t ptr_at = words;
        const size_t ptr_words = ((size_t)R + 1 + 63) & ~(size_t)63;
        constexpr int KP = kStripeChunkPairs;
        size_t n_entries = 0;
        for (int64_t r = 0; r < R; ++r) n_entries += ((size_t)(cnt[(size_t)r] + 1) / 2 + KP - 1) / KP * KP;
        W->staging.resize(ptr_at + ptr_words + 4 * n_entries + 64, 0);
        int32_t* ptr = W->staging.data() + ptr_at;
        int32_t* pr = ptr + ptr_words;
        const int32_t dead_off = INT32_MIN, dead_col = (int32_t)(k / bs_c);
        size_t q = 0;
        for (int64_t r = 0; r < R; ++r) {
            ptr[r] = (int32_t)q;
            const size_t row_first = q;
            for (int32_t p = index_pointer_host[r]; p < index_pointer_host[r + 1]; p += 2, ++q) {
                const bool two = p + 1 < index_pointer_host[r + 1];
                pr[4 * q] = p * 512;
                pr[4 * q + 1] = two ? (p + 1) * 512 : dead_off;
                pr[4 * q + 2] = block_indices_host[p];
                pr[4 * q + 3] = two ? block_indices_host[p + 1] : dead_col;
            }
            for (; (q - row_first) % KP != 0; ++q) {
                pr[4 * q] = pr[4 * q + 1] = dead_off;
                pr[4 * q + 2] = pr[4 * q + 3] = dead_col;
            }
        }
        ptr[R] = (int32_t)q;
        W->pair_ptr = W->row_order + ptr_at;
        W->pairs = W->pair_ptr + ptr_words;
        words = (ptr_at + ptr_words + 4 * n_entries + 63) & ~(size_t)63;
    }
    // Small blocks: group the stored blocks into 16x16 tiles of W.  Tile-row tr covers the block-rows
    // tr*SR .. tr*SR+SR-1 (SR = 16/bs_r), tile-column tc the block-columns tc*SC .. (SC = 16/bs_c); an
    // entry is one (tile-row, tile-column) with the byte offsets of its up to SR*SC blocks, position
    // (sub-row, sub-column) at index sub-row*SC + sub-column.  A second stored block at a position
    // already taken (duplicates are summed) opens a further entry of the same tile-column.
    const bool small = (bs_r == 8 || bs_r == 16) && (bs_c == 8 || bs_c == 16) && !(bs_r == 16 && bs_c == 16) &&
                       n % 16 == 0 && k % 16 == 0 && nnzb > 0 &&
                       nnzb * bs_r * bs_c * (dtype == BSR_F32 ? 4 : 2) < ((int64_t)1 << 31);
    if (small) {
        const int SR = 16 / bs_r, SC = 16 / bs_c;
        const int64_t TR = n / 16;
        const int32_t blk_bytes = bs_r * bs_c * (dtype == BSR_F32 ? 4 : 2);
        struct entry { int32_t tc; int32_t off[4]; };
        std::vector<std::vector<entry>> rows((size_t)TR);
        size_t n_entries = 0;
        for (int64_t tr = 0; tr < TR; ++tr) {
            auto& list = rows[(size_t)tr];
            for (int qa = 0; qa < SR; ++qa) {
                const int64_t r = tr * SR + qa;
                for (int32_t p = index_pointer_host[r]; p < index_pointer_host[r + 1]; ++p) {
                    const int32_t tc = block_indices_host[p] / SC, pos = qa * SC + block_indices_host[p] % SC;
                    entry* slot = nullptr;
                    for (auto& e : list)
                        if (e.tc == tc && e.off[pos] == INT32_MIN) { slot = &e; break; }
                    if (!slot) {
                        list.push_back(entry{tc, {INT32_MIN, INT32_MIN, INT32_MIN, INT32_MIN}});
                        slot = &list.back();
                    }
                    slot->off[pos] = p * blk_bytes;
                }
            }
            std::stable_sort(list.begin(), list.end(), [](const entry& a, const entry& b) { return a.tc < b.tc; });
            n_entries += list.size();
        }
        std::vector<int32_t> order((size_t)TR);
        std::iota(order.begin(), order.end(), 0);
        std::stable_sort(order.begin(), order.end(),
                         [&](int32_t a, int32_t b) { return rows[(size_t)a].size() > rows[(size_t)b].size(); });
        const size_t desc_at = words, ent_at = desc_at + (size_t)TR * kRowDescWords;
        const size_t col_at = ent_at + 4 * n_entries;
        W->staging.resize(col_at + n_entries + 64, 0);
        size_t e = 0;
        for (int64_t s = 0; s < TR; ++s) {
            const auto& list = rows[(size_t)order[(size_t)s]];
            int32_t* d = W->staging.data() + desc_at + (size_t)s * kRowDescWords;
            d[0] = order[(size_t)s];
            d[1] = (int32_t)e;
            d[2] = (int32_t)list.size();
            for (size_t j = 0; j < list.size(); ++j, ++e) {
                if (j < (size_t)kRowDescCols) d[kRowDescColsAt + j] = list[j].tc;
                for (int q = 0; q < 4; ++q) W->staging[ent_at + 4 * e + q] = list[j].off[q];
                W->staging[col_at + e] = list[j].tc;
            }
            W->sb_max_entries = std::max<int32_t>(W->sb_max_entries, (int32_t)list.size());
        }
        W->sb_desc = W->row_order + desc_at;
        W->sb_entries = W->row_order + ent_at;
        W->sb_cols = W->row_order + col_at;
        W->sb_rows = (int32_t)TR;
        words = (col_at + n_entries + 63) & ~(size_t)63;
    }
    if (nnzb > 0) {                                   // block-row of every stored block
        const size_t at = words;
        W->staging.resize(at + (size_t)nnzb + 64, 0);
        for (int64_t r = 0; r < R; ++r)
            for (int32_t p = index_pointer_host[r]; p < index_pointer_host[r + 1]; ++p) W->staging[at + (size_t)p] = (int32_t)r;
        W->block_row = W->row_order + at;
        words = (at + (size_t)nnzb + 63) & ~(size_t)63;
        // runs of the sampled product: ceil(count / NB) runs per block-row, lengths differing by at most 1
        const int NB = sddmm_run_blocks(bs_r, bs_c, dtype);
        const size_t run_at = words;
        W->staging.resize(run_at + 2 * (size_t)nnzb + 64, 0);
        size_t q = 0;
        for (int64_t r = 0; r < R; ++r) {
            const int32_t first = index_pointer_host[r], cnt = index_pointer_host[r + 1] - first;
            const int32_t parts = (cnt + NB - 1) / NB;
            for (int32_t j = 0, p = first; j < parts; ++j, ++q) {
                const int32_t len = cnt / parts + (j < cnt % parts ? 1 : 0);
                W->staging[run_at + 2 * q] = p;
                W->staging[run_at + 2 * q + 1] = len;
                p += len;
            }
        }
        W->sd_runs = W->row_order + run_at;
        W->sd_n_runs = (int32_t)q;
        words = (run_at + 2 * q + 63) & ~(size_t)63;
        // tiles of the sampled product, for the shapes its matrix-core kernel takes: a stored block goes
        // to the first tile of its (super-row, column group) whose position is free (a duplicate opens
        // another tile); tiles of a super-row by column group, super-rows in order
        int SR = 1, LC = 1;
        sddmm_tile_dims(bs_r, bs_c, dtype, &SR, &LC);
        const bool mfma_shape = (bs_r == 16 || bs_r == 32 || bs_r == 64) && (bs_c == 16 || bs_c == 32 || bs_c == 64);
        if (mfma_shape && SR * LC > 1 && SR * LC <= 16) {
            struct tile { int32_t cg; uint32_t mask; int32_t p[16]; };
            const size_t tile_at = words;
            W->staging.resize(tile_at + 5 * (size_t)nnzb + 128, 0);
            std::vector<int32_t> plist;
            plist.reserve((size_t)nnzb);
            std::vector<tile> list;
            size_t nt = 0;
            for (int64_t sr = 0; sr * SR < R; ++sr) {
                list.clear();
                for (int a = 0; a < SR && sr * SR + a < R; ++a) {
                    const int64_t r = sr * SR + a;
                    for (int32_t p = index_pointer_host[r]; p < index_pointer_host[r + 1]; ++p) {
                        const int32_t cg = block_indices_host[p] / LC, pos = a * LC + block_indices_host[p] % LC;
                        tile* slot = nullptr;
                        for (auto& t : list)
                            if (t.cg == cg && !((t.mask >> pos) & 1u)) { slot = &t; break; }
                        if (!slot) {
                            list.push_back(tile{cg, 0u, {}});
                            slot = &list.back();
                        }
                        slot->mask |= 1u << pos;
                        slot->p[pos] = p;
                    }
                }
                std::stable_sort(list.begin(), list.end(), [](const tile& x, const tile& y) { return x.cg < y.cg; });
                for (const tile& t : list) {
                    int32_t* d = W->staging.data() + tile_at + 4 * nt++;
                    d[0] = (int32_t)sr;
                    d[1] = t.cg;
                    d[2] = (int32_t)plist.size();
                    d[3] = (int32_t)t.mask;
                    for (int pos = 0; pos < SR * LC; ++pos)
                        if ((t.mask >> pos) & 1u) plist.push_back(t.p[pos]);
                }
            }
            const size_t plist_at = (tile_at + 4 * nt + 63) & ~(size_t)63;
            W->staging.resize(plist_at + plist.size() + 64, 0);
            std::copy(plist.begin(), plist.end(), W->staging.begin() + (ptrdiff_t)plist_at);
            W->sd_tiles = W->row_order + tile_at;
            W->sd_plist = W->row_order + plist_at;
            W->sd_n_tiles = (int32_t)nt;
            words = (plist_at + plist.size() + 63) & ~(size_t)63;
        }
    }
    build_group_plan(W, index_pointer_host, block_indices_host, &words);
    build_thinrow_plan(W, index_pointer_host, block_indices_host, &words);
    build_wide_plan(W, index_pointer_host, block_indices_host, &words);
    size_t upload_words = words;
    {   // the per-m tables sit behind everything else, 256-byte aligned
        W->item_desc = const_cast<int32_t*>(W->row_order) + words;
        W->item_capacity = item_table_bytes(R) / (kRowDescWords * sizeof(int32_t));
        words += kItemSlots * W->item_capacity * kRowDescWords;
        W->debug_out = const_cast<int32_t*>(W->row_order) + words;
        words += 64;
    }
    // the plan must fit what bsr_workspace_size promised (its bound is per block-row and per stored block)
    if (sizeof(int32_t) * words > workspace_bytes) { delete W; return BSR_ERR_WORKSPACE; }
    words = upload_words;
    {
        const char* dbg = std::getenv("BSR_SPMM_DEBUG");
        W->debug = dbg && dbg[0] && dbg[0] != '0';
        W->debug_words = words;
        if (W->debug) W->debug_sum = debug_plan_sum(W->staging.data(), words);
    }
    if (R > 0) {
        hipError_t e = hipMemcpyAsync(workspace_dev, W->staging.data(), sizeof(int32_t) * words,
                                      hipMemcpyHostToDevice, (hipStream_t)hip_stream);
        if (e != hipSuccess) { delete W; return BSR_ERR_HIP; }
        if (hipEventCreateWithFlags(&W->plan_uploaded, hipEventDisableTiming) == hipSuccess)
            (void)hipEventRecord(W->plan_uploaded, (hipStream_t)hip_stream);
        else
            W->plan_uploaded = nullptr;
        (void)hipGetLastError();
    }
    // thin blocks: look up the built-in scratch array's address for this device now, so that
    // bsr_spmm_static() has no set-up left to do
    if (mfma_thin_supports(W)) (void)mfma_thin_static_scratch(nullptr);
    *out = W;
    return BSR_OK;
}

void bsr_destroy(bsr_matrix* W)
{
    if (!W) return;
    std::vector<hipEvent_t> events{W->plan_uploaded};
    for (const auto& t : W->item_tables) events.push_back(t.uploaded);
    for (hipEvent_t e : events) {                     // uploads read the handle's host buffers
        if (!e) continue;
        (void)hipEventSynchronize(e);
        (void)hipEventDestroy(e);
        (void)hipGetLastError();
    }
    delete W;
}

bsr_status bsr_query_path(const bsr_matrix* W, int64_t m, bsr_path* path_out)
{
    if (!W || !path_out) return BSR_ERR_NULL;
    // Matrix-core tiles are at least 16 rows of X tall: below that most of a tile is padding and
    // the wavefront-reduction kernels (the paper's own regime, m <= 8) stream W once instead.
    // Thin 16x1 fp32 blocks take the matrix-core path when the caller has lent enough scratch for
    // the transposed copy of X, or when their block-rows are stored in block-column order (one launch,
    // no scratch).
    if ((mfma_supports(W) || mfma_small_supports(W)) && m >= 16) *path_out = BSR_PATH_MFMA;
    else if (mfma_thin_supports(W) && m >= 32 && W->scratch && W->scratch_bytes >= mfma_thin_scratch_bytes(W, m))
        *path_out = BSR_PATH_MFMA;
    else if (mfma_thinrow_supports(W) && m >= 16) *path_out = BSR_PATH_MFMA;   // no scratch: rows of X staged in LDS
    else if (mfma_wide_supports(W) && m >= 16) *path_out = BSR_PATH_MFMA;      // 1x16 blocks, by block-column
    else *path_out = BSR_PATH_WAVE;
    return BSR_OK;
}

bsr_status bsr_scratch_size(const bsr_matrix* W, int64_t m, size_t* bytes)
{
    if (!W || !bytes) return BSR_ERR_NULL;
    *bytes = 0;
    if (m < 0) return BSR_ERR_SHAPE;
    *bytes = mfma_thin_scratch_bytes(W, m);
    return BSR_OK;
}

bsr_status bsr_set_scratch(bsr_matrix* W, void* scratch_dev, size_t bytes)
{
    if (!W) return BSR_ERR_NULL;
    if (scratch_dev && !aligned16(scratch_dev)) return BSR_ERR_ALIGN;
    W->scratch = scratch_dev;
    W->scratch_bytes = scratch_dev ? bytes : 0;
    return BSR_OK;
}

namespace {

bsr_status check_product_args(const bsr_matrix* W, int64_t m, const void* X_dev, const void* Y_dev, bsr_dtype y_dtype)
{
    if (!W) return BSR_ERR_NULL;
    if (m < 0) return BSR_ERR_SHAPE;
    if (y_dtype != W->dtype && y_dtype != BSR_F32) return BSR_ERR_DTYPE;
    if (m == 0 || W->n == 0) return BSR_OK;
    if (!Y_dev || (W->k > 0 && !X_dev)) return BSR_ERR_NULL;
    if (m * std::max<int64_t>(W->k, W->n) >= kInt32Limit) return BSR_ERR_SHAPE;
    if (!aligned16(X_dev) || !aligned16(Y_dev)) return BSR_ERR_ALIGN;
    return BSR_OK;
}

// One product on a fixed family (never AUTO) with fixed settings.
bsr_status run_product(const spmm_args& a, bsr_path path, const tune_opts& t)
{
    order_after_upload(a.stream, a.W->plan_uploaded, a.W->plan_landed);
    if (a.W->debug) {
        const bsr_status dbg = debug_check_device_arrays(a.W, a.stream);
        if (dbg != BSR_OK) return dbg;
    }
    // no stored block (k == 0 included): every kernel family would only store zeros; the wavefront
    // kernels do that for any shape without touching X or W
    if (a.W->nnzb == 0) return launch_wave(a, t);
    if (path == BSR_PATH_MFMA) {
        if (mfma_thin_supports(a.W)) return launch_mfma_thin(a, t);
        if (mfma_small_supports(a.W)) return launch_mfma_small(a, t);
        if (mfma_wide_supports(a.W) && a.y_dtype == BSR_F32) return launch_mfma_wide(a, t);
        if (!mfma_supports(a.W)) return BSR_ERR_UNSUPPORTED;
        return launch_mfma(a, t);
    }
    return launch_wave(a, t);
}

}  // namespace

bsr_status bsr_spmm_ex(const bsr_matrix* W, int64_t m, const void* X_dev, void* Y_dev,
                       bsr_dtype y_dtype, bsr_path path, void* hip_stream)
{
    if (path != BSR_PATH_AUTO && path != BSR_PATH_WAVE && path != BSR_PATH_MFMA) return BSR_ERR_UNSUPPORTED;
    const bsr_status st = check_product_args(W, m, X_dev, Y_dev, y_dtype);
    if (st != BSR_OK || m == 0 || W->n == 0) return st;
    tune_opts t = W->env_tune;
    if (path == BSR_PATH_AUTO) {
        bool tuned = false;
        if (!t.from_env) {                            // what bsr_tune() remembered for this m, if anything
            std::lock_guard<std::mutex> lock(W->tune_mu);
            auto it = W->tuned.find({m, (int)y_dtype});
            if (it != W->tuned.end()) { path = it->second.path; t = it->second.opts; tuned = true; }
        }
        // a remembered thin-block choice needs its scratch still lent
        if (tuned && path == BSR_PATH_MFMA && mfma_thin_supports(W) && !(t.variant == 2 && mfma_thinrow_supports(W)) &&
            (!W->scratch || W->scratch_bytes < mfma_thin_scratch_bytes(W, m))) tuned = false;
        if (!tuned) { bsr_query_path(W, m, &path); if (!t.from_env) t = tune_opts{}; }
    }
    return run_product(spmm_args{W, m, X_dev, Y_dev, y_dtype, (hipStream_t)hip_stream}, path, t);
}

// Candidate settings per kernel family for this W and m (the search space of bsr_tune).
static std::vector<tuned_choice> tune_candidates(const bsr_matrix* W, int64_t m)
{
    std::vector<tuned_choice> c;
    auto add = [&](bsr_path path, int variant, int nw, int mt, int a, int b) {
        tuned_choice t;
        t.path = path;
        t.opts.variant = variant; t.opts.nw = nw; t.opts.mt = mt; t.opts.a = a; t.opts.b = b;
        c.push_back(t);
    };
    const bool thin = mfma_thin_supports(W);
    if (thin) {
        if (mfma_thinrow_supports(W) && m >= 8)
            add(BSR_PATH_MFMA, 2, 0, 0, 0, 0);
        if (W->scratch && W->scratch_bytes >= mfma_thin_scratch_bytes(W, m) && m >= 16)
            for (int a : {4, 6, 8, 10, 12, 14, 16}) add(BSR_PATH_MFMA, 1, 0, 0, a, 0);
    } else if (mfma_small_supports(W)) {
        if (m >= 8)
            for (int nw : {2, 4, 8})
                for (int per : {1, 2, 4}) add(BSR_PATH_MFMA, 0, nw, 0, per, 0);
    } else if (mfma_supports(W) && m >= 8) {
        add(BSR_PATH_MFMA, 0, 0, 0, 0, 0);                                  // the library's own choice
        for (int mt : {1, 2}) {
            if (mt == 2 && W->bs_r < 32) continue;
            for (int nw : {2, 4, 8})
                for (int per : {1, 2, 4}) add(BSR_PATH_MFMA, 2, nw, mt, per, 0);
        }
        if (mfma_group_supports(W) && m >= 64) add(BSR_PATH_MFMA, 5, 0, 0, 0, 0);   // long rows in row groups + tile kernel
        if (W->bs_r >= 32 && m >= 128) {
            for (int depth : {2, 3, 4}) add(BSR_PATH_MFMA, 3, 0, 1, depth, 0);
            for (int depth : {1, 2}) add(BSR_PATH_MFMA, 3, 0, 2, depth, 0);
        }
        for (int tm : {1, 2, 4})
            if (m >= 16 * tm && mfma_stripe_supports(W, 16 * tm)) add(BSR_PATH_MFMA, 4, 0, tm, 0, 0);
        add(BSR_PATH_MFMA, 1, 0, 0, 0, 0);
        if (W->bs_r >= 32) add(BSR_PATH_MFMA, 1, 4, 2, 0, 0);
    }
    if (m <= 64 || c.empty())                                               // the wavefront-reduction family
        for (int rows : {1, 2, 4, 8})
            if (rows <= std::max<int64_t>(m, 1) || rows == 1) add(BSR_PATH_WAVE, 0, 0, rows, 0, 0);
    return c;
}

bsr_status bsr_tune(bsr_matrix* W, int64_t m, const void* X_dev, void* Y_dev, bsr_dtype y_dtype,
                    int trials, void* hip_stream, int* tried_out, float* best_us_out)
{
    if (tried_out) *tried_out = 0;
    if (best_us_out) *best_us_out = 0.f;
    const bsr_status st = check_product_args(W, m, X_dev, Y_dev, y_dtype);
    if (st != BSR_OK || m == 0 || W->n == 0) return st;
    if (trials < 1) trials = 20;
    hipStream_t stream = (hipStream_t)hip_stream;
    const spmm_args a{W, m, X_dev, Y_dev, y_dtype, stream};
    hipEvent_t e0 = nullptr, e1 = nullptr;
    if (hipEventCreate(&e0) != hipSuccess) return BSR_ERR_HIP;
    if (hipEventCreate(&e1) != hipSuccess) { (void)hipEventDestroy(e0); return BSR_ERR_HIP; }
    tuned_choice best;
    int tried = 0;
    const bool verbose = std::getenv("BSR_TUNE_VERBOSE") != nullptr;   // one line per candidate on stderr
    bsr_status result = BSR_OK;
    for (tuned_choice cand : tune_candidates(W, m)) {
        bsr_status s = BSR_OK;
        for (int i = 0; i < 2 && s == BSR_OK; ++i) s = run_product(a, cand.path, cand.opts);     // warm-up
        if (s == BSR_ERR_UNSUPPORTED || s == BSR_ERR_WORKSPACE) continue;                         // not for this shape
        if (s != BSR_OK) { result = s; break; }
        if (hipEventRecord(e0, stream) != hipSuccess) { result = BSR_ERR_HIP; break; }
        for (int i = 0; i < trials && s == BSR_OK; ++i) s = run_product(a, cand.path, cand.opts);
        if (s != BSR_OK) { result = s; break; }
        float ms = 0.f;
        if (hipEventRecord(e1, stream) != hipSuccess || hipEventSynchronize(e1) != hipSuccess ||
            hipEventElapsedTime(&ms, e0, e1) != hipSuccess) { result = BSR_ERR_HIP; break; }
        cand.us = ms * 1000.f / (float)trials;
        ++tried;
        if (verbose)
            std::fprintf(stderr, "[bsr_tune] m=%lld path=%d variant=%d nw=%d mt=%d a=%d b=%d: %.2f us\n", (long long)m,
                         (int)cand.path, cand.opts.variant, cand.opts.nw, cand.opts.mt, cand.opts.a, cand.opts.b, cand.us);
        if (best.path == BSR_PATH_AUTO || cand.us < best.us) best = cand;
    }
    (void)hipEventDestroy(e0);
    (void)hipEventDestroy(e1);
    if (result != BSR_OK) return result;
    if (best.path != BSR_PATH_AUTO) {
        std::lock_guard<std::mutex> lock(W->tune_mu);
        W->tuned[{m, (int)y_dtype}] = best;
    }
    if (tried_out) *tried_out = tried;
    if (best_us_out) *best_us_out = best.us;
    return BSR_OK;
}

bsr_status bsr_tune_result(const bsr_matrix* W, int64_t m, bsr_dtype y_dtype, int32_t settings_out[6], float* us_out)
{
    if (!W || !settings_out) return BSR_ERR_NULL;
    std::lock_guard<std::mutex> lock(W->tune_mu);
    auto it = W->tuned.find({m, (int)y_dtype});
    if (it == W->tuned.end()) return BSR_ERR_UNSUPPORTED;
    const tuned_choice& c = it->second;
    const int32_t v[6] = {(int32_t)c.path, c.opts.variant, c.opts.nw, c.opts.mt, c.opts.a, c.opts.b};
    for (int i = 0; i < 6; ++i) settings_out[i] = v[i];
    if (us_out) *us_out = c.us;
    return BSR_OK;
}

bsr_status bsr_spmm(const bsr_matrix* W, int64_t m, const void* X_dev, void* Y_dev,
                    bsr_dtype y_dtype, void* hip_stream)
{
    return bsr_spmm_ex(W, m, X_dev, Y_dev, y_dtype, BSR_PATH_AUTO, hip_stream);
}

bsr_status bsr_spmm_static(const bsr_matrix* W, int64_t m, const void* X_dev, void* Y_dev,
                           bsr_dtype y_dtype, void* hip_stream)
{
    const bsr_status st = check_product_args(W, m, X_dev, Y_dev, y_dtype);
    if (st != BSR_OK) return st;
    if (!mfma_thin_supports(W) || y_dtype != BSR_F32) return BSR_ERR_UNSUPPORTED;
    if (m == 0 || W->n == 0) return BSR_OK;
    const spmm_args a{W, m, X_dev, Y_dev, y_dtype, (hipStream_t)hip_stream};
    if (mfma_thin_scratch_bytes(W, m) > (size_t)BSR_STATIC_SCRATCH_BYTES) return BSR_ERR_SCRATCH_LIMIT;
    order_after_upload(a.stream, W->plan_uploaded, W->plan_landed);
    if (W->debug) {
        const bsr_status dbg = debug_check_device_arrays(W, a.stream);
        if (dbg != BSR_OK) return dbg;
    }
    tune_opts t = W->env_tune;
    if (W->nnzb == 0) return launch_wave(a, t);
    return launch_mfma_thin_static(a, t);
}

const char* bsr_status_string(bsr_status s)
{
    switch (s) {
        case BSR_OK: return "ok";
        case BSR_ERR_NULL: return "a required pointer is NULL";
        case BSR_ERR_SHAPE: return "bad shape: negative size, block size not dividing n or k, or beyond int32 indexing";
        case BSR_ERR_INDPTR: return "index_pointer must start at 0, never decrease and end at the block count";
        case BSR_ERR_INDEX: return "block_indices entry outside [0, k / bs_c)";
        case BSR_ERR_DTYPE: return "unknown dtype, or output type neither the input type nor fp32";
        case BSR_ERR_ALIGN: return "device pointer not 16-byte aligned";
        case BSR_ERR_WORKSPACE: return "workspace smaller than bsr_workspace_size() reports";
        case BSR_ERR_HIP: return "HIP runtime call failed";
        case BSR_ERR_UNSUPPORTED: return "requested kernel path does not support this block shape";
        case BSR_ERR_SCRATCH_LIMIT: return "the product needs more scratch than the library's built-in array (BSR_STATIC_SCRATCH_BYTES)";
    }
    return "unknown status";
}

}  // extern "C"

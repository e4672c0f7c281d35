// Internal declarations shared by the translation units of libbsr_spmm (not installed).
#pragma once

#include <hip/hip_runtime.h>

#include <atomic>
#include <cstddef>
#include <cstdint>
#include <cstring>
#include <functional>
#include <map>
#include <mutex>
#include <vector>

#include "bsr_spmm.h"

// Row descriptor (128 bytes): {block-row, first stored block, block count, m-tile, 28 block-columns}.
constexpr int kRowDescWords = 32;
constexpr int kRowDescColsAt = 4;                 // word index of the first inline block-column
constexpr int kRowDescCols = kRowDescWords - kRowDescColsAt;
constexpr int kMaxKsplitItems = 4096;             // the k-split kernel is used below this many (block-row, m-tile) items
constexpr int kStripeChunkPairs = 3;              // the stripe kernel's pair table lists block-rows in chunks of this many pairs
constexpr int kItemSlots = 4;                     // k-split work-item tables a handle keeps (one per recent m)

// Development knobs, read from the environment variable BSR_SPMM_TUNE ("key=value,key=value"), and
// the settings bsr_tune() remembers per m.  Unset keys are 0 and mean "the library's own choice".
//   variant  1 direct, 2 ksplit, 3 tile, 4 stripe, 5 row groups + tile  (matrix-core kernel variant)
//   nw       wavefronts per workgroup      mt   MFMA tiles along m per wavefront (wave path: rows of X
//            per wavefront; ksplit: 1 = 16-row, 2 = 32-row tiles)
//   a, b     per-variant: ksplit a = blocks per wavefront; tile a = blocks in flight, b-1 = long rows
//            started first; stripe a = block-row groups; thin a = groups of 4 blocks in flight
//            thin blocks: variant 1 = transposed copy in scratch + gather, 2 = rows of X staged in LDS
//            (a = slots per wavefront)
struct tune_opts {
    int variant = 0, nw = 0, mt = 0, a = 0, b = 0;
    bool from_env = false;                   // BSR_SPMM_TUNE is set: it overrides what bsr_tune() remembered
};

// What bsr_tune() found fastest for one m: the kernel family and its settings.
struct tuned_choice {
    bsr_path path = BSR_PATH_AUTO;
    tune_opts opts;
    float us = 0.f;                          // its measured time per product
};

// Host-side description of one W.  Device pointers are borrowed from the caller.
struct bsr_matrix {
    int64_t n = 0, k = 0, nnzb = 0;
    int32_t bs_r = 0, bs_c = 0;
    int32_t R = 0, C = 0;                    // block-rows, block-columns
    bsr_dtype dtype = BSR_F32;
    const void* data = nullptr;              // [nnzb][bs_r][bs_c]
    const int32_t* indices = nullptr;        // [nnzb]
    const int32_t* indptr = nullptr;         // [R+1]

    // ---- plan (paper, Discussion: unequal block-rows need different treatment) ----
    // Block-rows ordered by stored-block count, longest first; a workgroup's slot s works on
    // block-row row_order[s], so the long rows are dispatched before the short ones.
    const int32_t* row_order = nullptr;      // device, [R]
    // Per slot, one row descriptor (m-tile word 0): one read starts a workgroup (device, [R][kRowDescWords]).
    const int32_t* row_desc = nullptr;
    // Work-item table of the k-split kernel (device, in the workspace behind row_desc): one row
    // descriptor per WORKGROUP with the m-tile filled in, ordered so that the workgroups the
    // dispatcher puts on one CU carry about the same number of stored blocks (see ksplit_items()).
    // Pair table of the stripe kernel (16x16 blocks): pair_ptr[R+1], pairs[entries][4] (see bsr_create).
    const int32_t* pair_ptr = nullptr;
    const int32_t* pairs = nullptr;
    int32_t* item_desc = nullptr;            // kItemSlots tables of item_capacity descriptors each
    size_t item_capacity = 0;                // descriptors that fit one table
    std::vector<int32_t> slot_blocks;        // stored blocks per slot (host)
    // One cached table per recent number of m-tiles; the least recently used one is replaced.
    struct item_table {
        int tiles = -1;                      // m-tiles the table was built for (-1: none)
        int grid = 0;                        // its workgroups
        uint64_t last_use = 0;
        std::vector<int32_t> host;           // host copy (kept alive for the asynchronous upload)
        hipEvent_t uploaded = nullptr;       // recorded behind the upload
        std::atomic<bool> landed{false};     // the upload is known to have finished
    };
    mutable std::mutex item_mu;              // guards the tables below
    mutable item_table item_tables[kItemSlots];
    mutable uint64_t item_clock = 0;
    // Row-group kernel (64x64 blocks of a 16-bit type, bsr_mfma_group.hip): the leading grp_slots slots (the
    // longest block-rows) are multiplied in groups of up to 8 that share their X tiles; the tile kernel takes
    // the slots behind them.  grp_desc = per group {8 block-rows (-1: none), first window record, windows, 0...}
    // (16 words), grp_recs = the window records (16 words each, layout in bsr_mfma_group.hip).
    int32_t grp_n = 0;                       // groups (0: the kernel is not used for this W)
    int32_t grp_slots = 0;                   // leading slots they cover
    int64_t grp_blocks = 0;                  // stored blocks of those slots
    const int32_t* grp_desc = nullptr;       // device
    const int32_t* grp_recs = nullptr;       // device
    std::vector<int32_t> grp_host;           // host copy of both (descriptors first), for the plan checker
    size_t grp_host_recs_at = 0;             // word offset of the records in grp_host
    // Thin blocks (16x1 fp32) whose block-rows store their blocks in non-decreasing block-column order
    // (bsr_mfma_thinrow.hip): per slot the stored-block positions where the block-columns cross the multiples
    // of 1024, [R][thin_nph + 1] (device); null when the kernel cannot take this W.
    const int32_t* thin_ph = nullptr;
    int32_t thin_nph = 0;
    int32_t thin_max_run = 0;                // stored blocks of the longest (block-row, 1024 columns) run
    // Blocks of one row (1x16 fp32: a thin W transposed) without duplicates (bsr_mfma_wide.hip): the stored blocks
    // by (block-column, block-row) as pairs {byte offset of the block, block-row}, [nnzb][2]; the chunks (at most
    // 16 pairs of one block-column inside one range of 256 block-rows) as {block-column, first pair, pairs, 0},
    // listed per (range, wavefront), and the lists' starts, [8 * wide_nq + 1] (all device); null when the kernel
    // cannot take this W.
    const int32_t* wide_pairs = nullptr;
    const int32_t* wide_chunks = nullptr;
    const int32_t* wide_chunk_ptr = nullptr;
    int32_t wide_nq = 0;
    // Debug mode (BSR_SPMM_DEBUG=1 at bsr_create, bsr_debug.hip): the device arrays are re-checked before every product
    bool debug = false;
    size_t debug_words = 0;                  // words of the plan that never change after bsr_create
    uint64_t debug_sum = 0;                  // their position-weighted sum
    int32_t* debug_out = nullptr;            // device, 4 words behind everything else in the workspace
    int n_cu = 256;                          // CUs of the device the handle was created on (entry b of a table runs on CU b mod n_cu)
    int device = 0;                          // that device
    tune_opts env_tune;                      // BSR_SPMM_TUNE as it was when the handle was created
    // Blocks smaller than an MFMA tile (bs_r, bs_c in {8,16}, not both 16; n and k multiples of 16),
    // grouped into 16x16 tiles of W (see bsr_create): descriptors of the tile-rows, longest first,
    // [sb_rows][kRowDescWords] = {tile-row, first entry, entries, 0, first tile-columns}; per entry the
    // byte offsets of the tile's blocks in block_data, [entries][4] (2^31: no block there), and its
    // tile-column, [entries].
    const int32_t* block_row = nullptr;      // device, [nnzb]: block-row of every stored block (sampled product)
    // Runs of the sampled product: every block-row cut into runs of at most sddmm_run_blocks() stored
    // blocks of about equal length, in storage order; [sd_n_runs][2] = {first block, blocks}.
    const int32_t* sd_runs = nullptr;
    int32_t sd_n_runs = 0;
    // Tiles of the sampled product (block shapes whose pieces of G or X are narrower than 128 bytes, see
    // sddmm_tile_dims): [sd_n_tiles][4] = {super-row, column group, first entry in sd_plist, position mask};
    // sd_plist holds the stored-block numbers of a tile's set positions in position order.
    const int32_t* sd_tiles = nullptr;
    const int32_t* sd_plist = nullptr;
    int32_t sd_n_tiles = 0;
    const int32_t* sb_desc = nullptr;
    const int32_t* sb_entries = nullptr;
    const int32_t* sb_cols = nullptr;
    int32_t sb_rows = 0, sb_max_entries = 0;
    int32_t max_row_blocks = 0;              // longest block-row
    int32_t long_rows = 0;                   // leading slots whose block count is > 4x the mean and > 8 ("long" bin)
    int32_t empty_rows = 0;                  // block-rows with no stored block
    double mean_row_blocks = 0.0;
    std::vector<int32_t> staging;            // host copy of what was uploaded (kept for the async copy)
    hipEvent_t plan_uploaded = nullptr;      // recorded behind that copy: products on other streams and bsr_destroy wait for it
    mutable std::atomic<bool> plan_landed{false};   // that copy is known to have finished
    // Optional per-call scratch lent by the caller (bsr_set_scratch): device memory some kernels
    // need beyond X, W and Y (the thin-block path keeps a transposed copy of X there).
    void* scratch = nullptr;
    size_t scratch_bytes = 0;
    // bsr_tune() results, keyed by (m, output type)
    mutable std::mutex tune_mu;
    std::map<std::pair<int64_t, int>, tuned_choice> tuned;
};

// Arguments every kernel launcher takes.
struct spmm_args {
    const bsr_matrix* W;
    int64_t m;
    const void* X;
    void* Y;
    bsr_dtype y_dtype;
    hipStream_t stream;
    int first_slot = 0;                      // tile kernel: leave out the slots before this one (another kernel multiplies them)
};

tune_opts read_tune_env();
// Debug mode: checks index_pointer, block_indices and the plan on the device (one launch, a copy and a stream
// synchronisation); BSR_OK when the handle is not in debug mode or the stream is being captured.
bsr_status debug_check_device_arrays(const bsr_matrix* W, hipStream_t stream);
uint64_t debug_plan_sum(const int32_t* words, size_t n);

// Stored blocks of one block-row that a workgroup of the sampled product takes together (they share
// the piece of G): 4 while a block is at most 2 KiB, else 2.
// Tile of the sampled product: sr adjacent block-rows x lc adjacent block-columns, as many as make a
// 128-byte line of a row of G and of X (1 when a block's piece is a line or more).
inline void sddmm_tile_dims(int bs_r, int bs_c, bsr_dtype t, int* sr, int* lc)
{
    const int s = t == BSR_F32 ? 4 : 2;
    *sr = bs_r * s >= 128 ? 1 : 128 / (bs_r * s);
    *lc = bs_c * s >= 128 ? 1 : 128 / (bs_c * s);
}
inline int sddmm_run_blocks(int bs_r, int bs_c, bsr_dtype t) { return bs_r * bs_c * (t == BSR_F32 ? 4 : 2) <= 2048 ? 4 : 2; }

// Each returns BSR_OK, BSR_ERR_UNSUPPORTED (shape not covered by that family) or BSR_ERR_HIP.
bsr_status launch_wave(const spmm_args& a, const tune_opts& t);
bsr_status launch_mfma(const spmm_args& a, const tune_opts& t);
bool mfma_supports(const bsr_matrix* W);

// matrix-core kernel variants (bsr_mfma*.hip)
bsr_status launch_mfma_direct(const spmm_args& a, const tune_opts& t);
bsr_status launch_mfma_ksplit(const spmm_args& a, const tune_opts& t);
// Builds (or reuses) the k-split work-item table for `tiles` m-tiles, queues its upload on `stream` (or
// makes `stream` wait for an upload another stream still has in flight); returns the number of
// workgroups and the table's device address, 0 if the table does not fit the workspace.
int ksplit_items(const bsr_matrix* W, int tiles, hipStream_t stream, const int32_t** table_out);
// One cached per-m table out of `tables` (kItemSlots of them, `capacity_words` int32 each, starting at
// `dev_base`): the one built for `key`, else `build` fills a host vector (returning the number of
// workgroups, 0 = does not fit) that is uploaded into the least recently used slot on `stream`.
// Returns the workgroups and the table's device address; 0 if there is no table.  Caller holds no lock.
int cached_table(const bsr_matrix* W, bsr_matrix::item_table* tables, int key, hipStream_t stream, int32_t* dev_base,
                 size_t capacity_words, const std::function<int(std::vector<int32_t>&)>& build, const int32_t** table_out);
// Makes `stream` wait (on the device) for the upload recorded as `ev`, unless it is known to have
// finished.  Under stream capture nothing is recorded: an event from outside the capture cannot be
// waited for there, and a caller that captures a handle's first product orders it itself.
void order_after_upload(hipStream_t stream, hipEvent_t ev, std::atomic<bool>& landed);
bsr_status launch_mfma_tile(const spmm_args& a, const tune_opts& t);
// Row-group kernel: the grouped (longest) block-rows of a W with 64x64 blocks of a 16-bit type; the caller
// launches the tile kernel with first_slot = W->grp_slots for the rest
bsr_status launch_mfma_group(const spmm_args& a, const tune_opts& t);
bool mfma_group_supports(const bsr_matrix* W);
// Chooses the grouped block-rows of W and appends their descriptors and window records to the plan being
// staged (`words` = its length so far, 64-word aligned on return); leaves W->grp_n = 0 when the shape is not
// the kernel's or no block-row is long enough.  group_plan_words: what the workspace must hold for it.
void build_group_plan(bsr_matrix* W, const int32_t* index_pointer_host, const int32_t* block_indices_host, size_t* words);
size_t group_plan_words(int64_t R, int32_t bs_r, int32_t bs_c, int64_t nnzb);
bsr_status launch_mfma_stripe(const spmm_args& a, const tune_opts& t);
bool mfma_stripe_supports(const bsr_matrix* W, int tm);   // 16x16 blocks, 16-bit type, tm rows of X fit in LDS
bsr_status launch_mfma_thin(const spmm_args& a, const tune_opts& t);    // bs_r = 16, bs_c = 1, fp32; needs scratch
// The same product on the library's built-in scratch array (no lent scratch needed); BSR_ERR_SCRATCH_LIMIT
// when the product needs more than BSR_STATIC_SCRATCH_BYTES.
bsr_status launch_mfma_thin_static(const spmm_args& a, const tune_opts& t);
// Resolves the built-in scratch array's device address for the current device (once per device).
bsr_status mfma_thin_static_scratch(void** out);
bool mfma_thin_supports(const bsr_matrix* W);
// The same product in one launch, rows of X staged in LDS (no scratch): needs sorted block-rows, k % 4 == 0
bsr_status launch_mfma_thinrow(const spmm_args& a, const tune_opts& t);
bool mfma_thinrow_supports(const bsr_matrix* W);
void build_thinrow_plan(bsr_matrix* W, const int32_t* index_pointer_host, const int32_t* block_indices_host, size_t* words);
size_t thinrow_plan_words(int64_t R, int64_t k, int32_t bs_r, int32_t bs_c);
// bs_r = 1, bs_c = 16, fp32, no block stored twice: by block-column on the matrix cores, sums in LDS
bsr_status launch_mfma_wide(const spmm_args& a, const tune_opts& t);
bool mfma_wide_supports(const bsr_matrix* W);
void build_wide_plan(bsr_matrix* W, const int32_t* index_pointer_host, const int32_t* block_indices_host, size_t* words);
size_t wide_plan_words(int64_t R, int64_t k, int64_t nnzb, int32_t bs_r, int32_t bs_c);
bsr_status launch_mfma_small(const spmm_args& a, const tune_opts& t);   // bs_r, bs_c in {8,16}, not both 16
bool mfma_small_supports(const bsr_matrix* W);
size_t mfma_thin_scratch_bytes(const bsr_matrix* W, int64_t m);   // bytes of the transposed copy of X
// XT[c][i] = X[i][c], rows of XT (m rounded up to 4) floats apart
bsr_status launch_transpose_f32(const float* X, float* XT, int m, int k, hipStream_t stream);

// Expands to a chain of `if (shape matches) return FN<T, O, BR, BC>(args...)` over the block
// shapes the matrix-core kernels are instantiated for.
#define BSR_MFMA_SHAPES(FN, T, O, br, bc, ...)                                             \
    do {                                                                                   \
        if (br == 16 && bc == 16) return FN<T, O, 16, 16>(__VA_ARGS__);                    \
        if (br == 16 && bc == 32) return FN<T, O, 16, 32>(__VA_ARGS__);                    \
        if (br == 16 && bc == 64) return FN<T, O, 16, 64>(__VA_ARGS__);                    \
        if (br == 32 && bc == 16) return FN<T, O, 32, 16>(__VA_ARGS__);                    \
        if (br == 32 && bc == 32) return FN<T, O, 32, 32>(__VA_ARGS__);                    \
        if (br == 32 && bc == 64) return FN<T, O, 32, 64>(__VA_ARGS__);                    \
        if (br == 64 && bc == 16) return FN<T, O, 64, 16>(__VA_ARGS__);                    \
        if (br == 64 && bc == 32) return FN<T, O, 64, 32>(__VA_ARGS__);                    \
        if (br == 64 && bc == 64) return FN<T, O, 64, 64>(__VA_ARGS__);                    \
    } while (0)

// Dispatch on (input type, output type) to FN<T, O, BR, BC>(args...).
#define BSR_MFMA_DISPATCH(FN, W, y_dtype, ...)                                                            \
    do {                                                                                                  \
        const int br_ = (W)->bs_r, bc_ = (W)->bs_c;                                                       \
        if ((W)->dtype == BSR_F32) BSR_MFMA_SHAPES(FN, float, float, br_, bc_, __VA_ARGS__);              \
        if ((W)->dtype == BSR_F16 && (y_dtype) == BSR_F32) BSR_MFMA_SHAPES(FN, _Float16, float, br_, bc_, __VA_ARGS__);   \
        if ((W)->dtype == BSR_F16) BSR_MFMA_SHAPES(FN, _Float16, _Float16, br_, bc_, __VA_ARGS__);        \
        if ((W)->dtype == BSR_BF16 && (y_dtype) == BSR_F32) BSR_MFMA_SHAPES(FN, __bf16, float, br_, bc_, __VA_ARGS__);    \
        if ((W)->dtype == BSR_BF16) BSR_MFMA_SHAPES(FN, __bf16, __bf16, br_, bc_, __VA_ARGS__);           \
    } while (0)

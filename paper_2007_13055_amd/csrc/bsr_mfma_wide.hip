// Matrix-core kernel for wide blocks of one row: bs_r = 1, bs_c = 16, fp32 -- the shape a thin (16x1) W has
// once it is transposed, i.e. the sibling product Z = G*W of a layer with thin blocks run through the handle
// of W^T (here, as everywhere in the library, the product is Y = X * W^T of the handle's own W; the paper's
// Introduction has the sparse layers trained as well as run, and training needs the product with W itself).
//
// A 1x16 block couples 16 columns of X with ONE column of Y, so in the definition's form (per output column:
// a sum over its stored blocks) no two output columns share a reduction index and a matrix-core tile would
// use one of its 16 columns.  Turned round, by block-COLUMN j of W, it is dense: all stored blocks p of
// block-column j multiply the same 16 columns of X,
//     D[i][p] = sum_a X[i][16 j + a] * block_data[p][0][a]          (16 rows of X) x (16 a) x (16 blocks p)
// which is one 16x16x16 product per 16 blocks, and D[i][p] is a term of Y[i][block-row of p].  The terms are
// added where they belong in LDS: a workgroup owns 16 rows of X and a range of 256 output columns, each of
// its 8 wavefronts keeps a private 16 x 256 tile of partial sums there, takes an eighth of the block-columns, and
// adds its D values into its own tile (LDS add instructions on addresses that differ within an instruction;
// a wavefront's LDS operations execute in order, so the order of additions is fixed and runs repeat bit for
// bit).  At the end the 8 tiles are summed in fixed order and stored as whole rows of 1 KiB.
//
// Plan (bsr_create): the stored blocks sorted by (block-column, block-row) as pairs {byte offset of the block,
// block-row}, and per (range, wavefront) the list of its chunks; a W that stores a block twice is left to the
// other kernels (two terms of one instruction would meet in one address).
//
// Per 16 blocks of a (block-column, range) run -- a CHUNK -- a wavefront issues three loads: the chunk's 16
// pairs (eight chunks ahead), then with their offsets the blocks as the MFMA's B operand (lane l: 16 bytes =
// entries 4*(l/16) .. +3 of block l%16) and the 16 x 16 piece of X as its A operand (lane l: row l%16, the
// same entries), four chunks ahead.  The four v_mfma_f32_16x16x4_f32 of a chunk take component s of both
// registers, so the reduction index of step s and lane group g is entry 4g + s on both sides.  Lanes past
// the chunk's end read zeros for their block (a buffer load past the end) and add them to a clamped address.
#include <algorithm>

#include "bsr_mfma_common.h"

using namespace bsr_dev;

namespace {

constexpr int kRowsX = 16;                            // rows of X per workgroup
constexpr int kQW = 256;                              // output columns per workgroup
constexpr int kTS = kQW + 4;                          // tile row stride in words: rows 4 apart shift by 16 banks
constexpr int kTile = kRowsX * kTS * 4;               // one wavefront's tile, bytes
constexpr int kWv = 8;                                // wavefronts per workgroup
constexpr int kLds = kWv * kTile;
constexpr int kThreads = 64 * kWv;
static_assert(kLds <= 160 * 1024 && kTile % 16 == 0, "LDS; 16-byte writes clear a tile");

struct chunk_t { int j, e, cnt; };                    // block-column, first pair, pairs (0: none)

__global__ __launch_bounds__(kThreads) void bsr_wide16_f32(const float* __restrict__ X, const float* __restrict__ data,
                                                          const int32_t* __restrict__ pairs,
                                                          const int32_t* __restrict__ chunks,
                                                          const int32_t* __restrict__ chunk_ptr, float* __restrict__ Y,
                                                          int m, int k, int n, int nq, int n_rg,
                                                          unsigned data_bytes)
{
    extern __shared__ __attribute__((aligned(1024))) unsigned char lds[];
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int lo = lane & 15, kk = lane >> 4;

    // Workgroup -> (row group, column range).  The 8 XCDs take workgroups round-robin and have private L2s:
    // XCD x works on the row groups x%4, x%4 + 4, ... and the ranges x/4, x/4 + 2, ..., so a row of X is
    // fetched into 2 of the 8 L2s and a block into 4.
    const int x = (int)(blockIdx.x % 8u), local = (int)(blockIdx.x / 8u);
    const int rgs_here = (n_rg - (x & 3) + 3) >> 2, qs_here = (nq - (x >> 2) + 1) >> 1;
    if (rgs_here <= 0 || qs_here <= 0) return;        // whole workgroup leaves together
    const int ri = local / qs_here, qi = local - ri * qs_here;
    if (ri >= rgs_here) return;
    const int rg = (x & 3) + 4 * ri, q = (x >> 2) + 2 * qi;
    const int i0 = rg * kRowsX, c0 = q * kQW;

    // this wavefront's tile, cleared
    unsigned char* const tile = lds + wave * kTile;
    for (int o = lane * 16; o < kTile; o += 64 * 16) *reinterpret_cast<u32x4*>(tile + o) = u32x4{0u, 0u, 0u, 0u};

    const int ln = lane >> 2, lp = lane & 3;          // line order: row (block) and 16-byte piece this lane loads
    const unsigned char* const xrow = reinterpret_cast<const unsigned char*>(X) + (size_t)min(i0 + ln, m - 1) * (size_t)k * 4u + lp * 16;
    // MFMA lane l (row or block l%16, piece l/16) takes what line-order lane 4*(l%16) + l/16 loaded
    const int from = (4 * lo + kk) * 4;
    auto to_mfma = [&](u32x4 v) __attribute__((always_inline)) {
        u32x4 r;
        r.x = (uint32_t)__builtin_amdgcn_ds_bpermute(from, (int)v.x);
        r.y = (uint32_t)__builtin_amdgcn_ds_bpermute(from, (int)v.y);
        r.z = (uint32_t)__builtin_amdgcn_ds_bpermute(from, (int)v.z);
        r.w = (uint32_t)__builtin_amdgcn_ds_bpermute(from, (int)v.w);
        return __builtin_bit_cast(f32x4, r);
    };
    const __amdgpu_buffer_rsrc_t wrsrc = __builtin_amdgcn_make_buffer_rsrc(const_cast<float*>(data), 0, (int)data_bytes, 0x00020000);
    // where this lane's four results of a chunk go: rows 4*kk + jj of the tile, column = the block's block-row
    unsigned char* const t_at = tile + (4 * kk) * (kTS * 4);

    // The wavefront's chunks (its share of this range's block-columns, their pairs 16 at a time) are
    // listed in the plan; their descriptors {block-column, first pair, pairs} come 64 at a time, one per lane.
    const int lst = __builtin_amdgcn_readfirstlane(chunk_ptr[q * kWv + wave]);
    const int lend = __builtin_amdgcn_readfirstlane(chunk_ptr[q * kWv + wave + 1]);
    for (int b0 = lst; b0 < lend; b0 += 64) {         // uniform
        const int n_chunks = min(64, lend - b0);
        const __amdgpu_buffer_rsrc_t crsrc =
            __builtin_amdgcn_make_buffer_rsrc(const_cast<int32_t*>(chunks + 4 * (size_t)b0), 0, n_chunks * 16, 0x00020000);
        const u32x4 desc = __builtin_bit_cast(u32x4, __builtin_amdgcn_raw_buffer_load_b128(crsrc, lane * 16, 0, 0));
        int next_s = 0;
        auto next_chunk = [&]() __attribute__((always_inline)) {
            const int s_ = next_s++;                  // a turn past the 64th (the ring looks 8 ahead): no chunk
            const int at = min(s_, 63);
            chunk_t c;
            c.j = __builtin_amdgcn_readlane((int)desc.x, at);
            c.e = __builtin_amdgcn_readlane((int)desc.y, at);
            c.cnt = s_ < 64 ? __builtin_amdgcn_readlane((int)desc.z, at) : 0;
            return c;
        };
        // Loads go out in LINE order: lanes 4n .. 4n+3 take the four 16-byte pieces of block n (of row n of X), so
        // that each quad of lanes falls into one line -- a load whose neighbouring lanes sit in 16 different lines
        // keeps the CU's memory pipeline busy four times as long, and that pipeline is what bounds this kernel.
        // The MFMA wants lane l to hold piece l/16 of block (row) l%16: to_mfma() moves a register there.
        // a chunk's pairs, pair n in lanes 4n .. 4n+3: {byte offset of the block, its block-row}; zeros past its end
        auto load_pairs = [&](const chunk_t& c) __attribute__((always_inline)) {
            const __amdgpu_buffer_rsrc_t r =
                __builtin_amdgcn_make_buffer_rsrc(const_cast<int32_t*>(pairs + 2 * (size_t)c.e), 0, c.cnt * 8, 0x00020000);
            return __builtin_amdgcn_raw_buffer_load_b64(r, ln * 8, 0, 0);
        };
        auto load_b = [&](const chunk_t& c, u32x2 pc) __attribute__((always_inline)) {
            const unsigned off = ln < c.cnt ? pc.x + (unsigned)lp * 16u : 0x80000000u;   // past the end of W: zeros
            return __builtin_bit_cast(u32x4, __builtin_amdgcn_raw_buffer_load_b128(wrsrc, (int)off, 0, 0));
        };
        auto load_a = [&](const chunk_t& c) __attribute__((always_inline)) {
            return *reinterpret_cast<const u32x4*>(xrow + (size_t)c.j * 64u);
        };

        // A ring of 8 chunks: the pairs of a chunk are loaded 8 chunks ahead of its turn, its operands 4 ahead
        // (with the pairs' offsets, which have had 4 turns to arrive), so a turn waits only for loads that are
        // several turns old.
        constexpr int kRing = 8, kAhead = 4;
        chunk_t ch[kRing];
        u32x2 pc[kRing];
        u32x4 av[kRing], bv[kRing];
#pragma unroll
        for (int u = 0; u < kRing; ++u) {
            ch[u] = next_chunk();
            pc[u] = __builtin_bit_cast(u32x2, load_pairs(ch[u]));
        }
#pragma unroll
        for (int u = 0; u < kAhead; ++u) {
            bv[u] = load_b(ch[u], pc[u]);
            av[u] = load_a(ch[u]);
        }
        // the turns are taken 8 at a time without branches (a turn behind the last chunk multiplies zeros and
        // adds them to the tile's padding), so every wait counts loads exactly
        for (int base = 0; base < n_chunks; base += kRing) {   // uniform
#pragma unroll
            for (int u = 0; u < kRing; ++u) {
                // D = A x B over the 16 entries: step s takes entry 4*kk + s from both sides
                const f32x4 am = to_mfma(av[u]), bm = to_mfma(bv[u]);
                const int row_of_block = __builtin_amdgcn_ds_bpermute(lo * 16, (int)pc[u].y);   // pair l%16 sits in lane 4*(l%16)
                f32x4 d0 = {0.f, 0.f, 0.f, 0.f}, d1 = {0.f, 0.f, 0.f, 0.f};
                d0 = __builtin_amdgcn_mfma_f32_16x16x4f32(am.x, bm.x, d0, 0, 0, 0);
                d1 = __builtin_amdgcn_mfma_f32_16x16x4f32(am.y, bm.y, d1, 0, 0, 0);
                d0 = __builtin_amdgcn_mfma_f32_16x16x4f32(am.z, bm.z, d0, 0, 0, 0);
                d1 = __builtin_amdgcn_mfma_f32_16x16x4f32(am.w, bm.w, d1, 0, 0, 0);
                // lane l holds rows 4*kk + jj (jj = 0..3) of D, column = block l%16 of the chunk
                // (lanes past the chunk's end: the row's padding, which nobody reads)
                const unsigned rel = lo < ch[u].cnt ? min((unsigned)(row_of_block - c0), (unsigned)(kQW - 1)) : (unsigned)kQW;
                float* dst = reinterpret_cast<float*>(t_at + rel * 4u);
#pragma unroll
                for (int jj = 0; jj < 4; ++jj) dst[jj * kTS] += d0[jj] + d1[jj];
                ch[u] = next_chunk();
                pc[u] = __builtin_bit_cast(u32x2, load_pairs(ch[u]));
                const int v = (u + kAhead) % kRing;
                bv[v] = load_b(ch[v], pc[v]);
                av[v] = load_a(ch[v]);
            }
        }
    }

    __syncthreads();
    // Y tile = the 8 tiles added in wavefront order; whole rows of the range, 16 bytes per thread
    const int cols = min(kQW, n - c0);
    if ((n & 3) == 0) {
        for (int idx = threadIdx.x; idx < kRowsX * (kQW / 4); idx += kThreads) {
            const int row = idx / (kQW / 4), c4 = idx % (kQW / 4);
            if (i0 + row < m && 4 * c4 < cols) {
                f32x4 sum = *reinterpret_cast<const f32x4*>(lds + (row * kTS + 4 * c4) * 4);
#pragma unroll
                for (int w = 1; w < kWv; ++w) sum += *reinterpret_cast<const f32x4*>(lds + w * kTile + (row * kTS + 4 * c4) * 4);
                *reinterpret_cast<f32x4*>(Y + (size_t)(i0 + row) * n + c0 + 4 * c4) = sum;
            }
        }
    } else {
        for (int idx = threadIdx.x; idx < kRowsX * kQW; idx += kThreads) {
            const int row = idx / kQW, c = idx % kQW;
            if (i0 + row < m && c < cols) {
                float sum = *reinterpret_cast<const float*>(lds + (row * kTS + c) * 4);
#pragma unroll
                for (int w = 1; w < kWv; ++w) sum += *reinterpret_cast<const float*>(lds + w * kTile + (row * kTS + c) * 4);
                Y[(size_t)(i0 + row) * n + c0 + c] = sum;
            }
        }
    }
}

}  // namespace

size_t wide_plan_words(int64_t R, int64_t k, int64_t nnzb, int32_t bs_r, int32_t bs_c)
{
    if (bs_r != 1 || bs_c != 16) return 0;
    // pairs (2 words per stored block), chunk descriptors (4 words; a chunk per 16 pairs of a run and one more per
    // run, and no more runs than stored blocks), the lists' starts (8 per range), padding
    return 2 * (size_t)nnzb + 4 * ((size_t)nnzb + (size_t)nnzb / 16 + 1) + (size_t)kWv * (size_t)((R + kQW - 1) / kQW) + 1 + 256;
}

bool mfma_wide_supports(const bsr_matrix* W) { return W->wide_pairs != nullptr; }

void build_wide_plan(bsr_matrix* W, const int32_t* ptr, const int32_t* idx, size_t* words)
{
    W->wide_pairs = nullptr;
    W->wide_chunks = nullptr;
    W->wide_chunk_ptr = nullptr;
    W->wide_nq = 0;
    if (W->bs_r != 1 || W->bs_c != 16 || W->dtype != BSR_F32 || W->R <= 0 || W->C <= 0) return;
    if (W->nnzb <= 0 || W->nnzb >= ((int64_t)1 << 25)) return;   // byte offsets into block_data are 32-bit
    const int R = W->R, C = W->C, nq = (R + kQW - 1) / kQW;
    // stored blocks per block-column; a block-row that stores a block-column twice leaves the kernel out
    std::vector<int32_t> first((size_t)C + 1, 0), seen((size_t)C, -1);
    for (int r = 0; r < R; ++r)
        for (int32_t p = ptr[r]; p < ptr[r + 1]; ++p) {
            if (seen[idx[p]] == r) return;
            seen[idx[p]] = r;
            ++first[(size_t)idx[p] + 1];
        }
    for (int j = 0; j < C; ++j) first[j + 1] += first[j];
    // block-rows in ascending order: every block-column's pairs come out sorted by block-row
    std::vector<int32_t> pairs(2 * (size_t)W->nnzb), at(first.begin(), first.end() - 1);
    for (int r = 0; r < R; ++r)
        for (int32_t p = ptr[r]; p < ptr[r + 1]; ++p) {
            const int32_t o = at[idx[p]]++;
            pairs[2 * (size_t)o] = p * 64;
            pairs[2 * (size_t)o + 1] = r;
        }
    // Chunk lists: for every range q and wavefront w, the runs of its block-columns (the pairs of block-column j
    // whose block-rows fall into the range) cut into chunks of at most 16 pairs: {j, first pair, pairs, 0}.
    std::vector<int32_t> chunks, chunk_ptr;
    std::vector<int32_t> cur(first.begin(), first.end() - 1);    // per block-column: first pair not yet listed
    for (int qq = 0; qq < nq; ++qq) {
        // the pairs of block-column j inside range qq are [cur[j], lim[j])
        std::vector<int32_t> lim((size_t)C);
        for (int j = 0; j < C; ++j) {
            int32_t o = cur[j];
            while (o < first[j + 1] && pairs[2 * (size_t)o + 1] < (qq + 1) * kQW) ++o;
            lim[j] = o;
        }
        // The block-columns go to the wavefronts so that all get about the same number of chunks: longest run
        // first, each to the wavefront with the fewest chunks so far (the workgroup waits for its slowest).
        std::vector<int32_t> order;
        for (int j = 0; j < C; ++j)
            if (lim[j] > cur[j]) order.push_back(j);
        std::stable_sort(order.begin(), order.end(), [&](int32_t x, int32_t y) {
            return (lim[x] - cur[x] + 15) / 16 > (lim[y] - cur[y] + 15) / 16;
        });
        std::vector<int32_t> mine[kWv];
        int64_t load[kWv] = {};
        for (const int32_t j : order) {
            int w = 0;
            for (int v = 1; v < kWv; ++v)
                if (load[v] < load[w]) w = v;
            mine[w].push_back(j);
            load[w] += (lim[j] - cur[j] + 15) / 16;
        }
        for (int w = 0; w < kWv; ++w) {
            chunk_ptr.push_back((int32_t)(chunks.size() / 4));
            std::sort(mine[w].begin(), mine[w].end());           // ascending block-column: neighbouring pieces of X in turn
            for (const int32_t j : mine[w])
                for (int32_t e = cur[j]; e < lim[j]; e += 16) {
                    chunks.push_back(j);
                    chunks.push_back(e);
                    chunks.push_back(std::min<int32_t>(16, lim[j] - e));
                    chunks.push_back(0);
                }
        }
        cur = lim;
    }
    chunk_ptr.push_back((int32_t)(chunks.size() / 4));
    const size_t pairs_at = *words, chunks_at = (pairs_at + pairs.size() + 63) & ~(size_t)63;
    const size_t ptr_at = (chunks_at + chunks.size() + 63) & ~(size_t)63;
    const size_t end = (ptr_at + chunk_ptr.size() + 63) & ~(size_t)63;
    W->staging.resize(end + 64, 0);
    std::copy(pairs.begin(), pairs.end(), W->staging.begin() + (ptrdiff_t)pairs_at);
    std::copy(chunks.begin(), chunks.end(), W->staging.begin() + (ptrdiff_t)chunks_at);
    std::copy(chunk_ptr.begin(), chunk_ptr.end(), W->staging.begin() + (ptrdiff_t)ptr_at);
    W->wide_pairs = W->row_order + pairs_at;
    W->wide_chunks = W->row_order + chunks_at;
    W->wide_chunk_ptr = W->row_order + ptr_at;
    W->wide_nq = nq;
    *words = end;
}

bsr_status launch_mfma_wide(const spmm_args& a, const tune_opts&)
{
    const bsr_matrix* W = a.W;
    if (!mfma_wide_supports(W) || a.y_dtype != BSR_F32) return BSR_ERR_UNSUPPORTED;
    const int m = (int)a.m, n = (int)W->n, k = (int)W->k;
    const int n_rg = (m + kRowsX - 1) / kRowsX, nq = W->wide_nq;
    const int64_t grid = 8 * (int64_t)((n_rg + 3) / 4) * ((nq + 1) / 2);
    if (grid >= ((int64_t)1 << 31)) return BSR_ERR_SHAPE;
    static const hipError_t attr = hipFuncSetAttribute(reinterpret_cast<const void*>(&bsr_wide16_f32),
                                                       hipFuncAttributeMaxDynamicSharedMemorySize, kLds);
    if (attr != hipSuccess) return BSR_ERR_HIP;
    hipLaunchKernelGGL(bsr_wide16_f32, dim3((unsigned)grid), dim3(kThreads), kLds, a.stream, (const float*)a.X,
                       (const float*)W->data, W->wide_pairs, W->wide_chunks, W->wide_chunk_ptr, (float*)a.Y, m, k, n,
                       nq, n_rg, (unsigned)(W->nnzb * 64));
    return hipGetLastError() == hipSuccess ? BSR_OK : BSR_ERR_HIP;
}

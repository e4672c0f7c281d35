// Matrix-core kernels for thin blocks: bs_r = 16, bs_c = 1, fp32.
//
// A 16x1 block couples one column of X with 16 columns of Y, so a block-row is a small dense
// product over a GATHER of X columns:
//     Y[:, r*16 : r*16+16] = X[:, block_indices[p0..p1)] * block_data[p0..p1, :, 0]
// Columns of a row-major X are strided (one element per 4k-byte row), so gathering them directly
// would move a cache line per element.  The product therefore runs in two launches:
//   1. transpose X (m x k) into a scratch XT (k x m): a column of X becomes a contiguous row;
//   2. per block-row and per 64 rows of X: MFMA 16x16x4 over 4 stored blocks at a time, the
//      A operand gathered from XT rows (16 consecutive floats per lane group), the B operand the
//      4 blocks themselves (64 consecutive floats = one coalesced read).
// The lanes that share an output element's reduction are inside the matrix core here; what the
// paper's reduction kernels do with explicit cross-thread sums (Sections 4.4.2-4.4.3) the MFMA
// does across its k = 4 lane groups.
#include "bsr_mfma_common.h"

using namespace bsr_dev;

namespace {

// XT[c][i] = X[i][c], rows of XT mp floats apart (m rounded up to a multiple of 4, so every row starts
// 16-byte aligned); tiles of 32 rows x 64 columns of X through LDS, 16 bytes per lane on both sides.
__global__ __launch_bounds__(256) void transpose_f32(const float* __restrict__ X, float* __restrict__ XT, int m, int k, int mp)
{
    constexpr int TI = 32, TC = 64;
    __shared__ float tile[TI][TC + 1];
    const int c0 = blockIdx.x * TC, i0 = blockIdx.y * TI;
    const bool full = c0 + TC <= k && i0 + TI <= m && (k & 3) == 0;
    if (full) {
        {   // read: 16 lanes cover one row's 64 columns
            const int tx = threadIdx.x & 15, ty = threadIdx.x >> 4;
#pragma unroll
            for (int j = 0; j < TI / 16; ++j) {
                const int i = ty + 16 * j;
                const f32x4 v = *reinterpret_cast<const f32x4*>(X + (size_t)(i0 + i) * k + c0 + 4 * tx);
                tile[i][4 * tx] = v.x; tile[i][4 * tx + 1] = v.y; tile[i][4 * tx + 2] = v.z; tile[i][4 * tx + 3] = v.w;
            }
        }
        __syncthreads();
        {   // write: 8 lanes cover one XT row's 32 entries
            const int tx = threadIdx.x & 7, ty = threadIdx.x >> 3;
#pragma unroll
            for (int j = 0; j < TC / 32; ++j) {
                const int c = ty + 32 * j;
                const f32x4 v = {tile[4 * tx][c], tile[4 * tx + 1][c], tile[4 * tx + 2][c], tile[4 * tx + 3][c]};
                *reinterpret_cast<f32x4*>(XT + (size_t)(c0 + c) * mp + i0 + 4 * tx) = v;
            }
        }
    } else {                                          // ragged edge tile: element by element
        for (int e = threadIdx.x; e < TI * TC; e += 256) {
            const int i = e / TC, c = e % TC;
            tile[i][c] = (i0 + i < m && c0 + c < k) ? X[(size_t)(i0 + i) * k + c0 + c] : 0.f;
        }
        __syncthreads();
        for (int e = threadIdx.x; e < TI * TC; e += 256) {
            const int c = e / TI, i = e % TI;
            if (c0 + c < k && i0 + i < m) XT[(size_t)(c0 + c) * mp + i0 + i] = tile[i][c];
        }
    }
}

// One workgroup: the block-row of slot `slot`, 64 rows of X.  Its 4 wavefronts share out the
// stored blocks of the block-row in contiguous quarters (the paper's concurrent reduction, Section
// 4.4: several threads share one output's reduction and the partial results are added at the end);
// each keeps a 64 x 16 partial result, and the partial results are summed through LDS in fixed
// order.  Per MFMA 16x16x4:
//   A operand (rows of the result = rows of X): lane l supplies XT[col(p + l/16)][i0 + 4*(l%16) + s]
//     for the s-th of the wavefront's 4 MFMAs -- the 16 rows of MFMA s are rows s, 4+s, 8+s, ... of
//     the 64-row tile, so that ONE 16-byte load per lane (4 consecutive entries of an XT row) feeds
//     all four; neighbouring lanes read neighbouring 16-byte pieces, which the memory pipeline
//     serves four times faster than four 4-byte reads 64 bytes apart
//   B operand (columns = the 16 outputs of the block-row): lane l supplies block_data[p + l/16][l%16]
//   result of MFMA s: lane l holds tile rows 16*(l/16) + 4*j + s (j = 0..3), column l%16
// A wavefront works through its share in chunks of U groups of 4 blocks.  Per chunk it reads the
// block-columns with one load (lane l takes block l of the chunk) and hands them to the lane groups
// with ds_bpermute, reads the blocks themselves as contiguous 16-byte pieces into its own LDS area
// and takes its B operands from there, then issues all U gathers from XT before the first MFMA, so
// one memory latency covers up to 4*U blocks.  (Reading W and the block-columns one float per lane
// cost 2*U load instructions per chunk, each occupying the memory pipeline for 16 cycles whatever
// it carries: 3.4 of the kernel's 8.9 us.)  Blocks and block-columns are read through buffer
// resources over the wavefront's share, so pieces past its end read as zero without branches.
template <int U>
__global__ __launch_bounds__(256) void bsr_thin16_f32(const float* __restrict__ XT, const float* __restrict__ data,
                                                      const int32_t* __restrict__ indices,
                                                      const int32_t* __restrict__ row_desc, float* __restrict__ Y,
                                                      int m, int n, int R, int mg)
{
    constexpr int SUBS = 4;                           // 16-row MFMA tiles per wavefront: 64 rows
    constexpr int WT = (U * 256 + 1023) / 1024;       // 1 KiB pieces of W per chunk (a block is 64 bytes)
    __shared__ float red[4][64][17];
    __shared__ __attribute__((aligned(16))) unsigned char wstage[4][WT * 1024];
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int lo = lane & 15, pp = lane >> 4;
    // Workgroup -> (m-tile, slot).  The 8 XCDs take workgroups round-robin and have private L2s; XCD x
    // works on the m-tiles t = x mod G (mod G) and the slots s = x div G (mod 8/G): it then gathers
    // only from its own m-tiles' columns of XT -- with G = 8 every part of XT is fetched by one XCD
    // only -- at the price of W being read by G XCDs (`mg` = G, a power of two up to 8).
    const int x = (int)(blockIdx.x % 8u), j = (int)(blockIdx.x / 8u);
    const int rg = 8 / mg;                            // slot groups
    const int slots_here = (R - x / mg + rg - 1) / rg;   // slots of this XCD: x div G, x div G + 8/G, ...
    const int ti = j / max(slots_here, 1), si = j - ti * max(slots_here, 1);
    const int tile = x % mg + ti * mg, slot = x / mg + si * rg;
    if (slots_here <= 0 || tile * 64 >= m) return;    // whole workgroup leaves together
    const int i0 = tile * 64;
    const int32_t* __restrict__ desc = row_desc + (size_t)slot * kRowDescWords;
    const int r = desc[0];
    const int p0 = desc[1], nb = desc[2];
    const unsigned row_bytes = (unsigned)((m + 3) & ~3) * 4u;      // one row of XT (padded to 16 bytes)
    const int share = ((nb + 3) / 4 + 3) / 4 * 4;     // blocks per wavefront, a multiple of 4
    const int qb = p0 + min(wave * share, nb), qe = p0 + min((wave + 1) * share, nb);

    f32x4 acc[SUBS];
#pragma unroll
    for (int s = 0; s < SUBS; ++s) acc[s] = f32x4{0.f, 0.f, 0.f, 0.f};

    // The gather for group u reads XT + (col*mp + i0 + 4*lo)*4 bytes, mp = m rounded up to 4.  It may
    // read up to 63 floats past the m valid entries of an XT row (rows of X past m in the last tile):
    // that lands in the next XT row, or in the scratch's tail padding for the last one; those rows of
    // the result are never stored.
    const unsigned char* xt_bytes = reinterpret_cast<const unsigned char*>(XT);
    const unsigned lane_x = (unsigned)(i0 + 4 * lo) * 4u;
    const __amdgpu_buffer_rsrc_t wrsrc =
        __builtin_amdgcn_make_buffer_rsrc(const_cast<float*>(data + (size_t)qb * 16), 0, (qe - qb) * 64, 0x00020000);
    const __amdgpu_buffer_rsrc_t irsrc =
        __builtin_amdgcn_make_buffer_rsrc(const_cast<int32_t*>(indices + qb), 0, (qe - qb) * 4, 0x00020000);
    unsigned char* wl = wstage[wave];

    for (int pb = qb; pb < qe; pb += 4 * U) {
        const int rel = pb - qb;                      // first block of the chunk inside the share
        const int idx = __builtin_amdgcn_raw_buffer_load_b32(irsrc, (rel + lane) * 4, 0, 0);   // 0 past the share
        u32x4 w4[WT];
#pragma unroll
        for (int t = 0; t < WT; ++t) w4[t] = __builtin_amdgcn_raw_buffer_load_b128(wrsrc, rel * 64 + t * 1024 + lane * 16, 0, 0);
        int col[U];
#pragma unroll
        for (int u = 0; u < U; ++u) col[u] = __builtin_amdgcn_ds_bpermute((4 * u + pp) * 4, idx);
        f32x4 xv[U];
#pragma unroll
        for (int u = 0; u < U; ++u)
            xv[u] = *reinterpret_cast<const f32x4*>(xt_bytes + ((unsigned)col[u] * row_bytes + lane_x));
        // the wavefront's own LDS area: its LDS operations complete in order, no barrier.  (Every lane
        // stores, to an address the compiler cannot tell from the one it reads next, so the reads stay
        // behind the stores without a compiler fence -- which would also pin the gathers above in place:
        // 15.7 instead of 13.3 us per product.)
#pragma unroll
        for (int t = 0; t < WT; ++t) *reinterpret_cast<u32x4*>(wl + t * 1024 + lane * 16) = w4[t];
        float wv[U];
#pragma unroll
        for (int u = 0; u < U; ++u) wv[u] = *reinterpret_cast<const float*>(wl + (4 * u + pp) * 64 + lo * 4);
        // groups past the share multiply zeros (blocks read as zero, block-column 0): no branch around
        // the MFMAs, so the accumulators stay where they are
#pragma unroll
        for (int u = 0; u < U; ++u)
#pragma unroll
            for (int s = 0; s < SUBS; ++s)
                acc[s] = __builtin_amdgcn_mfma_f32_16x16x4f32(xv[u][s], wv[u], acc[s], 0, 0, 0);
    }

#pragma unroll
    for (int s = 0; s < SUBS; ++s)
#pragma unroll
        for (int j = 0; j < 4; ++j) red[wave][16 * pp + 4 * j + s][lo] = acc[s][j];
    __syncthreads();

    // thread t: row t/4 of the tile, columns (t%4)*4 .. +3; 4 adjacent lanes write one row's 64 bytes
    const int row = threadIdx.x >> 2, c4 = (threadIdx.x & 3) * 4;
    f32x4 sum;
#pragma unroll
    for (int e = 0; e < 4; ++e) sum[e] = (red[0][row][c4 + e] + red[1][row][c4 + e]) + (red[2][row][c4 + e] + red[3][row][c4 + e]);
    if (i0 + row < m) *reinterpret_cast<f32x4*>(Y + (size_t)(i0 + row) * n + (size_t)r * 16 + c4) = sum;
}

}  // namespace

bool mfma_thin_supports(const bsr_matrix* W) { return W->bs_r == 16 && W->bs_c == 1 && W->dtype == BSR_F32 && W->R > 0; }

size_t mfma_thin_scratch_bytes(const bsr_matrix* W, int64_t m)
{
    // k rows of m floats, each padded to a multiple of 4, plus 256 bytes of tail padding (the last
    // tile's gathers may run past the last row)
    return mfma_thin_supports(W) ? (((size_t)((m + 3) & ~(int64_t)3) * (size_t)W->k * sizeof(float) + 256 + 255) & ~(size_t)255) : 0;
}

bsr_status launch_transpose_f32(const float* X, float* XT, int m, int k, hipStream_t stream)
{
    if (m <= 0 || k <= 0) return BSR_OK;
    hipLaunchKernelGGL(transpose_f32, dim3((k + 63) / 64, (m + 31) / 32), dim3(256), 0, stream, X, XT, m, k, (m + 3) & ~3);
    return hipGetLastError() == hipSuccess ? BSR_OK : BSR_ERR_HIP;
}

namespace {

// Transpose into `scratch` (at least mfma_thin_scratch_bytes() bytes, checked by the callers), then the product.
bsr_status launch_thin_with_scratch(const spmm_args& a, const tune_opts& tune, void* scratch)
{
    const bsr_matrix* W = a.W;
    const int m = (int)a.m, n = (int)W->n, k = (int)W->k, R = W->R;
    if ((a.m + 3) * W->k >= ((int64_t)1 << 30)) return BSR_ERR_SHAPE;      // byte offsets into XT are 32-bit
    float* XT = static_cast<float*>(scratch);
    hipLaunchKernelGGL(transpose_f32, dim3((k + 63) / 64, (m + 31) / 32), dim3(256), 0, a.stream,
                       (const float*)a.X, XT, m, k, (m + 3) & ~3);
    if (hipGetLastError() != hipSuccess) return BSR_ERR_HIP;
    auto go = [&](auto u_tag) -> bsr_status {
        constexpr int U = decltype(u_tag)::value;
        // m-tile groups over the XCDs: as many as there are m-tiles, up to 8 (a power of two)
        const int tiles = (m + 63) / 64;
        const int mg = tune.b > 0 ? tune.b : (tiles >= 8 ? 8 : (tiles >= 4 ? 4 : (tiles >= 2 ? 2 : 1)));
        const int64_t per_xcd = (int64_t)((tiles + mg - 1) / mg) * ((R + 8 / mg - 1) / (8 / mg));
        const int64_t blocks = 8 * per_xcd;
        if (blocks >= ((int64_t)1 << 31)) return BSR_ERR_SHAPE;
        hipLaunchKernelGGL((bsr_thin16_f32<U>), dim3((unsigned)blocks), dim3(256), 0, a.stream,
                           (const float*)XT, (const float*)W->data, W->indices, W->row_desc, (float*)a.Y, m, n, R, mg);
        return hipGetLastError() == hipSuccess ? BSR_OK : BSR_ERR_HIP;
    };
    // groups of 4 blocks per chunk: a quarter of the longest block-row in one chunk when that is at
    // most 16 groups (every chunk multiplies all its U groups, so U should not be much larger)
    int u = tune.a > 0 ? tune.a : ((W->max_row_blocks + 3) / 4 + 3) / 4;
    if (u <= 4) return go(std::integral_constant<int, 4>{});
    if (u <= 6) return go(std::integral_constant<int, 6>{});
    if (u <= 8) return go(std::integral_constant<int, 8>{});
    if (u <= 10) return go(std::integral_constant<int, 10>{});
    if (u <= 12) return go(std::integral_constant<int, 12>{});
    if (u <= 14) return go(std::integral_constant<int, 14>{});
    if (u <= 16) return go(std::integral_constant<int, 16>{});
    return go(std::integral_constant<int, 8>{});      // very long block-rows: several chunks of 32 blocks
}

}  // namespace

bsr_status launch_mfma_thin(const spmm_args& a, const tune_opts& tune)
{
    const bsr_matrix* W = a.W;
    if (!mfma_thin_supports(W) || a.y_dtype != BSR_F32) return BSR_ERR_UNSUPPORTED;
    // One launch with the rows of X staged in LDS when the plan allows it and the runs of a phase are short
    // enough to be loaded ahead (12 against 13.3 us on the 256 x 4096 x 4096 workload, and no scratch).  Else,
    // with enough scratch lent: the transposed copy of X, then the gather kernel (two launches).  variant 1 / 2
    // ask for the one or the other.
    const bool lent = W->scratch && W->scratch_bytes >= mfma_thin_scratch_bytes(W, a.m);
    const bool rows_ok = mfma_thinrow_supports(W);
    const bool rows_fit = rows_ok && W->nnzb <= (int64_t)80 * W->R * W->thin_nph;   // average run of a phase: at most 80 blocks
    if (tune.variant == 2 || (tune.variant != 1 && rows_ok && (rows_fit || !lent)))
        return rows_ok ? launch_mfma_thinrow(a, tune) : BSR_ERR_UNSUPPORTED;
    if (!lent) return BSR_ERR_WORKSPACE;
    return launch_thin_with_scratch(a, tune, W->scratch);
}

// ---- the library's own scratch, for callers that cannot allocate any (bsr_spmm_static) ----
//
// `scratch` is a device array that lives in this library's code object: every GPU the library is
// loaded on holds its own copy, at its own address, until the process ends.  In host code the
// name is only a handle for hipGetSymbolAddress(); the address it returns for the current device
// is what the kernels get.
namespace {

static __device__ __align__(256) unsigned char scratch[BSR_STATIC_SCRATCH_BYTES];

constexpr int kMaxDevices = 64;
std::mutex static_scratch_mu;
void* static_scratch_ptr[kMaxDevices] = {};          // per device, resolved once

}  // namespace

bsr_status mfma_thin_static_scratch(void** out)
{
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return BSR_ERR_HIP;
    std::lock_guard<std::mutex> lock(static_scratch_mu);
    if (!static_scratch_ptr[dev]) {
        void* ptr = nullptr;
        if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess || !ptr) {
            (void)hipGetLastError();
            return BSR_ERR_HIP;
        }
        static_scratch_ptr[dev] = ptr;
    }
    if (out) *out = static_scratch_ptr[dev];
    return BSR_OK;
}

bsr_status launch_mfma_thin_static(const spmm_args& a, const tune_opts& tune)
{
    const bsr_matrix* W = a.W;
    if (!mfma_thin_supports(W) || a.y_dtype != BSR_F32) return BSR_ERR_UNSUPPORTED;
    if (mfma_thin_scratch_bytes(W, a.m) > (size_t)BSR_STATIC_SCRATCH_BYTES) return BSR_ERR_SCRATCH_LIMIT;
    void* ptr = nullptr;
    const bsr_status st = mfma_thin_static_scratch(&ptr);
    if (st != BSR_OK) return st;
    // nothing in the array has to start at zero: the transpose writes every entry of XT the product
    // reads for rows below m, and what the last tile's gathers read beyond them is never stored
    return launch_thin_with_scratch(a, tune, ptr);
}

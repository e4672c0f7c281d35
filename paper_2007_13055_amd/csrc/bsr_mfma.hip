// Matrix-core (MFMA) kernels for Y = X * W^T, W in BSR, gfx950.
//
// Work unit: a wavefront owns a tile of Y that is one block-row of W wide (bs_r columns) and
// MT*MM rows of X tall, and walks the stored blocks of that block-row (Background: index_pointer
// gives the range, block_indices the block-column of each stored block).  This is the
// tile-per-thread-block design of the paper's "Utilizing shared memory" section, which the
// paper could not build because its compiler needed the cached extents at compile time; here
// the indices are read at run time and only the X columns of stored blocks are fetched.
//
// MFMA operand roles: the W block supplies the rows of the MFMA result (index a, the n side),
// the X tile supplies its columns (index i, the m side), so one lane ends up holding 4
// consecutive columns of Y for one row i, which are stored as one vector.  Both operands are
// read straight from their row-major storage: in both, the reduction index c is the contiguous
// one, so a lane's operand is a contiguous run of CH elements of a block row / an X row.  The
// lane groups split the bs_c columns of a block into 64/MM contiguous runs; W and X use the same
// split, so the sum over c is complete whatever order the instruction takes its k in.
#include "bsr_mfma_common.h"

using namespace bsr_dev;

namespace {

// Direct kernel: operands go from global memory (L1/L2) straight into registers.
//   MM   MFMA tile edge: 32 when bs_r >= 32, else 16          NA = BS_R / MM   result tiles along n
//   MT   result tiles along m per wavefront                    CH = BS_C / (64/MM) contiguous run per lane
// grid: blockIdx.x = slot + R * (m-tile); slot s works on block-row row_order[s] (longest first).
// No LDS and no barrier: wavefronts whose rows lie beyond m leave at once.
template <typename T, typename O, int BS_R, int BS_C, int MT>
__global__ __launch_bounds__(256) void bsr_mfma_direct(const T* __restrict__ X, const T* __restrict__ data,
                                                       const int32_t* __restrict__ indices,
                                                       const int32_t* __restrict__ indptr,
                                                       const int32_t* __restrict__ row_order, O* __restrict__ Y,
                                                       int m, int k, int n, int R)
{
    constexpr int MM = BS_R >= 32 ? 32 : 16;
    constexpr int NA = BS_R / MM;
    constexpr int G = 64 / MM;
    constexpr int CH = BS_C / G;
    typedef typename AccT<MM>::type acc_t;

    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, waves = blockDim.x >> 6;
    const int li = lane % MM, h = lane / MM;
    const int slot = (int)(blockIdx.x % (unsigned)R);
    const int tile = (int)(blockIdx.x / (unsigned)R);
    const int i_base = (tile * waves + wave) * (MT * MM);
    if (i_base >= m) return;
    const int r = row_order[slot];
    const int p0 = indptr[r], p1 = indptr[r + 1];

    acc_t acc[NA][MT];
#pragma unroll
    for (int u = 0; u < NA; ++u)
#pragma unroll
        for (int t = 0; t < MT; ++t)
#pragma unroll
            for (int e = 0; e < (MM == 32 ? 16 : 4); ++e) acc[u][t][e] = 0.f;

    // per-lane bases: X rows (clamped to m-1; the surplus rows are never stored) and the lane's run
    const T* xbase[MT];
#pragma unroll
    for (int t = 0; t < MT; ++t)
        xbase[t] = X + (size_t)min(i_base + t * MM + li, m - 1) * (size_t)k + h * CH;
    const T* wbase = data + (size_t)li * BS_C + h * CH;

    Frag<T, CH> wf[2][NA], xf[2][MT];
    auto fetch = [&](int buf, int p) {
        const int c = indices[p];
        const T* wp = wbase + (size_t)p * (BS_R * BS_C);
#pragma unroll
        for (int u = 0; u < NA; ++u) wf[buf][u].load(wp + u * (MM * BS_C));
#pragma unroll
        for (int t = 0; t < MT; ++t) xf[buf][t].load(xbase[t] + (size_t)c * BS_C);
    };
    auto compute = [&](int buf) {
#pragma unroll
        for (int u = 0; u < NA; ++u)
#pragma unroll
            for (int t = 0; t < MT; ++t) mfma_frag<T, MM, CH>(acc[u][t], wf[buf][u], xf[buf][t]);
    };

    // two-stage software pipeline over the stored blocks of the block-row
    int p = p0;
    if (p < p1) fetch(0, p);
    while (p < p1) {
        if (p + 1 < p1) fetch(1, p + 1);
        compute(0);
        ++p;
        if (p >= p1) break;
        if (p + 1 < p1) fetch(0, p + 1);
        compute(1);
        ++p;
    }

    // store: lane holds, for row i, columns r*BS_R + u*MM + (MM==32 ? 8*g + 4*h : 4*h) + 0..3
    O* yrow_base = Y + (size_t)r * BS_R;
#pragma unroll
    for (int t = 0; t < MT; ++t) {
        const int i = i_base + t * MM + li;
        if (i < m) {
            O* yrow = yrow_base + (size_t)i * (size_t)n;
#pragma unroll
            for (int u = 0; u < NA; ++u) {
                if constexpr (MM == 32) {
#pragma unroll
                    for (int g = 0; g < 4; ++g)
                        store4<O>(yrow + u * 32 + 8 * g + 4 * h, acc[u][t][4 * g], acc[u][t][4 * g + 1],
                                  acc[u][t][4 * g + 2], acc[u][t][4 * g + 3]);
                } else {
                    store4<O>(yrow + u * 16 + 4 * h, acc[u][t][0], acc[u][t][1], acc[u][t][2], acc[u][t][3]);
                }
            }
        }
    }
}

template <typename T, typename O, int BS_R, int BS_C>
bsr_status launch_direct_shape(const spmm_args& a, const tune_opts& tune)
{
    const bsr_matrix* W = a.W;
    const int m = (int)a.m, n = (int)W->n, k = (int)W->k, R = W->R;
    constexpr int MM = BS_R >= 32 ? 32 : 16;
    auto go = [&](auto mt_tag, int waves) -> bsr_status {
        constexpr int MT = decltype(mt_tag)::value;
        const int rows_per_wg = waves * MT * MM;
        const int64_t tiles = (m + rows_per_wg - 1) / rows_per_wg;
        const int64_t blocks = tiles * R;
        if (blocks >= ((int64_t)1 << 31) || blocks * 64 * waves >= ((int64_t)1 << 32)) return BSR_ERR_SHAPE;
        hipLaunchKernelGGL((bsr_mfma_direct<T, O, BS_R, BS_C, MT>), dim3((unsigned)blocks), dim3(64 * waves), 0,
                           a.stream, (const T*)a.X, (const T*)W->data, W->indices, W->indptr, W->row_order,
                           (O*)a.Y, m, k, n, R);
        return hipGetLastError() == hipSuccess ? BSR_OK : BSR_ERR_HIP;
    };
    // Tile height: enough workgroups to fill 256 CUs several times over when m allows it, taller
    // wavefront tiles (more reuse of each W block) when m is large.
    const int sub = (m + MM - 1) / MM;                 // MFMA tiles along m
    int mt = sub >= 64 ? 2 : 1, waves = sub >= 8 ? 4 : 1;
    if (tune.mt == 1 || tune.mt == 2) mt = tune.mt;
    if (tune.nw >= 1 && tune.nw <= 4) waves = tune.nw;
    if (mt == 2) return go(std::integral_constant<int, 2>{}, waves);
    return go(std::integral_constant<int, 1>{}, waves);
}

}  // namespace

bsr_status launch_mfma_direct(const spmm_args& a, const tune_opts& t)
{
    BSR_MFMA_DISPATCH(launch_direct_shape, a.W, a.y_dtype, a, t);
    return BSR_ERR_UNSUPPORTED;
}

bool mfma_supports(const bsr_matrix* W)
{
    const int br = W->bs_r, bc = W->bs_c;
    const bool r_ok = br == 16 || br == 32 || br == 64;
    const bool c_ok = bc == 16 || bc == 32 || bc == 64;
    return r_ok && c_ok && W->R > 0;
}

// Which matrix-core kernel serves this product.
//   ksplit  fewer than about 6000 (m-tile, block-row) items: the stored blocks of a block-row are spread over the
//           wavefronts of a workgroup, otherwise most of the chip would idle
//   tile    many rows of X and blocks at least 32 rows tall: 128 x bs_r tiles of Y, the W block and
//           the X tile staged in LDS with coalesced reads, XCD-aware launch order
//   stripe  16x16 blocks of a 16-bit type, many rows of X, and 64 full rows of X fit in LDS: the
//           stripe is copied to LDS once and many block-rows are multiplied against it
//   direct  everything else: block-rows of a block or two, where writing Y is most of the work
//           (operands straight from global memory)
bsr_status launch_mfma(const spmm_args& a, const tune_opts& tune)
{
    tune_opts t = tune;
    int variant = t.variant;
    if (variant == 0) {
        // thresholds from timed trials over many sizes (bsr_tune's candidates) on MI355X
        const int MM = a.W->bs_r >= 32 ? 32 : 16;
        const int64_t sub = (a.m + MM - 1) / MM;
        if (sub * a.W->R < 6000 && a.W->mean_row_blocks > 1.5) variant = 2;
        else if (a.W->bs_r >= 32 && a.m >= 512) variant = 3;
        else if (a.m >= 256 && mfma_stripe_supports(a.W, 16)) variant = 4;
        else if (a.W->mean_row_blocks > 4.0) variant = 2;     // 16-row blocks the tile kernel does not take
        else variant = 1;
        // 64x64 16-bit blocks with a few block-rows that hold much of W: those rows in row groups (their X
        // tiles shared through LDS), the rest through the tile kernel (112 against 135 us on the 8192^3
        // power-law workload, 403 instead of 825 MB fetched)
        if (variant == 3 && t.mt == 0 && a.m >= 1024 && mfma_group_supports(a.W) && a.W->grp_blocks * 5 >= a.W->nnzb * 2)
            variant = 5;
        if (variant == 3 && t.mt == 0) {
            // fp32 blocks: 256-row tiles with one block in flight once m is large (the W block is
            // staged half as often); otherwise 128-row tiles with two blocks in flight
            const bool tall = a.W->dtype == BSR_F32 && a.m >= 2048;
            t.mt = tall ? 2 : 1;
            if (t.a == 0) t.a = tall ? 1 : 2;
        }
    }
    if (variant == 5) {
        // the grouped (longest) block-rows in one launch, the other slots through the tile kernel
        if (!mfma_group_supports(a.W)) return launch_mfma_tile(a, t);   // no block-row long enough
        const bsr_status st = launch_mfma_group(a, t);
        if (st == BSR_ERR_UNSUPPORTED) return launch_mfma_tile(a, t);   // sizes beyond its 32-bit offsets: nothing was launched
        if (st != BSR_OK) return st;
        spmm_args rest = a;
        rest.first_slot = a.W->grp_slots;
        tune_opts tt = t;
        tt.variant = 3;
        tt.b = 0;
        tt.nw = 0;
        if (tt.mt == 0) tt.mt = 1;
        if (tt.a == 0) {
            // blocks in flight per workgroup: two pay only when the rows that are left still have a few blocks each
            // (the 8192^3 power-law workload, 2.2 per row: 111.4 us with one against 112.7 with two)
            const int64_t rows_left = a.W->R - a.W->grp_slots, blocks_left = a.W->nnzb - a.W->grp_blocks;
            tt.a = blocks_left >= 4 * rows_left ? 2 : 1;
        }
        return launch_mfma_tile(rest, tt);
    }
    if (variant == 2) return launch_mfma_ksplit(a, t);
    if (variant == 3) return launch_mfma_tile(a, t);
    if (variant == 4) return launch_mfma_stripe(a, t);
    return launch_mfma_direct(a, t);
}

// Matrix-core kernel for products with few rows of X (few MFMA tiles along m).
//
// One workgroup owns an (MM rows of X) x (one block-row of W) tile of Y.  Its wavefronts share
// out the stored blocks of the block-row -- wavefront w takes blocks p0+w, p0+w+NW, ... -- so a
// block-row's reduction runs NW-wide instead of serially; each wavefront keeps a full-tile fp32
// partial sum, and the partial sums are added through LDS in a fixed order (wavefront 0, 1, ...),
// which keeps the result deterministic.  This is the paper's concurrent reduction (Section 4.4:
// several threads share one output's reduction, partial results aggregated at the end) moved from
// single output elements to MFMA tiles.
#include "bsr_mfma_common.h"

using namespace bsr_dev;

namespace {

template <typename T, typename O, int BS_R, int BS_C>
__global__ __launch_bounds__(512) void bsr_mfma_ksplit(const T* __restrict__ X, const T* __restrict__ data,
                                                       const int32_t* __restrict__ indices,
                                                       const int32_t* __restrict__ row_desc, O* __restrict__ Y,
                                                       int m, int k, int n, int R, int per, int items)
{
    constexpr int MM = BS_R >= 32 ? 32 : 16;
    constexpr int NA = BS_R / MM;
    constexpr int G = 64 / MM;
    constexpr int CH = BS_C / G;
    constexpr int NE = MM == 32 ? 16 : 4;             // accumulator values per lane and tile
    constexpr int LD = BS_R + 4;                      // padded row of the LDS partial-sum tile
    typedef typename AccT<MM>::type acc_t;
    extern __shared__ float red[];                    // [NW][MM][LD]

    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int nw_max = blockDim.x >> 6;
    const int li = lane % MM, h = lane / MM;
    // one read of the workgroup's descriptor: block-row, first stored block, count, m-tile, first
    // block-columns.  With a work-item table (items != 0) workgroup b takes entry b -- the table is
    // laid out so that the workgroups sharing a CU carry about equal work -- and an entry with
    // block-row -1 is a filler; without one, workgroup b takes slot b mod R of m-tile b div R.
    const int32_t* __restrict__ desc =
        row_desc + (size_t)(items ? blockIdx.x : blockIdx.x % (unsigned)R) * kRowDescWords;
    const int r = desc[0];
    if (r < 0) return;                                // whole workgroup leaves together
    const int i_base = (items ? desc[3] : (int)(blockIdx.x / (unsigned)R)) * MM;
    const int p0 = desc[1], p1 = p0 + desc[2];
    // wavefronts that take part: about `per` stored blocks each, at most all of the workgroup's;
    // the others go straight to the barrier, so short block-rows cost no loads in idle wavefronts
    const int nw = max(1, min(nw_max, (p1 - p0 + per - 1) / per));

    acc_t acc[NA];
#pragma unroll
    for (int u = 0; u < NA; ++u)
#pragma unroll
        for (int e = 0; e < NE; ++e) acc[u][e] = 0.f;

    const T* xbase = X + (size_t)min(i_base + li, m - 1) * (size_t)k + h * CH;
    const T* wbase = data + (size_t)li * BS_C + h * CH;

    Frag<T, CH> wf[2][NA], xf[2];
    auto fetch = [&](int buf, int p) {
        const int j = p - p0;
        const int c = j < kRowDescCols ? desc[kRowDescColsAt + j] : indices[p];
        const T* wp = wbase + (size_t)p * (BS_R * BS_C);
#pragma unroll
        for (int u = 0; u < NA; ++u) wf[buf][u].load(wp + u * (MM * BS_C));
        xf[buf].load(xbase + (size_t)c * BS_C);
    };
    auto compute = [&](int buf) {
#pragma unroll
        for (int u = 0; u < NA; ++u) mfma_frag<T, MM, CH>(acc[u], wf[buf][u], xf[buf]);
    };

    int p = wave < nw ? p0 + wave : p1;
    if (p < p1) fetch(0, p);
    while (p < p1) {
        if (p + nw < p1) fetch(1, p + nw);
        compute(0);
        p += nw;
        if (p >= p1) break;
        if (p + nw < p1) fetch(0, p + nw);
        compute(1);
        p += nw;
    }
    // partial sums of the wavefronts that had at least one block -> LDS
    const int used = min(nw, p1 - p0);
    if (wave < used) {
        float* mine = red + ((size_t)wave * MM + li) * LD;
#pragma unroll
        for (int u = 0; u < NA; ++u) {
            if constexpr (MM == 32) {
#pragma unroll
                for (int g = 0; g < 4; ++g) {
                    const f32x4 v = {acc[u][4 * g], acc[u][4 * g + 1], acc[u][4 * g + 2], acc[u][4 * g + 3]};
                    *reinterpret_cast<f32x4*>(mine + u * 32 + 8 * g + 4 * h) = v;
                }
            } else {
                const f32x4 v = {acc[u][0], acc[u][1], acc[u][2], acc[u][3]};
                *reinterpret_cast<f32x4*>(mine + u * 16 + 4 * h) = v;
            }
        }
    }
    __syncthreads();

    // fixed-order sum over the partial tiles; each thread owns 4 consecutive columns of one row
    constexpr int QUADS = BS_R / 4;
    for (int t = threadIdx.x; t < MM * QUADS; t += blockDim.x) {
        const int i = t / QUADS, q = t - i * QUADS;
        f32x4 s = {0.f, 0.f, 0.f, 0.f};
        for (int w = 0; w < used; ++w) s += *reinterpret_cast<const f32x4*>(red + ((size_t)w * MM + i) * LD + 4 * q);
        if (i_base + i < m)
            store4<O>(Y + (size_t)(i_base + i) * (size_t)n + (size_t)r * BS_R + 4 * q, s.x, s.y, s.z, s.w);
    }
}

template <typename T, typename O, int BS_R, int BS_C>
bsr_status launch_ksplit_shape(const spmm_args& a, const tune_opts& tune)
{
    const bsr_matrix* W = a.W;
    const int m = (int)a.m, n = (int)W->n, k = (int)W->k, R = W->R;
    constexpr int MM = BS_R >= 32 ? 32 : 16;
    // wavefronts per workgroup: about one stored block each for the average block-row, 1..8
    // blocks per wavefront `per`, and as many wavefronts as the longest block-row then needs (1..8)
    int per = tune.a > 0 ? tune.a : 2;
    int nw = (W->max_row_blocks + per - 1) / per;
    nw = nw < 1 ? 1 : (nw > 8 ? 8 : nw);
    if (tune.nw >= 1 && tune.nw <= 8) nw = tune.nw;
    const int64_t tiles = (m + MM - 1) / MM;
    int64_t blocks = tiles * R;
    if (blocks >= ((int64_t)1 << 31) || blocks * 64 * nw >= ((int64_t)1 << 32)) return BSR_ERR_SHAPE;
    // CU-balanced work-item table when there are more items than CUs (else every item has a CU to itself)
    const int32_t* table = W->row_desc;
    int items = 0;
    if (tune.b != 1 && blocks > 256 && blocks <= kMaxKsplitItems) {
        const int grid = ksplit_items(W, (int)tiles, a.stream);
        if (grid > 0) { table = W->item_desc; items = 1; blocks = grid; }
    }
    const size_t lds = (size_t)nw * MM * (BS_R + 4) * sizeof(float);
    hipLaunchKernelGGL((bsr_mfma_ksplit<T, O, BS_R, BS_C>), dim3((unsigned)blocks), dim3(64 * nw), lds, a.stream,
                       (const T*)a.X, (const T*)W->data, W->indices, table, (O*)a.Y, m, k, n, R, per, items);
    return hipGetLastError() == hipSuccess ? BSR_OK : BSR_ERR_HIP;
}

}  // namespace

bsr_status launch_mfma_ksplit(const spmm_args& a, const tune_opts& t)
{
    BSR_MFMA_DISPATCH(launch_ksplit_shape, a.W, a.y_dtype, a, t);
    return BSR_ERR_UNSUPPORTED;
}

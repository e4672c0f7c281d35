// Matrix-core kernel for 16x16 blocks of a 16-bit type when a stripe of X fits in LDS.
//
// With blocks this small a stored block touches only 32 bytes of each X row, so fetching X tiles
// block by block would use a quarter of every cache line.  Instead a workgroup copies a whole
// stripe of X -- TM full rows, one contiguous piece of memory -- into LDS once, and then walks
// many block-rows of W against it: "cache the part of X that all outputs of the tile need"
// (the paper's "Utilizing shared memory" section) with the tile made TM rows x many block-rows.
//
// Work split: the grid is (m-tiles) x (groups of consecutive block-rows); inside a workgroup
// every wavefront owns 4 consecutive block-rows (64 columns of Y = one 128-byte line of bf16 per
// row) for all TM rows.  Two stored blocks of a block-row are multiplied per MFMA: the 16x16x32
// instruction takes k = 32, lanes 0-31 supply block p and lanes 32-63 block p+1 (an odd last
// block is paired with zeros).  W blocks stream from global memory into registers, a block-row
// ahead of the arithmetic; X operands come from the LDS stripe at the column block_indices names.
#include "bsr_mfma_common.h"

using namespace bsr_dev;

namespace {

constexpr int kXcds = 8;
constexpr int kRowsPerWave = 4;      // block-rows per wavefront: 4 x 16 columns = 64 outputs per row of Y
constexpr int kPairs = 8;            // pairs of blocks held in registers per block-row chunk

template <typename T, typename O, int TM>
__global__ __launch_bounds__(768) void bsr_mfma_stripe16(const T* __restrict__ X, const T* __restrict__ data,
                                                          const int32_t* __restrict__ indices,
                                                          const int32_t* __restrict__ indptr, O* __restrict__ Y,
                                                          int m, int k, int n, int R, int n_tiles, int n_groups,
                                                          int rows_per_group, unsigned cpr_magic, int nnzb)
{
    constexpr int SUB = TM / 16;                      // 16-row MFMA tiles along m
    extern __shared__ __attribute__((aligned(16))) unsigned char lds[];   // [TM][k*2 + 16]
    const int RB = k * (int)sizeof(T), RS = RB + 16;  // row bytes, padded LDS stride (rows shift by 4 banks)

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int li = lane & 15, h = lane >> 4;          // MFMA row/column index, k-group 0..3
    const int half = h >> 1;                          // which block of the pair this lane feeds

    // workgroup -> (m-tile, block-row group); the groups of one m-tile share an XCD (and its L2 copy
    // of the stripe)
    const int xcd = (int)(blockIdx.x % kXcds), local = (int)(blockIdx.x / kXcds);
    const int tile = (local / n_groups) * kXcds + xcd, group = local % n_groups;
    if (tile >= n_tiles) return;                      // whole workgroup leaves together
    const int i_base = tile * TM;

    const int r_first = group * rows_per_group + wave * kRowsPerWave;
    const int r_end = min(min((group + 1) * rows_per_group, R), r_first + kRowsPerWave);

    // lane's part of a pair: block p+half, row li of the block, 8 columns starting at (h&1)*8
    const unsigned char* wlane = reinterpret_cast<const unsigned char*>(data) + half * 512 + li * 32 + (h & 1) * 16;
    const int32_t* ilane = indices + half;
    const unsigned char* xlane = lds + (size_t)li * RS + (h & 1) * 16;

    // stored-block ranges of this wavefront's block-rows (rows past r_end get an empty range)
    int pb0[kRowsPerWave], pb1[kRowsPerWave];
#pragma unroll
    for (int j = 0; j < kRowsPerWave; ++j) {
        const int r = min(r_first + j, R - 1);
        pb0[j] = indptr[r];
        pb1[j] = r_first + j < r_end ? indptr[r + 1] : pb0[j];
    }

    // A chunk = up to kPairs pairs of blocks of one block-row: W operands and block-columns, all
    // loads independent of each other.  Two chunk buffers: the next block-row's chunk is loaded
    // while the current one is multiplied.
    u32x4 wreg[2][kPairs];
    int col[2][kPairs];
    auto load_chunk = [&](int buf, int pb, int p1) {
        if (pb >= p1) return;                         // uniform: empty block-row or past its end
        if (pb + 2 * kPairs <= nnzb) {
            // every block index of the chunk exists (blocks past p1 belong to later block-rows and
            // are discarded below): plain base + q*1024 addressing, no per-lane clamping
            const unsigned char* wb = wlane + (size_t)pb * 512;
            const int32_t* ib = ilane + pb;
#pragma unroll
            for (int q = 0; q < kPairs; ++q) {
                wreg[buf][q] = *reinterpret_cast<const u32x4*>(wb + q * 1024);
                col[buf][q] = ib[2 * q];
            }
        } else {                                      // the last blocks of W: clamp each lane's block index
#pragma unroll
            for (int q = 0; q < kPairs; ++q) {
                const int pc = min(pb + 2 * q + half, p1 - 1) - half;
                wreg[buf][q] = *reinterpret_cast<const u32x4*>(wlane + (size_t)pc * 512);
                col[buf][q] = ilane[pc];
            }
        }
#pragma unroll
        for (int q = 0; q < kPairs; ++q)              // odd tail / past the end of the block-row: zeros
            if (pb + 2 * q + 2 > p1 && pb + 2 * q + half >= p1) { wreg[buf][q] = u32x4{0u, 0u, 0u, 0u}; col[buf][q] = 0; }
    };

    load_chunk(0, pb0[0], pb1[0]);                    // in flight while the stripe is staged

    // ---- stage the stripe: TM rows x k columns, one contiguous piece of memory ----
    // chunk q (16 bytes) of the stripe lies in row q / cpr; the quotient comes from a multiply with
    // cpr_magic = floor(2^32 / cpr) + 1, exact for q < 2^16 (the stripe has at most 10240 chunks)
    {
        const int cpr = RB / 16;                      // 16-byte chunks per row
        const int total = TM * cpr;
        const unsigned char* xb = reinterpret_cast<const unsigned char*>(X) + (size_t)i_base * (size_t)RB;
        if (i_base + TM <= m) {                       // whole tile inside X (uniform)
            for (int q = tid; q < total; q += blockDim.x) {
                const int row = (int)__umulhi((unsigned)q, cpr_magic);
                *reinterpret_cast<u32x4*>(lds + (size_t)(q + row) * 16) = *reinterpret_cast<const u32x4*>(xb + (size_t)q * 16);
            }
        } else {                                      // last tile: rows past m repeat row m-1, never stored
            for (int q = tid; q < total; q += blockDim.x) {
                const int row = (int)__umulhi((unsigned)q, cpr_magic), cc = q - row * cpr;
                const size_t src = (size_t)min(row, m - 1 - i_base) * (size_t)RB + (size_t)cc * 16;
                *reinterpret_cast<u32x4*>(lds + (size_t)(q + row) * 16) = *reinterpret_cast<const u32x4*>(xb + src);
            }
        }
    }
    __syncthreads();
    if (r_first >= r_end) return;                     // no barrier after this point

    f32x4 acc[kRowsPerWave][SUB];
#pragma unroll
    for (int j = 0; j < kRowsPerWave; ++j)
#pragma unroll
        for (int s = 0; s < SUB; ++s) acc[j][s] = f32x4{0.f, 0.f, 0.f, 0.f};

    const unsigned char* xsub[SUB];                   // the lane's row of each 16-row tile of the stripe
#pragma unroll
    for (int s = 0; s < SUB; ++s) xsub[s] = xlane + (size_t)s * 16 * RS;
    auto compute_chunk = [&](int buf, int j, int pb, int p1) {
#pragma unroll
        for (int q = 0; q < kPairs; ++q) {
            if (pb + 2 * q < p1) {                    // uniform
                Frag<T, 8> wf, xf;
                wf.w[0] = wreg[buf][q].x; wf.w[1] = wreg[buf][q].y; wf.w[2] = wreg[buf][q].z; wf.w[3] = wreg[buf][q].w;
#pragma unroll
                for (int s = 0; s < SUB; ++s) {
                    xf.load(reinterpret_cast<const T*>(xsub[s] + col[buf][q] * 32));
                    mfma_frag<T, 16, 8>(acc[j][s], wf, xf);
                }
            }
        }
    };

#pragma unroll
    for (int j = 0; j < kRowsPerWave; ++j) {
        if (j + 1 < kRowsPerWave) load_chunk((j + 1) & 1, pb0[j + 1], pb1[j + 1]);
        compute_chunk(j & 1, j, pb0[j], pb1[j]);
        for (int pb = pb0[j] + 2 * kPairs; pb < pb1[j]; pb += 2 * kPairs) {   // block-rows longer than one chunk
            load_chunk(j & 1, pb, pb1[j]);
            compute_chunk(j & 1, j, pb, pb1[j]);
        }
    }

    // Epilogue.  A lane holds, for row i = s*16 + li, columns (r_first + j)*16 + 4h .. +3: neighbouring
    // lanes are neighbouring ROWS of Y, so direct stores would be 64 separate small writes per
    // instruction.  Each wavefront therefore passes its 64-column result through a private LDS
    // scratch (behind the stripe), SPP 16-row tiles at a time, and stores whole rows: OC consecutive
    // lanes write one row's 64 outputs as 16-byte pieces.
    constexpr int OB = kRowsPerWave * 16 * (int)sizeof(O);   // bytes of one output row of the wavefront's tile
    constexpr int OS = OB + 16, OC = OB / 16;                // padded LDS stride, 16-byte pieces per row
    constexpr int SPP = sizeof(O) == 2 ? (SUB >= 2 ? 2 : 1) : 1;   // 16-row tiles per pass (scratch <= 4.6 KB)
    constexpr int RPI = 64 / OC;                             // rows one store instruction covers
    unsigned char* scratch = lds + (size_t)TM * RS + (size_t)wave * (SPP * 16 * OS);
    unsigned char* ybytes = reinterpret_cast<unsigned char*>(Y + (size_t)r_first * 16);
    const int orow = lane / OC, opiece = lane - orow * OC;
    const int valid_bytes = (r_end - r_first) * 16 * (int)sizeof(O);   // the group's last wavefront may own < 4 block-rows
#pragma unroll
    for (int s0 = 0; s0 < SUB; s0 += SPP) {
#pragma unroll
        for (int ss = 0; ss < SPP; ++ss)
#pragma unroll
            for (int j = 0; j < kRowsPerWave; ++j)
                store4<O>(reinterpret_cast<O*>(scratch + (size_t)(ss * 16 + li) * OS) + j * 16 + 4 * h,
                          acc[j][s0 + ss][0], acc[j][s0 + ss][1], acc[j][s0 + ss][2], acc[j][s0 + ss][3]);
        // same wavefront wrote and now reads: its LDS operations complete in order, no barrier needed
#pragma unroll
        for (int pass = 0; pass < SPP * 16 / RPI; ++pass) {
            const int row = pass * RPI + orow;
            const u32x4 v = *reinterpret_cast<const u32x4*>(scratch + (size_t)row * OS + opiece * 16);
            const int i = i_base + s0 * 16 + row;
            if (i < m && opiece * 16 < valid_bytes)
                *reinterpret_cast<u32x4*>(ybytes + (size_t)i * (size_t)n * sizeof(O) + opiece * 16) = v;
        }
    }
}

template <typename T, typename O>
bsr_status launch_stripe_types(const spmm_args& a, const tune_opts& tune)
{
    const bsr_matrix* W = a.W;
    const int m = (int)a.m, n = (int)W->n, k = (int)W->k, R = W->R;
    auto go = [&](auto tm_tag) -> bsr_status {
        constexpr int TM = decltype(tm_tag)::value;
        const size_t lds_stripe = (size_t)TM * ((size_t)k * sizeof(T) + 16);
        constexpr int SPP = sizeof(O) == 2 ? (TM >= 32 ? 2 : 1) : 1;
        const size_t scratch_per_wave = (size_t)SPP * 16 * (kRowsPerWave * 16 * sizeof(O) + 16);
        const int n_tiles = (m + TM - 1) / TM;
        // groups of block-rows: enough workgroups for every CU, at most 12 wavefronts (48 block-rows) each
        int n_groups = tune.a > 0 ? tune.a : (256 + n_tiles - 1) / n_tiles;
        const int min_groups = (R + 12 * kRowsPerWave - 1) / (12 * kRowsPerWave);
        if (n_groups < min_groups) n_groups = min_groups;
        if (n_groups > (R + kRowsPerWave - 1) / kRowsPerWave) n_groups = (R + kRowsPerWave - 1) / kRowsPerWave;
        int rows_per_group = (R + n_groups - 1) / n_groups;
        rows_per_group = (rows_per_group + kRowsPerWave - 1) / kRowsPerWave * kRowsPerWave;
        n_groups = (R + rows_per_group - 1) / rows_per_group;
        const int waves = rows_per_group / kRowsPerWave;
        const size_t lds = lds_stripe + (size_t)waves * scratch_per_wave;
        if (lds > 160 * 1024) return BSR_ERR_UNSUPPORTED;
        const int64_t blocks = (int64_t)((n_tiles + kXcds - 1) / kXcds) * kXcds * n_groups;
        if (blocks >= ((int64_t)1 << 31)) return BSR_ERR_SHAPE;
        static const hipError_t attr =
            hipFuncSetAttribute(reinterpret_cast<const void*>(&bsr_mfma_stripe16<T, O, TM>),
                                hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
        if (attr != hipSuccess) return BSR_ERR_HIP;
        hipLaunchKernelGGL((bsr_mfma_stripe16<T, O, TM>), dim3((unsigned)blocks), dim3(64 * waves), lds, a.stream,
                           (const T*)a.X, (const T*)W->data, W->indices, W->indptr, (O*)a.Y, m, k, n, R, n_tiles,
                           n_groups, rows_per_group, (unsigned)(0x100000000ull / (unsigned)(k * sizeof(T) / 16)) + 1u, (int)W->nnzb);
        return hipGetLastError() == hipSuccess ? BSR_OK : BSR_ERR_HIP;
    };
    const int tm = tune.mt > 0 ? tune.mt * 16 : 64;
    if (tm == 16) return go(std::integral_constant<int, 16>{});
    if (tm == 32) return go(std::integral_constant<int, 32>{});
    return go(std::integral_constant<int, 64>{});
}

}  // namespace

bool mfma_stripe_supports(const bsr_matrix* W, int tm)
{
    if (W->bs_r != 16 || W->bs_c != 16 || W->dtype == BSR_F32) return false;
    return (size_t)tm * ((size_t)W->k * 2 + 16) + 12 * 16 * (kRowsPerWave * 16 * 4 + 16) <= 160 * 1024;
}

bsr_status launch_mfma_stripe(const spmm_args& a, const tune_opts& t)
{
    const bsr_matrix* W = a.W;
    if (W->bs_r != 16 || W->bs_c != 16) return BSR_ERR_UNSUPPORTED;
    if (W->dtype == BSR_F16) return a.y_dtype == BSR_F32 ? launch_stripe_types<_Float16, float>(a, t)
                                                         : launch_stripe_types<_Float16, _Float16>(a, t);
    if (W->dtype == BSR_BF16) return a.y_dtype == BSR_F32 ? launch_stripe_types<__bf16, float>(a, t)
                                                          : launch_stripe_types<__bf16, __bf16>(a, t);
    return BSR_ERR_UNSUPPORTED;
}

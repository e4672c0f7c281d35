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
// instruction takes k = 32, lanes 0-31 supply block p and lanes 32-63 block p+1.
//
// The arithmetic has no data-dependent branches.  The plan's pair table lists every block-row as
// whole CHUNKS of kStripeChunkPairs pairs; a slot without a stored block ("dead") carries a byte
// offset past the end of W, which a buffer load answers with zeros, and the index of an extra,
// all-zero LDS panel for X.  So a chunk is always kStripeChunkPairs x (TM/16) MFMAs, the
// compiler can schedule its LDS reads and MFMAs freely.  Chunks are short (3 pairs: the fewer slots a
// chunk has, the fewer of them are dead), so most block-rows take two or more: W travels through
// four register buffers, a pair per block-row in turn -- the chunk after next is loaded into the
// buffer a multiply has just freed, and the first two chunks of the row after next into the pair a
// finished row leaves behind.
//
// LDS layout of the stripe: one PANEL per block-column (TM rows x 32 bytes, panels PS bytes apart),
// so the 16-row tiles of a lane's operand are at compile-time offsets from one address; the two
// 16-byte halves of a row are swapped in rows with bit 2 set.
#include "bsr_mfma_common.h"

using namespace bsr_dev;

namespace {

constexpr int kXcds = 8;
constexpr int kRowsPerWave = 4;      // block-rows per wavefront: 4 x 16 columns = 64 outputs per row of Y
constexpr int KP = kStripeChunkPairs;
constexpr int kBufs = 4;             // W chunks in registers: a pair per block-row in turn, the other pair filling for the row after next
constexpr int kStageBatch = 8;       // 16-byte loads in flight per thread while the stripe is staged

typedef int i32x4 __attribute__((ext_vector_type(4)));

template <typename T, typename O, int TM>
__global__ __launch_bounds__(768) void bsr_mfma_stripe16(const T* __restrict__ X, const T* __restrict__ data,
                                                         unsigned w_bytes, const int32_t* __restrict__ pair_ptr,
                                                         const i32x4* __restrict__ pairs, O* __restrict__ Y,
                                                         int m, int k, int n, int R, int n_tiles, int n_groups,
                                                         int rows_per_group, unsigned cpr_magic)
{
    constexpr int SUB = TM / 16;                      // 16-row MFMA tiles along m
    constexpr int PS = TM * 32 + 32;                  // bytes from one panel to the next (+32: panels shift by 8 banks)
    extern __shared__ __attribute__((aligned(16))) unsigned char lds[];   // [k/16 + 1 panels][PS], then per-wavefront scratch
    const int RB = k * (int)sizeof(T);                // bytes of one row of X
    const int C = k / 16;                             // block-columns; panel C is the all-zero one

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int li = lane & 15, h = lane >> 4;          // MFMA row/column index, k-group 0..3
    const bool second = h >= 2;                       // this lane feeds the second block of a pair
    const int hh = h & 1;                             // which 8 of the block's 16 columns

    // workgroup -> (m-tile, block-row group); the groups of one m-tile share an XCD (and its L2 copy
    // of the stripe)
    const int xcd = (int)(blockIdx.x % kXcds), local = (int)(blockIdx.x / kXcds);
    const int tile = (local / n_groups) * kXcds + xcd, group = local % n_groups;
    if (tile >= n_tiles) return;                      // whole workgroup leaves together
    const int i_base = tile * TM;

    const int r_first = group * rows_per_group + wave * kRowsPerWave;
    const int r_end = min(min((group + 1) * rows_per_group, R), r_first + kRowsPerWave);

    // W through a buffer resource: a byte offset >= w_bytes (the dead slots) reads as zero
    const __amdgpu_buffer_rsrc_t wrsrc =
        __builtin_amdgcn_make_buffer_rsrc(const_cast<T*>(data), 0, (int)w_bytes, 0x00020000);
    // lane's part of a block: row li, 8 columns starting at hh*8
    const unsigned lane_w = (unsigned)(li * 32 + hh * 16);
    const unsigned lane_x = (unsigned)(li * 32 + ((hh ^ ((li >> 2) & 1)) * 16));

    u32x4 wreg[kBufs][KP];
    unsigned xoff[kBufs][KP];                         // LDS byte offset of the lane's X operand, 16-row tile 0
    auto load_chunk = [&](int buf, int qb) {          // pair entries qb .. qb+KP-1: {offset 1, offset 2, column 1, column 2}
        i32x4 e[KP];
#pragma unroll
        for (int q = 0; q < KP; ++q) e[q] = pairs[qb + q];
#pragma unroll
        for (int q = 0; q < KP; ++q) {
            // the entry is the same for the whole wavefront: its four words as scalars, so that each choice between
            // the pair's two blocks is one select (picked out of the vector by a lane-dependent index it was four)
            const int o1 = __builtin_amdgcn_readfirstlane(e[q].x), o2 = __builtin_amdgcn_readfirstlane(e[q].y);
            const int c1 = __builtin_amdgcn_readfirstlane(e[q].z) * PS, c2 = __builtin_amdgcn_readfirstlane(e[q].w) * PS;
            const unsigned off = (unsigned)(second ? o2 : o1) + lane_w;
            wreg[buf][q] = __builtin_amdgcn_raw_buffer_load_b128(wrsrc, (int)off, 0, 0);
            xoff[buf][q] = (unsigned)(second ? c2 : c1) + lane_x;
        }
    };

    // ---- stage the stripe: TM rows x k columns, one contiguous piece of memory ----
    // chunk q (16 bytes) of the stripe lies in row q / cpr; the quotient comes from a multiply with
    // cpr_magic = floor(2^32 / cpr) + 1, exact for q < 2^16 (the stripe has at most 10240 chunks).
    // kStageBatch loads are issued before the first LDS write; past the end the last chunk is
    // simply copied again (same bytes to the same place).
    // The first batch of loads goes out before anything else: it needs nothing but the workgroup's number, while
    // the wavefront's ranges in the pair table and its first chunks of W are two dependent reads away.
    int q0[kRowsPerWave], q1[kRowsPerWave];
    {
        const int cpr = RB / 16;                      // 16-byte chunks per row: 2 per block-column
        const int total = TM * cpr;
        const unsigned char* xb = reinterpret_cast<const unsigned char*>(X) + (size_t)i_base * (size_t)RB;
        const bool whole = i_base + TM <= m;          // uniform; else rows past m repeat row m-1, never stored
        const int step = (int)blockDim.x;
        u32x4 v[kStageBatch];
        int dst[kStageBatch];
        auto fetch = [&](int base) {
#pragma unroll
            for (int u = 0; u < kStageBatch; ++u) {
                const int q = min(base + u * step, total - 1);
                const int row = (int)__umulhi((unsigned)q, cpr_magic), cc = q - row * cpr;
                const size_t src = whole ? (size_t)q * 16 : (size_t)min(row, m - 1 - i_base) * (size_t)RB + (size_t)cc * 16;
                dst[u] = (cc >> 1) * PS + row * 32 + (((cc & 1) ^ ((row >> 2) & 1)) * 16);
                v[u] = *reinterpret_cast<const u32x4*>(xb + src);
            }
        };
        auto put = [&]() {
#pragma unroll
            for (int u = 0; u < kStageBatch; ++u) *reinterpret_cast<u32x4*>(lds + dst[u]) = v[u];
        };
        fetch(tid);                                   // every thread has a first batch (past the end: the last chunk again)
        __builtin_amdgcn_sched_barrier(0);

        // entry ranges of this wavefront's block-rows in the pair table, whole chunks each (rows past
        // r_end get an empty range)
#pragma unroll
        for (int j = 0; j < kRowsPerWave; ++j) {
            const int r = min(r_first + j, R - 1);
            q0[j] = pair_ptr[r];
            q1[j] = r_first + j < r_end ? pair_ptr[r + 1] : q0[j];
        }

        // first chunks of the first block-rows: in flight while the stripe is staged
#pragma unroll
        for (int j = 0; j < 2; ++j) {                     // the first two chunks of the first two block-rows (uniform)
            if (q0[j] < q1[j]) load_chunk(2 * j, q0[j]);
            if (q0[j] + KP < q1[j]) load_chunk(2 * j + 1, q0[j] + KP);
        }

        put();
        for (int base = tid + kStageBatch * step; base < total; base += kStageBatch * step) {
            fetch(base);
            put();
        }
        for (int z = tid; z < TM * 2; z += step) *reinterpret_cast<u32x4*>(lds + C * PS + z * 16) = u32x4{0u, 0u, 0u, 0u};
    }
    __syncthreads();
    if (r_first >= r_end) return;                     // no barrier after this point

    f32x4 acc[kRowsPerWave][SUB];
#pragma unroll
    for (int j = 0; j < kRowsPerWave; ++j)
#pragma unroll
        for (int s = 0; s < SUB; ++s) acc[j][s] = f32x4{0.f, 0.f, 0.f, 0.f};

    auto compute_chunk = [&](int buf, int j) {
#pragma unroll
        for (int q = 0; q < KP; ++q) {
            Frag<T, 8> wf, xf;
            wf.w[0] = wreg[buf][q].x; wf.w[1] = wreg[buf][q].y; wf.w[2] = wreg[buf][q].z; wf.w[3] = wreg[buf][q].w;
            const unsigned char* xp = lds + xoff[buf][q];
#pragma unroll
            for (int s = 0; s < SUB; ++s) {
                xf.load(reinterpret_cast<const T*>(xp + s * 512));
                mfma_frag<T, 16, 8>(acc[j][s], wf, xf);
            }
        }
    };

    // Block-row j multiplies out of the buffer pair (2 (j mod 2), + 1) in turn: while one chunk is multiplied the
    // chunk after next is loaded into the buffer just used, and when the row is done the pair takes the first two
    // chunks of the row after next.
#pragma unroll
    for (int j = 0; j < kRowsPerWave; ++j) {
        const int A = 2 * (j % 2), B = A + 1;
        for (int qb = q0[j]; qb < q1[j]; qb += 2 * KP) {          // chunks qb (in A) and qb + KP (in B)
            compute_chunk(A, j);
            if (qb + 2 * KP < q1[j]) load_chunk(A, qb + 2 * KP);
            if (qb + KP < q1[j]) {
                compute_chunk(B, j);
                if (qb + 3 * KP < q1[j]) load_chunk(B, qb + 3 * KP);
            }
        }
        if (j + 2 < kRowsPerWave) {
            if (q0[j + 2] < q1[j + 2]) load_chunk(A, q0[j + 2]);
            if (q0[j + 2] + KP < q1[j + 2]) load_chunk(B, q0[j + 2] + KP);
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
    unsigned char* scratch = lds + (size_t)(C + 1) * PS + (size_t)wave * (SPP * 16 * OS);
    unsigned char* ybytes = reinterpret_cast<unsigned char*>(Y + (size_t)r_first * 16);
    const int orow = lane / OC, opiece = lane - orow * OC;
    const int valid_bytes = (r_end - r_first) * 16 * (int)sizeof(O);   // the group's last wavefront may own < 4 block-rows
#pragma unroll
    for (int s0 = 0; s0 < SUB; s0 += SPP) {
        wave_lds_fence();
#pragma unroll
        for (int ss = 0; ss < SPP; ++ss)
#pragma unroll
            for (int j = 0; j < kRowsPerWave; ++j)
                store4<O>(reinterpret_cast<O*>(scratch + (size_t)(ss * 16 + li) * OS) + j * 16 + 4 * h,
                          acc[j][s0 + ss][0], acc[j][s0 + ss][1], acc[j][s0 + ss][2], acc[j][s0 + ss][3]);
        // same wavefront wrote and now reads: its LDS operations complete in order, no barrier needed
        wave_lds_fence();
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

size_t stripe_lds_bytes(int k, int tm, int waves, size_t out_size)
{
    const size_t panels = (size_t)(k / 16 + 1) * (size_t)(tm * 32 + 32);
    const int spp = out_size == 2 ? (tm >= 32 ? 2 : 1) : 1;
    return panels + (size_t)waves * (size_t)spp * 16 * (kRowsPerWave * 16 * out_size + 16);
}

template <typename T, typename O>
bsr_status launch_stripe_types(const spmm_args& a, const tune_opts& tune)
{
    const bsr_matrix* W = a.W;
    const int m = (int)a.m, n = (int)W->n, k = (int)W->k, R = W->R;
    auto go = [&](auto tm_tag) -> bsr_status {
        constexpr int TM = decltype(tm_tag)::value;
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
        const size_t lds = stripe_lds_bytes(k, TM, waves, sizeof(O));
        if (lds > 160 * 1024) return BSR_ERR_UNSUPPORTED;
        const int64_t blocks = (int64_t)((n_tiles + kXcds - 1) / kXcds) * kXcds * n_groups;
        if (blocks >= ((int64_t)1 << 31)) return BSR_ERR_SHAPE;
        static const hipError_t attr =
            hipFuncSetAttribute(reinterpret_cast<const void*>(&bsr_mfma_stripe16<T, O, TM>),
                                hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
        if (attr != hipSuccess) return BSR_ERR_HIP;
        hipLaunchKernelGGL((bsr_mfma_stripe16<T, O, TM>), dim3((unsigned)blocks), dim3(64 * waves), lds, a.stream,
                           (const T*)a.X, (const T*)W->data, (unsigned)(W->nnzb * 512), W->pair_ptr,
                           reinterpret_cast<const i32x4*>(W->pairs), (O*)a.Y, m, k, n, R, n_tiles,
                           n_groups, rows_per_group, (unsigned)(0x100000000ull / (unsigned)(k * sizeof(T) / 16)) + 1u);
        return hipGetLastError() == hipSuccess ? BSR_OK : BSR_ERR_HIP;
    };
    // rows of X per workgroup: the largest stripe that still leaves 32 m-tiles (fewer, taller stripes
    // read W less often; too few leave CUs idle while a stripe is staged)
    int tm = tune.mt > 0 ? tune.mt * 16 : (m >= 32 * 64 ? 64 : (m >= 32 * 32 ? 32 : 16));
    while (tm > 16 && !mfma_stripe_supports(W, tm)) tm /= 2;      // wide X: a shorter stripe still fits LDS
    if (tm == 16) return go(std::integral_constant<int, 16>{});
    if (tm == 32) return go(std::integral_constant<int, 32>{});
    return go(std::integral_constant<int, 64>{});
}

}  // namespace

bool mfma_stripe_supports(const bsr_matrix* W, int tm)
{
    if (W->bs_r != 16 || W->bs_c != 16 || W->dtype == BSR_F32) return false;
    // byte offsets into W are 32-bit with the top bit marking a dead slot; the stripe has < 2^16 chunks
    if (!W->pairs || W->nnzb * 512 >= ((int64_t)1 << 31) || (int64_t)tm * (W->k / 8) >= 65536) return false;
    return stripe_lds_bytes((int)W->k, tm, 12, 4) <= 160 * 1024;
}

bsr_status launch_mfma_stripe(const spmm_args& a, const tune_opts& t)
{
    const bsr_matrix* W = a.W;
    if (!mfma_stripe_supports(W, 16)) return BSR_ERR_UNSUPPORTED;
    if (W->dtype == BSR_F16) return a.y_dtype == BSR_F32 ? launch_stripe_types<_Float16, float>(a, t)
                                                         : launch_stripe_types<_Float16, _Float16>(a, t);
    if (W->dtype == BSR_BF16) return a.y_dtype == BSR_F32 ? launch_stripe_types<__bf16, float>(a, t)
                                                          : launch_stripe_types<__bf16, __bf16>(a, t);
    return BSR_ERR_UNSUPPORTED;
}

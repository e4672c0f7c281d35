// Matrix-core kernel for thin blocks (bs_r = 16, bs_c = 1, fp32) in ONE launch and without scratch: rows of
// X staged in LDS.
//
// A 16x1 block couples one column of X with 16 columns of Y, so a block-row is a small dense product
// over a GATHER of X columns:
//     Y[:, r*16 : r*16+16] = X[:, block_indices[p0..p1)] * block_data[p0..p1, :, 0]
// Columns of a row-major X are strided (one element per row), so gathering them from memory moves a
// cache line per element.  This is the paper's coalescing problem (Sections 4.4.2-4.4.3: reads are only
// contiguous along the reduction axis of a block) at its extreme, a block that is one element wide.
// Here the gather happens in LDS: a workgroup stages 16 whole rows of X, 1024 columns (a PHASE) at a time,
// with coalesced 16-byte reads, and its wavefronts pick the columns their stored blocks name with 4-byte
// LDS reads.  X is read row-major; no transposed copy exists anywhere.
//
// Plan (bsr_create): the stored blocks of every block-row must come in non-decreasing block-column
// order (else this kernel is not used); per slot the plan keeps the positions where the block-columns
// cross the multiples of 1024, so the blocks of a (block-row, phase) are a contiguous run.
//
// Workgroup = 16 rows of X x 16 slots; 16 wavefronts.  Wavefront w moves row w of the row group (4 KiB per
// phase through registers into one of two LDS buffers, one phase ahead of its use) and multiplies slot w:
// per phase its run of stored blocks, 4 blocks per v_mfma_f32_16x16x4_f32, with
//   A (rows of the result = rows of X): lane l supplies X[i0 + l%16][column of block 4g + l/16] from LDS
//   B (columns = the 16 outputs of the block-row): lane l supplies block_data[4g + l/16][l%16]
// on two alternating accumulators (a dependent MFMA would wait for its predecessor).  The blocks of a run
// sit in registers, one dword per lane and MFMA (up to CAP MFMAs), and every register is re-loaded with the
// next phase's run as soon as its MFMA has been issued: the only wait on memory inside a phase is the one at
// its start, for loads that have had a whole phase to arrive.  The run's block-columns come with one load of
// 64 (a CU takes one wavefront-wide load per 16 cycles whatever it carries, and the load instructions are what
// bounds this kernel), go to a wavefront-private LDS area at the end of the phase before, and are read back
// from there, four distinct values per MFMA.  Both are read through buffer resources over the run, so entries
// past its end read as zero without branches (no traffic); a run longer than 4*CAP blocks takes extra passes
// with loads of their own.  One barrier per phase.
#include <algorithm>

#include "bsr_mfma_common.h"

using namespace bsr_dev;

namespace {

constexpr int kRowsX = 16;                            // rows of X per workgroup
constexpr int kPW = 1024;                             // columns of X per phase
constexpr int kRS = kPW * 4 + 16;                     // LDS row stride in bytes: rows shift by 4 banks
constexpr int kXBuf = kRowsX * kRS;
constexpr int kNB = 2;                                // phase buffers: one in use, one being written
constexpr int kWaves = 16;                            // = slots per workgroup = rows of X per workgroup
constexpr int kMaxCap = 24;                           // MFMAs of a phase whose operands are loaded ahead, at most
constexpr int kCArea = kMaxCap * 16;                  // a wavefront's block-columns of one phase, bytes
constexpr int kLds = kNB * kXBuf + kWaves * 2 * kCArea;
constexpr int kThreads = 64 * kWaves;
constexpr int kMaxPhases = 63;                        // a slot's phase positions sit one per lane
static_assert(kLds <= 160 * 1024 && kWaves == kRowsX, "LDS; a wavefront moves one row");

// LDS writes of this wavefront done, then the workgroup's barrier (loads from memory stay in flight across it)
__device__ __forceinline__ void wg_barrier() { asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory"); }

template <int CAP>
__global__ __launch_bounds__(kThreads) void bsr_thin16_rows(const float* __restrict__ X, const float* __restrict__ data,
                                                           const int32_t* __restrict__ indices,
                                                           const int32_t* __restrict__ row_desc,
                                                           const int32_t* __restrict__ ph_ptr, float* __restrict__ Y,
                                                           int m, int k, int n, int R, int nph, int n_rg, int n_set)
{
    static_assert(CAP % 4 == 0 && CAP <= kMaxCap, "MFMAs are skipped four at a time");
    constexpr int NC = (4 * CAP + 63) / 64;           // loads of 64 block-columns per run
    extern __shared__ __attribute__((aligned(1024))) unsigned char lds[];

    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int lo = lane & 15, kk = lane >> 4;

    // Workgroup -> (row group, slot set).  The 8 XCDs take workgroups round-robin and have private L2s:
    // XCD x works on the row groups x%4, x%4 + 4, ... and the slot sets x/4, x/4 + 2, ..., so a row of X
    // is fetched into 2 of the 8 L2s and a block into 4.
    const int x = (int)(blockIdx.x % 8u), local = (int)(blockIdx.x / 8u);
    const int rgs_here = (n_rg - (x & 3) + 3) >> 2, sets_here = (n_set - (x >> 2) + 1) >> 1;
    if (rgs_here <= 0 || sets_here <= 0) return;      // whole workgroup leaves together
    const int ri = local / sets_here, si = local - ri * sets_here;
    if (ri >= rgs_here) return;
    const int rg = (x & 3) + 4 * ri, set = (x >> 2) + 2 * si;
    const int i0 = rg * kRowsX;
    // The workgroups of an XCD start together and would walk the phases in step, all of them asking for the
    // same column range of rows that are k*4 bytes apart.  Each workgroup therefore takes the phases in its
    // own rotation: step s is phase (s + rot) mod nph (the order of a block-row's additions is free).
    const int rot = local % nph;
    auto phase_of = [&](int s) { const int p = s + rot; return p >= nph ? p - nph : p; };

    // ---- moving X: this wavefront's row, four loads of 1 KiB per phase ----
    const unsigned row_bytes = (unsigned)k * 4u;
    const unsigned char* src = reinterpret_cast<const unsigned char*>(X) + (size_t)min(i0 + wave, m - 1) * row_bytes;
    auto stage_load = [&](u32x4 (&r)[4], int s) __attribute__((always_inline)) {
        // columns past k repeat the row's last 16 bytes (no stored block names them)
        const unsigned cb = (unsigned)phase_of(s) * (kPW * 4u) + (unsigned)lane * 16u;
#pragma unroll
        for (int q = 0; q < 4; ++q) r[q] = *reinterpret_cast<const u32x4*>(src + min(cb + q * 1024u, row_bytes - 16u));
    };
    auto stage_write = [&](const u32x4 (&r)[4], int s) __attribute__((always_inline)) {
        unsigned char* dst = lds + (s & 1) * kXBuf + wave * kRS + lane * 16;
#pragma unroll
        for (int q = 0; q < 4; ++q) *reinterpret_cast<u32x4*>(dst + q * 1024) = r[q];
    };

    // The first two phases' rows go out at once; the second one's stays in flight behind the first run's
    // loads, as in every later phase (a phase's row is always older than the run loaded after it).
    u32x4 st0[4], st[4];
    stage_load(st0, 0);

    // ---- multiplying: slot set*16 + wave ----
    const int slot = set * kWaves + wave;
    // phase positions of the slot, one per lane: lane l holds position min(l, nph); a slot past R has empty runs
    const int pp = slot < R ? ph_ptr[(size_t)slot * (size_t)(nph + 1) + min(lane, nph)] : 0;
    stage_load(st, nph > 1 ? 1 : 0);
    // the run of step s as a pair of buffer resources: its blocks (64 bytes each) and its block-columns
    struct run_t { __amdgpu_buffer_rsrc_t w, i; int cnt; };
    auto run_of = [&](int s) __attribute__((always_inline)) {
        int e = 0, end = 0;
        if (s < nph) {                                // uniform
            const int ph = phase_of(s);
            e = __builtin_amdgcn_readlane(pp, ph);
            end = __builtin_amdgcn_readlane(pp, ph + 1);
        }
        run_t r;
        r.cnt = max(end - e, 0);
        r.w = __builtin_amdgcn_make_buffer_rsrc(const_cast<float*>(data + (size_t)e * 16), 0, r.cnt * 64, 0x00020000);
        r.i = __builtin_amdgcn_make_buffer_rsrc(const_cast<int32_t*>(indices + e), 0, r.cnt * 4, 0x00020000);
        return r;
    };
    const int w_off = kk * 64 + lo * 4;               // lane's entry of MFMA 0; MFMA g: + 256 g
    unsigned char* const c_area = lds + kNB * kXBuf + wave * (2 * kCArea);   // this wavefront's two areas (steps alternate)
    auto c_load = [&](int (&cr)[NC], const run_t& r) __attribute__((always_inline)) {
#pragma unroll
        for (int j = 0; j < NC; ++j) cr[j] = __builtin_amdgcn_raw_buffer_load_b32(r.i, (64 * j + lane) * 4, 0, 0);
    };
    auto c_write = [&](const int (&cr)[NC], int s) __attribute__((always_inline)) {
#pragma unroll
        for (int j = 0; j < NC; ++j)
            if (64 * j + 64 <= 4 * CAP || 64 * j + lane < 4 * CAP)
                *reinterpret_cast<int*>(c_area + (s & 1) * kCArea + (64 * j + lane) * 4) = cr[j];
    };

    float wv[CAP];
    int cr[NC];
    run_t cur = run_of(0);
    c_load(cr, cur);
#pragma unroll
    for (int g = 0; g < CAP; ++g)
        wv[g] = __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(cur.w, w_off + g * 256, 0, 0));
    stage_write(st0, 0);
    c_write(cr, 0);

    f32x4 acc[2] = {f32x4{0.f, 0.f, 0.f, 0.f}, f32x4{0.f, 0.f, 0.f, 0.f}};

    for (int s = 0; s < nph; ++s) {
        wg_barrier();                                 // step s is in its buffer; everybody is done with step s-1
        if (s + 1 < nph) stage_write(st, s + 1);      // loaded a phase ago
        if (s + 2 < nph) stage_load(st, s + 2);
        const run_t nxt = run_of(s + 1);              // empty behind the last step
        c_load(cr, nxt);
        asm volatile("" ::: "memory");                // the row moves on before the multiplying starts, not behind it
        // byte address of column 0 of this lane's row; the phase's first column sits at the buffer's start
        const unsigned char* a_row = lds + (s & 1) * kXBuf + lo * kRS;
        const unsigned char* c_at = c_area + (s & 1) * kCArea + kk * 4;
        const int col0 = phase_of(s) * kPW;
        int c[CAP];
#pragma unroll
        for (int g = 0; g < CAP; ++g) c[g] = *reinterpret_cast<const int*>(c_at + g * 16);
#pragma unroll
        for (int G = 0; G < CAP / 4; ++G) {
            if (G * 16 < cur.cnt) {                   // uniform
#pragma unroll
                for (int g = 4 * G; g < 4 * G + 4; ++g) {
                    // an entry past the run's end read 0 for its block (and 0 for its column: clamped)
                    const unsigned rel = min((unsigned)(c[g] - col0), (unsigned)(kPW - 1));
                    const float av = *reinterpret_cast<const float*>(a_row + rel * 4u);
                    acc[g & 1] = __builtin_amdgcn_mfma_f32_16x16x4f32(av, wv[g], acc[g & 1], 0, 0, 0);
                }
            }
#pragma unroll
            for (int g = 4 * G; g < 4 * G + 4; ++g)
                wv[g] = __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(nxt.w, w_off + g * 256, 0, 0));
        }
        // a run longer than the registers hold: the rest with loads of its own, 4 blocks at a time
        for (int b = 4 * CAP; b < cur.cnt; b += 4) {  // uniform
            const float w = __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(cur.w, w_off + b * 64, 0, 0));
            const int cc = __builtin_amdgcn_raw_buffer_load_b32(cur.i, (b + kk) * 4, 0, 0);
            const unsigned rel = min((unsigned)(cc - col0), (unsigned)(kPW - 1));
            const float av = *reinterpret_cast<const float*>(a_row + rel * 4u);
            acc[0] = __builtin_amdgcn_mfma_f32_16x16x4f32(av, w, acc[0], 0, 0, 0);
        }
        c_write(cr, s + 1);                           // into the other area; read after the next barrier
        cur = nxt;
    }

    // result of the MFMA: lane l holds rows 4*(l/16) + j (j = 0..3) of the row group, column l%16
    if (slot < R) {
        const int r = row_desc[(size_t)slot * kRowDescWords];
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int i = i0 + 4 * kk + j;
            if (i < m) Y[(size_t)i * n + (size_t)r * 16 + lo] = acc[0][j] + acc[1][j];
        }
    }
}

}  // namespace

size_t thinrow_plan_words(int64_t R, int64_t k, int32_t bs_r, int32_t bs_c)
{
    if (bs_r != 16 || bs_c != 1) return 0;
    return (size_t)R * (size_t)((k + kPW - 1) / kPW + 1) + 64;
}

bool mfma_thinrow_supports(const bsr_matrix* W) { return W->thin_ph != nullptr; }

void build_thinrow_plan(bsr_matrix* W, const int32_t* ptr, const int32_t* idx, size_t* words)
{
    W->thin_ph = nullptr;
    W->thin_nph = 0;
    W->thin_max_run = 0;
    if (W->bs_r != 16 || W->bs_c != 1 || W->dtype != BSR_F32 || W->R <= 0 || W->k < 4 || (W->k & 3) != 0) return;
    if (W->nnzb <= 0 || W->nnzb >= ((int64_t)1 << 25)) return;   // byte offsets into block_data are 32-bit
    if ((W->k + kPW - 1) / kPW > kMaxPhases) return;
    const int R = W->R;
    for (int r = 0; r < R; ++r)
        for (int32_t p = ptr[r] + 1; p < ptr[r + 1]; ++p)
            if (idx[p] < idx[p - 1]) return;          // a block-row out of order: the other kernels take this W
    const int nph = (int)((W->k + kPW - 1) / kPW);
    const int32_t* order = W->staging.data();         // slot -> block-row
    const size_t at = *words, end = (at + (size_t)R * (size_t)(nph + 1) + 63) & ~(size_t)63;
    W->staging.resize(end + 64, 0);
    order = W->staging.data();
    int32_t longest = 0;
    for (int s = 0; s < R; ++s) {
        const int r = order[s];
        int32_t* out = W->staging.data() + at + (size_t)s * (size_t)(nph + 1);
        for (int ph = 0; ph <= nph; ++ph)
            out[ph] = (int32_t)(std::lower_bound(idx + ptr[r], idx + ptr[r + 1], ph * kPW) - idx);
        out[nph] = ptr[r + 1];
        for (int ph = 0; ph < nph; ++ph) longest = std::max(longest, out[ph + 1] - out[ph]);
    }
    W->thin_ph = W->row_order + at;
    W->thin_nph = nph;
    W->thin_max_run = longest;
    *words = end;
}

bsr_status launch_mfma_thinrow(const spmm_args& a, const tune_opts& tune)
{
    const bsr_matrix* W = a.W;
    if (!mfma_thinrow_supports(W) || a.y_dtype != BSR_F32) return BSR_ERR_UNSUPPORTED;
    const int m = (int)a.m, n = (int)W->n, k = (int)W->k, R = W->R;
    auto go = [&](auto cap_tag) -> bsr_status {
        constexpr int CAP = decltype(cap_tag)::value;
        const int n_rg = (m + kRowsX - 1) / kRowsX, n_set = (R + kWaves - 1) / kWaves;
        const int64_t grid = 8 * (int64_t)((n_rg + 3) / 4) * ((n_set + 1) / 2);
        if (grid >= ((int64_t)1 << 31)) return BSR_ERR_SHAPE;
        static const hipError_t attr = hipFuncSetAttribute(reinterpret_cast<const void*>(&bsr_thin16_rows<CAP>),
                                                           hipFuncAttributeMaxDynamicSharedMemorySize, kLds);
        if (attr != hipSuccess) return BSR_ERR_HIP;
        hipLaunchKernelGGL((bsr_thin16_rows<CAP>), dim3((unsigned)grid), dim3(kThreads), kLds, a.stream, (const float*)a.X,
                           (const float*)W->data, W->indices, W->row_desc, W->thin_ph, (float*)a.Y, m, k, n, R,
                           W->thin_nph, n_rg, n_set);
        return hipGetLastError() == hipSuccess ? BSR_OK : BSR_ERR_HIP;
    };
    // MFMAs of a phase whose operands are loaded ahead (4 blocks each): enough for the average run and a
    // quarter more; the few longer runs take their tails with loads of their own
    const int64_t runs = (int64_t)R * W->thin_nph;
    const int cap = tune.a > 0 ? tune.a : (int)((W->nnzb * 5 / 4 + runs - 1) / runs + 3) / 4;
    if (cap <= 8) return go(std::integral_constant<int, 8>{});
    if (cap <= 16) return go(std::integral_constant<int, 16>{});
    return go(std::integral_constant<int, 24>{});
}

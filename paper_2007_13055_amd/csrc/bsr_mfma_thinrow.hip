// Matrix-core kernel for thin blocks (bs_r = 16, bs_c = 1, fp32) in ONE launch and without scratch: rows of
// X staged in LDS.
//
// A 16x1 block couples one column of X with 16 columns of Y, so a block-row is a small dense product
// over a GATHER of X columns:
//     Y[:, r*16 : r*16+16] = X[:, block_indices[p0..p1)] * block_data[p0..p1, :, 0]
// Columns of a row-major X are strided (one element per row), so gathering them from memory moves a
// cache line per element.  This is the paper's coalescing problem (Sections 4.4.2-4.4.3: reads are only
// contiguous along the reduction axis of a block) at its extreme, a block that is one element wide.
// Here the gather happens in LDS: a workgroup stages 16 whole rows of X, 256 columns (a PHASE) at a time,
// with coalesced 16-byte reads, and its wavefronts pick the columns their stored blocks name with 4-byte
// LDS reads.  X is read row-major; no transposed copy exists anywhere.  The kernel with the transposed
// copy in caller-lent scratch (bsr_mfma_thin.hip) is about 2.5 times faster and is preferred when the
// scratch is there: here every 16 stored blocks cost a round of bookkeeping (cursor, clamps, loads)
// that outweighs their four MFMAs.
//
// Plan (bsr_create): the stored blocks of every block-row must come in non-decreasing block-column
// order (else this kernel is not used); per slot the plan keeps the positions where the block-columns
// cross the multiples of 256, so the blocks of a (block-row, phase) are a contiguous run.
//
// Workgroup = 16 rows of X x a set of 8*SPW slots; 12 wavefronts.  Wavefronts 8-11 only move X: each
// takes 4 of the 16 rows through registers, six phases ahead, into two alternating LDS buffers.
// Wavefronts 0-7 take SPW slots each; per phase and ROUND they take the next 16 stored blocks of each
// slot: the block-columns and the blocks themselves (1 KiB, contiguous) arrive in a wavefront-private
// LDS ring several rounds ahead (global_load_lds), and per 4 blocks one v_mfma_f32_16x16x4_f32 runs with
//   A (rows of the result = rows of X): lane l supplies X[i0 + l%16][column of block 4g + l/16] from LDS
//   B (columns = the 16 outputs of the block-row): lane l supplies block_data[4g + l/16][l%16]
// on two alternating accumulators per slot (a dependent MFMA would wait for its predecessor).
// Entries past the end of a run multiply zeros: their B operand is replaced by zero.
#include <algorithm>

#include "bsr_mfma_common.h"

using namespace bsr_dev;

namespace {

constexpr int kRowsX = 16;                            // rows of X per workgroup
constexpr int kPW = 256;                              // columns of X per phase
constexpr int kRS = kPW * 4 + 16;                     // LDS row stride in bytes: rows shift by 4 banks
constexpr int kXBuf = kRowsX * kRS;
constexpr int kNB = 2;                                // phase buffers: one in use, one being written
constexpr int kConsumers = 8, kProducers = 4;
constexpr int kChunk = 16;                            // stored blocks per chunk
constexpr int kDepth = 6;                             // chunks a multiplying wavefront keeps in LDS: one in use, five on their way
constexpr int kEntry = kChunk * 64 + 256;             // a chunk in LDS: its blocks (1 KiB), then 64 block-columns
constexpr int kRing = kDepth * kEntry;                // per multiplying wavefront
constexpr int kLds = kNB * kXBuf + kConsumers * kRing;
constexpr int kThreads = 64 * (kConsumers + kProducers);
constexpr int kMaxPhases = 63;                        // a slot's phase positions sit one per lane
static_assert(kLds <= 160 * 1024 && kDepth % 2 == 0, "LDS; the ring holds whole rounds of 1 or 2 chunks");
static_assert(kPW * 4 == 1024 && kRowsX == 4 * kProducers, "a moving wavefront takes 4 rows, one 1 KiB load each");

template <int N>
__device__ __forceinline__ void wait_vm() { asm volatile("s_waitcnt vmcnt(%0)" ::"n"(N) : "memory"); }

__device__ __forceinline__ void wg_barrier() { asm volatile("s_barrier" ::: "memory"); }

template <int SPW>
__global__ __launch_bounds__(kThreads) void bsr_thin16_rows(const float* __restrict__ X, const float* __restrict__ data,
                                                           const int32_t* __restrict__ indices,
                                                           const int32_t* __restrict__ row_desc,
                                                           const int32_t* __restrict__ ph_ptr, float* __restrict__ Y,
                                                           int m, int k, int n, int R, int nph, int n_rg, int n_set,
                                                           unsigned data_bytes, unsigned index_bytes)
{
    typedef __attribute__((address_space(3))) void lds_void;
    typedef __attribute__((address_space(1))) const void glob_void;
    extern __shared__ __attribute__((aligned(1024))) unsigned char lds[];

    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);

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
    // The workgroups of an XCD start at about the same time and would walk the phases in step: all of them
    // reading the same 1 KiB column range of their 16 rows, rows that are k*4 bytes apart and fall into the
    // same L2 channel when k is a power of two.  Each workgroup therefore takes the phases in its own
    // rotation: step i is phase (i + rot) mod nph (the order of a block-row's additions is free).
    const int rot = local % nph;
    auto phase_of = [&](int i) { const int p = i + rot; return p >= nph ? p - nph : p; };

    if (wave >= kConsumers) {
        // ---- moving X: rows 4q .. 4q+3 of the row group, one load of 1 KiB per row and phase ----
        const int q = wave - kConsumers;
        const unsigned row_bytes = (unsigned)k * 4u;
        const unsigned char* Xb = reinterpret_cast<const unsigned char*>(X);
        const unsigned char* src[4];
#pragma unroll
        for (int rr = 0; rr < 4; ++rr) src[rr] = Xb + (size_t)min(i0 + 4 * q + rr, m - 1) * row_bytes;
        // Rows travel through registers (16 bytes per lane and row), kAhead steps ahead, and are written to
        // the step's buffer with 16-byte LDS writes.  (Loads that write LDS directly kept the LDS busy for
        // about four times as long as these writes do, and the operand reads waited behind them.)
        constexpr int kAhead = 6;
        u32x4 st[kAhead][4];
        auto load = [&](u32x4 (&r)[4], int i) __attribute__((always_inline)) {
            // columns past k repeat the row's last 16 bytes (never read back)
            const unsigned cb = min((unsigned)phase_of(i) * (kPW * 4u) + (unsigned)lane * 16u, row_bytes - 16u);
#pragma unroll
            for (int rr = 0; rr < 4; ++rr) r[rr] = *reinterpret_cast<const u32x4*>(src[rr] + cb);
        };
#pragma unroll
        for (int d = 0; d < kAhead; ++d)
            if (d < nph) load(st[d], d);
        for (int base = 0; base < nph; base += kAhead) {
#pragma unroll
            for (int d = 0; d < kAhead; ++d) {
                const int i = base + d;
                if (i < nph) {                        // uniform
                    unsigned char* buf = lds + (i % kNB) * kXBuf + (4 * q) * kRS + lane * 16;
#pragma unroll
                    for (int rr = 0; rr < 4; ++rr) *reinterpret_cast<u32x4*>(buf + rr * kRS) = st[d][rr];
                    if (i + kAhead < nph) load(st[d], i + kAhead);
                    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
                    wg_barrier();                     // step i is in its buffer; everybody is done with step i-1
                }
            }
        }
        return;
    }

    // ---- multiplying wavefront: slots set*8*SPW + wave + 8*sl ----
    const int lo = lane & 15, kk = lane >> 4;
    const int slot0 = set * (kConsumers * SPW) + wave;
    unsigned char* wr = lds + kNB * kXBuf + wave * kRing;
    const unsigned char* Wb = reinterpret_cast<const unsigned char*>(data);

    f32x4 acc[SPW][2];
#pragma unroll
    for (int s = 0; s < SPW; ++s) acc[s][0] = acc[s][1] = f32x4{0.f, 0.f, 0.f, 0.f};

    // phase positions of the wavefront's slots, one per lane: lane l holds position min(l, nph)
    int pp[SPW];
#pragma unroll
    for (int s = 0; s < SPW; ++s) {
        const int slot = slot0 + kConsumers * s;
        pp[s] = slot < R ? ph_ptr[(size_t)slot * (size_t)(nph + 1) + min(lane, nph)] : 0;
    }
    // The wavefront's work, step by step (a step = a phase in this workgroup's rotation): in every ROUND it
    // takes the next chunk of 16 stored blocks of each of its SPW slots (a slot whose run is used up takes
    // part with an empty chunk), so a round is straight-line code for SPW independent chunks, and a step has
    // as many rounds as its longest run needs.  Two cursors walk the rounds: one issues their loads, the
    // other, kRounds - 1 rounds behind, multiplies.
    constexpr int kRounds = kDepth / SPW;             // rounds the ring holds
    struct cursor { int step, r, rounds; };
    auto run_of = [&](int step, int s, int& e, int& end) __attribute__((always_inline)) {
        const int phase = phase_of(step);
        e = __builtin_amdgcn_readlane(pp[s], phase);
        end = __builtin_amdgcn_readlane(pp[s], phase + 1);
    };
    auto rounds_of = [&](int step) __attribute__((always_inline)) {
        int most = 0;
#pragma unroll
        for (int s = 0; s < SPW; ++s) {
            int e, end;
            run_of(step, s, e, end);
            most = max(most, end - e);
        }
        return (most + kChunk - 1) / kChunk;
    };
    auto advance = [&](cursor& c) __attribute__((always_inline)) {   // c.step == nph: no round left
        if (c.step >= nph) return;
        ++c.r;
        while (c.r >= c.rounds) {
            c.r = 0;
            if (++c.step >= nph) return;
            c.rounds = rounds_of(c.step);
        }
    };
    // A round into ring position d: per slot the chunk's blocks (lane l: 16-byte piece l of the 1 KiB run) and
    // 64 block-columns (lane l: block e + l), clamped to the arrays.  An empty chunk, and every chunk of the
    // rounds behind the last one, reads the start of the arrays: every round issues 2*SPW loads, so "all but
    // the youngest 2*SPW*(kRounds-1) have landed" always means the round in turn has.
    const unsigned last_piece = data_bytes - 16u;
    const int last_block = (int)(index_bytes >> 2) - 1;
    auto issue = [&](const cursor& c, int d) __attribute__((always_inline)) {
#pragma unroll
        for (int s = 0; s < SPW; ++s) {
            int e = 0, end = 0;
            if (c.step < nph) run_of(c.step, s, e, end);
            e = min(e + kChunk * c.r, max(end, 0));
            unsigned char* dst = wr + (d * SPW + s) * kEntry;
            const unsigned o = (unsigned)e * 64u + (unsigned)lane * 16u;
            __builtin_amdgcn_global_load_lds((glob_void*)(Wb + min(o, last_piece)), (lds_void*)dst, 16, 0, 0);
            __builtin_amdgcn_global_load_lds((glob_void*)(indices + min(e + lane, last_block)), (lds_void*)(dst + kChunk * 64), 4, 0, 0);
        }
    };
    cursor ci{-1, 0, 0};
    advance(ci);
    cursor cc = ci;
#pragma unroll
    for (int d = 0; d < kRounds - 1; ++d) {
        issue(ci, d);
        advance(ci);
    }
    int d_c = 0, d_i = kRounds - 1;

    for (int step = 0; step < nph; ++step) {
        wg_barrier();                                 // this step's columns of X are in their buffer
        const unsigned char* a_base = lds + (step % kNB) * kXBuf + lo * kRS;
        const int col0 = phase_of(step) * kPW;
        while (cc.step == step) {                     // uniform
            issue(ci, d_i);
            advance(ci);
            d_i = d_i + 1 == kRounds ? 0 : d_i + 1;
            wait_vm<2 * SPW * (kRounds - 1)>();
#pragma unroll
            for (int s = 0; s < SPW; ++s) {
                int e, end;
                run_of(step, s, e, end);
                const int cnt = min(max(end - e - kChunk * cc.r, 0), kChunk);   // blocks of this slot's chunk (may be none)
                const unsigned char* ent = wr + (d_c * SPW + s) * kEntry;
                const int col = *reinterpret_cast<const int*>(ent + kChunk * 64 + lo * 4);
                const int rel = min(max(col - col0, 0), kPW - 1) * 4;         // byte offset of the column inside the phase
                const unsigned char* b_base = ent + kk * 64 + lo * 4;
#pragma unroll
                for (int g = 0; g < kChunk / 4; ++g) {
                    const int cb = __builtin_amdgcn_ds_bpermute((4 * g + kk) * 4, rel);
                    const float av = *reinterpret_cast<const float*>(a_base + cb);
                    float bv = *reinterpret_cast<const float*>(b_base + g * 256);
                    bv = 4 * g + kk < cnt ? bv : 0.f;                         // entries past the run's end are zeros
                    acc[s][g & 1] = __builtin_amdgcn_mfma_f32_16x16x4f32(av, bv, acc[s][g & 1], 0, 0, 0);
                }
            }
            advance(cc);
            d_c = d_c + 1 == kRounds ? 0 : d_c + 1;
        }
    }

    // result of the MFMA: lane l holds rows 4*(l/16) + j (j = 0..3) of the row group, column l%16
#pragma unroll
    for (int sl = 0; sl < SPW; ++sl) {
        const int slot = slot0 + kConsumers * sl;
        if (slot < R) {
            const int r = row_desc[(size_t)slot * kRowDescWords];
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const int i = i0 + 4 * kk + j;
                if (i < m) Y[(size_t)i * n + (size_t)r * 16 + lo] = acc[sl][0][j] + acc[sl][1][j];
            }
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
    for (int s = 0; s < R; ++s) {
        const int r = order[s];
        int32_t* out = W->staging.data() + at + (size_t)s * (size_t)(nph + 1);
        for (int ph = 0; ph <= nph; ++ph)
            out[ph] = (int32_t)(std::lower_bound(idx + ptr[r], idx + ptr[r + 1], ph * kPW) - idx);
        out[nph] = ptr[r + 1];
    }
    W->thin_ph = W->row_order + at;
    W->thin_nph = nph;
    *words = end;
}

bsr_status launch_mfma_thinrow(const spmm_args& a, const tune_opts& tune)
{
    const bsr_matrix* W = a.W;
    if (!mfma_thinrow_supports(W) || a.y_dtype != BSR_F32) return BSR_ERR_UNSUPPORTED;
    const int m = (int)a.m, n = (int)W->n, k = (int)W->k, R = W->R;
    auto go = [&](auto spw_tag) -> bsr_status {
        constexpr int SPW = decltype(spw_tag)::value;
        const int n_rg = (m + kRowsX - 1) / kRowsX, n_set = (R + kConsumers * SPW - 1) / (kConsumers * SPW);
        const int64_t grid = 8 * (int64_t)((n_rg + 3) / 4) * ((n_set + 1) / 2);
        if (grid >= ((int64_t)1 << 31)) return BSR_ERR_SHAPE;
        static const hipError_t attr = hipFuncSetAttribute(reinterpret_cast<const void*>(&bsr_thin16_rows<SPW>),
                                                           hipFuncAttributeMaxDynamicSharedMemorySize, kLds);
        if (attr != hipSuccess) return BSR_ERR_HIP;
        hipLaunchKernelGGL((bsr_thin16_rows<SPW>), dim3((unsigned)grid), dim3(kThreads), kLds, a.stream, (const float*)a.X,
                           (const float*)W->data, W->indices, W->row_desc, W->thin_ph, (float*)a.Y, m, k, n, R,
                           W->thin_nph, n_rg, n_set, (unsigned)(W->nnzb * 64), (unsigned)(W->nnzb * 4));
        return hipGetLastError() == hipSuccess ? BSR_OK : BSR_ERR_HIP;
    };
    // slots per multiplying wavefront: 2 unless that leaves most CUs without a workgroup
    int spw = tune.a > 0 ? tune.a : 2;
    if (tune.a <= 0) {
        const int64_t wgs2 = (int64_t)((m + kRowsX - 1) / kRowsX) * ((R + 15) / 16);
        if (wgs2 < W->n_cu && R > kConsumers) spw = 1;
    }
    if (spw <= 1) return go(std::integral_constant<int, 1>{});
    return go(std::integral_constant<int, 2>{});
}



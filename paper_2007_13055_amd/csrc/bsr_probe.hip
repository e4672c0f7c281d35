// Peak probe for the benchmark: a loop of independent MFMAs with no memory traffic, so that roofline
// fractions can also be stated against what this chip delivers rather than against the data sheet.
// Not part of the product path.
#include "bsr_mfma_common.h"

using namespace bsr_dev;

namespace {

constexpr int kChains = 8;                            // independent accumulators per wavefront

template <typename T>
__global__ __launch_bounds__(256) void mfma_loop(int iters, float* __restrict__ sink)
{
    f32x16 acc[kChains];
#pragma unroll
    for (int c = 0; c < kChains; ++c)
#pragma unroll
        for (int e = 0; e < 16; ++e) acc[c][e] = 0.f;
    // operand values that keep every partial sum finite and lane-dependent
    const float seed = 1.0f / (float)(1 + (threadIdx.x & 7));
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int c = 0; c < kChains; ++c) {
            if constexpr (std::is_same<T, float>::value) {
                acc[c] = __builtin_amdgcn_mfma_f32_32x32x2f32(seed, 0.5f, acc[c], 0, 0, 0);
            } else if constexpr (std::is_same<T, f16_t>::value) {
                const f16_t a = (f16_t)seed, b = (f16_t)0.5f;
                const f16x8 av = {a, a, a, a, a, a, a, a}, bv = {b, b, b, b, b, b, b, b};
                acc[c] = __builtin_amdgcn_mfma_f32_32x32x16_f16(av, bv, acc[c], 0, 0, 0);
            } else {
                const bf16_t a = (bf16_t)seed, b = (bf16_t)0.5f;
                const bf16x8 av = {a, a, a, a, a, a, a, a}, bv = {b, b, b, b, b, b, b, b};
                acc[c] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(av, bv, acc[c], 0, 0, 0);
            }
        }
    }
    float s = 0.f;
#pragma unroll
    for (int c = 0; c < kChains; ++c)
#pragma unroll
        for (int e = 0; e < 16; ++e) s += acc[c][e];
    if (s == -1.0f) *sink = s;                        // never true (all terms are positive): keeps the loop alive
}

}  // namespace

extern "C" bsr_status bsr_probe_mfma(bsr_dtype dtype, int32_t iters, void* sink_dev, void* hip_stream, double* flops_out)
{
    if (!sink_dev || !flops_out) return BSR_ERR_NULL;
    if (iters < 1 || iters > (1 << 20)) return BSR_ERR_SHAPE;
    int dev = 0, n_cu = 256;
    if (hipGetDevice(&dev) != hipSuccess) return BSR_ERR_HIP;
    if (hipDeviceGetAttribute(&n_cu, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || n_cu <= 0) n_cu = 256;
    const unsigned blocks = (unsigned)n_cu * 8u;      // 8 workgroups of 4 wavefronts per CU
    hipStream_t stream = (hipStream_t)hip_stream;
    double per_mfma = 0.0;
    if (dtype == BSR_F32) {
        hipLaunchKernelGGL(mfma_loop<float>, dim3(blocks), dim3(256), 0, stream, (int)iters, (float*)sink_dev);
        per_mfma = 2.0 * 32 * 32 * 2;
    } else if (dtype == BSR_F16) {
        hipLaunchKernelGGL(mfma_loop<f16_t>, dim3(blocks), dim3(256), 0, stream, (int)iters, (float*)sink_dev);
        per_mfma = 2.0 * 32 * 32 * 16;
    } else if (dtype == BSR_BF16) {
        hipLaunchKernelGGL(mfma_loop<bf16_t>, dim3(blocks), dim3(256), 0, stream, (int)iters, (float*)sink_dev);
        per_mfma = 2.0 * 32 * 32 * 16;
    } else {
        return BSR_ERR_DTYPE;
    }
    if (hipGetLastError() != hipSuccess) return BSR_ERR_HIP;
    *flops_out = per_mfma * kChains * (double)iters * 4.0 * (double)blocks;
    return BSR_OK;
}

// Debug mode (environment BSR_SPMM_DEBUG=1 when the handle is created): before every product the device
// arrays that all kernel addresses derive from are checked ON THE DEVICE, as they are at that moment:
//   - index_pointer starts at 0, does not decrease, ends at the number of stored blocks;
//   - every block_indices entry lies in [0, k/bs_c) (the paper's three BSR arrays, Background);
//   - every row descriptor of the plan still names its block-row's range of index_pointer;
//   - the plan in the caller's workspace still holds what bsr_create() wrote (a position-weighted sum).
// Together with the host checks of m, k, n, alignment and types this bounds every address a kernel forms:
// rows of X and Y come from m and the launch grid, columns from block_indices and the plan.  The check
// costs one extra launch, a 16-byte copy and a stream synchronisation per product; it is skipped while the
// stream is being captured into a graph.
#include "bsr_internal.h"

namespace {

// out[0] = smallest failing code found (0: none), out[1] = position of one failure, out[2..3] = plan sum
__global__ __launch_bounds__(256) void bsr_debug_check(const int32_t* __restrict__ indptr, const int32_t* __restrict__ indices,
                                                       const int32_t* __restrict__ plan, const int32_t* __restrict__ row_desc,
                                                       int R, int C, int nnzb, int plan_words, int32_t* __restrict__ out)
{
    const int stride = (int)(gridDim.x * blockDim.x);
    const int t0 = (int)(blockIdx.x * blockDim.x + threadIdx.x);
    auto fail = [&](int code, int pos) {
        atomicMax(&out[0], 16 - code);                // the smallest code wins (reported as 16 - value)
        out[1] = pos;
    };
    if (t0 == 0 && (indptr[0] != 0 || indptr[R] != nnzb)) fail((int)BSR_ERR_INDPTR, indptr[0] != 0 ? 0 : R);
    for (int r = t0; r < R; r += stride)
        if (indptr[r + 1] < indptr[r]) fail((int)BSR_ERR_INDPTR, r + 1);
    for (int p = t0; p < nnzb; p += stride)
        if (indices[p] < 0 || indices[p] >= C) fail((int)BSR_ERR_INDEX, p);
    for (int s = t0; s < R; s += stride) {
        const int32_t* d = row_desc + (size_t)s * kRowDescWords;
        const int r = d[0];
        if (r < 0 || r >= R || d[1] != indptr[r] || d[2] != indptr[r + 1] - indptr[r]) fail((int)BSR_ERR_WORKSPACE, s);
    }
    unsigned long long sum = 0;
    for (int i = t0; i < plan_words; i += stride) sum += (unsigned long long)(uint32_t)plan[i] * (unsigned long long)(i + 1);
    if (sum) atomicAdd(reinterpret_cast<unsigned long long*>(out + 2), sum);
}

__global__ void bsr_debug_clear(int32_t* out)
{
    if (threadIdx.x < 4) out[threadIdx.x] = 0;
}

}  // namespace

uint64_t debug_plan_sum(const int32_t* words, size_t n)
{
    uint64_t sum = 0;
    for (size_t i = 0; i < n; ++i) sum += (uint64_t)(uint32_t)words[i] * (uint64_t)(i + 1);
    return sum;
}

bsr_status debug_check_device_arrays(const bsr_matrix* W, hipStream_t stream)
{
    if (!W->debug || W->R <= 0 || !W->debug_out) return BSR_OK;
    hipStreamCaptureStatus cap = hipStreamCaptureStatusNone;
    if (hipStreamIsCapturing(stream, &cap) != hipSuccess || cap != hipStreamCaptureStatusNone) {
        (void)hipGetLastError();
        return BSR_OK;                                // cannot synchronise inside a capture
    }
    hipLaunchKernelGGL(bsr_debug_clear, dim3(1), dim3(64), 0, stream, W->debug_out);
    hipLaunchKernelGGL(bsr_debug_check, dim3(256), dim3(256), 0, stream, W->indptr, W->indices, W->row_order, W->row_desc,
                       W->R, W->C, (int)W->nnzb, (int)W->debug_words, W->debug_out);
    int32_t host[4] = {0, 0, 0, 0};
    if (hipGetLastError() != hipSuccess) return BSR_ERR_HIP;
    if (hipMemcpyAsync(host, W->debug_out, sizeof(host), hipMemcpyDeviceToHost, stream) != hipSuccess) return BSR_ERR_HIP;
    if (hipStreamSynchronize(stream) != hipSuccess) return BSR_ERR_HIP;
    if (host[0] != 0) return (bsr_status)(16 - host[0]);
    uint64_t sum;
    std::memcpy(&sum, host + 2, sizeof(sum));
    return sum == W->debug_sum ? BSR_OK : BSR_ERR_WORKSPACE;
}

// The transposed matrix W^T in BSR, for the sibling product Z = G * W.
//
// The product kernels compute Y = X * W^T for a W stored by block-rows.  The gradient of a sparse
// layer's input is Z = G * W (G = dL/dY): the same product with W^T in place of W, because
// G * W = G * (W^T)^T.  So the library does not need a second family of kernels, only W^T in the
// same storage format: a (k, n) matrix whose block-rows are W's block-columns and whose blocks are
// the bs_c x bs_r transposes of W's blocks.  The pattern is transposed on the host (a stable
// counting sort of the stored blocks by block-column, so the blocks of a block-row of W^T come in
// ascending block-row of W), the values on the device, into memory the caller provides.
#include <numeric>
#include <vector>

#include "bsr_internal.h"

namespace {

// t_data[q][c][a] = data[perm[q]][a][c].  A workgroup takes `per` stored blocks (one when a block has
// more than 128 elements, else as many as its 256 threads cover); a bs_r x bs_c block is at most
// 64 x 64 elements here, staged through LDS so that both the read and the write run along the
// contiguous index.
template <typename T>
__global__ __launch_bounds__(256) void transpose_blocks(const T* __restrict__ data, const int32_t* __restrict__ perm,
                                                        T* __restrict__ t_data, int bs_r, int bs_c, int per, int nnzb)
{
    extern __shared__ __attribute__((aligned(16))) unsigned char raw[];
    T* tiles = reinterpret_cast<T*>(raw);             // [per][bs_r][bs_c + 1]
    const int elems = bs_r * bs_c, pitch = bs_c + 1;
    // thread -> (block of the workgroup, first element): threads_per_block threads stride over a block
    const int tpb = 256 / per;
    const int lb = (int)threadIdx.x / tpb, t = (int)threadIdx.x - lb * tpb;
    const int q = (int)blockIdx.x * per + lb;
    const bool live = lb < per && q < nnzb;
    T* tile = tiles + (size_t)lb * bs_r * pitch;
    if (live) {
        const T* src = data + (size_t)perm[q] * elems;
        for (int e = t; e < elems; e += tpb) {
            const int a = e / bs_c, c = e - a * bs_c;
            tile[a * pitch + c] = src[e];
        }
    }
    __syncthreads();
    if (live) {
        T* dst = t_data + (size_t)q * elems;
        for (int e = t; e < elems; e += tpb) {
            const int c = e / bs_r, a = e - c * bs_r;
            dst[e] = tile[a * pitch + c];
        }
    }
}

}  // namespace

extern "C" {

bsr_status bsr_transpose_pattern(int64_t n, int64_t k, int32_t bs_r, int32_t bs_c, int64_t nnzb,
                                 const int32_t* index_pointer_host, const int32_t* block_indices_host,
                                 int32_t* t_index_pointer_host, int32_t* t_block_indices_host, int32_t* perm_host)
{
    if (!t_index_pointer_host || (nnzb > 0 && (!t_block_indices_host || !perm_host))) return BSR_ERR_NULL;
    const bsr_status st = bsr_validate(n, k, bs_r, bs_c, nnzb, index_pointer_host, block_indices_host);
    if (st != BSR_OK) return st;
    const int64_t R = n / bs_r, C = k / bs_c;
    std::vector<int64_t> count((size_t)C + 1, 0);
    for (int64_t p = 0; p < nnzb; ++p) ++count[(size_t)block_indices_host[p] + 1];
    std::partial_sum(count.begin(), count.end(), count.begin());
    for (int64_t c = 0; c <= C; ++c) t_index_pointer_host[c] = (int32_t)count[(size_t)c];
    // stable: block-rows of W are visited in ascending order, so each block-row of W^T lists its
    // blocks by ascending block-row of W (and duplicates keep their order)
    for (int64_t r = 0; r < R; ++r)
        for (int64_t p = index_pointer_host[r]; p < index_pointer_host[r + 1]; ++p) {
            const int64_t q = count[(size_t)block_indices_host[p]]++;
            t_block_indices_host[q] = (int32_t)r;
            perm_host[q] = (int32_t)p;
        }
    return BSR_OK;
}

bsr_status bsr_transpose_values(bsr_dtype dtype, int32_t bs_r, int32_t bs_c, int64_t nnzb, const int32_t* perm_dev,
                                const void* block_data_dev, void* t_block_data_dev, void* hip_stream)
{
    if (dtype != BSR_F32 && dtype != BSR_F16 && dtype != BSR_BF16) return BSR_ERR_DTYPE;
    if (bs_r <= 0 || bs_c <= 0 || nnzb < 0 || nnzb >= ((int64_t)1 << 31)) return BSR_ERR_SHAPE;
    if (nnzb == 0) return BSR_OK;
    if (!perm_dev || !block_data_dev || !t_block_data_dev) return BSR_ERR_NULL;
    const size_t es = dtype == BSR_F32 ? 4 : 2;
    const int elems = bs_r * bs_c;
    const int per = elems > 128 ? 1 : 256 / elems;        // stored blocks per workgroup
    const size_t lds = (size_t)per * (size_t)bs_r * (size_t)(bs_c + 1) * es;
    if (lds > 64 * 1024) return BSR_ERR_UNSUPPORTED;      // blocks beyond 64 KiB are not staged
    const unsigned grid = (unsigned)((nnzb + per - 1) / per);
    hipStream_t stream = (hipStream_t)hip_stream;
    if (es == 4)
        hipLaunchKernelGGL(transpose_blocks<uint32_t>, dim3(grid), dim3(256), lds, stream,
                           (const uint32_t*)block_data_dev, perm_dev, (uint32_t*)t_block_data_dev, bs_r, bs_c, per,
                           (int)nnzb);
    else
        hipLaunchKernelGGL(transpose_blocks<uint16_t>, dim3(grid), dim3(256), lds, stream,
                           (const uint16_t*)block_data_dev, perm_dev, (uint16_t*)t_block_data_dev, bs_r, bs_c, per,
                           (int)nnzb);
    return hipGetLastError() == hipSuccess ? BSR_OK : BSR_ERR_HIP;
}

}  // extern "C"

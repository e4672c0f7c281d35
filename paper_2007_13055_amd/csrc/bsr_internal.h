// Internal declarations shared by the translation units of libbsr_spmm (not installed).
#pragma once

#include <hip/hip_runtime.h>

#include <cstddef>
#include <cstdint>
#include <vector>

#include "bsr_spmm.h"

// Host-side description of one W.  Device pointers are borrowed from the caller.
struct bsr_matrix {
    int64_t n = 0, k = 0, nnzb = 0;
    int32_t bs_r = 0, bs_c = 0;
    int32_t R = 0, C = 0;                    // block-rows, block-columns
    bsr_dtype dtype = BSR_F32;
    const void* data = nullptr;              // [nnzb][bs_r][bs_c]
    const int32_t* indices = nullptr;        // [nnzb]
    const int32_t* indptr = nullptr;         // [R+1]

    // ---- plan (paper, Discussion: unequal block-rows need different treatment) ----
    // Block-rows ordered by stored-block count, longest first; a workgroup's slot s works on
    // block-row row_order[s], so the long rows are dispatched before the short ones.
    const int32_t* row_order = nullptr;      // device, [R]
    int32_t max_row_blocks = 0;              // longest block-row
    int32_t empty_rows = 0;                  // block-rows with no stored block
    double mean_row_blocks = 0.0;
    std::vector<int32_t> staging;            // host copy of what was uploaded (kept for the async copy)
};

// Arguments every kernel launcher takes.
struct spmm_args {
    const bsr_matrix* W;
    int64_t m;
    const void* X;
    void* Y;
    bsr_dtype y_dtype;
    hipStream_t stream;
};

// Each returns BSR_OK, BSR_ERR_UNSUPPORTED (shape not covered by that family) or BSR_ERR_HIP.
bsr_status launch_wave(const spmm_args& a);
bsr_status launch_mfma(const spmm_args& a);
bool mfma_supports(const bsr_matrix* W);

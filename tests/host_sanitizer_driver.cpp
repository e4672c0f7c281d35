// Host-side sanitizer driver (test infrastructure): builds the library's plans -- row descriptors, pair, tile
// and run tables of bsr_create, the counting sort of bsr_transpose_pattern -- for 1440 random and adversarial
// patterns (empty, full, single-block and over-full block-rows, unsorted and repeated block-columns) over
// twelve block shapes and the three types, in a binary whose HOST code is compiled with AddressSanitizer and
// UndefinedBehaviorSanitizer.  No GPU is needed: without one the upload at the end of bsr_create fails with
// BSR_ERR_HIP after the whole plan has been built, which this driver accepts.
// Build and run (about 2.5 minutes, most of it the device pass of the kernels it links):
//   hipcc --offload-arch=gfx950 -O1 -g -std=c++17 -Xarch_host -fsanitize=address -Xarch_host -fsanitize=undefined \
//         -Xclang -target-feature -Xclang -packed-fp32-ops -I include -I paper_2007_13055_amd/csrc \
//         tests/host_sanitizer_driver.cpp paper_2007_13055_amd/csrc/*.hip -o /tmp/host_sanitizer_driver \
//         -fsanitize=address -fsanitize=undefined && ASAN_OPTIONS=detect_leaks=0 /tmp/host_sanitizer_driver
// tests/test_host_sanitizer.py does exactly that when BSR_RUN_SANITIZER=1 is set (it is too slow for every run).
#include <cstdio>
#include <cstdlib>
#include <vector>
#include <numeric>
#include "bsr_spmm.h"
static int run(int bs_r, int bs_c, bsr_dtype t, int R, int C, const std::vector<int>& counts, const std::vector<int>& idx)
{
    std::vector<int32_t> ptr(R + 1, 0);
    for (int r = 0; r < R; ++r) ptr[r + 1] = ptr[r] + counts[r];
    const int64_t nnzb = ptr[R];
    size_t need = 0;
    if (bsr_workspace_size((int64_t)R * bs_r, (int64_t)C * bs_c, bs_r, bs_c, nnzb, &need) != BSR_OK) return 100;
    std::vector<unsigned char> ws(need + 64), data((size_t)nnzb * bs_r * bs_c * 4 + 64);
    auto al = [](std::vector<unsigned char>& v) { return (void*)(((uintptr_t)v.data() + 15) & ~(uintptr_t)15); };
    bsr_matrix* W = nullptr;
    std::vector<int32_t> ix(idx.begin(), idx.end());
    bsr_status st = bsr_create(&W, (int64_t)R * bs_r, (int64_t)C * bs_c, bs_r, bs_c, nnzb, t, al(data), ix.data(), ptr.data(),
                               ix.data(), ptr.data(), al(ws), need, nullptr);
    if (st == BSR_OK) bsr_destroy(W);
    std::vector<int32_t> tp(C + 1), ti(nnzb + 1), perm(nnzb + 1);
    bsr_status s2 = bsr_transpose_pattern((int64_t)R * bs_r, (int64_t)C * bs_c, bs_r, bs_c, nnzb, ptr.data(), ix.data(), tp.data(), ti.data(), perm.data());
    return (int)st * 10 + (int)s2;
}
int main()
{
    const int shapes[][2] = {{16, 16}, {8, 8}, {8, 16}, {16, 8}, {32, 32}, {64, 64}, {16, 64}, {64, 16}, {16, 1}, {1, 16}, {3, 5}, {32, 16}};
    const bsr_dtype types[] = {BSR_F32, BSR_F16, BSR_BF16};
    srand(7);
    int n = 0;
    for (auto& sh : shapes)
        for (bsr_dtype t : types)
            for (int trial = 0; trial < 40; ++trial) {
                const int R = 1 + rand() % 70, C = 1 + rand() % 70;
                std::vector<int> counts(R), idx;
                for (int r = 0; r < R; ++r) {
                    const int mode = rand() % 5;
                    int c = mode == 0 ? 0 : mode == 1 ? C : mode == 2 ? 1 : rand() % (C + 1);
                    if (trial % 7 == 3) c = c * 3;                      // duplicates: more blocks than columns
                    counts[r] = c;
                    for (int j = 0; j < c; ++j) idx.push_back(trial % 5 == 0 ? rand() % C : (j * 7 + r) % C);   // unsorted / repeated
                }
                const int rc = run(sh[0], sh[1], t, R, C, counts, idx);
                if (rc / 10 != BSR_OK && rc / 10 != BSR_ERR_HIP) { printf("unexpected status %d shape %dx%d R=%d C=%d\n", rc, sh[0], sh[1], R, C); return 1; }
                if (rc % 10 != BSR_OK) { printf("transpose_pattern status %d\n", rc % 10); return 1; }
                ++n;
            }
    printf("plans built under the sanitizer: %d, no report\n", n);
    return 0;
}

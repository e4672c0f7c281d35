/*
 * CPU oracle for the block-sparse product  Y = X * W^T  (TEST INFRASTRUCTURE).
 *
 * This file is the correctness reference that the GPU library is checked
 * against.  It is deliberately plain and slow: the definition of the product
 * written out as loops, in IEEE double, in a fixed order.  It shares no code,
 * header, table or helper with the GPU library and must never be called from
 * the product path; only the tests, the smoke check and the benchmark's
 * cpu_baseline leg use it.
 *
 * What is computed (paper: Background, the three BSR arrays; Approaches, the
 * unnumbered equation X W_B^T = Y with b_r | n and b_c | k):
 *
 *   W is an (n, k) matrix cut into blocks of b_r rows and b_c columns.  Only
 *   some blocks are stored.  block_data[p] is the p-th stored block, a
 *   b_r x b_c row-major array; block_indices[p] is its block-column;
 *   index_pointer[r] .. index_pointer[r+1]-1 are the stored blocks of
 *   block-row r (CSR over blocks: length n/b_r + 1, first entry 0, last entry
 *   the number of stored blocks).  So
 *
 *     block_data[p][a][c] = W[r*b_r + a][block_indices[p]*b_c + c]
 *
 *   and for every row i of X, block-row r and row a inside the block
 *
 *     Y[i][r*b_r + a] = sum over p in block-row r, sum over c in [0, b_c) of
 *                         X[i][block_indices[p]*b_c + c] * block_data[p][a][c]
 *
 *   A block-row with no stored block gives exact zeros.  Two stored blocks
 *   with the same (block-row, block-column) both contribute (the sum runs over
 *   stored blocks, not over positions).  Blocks of a block-row may come in any
 *   order.
 *
 * Alongside Y the oracle returns S, the same double sum taken over the
 * absolute values of the products.  S is the scale of the admissible
 * difference: a GPU result passes when |Y_gpu - Y| <= tau * S elementwise.
 *
 * Inputs arrive as float because every input type the library accepts (fp32,
 * fp16, bf16) converts to float without change; each value is widened to
 * double before any arithmetic.  Products and sums are double; the order is p
 * ascending, then c ascending; nothing is blocked, fused or reordered.
 */
#include <stddef.h>
#include <stdint.h>
#include <math.h>
#ifdef _OPENMP
#include <omp.h>
#endif

enum {
    ORACLE_OK = 0,
    ORACLE_BAD_ARGUMENT = 1,   /* null pointer, non-positive size, b_r !| n, b_c !| k */
    ORACLE_BAD_POINTER = 2,    /* index_pointer not 0-based / non-decreasing / wrong end */
    ORACLE_BAD_INDEX = 3,      /* a block-column outside [0, k/b_c) */
    ORACLE_BAD_ROW = 4         /* a requested row of X outside [0, m) */
};

/* Number of threads the loops below will use. */
int oracle_num_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

void oracle_set_num_threads(int t)
{
#ifdef _OPENMP
    if (t > 0) omp_set_num_threads(t);
#else
    (void)t;
#endif
}

/* Structural check of the three BSR arrays (own code, not the library's). */
static int check_structure(int64_t k, int64_t n, int32_t b_r, int32_t b_c, int64_t nnzb,
                           const int32_t* block_indices, const int32_t* index_pointer)
{
    if (n < 0 || k < 0 || b_r <= 0 || b_c <= 0 || nnzb < 0) return ORACLE_BAD_ARGUMENT;
    if (n % b_r != 0 || k % b_c != 0) return ORACLE_BAD_ARGUMENT;
    if (!index_pointer) return ORACLE_BAD_ARGUMENT;
    if (nnzb > 0 && !block_indices) return ORACLE_BAD_ARGUMENT;
    const int64_t R = n / b_r, C = k / b_c;
    if (index_pointer[0] != 0) return ORACLE_BAD_POINTER;
    for (int64_t r = 0; r < R; ++r)
        if (index_pointer[r + 1] < index_pointer[r]) return ORACLE_BAD_POINTER;
    if (index_pointer[R] != nnzb) return ORACLE_BAD_POINTER;
    for (int64_t p = 0; p < nnzb; ++p)
        if (block_indices[p] < 0 || block_indices[p] >= C) return ORACLE_BAD_INDEX;
    return ORACLE_OK;
}

/*
 * Rows rows[0..n_rows) of the product (rows == NULL means rows 0..n_rows-1,
 * and then n_rows must equal m for the whole product).  Y and S are
 * [n_rows][n] row-major doubles; S may be NULL.
 */
int oracle_bsr_spmm_rows(int64_t m, int64_t k, int64_t n, int32_t b_r, int32_t b_c, int64_t nnzb,
                         const float* X, const float* block_data,
                         const int32_t* block_indices, const int32_t* index_pointer,
                         int64_t n_rows, const int64_t* rows, double* Y, double* S)
{
    if (m < 0 || n_rows < 0) return ORACLE_BAD_ARGUMENT;
    int st = check_structure(k, n, b_r, b_c, nnzb, block_indices, index_pointer);
    if (st != ORACLE_OK) return st;
    if (n_rows == 0 || n == 0) return ORACLE_OK;
    if (!Y || (m > 0 && k > 0 && !X) || (nnzb > 0 && !block_data)) return ORACLE_BAD_ARGUMENT;
    if (!rows && n_rows > m) return ORACLE_BAD_ROW;
    if (rows)
        for (int64_t q = 0; q < n_rows; ++q)
            if (rows[q] < 0 || rows[q] >= m) return ORACLE_BAD_ROW;

    const int64_t R = n / b_r;
    const int64_t block_elems = (int64_t)b_r * b_c;

#pragma omp parallel for schedule(static)
    for (int64_t q = 0; q < n_rows; ++q) {
        const int64_t i = rows ? rows[q] : q;
        const float* x_row = X + i * k;
        for (int64_t r = 0; r < R; ++r) {
            for (int32_t a = 0; a < b_r; ++a) {
                double y = 0.0, s = 0.0;
                for (int64_t p = index_pointer[r]; p < index_pointer[r + 1]; ++p) {
                    const float* w_row = block_data + p * block_elems + (int64_t)a * b_c;
                    const float* x_seg = x_row + (int64_t)block_indices[p] * b_c;
                    for (int32_t c = 0; c < b_c; ++c) {
                        const double prod = (double)x_seg[c] * (double)w_row[c];
                        y += prod;
                        s += fabs(prod);
                    }
                }
                Y[q * n + r * b_r + a] = y;
                if (S) S[q * n + r * b_r + a] = s;
            }
        }
    }
    return ORACLE_OK;
}

/*
 * The sibling product  Z = G * W  (G dense (m, n), same BSR arrays of W; Z is (m, k)).
 *
 * The paper gives Y = X W_B^T for the forward pass of a sparse fully connected layer and names
 * training as the use (Introduction); the gradient with respect to X of any function of Y is
 * (dL/dY) W, i.e. this product with G = dL/dY.  Written out from the same storage definition:
 *
 *   Z[i][block_indices[p]*b_c + c] = sum over block-rows r, over the stored blocks p of r, over
 *                                    a in [0, b_r) of  G[i][r*b_r + a] * block_data[p][a][c]
 *
 * Columns of Z whose block-column holds no stored block are exact zeros.  S is the same sum over
 * absolute values.  Order: r ascending, p ascending, a ascending (a plain scatter into Z, one row
 * of G at a time); double throughout.
 */
int oracle_bsr_spmm_w(int64_t m, int64_t k, int64_t n, int32_t b_r, int32_t b_c, int64_t nnzb,
                      const float* G, const float* block_data,
                      const int32_t* block_indices, const int32_t* index_pointer,
                      double* Z, double* S)
{
    if (m < 0) return ORACLE_BAD_ARGUMENT;
    int st = check_structure(k, n, b_r, b_c, nnzb, block_indices, index_pointer);
    if (st != ORACLE_OK) return st;
    if (m == 0 || k == 0) return ORACLE_OK;
    if (!Z || (n > 0 && !G) || (nnzb > 0 && !block_data)) return ORACLE_BAD_ARGUMENT;

    const int64_t R = n / b_r;
    const int64_t block_elems = (int64_t)b_r * b_c;

#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < m; ++i) {
        double* z_row = Z + i * k;
        double* s_row = S ? S + i * k : NULL;
        for (int64_t j = 0; j < k; ++j) {
            z_row[j] = 0.0;
            if (s_row) s_row[j] = 0.0;
        }
        const float* g_row = G + i * n;
        for (int64_t r = 0; r < R; ++r) {
            for (int64_t p = index_pointer[r]; p < index_pointer[r + 1]; ++p) {
                const int64_t col0 = (int64_t)block_indices[p] * b_c;
                for (int32_t a = 0; a < b_r; ++a) {
                    const double g = (double)g_row[r * b_r + a];
                    const float* w_row = block_data + p * block_elems + (int64_t)a * b_c;
                    for (int32_t c = 0; c < b_c; ++c) {
                        const double prod = g * (double)w_row[c];
                        z_row[col0 + c] += prod;
                        if (s_row) s_row[col0 + c] += fabs(prod);
                    }
                }
            }
        }
    }
    return ORACLE_OK;
}

/*
 * The sampled sibling: the gradient of the stored blocks,
 *
 *   D[p][a][c] = sum over i in [0, m) of  G[i][r*b_r + a] * X[i][block_indices[p]*b_c + c]
 *
 * for every stored block p of block-row r -- the entries of G^T X at the positions W stores, and
 * nothing else (positions of W without a stored block have no gradient).  It follows from the
 * same definition: Y = X W^T is linear in block_data[p][a][c] with coefficient X[i][col*b_c + c]
 * in Y[i][r*b_r + a].  D has the shape of block_data; S is the same sum over absolute values.
 * Order: i ascending; double throughout.
 */
int oracle_bsr_sddmm(int64_t m, int64_t k, int64_t n, int32_t b_r, int32_t b_c, int64_t nnzb,
                     const float* G, const float* X,
                     const int32_t* block_indices, const int32_t* index_pointer,
                     double* D, double* S)
{
    if (m < 0) return ORACLE_BAD_ARGUMENT;
    int st = check_structure(k, n, b_r, b_c, nnzb, block_indices, index_pointer);
    if (st != ORACLE_OK) return st;
    if (nnzb == 0) return ORACLE_OK;
    if (!D || (m > 0 && (!G || !X))) return ORACLE_BAD_ARGUMENT;

    const int64_t R = n / b_r;
    const int64_t block_elems = (int64_t)b_r * b_c;

#pragma omp parallel for schedule(dynamic)
    for (int64_t r = 0; r < R; ++r) {
        for (int64_t p = index_pointer[r]; p < index_pointer[r + 1]; ++p) {
            const int64_t col0 = (int64_t)block_indices[p] * b_c;
            for (int32_t a = 0; a < b_r; ++a) {
                for (int32_t c = 0; c < b_c; ++c) {
                    double d = 0.0, s = 0.0;
                    for (int64_t i = 0; i < m; ++i) {
                        const double prod = (double)G[i * n + r * b_r + a] * (double)X[i * k + col0 + c];
                        d += prod;
                        s += fabs(prod);
                    }
                    D[p * block_elems + (int64_t)a * b_c + c] = d;
                    if (S) S[p * block_elems + (int64_t)a * b_c + c] = s;
                }
            }
        }
    }
    return ORACLE_OK;
}

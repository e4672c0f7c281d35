"""Independent checkers used to pin the oracle (none of them is the oracle or the GPU path)."""
import numpy as np


def dense_expand(block_data, block_indices, index_pointer, n, k):
    """Dense (n, k) float64 W: stored blocks scatter-ADDED at their positions."""
    nnzb, bs_r, bs_c = block_data.shape
    W = np.zeros((n, k), dtype=np.float64)
    for r in range(n // bs_r):
        for p in range(int(index_pointer[r]), int(index_pointer[r + 1])):
            c = int(block_indices[p])
            W[r * bs_r:(r + 1) * bs_r, c * bs_c:(c + 1) * bs_c] += block_data[p].astype(np.float64)
    return W


def brute_force(X, W):
    """Y[i][j] = sum_l X[i][l] * W[j][l] over ALL l (zeros included), pure Python floats."""
    m, k = X.shape
    n = W.shape[0]
    Y = [[0.0] * n for _ in range(m)]
    S = [[0.0] * n for _ in range(m)]
    for i in range(m):
        for j in range(n):
            y = 0.0
            s = 0.0
            for l in range(k):
                t = float(X[i, l]) * float(W[j, l])
                y += t
                s += abs(t)
            Y[i][j] = y
            S[i][j] = s
    return np.array(Y).reshape(m, n), np.array(S).reshape(m, n)

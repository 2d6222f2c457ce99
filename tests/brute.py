"""O(N^2) kernel-score attention in numpy float64: the definition that linear
attention re-brackets (Sec. 3.2: the right-hand form of the linear-attention
equation equals sum_j sim(Q_i, K_j) V_j / sum_j sim(Q_i, K_j) with
sim(q, k) = phi(q) . phi(k), by associativity).  Tiny inputs only.
"""
import numpy as np


def kernel_score_attention(Q, K, V, eps, block_of=None):
    """Q, K, V: float arrays [N][d] of one head.  `block_of[i]` is the block
    index of token i; token i attends to token j iff block_of[j] <= block_of[i]
    (all pairs when block_of is None)."""
    Q = np.asarray(Q, np.float64)
    K = np.asarray(K, np.float64)
    V = np.asarray(V, np.float64)
    N = Q.shape[0]
    O = np.zeros_like(V)
    for i in range(N):
        qi = np.maximum(Q[i], 0.0)
        num = np.zeros(V.shape[1])
        den = 0.0
        for j in range(N):
            if block_of is not None and block_of[j] > block_of[i]:
                continue
            a = float(np.dot(qi, np.maximum(K[j], 0.0)))
            num += a * V[j]
            den += a
        O[i] = num / (den + eps)
    return O


def kernel_score_attention_dense(Q, K, V, eps, block_of=None):
    """Same quantity through an explicit N x N score matrix (faster for N~1000)."""
    Q = np.asarray(Q, np.float64)
    K = np.asarray(K, np.float64)
    V = np.asarray(V, np.float64)
    A = np.maximum(Q, 0.0) @ np.maximum(K, 0.0).T
    if block_of is not None:
        b = np.asarray(block_of)
        A = A * (b[None, :] <= b[:, None])
    return (A @ V) / (A.sum(axis=1, keepdims=True) + eps)


def rotate_pairs(X, table):
    """rot_t(x) for every token: adjacent feature pairs (2p, 2p+1) of row t turned
    by the angle whose (cos, sin) is table[t][p]."""
    X = np.asarray(X, np.float64)
    c = np.asarray(table, np.float64)[..., 0]
    s = np.asarray(table, np.float64)[..., 1]
    Y = np.empty_like(X)
    Y[:, 0::2] = X[:, 0::2] * c - X[:, 1::2] * s
    Y[:, 1::2] = X[:, 0::2] * s + X[:, 1::2] * c
    return Y


def kernel_score_attention_rope(Q, K, V, table, eps, block_of=None):
    """The full Sec. 3.2 equation as O(N^2) attention with TWO score matrices:
    numerator scores from rotated ReLU features, denominator scores from the
    un-rotated ones."""
    pQ = np.maximum(np.asarray(Q, np.float64), 0.0)
    pK = np.maximum(np.asarray(K, np.float64), 0.0)
    V = np.asarray(V, np.float64)
    A_num = rotate_pairs(pQ, table) @ rotate_pairs(pK, table).T
    A_den = pQ @ pK.T
    if block_of is not None:
        b = np.asarray(block_of)
        mask = b[None, :] <= b[:, None]
        A_num, A_den = A_num * mask, A_den * mask
    return (A_num @ V) / (A_den.sum(axis=1, keepdims=True) + eps)

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

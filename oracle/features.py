"""CPU oracle of the RIB feature generator -- TEST INFRASTRUCTURE, not product code.

Direct evaluation, in float64 numpy, of the paper's Sec. 3.1 Eq. 1-3: per-token
coordinates of an M x M window -> Fourier features -> one shared ReLU layer ->
per-head linear projections to the rank-r positional features f_q, f_k that the
attention operator concatenates to q and k (Eq. 5).  The backward pass is the
chain rule through those three lines.

Readings where the paper leaves a choice (each also listed in the design notes):
  * coordinates: M equally spaced values from -1 to 1 inclusive per axis
    (x_i = -1 + 2 i / (M - 1); the single token of M = 1 sits at 0);
  * the first coordinate is the row iy, the second the column ix, tokens in
    row-major order n = iy*M + ix (the order the attention operator uses);
  * frequencies are 2^l as printed in Eq. 1 (no factor pi);
  * feature order as printed: [x, sin(2^0 x), cos(2^0 x), ..., sin(2^(L-1) x),
    cos(2^(L-1) x)], every block holding the (row, column) pair: width 2 + 4L;
  * Eq. 3 prints no bias for the head-wise projections: none is used.

Nothing here imports the GPU package; only tests/, the smoke check and bench.py's
cpu_baseline leg may import this module.
"""
import numpy as np


def coordinates(M: int) -> np.ndarray:
    """[N, 2] float64: (row, column) coordinate of every token, in [-1, 1] (Sec. 3.1)."""
    axis = np.zeros(1) if M == 1 else -1.0 + 2.0 * np.arange(M, dtype=np.float64) / (M - 1)
    yy, xx = np.meshgrid(axis, axis, indexing="ij")
    return np.stack([yy.reshape(-1), xx.reshape(-1)], axis=1)


def fourier(x: np.ndarray, L: int) -> np.ndarray:
    """gamma(x) of Eq. 1: [N, 2 + 4L]."""
    blocks = [x]
    for l in range(L):
        blocks.append(np.sin((2.0 ** l) * x))
        blocks.append(np.cos((2.0 ** l) * x))
    return np.concatenate(blocks, axis=1)


def features_fwd(M, L, W_h, b_h, W_pq, W_pk):
    """Eq. 1-3.  W_h [2+4L, d_h], b_h [d_h], W_pq / W_pk [heads, d_h, r].
    Returns f_q, f_k as float64 [heads, N, r]."""
    W_h, b_h, W_pq, W_pk = (np.asarray(a, np.float64) for a in (W_h, b_h, W_pq, W_pk))
    r_in = fourier(coordinates(M), L)                     # Eq. 1
    h = np.maximum(r_in @ W_h + b_h, 0.0)                 # Eq. 2
    f_q = np.stack([h @ W_pq[hd] for hd in range(W_pq.shape[0])])     # Eq. 3, one projection per head
    f_k = np.stack([h @ W_pk[hd] for hd in range(W_pk.shape[0])])
    return f_q, f_k


def features_bwd(M, L, W_h, b_h, W_pq, W_pk, df_q, df_k):
    """Gradients of sum(f_q * df_q) + sum(f_k * df_k) with respect to the four
    parameter tensors: returns dW_h, db_h, dW_pq, dW_pk (float64)."""
    W_h, b_h, W_pq, W_pk, df_q, df_k = (np.asarray(a, np.float64) for a in (W_h, b_h, W_pq, W_pk, df_q, df_k))
    r_in = fourier(coordinates(M), L)
    pre = r_in @ W_h + b_h
    h = np.maximum(pre, 0.0)
    heads = W_pq.shape[0]
    dW_pq = np.stack([h.T @ df_q[hd] for hd in range(heads)])
    dW_pk = np.stack([h.T @ df_k[hd] for hd in range(heads)])
    dh = np.zeros_like(h)
    for hd in range(heads):
        dh += df_q[hd] @ W_pq[hd].T + df_k[hd] @ W_pk[hd].T
    dpre = dh * (pre > 0.0)
    return r_in.T @ dpre, dpre.sum(axis=0), dW_pq, dW_pk

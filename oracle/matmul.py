"""Oracle for the stand-alone masked product.  TEST INFRASTRUCTURE ONLY.

The operation behind the two matrix-multiplication latency figures of the paper's Section 3 (a dense input batch times
a square weight matrix, dense or sparse), with the sparsity expressed by the mask-based approach of Section 4:

    Y[b, r] = sum_k (Msk[r, k] ? W[r, k] : 0) * X[b, k]

in float64.  The mask selects: a value under a zero mask byte never enters the sum, whatever it is.
"""
import numpy as np


def masked_product(X: np.ndarray, W: np.ndarray, M) -> np.ndarray:
    X = np.asarray(X, dtype=np.float64)
    W = np.asarray(W, dtype=np.float64)
    batch, n_in = X.shape
    n_out = W.shape[0]
    assert W.shape == (n_out, n_in)
    Y = np.zeros((batch, n_out), np.float64)
    for r in range(n_out):
        kept = np.arange(n_in) if M is None else np.flatnonzero(np.asarray(M)[r] != 0)
        Y[:, r] = X[:, kept] @ W[r, kept]
    return Y

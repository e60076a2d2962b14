"""Pins of the stand-alone masked-product oracle (no GPU): a product worked by hand, brute force with plain Python
loops, and the selection semantics of the mask."""
import numpy as np

from oracle import matmul as omm


def test_hand_example():
    X = np.array([[1.0, 2.0, 3.0], [0.5, -1.0, 4.0]])
    W = np.array([[1.0, 0.0, -1.0], [2.0, 2.0, 2.0], [0.0, 1.0, 0.5]])
    M = np.array([[1, 1, 1], [1, 0, 1], [0, 1, 0]], np.uint8)
    # row 0: x0 - x2 ; row 1: 2 x0 + 2 x2 (middle entry masked) ; row 2: x1 (only the middle entry kept)
    want = np.array([[1 - 3, 2 + 6, 2], [0.5 - 4, 1 + 8, -1.0]])
    np.testing.assert_array_equal(omm.masked_product(X, W, M), want)
    # Y = X W^T, not X W: an asymmetric W tells them apart
    np.testing.assert_array_equal(omm.masked_product(X, W, None), X @ W.T)
    assert not np.array_equal(omm.masked_product(X, W, None), X @ W)


def test_brute_force_and_mask_selects():
    rng = np.random.default_rng(3)
    n, b = 7, 3
    X = rng.standard_normal((b, n)).astype(np.float32)
    W = rng.uniform(-0.1, 0.1, (n, n)).astype(np.float32)
    M = (rng.random((n, n)) < 0.4).astype(np.uint8)
    Y = omm.masked_product(X, W, M)
    for i in range(b):
        for r in range(n):
            s = 0.0
            for k in range(n):
                if M[r, k]:
                    s += float(W[r, k]) * float(X[i, k])
            assert abs(Y[i, r] - s) <= 1e-15
    Wj = W.copy()
    Wj[M == 0] = np.nan
    np.testing.assert_array_equal(omm.masked_product(X, Wj, M), Y)
    np.testing.assert_array_equal(omm.masked_product(X, W, np.zeros((n, n), np.uint8)), np.zeros((b, n)))

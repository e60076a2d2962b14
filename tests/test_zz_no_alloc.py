"""The allocation-free row/column pruning entry point against the allocating one (GPU, through the C ABI): the same
masks, weights and counts, bit for bit, on two calls in a row of which the second is smaller (it must not see what the
first left in the library's fixed scratch array), and a clear error above the fixed limit."""
import numpy as np
import pytest

from paper_1901_10997_amd import binding as B

pytestmark = pytest.mark.gpu


def _case(M, N, keep, seed):
    rng = np.random.default_rng(seed)
    W = (rng.standard_normal((M, N)) * np.exp(rng.uniform(-10, 3, (M, N)))).astype(np.float32)
    mask = (rng.random((M, N)) < keep).astype(np.uint8)
    return W, mask


def _both(W, mask, pr, pc):
    import torch
    dev = torch.device("cuda:0")
    M, N = W.shape
    Wa, ma = torch.from_numpy(W).to(dev), torch.from_numpy(mask).to(dev)
    Wb, mb = torch.from_numpy(W).to(dev), torch.from_numpy(mask).to(dev)
    removed = torch.full((2,), -7, dtype=torch.int32, device=dev)
    torch.cuda.synchronize()
    rows, cols = B.lstm_prune_rows_cols(Wa.data_ptr(), ma.data_ptr(), M, N, pr, pc)
    B.lstm_prune_rows_cols_static(Wb.data_ptr(), mb.data_ptr(), M, N, pr, pc, removed.data_ptr())
    torch.cuda.synchronize()
    assert np.array_equal(ma.cpu().numpy(), mb.cpu().numpy())
    assert np.array_equal(Wa.cpu().numpy().view(np.uint32), Wb.cpu().numpy().view(np.uint32))
    assert removed.cpu().tolist() == [rows, cols]
    return rows, cols


def test_static_scratch_variant_equals_the_allocating_one_twice_in_a_row():
    W1, m1 = _case(1500, 1900, 0.6, 1)          # a gate matrix of the language-model shape
    r1, c1 = _both(W1, m1, 0.2, 0.0)
    assert r1 >= 300
    W2, m2 = _case(257, 130, 0.5, 2)            # smaller: fewer sums than the first call left in the array
    r2, c2 = _both(W2, m2, 0.1, 0.25)
    assert r2 >= 26 and c2 >= 33
    W3, m3 = _case(64, 2000, 0.9, 3)            # and a third that is wider than the second
    _both(W3, m3, 0.0, 0.3)


def test_static_scratch_variant_without_counts_and_above_the_limit():
    import torch
    W, m = _case(40, 30, 0.8, 4)
    dev = torch.device("cuda:0")
    Wa, ma = torch.from_numpy(W).to(dev), torch.from_numpy(m).to(dev)
    Wb, mb = torch.from_numpy(W).to(dev), torch.from_numpy(m).to(dev)
    B.lstm_prune_rows_cols(Wa.data_ptr(), ma.data_ptr(), 40, 30, 0.25, 0.1)
    B.lstm_prune_rows_cols_static(Wb.data_ptr(), mb.data_ptr(), 40, 30, 0.25, 0.1, None)
    torch.cuda.synchronize()
    assert np.array_equal(ma.cpu().numpy(), mb.cpu().numpy())
    with pytest.raises(B.LstmError) as ei:
        B.lstm_prune_rows_cols_static(Wb.data_ptr(), mb.data_ptr(), 16385, 1, 0.1, 0.1, None)
    assert ei.value.code == B.LSTM_ERR_ARG and "16384" in str(ei.value)
    with pytest.raises(B.LstmError):
        B.lstm_prune_rows_cols_static(Wb.data_ptr(), mb.data_ptr(), 1, 16385, 0.1, 0.1, None)

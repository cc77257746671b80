"""Pins for the oracle's per-row top-k of the prefill logits (no GPU)."""
import numpy as np
import pytest

from oracle.calibration import topk_rows
from oracle.acceptance import _argmax_rows


def test_hand_worked_rows_with_ties():
    z = np.array([[1.0, 5.0, 3.0, 5.0, -2.0, 3.0],      # 5.0 twice, 3.0 twice: lower id first
                  [0.0, 0.0, 0.0, 0.0, 0.0, 0.0],       # all equal: ids in order
                  [-1.0, -3.0, -2.0, -0.5, -9.0, -0.5]], dtype=np.float32)
    v, i = topk_rows(z, 4)
    assert i.tolist() == [[1, 3, 2, 5], [0, 1, 2, 3], [3, 5, 0, 2]]
    assert v.tolist() == [[5.0, 5.0, 3.0, 3.0], [0.0] * 4, [-0.5, -0.5, -1.0, -2.0]]


def test_against_repeated_maximum_and_partition_routes():
    rng = np.random.default_rng(0)
    for V, k in ((7, 7), (50, 3), (1000, 8), (4096, 5)):
        z = rng.standard_normal((6, V)).astype(np.float32)
        z[:, rng.integers(0, V, V // 3)] = np.float32(0.25)          # many exact ties
        v, ids = topk_rows(z, k)
        for r in range(6):
            # brute force: take the maximum (lowest id among equals) k times
            left = z[r].astype(np.float64).copy()
            want = []
            for _ in range(k):
                j = int(np.argmax(left))
                want.append(j)
                left[j] = -np.inf
            assert ids[r].tolist() == want
            # library route: the k-th largest value by partition bounds the selection
            kth = np.partition(z[r], V - k)[V - k]
            assert v[r, -1] == kth and np.all(np.diff(v[r]) <= 0)
            assert np.count_nonzero(z[r] > kth) <= k - 1 or np.count_nonzero(z[r] > kth) < k
        assert np.array_equal(ids[:, 0], _argmax_rows(z))             # the first entry is the arg-max


def test_k_out_of_range():
    z = np.zeros((2, 5), dtype=np.float32)
    for k in (0, 6):
        with pytest.raises(ValueError):
            topk_rows(z, k)

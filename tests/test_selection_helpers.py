"""The test-side selection helpers of gpu_util (used to check the device's top-k against the
device's own scores and for validity under the score tolerance) are themselves checked here, on
the CPU, against the oracle's full-sort selection and on hand-made cases."""
import numpy as np
import pytest

import oracle
from gpu_util import check_selection_valid, full_sort_selection


@pytest.mark.parametrize("seed", range(5))
def test_full_sort_selection_equals_the_oracle_on_random_scores_with_ties(seed):
    rng = np.random.default_rng(seed)
    for n in (1, 2, 7, 64, 300):
        scores = rng.standard_normal((3, n)).astype(np.float32)
        scores[:, rng.integers(0, n, size=max(1, n // 3))] = 0.25          # exact ties
        for k in (0, 1, n // 2, n, n + 3):
            idx, mask = full_sort_selection(scores, k)
            widx, wmask = oracle.select_topk(scores, k)
            assert np.array_equal(idx, widx) and np.array_equal(mask, wmask)


def test_validity_check_accepts_swaps_inside_the_tolerance_only():
    want = np.array([[5.0, 4.0, 3.0 + 1e-7, 3.0, 1.0]])
    wmask = oracle.select_topk(want, 3)[1]
    assert wmask.tolist() == [[1, 1, 1, 0, 0]]
    # chunk 3 instead of chunk 2: their scores differ by less than the tolerance -> valid
    check_selection_valid(np.array([[0, 1, 3]]), np.array([[1, 1, 0, 1, 0]], np.uint8), want, wmask, 3, tol=1e-6)
    # chunk 4 instead of chunk 2: clearly worse -> rejected
    with pytest.raises(AssertionError):
        check_selection_valid(np.array([[0, 1, 4]]), np.array([[1, 1, 0, 0, 1]], np.uint8), want, wmask, 3, tol=1e-6)
    # a clear margin at rank k: only the oracle's mask passes
    with pytest.raises(AssertionError):
        check_selection_valid(np.array([[0, 2, 3]]), np.array([[1, 0, 1, 1, 0]], np.uint8), want, wmask, 3, tol=1e-6)
    # wrong count, or an index list that disagrees with the mask
    with pytest.raises(AssertionError):
        check_selection_valid(np.array([[0, 1]]), np.array([[1, 1, 0, 0, 0]], np.uint8), want, wmask, 3, tol=1e-6)
    with pytest.raises(AssertionError):
        check_selection_valid(np.array([[0, 1, 2]]), np.array([[1, 1, 0, 1, 0]], np.uint8), want, wmask, 3, tol=1e-6)

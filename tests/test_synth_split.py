"""Host-side input recipe for the data-splitting arrangement of Section 5 (no GPU, no method arithmetic)."""
import numpy as np
import pytest

from paper_1707_00424_amd import synth


@pytest.mark.parametrize("n,fraction", [(3, 0.5), (6, 0.25), (4, 0.25), (3, 1.0)])
def test_subsets_have_equal_size_and_cover_the_set(n, fraction):
    S = 1001
    shards = synth.split_shards(7, S, n, fraction)
    assert shards.shape == (n, int(np.ceil(fraction * S)))
    assert all(len(np.unique(s)) == shards.shape[1] for s in shards)       # no sample twice in one subset
    assert np.array_equal(np.unique(shards), np.arange(S))                  # every sample lies in a subset
    if n * fraction > 1.0 and fraction < 1.0:
        assert len(np.intersect1d(shards[0], shards[1])) > 0               # Table 2's cases overlap
        assert len(np.setdiff1d(shards[0], shards[1])) > 0                 # and still differ


def test_subsets_that_cannot_cover_are_refused():
    with pytest.raises(ValueError):
        synth.split_shards(0, 100, 3, 0.25)


def test_replicas_draw_only_from_their_own_subset_in_epochs():
    n, B, steps, S = 3, 16, 9, 96
    X, Y, idx, shards = synth.split_image_batches(3, steps, n, B, 4, 4, 3, S, 0.5)
    assert X.shape == (steps, n, B, 4, 4, 3) and Y.shape == (steps, n, B) and X.dtype == np.float32
    m = shards.shape[1]
    for a in range(n):
        walk = idx[:, a].reshape(-1)
        assert np.isin(walk, shards[a]).all()
        assert np.array_equal(np.sort(walk[:m]), np.sort(shards[a]))       # first epoch visits the subset once
    # the same sample is the same image and label wherever it is drawn
    flat_i, flat_x, flat_y = idx.reshape(-1), X.reshape(-1, 48), Y.reshape(-1)
    first = {}
    for i, x, y in zip(flat_i, flat_x, flat_y):
        if i in first:
            assert np.array_equal(first[i][0], x) and first[i][1] == y
        first[i] = (x, y)
    X2, Y2, idx2, _ = synth.split_image_batches(3, steps, n, B, 4, 4, 3, S, 0.5)
    assert np.array_equal(X, X2) and np.array_equal(idx, idx2)             # seeded

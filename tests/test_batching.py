"""Host logic that batches sentences of different lengths for the padded entry points."""
import numpy as np
import pytest

from paper_2209_12708_amd import batching as bt


def test_padded_length_rounds_up_to_the_multiple():
    assert [bt.padded_length(n) for n in (1, 4, 5, 8, 61)] == [4, 4, 8, 8, 64]


def test_buckets_cover_every_sentence_once_and_share_a_padded_length():
    rng = np.random.default_rng(0)
    lens = rng.integers(4, 63, 200)                       # the spread of the shorter of the paper's data sets
    batches = bt.bucket_by_length(lens, max_batch=16)
    seen = np.concatenate([idx for idx, _ in batches])
    assert sorted(seen) == list(range(200))
    for idx, L in batches:
        assert 1 <= len(idx) <= 16 and L % 4 == 0
        assert np.all(lens[idx] <= L) and np.all(lens[idx] > L - 4)      # nobody is padded by a whole group of 4
    # padding waste is bounded by the rounding alone
    assert sum(len(idx) * L for idx, L in batches) <= lens.sum() + 3 * 200


def test_bucket_order_is_stable_and_batches_close_at_max_batch():
    batches = bt.bucket_by_length([8, 8, 8, 5, 8], max_batch=2)
    assert [(list(i), L) for i, L in batches] == [([3, 0], 8), ([1, 2], 8), ([4], 8)]
    with pytest.raises(ValueError):
        bt.bucket_by_length([3, 0], 4)
    with pytest.raises(ValueError):
        bt.bucket_by_length([], 4)


def test_pad_batch_fills_rows_and_reports_lengths():
    sents = [[5, 6, 7], [1], [9, 9, 9, 9, 9]]
    tok, lens = bt.pad_batch(sents, np.array([2, 0]), 8, pad_token=3)
    assert tok.dtype == np.int32 and tok.shape == (2, 8)
    assert list(tok[0]) == [9, 9, 9, 9, 9, 3, 3, 3] and list(tok[1]) == [5, 6, 7, 3, 3, 3, 3, 3]
    assert list(lens) == [5, 3]
    with pytest.raises(ValueError):
        bt.pad_batch(sents, np.array([2]), 4)

"""Pins for the host packing step's oracle."""
from oracle.packing import pack_microbatches


def test_skip_zero_length_and_keep_order():
    order, off, cus = pack_microbatches([5, 0, 3, 0, 4], 8, 0)
    assert order == [0, 2, 4] and off == [0, 2, 3] and cus == [[0, 5, 8], [0, 4]]


def test_longest_first_is_stable_and_oversized_sample_alone():
    order, off, cus = pack_microbatches([2, 9, 2, 20, 9], 10, 1)
    assert order == [3, 1, 4, 0, 2]
    assert cus == [[0, 20], [0, 9], [0, 9], [0, 2, 4]] and off == [0, 1, 2, 3, 5]


def test_all_text_only_gives_no_microbatch():
    assert pack_microbatches([0, 0], 16, 0) == ([], [0], [])


def test_every_kept_token_appears_once():
    lens = [7, 0, 1, 12, 5, 5, 0, 9]
    order, off, cus = pack_microbatches(lens, 16, 1)
    assert sorted(order) == [i for i, n in enumerate(lens) if n > 0]
    assert sum(c[-1] for c in cus) == sum(lens)
    assert all(c[-1] <= 16 for c in cus)

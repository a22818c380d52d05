"""Host logic: the tile ranges the matrix-core plan gives its waves (odma_stream_plan_ranges, the same arithmetic the
plan kernel runs on the device).

The attention kernel lets a wave whose segment runs on past its range wait for the first piece of its right-hand
neighbour inside the work-group; an empty wave hands nothing over, so a range that holds tiles must never have an
empty range to its right among the used waves.  These tests pin that, and the plain properties of a partition,
over small totals, both work-group sizes, every tile minimum and the whole range of the share weights.
"""
import itertools

import numpy as np
import pytest

from paper_2512_09427_amd import binding as B


def ranges(total, n_waves, wpw, q_min, odd=256, late=256):
    start, used = B.odma_stream_plan_ranges(total, n_waves, wpw, q_min, odd, late)
    return start.astype(np.int64), used


def check_partition(total, n_waves, wpw, q_min, odd=256, late=256):
    start, used = ranges(total, n_waves, wpw, q_min, odd, late)
    what = f"total={total} n_waves={n_waves} wpw={wpw} q_min={q_min} odd={odd} late={late}"
    assert start[0] == 0 and start[-1] == total, what
    assert (np.diff(start) >= 0).all(), what
    assert 1 <= used <= n_waves and used % wpw == 0, what
    assert (start[used:] == total).all(), what                      # waves past `used` hold nothing
    sizes = np.diff(start)[:used]
    holding = np.nonzero(sizes > 0)[0]
    if len(holding):
        # empty ranges form a prefix of the used waves
        assert (sizes[holding[0]:] > 0).all(), what + f" sizes={sizes.tolist()}"
    return sizes, used


@pytest.mark.parametrize("wpw", [4, 8])
def test_no_empty_range_right_of_a_range_with_tiles_small_totals(wpw):
    for n_waves in (wpw, 2 * wpw, 1024):
        for q_min in (1, 2, 4, 8):
            for total in range(0, 6 * wpw * 4 + 3):
                sizes, used = check_partition(total, n_waves, wpw, q_min)
                if total >= used:
                    assert sizes.max() - sizes.min() <= 1              # equal weights: shares differ by at most a tile


def test_the_shapes_that_used_to_interleave_empty_ranges():
    # one request of two tiles on one KV head, default shape: two tiles over a four-wave work-group
    sizes, used = check_partition(2, 1024, 4, 4)
    assert used == 4 and sizes.tolist() == [0, 0, 1, 1]
    # eight-wave work-groups, 2..6 tiles
    for total in range(2, 7):
        sizes, used = check_partition(total, 2048, 8, 4)
        assert used == 8 and sizes.tolist() == [0] * (8 - total) + [1] * total


@pytest.mark.parametrize("wpw", [4, 8])
def test_weighted_shares_never_round_to_nothing(wpw):
    rng = np.random.default_rng(7)
    weights = [128, 160, 232, 256, 300, 512]
    for odd, late in itertools.product(weights, weights):
        for n_waves in (wpw, 8 * wpw, 1024):
            totals = np.unique(np.concatenate([np.arange(0, 5 * n_waves + 2, max(1, n_waves // 16)),
                                               rng.integers(0, 40 * n_waves, 12)]))
            for q_min in (1, 2, 4):
                for total in totals:
                    sizes, used = check_partition(int(total), n_waves, wpw, q_min, odd, late)
                    if total >= 4 * used:
                        assert sizes.min() >= 1


def test_full_size_shares_are_even_and_weights_shift_them():
    total = 26240                                                     # about config 3: 104 745 tokens, 4 KV heads
    sizes, used = check_partition(total, 1024, 4, 4)
    assert used == 1024 and sizes.sum() == total and sizes.max() - sizes.min() <= 1
    light, _ = check_partition(total, 1024, 4, 4, odd=232)
    wg = light.reshape(256, 4).sum(axis=1)
    assert wg[1::2].mean() < wg[0::2].mean()                          # odd work-groups (odd XCDs) got less
    assert abs(wg[1::2].mean() / wg[0::2].mean() - 232 / 256) < 0.01


def test_invalid_arguments_are_refused():
    for args in [(-1, 8, 4, 4), (10, 0, 4, 4), (10, 6, 4, 4), (10, 8, 5, 4), (10, 8, 4, 0)]:
        with pytest.raises(B.OdmaError):
            B.odma_stream_plan_ranges(*args)
    with pytest.raises(B.OdmaError):
        B.odma_stream_plan_ranges(10, 8, 4, 4, 100, 256)

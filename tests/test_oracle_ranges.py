"""Pins of the oracle's range bookkeeping across steps (Sec. 4.1, Eq. 9-11): the append rule of
Eq. 10 against a from-scratch segmentation of the whole token stream, and its composition with the
remapping of Eq. 11."""
import numpy as np
import pytest

import oracle


def scratch_offsets(starts_flag):
    """Offsets of the sentences of a token stream given per-token 'starts a sentence' flags
    (token 0 always starts one): the plain definition, nothing incremental."""
    f = np.asarray(starts_flag, dtype=bool).copy()
    if f.size:
        f[0] = True
    return np.concatenate([np.flatnonzero(f), [f.size]]).astype(np.int64)


def test_no_start_only_moves_the_end():
    off = np.array([0, 4, 9, 15])
    np.testing.assert_array_equal(oracle.append_ranges(off, 6, []), [0, 4, 9, 21])


def test_start_at_zero_closes_the_last_sentence():
    off = np.array([0, 4, 9, 15])
    np.testing.assert_array_equal(oracle.append_ranges(off, 6, [0]), [0, 4, 9, 15, 21])
    np.testing.assert_array_equal(oracle.append_ranges(off, 6, [0, 2]), [0, 4, 9, 15, 17, 21])
    np.testing.assert_array_equal(oracle.append_ranges(off, 6, [2]), [0, 4, 9, 17, 21])


def test_empty_cache_opens_the_first_sentence():
    np.testing.assert_array_equal(oracle.append_ranges(np.array([0]), 5, []), [0, 5])
    np.testing.assert_array_equal(oracle.append_ranges(np.array([0]), 5, [0, 3]), [0, 3, 5])
    np.testing.assert_array_equal(oracle.append_ranges(np.array([0]), 5, [3]), [0, 3, 5])


@pytest.mark.parametrize("seed", range(8))
def test_incremental_appends_equal_from_scratch_segmentation(seed):
    rng = np.random.default_rng(seed)
    m = int(rng.integers(1, 400))
    flags = rng.random(m) < 0.15
    want = scratch_offsets(flags)
    off = np.array([0], dtype=np.int64)
    pos = 0
    while pos < m:
        n = int(rng.integers(1, 40))
        n = min(n, m - pos)
        starts = np.flatnonzero(flags[pos:pos + n])
        off = oracle.append_ranges(off, n, starts)
        pos += n
        np.testing.assert_array_equal(off, scratch_offsets(flags[:pos]))
    np.testing.assert_array_equal(off, want)


def test_append_after_eviction_keeps_surviving_ranges_and_shifts_new_ones():
    # Eq. 11 then Eq. 10: sentences 1 and 3 of five are evicted, then 7 tokens arrive, the third
    # of which starts a sentence.  Surviving ranges keep their lengths, the new ones follow.
    off = np.array([0, 5, 8, 14, 16, 20])
    kept = np.concatenate([np.arange(0, 5), np.arange(8, 14), np.arange(16, 20)])
    ranges = oracle.remap_ranges(off, kept)
    new_off = np.array([b for b, _ in ranges] + [ranges[-1][1] + 1])
    np.testing.assert_array_equal(new_off, [0, 5, 11, 15])
    np.testing.assert_array_equal(oracle.append_ranges(new_off, 7, [2]), [0, 5, 11, 17, 22])

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


def test_sentence_numbers_follow_the_surviving_ranges():
    # pins: (1) as many numbers as Eq. 11 leaves ranges, for sentence-level and token-level evictions;
    # (2) a worked case with a sentence that straddles the protected window: its candidate part goes,
    # its tail stays, so its number stays; (3) composition over two evictions equals one lookup.
    rng = np.random.default_rng(8)
    for trial in range(30):
        n_sent = int(rng.integers(1, 30))
        off = np.concatenate([[0], np.cumsum(rng.integers(1, 9, size=n_sent))])
        score = rng.standard_normal(int(off[-1]))
        budget, protect = int(rng.integers(4, off[-1] + 3)), int(rng.integers(0, 5))
        if budget < protect:
            budget = protect
        tok = oracle.select_tokens(score, off, budget, protect)
        ids = oracle.surviving_sentence_ids(off, tok["kept_idx"])
        assert len(ids) == len(tok["new_off"]) - 1 == len(oracle.remap_ranges(off, tok["kept_idx"]))
        assert list(ids) == sorted(set(ids)) and all(0 <= i < n_sent for i in ids)
        imp = rng.random(int(off[-1]))
        lam = rng.uniform(-1, 1, n_sent)
        sc, candlen = oracle.sentence_scores(imp, lam, off, protect)
        sel = oracle.select_sentences(sc, candlen, off, budget, protect)
        ids_s = oracle.surviving_sentence_ids(off, sel["kept_idx"])
        assert len(ids_s) == len(sel["new_off"]) - 1
        # the lengths of the surviving sentences are the kept tokens inside each
        kept = set(int(t) for t in sel["kept_idx"])
        want_len = [sum(t in kept for t in range(off[s], off[s + 1])) for s in ids_s]
        np.testing.assert_array_equal(np.diff(sel["new_off"]), want_len)
    off = np.array([0, 4, 9, 12, 20])           # 20 tokens, window = last 10: sentence 2 = [9, 12) straddles position 10
    kept = np.concatenate([np.arange(0, 4), np.arange(10, 20)])   # sentence 1 evicted, candidate part of sentence 2 evicted
    np.testing.assert_array_equal(oracle.surviving_sentence_ids(off, kept), [0, 2, 3])
    np.testing.assert_array_equal(oracle.surviving_sentence_ids(off, kept, ids=[5, 7, 8, 11]), [5, 8, 11])
    np.testing.assert_array_equal(oracle.append_sentence_ids([5, 8, 11], 2), [5, 8, 11, 12, 13])
    np.testing.assert_array_equal(oracle.append_sentence_ids([], 3), [0, 1, 2])
    first = oracle.surviving_sentence_ids(off, kept)
    off2 = np.array([0, 4, 6, 14])               # the compacted ranges of the three survivors
    second = oracle.surviving_sentence_ids(off2, np.arange(4, 14), ids=first)
    np.testing.assert_array_equal(second, [2, 3])

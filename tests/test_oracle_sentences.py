"""Pins for sentence pooling, redundancy and the fused sentence score
(Sec. 4.1 Eq.1-3 and Eq.6)."""
import numpy as np
import pytest
from sklearn.metrics.pairwise import cosine_similarity

from oracle import sentence_embeddings, sentence_redundancy, sentence_scores


def _rand(shape, seed):
    return np.random.default_rng(seed).standard_normal(shape)


# ---------------------------------------------------------------- pooling (Eq.2)
def test_length_one_sentences_return_the_rows():
    k = _rand((17, 32), 1)
    np.testing.assert_array_equal(sentence_embeddings(k, np.arange(18)), k)


def test_equal_length_sentences_are_reshape_mean():
    k = _rand((60, 16), 2)
    ref = k.reshape(12, 5, 16).mean(axis=1)
    np.testing.assert_allclose(sentence_embeddings(k, np.arange(0, 61, 5)), ref, rtol=1e-14)


def test_ragged_pooling_matches_segment_sum_over_length():
    k = _rand((40, 8), 3)
    off = np.array([0, 3, 4, 11, 30, 40])
    ref = np.add.reduceat(k, off[:-1], axis=0) / np.diff(off)[:, None]
    np.testing.assert_allclose(sentence_embeddings(k, off), ref, rtol=1e-13)


# ---------------------------------------------------------------- redundancy (Eq.1, Eq.3)
def test_redundancy_is_max_cosine_over_later_sentences():
    v = _rand((25, 64), 4)
    g = cosine_similarity(v)                      # library normalised Gram matrix
    ref = np.array([g[s, s + 1:].max() if s < 24 else -np.inf for s in range(25)])
    np.testing.assert_allclose(sentence_redundancy(v), ref, rtol=1e-11)


def test_exact_duplicate_scores_maximal_redundancy():
    v = _rand((10, 128), 5)
    v[7] = v[2]
    lam = sentence_redundancy(v)
    assert abs(lam[2] - 1.0) < 1e-12
    # only the EARLIER sentence of the pair is flagged by that pair
    assert lam[7] < 0.9
    assert lam[-1] == -np.inf


def test_orthogonal_sentences_have_zero_redundancy():
    lam = sentence_redundancy(np.eye(6)[:, :6] * np.arange(1, 7)[:, None])
    np.testing.assert_array_equal(lam[:-1], 0.0)


def test_redundancy_invariant_under_positive_rescaling():
    v = _rand((12, 32), 6)
    scale = np.random.default_rng(7).uniform(0.1, 50.0, size=12)
    np.testing.assert_allclose(sentence_redundancy(v * scale[:, None]), sentence_redundancy(v), rtol=1e-11)


def test_zero_embedding_is_never_redundant():
    v = _rand((5, 16), 8)
    v[1] = 0.0
    lam = sentence_redundancy(v)
    assert lam[1] == 0.0 and np.all(np.isfinite(lam[:-1]))


def test_planted_copy_has_the_expected_cosine():
    # keys N(0,1), copy = source + 0.05 N(0,1): cos ~ 1/sqrt(1 + 0.05^2) = 0.99875,
    # unrelated sentences ~ N(0, 1/128).
    rng = np.random.default_rng(9)
    k = rng.standard_normal((2000, 128))
    off = np.arange(0, 2001, 20)
    k[off[60]:off[61]] = k[off[10]:off[11]] + 0.05 * rng.standard_normal((20, 128))
    lam = sentence_redundancy(sentence_embeddings(k, off))
    assert lam[10] == pytest.approx(1 / np.sqrt(1.0025), abs(3e-4))
    others = np.delete(lam[:-1], 10)
    assert others.max() < 0.6


# ---------------------------------------------------------------- fused score (Eq.6)
def test_redundant_sentences_rank_below_all_others():
    # sigma * I <= sigma = 0.1 < tau, so a penalised sentence is negative, others >= 0:
    # redundant sentences are evicted before any importance-based eviction.
    rng = np.random.default_rng(10)
    off = np.concatenate([[0], np.cumsum(rng.integers(1, 9, size=30))])
    imp = rng.uniform(0, 1, size=off[-1])
    lam = rng.uniform(0.5, 1.0, size=30)
    score, _ = sentence_scores(imp, lam, off, protect=0, sigma=0.1, tau=0.95)
    pen = lam > 0.95
    assert pen.any() and (~pen).any()
    assert score[pen].max() < 0 <= score[~pen].min()


def test_score_terms_and_threshold_are_strict():
    off = np.array([0, 2, 4, 6])
    imp = np.array([0.2, 0.4, 0.1, 0.1, 0.6, 0.0])
    red = np.array([0.5, 0.5, 0.0, 1.0, 0.0, 0.0])
    lam = np.array([0.95, 0.96, -np.inf])          # 0.95 is NOT > tau
    score, candlen = sentence_scores(imp, lam, off, protect=0, sigma=0.25, tau=0.95, red=red)
    np.testing.assert_allclose(score, [0.25 * 0.3 - 0.75 * 0.5, 0.25 * 0.1 - 0.75 * 0.5 - 0.96, 0.25 * 0.3])
    np.testing.assert_array_equal(candlen, [2, 2, 2])


def test_protected_window_clips_the_straddling_sentence():
    off = np.array([0, 4, 10, 14])                 # N = 14, window 6 -> p = 8
    imp = np.arange(14, dtype=float)
    lam = np.full(3, -np.inf)
    score, candlen = sentence_scores(imp, lam, off, protect=6, sigma=1.0, tau=0.95)
    np.testing.assert_array_equal(candlen, [4, 4, 0])     # sentence 1 contributes tokens 4..7 only
    assert score[0] == pytest.approx(1.5) and score[1] == pytest.approx(5.5)
    assert score[2] == np.inf


def test_window_larger_than_cache_leaves_no_candidates():
    off = np.array([0, 3, 5])
    score, candlen = sentence_scores(np.ones(5), np.zeros(2), off, protect=9)
    assert np.all(np.isinf(score)) and candlen.sum() == 0

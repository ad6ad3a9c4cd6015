"""Pins of the oracle's token-level scores and selection (Eq.6 as printed and the eviction rule
after it; ranges after eviction: Eq.11)."""
import itertools

import numpy as np
import pytest

import oracle


def test_token_scores_hand_example():
    # three sentences of lengths 2, 3, 1; only the second is in the redundant set (0.97 > 0.95)
    off = [0, 2, 5, 6]
    imp = np.array([0.5, 0.1, 0.2, 0.3, 0.4, 0.6])
    red = np.array([0.1, 0.2, 0.3, 0.1, 0.2, 0.3])
    lam = np.array([0.90, 0.97, -np.inf])
    got = oracle.token_scores(imp, red, lam, off, sigma=0.1, tau=0.95)
    want = [0.05 - 0.09, 0.01 - 0.18, 0.02 - 0.27 - 0.97, 0.03 - 0.09 - 0.97, 0.04 - 0.18 - 0.97, 0.06 - 0.27]
    np.testing.assert_allclose(got, want, rtol=1e-12)
    # without R, and with a threshold nothing passes
    np.testing.assert_allclose(oracle.token_scores(imp, None, lam, off, 0.5, 0.99), 0.5 * imp, rtol=1e-12)
    # every token of a redundant sentence scores below every token of the others when I, R <= 1 (order-of-magnitude remark after Eq.6)
    assert got[2:5].max() < min(got[:2].min(), got[5])


def _brute_best(score, n_tok, budget, protect):
    """Exhaustive: among all subsets of the unprotected tokens of size `room`, the kept set is the
    one that is upward closed in the order (score desc, index desc) - it is unique."""
    p = n_tok - min(protect, n_tok)
    room = budget - (n_tok - p)
    rank = sorted(range(p), key=lambda t: (-score[t], -t))
    pos = {t: i for i, t in enumerate(rank)}
    best = None
    for sub in itertools.combinations(range(p), room):
        if all(pos[t] < room for t in sub):  # upward closed <=> its members are the `room` best
            assert best is None
            best = set(sub)
    return best


@pytest.mark.parametrize("seed", range(6))
def test_select_tokens_matches_exhaustive_search(seed):
    rng = np.random.default_rng(seed)
    n_tok, protect = 11, 3
    budget = int(rng.integers(protect, n_tok))
    score = rng.choice([0.0, 0.5, -0.5, 1.0], size=n_tok)  # many ties: the later token wins
    off = [0, 4, 5, 9, 11]
    got = oracle.select_tokens(score, off, budget, protect)
    best = _brute_best(score, n_tok, budget, protect)
    assert set(got["kept_idx"].tolist()) == best | set(range(n_tok - protect, n_tok))
    assert got["new_len"] == budget == int(got["keep"].sum())


def test_select_tokens_invariants_and_ranges():
    rng = np.random.default_rng(9)
    lens = rng.integers(1, 9, size=40)
    off = np.concatenate([[0], np.cumsum(lens)])
    n_tok = int(off[-1])
    score = rng.standard_normal(n_tok)
    for budget, protect in [(n_tok + 5, 8), (n_tok, 8), (n_tok - 1, 8), (60, 16), (16, 16), (40, 0)]:
        got = oracle.select_tokens(score, off, budget, protect)
        kept = got["kept_idx"]
        assert (np.diff(kept) > 0).all()
        assert got["new_len"] == min(n_tok, budget)
        assert set(range(n_tok - min(protect, n_tok), n_tok)) <= set(kept.tolist())
        if n_tok > budget:  # every evicted unprotected token ranks below every kept one
            p = n_tok - protect
            kept_u = [t for t in kept if t < p]
            gone = [t for t in range(p) if t not in set(kept_u)]
            if kept_u and gone:
                assert min((score[t], t) for t in kept_u) > max((score[t], t) for t in gone)
        # ranges after eviction agree with the remapping rule of Eq.11, written for inclusive ranges
        ranges = oracle.remap_ranges(off, kept)
        new_off = got["new_off"]
        assert len(ranges) == len(new_off) - 1
        for (b, e), lo, hi in zip(ranges, new_off[:-1], new_off[1:]):
            assert (b, e) == (lo, hi - 1)


def test_select_tokens_equals_library_partition_when_scores_are_distinct():
    rng = np.random.default_rng(4)
    n_tok, protect, budget = 500, 32, 200
    score = rng.permutation(n_tok).astype(np.float64)  # distinct
    got = oracle.select_tokens(score, [0, n_tok], budget, protect)
    p = n_tok - protect
    top = np.argpartition(-score[:p], budget - protect - 1)[:budget - protect]
    want = np.sort(np.concatenate([top, np.arange(p, n_tok)]))
    np.testing.assert_array_equal(got["kept_idx"], want)

"""Pins for budgeted whole-sentence selection, the surviving index set, the range remap
(Eq.11) and compaction (Alg.1 eviction line)."""
import itertools

import numpy as np
import pytest

from oracle import compact, compress_head, remap_ranges, select_sentences, sentence_scores


def _random_case(rng, n_sent, max_len=6):
    off = np.concatenate([[0], np.cumsum(rng.integers(1, max_len + 1, size=n_sent))])
    n_tok = int(off[-1])
    protect = int(rng.integers(0, max(1, n_tok // 3)))
    budget = int(rng.integers(protect, n_tok + 3))
    # coarse scores so that exact ties are common and the tie rule is exercised
    imp = rng.integers(0, 4, size=n_tok).astype(float)
    lam = np.where(rng.random(n_sent) < 0.3, 0.97, 0.1)
    score, candlen = sentence_scores(imp, lam, off, protect, sigma=0.1, tau=0.95)
    return off, n_tok, protect, budget, score, candlen


def _brute_force(off, n_tok, protect, budget, score, candlen):
    """Definition-level answer: among all subsets of candidate sentences that fit the
    room left by the protected window AND are upward-closed in the total order
    (score desc, index desc), the one with most sentences.  It is unique."""
    n_sent = len(off) - 1
    if n_tok <= budget:
        return np.ones(n_sent, dtype=bool)
    p = n_tok - min(protect, n_tok)
    cands = [s for s in range(n_sent) if off[s] < p]
    room = budget - (n_tok - p)

    def ranks_above(a, b):  # a is evicted later than b
        return (score[a], a) > (score[b], b)

    best = None
    for r in range(len(cands) + 1):
        for sub in itertools.combinations(cands, r):
            ss = set(sub)
            if sum(candlen[s] for s in sub) > room:
                continue
            if any(ranks_above(o, s) for s in ss for o in cands if o not in ss):
                continue
            if best is None or len(ss) > len(best):
                best = ss
    keep = np.ones(n_sent, dtype=bool)
    for s in cands:
        keep[s] = s in best
    return keep


@pytest.mark.parametrize("seed", range(40))
def test_selection_equals_brute_force(seed):
    rng = np.random.default_rng(seed)
    case = _random_case(rng, int(rng.integers(1, 12)))
    off, n_tok, protect, budget, score, candlen = case
    got = select_sentences(score, candlen, off, budget, protect)
    np.testing.assert_array_equal(got["keep"], _brute_force(*case))


@pytest.mark.parametrize("seed", range(60))
def test_selection_invariants(seed):
    rng = np.random.default_rng(1000 + seed)
    off, n_tok, protect, budget, score, candlen = _random_case(rng, int(rng.integers(1, 60)), 12)
    sel = select_sentences(score, candlen, off, budget, protect)
    kept, keep = sel["kept_idx"], sel["keep"]
    p = n_tok - min(protect, n_tok)
    # strictly ascending, in range
    assert np.all(np.diff(kept) > 0)
    assert kept.size == 0 or (kept[0] >= 0 and kept[-1] < n_tok)
    assert sel["new_len"] == kept.size
    # budget respected, or nothing evicted when the cache already fits
    if n_tok <= budget:
        np.testing.assert_array_equal(kept, np.arange(n_tok))
    else:
        assert kept.size <= budget
    # protected window always kept
    assert set(range(p, n_tok)) <= set(kept.tolist())
    # whole sentences: the unprotected part of each sentence is all-in or all-out
    ks = set(kept.tolist())
    for s in range(len(off) - 1):
        span = range(int(off[s]), min(int(off[s + 1]), p))
        inside = [t in ks for t in span]
        assert all(inside) or not any(inside)
        if len(span):
            assert all(inside) == bool(keep[s])
    # maximality: the best-ranked evicted sentence would overflow the budget
    if n_tok > budget:
        ev = [s for s in range(len(off) - 1) if off[s] < p and not keep[s]]
        if ev:
            top = max(ev, key=lambda s: (score[s], s))
            assert kept.size + candlen[top] > budget
            # and everything kept outranks everything evicted
            kp = [s for s in range(len(off) - 1) if off[s] < p and keep[s]]
            if kp:
                low = min(kp, key=lambda s: (score[s], s))
                assert (score[low], low) > (score[top], top)


def test_tie_keeps_the_later_sentence():
    off = np.array([0, 2, 4, 6, 8])
    score = np.array([1.0, 1.0, 1.0, 1.0])
    candlen = np.array([2, 2, 2, 2])
    sel = select_sentences(score, candlen, off, budget=4, protect=0)
    np.testing.assert_array_equal(sel["keep"], [False, False, True, True])
    np.testing.assert_array_equal(sel["kept_idx"], [4, 5, 6, 7])


def test_no_skip_and_fill():
    # ranks: s0 (3 tokens) > s1 (4 tokens) > s2 (1 token); room 4: keep s0 only.
    off = np.array([0, 3, 7, 8])
    sel = select_sentences(np.array([3.0, 2.0, 1.0]), np.array([3, 4, 1]), off, budget=4, protect=0)
    np.testing.assert_array_equal(sel["keep"], [True, False, False])


def test_new_offsets_follow_the_range_remap():
    # Eq.11 with searchsorted as an independent closed form, on inclusive ranges
    rng = np.random.default_rng(7)
    for _ in range(30):
        off, n_tok, protect, budget, score, candlen = _random_case(rng, int(rng.integers(2, 30)), 9)
        sel = select_sentences(score, candlen, off, budget, protect)
        kept = sel["kept_idx"]
        ref = []
        for s in range(len(off) - 1):
            b = np.searchsorted(kept, off[s], "left")
            e = np.searchsorted(kept, off[s + 1] - 1, "right") - 1
            if b <= e:
                ref.append((int(b), int(e)))
        assert remap_ranges(off, kept) == ref
        new_off = sel["new_off"]
        assert [(int(new_off[i]), int(new_off[i + 1]) - 1) for i in range(len(new_off) - 1)] == ref
        assert new_off[-1] == sel["new_len"]


def test_compact_is_library_gather_and_identity():
    rng = np.random.default_rng(8)
    k, v = rng.standard_normal((30, 8)), rng.standard_normal((30, 8))
    idx = np.array([0, 1, 5, 6, 7, 20, 29])
    k2, v2 = compact(k, v, idx)
    np.testing.assert_array_equal(k2, np.take(k, idx, axis=0))
    np.testing.assert_array_equal(v2, np.take(v, idx, axis=0))
    k3, v3 = compact(k, v, np.arange(30))
    np.testing.assert_array_equal(k3, k)
    np.testing.assert_array_equal(v3, v)


def test_whole_step_on_a_planted_duplicate():
    # the source of a later exact copy is evicted first; the copy is not penalised by it
    rng = np.random.default_rng(9)
    n_tok, d = 160, 32
    off = np.arange(0, n_tok + 1, 8)
    k = rng.standard_normal((n_tok, d))
    v = rng.standard_normal((n_tok, d))
    k[off[12]:off[13]] = k[off[3]:off[4]]
    q = rng.standard_normal((2, 4, d))
    out = compress_head(q, k, v, off, budget=n_tok - 8, protect=16)
    assert out["lam"][3] == pytest.approx(1.0, abs=1e-11) and out["score"][3] < 0
    assert not out["keep"][3] and out["keep"][12]
    assert out["new_len"] == n_tok - 8
    np.testing.assert_array_equal(out["k"], k[out["kept_idx"]])
    np.testing.assert_array_equal(out["v"], v[out["kept_idx"]])

"""Pins for the oracle's token-importance step (Sec. 4.1 "Token Importance Score", Eq.4).

Each pin is something other than the oracle's own formula: a library routine, a closed
form, a pure-Python brute force, or an invariant that a dropped term / wrong axis /
wrong group mapping would break.
"""
import math

import numpy as np
import pytest
import scipy.special
import torch

from oracle import token_importance


def _rand(shape, seed):
    return np.random.default_rng(seed).standard_normal(shape)


def test_single_head_single_query_is_library_softmax():
    # n = 1, alpha = 1: I is just softmax(q K^T / sqrt(D)) over all keys.
    q, k = _rand((1, 1, 128), 1), _rand((300, 128), 2)
    ref = scipy.special.softmax(k @ q[0, 0] / math.sqrt(128))
    np.testing.assert_allclose(token_importance(q, k), ref, rtol=1e-12, atol=0)


def test_matches_library_attention_with_gqa_and_causal_mask():
    # torch's scaled_dot_product_attention with V = identity returns the attention
    # probabilities; enable_gqa maps query head i to KV head i // n, which is the
    # 0-based reading of g(i); the boolean mask is the causal part of M.
    n, hk, alpha, n_tok, d = 4, 2, 8, 96, 128
    q = torch.from_numpy(_rand((hk * n, alpha, d), 3))
    k = torch.from_numpy(_rand((hk, n_tok, d), 4))
    eye = torch.eye(n_tok, dtype=torch.float64).expand(hk, n_tok, n_tok)
    pos = n_tok - alpha + torch.arange(alpha)
    mask = torch.arange(n_tok)[None, :] <= pos[:, None]
    probs = torch.nn.functional.scaled_dot_product_attention(
        q[None], k[None], eye[None], attn_mask=mask, enable_gqa=True)[0]   # [Hq, alpha, N]
    for h in range(hk):
        ref = probs[h * n:(h + 1) * n].max(dim=0).values.mean(dim=0).numpy()
        got = token_importance(q[h * n:(h + 1) * n].numpy(), k[h].numpy())
        np.testing.assert_allclose(got, ref, rtol=1e-10, atol=1e-15)


def test_zero_queries_closed_form():
    # Q = 0: every visible key gets 1/(number visible); query a sees N-alpha+a+1 keys.
    n, alpha, n_tok = 3, 5, 40
    got = token_importance(np.zeros((n, alpha, 16)), _rand((n_tok, 16), 5))
    ref = np.zeros(n_tok)
    for t in range(n_tok):
        for a in range(alpha):
            if t <= n_tok - alpha + a:
                ref[t] += 1.0 / (n_tok - alpha + a + 1)
    np.testing.assert_allclose(got, ref / alpha, rtol=1e-13)


def test_identical_keys_give_uniform_rows():
    n, alpha, n_tok = 2, 4, 30
    k = np.tile(_rand((1, 32), 6), (n_tok, 1))
    got = token_importance(_rand((n, alpha, 32), 7), k)
    ref = np.zeros(n_tok)
    for a in range(alpha):
        vis = n_tok - alpha + a + 1
        ref[:vis] += 1.0 / vis
    np.testing.assert_allclose(got, ref / alpha, rtol=1e-12)


def test_mass_between_one_and_group_size():
    # each (head, query) row sums to 1; the max over n heads sums to something in [1, n];
    # exactly 1 when all heads of the group carry the same queries.
    n, alpha = 4, 8
    q, k = _rand((n, alpha, 64), 8), _rand((200, 64), 9)
    total = token_importance(q, k).sum()
    assert 1.0 - 1e-12 <= total <= n + 1e-12
    assert total > 1.05  # independent heads do disagree
    same = np.repeat(q[:1], n, axis=0)
    assert abs(token_importance(same, k).sum() - 1.0) < 1e-12


def test_brute_force_scalar_loops():
    n, alpha, n_tok, d = 2, 3, 11, 8
    q, k = _rand((n, alpha, d), 10), _rand((n_tok, d), 11)
    ref = [0.0] * n_tok
    for a in range(alpha):
        last = n_tok - alpha + a
        rows = []
        for i in range(n):
            lg = [sum(q[i, a, c] * k[t, c] for c in range(d)) / math.sqrt(d) for t in range(last + 1)]
            z = sum(math.exp(x) for x in lg)
            rows.append([math.exp(x) / z for x in lg])
        for t in range(last + 1):
            ref[t] += max(r[t] for r in rows) / alpha
    np.testing.assert_allclose(token_importance(q, k), ref, rtol=1e-12)


def test_causal_mask_hides_later_window_keys():
    # the key at the last position is visible to the last window query only
    n, alpha, n_tok = 1, 4, 20
    q, k = _rand((n, alpha, 16), 12), _rand((n_tok, 16), 13)
    imp = token_importance(q, k)
    lg = k @ q[0, alpha - 1] / 4.0
    assert imp[-1] == pytest.approx(scipy.special.softmax(lg)[-1] / alpha, rel=1e-12)


def test_group_mapping_is_per_kv_head_not_strided():
    # importance of a KV head must not change when OTHER groups' queries change
    q, k = _rand((2, 4, 32), 14), _rand((50, 32), 15)
    base = token_importance(q, k)
    np.testing.assert_array_equal(base, token_importance(q.copy(), k))
    # and max-pool (not mean, not sum) over the group: adding a head can only raise I
    more = np.concatenate([q, _rand((1, 4, 32), 16)], axis=0)
    assert np.all(token_importance(more, k) >= base - 1e-15)


def test_short_cache_rows_without_keys_contribute_zero():
    # N < alpha: the first alpha-N window queries precede the cache
    q, k = _rand((2, 6, 8), 17), _rand((4, 8), 18)
    imp = token_importance(q, k)
    assert imp.shape == (4,)
    # visible rows: a = 2..5 see 1..4 keys; each contributes a max over heads that sums >= 1
    assert 4.0 / 6 - 1e-12 <= imp.sum() <= 2 * 4.0 / 6 + 1e-12

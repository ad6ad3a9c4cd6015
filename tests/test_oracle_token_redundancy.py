"""Pins of the oracle's token redundancy (Sec. 4.1 "Token Redundancy Score", Eq.5) against what
the mathematics fixes: closed forms on structured keys, brute force with plain loops, invariants."""
import math

import numpy as np
import pytest

import oracle


def _brute(k, eps=1e-12):
    """Eq.5 with plain Python loops (tiny inputs only)."""
    n, d = len(k), len(k[0])
    unit = []
    for row in k:
        norm = math.sqrt(sum(x * x for x in row)) + eps
        unit.append([x / norm for x in row])
    red = [0.0] * n
    for i in range(n):
        logits = [sum(unit[i][c] * unit[j][c] for c in range(d)) for j in range(n)]
        z = sum(math.exp(x) for x in logits)
        for j in range(n):
            red[j] += math.exp(logits[j]) / z / n
    return np.array(red)


def test_identical_keys_share_the_mass_equally():
    k = np.tile(np.array([[0.3, -1.2, 2.0, 0.7]]), (9, 1)) * np.arange(1, 10)[:, None]  # same direction, any length
    np.testing.assert_allclose(oracle.token_redundancy(k), np.full(9, 1 / 9), rtol=1e-12)


def test_two_orthogonal_clusters_closed_form():
    # m copies of direction a, N-m copies of direction b, a orthogonal to b: cosines are 1 inside a
    # cluster and 0 across.  A row of cluster A gives e/(m e + N - m) to each member of A and
    # 1/(m e + N - m) to each member of B; likewise for rows of B.
    m, n = 3, 10
    a = np.zeros(8); a[0] = 2.5
    b = np.zeros(8); b[5] = -0.4
    k = np.stack([a] * m + [b] * (n - m))
    za, zb = m * math.e + (n - m), (n - m) * math.e + m
    r_a = (m * math.e / za + (n - m) * 1.0 / zb) / n
    r_b = (m * 1.0 / za + (n - m) * math.e / zb) / n
    got = oracle.token_redundancy(k)
    np.testing.assert_allclose(got[:m], r_a, rtol=1e-10)  # eps = 1e-12 in the norm moves the cosines by ~1e-12
    np.testing.assert_allclose(got[m:], r_b, rtol=1e-10)
    assert r_b > r_a  # the larger cluster is the more redundant one


def test_antipodal_pair_and_single_token():
    np.testing.assert_allclose(oracle.token_redundancy(np.array([[1.0, 2.0]])), [1.0])
    k = np.array([[1.0, 0.0], [-3.0, 0.0], [0.0, 2.0]])
    # cosines: (0,1) = -1, (0,2) = 0, (1,2) = 0
    e, ei = math.e, 1 / math.e
    rows = np.array([[e, ei, 1.0], [ei, e, 1.0], [1.0, 1.0, e]])
    want = (rows / rows.sum(axis=1, keepdims=True)).mean(axis=0)
    np.testing.assert_allclose(oracle.token_redundancy(k), want, rtol=1e-12)


@pytest.mark.parametrize("seed,n,d", [(0, 5, 3), (1, 12, 7), (2, 17, 128)])
def test_matches_brute_force_loops(seed, n, d):
    k = np.random.default_rng(seed).standard_normal((n, d))
    np.testing.assert_allclose(oracle.token_redundancy(k), _brute(k.tolist()), rtol=1e-11)


def test_invariants_sum_scaling_permutation_and_duplicates():
    rng = np.random.default_rng(7)
    k = rng.standard_normal((40, 16))
    r = oracle.token_redundancy(k)
    assert abs(r.sum() - 1.0) < 1e-12 and (r > 0).all()
    # positive rescaling of any key leaves R unchanged (cosines)
    np.testing.assert_allclose(oracle.token_redundancy(k * rng.uniform(0.1, 9.0, size=(40, 1))), r, rtol=1e-10)
    # relabelling the tokens relabels R
    perm = rng.permutation(40)
    np.testing.assert_allclose(oracle.token_redundancy(k[perm]), r[perm], rtol=1e-12)
    # a key that has exact copies collects more mass than it did alone, and the copies tie
    k2 = np.concatenate([k, k[:1], k[:1]])
    r2 = oracle.token_redundancy(k2)
    np.testing.assert_allclose(r2[[0, 40, 41]], r2[0], rtol=1e-12)
    assert r2[0] * 42 > r[0] * 40


def test_zero_key_is_orthogonal_to_everything():
    k = np.array([[0.0, 0.0], [1.0, 0.0], [0.0, 1.0]])
    rows = np.array([[1.0, 1.0, 1.0], [1.0, math.e, 1.0], [1.0, 1.0, math.e]])  # zero row: all cosines 0
    want = (rows / rows.sum(axis=1, keepdims=True)).mean(axis=0)
    np.testing.assert_allclose(oracle.token_redundancy(k), want, rtol=1e-12)

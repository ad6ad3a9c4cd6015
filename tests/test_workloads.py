"""The synthetic workloads have the stated shapes and statistics, and the oracle's whole
step on the tiny config obeys the invariants of the method."""
import numpy as np
import pytest

from oracle import compress_head
from paper_2512_07993_amd import workloads as W


@pytest.mark.parametrize("cid", [1, 2, 3, 4, 5])
def test_structure_statistics(cid):
    cfg = W.CONFIGS[cid]
    st = W.make_structure(cfg)
    assert st.seq_len.min() >= cfg.len_lo and st.seq_len.max() <= cfg.len_hi
    assert st.seq_off[-1] == st.seq_len.sum()
    lens = []
    for b in range(cfg.batch):
        off = st.offsets(b)
        assert off[0] == 0 and off[-1] == st.seq_len[b] and np.all(np.diff(off) >= 1)
        lens.append(np.diff(off)[:-1])
        src = st.dup_src[b]
        assert np.all(src < np.arange(len(src)))
    lens = np.concatenate(lens)
    assert lens.min() >= cfg.sent_min and lens.max() <= cfg.sent_max
    assert abs(lens.mean() - cfg.sent_mean) < 0.12 * cfg.sent_mean
    frac = np.concatenate([s >= 0 for s in st.dup_src]).mean()
    assert abs(frac - cfg.dup_frac) < 0.05
    # same seed, same structure
    st2 = W.make_structure(cfg)
    np.testing.assert_array_equal(st.sent_off, st2.sent_off)


def test_tiny_config_whole_step_invariants():
    cfg = W.CONFIGS[1]
    st = W.make_structure(cfg)
    k, v, q = W.fill_cache(cfg, st)
    assert k.shape == (1, 8, 1152, 128) and q.shape == (1, 1, 32, 8, 128)
    n_dup = int((st.dup_src[0] >= 0).sum())
    for h in range(cfg.n_kv_heads):
        qq, kk, vv, off = W.head_arrays(cfg, st, k, v, q, 0, h, 0)
        out = compress_head(qq, kk, vv, off, cfg.budget, cfg.protect_window)
        assert out["new_len"] <= cfg.budget
        assert out["new_len"] > cfg.budget - cfg.sent_max
        kept = set(out["kept_idx"].tolist())
        assert set(range(1152 - 32, 1152)) <= kept
        # every source of a planted copy is flagged (cos ~ 0.9988 > tau); anything else
        # flagged is itself a copy with a later sibling copy of the same source
        flagged = out["lam"] > 0.95
        srcs = set(int(j) for j in st.dup_src[0] if j >= 0)
        copies = set(int(s) for s, j in enumerate(st.dup_src[0]) if j >= 0)
        got = set(np.nonzero(flagged)[0].tolist())
        assert srcs <= got <= (srcs | copies)
        assert len(srcs) <= n_dup
        # flagged sentences go first
        p = 1152 - 32
        cand = off[:-1] < p
        if (~out["keep"][cand]).sum() > flagged[cand].sum():
            assert not out["keep"][cand & flagged].any()
        np.testing.assert_array_equal(out["k"], kk[out["kept_idx"]])

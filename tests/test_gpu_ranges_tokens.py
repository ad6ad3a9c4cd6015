"""The token-level flow on per-head ranges through the C ABI (Sec. 4.1: token redundancy Eq. 5,
token scores Eq. 6 as printed, eviction, ranges per Eq. 11, repeated over two steps): where the
per-head description says the same as the shared one the results are those of the shared-range
calls bit for bit; after a first token-level step (heads differ, sentences have shrunk) the second
step is checked against the oracle head by head."""
import numpy as np
import pytest
import torch

import oracle
from paper_2512_07993_amd import binding as B
from paper_2512_07993_amd import workloads as W

from helpers import make_cache
from test_gpu_ranges import shared_as_ranges

pytestmark = pytest.mark.gpu


def _bytes(n):
    return torch.empty(n + 256, dtype=torch.uint8, device="cuda")


def _token_step(cfg, st, cache, q, budget, ranges=None):
    """token redundancy -> score -> token-level selection -> compaction; with `ranges` through the per-head calls."""
    L, H, Bn, S, T = cfg.n_layers, cfg.n_kv_heads, cfg.batch, st.total_sentences, st.total_tokens
    status = torch.zeros(1, dtype=torch.int32, device="cuda")
    params = B.Params(cfg.obs_window, cfg.protect_window, budget, dev_status=status)
    f32 = lambda *shape: torch.full(shape, float("nan"), dtype=torch.float32, device="cuda")
    red, imp, score, lam, tok_score = f32(L, H, T), f32(L, H, T), f32(L, H, S), f32(L, H, S), f32(L, H, T)
    kept_stride = max(1, min(budget, T))
    tok_keep = torch.full((L, H, T), 77, dtype=torch.uint8, device="cuda")
    kept_idx = torch.full((L, H, Bn, kept_stride), -1, dtype=torch.int32, device="cuda")
    new_len = torch.full((L, H, Bn), -1, dtype=torch.int32, device="cuda")
    new_off = torch.full((L, H, S + Bn), -1, dtype=torch.int32, device="cuda")
    new_cnt = torch.full((L, H, Bn), -1, dtype=torch.int32, device="cuda")
    if ranges is None:
        B.skipkv_token_redundancy(cache, red, _bytes(B.skipkv_redundancy_workspace_bytes(cache)))
        B.skipkv_score(cache, params, q, red, score, lam, imp, _bytes(B.skipkv_workspace_bytes(cache, params)))
        B.skipkv_select_tokens(cache, params, imp, red, lam, tok_score, tok_keep, kept_idx, new_len, new_off, new_cnt, kept_stride)
    else:
        ws = _bytes(B.skipkv_ranges_workspace_bytes(cache, params))
        B.skipkv_token_redundancy_ranges(cache, ranges, red, _bytes(B.skipkv_redundancy_workspace_bytes(cache)))
        B.skipkv_score_ranges(cache, ranges, params, q, red, score, lam, imp, ws)
        B.skipkv_select_tokens_ranges(cache, ranges, params, imp, red, lam, tok_score, tok_keep, kept_idx, new_len, new_off,
                                      new_cnt, kept_stride, ws)
    B.skipkv_compact(cache, kept_idx, new_len, kept_stride)
    torch.cuda.synchronize()
    assert int(status.item()) == 0
    return dict(red=red, imp=imp, score=score, lam=lam, tok_score=tok_score, tok_keep=tok_keep, kept_idx=kept_idx,
                new_len=new_len, new_off=new_off, new_cnt=new_cnt)


@pytest.mark.parametrize("config_id,kw", [
    (3, dict(n_layers=2, batch=3, len_lo=300, len_hi=1700, budget=512)),
    (1, dict()),
])
def test_per_head_calls_equal_the_shared_ones_on_the_same_cache(config_id, kw):
    cfg = W.CONFIGS[config_id].scaled(**kw) if kw else W.CONFIGS[config_id]
    st = W.make_structure(cfg)
    k0, v0, q = W.fill_cache(cfg, st, device="cuda")
    ka, va = k0.clone(), v0.clone()
    a = _token_step(cfg, st, make_cache(cfg, st, ka, va), q, cfg.budget)
    kb, vb = k0.clone(), v0.clone()
    b = _token_step(cfg, st, make_cache(cfg, st, kb, vb), q, cfg.budget, shared_as_ranges(cfg, st))
    for name in a:
        x, y = a[name], b[name]
        assert torch.equal(x.view(torch.uint8) if x.dtype != torch.uint8 else x, y.view(torch.uint8) if y.dtype != torch.uint8 else y), name
    nl = a["new_len"].cpu().numpy()
    for l in range(cfg.n_layers):
        for h in range(cfg.n_kv_heads):
            for s in range(cfg.batch):
                t0, n = int(st.seq_off[s]), int(nl[l, h, s])
                assert torch.equal(ka[l, h, t0:t0 + n], kb[l, h, t0:t0 + n]) and torch.equal(va[l, h, t0:t0 + n], vb[l, h, t0:t0 + n])


def test_second_token_level_step_on_per_head_ranges_matches_the_oracle():
    cfg = W.CONFIGS[3].scaled(n_layers=2, n_kv_heads=2, n_q_heads=8, batch=3, len_lo=700, len_hi=1900, budget=512)
    st = W.make_structure(cfg)
    k, v, q1 = W.fill_cache(cfg, st, device="cuda")
    cache = make_cache(cfg, st, k, v)
    s1 = _token_step(cfg, st, cache, q1, cfg.budget)
    L, H, Bn = cfg.n_layers, cfg.n_kv_heads, cfg.batch
    len1, cnt1, off1 = s1["new_len"].cpu().numpy(), s1["new_cnt"].cpu().numpy(), s1["new_off"].cpu().numpy()
    assert (len1 == np.minimum(cfg.budget, st.seq_len)[None, None, :]).all()
    assert len({tuple(off1[l, h]) for l in range(L) for h in range(H)}) > 1     # the heads' ranges really differ
    ranges = B.Ranges(s1["new_len"].clone(), s1["new_cnt"].clone(), s1["new_off"].clone())
    # per-head budgets for the second step, so that the heads' lengths differ afterwards too
    rng = np.random.default_rng(4)
    bud2 = rng.integers(cfg.protect_window + 40, cfg.budget // 2, size=(L, H, Bn)).astype(np.int32)
    g = torch.Generator(device="cuda")
    g.manual_seed(5)
    q2 = torch.randn(q1.shape, generator=g, device="cuda").to(q1.dtype)
    k_in, v_in = k.clone(), v.clone()
    status = torch.zeros(1, dtype=torch.int32, device="cuda")
    T, S = st.total_tokens, st.total_sentences
    params = B.Params(cfg.obs_window, cfg.protect_window, torch.from_numpy(bud2).cuda(), max_budget=int(bud2.max()), dev_status=status)
    f32 = lambda *shape: torch.full(shape, float("nan"), dtype=torch.float32, device="cuda")
    red, imp, score, lam, tok_score = f32(L, H, T), f32(L, H, T), f32(L, H, S), f32(L, H, S), f32(L, H, T)
    kept_stride = int(bud2.max())
    tok_keep = torch.full((L, H, T), 77, dtype=torch.uint8, device="cuda")
    kept_idx = torch.full((L, H, Bn, kept_stride), -1, dtype=torch.int32, device="cuda")
    new_len = torch.full((L, H, Bn), -1, dtype=torch.int32, device="cuda")
    new_off = torch.full((L, H, S + Bn), -1, dtype=torch.int32, device="cuda")
    new_cnt = torch.full((L, H, Bn), -1, dtype=torch.int32, device="cuda")
    ws = _bytes(B.skipkv_ranges_workspace_bytes(cache, params))
    B.skipkv_token_redundancy_ranges(cache, ranges, red, _bytes(B.skipkv_redundancy_workspace_bytes(cache)))
    B.skipkv_score_ranges(cache, ranges, params, q2, red, score, lam, imp, ws)
    B.skipkv_select_tokens_ranges(cache, ranges, params, imp, red, lam, tok_score, tok_keep, kept_idx, new_len, new_off, new_cnt,
                                  kept_stride, ws)
    B.skipkv_compact(cache, kept_idx, new_len, kept_stride)
    torch.cuda.synchronize()
    assert int(status.item()) == 0
    n = cfg.group
    for l in range(L):
        for h in range(H):
            for b in range(Bn):
                t0, p0, n1, c1 = int(st.seq_off[b]), int(st.sent_ptr[b]), int(len1[l, h, b]), int(cnt1[l, h, b])
                off = off1[l, h, p0:p0 + c1 + 1].astype(np.int64)
                assert off[0] == 0 and off[-1] == n1
                tag = "head (l=%d, h=%d, b=%d, N=%d, S=%d, budget=%d)" % (l, h, b, n1, c1, bud2[l, h, b])
                kh = k_in[l, h, t0:t0 + n1].to(torch.float64).cpu().numpy()
                # Eq. 5 over the head's own tokens
                got_r = red[l, h, t0:t0 + n1].cpu().numpy().astype(np.float64)
                np.testing.assert_allclose(got_r, oracle.token_redundancy(kh), rtol=1e-4, atol=0, err_msg="R " + tag)
                # token importance and lambda over the head's own ranges, with the query rows of the real head
                qh = q2[l, b, h * n:(h + 1) * n].to(torch.float64).cpu().numpy()
                want_imp = oracle.token_importance(qh, kh)
                np.testing.assert_allclose(imp[l, h, t0:t0 + n1].cpu().numpy(), want_imp, rtol=1e-3, atol=1e-12, err_msg="importance " + tag)
                s0 = p0 - b
                want_lam = oracle.sentence_redundancy(oracle.sentence_embeddings(kh, off))
                got_lam = lam[l, h, s0:s0 + c1].cpu().numpy().astype(np.float64)
                assert got_lam[-1] == -np.inf
                np.testing.assert_allclose(got_lam[:-1], want_lam[:-1], rtol=1e-3, atol=1e-5, err_msg="lambda " + tag)
                # Eq. 6 as printed and the eviction, both sides ranking the same fp32 scores
                sc = tok_score[l, h, t0:t0 + n1].cpu().numpy()
                want_sc = oracle.token_scores(imp[l, h, t0:t0 + n1].cpu().numpy(), red[l, h, t0:t0 + n1].cpu().numpy(),
                                              got_lam, off, 0.1, 0.95)
                np.testing.assert_allclose(sc, want_sc, rtol=1e-6, atol=1e-9, err_msg="token scores " + tag)
                ora = oracle.select_tokens(sc.astype(np.float64), off, int(bud2[l, h, b]), cfg.protect_window)
                nl = int(new_len[l, h, b])
                assert nl == ora["new_len"] == min(int(bud2[l, h, b]), n1), tag
                np.testing.assert_array_equal(kept_idx[l, h, b, :nl].cpu().numpy(), ora["kept_idx"], err_msg=tag)
                np.testing.assert_array_equal(tok_keep[l, h, t0:t0 + n1].cpu().numpy().astype(bool), ora["keep"], err_msg=tag)
                c2 = int(new_cnt[l, h, b])
                assert c2 == len(ora["new_off"]) - 1, tag
                np.testing.assert_array_equal(new_off[l, h, p0:p0 + c2 + 1].cpu().numpy(), ora["new_off"], err_msg=tag)
                kept = torch.from_numpy(ora["kept_idx"].astype(np.int64)).cuda()
                assert torch.equal(k[l, h, t0:t0 + nl], k_in[l, h, t0 + kept]) and torch.equal(v[l, h, t0:t0 + nl], v_in[l, h, t0 + kept]), tag

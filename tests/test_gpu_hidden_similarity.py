"""Sentence similarity from the last layer's hidden states (Sec. 4.1, Eq. 1-3 as printed) and the
scores of Eq. 6 with that shared lambda, through the C ABI, against the oracle."""
import numpy as np
import pytest
import torch

import oracle
from paper_2512_07993_amd import binding as B
from paper_2512_07993_amd import workloads as W
from helpers import SCORE_RTOL, make_cache

pytestmark = pytest.mark.gpu


def _hidden_with_copies(st, d_model, dtype, seed, p_copy=0.2, noise=0.05):
    """Hidden states [T, d_model]: iid N(0,1) rows, except that a sentence is, with probability
    p_copy, a noisy copy of an earlier sentence of the same length range (near-duplicates as in the
    key recipe of the workloads)."""
    g = torch.Generator(device="cuda")
    g.manual_seed(seed)
    h = torch.randn((st.total_tokens, d_model), generator=g, device="cuda")
    rng = np.random.default_rng(seed)
    for b in range(len(st.seq_len)):
        off = st.offsets(b)
        t0 = int(st.seq_off[b])
        for s in range(1, len(off) - 1):
            if rng.random() < p_copy:
                j = int(rng.integers(0, s))
                n = int(min(off[s + 1] - off[s], off[j + 1] - off[j]))
                src = h[t0 + off[j]:t0 + off[j] + n]
                h[t0 + off[s]:t0 + off[s] + n] = src + noise * torch.randn(src.shape, generator=g, device="cuda")
    return h.to(dtype)


def _oracle_lambda(st, h, b):
    t0, t1 = int(st.seq_off[b]), int(st.seq_off[b + 1])
    hh = h[t0:t1].to(torch.float64).cpu().numpy()
    emb = oracle.sentence_embeddings(hh, st.offsets(b).astype(np.int64))
    return oracle.sentence_redundancy(emb)


@pytest.mark.parametrize("dtype,d_model", [(torch.bfloat16, 512), (torch.float32, 384), (torch.bfloat16, 4096)])
def test_hidden_state_similarity_matches_oracle(dtype, d_model):
    cfg = W.CONFIGS[3].scaled(n_layers=1, batch=4, len_lo=200, len_hi=2400 if d_model < 4096 else 900)
    st = W.make_structure(cfg)
    h = _hidden_with_copies(st, d_model, dtype, 7)
    k = torch.zeros((1, 1, st.total_tokens, 128), dtype=torch.bfloat16, device="cuda")
    cache = make_cache(cfg.scaled(n_kv_heads=1, n_q_heads=4), st, k, k)
    lam = torch.full((st.total_sentences,), float("nan"), dtype=torch.float32, device="cuda")
    ws = torch.empty(B.skipkv_similarity_workspace_bytes(cache, d_model) + 256, dtype=torch.uint8, device="cuda")
    B.skipkv_sentence_similarity(cache, h, lam, ws)
    torch.cuda.synchronize()
    got = lam.cpu().numpy().astype(np.float64)
    n_dup = 0
    for b in range(cfg.batch):
        want = _oracle_lambda(st, h, b)
        sb, S = st.sent_base(b), int(st.n_sent[b])
        assert got[sb + S - 1] == -np.inf
        np.testing.assert_allclose(got[sb:sb + S - 1], want[:-1], rtol=SCORE_RTOL, atol=1e-5)
        n_dup += int((want[:-1] > 0.95).sum())
    assert n_dup > 0  # the planted copies are found


def _check_scores_with_shared_lambda(cfg, d_model, heads):
    st = W.make_structure(cfg)
    k0, v0, q = W.fill_cache(cfg, st, device="cuda")
    h = _hidden_with_copies(st, d_model, torch.bfloat16, 5)
    cache = make_cache(cfg, st, k0, v0)
    L, H, S, T = cfg.n_layers, cfg.n_kv_heads, st.total_sentences, st.total_tokens
    shared = torch.empty((S,), dtype=torch.float32, device="cuda")
    ws1 = torch.empty(B.skipkv_similarity_workspace_bytes(cache, d_model) + 256, dtype=torch.uint8, device="cuda")
    B.skipkv_sentence_similarity(cache, h, shared, ws1)
    status = torch.zeros(1, dtype=torch.int32, device="cuda")
    params = B.Params(cfg.obs_window, cfg.protect_window, cfg.budget, dev_status=status)
    ws = torch.empty(B.skipkv_workspace_bytes(cache, params) + 256, dtype=torch.uint8, device="cuda")
    score = torch.full((L, H, S), float("nan"), dtype=torch.float32, device="cuda")
    lam_out = torch.full((L, H, S), float("nan"), dtype=torch.float32, device="cuda")
    imp = torch.full((L, H, T), float("nan"), dtype=torch.float32, device="cuda")
    B.skipkv_score_shared(cache, params, q, None, shared, score, lam_out, imp, ws)
    torch.cuda.synchronize()
    assert int(status.item()) == 0
    # every head carries the sequence's lambda unchanged, and nothing is left unwritten
    assert torch.equal(lam_out.view(torch.int32), shared.view(torch.int32).expand(L, H, S))
    assert not bool(torch.isnan(score).any()) and not bool(torch.isnan(imp).any())
    shared_np = shared.cpu().numpy().astype(np.float64)
    for (l, hh, b) in heads(cfg, st):
        qq, kk, vv, off = W.head_arrays(cfg, st, k0, v0, q, l, hh, b)
        t0, t1 = int(st.seq_off[b]), int(st.seq_off[b + 1])
        sb, Sb = st.sent_base(b), int(st.n_sent[b])
        want_imp = oracle.token_importance(qq, kk)
        np.testing.assert_allclose(imp[l, hh, t0:t1].cpu().numpy(), want_imp, rtol=SCORE_RTOL, atol=1e-12)
        lam_b = shared_np[sb:sb + Sb]
        want, candlen = oracle.sentence_scores(want_imp, lam_b, off, cfg.protect_window)
        got = score[l, hh, sb:sb + Sb].cpu().numpy().astype(np.float64)
        cand = candlen > 0
        np.testing.assert_array_equal(np.isinf(got) & (got > 0), ~cand)
        np.testing.assert_allclose(got[cand], want[cand], rtol=SCORE_RTOL, atol=1e-12)


def test_scores_with_shared_lambda_match_oracle():
    cfg = W.CONFIGS[3].scaled(n_layers=2, batch=3, len_lo=500, len_hi=2500, budget=512)
    _check_scores_with_shared_lambda(cfg, 1024, lambda cfg, st: [(l, h, b) for l in range(cfg.n_layers) for h in range(cfg.n_kv_heads)
                                                                  for b in range(cfg.batch)])


def test_scores_with_shared_lambda_config3_full_size():
    """The workload that bench.py --shared-lambda times (all 32 layers, 16 sequences, d_model 4096), on heads
    sampled across layers, heads and sequences."""
    from helpers import sample_heads
    _check_scores_with_shared_lambda(W.CONFIGS[3], 4096, lambda cfg, st: sample_heads(cfg, st, 8, 9))

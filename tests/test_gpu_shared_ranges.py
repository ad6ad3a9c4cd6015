"""The shared lambda (hidden-state sentence similarity, Sec. 4.1 Eq. 1-3 as printed) on per-head
ranges (Eq. 9-11), through the C ABI: two compression steps with a decode-like append in between.
After the first step every head keeps its own subsequence of the sequence's sentences; the second
step must look every head's lambda up by the number its sentence has in the sequence's own list.
Checked against the oracle head by head: the sentence numbers, token importance, scores (rel 1e-3),
the selection (both sides ranking the same fp32 scores, so exactly) and the compacted rows."""
import numpy as np
import pytest
import torch

import oracle
from paper_2512_07993_amd import binding as B
from paper_2512_07993_amd import workloads as W

from helpers import SCORE_RTOL, make_cache
from test_gpu_hidden_similarity import _hidden_with_copies

pytestmark = pytest.mark.gpu


def _bytes(n):
    return torch.empty(n + 256, dtype=torch.uint8, device="cuda")


def test_two_steps_with_shared_lambda_on_per_head_ranges():
    cfg = W.CONFIGS[3].scaled(n_layers=2, n_kv_heads=2, n_q_heads=8, batch=3, len_lo=900, len_hi=2200, budget=512)
    st = W.make_structure(cfg)
    k, v, q1 = W.fill_cache(cfg, st, device="cuda")
    cache = make_cache(cfg, st, k, v)
    L, H, Bn, S, T = cfg.n_layers, cfg.n_kv_heads, cfg.batch, st.total_sentences, st.total_tokens
    n = cfg.group
    dev = lambda a: torch.from_numpy(np.ascontiguousarray(a)).cuda()
    f32 = lambda *shape: torch.full(shape, float("nan"), dtype=torch.float32, device="cuda")
    status = torch.zeros(1, dtype=torch.int32, device="cuda")
    params = B.Params(cfg.obs_window, cfg.protect_window, cfg.budget, dev_status=status)
    kept_stride = min(cfg.budget, T)

    def outputs():
        return dict(keep=torch.full((L, H, S), 77, dtype=torch.uint8, device="cuda"),
                    kept_idx=torch.full((L, H, Bn, kept_stride), -1, dtype=torch.int32, device="cuda"),
                    new_len=torch.full((L, H, Bn), -1, dtype=torch.int32, device="cuda"),
                    new_off=torch.full((L, H, S + Bn), -1, dtype=torch.int32, device="cuda"),
                    new_cnt=torch.full((L, H, Bn), -1, dtype=torch.int32, device="cuda"))

    # ---- step 1 on the shared ranges: similarity from hidden states, scores, selection, compaction, numbers
    hid = _hidden_with_copies(st, 512, torch.bfloat16, 7)
    lam1 = torch.empty((S,), dtype=torch.float32, device="cuda")
    B.skipkv_sentence_similarity(cache, hid, lam1, _bytes(B.skipkv_similarity_workspace_bytes(cache, 512)))
    score1, imp1 = f32(L, H, S), f32(L, H, T)
    B.skipkv_score_shared(cache, params, q1, None, lam1, score1, None, imp1, _bytes(B.skipkv_workspace_bytes(cache, params)))
    o1 = outputs()
    B.skipkv_select(cache, params, score1, o1["keep"], o1["kept_idx"], o1["new_len"], o1["new_off"], o1["new_cnt"], kept_stride)
    B.skipkv_compact(cache, o1["kept_idx"], o1["new_len"], kept_stride)
    ids = torch.full((L, H, S), -5, dtype=torch.int32, device="cuda")
    B.skipkv_ranges_ids_select(cache, None, cfg.protect_window, o1["keep"], None, ids)
    torch.cuda.synchronize()
    assert int(status.item()) == 0
    keep1, cnt1, off1, len1 = o1["keep"].cpu().numpy(), o1["new_cnt"].cpu().numpy(), o1["new_off"].cpu().numpy(), o1["new_len"].cpu().numpy()
    want_ids = {}
    straddlers = 0
    for l in range(L):
        for h in range(H):
            for b in range(Bn):
                off = st.offsets(b).astype(np.int64)
                p = int(off[-1]) - min(cfg.protect_window, int(off[-1]))
                sb, ns = st.sent_base(b), int(st.n_sent[b])
                straddlers += int((~keep1[l, h, sb:sb + ns].astype(bool) & (off[1:] > p)).sum())
                want_ids[(l, h, b)] = oracle.surviving_sentence_ids(off, o1["kept_idx"][l, h, b, :int(len1[l, h, b])].cpu().numpy())
                assert len(want_ids[(l, h, b)]) == cnt1[l, h, b]
                np.testing.assert_array_equal(ids[l, h, sb:sb + cnt1[l, h, b]].cpu().numpy(), want_ids[(l, h, b)])
    assert len({tuple(x) for x in want_ids.values()}) > Bn  # heads of a sequence keep different sentences

    # ---- decode-like phase: new tokens and sentence boundaries, the same text for every head
    rng = np.random.default_rng(3)
    g = torch.Generator(device="cuda")
    g.manual_seed(99)
    n_new = rng.integers(40, 120, size=Bn).astype(np.int32)
    bnds = [np.unique(np.concatenate([[0] if b != 1 else [], rng.choice(np.arange(1, m), size=3, replace=False)])).astype(np.int32)
            for b, m in enumerate(n_new)]
    bnd_ptr = np.concatenate([[0], np.cumsum([len(x) for x in bnds])]).astype(np.int32)
    ranges = B.Ranges(o1["new_len"].clone(), o1["new_cnt"].clone(), o1["new_off"].clone())
    for l in range(L):
        for h in range(H):
            for b in range(Bn):
                t = int(st.seq_off[b]) + int(len1[l, h, b])
                m = int(n_new[b])
                k[l, h, t:t + m] = torch.randn((m, 128), generator=g, device="cuda").to(k.dtype)
                v[l, h, t:t + m] = torch.randn((m, 128), generator=g, device="cuda").to(v.dtype)
    old_cnt = ranges.sent_cnt.clone()
    B.skipkv_ranges_append(cache, ranges, dev(n_new), dev(bnd_ptr), dev(np.concatenate(bnds).astype(np.int32)), status)
    B.skipkv_ranges_ids_append(cache, old_cnt, ranges.sent_cnt, ids)
    torch.cuda.synchronize()
    assert int(status.item()) == 0
    # the sequences' own lists now: the original sentences plus the new ones (sequence 1 continues its last sentence first)
    added = np.array([len(x) for x in bnds])
    n_glob = st.n_sent + added
    cnt2, off2, len2 = ranges.sent_cnt.cpu().numpy(), ranges.sent_off.cpu().numpy(), ranges.len.cpu().numpy()
    for key, w in want_ids.items():
        l, h, b = key
        assert cnt2[l, h, b] == len(w) + added[b]
        want_ids[key] = oracle.append_sentence_ids(w, added[b])
        assert want_ids[key][-1] == n_glob[b] - 1   # a head's last sentence is the sequence's last
        np.testing.assert_array_equal(ids[l, h, st.sent_base(b):st.sent_base(b) + cnt2[l, h, b]].cpu().numpy(), want_ids[key])

    # ---- step 2: a lambda per sentence of the sequences' own lists (any values serve the lookup: a quarter above tau)
    lam_ptr = np.concatenate([[0], np.cumsum(n_glob)]).astype(np.int32)
    lam2 = np.where(rng.random(int(lam_ptr[-1])) < 0.25, rng.uniform(0.951, 0.999, int(lam_ptr[-1])), rng.uniform(-0.2, 0.9, int(lam_ptr[-1]))).astype(np.float32)
    lam2[lam_ptr[1:] - 1] = -np.inf
    q2 = torch.randn(q1.shape, generator=g, device="cuda").to(q1.dtype)
    k_in, v_in = k.clone(), v.clone()
    score2, lamo2, imp2 = f32(L, H, S), f32(L, H, S), f32(L, H, T)
    ws = _bytes(B.skipkv_ranges_workspace_bytes(cache, params))
    B.skipkv_score_shared_ranges(cache, ranges, ids, dev(lam_ptr), params, q2, None, dev(lam2), score2, lamo2, imp2, ws)
    o2 = outputs()
    B.skipkv_select_ranges(cache, ranges, params, score2, o2["keep"], o2["kept_idx"], o2["new_len"], o2["new_off"], o2["new_cnt"],
                           kept_stride, ws)
    B.skipkv_compact(cache, o2["kept_idx"], o2["new_len"], kept_stride)
    ids3 = torch.full((L, H, S), -5, dtype=torch.int32, device="cuda")
    B.skipkv_ranges_ids_select(cache, ranges, cfg.protect_window, o2["keep"], ids, ids3)
    torch.cuda.synchronize()
    assert int(status.item()) == 0
    evicted = 0
    for l in range(L):
        for h in range(H):
            for b in range(Bn):
                t0, p0, sb = int(st.seq_off[b]), int(st.sent_ptr[b]), st.sent_base(b)
                n2, c2 = int(len2[l, h, b]), int(cnt2[l, h, b])
                off = off2[l, h, p0:p0 + c2 + 1].astype(np.int64)
                assert off[0] == 0 and off[-1] == n2
                tag = "head (l=%d, h=%d, b=%d, N=%d, S=%d)" % (l, h, b, n2, c2)
                kh = k_in[l, h, t0:t0 + n2].to(torch.float64).cpu().numpy()
                qh = q2[l, b, h * n:(h + 1) * n].to(torch.float64).cpu().numpy()
                want_imp = oracle.token_importance(qh, kh)
                np.testing.assert_allclose(imp2[l, h, t0:t0 + n2].cpu().numpy(), want_imp, rtol=SCORE_RTOL, atol=1e-12, err_msg=tag)
                lam_h = lam2[lam_ptr[b] + want_ids[(l, h, b)]]
                np.testing.assert_array_equal(lamo2[l, h, sb:sb + c2].cpu().numpy(), lam_h, err_msg=tag)
                want, candlen = oracle.sentence_scores(want_imp, lam_h.astype(np.float64), off, cfg.protect_window)
                got = score2[l, h, sb:sb + c2].cpu().numpy()
                cand = candlen > 0
                np.testing.assert_array_equal(np.isinf(got) & (got > 0), ~cand, err_msg=tag)
                np.testing.assert_allclose(got[cand], want[cand], rtol=SCORE_RTOL, atol=1e-12, err_msg=tag)
                ora = oracle.select_sentences(got.astype(np.float64), candlen, off, cfg.budget, cfg.protect_window)
                nl = int(o2["new_len"][l, h, b])
                assert nl == ora["new_len"], tag
                np.testing.assert_array_equal(o2["keep"][l, h, sb:sb + c2].cpu().numpy().astype(bool), ora["keep"], err_msg=tag)
                np.testing.assert_array_equal(o2["kept_idx"][l, h, b, :nl].cpu().numpy(), ora["kept_idx"], err_msg=tag)
                c3 = int(o2["new_cnt"][l, h, b])
                assert c3 == len(ora["new_off"]) - 1, tag
                np.testing.assert_array_equal(o2["new_off"][l, h, p0:p0 + c3 + 1].cpu().numpy(), ora["new_off"], err_msg=tag)
                kept = torch.from_numpy(ora["kept_idx"]).cuda()
                assert torch.equal(k[l, h, t0:t0 + nl], k_in[l, h, t0 + kept]) and torch.equal(v[l, h, t0:t0 + nl], v_in[l, h, t0 + kept]), tag
                want3 = oracle.surviving_sentence_ids(off, ora["kept_idx"], ids=want_ids[(l, h, b)])
                evicted += c2 - len(want3)
                np.testing.assert_array_equal(ids3[l, h, sb:sb + c3].cpu().numpy(), want3, err_msg=tag)
    assert evicted > 0
    print("straddling sentences after step 1:", straddlers, "sentences evicted in step 2:", evicted, flush=True)


def test_a_number_outside_the_sequences_list_is_reported():
    cfg = W.CONFIGS[3].scaled(n_layers=1, n_kv_heads=2, n_q_heads=8, batch=2, len_lo=400, len_hi=700, budget=256)
    st = W.make_structure(cfg)
    k, v, q = W.fill_cache(cfg, st, device="cuda")
    cache = make_cache(cfg, st, k, v)
    from test_gpu_ranges import shared_as_ranges
    L, H, S, T = cfg.n_layers, cfg.n_kv_heads, st.total_sentences, st.total_tokens
    ids = torch.zeros((L, H, S), dtype=torch.int32, device="cuda")
    ids[0, 1, 3] = int(st.n_sent[0]) + 7
    lam_ptr = torch.from_numpy(np.concatenate([[0], np.cumsum(st.n_sent)]).astype(np.int32)).cuda()
    lam = torch.zeros((S,), dtype=torch.float32, device="cuda")
    status = torch.zeros(1, dtype=torch.int32, device="cuda")
    params = B.Params(cfg.obs_window, cfg.protect_window, cfg.budget, dev_status=status)
    score = torch.empty((L, H, S), dtype=torch.float32, device="cuda")
    B.skipkv_score_shared_ranges(cache, shared_as_ranges(cfg, st), ids, lam_ptr, params, q, None, lam, score, None, None,
                                 _bytes(B.skipkv_ranges_workspace_bytes(cache, params)))
    torch.cuda.synchronize()
    assert int(status.item()) & B.DEV_BAD_OFFSETS

"""Per-head ranges (Sec. 4.1, Eq. 9-11) on a paged KV cache (Appendix, "System-Level Evaluation on
vLLM") through the C ABI.  A first step on the contiguous cache leaves every head with its own
length and sentence ranges; the second step then runs twice on the same numbers, once on the
contiguous cache (whose parity with the oracle test_gpu_ranges.py establishes) and once on pools of
blocks that the cache was scattered into, and the two must agree: token importance, selection and
the compacted rows bit for bit, scores bit for bit through the single-pass scan and to rounding
through the two-pass one (whose pooling order varies from run to run)."""
import numpy as np
import pytest
import torch

from paper_2512_07993_amd import binding as B
from paper_2512_07993_amd import workloads as W

from helpers import GpuStep, device_structure, run_step
from test_gpu_paged import SENTINEL, _from_pages, _to_pages, _token_slots
from test_gpu_ranges import _outputs, run_step_ranges

pytestmark = pytest.mark.gpu


def _run_ranges_paged(cfg, st, kp, vp, table, q, ranges, budget):
    dev = kp.device
    so, sp, sf = device_structure(st, dev)
    cache = B.PagedCache(kp, vp, table, cfg.n_q_heads, so, sp, sf, st.total_tokens, st.total_sentences)
    status = torch.zeros(1, dtype=torch.int32, device=dev)
    params = B.Params(cfg.obs_window, cfg.protect_window, budget, dev_status=status)
    ws = torch.empty(B.skipkv_ranges_paged_workspace_bytes(cache, params) + 256, dtype=torch.uint8, device=dev)
    kept_stride = max(1, min(budget, st.total_tokens))
    o = _outputs(cfg, st, kept_stride)
    B.skipkv_step_ranges_paged(cache, ranges, params, q, None, o["sent_score"], o["sent_lambda"], o["tok_imp"],
                               o["sent_keep"], o["kept_idx"], o["new_len"], o["new_sent_off"], o["new_sent_cnt"],
                               kept_stride, ws)
    torch.cuda.synchronize()
    return GpuStep(cache, params, o["sent_score"], o["sent_lambda"], o["tok_imp"], o["sent_keep"], o["kept_idx"],
                   o["new_len"], o["new_sent_off"], o["new_sent_cnt"], kept_stride, status)


def _first_step(cfg):
    st = W.make_structure(cfg)
    k, v, q = W.fill_cache(cfg, st, device="cuda")
    s1 = run_step(cfg, st, k, v, q)
    assert int(s1.dev_status.item()) == 0
    assert len({int(x) for x in s1.new_len.flatten()}) > 1  # heads really differ after the first step
    g = torch.Generator(device="cuda")
    g.manual_seed(17)
    q2 = torch.randn(q.shape, generator=g, device="cuda").to(q.dtype)
    return st, k, v, q2, s1


def _ranges_of(s1):
    return B.Ranges(s1.new_len.clone(), s1.new_sent_cnt.clone(), s1.new_sent_off.clone())


@pytest.mark.parametrize("config_id,kw,block_size,heads_before_slots", [
    (3, dict(n_layers=2, batch=4, len_lo=900, len_hi=3000, budget=768), 16, False),
    (3, dict(n_layers=2, batch=4, len_lo=900, len_hi=3000, budget=768), 32, True),
    (3, dict(n_layers=1, batch=3, len_lo=700, len_hi=1800, budget=512), 24, False),
    (4, dict(n_layers=2, batch=3, len_lo=700, len_hi=1800, budget=512), 16, False),
    (1, dict(), 16, False),
])
def test_paged_per_head_step_equals_the_contiguous_one(config_id, kw, block_size, heads_before_slots, monkeypatch):
    cfg = W.CONFIGS[config_id].scaled(**kw) if kw else W.CONFIGS[config_id]
    st, k1, v1, q2, s1 = _first_step(cfg)
    budget2 = cfg.budget // 2
    print("paged ranges", cfg.name, "block", block_size, "tokens", st.total_tokens, flush=True)
    kp, vp, table = _to_pages(cfg, st, k1, v1, block_size, seed=block_size + 1, heads_before_slots=heads_before_slots)
    kp0 = kp.clone()
    out = _run_ranges_paged(cfg, st, kp, vp, table, q2, _ranges_of(s1), budget2)
    assert int(out.dev_status.item()) == 0
    two_pass = block_size < 16 or (block_size & (block_size - 1)) != 0
    k, v = k1.clone(), v1.clone()
    ref = run_step_ranges(cfg, st, k, v, q2, _ranges_of(s1), budget2, flags=B.FLAG_FORCE_TWO_PASS if two_pass else 0)
    assert int(ref.dev_status.item()) == 0
    # per-token and per-sentence arrays are defined inside every head's own ranges only
    len1, cnt1 = s1.new_len.cpu().numpy(), s1.new_sent_cnt.cpu().numpy()
    new_len, new_cnt = out.new_len.cpu().numpy(), out.new_sent_cnt.cpu().numpy()
    assert np.array_equal(new_len, ref.new_len.cpu().numpy()) and np.array_equal(new_cnt, ref.new_sent_cnt.cpu().numpy())
    assert (new_len <= budget2).all() and (new_len < len1).any()
    exact = not two_pass and cfg.dtype != "fp32"
    kg, vg = _from_pages(cfg, st, kp, table, block_size), _from_pages(cfg, st, vp, table, block_size)
    for l in range(cfg.n_layers):
        for h in range(cfg.n_kv_heads):
            for b in range(cfg.batch):
                t0, p0 = int(st.seq_off[b]), int(st.sent_ptr[b])
                n1, c1, n2, c2 = int(len1[l, h, b]), int(cnt1[l, h, b]), int(new_len[l, h, b]), int(new_cnt[l, h, b])
                tag = (l, h, b)
                assert torch.equal(out.tok_imp[l, h, t0:t0 + n1].view(torch.int32), ref.tok_imp[l, h, t0:t0 + n1].view(torch.int32)), tag
                s0 = p0 - b
                assert torch.equal(out.sent_keep[l, h, s0:s0 + c1], ref.sent_keep[l, h, s0:s0 + c1]), tag
                for name in ("sent_lambda", "sent_score"):
                    x, y = getattr(out, name)[l, h, s0:s0 + c1], getattr(ref, name)[l, h, s0:s0 + c1]
                    if exact:
                        assert torch.equal(x.view(torch.int32), y.view(torch.int32)), (name, tag)
                    else:
                        torch.testing.assert_close(x, y, rtol=1e-5, atol=1e-6)
                assert torch.equal(out.kept_idx[l, h, b, :n2], ref.kept_idx[l, h, b, :n2]), tag
                assert torch.equal(out.new_sent_off[l, h, p0:p0 + c2 + 1], ref.new_sent_off[l, h, p0:p0 + c2 + 1]), tag
                assert torch.equal(kg[l, h, t0:t0 + n2].view(torch.uint8), k[l, h, t0:t0 + n2].view(torch.uint8)), tag
                assert torch.equal(vg[l, h, t0:t0 + n2].view(torch.uint8), v[l, h, t0:t0 + n2].view(torch.uint8)), tag
    # slots that hold no token were not written
    blk, slot = _token_slots(cfg, st, table.cpu().numpy(), block_size, kp.device)
    free = torch.ones(kp.shape[1], kp.shape[2], dtype=torch.bool, device=kp.device)
    free[blk, slot] = False
    assert torch.equal(kp[:, free].view(torch.uint8), kp0[:, free].view(torch.uint8))
    assert bool((vp[:, free] == SENTINEL).all())


def test_paged_per_head_step_reports_a_bad_block_id_and_leaves_the_sequence_alone():
    cfg = W.CONFIGS[3].scaled(n_layers=2, batch=3, len_lo=900, len_hi=2000, budget=512)
    st, k1, v1, q2, s1 = _first_step(cfg)
    kp, vp, table = _to_pages(cfg, st, k1, v1, 16, seed=9)
    table[2, 1] = -4
    kp0, vp0 = kp.clone(), vp.clone()
    out = _run_ranges_paged(cfg, st, kp, vp, table, q2, _ranges_of(s1), cfg.budget // 2)
    assert int(out.dev_status.item()) & B.DEV_BAD_BLOCK_TABLE
    n2 = (int(st.seq_off[3] - st.seq_off[2]) + 15) // 16
    own = table[2, :n2].cpu().numpy()
    own = torch.from_numpy(own[(own >= 0) & (own < kp.shape[1])].astype(np.int64)).to(kp.device)
    assert torch.equal(kp[:, own].view(torch.uint8), kp0[:, own].view(torch.uint8))
    assert torch.equal(vp[:, own].view(torch.uint8), vp0[:, own].view(torch.uint8))
    # the other sequences were compacted
    new_len = out.new_len.cpu().numpy()
    assert (new_len >= 0).all() and (new_len <= cfg.budget // 2).all()
    assert not torch.equal(kp.view(torch.uint8), kp0.view(torch.uint8))


def test_token_level_flow_and_shared_lambda_on_per_head_ranges_and_pages():
    """After a first step on the contiguous cache: the token-level flow (R, scores, token selection,
    compaction) and the scores with a shared lambda, on pages and on the contiguous cache."""
    from test_gpu_ranges_tokens import _bytes
    cfg = W.CONFIGS[3].scaled(n_layers=2, batch=3, len_lo=900, len_hi=2400, budget=768)
    st, k1, v1, q2, s1 = _first_step(cfg)
    L, H, Bn, S, T = cfg.n_layers, cfg.n_kv_heads, cfg.batch, st.total_sentences, st.total_tokens
    budget2 = cfg.budget // 2
    kept_stride = budget2
    kp, vp, table = _to_pages(cfg, st, k1, v1, 16, seed=41)
    so, sp, sf = device_structure(st, kp.device)
    paged = B.PagedCache(kp, vp, table, cfg.n_q_heads, so, sp, sf, T, S)
    k, v = k1.clone(), v1.clone()
    from helpers import make_cache
    flat = make_cache(cfg, st, k, v)
    f32 = lambda *shape: torch.full(shape, float("nan"), dtype=torch.float32, device="cuda")
    ids = torch.arange(S, dtype=torch.int32, device="cuda").expand(L, H, S).contiguous() % 7   # any numbers inside the lists
    lam_ptr = torch.from_numpy(np.concatenate([[0], np.cumsum(st.n_sent)]).astype(np.int32)).cuda()
    shared = torch.from_numpy(np.random.default_rng(6).uniform(0.6, 1.0, S).astype(np.float32)).cuda()
    res = {}
    for name, cache in (("flat", flat), ("paged", paged)):
        status = torch.zeros(1, dtype=torch.int32, device="cuda")
        params = B.Params(cfg.obs_window, cfg.protect_window, budget2, dev_status=status)
        ranges = _ranges_of(s1)
        red, imp, score, lam, tok_score, score_sh, lam_sh = f32(L, H, T), f32(L, H, T), f32(L, H, S), f32(L, H, S), f32(L, H, T), f32(L, H, S), f32(L, H, S)
        tok_keep = torch.full((L, H, T), 77, dtype=torch.uint8, device="cuda")
        kept_idx = torch.full((L, H, Bn, kept_stride), -1, dtype=torch.int32, device="cuda")
        new_len = torch.full((L, H, Bn), -1, dtype=torch.int32, device="cuda")
        new_off = torch.full((L, H, S + Bn), -1, dtype=torch.int32, device="cuda")
        new_cnt = torch.full((L, H, Bn), -1, dtype=torch.int32, device="cuda")
        if name == "flat":
            ws = _bytes(B.skipkv_ranges_workspace_bytes(cache, params))
            B.skipkv_token_redundancy_ranges(cache, ranges, red, _bytes(B.skipkv_redundancy_workspace_bytes(cache)))
            B.skipkv_score_shared_ranges(cache, ranges, ids, lam_ptr, params, q2, red, shared, score_sh, lam_sh, None, ws)
            B.skipkv_score_ranges(cache, ranges, params, q2, red, score, lam, imp, ws)
        else:
            ws = _bytes(B.skipkv_ranges_paged_workspace_bytes(cache, params))
            B.skipkv_token_redundancy_ranges_paged(cache, ranges, red, status, _bytes(B.skipkv_redundancy_paged_workspace_bytes(cache)))
            B.skipkv_score_ranges_paged(cache, ranges, ids, lam_ptr, shared, params, q2, red, score_sh, lam_sh, None, ws)
            B.skipkv_score_ranges_paged(cache, ranges, None, None, None, params, q2, red, score, lam, imp, ws)
        B.skipkv_select_tokens_ranges(cache, ranges, params, imp, red, lam, tok_score, tok_keep, kept_idx, new_len, new_off, new_cnt,
                                      kept_stride, ws)
        if name == "flat":
            B.skipkv_compact(cache, kept_idx, new_len, kept_stride)
        else:
            B.skipkv_compact_paged(cache, kept_idx, new_len, kept_stride, status, _bytes(B.skipkv_compact_paged_workspace_bytes(cache, kept_stride)))
        torch.cuda.synchronize()
        assert int(status.item()) == 0
        res[name] = dict(red=red, imp=imp, score=score, lam=lam, tok_score=tok_score, score_sh=score_sh, lam_sh=lam_sh,
                         tok_keep=tok_keep, kept_idx=kept_idx, new_len=new_len, new_off=new_off, new_cnt=new_cnt)
    len1, cnt1 = s1.new_len.cpu().numpy(), s1.new_sent_cnt.cpu().numpy()
    nl = res["flat"]["new_len"].cpu().numpy()
    assert np.array_equal(nl, res["paged"]["new_len"].cpu().numpy()) and np.array_equal(res["flat"]["new_cnt"].cpu().numpy(), res["paged"]["new_cnt"].cpu().numpy())
    assert (nl == np.minimum(budget2, len1)).all()
    kg, vg = _from_pages(cfg, st, kp, table, 16), _from_pages(cfg, st, vp, table, 16)
    a, b_ = res["flat"], res["paged"]
    for l in range(L):
        for h in range(H):
            for b in range(Bn):
                t0, p0, n1, c1, n2 = int(st.seq_off[b]), int(st.sent_ptr[b]), int(len1[l, h, b]), int(cnt1[l, h, b]), int(nl[l, h, b])
                s0 = p0 - b
                for name in ("red", "imp", "tok_score"):
                    assert torch.equal(a[name][l, h, t0:t0 + n1].view(torch.int32), b_[name][l, h, t0:t0 + n1].view(torch.int32)), (name, l, h, b)
                for name in ("score", "lam", "score_sh", "lam_sh"):
                    assert torch.equal(a[name][l, h, s0:s0 + c1].view(torch.int32), b_[name][l, h, s0:s0 + c1].view(torch.int32)), (name, l, h, b)
                assert torch.equal(a["tok_keep"][l, h, t0:t0 + n1], b_["tok_keep"][l, h, t0:t0 + n1])
                assert torch.equal(a["kept_idx"][l, h, b, :n2], b_["kept_idx"][l, h, b, :n2])
                c2 = int(a["new_cnt"][l, h, b])
                assert torch.equal(a["new_off"][l, h, p0:p0 + c2 + 1], b_["new_off"][l, h, p0:p0 + c2 + 1])
                assert torch.equal(kg[l, h, t0:t0 + n2].view(torch.uint8), k[l, h, t0:t0 + n2].view(torch.uint8)), (l, h, b)
                assert torch.equal(vg[l, h, t0:t0 + n2].view(torch.uint8), v[l, h, t0:t0 + n2].view(torch.uint8)), (l, h, b)
    # the looked-up lambda is the one of the sentence's number
    sh = shared.cpu().numpy()
    for (l, h, b) in [(0, 0, 0), (1, 3, 2)]:
        s0, c1 = int(st.sent_ptr[b]) - b, int(cnt1[l, h, b])
        want = sh[int(lam_ptr[b]) + ids[l, h, s0:s0 + c1].cpu().numpy()]
        np.testing.assert_array_equal(b_["lam_sh"][l, h, s0:s0 + c1].cpu().numpy(), want)


def test_paged_per_head_step_replays_from_a_hip_graph():
    """Like the contiguous step, the per-head step on pages allocates nothing, never synchronises and
    clears its flags with fill kernels: captured into a HIP graph, every replay (with eager work and
    synchronisations in between) reproduces the eager result bit for bit."""
    cfg = W.CONFIGS[3].scaled(n_layers=1, batch=3, len_lo=900, len_hi=2000, budget=512)
    st, k1, v1, q2, s1 = _first_step(cfg)
    budget2 = cfg.budget // 2
    kp0, vp0, table = _to_pages(cfg, st, k1, v1, 16, seed=77)
    ka, va = kp0.clone(), vp0.clone()
    eager = _run_ranges_paged(cfg, st, ka, va, table, q2, _ranges_of(s1), budget2)
    assert int(eager.dev_status.item()) == 0
    kp, vp = kp0.clone(), vp0.clone()
    so, sp, sf = device_structure(st, kp.device)
    cache = B.PagedCache(kp, vp, table, cfg.n_q_heads, so, sp, sf, st.total_tokens, st.total_sentences)
    status = torch.zeros(1, dtype=torch.int32, device="cuda")
    params = B.Params(cfg.obs_window, cfg.protect_window, budget2, dev_status=status)
    ws = torch.empty(B.skipkv_ranges_paged_workspace_bytes(cache, params) + 256, dtype=torch.uint8, device="cuda")
    ranges = _ranges_of(s1)
    o = _outputs(cfg, st, eager.kept_stride)
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        with torch.cuda.graph(graph, stream=side):
            B.skipkv_step_ranges_paged(cache, ranges, params, q2, None, o["sent_score"], o["sent_lambda"], o["tok_imp"],
                                       o["sent_keep"], o["kept_idx"], o["new_len"], o["new_sent_off"], o["new_sent_cnt"],
                                       eager.kept_stride, ws)
    torch.cuda.synchronize()
    len1, cnt1 = s1.new_len.cpu().numpy(), s1.new_sent_cnt.cpu().numpy()
    for rep in range(3):
        kp.copy_(kp0)
        vp.copy_(vp0)
        for t in (o["sent_score"], o["kept_idx"], o["new_len"]):
            t.fill_(-7)                       # eager work between the replays
        ws.fill_(0xAB)                        # nothing in the workspace is carried from call to call
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert int(status.item()) == 0
        assert torch.equal(o["new_len"], eager.new_len) and torch.equal(o["new_sent_cnt"], eager.new_sent_cnt), rep
        nl = o["new_len"].cpu().numpy()
        for l in range(cfg.n_layers):
            for h in range(cfg.n_kv_heads):
                for b in range(cfg.batch):
                    s0, c1, n2 = int(st.sent_ptr[b]) - b, int(cnt1[l, h, b]), int(nl[l, h, b])
                    assert torch.equal(o["sent_score"][l, h, s0:s0 + c1].view(torch.int32), eager.sent_score[l, h, s0:s0 + c1].view(torch.int32)), (rep, l, h, b)
                    assert torch.equal(o["kept_idx"][l, h, b, :n2], eager.kept_idx[l, h, b, :n2]), (rep, l, h, b)
        # the pools: wherever a kept token lives the replay wrote what the eager call wrote
        kg, kr = _from_pages(cfg, st, kp, table, 16), _from_pages(cfg, st, ka, table, 16)
        vg, vr = _from_pages(cfg, st, vp, table, 16), _from_pages(cfg, st, va, table, 16)
        for l in range(cfg.n_layers):
            for h in range(cfg.n_kv_heads):
                for b in range(cfg.batch):
                    t0, n2 = int(st.seq_off[b]), int(nl[l, h, b])
                    assert torch.equal(kg[l, h, t0:t0 + n2], kr[l, h, t0:t0 + n2]) and torch.equal(vg[l, h, t0:t0 + n2], vr[l, h, t0:t0 + n2]), (rep, l, h, b)

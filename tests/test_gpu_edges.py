"""GPU parity on the degenerate and ragged cases of the method, and on the optional inputs
and outputs of the C ABI."""
import numpy as np
import pytest
import torch

import oracle
from paper_2512_07993_amd import binding as B
from paper_2512_07993_amd import workloads as W

from helpers import compare_head, make_cache, oracle_head, run_step

pytestmark = pytest.mark.gpu


def _structure(offsets):
    """Structure from explicit per-sequence sentence offsets."""
    seq_len = np.asarray([o[-1] for o in offsets], dtype=np.int32)
    seq_off = np.concatenate([[0], np.cumsum(seq_len)]).astype(np.int32)
    sent_ptr = np.concatenate([[0], np.cumsum([len(o) for o in offsets])]).astype(np.int32)
    sent_off = np.concatenate([np.asarray(o, dtype=np.int32) for o in offsets])
    return W.Structure(seq_len, seq_off, sent_ptr, sent_off, [np.full(len(o) - 1, -1) for o in offsets])


def _random_kvq(cfg, st, seed, stride_tok=128):
    g = torch.Generator(device="cuda")
    g.manual_seed(seed)
    dt = W.torch_dtype(cfg)
    shape = (cfg.n_layers, cfg.n_kv_heads, st.total_tokens, stride_tok)
    k = torch.randn(shape, generator=g, device="cuda").to(dt)[..., :128]
    v = torch.randn(shape, generator=g, device="cuda").to(dt)[..., :128]
    q = torch.randn((cfg.n_layers, cfg.batch, cfg.n_q_heads, cfg.obs_window, 128), generator=g, device="cuda").to(dt)
    return k, v, q


def _clone(t):
    """Clone that preserves strides (a strided cache stays strided)."""
    out = torch.empty_strided(t.shape, t.stride(), dtype=t.dtype, device=t.device)
    out.copy_(t)
    return out


def _compare_all(cfg, st, out, k, v, k0, v0, q, budgets=None, red=None, skip_empty=True):
    stats = {}
    for l in range(cfg.n_layers):
        for h in range(cfg.n_kv_heads):
            for b in range(cfg.batch):
                if st.seq_len[b] == 0:
                    assert int(out.new_len[l, h, b]) == 0 and int(out.new_sent_cnt[l, h, b]) == 0
                    continue
                bud = None if budgets is None else int(budgets[b])
                ora = oracle_head(cfg, st, k0, v0, q, l, h, b, budget=bud, red=red)
                compare_head(cfg, st, out, k, v, k0, v0, ora, l, h, b, stats, budget=bud)
    return stats


def _edge_cfg(dtype="bf16", batch=5):
    return W.Config("edges", 9, batch, 1, 2, 8, dtype, 0, 0, 64, 8, 16, 16.0, 0.0)


def _edge_offsets():
    rng = np.random.default_rng(5)
    long_seq = [0, 3, 4, 5, 705]                       # a 700-token sentence spanning several chunks and tiles
    while long_seq[-1] < 1500:
        long_seq.append(min(1500, long_seq[-1] + int(rng.integers(1, 40))))
    return [
        [0],                                           # empty sequence
        [0, 2, 5],                                     # shorter than the observation window
        [0, 7, 19, 40],                                # fits the budget: nothing evicted
        long_seq,
        list(range(0, 301)),                           # 300 one-token sentences (more than a chunk may hold)
    ]


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_ragged_degenerate_batch(dtype):
    cfg = _edge_cfg(dtype)
    st = _structure(_edge_offsets())
    k0, v0, q = _random_kvq(cfg, st, 11)
    k, v = k0.clone(), v0.clone()
    out = run_step(cfg, st, k, v, q)
    assert int(out.dev_status.item()) == 0
    stats = _compare_all(cfg, st, out, k, v, k0, v0, q)
    assert stats["heads"] == 8
    # sequences that fit are untouched, bit for bit
    for b in (1, 2):
        t0, t1 = int(st.seq_off[b]), int(st.seq_off[b + 1])
        assert torch.equal(k[:, :, t0:t1], k0[:, :, t0:t1]) and torch.equal(v[:, :, t0:t1], v0[:, :, t0:t1])
        assert int(out.new_len[0, 0, b]) == t1 - t0


def test_per_sequence_budgets_and_token_redundancy_input():
    cfg = W.CONFIGS[3].scaled(n_layers=1, batch=4, len_lo=600, len_hi=2500, budget=512)
    st = W.make_structure(cfg)
    k0, v0, q = W.fill_cache(cfg, st, device="cuda")
    k, v = k0.clone(), v0.clone()
    budgets = torch.tensor([256, 512, 300, 4000], dtype=torch.int32, device="cuda")
    g = torch.Generator(device="cuda")
    g.manual_seed(3)
    red = torch.rand((cfg.n_layers, cfg.n_kv_heads, st.total_tokens), generator=g, device="cuda") * 1e-3
    out = run_step(cfg, st, k, v, q, budget=budgets, red=red)
    stats = _compare_all(cfg, st, out, k, v, k0, v0, q, budgets=budgets.cpu().numpy(), red=red)
    assert stats["heads"] == 32
    assert (out.new_len[0, 0].cpu().numpy() <= budgets.cpu().numpy()).all()


def test_strided_cache_rows():
    cfg = W.CONFIGS[2].scaled(n_layers=1, len_lo=900, len_hi=900, budget=512)
    st = W.make_structure(cfg)
    k0, v0, q = _random_kvq(cfg, st, 21, stride_tok=192)
    assert k0.stride(2) == 192
    k, v = _clone(k0), _clone(v0)
    assert k.stride() == k0.stride()
    out = run_step(cfg, st, k, v, q)
    _compare_all(cfg, st, out, k, v, k0, v0, q)


def test_exact_duplicates_score_maximal_redundancy():
    cfg = W.CONFIGS[1]
    st = W.make_structure(cfg)
    k0, v0, q = W.fill_cache(cfg, st, device="cuda", dup_noise=0.0)
    k, v = k0.clone(), v0.clone()
    out = run_step(cfg, st, k, v, q)
    lam = out.sent_lambda[0].cpu().numpy()
    srcs = sorted(set(int(j) for j in st.dup_src[0] if j >= 0))
    # Unit embeddings are carried as bf16 hi + lo (16 significant bits per component) and normalised
    # with 1-ulp reciprocal and square root: |v|^2 deviates from 1 by a few 1e-6 at most.
    np.testing.assert_allclose(lam[:, srcs], 1.0, atol=5e-6)
    _compare_all(cfg, st, out, k, v, k0, v0, q)


def test_bad_offsets_are_reported_not_executed():
    """A sequence whose ranges are not strictly ascending (all offsets still inside the sequence) is
    reported and left whole: new_len = N, identity indices, K and V bit-identical to the input;
    the other sequence of the batch is processed as usual."""
    cfg = _edge_cfg(batch=2)
    st = _structure([[0, 10, 10, 30], [0, 5, 40]])         # first sequence: an empty sentence
    k0, v0, q = _random_kvq(cfg, st, 31)
    k, v = k0.clone(), v0.clone()
    out = run_step(cfg, st, k, v, q, budget=24)
    assert int(out.dev_status.item()) & B.DEV_BAD_OFFSETS
    assert not int(out.dev_status.item()) & ~B.DEV_BAD_OFFSETS
    n0 = 30
    assert (out.new_len[:, :, 0] == n0).all()
    assert torch.equal(k[:, :, :n0], k0[:, :, :n0]) and torch.equal(v[:, :, :n0], v0[:, :, :n0])
    kept = out.kept_idx[:, :, 0, :24].cpu().numpy()
    assert (kept == np.arange(24)[None, None, :]).all()
    stats = {}
    for l, h in ((0, 0), (cfg.n_layers - 1, cfg.n_kv_heads - 1)):
        ora = oracle_head(cfg, st, k0, v0, q, l, h, 1, budget=24)
        compare_head(cfg, st, out, k, v, k0, v0, ora, l, h, 1, stats, budget=24)


def test_many_tiny_sequences_more_items_than_workgroups():
    """Sequences of a few tokens: every work item of the single-pass scan has at most two stages
    per wave, so its load stream runs two items ahead of the compute, and there are more items
    than resident workgroups, so that every workgroup walks through several of them."""
    rng = np.random.default_rng(23)
    offsets = []
    for _ in range(40):
        n_sent = int(rng.integers(1, 7))
        lens = rng.integers(1, 12, size=n_sent)
        offsets.append(np.concatenate([[0], np.cumsum(lens)]).tolist())
    st = _structure(offsets)
    cfg = W.Config("tiny-seqs", 9, len(offsets), 4, 8, 32, "bf16", 0, 0, 12, 4, 4, 6.0, 0.0)
    assert cfg.n_layers * cfg.n_kv_heads * cfg.batch > 1024
    k0, v0, q = _random_kvq(cfg, st, 41)
    k, v = k0.clone(), v0.clone()
    out = run_step(cfg, st, k, v, q)
    assert int(out.dev_status.item()) == 0
    rs = np.random.default_rng(1)
    stats = {}
    for _ in range(60):
        l, h, b = int(rs.integers(cfg.n_layers)), int(rs.integers(cfg.n_kv_heads)), int(rs.integers(cfg.batch))
        ora = oracle_head(cfg, st, k0, v0, q, l, h, b)
        compare_head(cfg, st, out, k, v, k0, v0, ora, l, h, b, stats)


def test_select_ties_signs_and_all_group_sizes():
    """skipkv_select on hand-made scores: heavy ties across the cut (index order decides), both
    signed zeros, negative scores, denormals; sequences from 1 to 4096 sentences so that both the
    one-wave and the four-wave ranking run, with budgets that cut at different depths.  Integer
    work: everything must equal the oracle's selection exactly."""
    rng = np.random.default_rng(11)
    n_sents = [1, 2, 63, 64, 65, 500, 1023, 1024, 1025, 2500, 4096]
    offsets = []
    for ns in n_sents:
        lens = rng.integers(1, 9, size=ns)
        offsets.append(np.concatenate([[0], np.cumsum(lens)]).tolist())
    st = _structure(offsets)
    cfg = W.Config("select", 9, len(n_sents), 1, 2, 8, "bf16", 0, 0, 0, 8, 16, 4.0, 0.0)
    k = torch.zeros((1, 2, st.total_tokens, 128), dtype=torch.bfloat16, device="cuda")
    cache = make_cache(cfg, st, k, k.clone())
    L, H, Bn, S, T = 1, 2, cfg.batch, st.total_sentences, st.total_tokens
    palettes = [
        np.array([0.0, -0.0, 1.0, -1.0, 0.5], dtype=np.float32),                       # few values: ties everywhere
        np.array([1e-42, -1e-42, 3e38, -3e38, 0.25, 0.250001], dtype=np.float32),      # denormals and extremes
    ]
    score = np.empty((L, H, S), dtype=np.float32)
    score[0, 0] = palettes[0][rng.integers(0, len(palettes[0]), size=S)]
    score[0, 1] = np.where(rng.random(S) < 0.5, palettes[1][rng.integers(0, len(palettes[1]), size=S)],
                           rng.standard_normal(S).astype(np.float32))
    for frac in (0.05, 0.5, 0.97):
        budgets = np.maximum(16, (st.seq_len * frac).astype(np.int32))
        bud_t = torch.from_numpy(budgets).cuda()
        max_budget = int(budgets.max())
        status = torch.zeros(1, dtype=torch.int32, device="cuda")
        params = B.Params(cfg.obs_window, cfg.protect_window, bud_t, max_budget=max_budget, dev_status=status)
        kept_stride = min(max_budget, T)
        sent_keep = torch.full((L, H, S), 77, dtype=torch.uint8, device="cuda")
        kept_idx = torch.full((L, H, Bn, kept_stride), -1, dtype=torch.int32, device="cuda")
        new_len = torch.full((L, H, Bn), -1, dtype=torch.int32, device="cuda")
        new_off = torch.full((L, H, S + Bn), -1, dtype=torch.int32, device="cuda")
        new_cnt = torch.full((L, H, Bn), -1, dtype=torch.int32, device="cuda")
        B.skipkv_select(cache, params, torch.from_numpy(score).cuda(), sent_keep, kept_idx, new_len, new_off,
                        new_cnt, kept_stride)
        torch.cuda.synchronize()
        assert int(status.item()) == 0
        for h in range(H):
            for b in range(Bn):
                off = st.offsets(b).astype(np.int64)
                sb, ns, n_tok = st.sent_base(b), int(st.n_sent[b]), int(off[-1])
                p = n_tok - min(cfg.protect_window, n_tok)
                candlen = np.clip(np.minimum(off[1:], p) - off[:-1], 0, None)
                sc = score[0, h, sb:sb + ns].astype(np.float64)
                ora = oracle.select_sentences(np.where(candlen > 0, sc, np.inf), candlen, off, int(budgets[b]),
                                              cfg.protect_window)
                tag = "frac %.2f head %d seq %d (S=%d)" % (frac, h, b, ns)
                nl = int(new_len[0, h, b])
                assert nl == ora["new_len"], tag
                np.testing.assert_array_equal(kept_idx[0, h, b, :nl].cpu().numpy(), ora["kept_idx"], err_msg=tag)
                np.testing.assert_array_equal(sent_keep[0, h, sb:sb + ns].cpu().numpy().astype(bool), ora["keep"],
                                              err_msg=tag)
                cnt = int(new_cnt[0, h, b])
                assert cnt == len(ora["new_off"]) - 1, tag
                np.testing.assert_array_equal(new_off[0, h, st.sent_ptr[b]:st.sent_ptr[b] + cnt + 1].cpu().numpy(),
                                              ora["new_off"], err_msg=tag)


def test_untrusted_heads_keep_everything_and_are_not_compacted():
    """skipkv_select + skipkv_compact on inputs the library must refuse per head: a device budget
    larger than the row of kept indices can hold, one below the protected window, a negative one, and a
    NaN score.  Those heads report their full length, identity indices and the matching status bit,
    and their K/V stay bit-identical; the healthy heads of the batch, whose rows of kept indices lie between
    those of the refused ones, are selected and compacted as usual."""
    rng = np.random.default_rng(3)
    offsets = []
    for _ in range(5):
        lens = rng.integers(2, 9, size=40)
        offsets.append(np.concatenate([[0], np.cumsum(lens)]).tolist())
    st = _structure(offsets)
    cfg = W.Config("untrusted", 9, 5, 1, 2, 8, "bf16", 0, 0, 0, 8, 16, 4.0, 0.0)
    T, S, Bn, L, H = st.total_tokens, st.total_sentences, 5, 1, 2
    g = torch.Generator(device="cuda").manual_seed(5)
    k0 = torch.randn((L, H, T, 128), device="cuda", generator=g).to(torch.bfloat16)
    v0 = torch.randn((L, H, T, 128), device="cuda", generator=g).to(torch.bfloat16)
    k, v = k0.clone(), v0.clone()
    cache = make_cache(cfg, st, k, v)
    score = rng.standard_normal((L, H, S)).astype(np.float32)
    score[0, :, st.sent_base(4) + 7] = np.nan                      # sequence 4: a score that cannot be ranked
    max_budget = 64
    budgets = np.array([64, 100000, 8, -5, 64], dtype=np.int32)   # 1: beyond max_budget, 2: below the window, 3: negative
    status = torch.zeros(1, dtype=torch.int32, device="cuda")
    params = B.Params(cfg.obs_window, cfg.protect_window, torch.from_numpy(budgets).cuda(), max_budget=max_budget,
                      dev_status=status)
    kept_stride = max_budget
    kept_idx = torch.full((L, H, Bn, kept_stride), -99, dtype=torch.int32, device="cuda")
    new_len = torch.full((L, H, Bn), -1, dtype=torch.int32, device="cuda")
    sent_keep = torch.full((L, H, S), 77, dtype=torch.uint8, device="cuda")
    B.skipkv_select(cache, params, torch.from_numpy(score).cuda(), sent_keep, kept_idx, new_len, None, None, kept_stride)
    B.skipkv_compact(cache, kept_idx, new_len, kept_stride)
    torch.cuda.synchronize()
    assert int(status.item()) == (B.DEV_BAD_BUDGET | B.DEV_BAD_SCORES)
    for h in range(H):
        for b in (1, 2, 3, 4):
            t0, t1 = int(st.seq_off[b]), int(st.seq_off[b + 1])
            assert int(new_len[0, h, b]) == t1 - t0 > kept_stride
            assert torch.equal(kept_idx[0, h, b], torch.arange(kept_stride, dtype=torch.int32, device="cuda"))
            assert torch.equal(k[0, h, t0:t1], k0[0, h, t0:t1]) and torch.equal(v[0, h, t0:t1], v0[0, h, t0:t1])
        for b in (0,):
            t0, t1 = int(st.seq_off[b]), int(st.seq_off[b + 1])
            n = int(new_len[0, h, b])
            assert 16 <= n <= 64
            idx = kept_idx[0, h, b, :n].long()
            assert torch.equal(k[0, h, t0:t0 + n], k0[0, h, t0:t1][idx]) and torch.equal(v[0, h, t0:t0 + n], v0[0, h, t0:t1][idx])


@pytest.mark.parametrize("dtype", [torch.bfloat16, torch.float32])
def test_compact_generic_gather(dtype):
    # token-level kept sets (not whole sentences): shift-by-one, every other row, random subset
    L, H, n_tok = 2, 3, 777
    st = _structure([[0, n_tok], [0, n_tok], [0, n_tok]])
    g = torch.Generator(device="cuda")
    g.manual_seed(5)
    k0 = torch.randn((L, H, st.total_tokens, 128), generator=g, device="cuda").to(dtype)
    v0 = torch.randn((L, H, st.total_tokens, 128), generator=g, device="cuda").to(dtype)
    k, v = k0.clone(), v0.clone()
    rng = np.random.default_rng(6)
    rows = [np.arange(1, n_tok), np.arange(0, n_tok, 2), np.sort(rng.choice(n_tok, 300, replace=False))]
    stride = n_tok
    kept = torch.full((L, H, 3, stride), -1, dtype=torch.int32, device="cuda")
    new_len = torch.zeros((L, H, 3), dtype=torch.int32, device="cuda")
    for b, r in enumerate(rows):
        kept[:, :, b, :len(r)] = torch.from_numpy(r.astype(np.int32)).cuda()
        new_len[:, :, b] = len(r)
    cfg = W.Config("gather", 9, 3, L, H, H, "bf16" if dtype == torch.bfloat16 else "f32", 0, 0, 0, 1, 1, 1.0, 0.0)
    B.skipkv_compact(make_cache(cfg, st, k, v), kept, new_len, stride)
    torch.cuda.synchronize()
    for b, r in enumerate(rows):
        t0 = int(st.seq_off[b])
        idx = torch.from_numpy(r).cuda() + t0
        assert torch.equal(k[:, :, t0:t0 + len(r)], k0[:, :, idx]) and torch.equal(v[:, :, t0:t0 + len(r)], v0[:, :, idx])


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_steer_add_matches_oracle_bit_for_bit(dtype):
    cfg = W.CONFIGS[4]
    dt = torch.bfloat16 if dtype == "bf16" else torch.float32
    h0, vec, coef = W.fill_steer(cfg, device="cuda")
    h0, vec = h0.to(dt), vec.to(dt)
    assert h0.shape == (64, 3584)
    # scalar coefficient on every row (the config's recipe)
    h = h0.clone()
    B.skipkv_steer_add(h, vec, None, coef, None)
    ref = oracle.steer_add(h0.double().cpu().numpy(), vec.double().cpu().numpy(), coef, dtype=dtype)
    np.testing.assert_array_equal(h.double().cpu().numpy(), ref)
    # adaptive per-sample strength alpha_0 + gamma * N_o and a delimiter-row mask
    n_o = torch.arange(64, device="cuda", dtype=torch.int32)
    coefs = torch.empty(64, dtype=torch.float32, device="cuda")
    B.skipkv_steer_strength(n_o, 1.0, 0.02, coefs)
    want = oracle.steer_strength(n_o.cpu().numpy(), np.float32(1.0), np.float32(0.02)).astype(np.float32)
    np.testing.assert_array_equal(coefs.cpu().numpy(), want)
    mask = (torch.arange(64, device="cuda") % 3 != 1).to(torch.uint8)
    h = h0.clone()
    B.skipkv_steer_add(h, vec, coefs, 0.0, mask)
    ref = oracle.steer_add(h0.double().cpu().numpy(), vec.double().cpu().numpy(), coefs.cpu().numpy(),
                           mask.cpu().numpy(), dtype=dtype)
    np.testing.assert_array_equal(h.double().cpu().numpy(), ref)


def test_step_replays_from_a_hip_graph():
    """The step allocates nothing, never synchronises and clears its counters with a fill kernel, so
    it can be captured into a HIP graph: every replay (with eager work and synchronisations between
    the replays) must reproduce the eager result bit for bit."""
    cfg = W.CONFIGS[3].scaled(n_layers=1, batch=3)
    st = W.make_structure(cfg)
    k0, v0, q = W.fill_cache(cfg, st, device="cuda")
    k, v = k0.clone(), v0.clone()
    eager = run_step(cfg, st, k, v, q)
    want = [t.clone() for t in (eager.sent_score, eager.sent_keep, eager.kept_idx, eager.new_len, k, v)]

    kg, vg = k0.clone(), v0.clone()
    cache = make_cache(cfg, st, kg, vg)
    status = torch.zeros(1, dtype=torch.int32, device="cuda")
    params = B.Params(cfg.obs_window, cfg.protect_window, cfg.budget, dev_status=status)
    ws = torch.empty(B.skipkv_workspace_bytes(cache, params), dtype=torch.uint8, device="cuda")
    L, H, Bn, S, T = cfg.n_layers, cfg.n_kv_heads, cfg.batch, st.total_sentences, st.total_tokens
    ks = min(cfg.budget, T)
    sent_score = torch.empty((L, H, S), dtype=torch.float32, device="cuda")
    sent_lambda = torch.empty_like(sent_score)
    sent_keep = torch.empty((L, H, S), dtype=torch.uint8, device="cuda")
    kept_idx = torch.empty((L, H, Bn, ks), dtype=torch.int32, device="cuda")
    new_len = torch.empty((L, H, Bn), dtype=torch.int32, device="cuda")
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        with torch.cuda.graph(graph, stream=side):
            B.skipkv_step(cache, params, q, None, sent_score, sent_lambda, None, sent_keep, kept_idx, new_len,
                          None, None, ks, ws)
    torch.cuda.synchronize()
    for rep in range(3):
        kg.copy_(k0)
        vg.copy_(v0)
        for t in (sent_score, kept_idx, new_len):
            t.fill_(-7)                       # eager work between the replays
        ws.fill_(0xAB if rep % 2 else 0)      # nothing in the workspace is carried from call to call
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert int(status.item()) == 0
        got = (sent_score, sent_keep, kept_idx, new_len, kg, vg)
        for name, g_, w_ in zip(("score", "keep", "kept_idx", "new_len", "K", "V"), got, want):
            if name == "kept_idx":  # entries beyond new_len are unspecified
                ar = torch.arange(ks, device="cuda")[None, None, None, :]
                valid = ar < new_len[..., None]
                assert torch.equal(g_[valid], w_[valid]), (rep, name)
            elif name in ("K", "V"):  # rows beyond new_len are unspecified
                for b in range(Bn):
                    t0 = int(st.seq_off[b])
                    for h in range(H):
                        n = int(new_len[0, h, b])
                        assert torch.equal(g_[0, h, t0:t0 + n], w_[0, h, t0:t0 + n]), (rep, name, h, b)
            else:
                assert torch.equal(g_.view(torch.uint8) if g_.dtype != torch.uint8 else g_,
                                   w_.view(torch.uint8) if w_.dtype != torch.uint8 else w_), (rep, name)


def _boundary_structure(sent_hi):
    rng = np.random.default_rng(sent_hi)
    lens = [15, 16, 17, 65, 255, 256, 257, 511, 512, 513, 1023, 1024, 1025, 1280]
    offsets = []
    for n in lens:
        off = [0]
        while off[-1] < n:
            off.append(min(n, off[-1] + int(rng.integers(1, sent_hi))))
        offsets.append(off)
    return _structure(offsets), lens


@pytest.mark.parametrize("dtype,sent_hi", [("bf16", 9), ("bf16", 2), ("f32", 40)])
def test_lengths_around_chunk_and_stage_edges(dtype, sent_hi):
    """Sequence lengths one below, at and one above the multiples of the scan's chunk (256 tokens) and
    stage (16 tokens) sizes, with short, one-token and long sentences: every head against the oracle."""
    st, lens = _boundary_structure(sent_hi)
    cfg = W.Config("edges", 9, len(lens), 1, 2, 8, dtype, 0, 0, 96, 8, 16, 16.0, 0.0)
    k0, v0, q = _random_kvq(cfg, st, 23 + sent_hi)
    k, v = k0.clone(), v0.clone()
    out = run_step(cfg, st, k, v, q)
    assert int(out.dev_status.item()) == 0
    stats = _compare_all(cfg, st, out, k, v, k0, v0, q)
    assert stats["heads"] == 2 * len(lens)

"""GPU parity of the step on a paged KV cache (block table): against the same step on the
contiguous cache (through the same form of the key scan: token importance, selection and the
compacted rows bit for bit) and against the oracle on sampled heads.  The pools are filled by scattering a seeded contiguous cache into randomly
permuted blocks; slots that hold no token carry a sentinel that must survive the step."""
import numpy as np
import pytest
import torch

from paper_2512_07993_amd import binding as B
from paper_2512_07993_amd import workloads as W

from helpers import GpuStep, compare_head, device_structure, oracle_head, run_step, sample_heads

pytestmark = pytest.mark.gpu

SENTINEL = -7.0


def _to_pages(cfg, st, k, v, block_size, seed, heads_before_slots=False, spare=3):
    """Pools [L, blocks, slots, Hk, D] (or the same shape as a view of [L, blocks, Hk, slots, D]) and
    the block table [B, max blocks per sequence] of a random placement."""
    L, H, T, D = k.shape
    lens = [int(st.seq_off[b + 1] - st.seq_off[b]) for b in range(cfg.batch)]
    nblk = [(n + block_size - 1) // block_size for n in lens]
    n_blocks = sum(nblk) + spare
    rng = np.random.default_rng(seed)
    perm = rng.permutation(n_blocks)
    table = np.full((cfg.batch, max(1, max(nblk)) + 2), -1, dtype=np.int32)
    pos = 0
    for b in range(cfg.batch):
        table[b, :nblk[b]] = perm[pos:pos + nblk[b]]
        pos += nblk[b]
    if heads_before_slots:
        kp = torch.full((L, n_blocks, H, block_size, D), SENTINEL, dtype=k.dtype, device=k.device).permute(0, 1, 3, 2, 4)
        vp = torch.full((L, n_blocks, H, block_size, D), SENTINEL, dtype=k.dtype, device=k.device).permute(0, 1, 3, 2, 4)
    else:
        kp = torch.full((L, n_blocks, block_size, H, D), SENTINEL, dtype=k.dtype, device=k.device)
        vp = torch.full((L, n_blocks, block_size, H, D), SENTINEL, dtype=k.dtype, device=k.device)
    blk, slot = _token_slots(cfg, st, table, block_size, k.device)
    kp[:, blk, slot] = k.permute(0, 2, 1, 3)
    vp[:, blk, slot] = v.permute(0, 2, 1, 3)
    return kp, vp, torch.from_numpy(table).to(k.device)


def _token_slots(cfg, st, table, block_size, device):
    blk = np.empty(st.total_tokens, dtype=np.int64)
    slot = np.empty(st.total_tokens, dtype=np.int64)
    for b in range(cfg.batch):
        t0, t1 = int(st.seq_off[b]), int(st.seq_off[b + 1])
        t = np.arange(t1 - t0)
        blk[t0:t1] = table[b, t // block_size]
        slot[t0:t1] = t % block_size
    return torch.from_numpy(blk).to(device), torch.from_numpy(slot).to(device)


def _from_pages(cfg, st, kp, table, block_size):
    blk, slot = _token_slots(cfg, st, table.cpu().numpy(), block_size, kp.device)
    return kp[:, blk, slot].permute(0, 2, 1, 3).contiguous()


def _run_paged(cfg, st, kp, vp, table, q):
    dev = kp.device
    so, sp, sf = device_structure(st, dev)
    cache = B.PagedCache(kp, vp, table, cfg.n_q_heads, so, sp, sf, st.total_tokens, st.total_sentences)
    L, H, Bn = cfg.n_layers, cfg.n_kv_heads, cfg.batch
    status = torch.zeros(1, dtype=torch.int32, device=dev)
    params = B.Params(cfg.obs_window, cfg.protect_window, cfg.budget, dev_status=status)
    ws = torch.empty(B.skipkv_paged_workspace_bytes(cache, params) + 256, dtype=torch.uint8, device=dev)
    S, T = st.total_sentences, st.total_tokens
    kept_stride = max(1, min(cfg.budget, T))
    out = GpuStep(
        cache, params,
        torch.full((L, H, S), float("nan"), dtype=torch.float32, device=dev),
        torch.full((L, H, S), float("nan"), dtype=torch.float32, device=dev),
        torch.full((L, H, T), float("nan"), dtype=torch.float32, device=dev),
        torch.full((L, H, S), 77, dtype=torch.uint8, device=dev),
        torch.full((L, H, Bn, kept_stride), -1, dtype=torch.int32, device=dev),
        torch.full((L, H, Bn), -1, dtype=torch.int32, device=dev),
        torch.full((L, H, S + Bn), -1, dtype=torch.int32, device=dev),
        torch.full((L, H, Bn), -1, dtype=torch.int32, device=dev),
        kept_stride, status)
    B.skipkv_step_paged(cache, params, q, None, out.sent_score, out.sent_lambda, out.tok_imp, out.sent_keep,
                        out.kept_idx, out.new_len, out.new_sent_off, out.new_sent_cnt, kept_stride, ws)
    torch.cuda.synchronize()
    return out


def _check_against_contiguous(cfg, block_size, heads_before_slots, monkeypatch, n_oracle_heads=4):
    st = W.make_structure(cfg)
    k0, v0, q = W.fill_cache(cfg, st, device="cuda")
    kp, vp, table = _to_pages(cfg, st, k0, v0, block_size, seed=block_size, heads_before_slots=heads_before_slots)
    kp0 = kp.clone()
    print("paged", cfg.name, "block", block_size, "blocks", kp.shape[1], "tokens", st.total_tokens, flush=True)
    out = _run_paged(cfg, st, kp, vp, table, q)
    assert int(out.dev_status.item()) == 0
    # the same step on the contiguous cache, through the same form of the key scan: blocks of a power
    # of two >= 16 slots take the single-pass scan, other sizes the two-pass one
    two_pass = block_size < 16 or (block_size & (block_size - 1)) != 0
    k, v = k0.clone(), v0.clone()
    ref = run_step(cfg, st, k, v, q, flags=B.FLAG_FORCE_TWO_PASS if two_pass else 0)
    for name in ("tok_imp", "sent_keep", "kept_idx", "new_len", "new_sent_off", "new_sent_cnt"):
        a, b = getattr(out, name), getattr(ref, name)
        assert torch.equal(a.view(torch.uint8) if a.dtype != torch.uint8 else a, b.view(torch.uint8) if b.dtype != torch.uint8 else b), name
    # both forms of the scan add a sentence's keys up in a fixed order: embeddings, lambda and scores are the same bits
    for name in ("sent_lambda", "sent_score"):
        a, b = getattr(out, name), getattr(ref, name)
        assert torch.equal(a.view(torch.int32), b.view(torch.int32)), name
    kg, vg = _from_pages(cfg, st, kp, table, block_size), _from_pages(cfg, st, vp, table, block_size)
    new_len = out.new_len.cpu().numpy()
    for b in range(cfg.batch):
        t0 = int(st.seq_off[b])
        for l in range(cfg.n_layers):
            for h in range(cfg.n_kv_heads):
                n = int(new_len[l, h, b])
                assert torch.equal(kg[l, h, t0:t0 + n].view(torch.uint8), k[l, h, t0:t0 + n].view(torch.uint8)), (l, h, b)
                assert torch.equal(vg[l, h, t0:t0 + n].view(torch.uint8), v[l, h, t0:t0 + n].view(torch.uint8)), (l, h, b)
    # slots that hold no token were not written
    blk, slot = _token_slots(cfg, st, table.cpu().numpy(), block_size, kp.device)
    free = torch.ones(kp.shape[1], kp.shape[2], dtype=torch.bool, device=kp.device)
    free[blk, slot] = False
    assert torch.equal(kp[:, free].view(torch.uint8), kp0[:, free].view(torch.uint8))
    assert bool((vp[:, free] == SENTINEL).all())
    # and against the oracle
    stats = {}
    for (l, h, b) in sample_heads(cfg, st, n_oracle_heads, seed=block_size):
        ora = oracle_head(cfg, st, k0, v0, q, l, h, b)
        compare_head(cfg, st, out, kg, vg, k0, v0, ora, l, h, b, stats)
    print(stats, flush=True)


@pytest.mark.parametrize("block_size,heads_before_slots", [(16, False), (16, True), (24, False), (128, True), (8, False)])
def test_paged_step_matches_contiguous_and_oracle(block_size, heads_before_slots, monkeypatch):
    _check_against_contiguous(W.CONFIGS[3].scaled(n_layers=2, batch=4), block_size, heads_before_slots, monkeypatch)


def test_paged_step_config3_full_size(monkeypatch):
    """The workload that bench.py --paged 16 times (all 32 layers, 16 sequences, 9678 blocks of 16 slots): every
    head bit for bit against the contiguous step, sampled heads against the oracle."""
    _check_against_contiguous(W.CONFIGS[3], 16, False, monkeypatch, n_oracle_heads=6)


def test_paged_step_fp32(monkeypatch):
    _check_against_contiguous(W.CONFIGS[1], 16, False, monkeypatch, n_oracle_heads=3)


def test_paged_step_gqa7(monkeypatch):
    _check_against_contiguous(W.CONFIGS[4].scaled(n_layers=1, batch=3), 32, False, monkeypatch, n_oracle_heads=3)


def test_bad_block_id_is_reported_and_that_sequence_left_alone():
    cfg = W.CONFIGS[3].scaled(n_layers=1, batch=3)
    st = W.make_structure(cfg)
    k0, v0, q = W.fill_cache(cfg, st, device="cuda")
    kp, vp, table = _to_pages(cfg, st, k0, v0, 16, seed=5)
    table[1, 3] = kp.shape[1] + 9          # out of range
    kp0, vp0 = kp.clone(), vp.clone()
    out = _run_paged(cfg, st, kp, vp, table, q)
    assert int(out.dev_status.item()) & B.DEV_BAD_BLOCK_TABLE
    # the blocks of sequence 1 hold what they held
    n1 = (int(st.seq_off[2] - st.seq_off[1]) + 15) // 16
    own = table[1, :n1].cpu().numpy()
    own = torch.from_numpy(own[(own >= 0) & (own < kp.shape[1])].astype(np.int64)).to(kp.device)
    assert torch.equal(kp[:, own].view(torch.uint8), kp0[:, own].view(torch.uint8))
    assert torch.equal(vp[:, own].view(torch.uint8), vp0[:, own].view(torch.uint8))
    new_len = out.new_len.cpu().numpy()
    assert (new_len >= 0).all() and (new_len <= cfg.budget).all()


@pytest.mark.parametrize("block_size", [16, 1])
def test_paged_degenerate_batch(block_size):
    """The ragged and degenerate sequences of the edge tests (an empty sequence, one shorter than the
    observation window, one that fits its budget, a 700-token sentence that takes its sequence to the
    two-pass scan, 300 one-token sentences) on a paged cache, every head against the oracle."""
    from test_gpu_edges import _compare_all, _edge_cfg, _edge_offsets, _random_kvq, _structure
    cfg = _edge_cfg("bf16")
    st = _structure(_edge_offsets())
    k0, v0, q = _random_kvq(cfg, st, 11)
    kp, vp, table = _to_pages(cfg, st, k0, v0, block_size, seed=3)
    kp0 = kp.clone()
    out = _run_paged(cfg, st, kp, vp, table, q)
    assert int(out.dev_status.item()) == 0
    kg, vg = _from_pages(cfg, st, kp, table, block_size), _from_pages(cfg, st, vp, table, block_size)
    stats = _compare_all(cfg, st, out, kg, vg, k0, v0, q)
    assert stats["heads"] == 8
    for b in (1, 2):     # sequences that fit are untouched, bit for bit
        t0, t1 = int(st.seq_off[b]), int(st.seq_off[b + 1])
        assert torch.equal(kg[:, :, t0:t1], k0[:, :, t0:t1]) and torch.equal(vg[:, :, t0:t1], v0[:, :, t0:t1])
    blk, slot = _token_slots(cfg, st, table.cpu().numpy(), block_size, kp.device)
    free = torch.ones(kp.shape[1], kp.shape[2], dtype=torch.bool, device=kp.device)
    free[blk, slot] = False
    assert torch.equal(kp[:, free].view(torch.uint8), kp0[:, free].view(torch.uint8))


def _paged_cache(cfg, st, kp, vp, table):
    so, sp, sf = device_structure(st, kp.device)
    return B.PagedCache(kp, vp, table, cfg.n_q_heads, so, sp, sf, st.total_tokens, st.total_sentences)


@pytest.mark.parametrize("block_size", [16, 24])
def test_score_select_compact_on_pages_equal_the_paged_step(block_size):
    cfg = W.CONFIGS[3].scaled(n_layers=2, batch=4)
    st = W.make_structure(cfg)
    k0, v0, q = W.fill_cache(cfg, st, device="cuda")
    kp, vp, table = _to_pages(cfg, st, k0, v0, block_size, seed=21)
    ka, va = kp.clone(), vp.clone()
    ref = _run_paged(cfg, st, ka, va, table, q)
    assert int(ref.dev_status.item()) == 0
    cache = _paged_cache(cfg, st, kp, vp, table)
    L, H, Bn, S, T = cfg.n_layers, cfg.n_kv_heads, cfg.batch, st.total_sentences, st.total_tokens
    status = torch.zeros(1, dtype=torch.int32, device="cuda")
    params = B.Params(cfg.obs_window, cfg.protect_window, cfg.budget, dev_status=status)
    ws = torch.empty(B.skipkv_paged_workspace_bytes(cache, params) + 256, dtype=torch.uint8, device="cuda")
    score = torch.full((L, H, S), float("nan"), dtype=torch.float32, device="cuda")
    lam, imp = torch.full_like(score, float("nan")), torch.full((L, H, T), float("nan"), dtype=torch.float32, device="cuda")
    B.skipkv_score_paged(cache, params, q, None, score, lam, imp, ws)
    torch.cuda.synchronize()  # scoring alone wrote nothing into the pools:
    assert torch.equal(kp.view(torch.uint8), _to_pages(cfg, st, k0, v0, block_size, seed=21)[0].view(torch.uint8))
    kept_stride = ref.kept_stride
    keep = torch.full((L, H, S), 77, dtype=torch.uint8, device="cuda")
    kept_idx = torch.full((L, H, Bn, kept_stride), -1, dtype=torch.int32, device="cuda")
    new_len = torch.full((L, H, Bn), -1, dtype=torch.int32, device="cuda")
    new_off = torch.full((L, H, S + Bn), -1, dtype=torch.int32, device="cuda")
    new_cnt = torch.full((L, H, Bn), -1, dtype=torch.int32, device="cuda")
    B.skipkv_select(cache, params, score, keep, kept_idx, new_len, new_off, new_cnt, kept_stride)
    ws2 = torch.empty(B.skipkv_compact_paged_workspace_bytes(cache, kept_stride) + 256, dtype=torch.uint8, device="cuda")
    B.skipkv_compact_paged(cache, kept_idx, new_len, kept_stride, status, ws2)
    torch.cuda.synchronize()
    assert int(status.item()) == 0
    assert torch.equal(imp.view(torch.int32), ref.tok_imp.view(torch.int32))
    # blocks of 24 slots take the two-pass scan, whose pooling order varies from run to run
    if block_size == 16:
        assert torch.equal(score.view(torch.int32), ref.sent_score.view(torch.int32)) and torch.equal(lam.view(torch.int32), ref.sent_lambda.view(torch.int32))
    else:
        torch.testing.assert_close(score, ref.sent_score, rtol=1e-5, atol=1e-6)
        torch.testing.assert_close(lam, ref.sent_lambda, rtol=1e-5, atol=1e-6)
    assert torch.equal(keep, ref.sent_keep) and torch.equal(new_len, ref.new_len) and torch.equal(new_cnt, ref.new_sent_cnt)
    assert torch.equal(kept_idx, ref.kept_idx) and torch.equal(new_off, ref.new_sent_off)
    # the pools end up the same wherever a kept token lives (rows past the new lengths are unspecified)
    kg, vg = _from_pages(cfg, st, kp, table, block_size), _from_pages(cfg, st, vp, table, block_size)
    kr, vr = _from_pages(cfg, st, ka, table, block_size), _from_pages(cfg, st, va, table, block_size)
    nl = new_len.cpu().numpy()
    for l in range(L):
        for h in range(H):
            for b in range(Bn):
                t0, n = int(st.seq_off[b]), int(nl[l, h, b])
                assert torch.equal(kg[l, h, t0:t0 + n].view(torch.uint8), kr[l, h, t0:t0 + n].view(torch.uint8)), (l, h, b)
                assert torch.equal(vg[l, h, t0:t0 + n].view(torch.uint8), vr[l, h, t0:t0 + n].view(torch.uint8)), (l, h, b)


def test_token_level_flow_on_pages_equals_the_contiguous_one():
    """token redundancy -> score -> token-level selection (Eq. 6 as printed) -> compaction, on pages and on the
    contiguous cache."""
    from helpers import make_cache
    cfg = W.CONFIGS[3].scaled(n_layers=1, batch=3)
    st = W.make_structure(cfg)
    k0, v0, q = W.fill_cache(cfg, st, device="cuda")
    L, H, Bn, S, T = cfg.n_layers, cfg.n_kv_heads, cfg.batch, st.total_sentences, st.total_tokens
    flat = make_cache(cfg, st, k0, v0)
    red = torch.empty((L, H, T), dtype=torch.float32, device="cuda")
    B.skipkv_token_redundancy(flat, red, torch.empty(B.skipkv_redundancy_workspace_bytes(flat) + 256, dtype=torch.uint8, device="cuda"))
    kept_stride = min(cfg.budget, T)
    kp, vp, table = _to_pages(cfg, st, k0, v0, 16, seed=33)
    paged_cache = _paged_cache(cfg, st, kp, vp, table)
    red_p = torch.full((L, H, T), float("nan"), dtype=torch.float32, device="cuda")
    st_r = torch.zeros(1, dtype=torch.int32, device="cuda")
    B.skipkv_token_redundancy_paged(paged_cache, red_p, st_r, torch.empty(
        B.skipkv_redundancy_paged_workspace_bytes(paged_cache) + 256, dtype=torch.uint8, device="cuda"))
    torch.cuda.synchronize()
    assert int(st_r.item()) == 0
    assert torch.equal(red_p.view(torch.int32), red.view(torch.int32))   # same rows, same order of operations

    def flow(cache, paged):
        status = torch.zeros(1, dtype=torch.int32, device="cuda")
        params = B.Params(cfg.obs_window, cfg.protect_window, cfg.budget, dev_status=status)
        score = torch.empty((L, H, S), dtype=torch.float32, device="cuda")
        lam, imp = torch.empty_like(score), torch.empty((L, H, T), dtype=torch.float32, device="cuda")
        if paged:
            ws = torch.empty(B.skipkv_paged_workspace_bytes(cache, params) + 256, dtype=torch.uint8, device="cuda")
            B.skipkv_score_paged(cache, params, q, red, score, lam, imp, ws)
        else:
            ws = torch.empty(B.skipkv_workspace_bytes(cache, params) + 256, dtype=torch.uint8, device="cuda")
            B.skipkv_score(cache, params, q, red, score, lam, imp, ws)
        tok_score = torch.empty((L, H, T), dtype=torch.float32, device="cuda")
        tok_keep = torch.empty((L, H, T), dtype=torch.uint8, device="cuda")
        kept_idx = torch.full((L, H, Bn, kept_stride), -1, dtype=torch.int32, device="cuda")
        new_len = torch.empty((L, H, Bn), dtype=torch.int32, device="cuda")
        new_off = torch.full((L, H, S + Bn), -1, dtype=torch.int32, device="cuda")
        new_cnt = torch.empty((L, H, Bn), dtype=torch.int32, device="cuda")
        B.skipkv_select_tokens(cache, params, imp, red, lam, tok_score, tok_keep, kept_idx, new_len, new_off, new_cnt, kept_stride)
        if paged:
            ws2 = torch.empty(B.skipkv_compact_paged_workspace_bytes(cache, kept_stride) + 256, dtype=torch.uint8, device="cuda")
            B.skipkv_compact_paged(cache, kept_idx, new_len, kept_stride, status, ws2)
        else:
            B.skipkv_compact(cache, kept_idx, new_len, kept_stride)
        torch.cuda.synchronize()
        assert int(status.item()) == 0
        return tok_score, tok_keep, kept_idx, new_len, new_off, new_cnt

    k, v = k0.clone(), v0.clone()
    a = flow(make_cache(cfg, st, k, v), False)
    b = flow(paged_cache, True)
    for x, y in zip(a, b):
        assert torch.equal(x.view(torch.uint8) if x.dtype != torch.uint8 else x, y.view(torch.uint8) if y.dtype != torch.uint8 else y)
    kg, vg = _from_pages(cfg, st, kp, table, 16), _from_pages(cfg, st, vp, table, 16)
    nl = a[3].cpu().numpy()
    assert (nl == np.minimum(cfg.budget, st.seq_len)[None, None, :]).all()
    for h in range(H):
        for s in range(Bn):
            t0, n = int(st.seq_off[s]), int(nl[0, h, s])
            assert torch.equal(kg[0, h, t0:t0 + n], k[0, h, t0:t0 + n]) and torch.equal(vg[0, h, t0:t0 + n], v[0, h, t0:t0 + n])


@pytest.mark.parametrize("config_id,block_size,heads_before_slots", [(1, 8, False), (3, 24, True)])
def test_token_redundancy_on_pages_equals_the_contiguous_one(config_id, block_size, heads_before_slots):
    from helpers import make_cache
    cfg = W.CONFIGS[config_id] if config_id == 1 else W.CONFIGS[config_id].scaled(n_layers=1, batch=3, len_lo=200, len_hi=1500)
    st = W.make_structure(cfg)
    k0, v0, q = W.fill_cache(cfg, st, device="cuda")
    L, H, T = cfg.n_layers, cfg.n_kv_heads, st.total_tokens
    flat = make_cache(cfg, st, k0, v0)
    red = torch.empty((L, H, T), dtype=torch.float32, device="cuda")
    B.skipkv_token_redundancy(flat, red, torch.empty(B.skipkv_redundancy_workspace_bytes(flat) + 256, dtype=torch.uint8, device="cuda"))
    kp, vp, table = _to_pages(cfg, st, k0, v0, block_size, seed=5, heads_before_slots=heads_before_slots)
    cache = _paged_cache(cfg, st, kp, vp, table)
    red_p = torch.full((L, H, T), float("nan"), dtype=torch.float32, device="cuda")
    status = torch.zeros(1, dtype=torch.int32, device="cuda")
    B.skipkv_token_redundancy_paged(cache, red_p, status, torch.empty(
        B.skipkv_redundancy_paged_workspace_bytes(cache) + 256, dtype=torch.uint8, device="cuda"))
    torch.cuda.synchronize()
    assert int(status.item()) == 0
    assert torch.equal(red_p.view(torch.int32), red.view(torch.int32))
    # R sums to 1 over the tokens of every head and sequence (Eq. 5)
    for b in range(cfg.batch):
        t0, t1 = int(st.seq_off[b]), int(st.seq_off[b + 1])
        if t1 > t0:
            torch.testing.assert_close(red_p[:, :, t0:t1].double().sum(-1), torch.ones((L, H), dtype=torch.float64, device="cuda"), rtol=1e-4, atol=0)


def test_scores_with_shared_lambda_on_pages_equal_the_contiguous_ones():
    from helpers import make_cache
    cfg = W.CONFIGS[3].scaled(n_layers=2, batch=3, len_lo=500, len_hi=2500, budget=512)
    st = W.make_structure(cfg)
    k0, v0, q = W.fill_cache(cfg, st, device="cuda")
    L, H, S, T = cfg.n_layers, cfg.n_kv_heads, st.total_sentences, st.total_tokens
    lam = torch.from_numpy(np.random.default_rng(2).uniform(0.5, 1.0, S).astype(np.float32)).cuda()
    status = torch.zeros(1, dtype=torch.int32, device="cuda")
    params = B.Params(cfg.obs_window, cfg.protect_window, cfg.budget, dev_status=status)
    flat = make_cache(cfg, st, k0, v0)
    sa, la, ia = (torch.full(s, float("nan"), dtype=torch.float32, device="cuda") for s in ((L, H, S), (L, H, S), (L, H, T)))
    B.skipkv_score_shared(flat, params, q, None, lam, sa, la, ia, torch.empty(B.skipkv_workspace_bytes(flat, params) + 256, dtype=torch.uint8, device="cuda"))
    kp, vp, table = _to_pages(cfg, st, k0, v0, 16, seed=12)
    cache = _paged_cache(cfg, st, kp, vp, table)
    sb, lb, ib = (torch.full(s, float("nan"), dtype=torch.float32, device="cuda") for s in ((L, H, S), (L, H, S), (L, H, T)))
    B.skipkv_score_shared_paged(cache, params, q, None, lam, sb, lb, ib, torch.empty(B.skipkv_paged_workspace_bytes(cache, params) + 256, dtype=torch.uint8, device="cuda"))
    torch.cuda.synchronize()
    assert int(status.item()) == 0
    for x, y in ((sa, sb), (la, lb), (ia, ib)):
        assert torch.equal(x.view(torch.int32), y.view(torch.int32))
    assert torch.equal(la, lam.expand(L, H, S))


@pytest.mark.parametrize("block_size,sent_hi", [(16, 9), (64, 2), (32, 40)])
def test_paged_lengths_around_chunk_stage_and_block_edges(block_size, sent_hi):
    """Sequence lengths one below, at and one above the multiples of the scan's chunk and stage sizes
    (and so of the blocks) on a paged cache, every head against the oracle."""
    from test_gpu_edges import _boundary_structure, _compare_all, _random_kvq
    st, lens = _boundary_structure(sent_hi)
    cfg = W.Config("edges", 9, len(lens), 1, 2, 8, "bf16", 0, 0, 96, 8, 16, 16.0, 0.0)
    k0, v0, q = _random_kvq(cfg, st, 50 + block_size)
    kp, vp, table = _to_pages(cfg, st, k0, v0, block_size, seed=block_size + 7)
    out = _run_paged(cfg, st, kp, vp, table, q)
    assert int(out.dev_status.item()) == 0
    kg, vg = _from_pages(cfg, st, kp, table, block_size), _from_pages(cfg, st, vp, table, block_size)
    stats = _compare_all(cfg, st, out, kg, vg, k0, v0, q)
    assert stats["heads"] == 2 * len(lens)

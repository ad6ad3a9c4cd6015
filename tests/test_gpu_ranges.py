"""Per-head sentence ranges across compression steps (Sec. 4.1, Eq. 9-11) through the C ABI:
the append rule against the oracle, the per-head step against the shared-range step where both
describe the same cache, and a two-step decode-like pipeline against the oracle head by head."""
import numpy as np
import pytest
import torch

import oracle
from paper_2512_07993_amd import binding as B
from paper_2512_07993_amd import workloads as W
from helpers import GpuStep, compare_head, make_cache, run_step

pytestmark = pytest.mark.gpu


def _outputs(cfg, st, kept_stride, want_tok_imp=True):
    dev = "cuda"
    L, H, Bn, S, T = cfg.n_layers, cfg.n_kv_heads, cfg.batch, st.total_sentences, st.total_tokens
    return dict(
        sent_score=torch.full((L, H, S), float("nan"), dtype=torch.float32, device=dev),
        sent_lambda=torch.full((L, H, S), float("nan"), dtype=torch.float32, device=dev),
        tok_imp=torch.full((L, H, T), float("nan"), dtype=torch.float32, device=dev) if want_tok_imp else None,
        sent_keep=torch.full((L, H, S), 77, dtype=torch.uint8, device=dev),
        kept_idx=torch.full((L, H, Bn, kept_stride), -1, dtype=torch.int32, device=dev),
        new_len=torch.full((L, H, Bn), -1, dtype=torch.int32, device=dev),
        new_sent_off=torch.full((L, H, S + Bn), -1, dtype=torch.int32, device=dev),
        new_sent_cnt=torch.full((L, H, Bn), -1, dtype=torch.int32, device=dev))


def run_step_ranges(cfg, st, k, v, q, ranges, budget, flags=0):
    cache = make_cache(cfg, st, k, v)
    status = torch.zeros(1, dtype=torch.int32, device="cuda")
    params = B.Params(cfg.obs_window, cfg.protect_window, budget, dev_status=status, flags=flags)
    ws = torch.empty(B.skipkv_ranges_workspace_bytes(cache, params) + 256, dtype=torch.uint8, device="cuda")
    kept_stride = max(1, min(budget, st.total_tokens))
    o = _outputs(cfg, st, kept_stride)
    B.skipkv_step_ranges(cache, ranges, params, q, None, o["sent_score"], o["sent_lambda"], o["tok_imp"], o["sent_keep"],
                         o["kept_idx"], o["new_len"], o["new_sent_off"], o["new_sent_cnt"], kept_stride, ws)
    torch.cuda.synchronize()
    return GpuStep(cache, params, o["sent_score"], o["sent_lambda"], o["tok_imp"], o["sent_keep"], o["kept_idx"],
                   o["new_len"], o["new_sent_off"], o["new_sent_cnt"], kept_stride, status)


def shared_as_ranges(cfg, st):
    """The shared structure written out per head."""
    L, H, Bn = cfg.n_layers, cfg.n_kv_heads, cfg.batch
    ln = torch.from_numpy(st.seq_len.astype(np.int32)).cuda().expand(L, H, Bn).contiguous()
    cnt = torch.from_numpy(st.n_sent.astype(np.int32)).cuda().expand(L, H, Bn).contiguous()
    off = torch.from_numpy(st.sent_off.astype(np.int32)).cuda().expand(L, H, st.sent_off.size).contiguous()
    return B.Ranges(ln, cnt, off)


@pytest.mark.parametrize("config_id,kw", [
    (2, dict(n_layers=2, len_lo=1500, len_hi=1500, budget=640)),
    (3, dict(n_layers=1, batch=5, len_lo=300, len_hi=2600, budget=512)),
    (4, dict(n_layers=2, batch=3, len_lo=700, len_hi=1800, budget=512)),
    (3, dict()),  # the workload that bench.py --ranges times, at full size
])
def test_per_head_step_equals_shared_step_on_the_same_cache(config_id, kw):
    cfg = W.CONFIGS[config_id].scaled(**kw)
    st = W.make_structure(cfg)
    k0, v0, q = W.fill_cache(cfg, st, device="cuda")
    ka, va = k0.clone(), v0.clone()
    a = run_step(cfg, st, ka, va, q)
    kb, vb = k0.clone(), v0.clone()
    b = run_step_ranges(cfg, st, kb, vb, q, shared_as_ranges(cfg, st), cfg.budget)
    assert int(a.dev_status.item()) == 0 and int(b.dev_status.item()) == 0
    # the same kernels on the same numbers: everything is bit-identical
    for name in ("sent_score", "sent_lambda", "tok_imp", "sent_keep", "new_len", "new_sent_cnt"):
        x, y = getattr(a, name), getattr(b, name)
        assert torch.equal(x.view(torch.uint8), y.view(torch.uint8)), name
    L, H, Bn = cfg.n_layers, cfg.n_kv_heads, cfg.batch
    new_len, new_cnt = a.new_len.cpu().numpy(), a.new_sent_cnt.cpu().numpy()
    for l in range(L):
        for h in range(H):
            for s in range(Bn):
                n = int(new_len[l, h, s])
                assert torch.equal(a.kept_idx[l, h, s, :n], b.kept_idx[l, h, s, :n])
                c = int(new_cnt[l, h, s])
                p = int(st.sent_ptr[s])
                assert torch.equal(a.new_sent_off[l, h, p:p + c + 1], b.new_sent_off[l, h, p:p + c + 1])
                t0 = int(st.seq_off[s])
                assert torch.equal(ka[l, h, t0:t0 + n], kb[l, h, t0:t0 + n]) and torch.equal(va[l, h, t0:t0 + n], vb[l, h, t0:t0 + n])


def _assert_same_step(cfg, st, a, ka, va, b, kb, vb):
    for name in ("sent_score", "sent_lambda", "tok_imp", "sent_keep", "new_len", "new_sent_cnt"):
        x, y = getattr(a, name), getattr(b, name)
        assert torch.equal(x.view(torch.uint8), y.view(torch.uint8)), name
    for l in range(cfg.n_layers):
        for h in range(cfg.n_kv_heads):
            for s in range(cfg.batch):
                n = int(a.new_len[l, h, s])
                assert torch.equal(a.kept_idx[l, h, s, :n], b.kept_idx[l, h, s, :n])
                t0 = int(st.seq_off[s])
                assert torch.equal(ka[l, h, t0:t0 + n], kb[l, h, t0:t0 + n]) and torch.equal(va[l, h, t0:t0 + n], vb[l, h, t0:t0 + n])


def test_per_head_step_through_the_two_pass_scan():
    two = B.FLAG_FORCE_TWO_PASS
    cfg = W.CONFIGS[4].scaled(n_layers=1, batch=3, len_lo=500, len_hi=1300, budget=384)
    st = W.make_structure(cfg)
    k0, v0, q = W.fill_cache(cfg, st, device="cuda")
    ka, va = k0.clone(), v0.clone()
    a = run_step(cfg, st, ka, va, q, flags=two)
    kb, vb = k0.clone(), v0.clone()
    b = run_step_ranges(cfg, st, kb, vb, q, shared_as_ranges(cfg, st), cfg.budget, flags=two)
    assert int(a.dev_status.item()) == 0 and int(b.dev_status.item()) == 0
    _assert_same_step(cfg, st, a, ka, va, b, kb, vb)


def test_per_head_step_on_degenerate_sequences():
    # empty sequence, shorter than the window, fits the budget, a 700-token sentence (two-pass scan),
    # 300 one-token sentences
    from test_gpu_edges import _edge_cfg, _edge_offsets, _random_kvq, _structure
    cfg = _edge_cfg("bf16")
    st = _structure(_edge_offsets())
    k0, v0, q = _random_kvq(cfg, st, 11)
    ka, va = k0.clone(), v0.clone()
    a = run_step(cfg, st, ka, va, q)
    kb, vb = k0.clone(), v0.clone()
    b = run_step_ranges(cfg, st, kb, vb, q, shared_as_ranges(cfg, st), cfg.budget)
    assert int(a.dev_status.item()) == 0 and int(b.dev_status.item()) == 0
    _assert_same_step(cfg, st, a, ka, va, b, kb, vb)


def test_per_head_length_beyond_the_room_is_reported():
    cfg = W.CONFIGS[3].scaled(n_layers=1, n_kv_heads=2, n_q_heads=8, batch=2, len_lo=400, len_hi=700, budget=256)
    st = W.make_structure(cfg)
    k0, v0, q = W.fill_cache(cfg, st, device="cuda")
    r = shared_as_ranges(cfg, st)
    r.len[0, 1, 0] += 5  # more tokens than the sequence's rows can hold
    out = run_step_ranges(cfg, st, k0.clone(), v0.clone(), q, r, cfg.budget)
    assert int(out.dev_status.item()) & B.DEV_BAD_OFFSETS


def test_ranges_append_matches_oracle_and_reports_overflow():
    rng = np.random.default_rng(11)
    L, H, Bn = 2, 3, 4
    cap_s = np.array([12, 40, 6, 25])
    cap_t = np.array([400, 900, 50, 300])
    seq_off = np.concatenate([[0], np.cumsum(cap_t)]).astype(np.int32)
    sent_ptr = np.concatenate([[0], np.cumsum(cap_s + 1)]).astype(np.int32)
    S_tot, T_tot = int(cap_s.sum()), int(cap_t.sum())
    ln = np.zeros((L, H, Bn), np.int32)
    cnt = np.zeros((L, H, Bn), np.int32)
    off = np.full((L, H, S_tot + Bn), -7, np.int32)
    heads = {}
    for l in range(L):
        for h in range(H):
            for b in range(Bn):
                s = int(rng.integers(0, cap_s[b] // 2 + 1))
                if b == 2:
                    s = cap_s[b] - 1  # nearly full: one more sentence fits, two do not
                o = np.concatenate([[0], np.sort(rng.choice(np.arange(1, cap_t[b] // 2), size=s, replace=False))]) if s else np.array([0])
                heads[(l, h, b)] = o.astype(np.int64)
                ln[l, h, b], cnt[l, h, b] = o[-1], s
                off[l, h, sent_ptr[b]:sent_ptr[b] + s + 1] = o
    n_new = np.array([30, 55, 9, 0], np.int32)
    bnds = [np.array([0, 7, 20]), np.array([3, 4, 50]), np.array([0, 5]), np.array([], int)]
    bnd_ptr = np.concatenate([[0], np.cumsum([len(x) for x in bnds])]).astype(np.int32)
    bnd_off = np.concatenate(bnds).astype(np.int32)
    dev = lambda a: torch.from_numpy(np.ascontiguousarray(a)).cuda()
    k = torch.zeros((L, H, T_tot, 128), dtype=torch.bfloat16, device="cuda")
    cache = B.Cache(k, k, H * 4, dev(seq_off), dev(sent_ptr), dev(np.zeros(S_tot + Bn, np.int32)), T_tot, S_tot)
    r = B.Ranges(dev(ln), dev(cnt), dev(off))
    status = torch.zeros(1, dtype=torch.int32, device="cuda")
    B.skipkv_ranges_append(cache, r, dev(n_new), dev(bnd_ptr), dev(bnd_off), status)
    torch.cuda.synchronize()
    got_len, got_cnt, got_off = r.len.cpu().numpy(), r.sent_cnt.cpu().numpy(), r.sent_off.cpu().numpy()
    assert int(status.item()) == B.DEV_TOO_MANY_SENT  # sequence 2: two new sentences do not fit
    for (l, h, b), o in heads.items():
        if b == 2 or n_new[b] == 0:  # unchanged
            want = o
        else:
            want = oracle.append_ranges(o, int(n_new[b]), bnds[b])
        assert got_len[l, h, b] == want[-1] and got_cnt[l, h, b] == len(want) - 1, (l, h, b)
        np.testing.assert_array_equal(got_off[l, h, sent_ptr[b]:sent_ptr[b] + len(want)], want)


class _HeadView:
    """What compare_head reads from a Structure, for one head with its own length and ranges."""

    def __init__(self, st, b, n_tok, off):
        self.seq_off = {b: int(st.seq_off[b]), b + 1: int(st.seq_off[b]) + int(n_tok)}
        self.sent_ptr = st.sent_ptr
        self.n_sent = {b: len(off) - 1}
        self._off, self._b, self._base = np.asarray(off), b, int(st.sent_ptr[b]) - b

    def sent_base(self, b):
        return self._base

    def offsets(self, b):
        return self._off


def test_two_steps_with_appended_tokens_match_the_oracle_head_by_head():
    cfg = W.CONFIGS[3].scaled(n_layers=2, n_kv_heads=2, n_q_heads=8, batch=3, len_lo=900, len_hi=2200, budget=512)
    st = W.make_structure(cfg)
    k0, v0, q1 = W.fill_cache(cfg, st, device="cuda")
    k, v = k0.clone(), v0.clone()
    s1 = run_step(cfg, st, k, v, q1)
    assert int(s1.dev_status.item()) == 0
    L, H, Bn = cfg.n_layers, cfg.n_kv_heads, cfg.batch
    assert len({int(x) for x in s1.new_len.flatten()}) > 1  # heads really differ after the first step

    # decode-like phase: every sequence receives new tokens (the same text for every head), the
    # caller writes their K/V rows behind each head's own length
    rng = np.random.default_rng(3)
    g = torch.Generator(device="cuda")
    g.manual_seed(99)
    n_new = rng.integers(40, 120, size=Bn).astype(np.int32)
    bnds = [np.unique(np.concatenate([[0] if rng.random() < 0.5 else [], rng.choice(np.arange(1, n), size=3, replace=False)])).astype(np.int32)
            for n in n_new]
    bnd_ptr = np.concatenate([[0], np.cumsum([len(x) for x in bnds])]).astype(np.int32)
    dev = lambda a: torch.from_numpy(np.ascontiguousarray(a)).cuda()
    ranges = B.Ranges(s1.new_len.clone(), s1.new_sent_cnt.clone(), s1.new_sent_off.clone())
    len1 = s1.new_len.cpu().numpy()
    for l in range(L):
        for h in range(H):
            for b in range(Bn):
                t = int(st.seq_off[b]) + int(len1[l, h, b])
                n = int(n_new[b])
                k[l, h, t:t + n] = torch.randn((n, 128), generator=g, device="cuda").to(k.dtype)
                v[l, h, t:t + n] = torch.randn((n, 128), generator=g, device="cuda").to(v.dtype)
    status = torch.zeros(1, dtype=torch.int32, device="cuda")
    B.skipkv_ranges_append(s1.cache, ranges, dev(n_new), dev(bnd_ptr), dev(np.concatenate(bnds).astype(np.int32)), status)
    torch.cuda.synchronize()
    assert int(status.item()) == 0
    q2 = torch.randn(q1.shape, generator=g, device="cuda").to(q1.dtype)
    k_in, v_in = k.clone(), v.clone()
    s2 = run_step_ranges(cfg, st, k, v, q2, ranges, cfg.budget)
    assert int(s2.dev_status.item()) == 0

    len2, cnt2, off2 = ranges.len.cpu().numpy(), ranges.sent_cnt.cpu().numpy(), ranges.sent_off.cpu().numpy()
    off1 = s1.new_sent_off.cpu().numpy()
    cnt1 = s1.new_sent_cnt.cpu().numpy()
    stats = {}
    n = cfg.group
    for l in range(L):
        for h in range(H):
            for b in range(Bn):
                p = int(st.sent_ptr[b])
                # ranges after the append: the oracle's rule on the first step's output
                want_off = oracle.append_ranges(off1[l, h, p:p + cnt1[l, h, b] + 1], int(n_new[b]), bnds[b])
                got_off = off2[l, h, p:p + cnt2[l, h, b] + 1]
                np.testing.assert_array_equal(got_off, want_off)
                assert len2[l, h, b] == want_off[-1]
                # second step of this head against the oracle on exactly its rows
                t0, N = int(st.seq_off[b]), int(len2[l, h, b])
                kk = k_in[l, h, t0:t0 + N].to(torch.float64).cpu().numpy()
                vv = v_in[l, h, t0:t0 + N].to(torch.float64).cpu().numpy()
                qq = q2[l, b, h * n:(h + 1) * n].to(torch.float64).cpu().numpy()
                ora = oracle.compress_head(qq, kk, vv, want_off, cfg.budget, cfg.protect_window)
                hv = _HeadView(st, b, N, want_off)
                compare_head(cfg, hv, s2, k, v, k_in, v_in, ora, l, h, b, stats)
    assert stats["heads"] == L * H * Bn

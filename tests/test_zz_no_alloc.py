"""skipkv_step_static (the entry point for callers that cannot allocate: its scratch is an array
the library holds on the GPU) against skipkv_step on the same inputs, through the C ABI: two calls
in a row on the shared array, the second on a smaller problem, then a problem that is too large."""
import pytest
import torch

from paper_2512_07993_amd import binding as B
from paper_2512_07993_amd import workloads as W

from helpers import make_cache, run_step

pytestmark = pytest.mark.gpu


def _bits(t):
    return t.view(torch.int16 if t.dtype == torch.bfloat16 else torch.int32)


def _run_static(cfg, st, k, v, q):
    dev = k.device
    cache = make_cache(cfg, st, k, v)
    L, H, Bn, S, T = cfg.n_layers, cfg.n_kv_heads, cfg.batch, st.total_sentences, st.total_tokens
    status = torch.zeros(1, dtype=torch.int32, device=dev)
    params = B.Params(cfg.obs_window, cfg.protect_window, cfg.budget, dev_status=status)
    kept_stride = max(1, min(cfg.budget, T))
    out = dict(
        sent_score=torch.full((L, H, S), float("nan"), dtype=torch.float32, device=dev),
        sent_lambda=torch.full((L, H, S), float("nan"), dtype=torch.float32, device=dev),
        tok_imp=torch.full((L, H, T), float("nan"), dtype=torch.float32, device=dev),
        sent_keep=torch.full((L, H, S), 77, dtype=torch.uint8, device=dev),
        kept_idx=torch.full((L, H, Bn, kept_stride), -1, dtype=torch.int32, device=dev),
        new_len=torch.full((L, H, Bn), -1, dtype=torch.int32, device=dev),
        new_sent_off=torch.full((L, H, S + Bn), -1, dtype=torch.int32, device=dev),
        new_sent_cnt=torch.full((L, H, Bn), -1, dtype=torch.int32, device=dev))
    B.skipkv_step_static(cache, params, q, None, out["sent_score"], out["sent_lambda"], out["tok_imp"], out["sent_keep"],
                         out["kept_idx"], out["new_len"], out["new_sent_off"], out["new_sent_cnt"], kept_stride)
    torch.cuda.synchronize()
    assert int(status.item()) == 0
    return out


def _check_against_step(cfg):
    st = W.make_structure(cfg)
    k0, v0, q = W.fill_cache(cfg, st, device="cuda")
    k_ref, v_ref = k0.clone(), v0.clone()
    ref = run_step(cfg, st, k_ref, v_ref, q)
    assert int(ref.dev_status.item()) == 0
    k, v = k0.clone(), v0.clone()
    got = _run_static(cfg, st, k, v, q)
    # integer, byte and index outputs and the compacted cache: bit for bit
    for name in ("sent_keep", "kept_idx", "new_len", "new_sent_off", "new_sent_cnt"):
        assert torch.equal(got[name], getattr(ref, name)), name
    for b in range(cfg.batch):
        t0 = int(st.seq_off[b])
        for l in range(cfg.n_layers):
            for h in range(cfg.n_kv_heads):
                n = int(ref.new_len[l, h, b].item())
                assert torch.equal(_bits(k[l, h, t0:t0 + n]), _bits(k_ref[l, h, t0:t0 + n])), ("K", l, h, b)
                assert torch.equal(_bits(v[l, h, t0:t0 + n]), _bits(v_ref[l, h, t0:t0 + n])), ("V", l, h, b)
    # floating point: the same kernels on the same bits (bar: rel 1e-3; observed: identical)
    for name, r in (("sent_score", ref.sent_score), ("sent_lambda", ref.sent_lambda), ("tok_imp", ref.tok_imp)):
        g = got[name]
        fin = torch.isfinite(r)
        assert torch.equal(torch.isfinite(g), fin), name
        assert torch.equal(g[~fin], r[~fin]), name
        torch.testing.assert_close(g[fin], r[fin], rtol=1e-3, atol=1e-12, msg=name)


def test_static_scratch_step_matches_step_twice_in_a_row_then_refuses_what_does_not_fit():
    big = W.CONFIGS[2].scaled(n_layers=4)       # 32 heads of 4224 tokens, several scan items each
    small = W.CONFIGS[3].scaled(n_layers=1, n_kv_heads=2, n_q_heads=8, batch=3, len_lo=300, len_hi=2500, budget=256)
    _check_against_step(big)
    _check_against_step(small)                  # the array still holds what the larger call left
    # a problem whose workspace exceeds the array is refused on the host, nothing is enqueued
    cfg = W.CONFIGS[3].scaled(n_layers=4)
    st = W.make_structure(cfg)
    dev = torch.device("cuda")
    T, S = st.total_tokens, st.total_sentences
    k = torch.zeros((cfg.n_layers, cfg.n_kv_heads, T, 128), dtype=torch.bfloat16, device=dev)
    q = torch.zeros((cfg.n_layers, cfg.batch, cfg.n_q_heads, cfg.obs_window, 128), dtype=torch.bfloat16, device=dev)
    cache = make_cache(cfg, st, k, k.clone())
    params = B.Params(cfg.obs_window, cfg.protect_window, cfg.budget)
    assert B.skipkv_workspace_bytes(cache, params) > B.STATIC_WS_BYTES
    L, H, Bn = cfg.n_layers, cfg.n_kv_heads, cfg.batch
    f = lambda *s: torch.zeros(s, dtype=torch.float32, device=dev)
    i = lambda *s: torch.full(s, -7, dtype=torch.int32, device=dev)
    new_len = i(L, H, Bn)
    with pytest.raises(B.SkipKVError) as e:
        B.skipkv_step_static(cache, params, q, None, f(L, H, S), f(L, H, S), None, None, i(L, H, Bn, cfg.budget), new_len,
                             None, None, cfg.budget)
    assert e.value.status == -4
    torch.cuda.synchronize()
    assert int((new_len != -7).sum().item()) == 0

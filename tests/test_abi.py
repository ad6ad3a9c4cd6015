"""CPU-side checks of the C-ABI library: it loads, exports every declared symbol, and
rejects bad arguments on the host before anything touches a GPU."""
import ctypes as C
import os
import re

import pytest

from paper_2512_07993_amd import binding as B

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module", autouse=True)
def _built():
    """The library under test: the product library, or (tests/test_abi_sanitized.py runs this file again
    in a child process with SKIPKV_ABI_TEST_LIB set) a build whose host side is sanitizer-instrumented."""
    other = os.environ.get("SKIPKV_ABI_TEST_LIB")
    if other:
        saved = (B._LIB_PATH, B._lib)
        B._LIB_PATH, B._lib = other, None
        yield
        B._LIB_PATH, B._lib = saved
        return
    if not os.path.exists(B._LIB_PATH):
        from paper_2512_07993_amd.build import build_library
        build_library()
    yield


def _declared():
    text = open(os.path.join(ROOT, "include", "skipkv.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(skipkv_[a-z_]+)\s*\(", text)))


def test_every_declared_symbol_is_exported():
    names = _declared()
    assert {"skipkv_score", "skipkv_select", "skipkv_compact", "skipkv_steer_add", "skipkv_step",
            "skipkv_workspace_bytes", "skipkv_strerror", "skipkv_version"} <= set(names)
    lib = B.lib()
    for n in names:
        assert hasattr(lib, n), n
    assert B.skipkv_version() == 101
    for code in (0, -1, -2, -3, -4, -5, -99):
        assert len(B.skipkv_strerror(code)) > 0


def _cache(**kw):
    d = dict(k=0x1000, v=0x2000, stride_layer=8 * 4096 * 128, stride_head=4096 * 128, stride_tok=128, dtype=B.BF16,
             n_layers=2, n_kv_heads=8, n_q_heads=32, head_dim=128, batch=1, total_tokens=4096, total_sentences=200,
             seq_off=0x3000, sent_ptr=0x4000, sent_off=0x5000)
    d.update(kw)
    return B.CCache(*[d[f[0]] for f in B.CCache._fields_])


def _params(**kw):
    d = dict(obs_window=16, protect_window=64, sigma=0.1, tau=0.95, budget=None, budget_scalar=2048, max_budget=2048,
             dev_status=None, profile=None, flags=0, spin_limit=0)
    d.update(kw)
    return B.CParams(*[d[f[0]] for f in B.CParams._fields_])


def _ws_bytes(cache, params):
    out = C.c_size_t(0)
    return B.lib().skipkv_workspace_bytes(C.byref(cache), C.byref(params), C.byref(out)), out.value


def test_workspace_size_is_computed_on_the_host():
    rc, n = _ws_bytes(_cache(), _params())
    assert rc == B.OK and n > 2 * 16 * 200 * 128 * 2 and n % 256 == 0
    rc2, n2 = _ws_bytes(_cache(total_tokens=8192), _params())
    assert rc2 == B.OK and n2 > n


@pytest.mark.parametrize("ckw,pkw,expect", [
    (dict(head_dim=64), {}, B.ECAPACITY),
    (dict(dtype=7), {}, B.EINVAL),
    (dict(k=None), {}, B.EINVAL),
    (dict(k=0x1004), {}, B.EINVAL),                       # not 16-byte aligned
    (dict(stride_tok=64), {}, B.EINVAL),
    (dict(stride_tok=132), {}, B.EINVAL),                 # rows would lose 16-byte alignment
    (dict(n_q_heads=30), {}, B.EINVAL),                   # not a multiple of the KV heads
    (dict(n_q_heads=8 * 9), {}, B.ECAPACITY),             # group larger than supported
    (dict(seq_off=None), {}, B.EINVAL),
    (dict(sent_off=None), {}, B.EINVAL),
    ({}, dict(obs_window=0), B.EINVAL),
    ({}, dict(obs_window=64, protect_window=32), B.EBUDGET),
    ({}, dict(budget_scalar=32), B.EBUDGET),              # budget < protected window
    ({}, dict(obs_window=33, protect_window=64), B.ECAPACITY),
    ({}, dict(sigma=1.5), B.EINVAL),
])
def test_validation_errors(ckw, pkw, expect):
    rc, _ = _ws_bytes(_cache(**ckw), _params(**pkw))
    assert rc == expect


def test_score_rejects_missing_or_small_workspace_and_null_outputs():
    lib, cache, params = B.lib(), _cache(), _params()
    rc, need = _ws_bytes(cache, params)
    assert rc == B.OK
    args = lambda ws, n, score=0x7000: (C.byref(cache), C.byref(params), 0x6000, None, score, 0x8000, None, ws, n, None)
    assert lib.skipkv_score(*args(None, need)) == B.EWORKSPACE
    assert lib.skipkv_score(*args(0x10000, need - 1)) == B.EWORKSPACE
    assert lib.skipkv_score(*args(0x10010, need)) == B.EWORKSPACE     # not 256-byte aligned
    assert lib.skipkv_score(*args(0x10000, need, score=None)) == B.EINVAL
    assert lib.skipkv_score(C.byref(cache), C.byref(params), None, None, 0x7000, 0x8000, None, 0x10000, need, None) == B.EINVAL


def test_select_and_compact_reject_bad_arguments():
    lib, cache, params = B.lib(), _cache(), _params()
    sel = lambda **kw: lib.skipkv_select(C.byref(cache), C.byref(params), kw.get("score", 0x7000), None,
                                         kw.get("kept", 0x9000), kw.get("new_len", 0xA000), kw.get("noff"),
                                         kw.get("ncnt"), kw.get("stride", 2048), None)
    assert sel(stride=100) == B.EINVAL                    # kept_idx rows shorter than the budget
    assert sel(new_len=None) == B.EINVAL
    assert sel(noff=0xB000) == B.EINVAL                   # offsets without counts
    assert lib.skipkv_compact(C.byref(cache), None, 0xA000, 2048, None) == B.EINVAL
    assert lib.skipkv_compact(C.byref(cache), 0x9000, None, 2048, None) == B.EINVAL
    assert lib.skipkv_compact(None, 0x9000, 0xA000, 2048, None) == B.EINVAL


def test_empty_problems_are_accepted_without_launching():
    lib = B.lib()
    cache, params = _cache(batch=0, total_tokens=0, total_sentences=0, k=None, v=None), _params()
    assert lib.skipkv_score(C.byref(cache), C.byref(params), None, None, None, None, None, None, 0, None) == B.OK
    assert lib.skipkv_compact(C.byref(cache), None, None, 0, None) == B.OK
    assert lib.skipkv_steer_add(None, None, None, 1.0, None, 0, 128, B.BF16, None) == B.OK
    assert lib.skipkv_steer_add(None, None, None, 1.0, None, 4, 128, B.BF16, None) == B.EINVAL
    assert lib.skipkv_steer_add(0x1000, 0x2000, None, 1.0, None, 4, 128, 9, None) == B.EINVAL


def test_binding_refuses_to_run_without_the_library(monkeypatch):
    monkeypatch.setattr(B, "_lib", None)
    monkeypatch.setattr(B, "_LIB_PATH", "/nonexistent/libskipkv.so")
    with pytest.raises(RuntimeError, match="no CPU fallback"):
        B.lib()


def test_ranges_and_similarity_entry_points_validate_on_the_host():
    lib, cache, params = B.lib(), _cache(), _params()
    out = C.c_size_t(0)
    # per-head ranges: workspace larger than the shared one, contiguous K/V required, ranges required
    assert lib.skipkv_ranges_workspace_bytes(C.byref(cache), C.byref(params), C.byref(out)) == B.OK
    assert out.value > _ws_bytes(cache, params)[1]
    need = out.value
    strided = _cache(stride_head=8192 * 128, stride_layer=8 * 8192 * 128)
    assert lib.skipkv_ranges_workspace_bytes(C.byref(strided), C.byref(params), C.byref(out)) == B.ECAPACITY
    rng = B.CRanges(0x6000, 0x6100, 0x6200)
    step = lambda r, ws=0x10000, n=need, noff=0xB000, ncnt=0xC000: lib.skipkv_step_ranges(
        C.byref(cache), r, C.byref(params), 0x6400, None, 0x7000, 0x8000, None, None, 0x9000, 0xA000, noff, ncnt,
        2048, ws, n, None)
    assert step(None) == B.EINVAL
    assert step(C.byref(B.CRanges(0x6000, None, 0x6200))) == B.EINVAL
    assert step(C.byref(rng), n=need - 1) == B.EWORKSPACE
    assert step(C.byref(rng), noff=0x6200) == B.EINVAL     # outputs must not alias the input ranges
    assert lib.skipkv_ranges_append(C.byref(cache), None, 0x6300, 0x6400, 0x6500, None, None) == B.EINVAL
    assert lib.skipkv_ranges_append(C.byref(cache), C.byref(rng), None, 0x6400, 0x6500, None, None) == B.EINVAL
    # hidden-state similarity: d_model a multiple of 128, workspace, pointers
    assert lib.skipkv_similarity_workspace_bytes(C.byref(cache), 4096, C.byref(out)) == B.OK
    assert out.value >= 200 * 4096 * 8
    assert lib.skipkv_similarity_workspace_bytes(C.byref(cache), 100, C.byref(out)) == B.EINVAL
    sim = lambda h=0x6400, d=4096, dt=B.BF16, lam=0x7000, ws=0x10000, n=1 << 30: lib.skipkv_sentence_similarity(
        C.byref(cache), h, d, dt, lam, ws, n, None)
    assert sim(h=None) == B.EINVAL and sim(lam=None) == B.EINVAL and sim(d=130) == B.EINVAL and sim(dt=7) == B.EINVAL
    assert sim(n=1024) == B.EWORKSPACE and sim(ws=0x10010) == B.EWORKSPACE
    assert lib.skipkv_score_shared(C.byref(cache), C.byref(params), 0x6400, None, None, 0x7000, None, None, 0x10000,
                                   1 << 40, None) == B.EINVAL  # lambda missing
    assert lib.skipkv_steer_strength(None, 1.0, 0.1, 0x7000, 4, None) == B.EINVAL
    assert lib.skipkv_steer_strength(None, 1.0, 0.1, None, 0, None) == B.OK


def test_paged_entry_points_validate_on_the_host():
    lib, cache, params = B.lib(), _cache(), _params()
    out = C.c_size_t(0)
    good = dict(block_table=0x6000, table_stride=600, block_size=16, n_blocks=700, stride_block=16 * cache.stride_tok)
    pg = lambda **kw: B.CPaging(**{**good, **kw})
    size = lambda p: lib.skipkv_paged_workspace_bytes(C.byref(cache), p, C.byref(params), C.byref(out))
    assert size(C.byref(pg())) == B.OK
    need = out.value
    assert need >= _ws_bytes(cache, params)[1] + 4 * cache.total_tokens   # the step's workspace plus the row map
    assert size(None) == B.EINVAL
    assert size(C.byref(pg(block_size=0))) == B.EINVAL
    assert size(C.byref(pg(n_blocks=0))) == B.EINVAL
    assert size(C.byref(pg(block_table=None))) == B.EINVAL
    assert size(C.byref(pg(stride_block=16 * cache.stride_tok + 8))) == B.EINVAL   # not a whole number of rows
    assert size(C.byref(pg(stride_block=8 * cache.stride_tok))) == B.EINVAL        # blocks would overlap
    assert size(C.byref(pg(n_blocks=1 << 30))) == B.ECAPACITY                      # slot rows are 32-bit
    step = lambda p, ws=0x10000, n=need, q=0x6400: lib.skipkv_step_paged(
        C.byref(cache), p, C.byref(params), q, None, 0x7000, 0x8000, None, None, 0x9000, 0xA000, 0xB000, 0xC000,
        2048, ws, n, None)
    assert step(None) == B.EINVAL
    assert step(C.byref(pg()), q=None) == B.EINVAL
    assert step(C.byref(pg()), n=need - 1) == B.EWORKSPACE
    assert step(C.byref(pg()), ws=0x10010) == B.EWORKSPACE


def test_paged_ranges_entry_points_validate_on_the_host():
    lib, params = B.lib(), _params()
    # pools laid out [layers, blocks, slots, heads, 128]: 700 blocks of 16 slots
    cache = _cache(stride_tok=8 * 128, stride_head=128, stride_layer=700 * 16 * 8 * 128)
    out = C.c_size_t(0)
    good = dict(block_table=0x6000, table_stride=600, block_size=16, n_blocks=700, stride_block=16 * cache.stride_tok)
    pg = lambda **kw: B.CPaging(**{**good, **kw})
    size = lambda p, c=cache: lib.skipkv_ranges_paged_workspace_bytes(C.byref(c), p, C.byref(params), C.byref(out))
    assert size(C.byref(pg())) == B.OK
    need = out.value
    n_lh = cache.n_layers * cache.n_kv_heads
    assert need >= 4 * n_lh * cache.total_tokens               # one row map per (layer, head)
    assert size(None) == B.EINVAL
    assert size(C.byref(pg(block_size=0))) == B.EINVAL
    assert size(C.byref(pg(stride_block=8 * cache.stride_tok))) == B.EINVAL        # blocks would overlap
    assert size(C.byref(pg()), _cache(stride_tok=8 * 128, stride_head=128 + 8, stride_layer=700 * 16 * 8 * 128)) == B.EINVAL  # head rows off the 128-element grid
    assert size(C.byref(pg(n_blocks=1 << 30))) == B.ECAPACITY                      # slot rows are 32-bit
    rng = B.CRanges(0x6000, 0x6100, 0x6200)
    step = lambda r, p, ws=0x10000, n=need, q=0x6400, noff=0xB000: lib.skipkv_step_ranges_paged(
        C.byref(cache), r, p, C.byref(params), q, None, 0x7000, 0x8000, None, None, 0x9000, 0xA000, noff, 0xC000,
        2048, ws, n, None)
    assert step(None, C.byref(pg())) == B.EINVAL
    assert step(C.byref(rng), None) == B.EINVAL
    assert step(C.byref(rng), C.byref(pg()), q=None) == B.EINVAL
    assert step(C.byref(rng), C.byref(pg()), n=need - 1) == B.EWORKSPACE
    assert step(C.byref(rng), C.byref(pg()), ws=0x10010) == B.EWORKSPACE
    assert step(C.byref(rng), C.byref(pg()), noff=0x6200) == B.EINVAL               # outputs must not alias the input ranges


def test_paged_score_and_compaction_validate_on_the_host():
    lib, cache, params = B.lib(), _cache(), _params()
    out = C.c_size_t(0)
    good = dict(block_table=0x6000, table_stride=600, block_size=16, n_blocks=700, stride_block=16 * cache.stride_tok)
    pg = lambda **kw: B.CPaging(**{**good, **kw})
    assert lib.skipkv_paged_workspace_bytes(C.byref(cache), C.byref(pg()), C.byref(params), C.byref(out)) == B.OK
    need = out.value
    score = lambda p, ws=0x10000, n=need, q=0x6400, lam=0x8000: lib.skipkv_score_paged(
        C.byref(cache), p, C.byref(params), q, None, 0x7000, lam, None, ws, n, None)
    assert score(None) == B.EINVAL and score(C.byref(pg()), q=None) == B.EINVAL and score(C.byref(pg()), lam=None) == B.EINVAL
    assert score(C.byref(pg()), n=need - 1) == B.EWORKSPACE and score(C.byref(pg(block_size=0))) == B.EINVAL
    size = lambda p, ks=2048: lib.skipkv_compact_paged_workspace_bytes(C.byref(cache), p, ks, C.byref(out))
    assert size(C.byref(pg())) == B.OK
    need = out.value
    assert need >= 4 * cache.total_tokens + 4 * cache.n_layers * cache.n_kv_heads * cache.batch * 2048
    assert size(None) == B.EINVAL and size(C.byref(pg()), ks=-1) == B.EINVAL
    assert size(C.byref(pg(n_blocks=1 << 30))) == B.ECAPACITY
    comp = lambda p, ws=0x10000, n=need, kept=0x9000, nl=0xA000: lib.skipkv_compact_paged(
        C.byref(cache), p, kept, nl, 2048, None, ws, n, None)
    assert comp(None) == B.EINVAL and comp(C.byref(pg()), kept=None) == B.EINVAL and comp(C.byref(pg()), nl=None) == B.EINVAL
    assert comp(C.byref(pg()), n=need - 1) == B.EWORKSPACE and comp(C.byref(pg()), ws=0x10010) == B.EWORKSPACE


def test_paged_token_redundancy_validates_on_the_host():
    lib, cache = B.lib(), _cache()
    out = C.c_size_t(0)
    good = dict(block_table=0x6000, table_stride=600, block_size=16, n_blocks=700, stride_block=16 * cache.stride_tok)
    pg = lambda **kw: B.CPaging(**{**good, **kw})
    size = lambda p: lib.skipkv_redundancy_paged_workspace_bytes(C.byref(cache), p, C.byref(out))
    assert size(C.byref(pg())) == B.OK
    need = out.value
    flat = C.c_size_t(0)
    assert lib.skipkv_redundancy_workspace_bytes(C.byref(cache), C.byref(flat)) == B.OK
    assert need >= flat.value + 4 * cache.total_tokens
    assert size(None) == B.EINVAL and size(C.byref(pg(block_size=0))) == B.EINVAL
    run = lambda p, ws=0x10000, n=need, red=0x7000: lib.skipkv_token_redundancy_paged(C.byref(cache), p, red, None, ws, n, None)
    assert run(None) == B.EINVAL and run(C.byref(pg()), red=None) == B.EINVAL
    assert run(C.byref(pg()), n=need - 1) == B.EWORKSPACE and run(C.byref(pg()), ws=0x10010) == B.EWORKSPACE


def test_token_level_range_entry_points_validate_on_the_host():
    lib, cache, params = B.lib(), _cache(), _params()
    out = C.c_size_t(0)
    assert lib.skipkv_ranges_workspace_bytes(C.byref(cache), C.byref(params), C.byref(out)) == B.OK
    need = out.value
    rng = B.CRanges(0x6000, 0x6100, 0x6200)
    score = lambda r, ws=0x10000, n=need, q=0x6400: lib.skipkv_score_ranges(
        C.byref(cache), r, C.byref(params), q, None, 0x7000, 0x8000, None, ws, n, None)
    assert score(None) == B.EINVAL and score(C.byref(rng), q=None) == B.EINVAL
    assert score(C.byref(rng), n=need - 1) == B.EWORKSPACE and score(C.byref(rng), ws=0x10010) == B.EWORKSPACE
    strided = _cache(stride_head=8192 * 128, stride_layer=8 * 8192 * 128)
    assert lib.skipkv_score_ranges(C.byref(strided), C.byref(rng), C.byref(params), 0x6400, None, 0x7000, 0x8000, None,
                                   0x10000, 1 << 40, None) == B.ECAPACITY
    sel = lambda r, ws=0x10000, n=need, imp=0x7000, noff=0xB000: lib.skipkv_select_tokens_ranges(
        C.byref(cache), r, C.byref(params), imp, None, 0x8000, 0x8800, None, 0x9000, 0xA000, noff, 0xC000, 2048, ws, n, None)
    assert sel(None) == B.EINVAL and sel(C.byref(rng), imp=None) == B.EINVAL
    assert sel(C.byref(rng), n=16) == B.EWORKSPACE and sel(C.byref(rng), ws=0x10010) == B.EWORKSPACE
    assert sel(C.byref(rng), noff=0x6200) == B.EINVAL      # outputs must not alias the input ranges
    flat = C.c_size_t(0)
    assert lib.skipkv_redundancy_workspace_bytes(C.byref(cache), C.byref(flat)) == B.OK
    red = lambda r, ws=0x10000, n=flat.value, o=0x7000: lib.skipkv_token_redundancy_ranges(C.byref(cache), r, o, ws, n, None)
    assert red(None) == B.EINVAL and red(C.byref(rng), o=None) == B.EINVAL and red(C.byref(B.CRanges(None, 0x6100, 0x6200))) == B.EINVAL
    assert red(C.byref(rng), n=flat.value - 1) == B.EWORKSPACE


def test_shared_lambda_range_entry_points_validate_on_the_host():
    lib, cache, params = B.lib(), _cache(), _params()
    out = C.c_size_t(0)
    assert lib.skipkv_ranges_workspace_bytes(C.byref(cache), C.byref(params), C.byref(out)) == B.OK
    need = out.value
    rng = B.CRanges(0x6000, 0x6100, 0x6200)
    ids_sel = lambda r=None, w=64, keep=0x7000, out_=0x7800: lib.skipkv_ranges_ids_select(C.byref(cache), r, w, keep, None, out_, None)
    assert ids_sel(keep=None) == B.EINVAL and ids_sel(out_=None) == B.EINVAL and ids_sel(w=-1) == B.EINVAL
    assert ids_sel(r=C.byref(B.CRanges(0x6000, None, 0x6200))) == B.EINVAL
    ids_app = lambda old=0x6100, new=0x6300, ids=0x7800: lib.skipkv_ranges_ids_append(C.byref(cache), old, new, ids, None)
    assert ids_app(old=None) == B.EINVAL and ids_app(ids=None) == B.EINVAL
    assert ids_app(new=0x6100) == B.EINVAL                    # the counts from before the append must be a copy
    score = lambda r, ids=0x7800, lp=0x7900, lam=0x7A00, ws=0x10000, n=need: lib.skipkv_score_shared_ranges(
        C.byref(cache), r, ids, lp, C.byref(params), 0x6400, None, lam, 0x7000, None, None, ws, n, None)
    assert score(None) == B.EINVAL and score(C.byref(rng), ids=None) == B.EINVAL and score(C.byref(rng), lp=None) == B.EINVAL
    assert score(C.byref(rng), lam=None) == B.EINVAL and score(C.byref(rng), n=need - 1) == B.EWORKSPACE
    sel = lambda r, ws=0x10000, n=need, sc=0x7000, noff=0xB000: lib.skipkv_select_ranges(
        C.byref(cache), r, C.byref(params), sc, None, 0x9000, 0xA000, noff, 0xC000, 2048, ws, n, None)
    assert sel(None) == B.EINVAL and sel(C.byref(rng), sc=None) == B.EINVAL
    assert sel(C.byref(rng), n=16) == B.EWORKSPACE and sel(C.byref(rng), noff=0x6200) == B.EINVAL


def test_paged_shared_lambda_score_validates_on_the_host():
    lib, cache, params = B.lib(), _cache(), _params()
    out = C.c_size_t(0)
    pg = B.CPaging(block_table=0x6000, table_stride=600, block_size=16, n_blocks=700, stride_block=16 * cache.stride_tok)
    assert lib.skipkv_paged_workspace_bytes(C.byref(cache), C.byref(pg), C.byref(params), C.byref(out)) == B.OK
    need = out.value
    score = lambda p=C.byref(pg), lam=0x7A00, sc=0x7000, n=need: lib.skipkv_score_shared_paged(
        C.byref(cache), p, C.byref(params), 0x6400, None, lam, sc, None, None, 0x10000, n, None)
    assert score(p=None) == B.EINVAL and score(lam=None) == B.EINVAL and score(sc=None) == B.EINVAL
    assert score(n=need - 1) == B.EWORKSPACE


def test_paged_per_head_parts_validate_on_the_host():
    lib, params = B.lib(), _params()
    cache = _cache(stride_tok=8 * 128, stride_head=128, stride_layer=700 * 16 * 8 * 128)
    out = C.c_size_t(0)
    pg = B.CPaging(block_table=0x6000, table_stride=600, block_size=16, n_blocks=700, stride_block=16 * cache.stride_tok)
    assert lib.skipkv_ranges_paged_workspace_bytes(C.byref(cache), C.byref(pg), C.byref(params), C.byref(out)) == B.OK
    need = out.value
    rng = B.CRanges(0x6000, 0x6100, 0x6200)
    score = lambda r=C.byref(rng), p=C.byref(pg), ids=None, lp=None, lam=None, sl=0x8000, n=need: lib.skipkv_score_ranges_paged(
        C.byref(cache), r, p, ids, lp, lam, C.byref(params), 0x6400, None, 0x7000, sl, None, 0x10000, n, None)
    assert score(r=None) == B.EINVAL and score(p=None) == B.EINVAL and score(sl=None) == B.EINVAL
    assert score(lam=0x7A00) == B.EINVAL                       # a shared lambda needs the sentence numbers and its CSR
    assert score(n=need - 1) == B.EWORKSPACE
    assert lib.skipkv_redundancy_paged_workspace_bytes(C.byref(cache), C.byref(pg), C.byref(out)) == B.OK
    red = lambda r=C.byref(rng), o=0x7000, n=out.value: lib.skipkv_token_redundancy_ranges_paged(
        C.byref(cache), r, C.byref(pg), o, None, 0x10000, n, None)
    assert red(r=None) == B.EINVAL and red(o=None) == B.EINVAL and red(n=out.value - 1) == B.EWORKSPACE


_I = 2 ** 31 - 1


@pytest.mark.parametrize("ckw", [
    dict(total_tokens=_I, total_sentences=_I), dict(n_layers=_I), dict(n_layers=1 << 20, n_kv_heads=1 << 10, n_q_heads=1 << 10),
    dict(batch=_I), dict(total_tokens=_I, total_sentences=_I, n_layers=4096, batch=1 << 20),
    dict(stride_tok=_I // 128 * 128, stride_head=1 << 62, stride_layer=1 << 62),
    dict(total_tokens=-5), dict(total_sentences=-1), dict(batch=-1), dict(n_layers=-3),
])
@pytest.mark.parametrize("pkw", [{}, dict(max_budget=_I, budget_scalar=_I),
                                 dict(obs_window=32, protect_window=_I, budget_scalar=_I, max_budget=_I)])
def test_extreme_sizes_give_an_error_or_a_sane_size(ckw, pkw):
    """Sizes at the edge of the 32-bit fields: every size query either refuses (negative counts: EINVAL;
    more than the 32-bit indices of the kernels can address: ECAPACITY) or returns a 256-byte multiple that
    did not wrap.  Run again under the sanitizer by tests/test_abi_sanitized.py."""
    lib, cache, params = B.lib(), _cache(**ckw), _params(**pkw)
    negative = any(v < 0 for v in ckw.values())
    out = C.c_size_t(0)
    for fn, extra in ((lib.skipkv_workspace_bytes, (C.byref(params),)), (lib.skipkv_ranges_workspace_bytes, (C.byref(params),)),
                      (lib.skipkv_similarity_workspace_bytes, (4096,))):
        out.value = 0
        rc = fn(C.byref(cache), *extra, C.byref(out))
        if negative:
            assert rc == B.EINVAL
        else:
            assert rc in (B.OK, B.ECAPACITY)
        if rc == B.OK:
            lower = 2 * cache.total_sentences * 128 * 2 if fn is not lib.skipkv_similarity_workspace_bytes else cache.total_sentences * 4096 * 4
            assert out.value % 256 == 0 and out.value >= lower

#!/usr/bin/env python3
"""Benchmark of the SkipKV compression step on one MI355X.

A "step" is one pass of the whole hot path (score -> select -> compact, one skipkv_step call)
over one batch of synthetic input already resident in HBM.  Prints ONE JSON line.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--config 3]

Compaction rewrites the cache in place, so every timed step gets its own pristine copy of
K and V (copied outside the timed region); steps are timed in groups of as many copies as
were allocated, each group bracketed by torch.cuda.synchronize().
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0  # MI355X published HBM3E bandwidth

# HBM bytes per launch from rocprofv3 counters (FETCH_SIZE and WRITE_SIZE, each scaled by what the same counter
# reads for a copy of known size).  They are NOT measured by this run: they are the stored result of the
# profiler runs written up in the file below, valid only for the workload they were taken on, and the JSON
# line names that file as their source.
TRAFFIC_PROFILE = os.path.join("profiles", "scan_fused_config3_hbm_traffic.txt")


def stored_traffic(config: int, kernel: str):
    """Bytes per launch from the profile's `traffic config=C kernel=K bytes=B` lines, None if there is none."""
    try:
        with open(os.path.join(ROOT, TRAFFIC_PROFILE)) as f:
            for line in f:
                w = line.split()
                if len(w) == 4 and w[0] == "traffic" and w[1] == "config=%d" % config and w[2] == "kernel=" + kernel:
                    return float(w[3].split("=", 1)[1])
    except OSError:
        pass
    return None


def _oracle_worker(args):
    import oracle  # test infrastructure, used here only for the reported CPU baseline
    from threadpoolctl import threadpool_limits
    qq, kk, vv, off, budget, protect = args
    with threadpool_limits(limits=1):
        t = time.perf_counter()
        oracle.compress_head(qq, kk, vv, off, budget, protect)
        return time.perf_counter() - t


def cpu_baseline(cfg, st, k0, v0, q, n_heads=640, seed=1):
    """Times the oracle as it stands on a bounded sample of heads of the same workload."""
    import multiprocessing as mp

    import numpy as np

    from paper_2512_07993_amd import workloads as W
    rng = np.random.default_rng(seed)
    cores = min(os.cpu_count() or 1, 16, n_heads)
    # heads spanning the length distribution: stratify over sequences sorted by length
    order = np.argsort(st.seq_len)
    picks = [int(order[int(i)]) for i in np.linspace(0, len(order) - 1, min(n_heads, len(order)))]
    while len(picks) < n_heads:
        picks.append(int(rng.integers(0, cfg.batch)))
    jobs, tok_heads = [], 0
    for b in picks:
        l, h = int(rng.integers(0, cfg.n_layers)), int(rng.integers(0, cfg.n_kv_heads))
        qq, kk, vv, off = W.head_arrays(cfg, st, k0, v0, q, l, h, b)
        jobs.append((qq, kk, vv, off, cfg.budget, cfg.protect_window))
        tok_heads += kk.shape[0]
    t = time.perf_counter()
    with mp.get_context("spawn").Pool(cores) as pool:
        pool.map(_oracle_worker, jobs)
    wall = time.perf_counter() - t
    lh = cfg.n_layers * cfg.n_kv_heads
    return {
        "value": tok_heads / wall / lh,
        "unit": "tokens/s",
        "cores": cores,
        "kind": "oracle",
        "sample": "%d heads of the same workload stratified over sequence length (%d token-heads, %.1f s wall), "
                  "scaled by token-heads to all %d heads" % (n_heads, tok_heads, wall, lh * cfg.batch),
    }


def calib_copy(reps: int = 3) -> int:
    """Counter calibration: a plain shifted copy of known size through skipkv_compact (row k <- row
    k+1 of every head: every byte of K and V is read once and written once), so that what
    rocprofv3's FETCH_SIZE / WRITE_SIZE read for a known amount of HBM traffic can be compared."""
    import torch

    from paper_2512_07993_amd import binding as B
    torch.cuda.set_device(0)
    L, H, T = 8, 8, 65536
    k = torch.randn((L, H, T, 128), device="cuda").to(torch.bfloat16)
    v = torch.randn((L, H, T, 128), device="cuda").to(torch.bfloat16)
    so = torch.tensor([0, T], dtype=torch.int32, device="cuda")
    sp = torch.tensor([0, 2], dtype=torch.int32, device="cuda")
    sf = torch.tensor([0, T], dtype=torch.int32, device="cuda")
    cache = B.Cache(k, v, H, so, sp, sf, T, 1)
    kept = (torch.arange(T - 1, dtype=torch.int32, device="cuda") + 1).repeat(L, H, 1, 1).contiguous()
    new_len = torch.full((L, H, 1), T - 1, dtype=torch.int32, device="cuda")
    for _ in range(reps):
        B.skipkv_compact(cache, kept, new_len, T - 1)
    torch.cuda.synchronize()
    moved = 2 * L * H * (T - 1) * 256
    print(json.dumps({"calibration": "shifted copy through k_compact", "launches": reps,
                      "bytes_read_per_launch": moved, "bytes_written_per_launch": moved}))
    return 0


def time_redundancy(config: int, reps: int = 3) -> int:
    """Times skipkv_token_redundancy (Eq.5, optional input of the step, quadratic in the cache
    length) on a workload's keys; prints one JSON line of its own.  Not part of the headline step."""
    import torch

    from paper_2512_07993_amd import binding as B
    from paper_2512_07993_amd import workloads as W
    torch.cuda.set_device(0)
    cfg = W.CONFIGS[config]
    st = W.make_structure(cfg)
    k0, v0, _ = W.fill_cache(cfg, st, device="cuda:0")
    so = torch.from_numpy(st.seq_off).cuda()
    sp = torch.from_numpy(st.sent_ptr).cuda()
    sf = torch.from_numpy(st.sent_off).cuda()
    cache = B.Cache(k0, v0, cfg.n_q_heads, so, sp, sf, st.total_tokens, st.total_sentences)
    ws = torch.empty(B.skipkv_redundancy_workspace_bytes(cache), dtype=torch.uint8, device="cuda")
    out = torch.empty((cfg.n_layers, cfg.n_kv_heads, st.total_tokens), dtype=torch.float32, device="cuda")
    B.skipkv_token_redundancy(cache, out, ws)
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(reps):
        B.skipkv_token_redundancy(cache, out, ws)
    e1.record()
    torch.cuda.synchronize()
    ms = e0.elapsed_time(e1) / reps
    # token-level selection on top of it (importance and lambda are random stand-ins: only its time is of interest here)
    L, H, Bn, S, T = cfg.n_layers, cfg.n_kv_heads, cfg.batch, st.total_sentences, st.total_tokens
    imp = torch.rand((L, H, T), device="cuda")
    lam = torch.rand((L, H, S), device="cuda")
    params = B.Params(cfg.obs_window, cfg.protect_window, cfg.budget)
    kept_stride = min(cfg.budget, T)
    tok_score = torch.empty((L, H, T), dtype=torch.float32, device="cuda")
    kept_idx = torch.empty((L, H, Bn, kept_stride), dtype=torch.int32, device="cuda")
    new_len = torch.empty((L, H, Bn), dtype=torch.int32, device="cuda")
    B.skipkv_select_tokens(cache, params, imp, out, lam, tok_score, None, kept_idx, new_len, None, None, kept_stride)
    torch.cuda.synchronize()
    e0.record()
    for _ in range(reps):
        B.skipkv_select_tokens(cache, params, imp, out, lam, tok_score, None, kept_idx, new_len, None, None, kept_stride)
    e1.record()
    torch.cuda.synchronize()
    ms_sel = e0.elapsed_time(e1) / reps
    pairs = float((st.seq_len.astype("float64") ** 2).sum()) * cfg.n_layers * cfg.n_kv_heads
    # what the kernels compute: the blocks at and right of the diagonal (256-row blocks, the diagonal square in full)
    done = float((st.seq_len.astype("float64") * (st.seq_len + 256.0) / 2).sum()) * cfg.n_layers * cfg.n_kv_heads
    flops = 2 * done * 128 * 2           # two sweeps over the computed half of the symmetric cosine matrix
    print(json.dumps({"op": "token_redundancy", "workload": "config %d: %s" % (cfg.config_id, cfg.name), "ms": ms,
                      "key_pairs_per_sweep": pairs, "computed_pairs_per_sweep": done,
                      "mfma_tflops": flops / (ms * 1e-3) / 1e12,
                      "frac_of_bf16_mfma_peak": flops / (ms * 1e-3) / 2.5e15,
                      "exp_per_s": 2 * done / (ms * 1e-3), "select_tokens_ms": ms_sel}))
    return 0


def time_ranges(config_id: int, steps: int = 5) -> int:
    """Times skipkv_step_ranges (per-head sentence ranges, Eq. 9-11) on the workload, with ranges that
    describe the same cache as the shared structure, next to skipkv_step on the same data."""
    import torch

    from paper_2512_07993_amd import binding as B
    from paper_2512_07993_amd import workloads as W

    torch.cuda.set_device(0)
    dev = "cuda:0"
    cfg = W.CONFIGS[config_id]
    st = W.make_structure(cfg)
    k0, v0, q = W.fill_cache(cfg, st, device=dev)
    L, H, Bn, S, T = cfg.n_layers, cfg.n_kv_heads, cfg.batch, st.total_sentences, st.total_tokens
    so, sp, sf = (torch.from_numpy(x).to(dev) for x in (st.seq_off, st.sent_ptr, st.sent_off))
    k, v = torch.empty_like(k0), torch.empty_like(v0)
    cache = B.Cache(k, v, cfg.n_q_heads, so, sp, sf, T, S)
    status = torch.zeros(1, dtype=torch.int32, device=dev)
    prof = B.skipkv_profile_create()
    params = B.Params(cfg.obs_window, cfg.protect_window, cfg.budget, dev_status=status, profile=prof)
    ws = torch.empty(B.skipkv_ranges_workspace_bytes(cache, params), dtype=torch.uint8, device=dev)
    ranges = B.Ranges(torch.from_numpy(st.seq_len.astype("int32")).to(dev).expand(L, H, Bn).contiguous(),
                      torch.from_numpy(st.n_sent.astype("int32")).to(dev).expand(L, H, Bn).contiguous(),
                      sf.expand(L, H, sf.numel()).contiguous())
    kept_stride = min(cfg.budget, T)
    sent_score = torch.empty((L, H, S), dtype=torch.float32, device=dev)
    sent_lambda = torch.empty_like(sent_score)
    sent_keep = torch.empty((L, H, S), dtype=torch.uint8, device=dev)
    kept_idx = torch.empty((L, H, Bn, kept_stride), dtype=torch.int32, device=dev)
    new_len = torch.empty((L, H, Bn), dtype=torch.int32, device=dev)
    new_off = torch.empty((L, H, S + Bn), dtype=torch.int32, device=dev)
    new_cnt = torch.empty((L, H, Bn), dtype=torch.int32, device=dev)
    out = {}
    for name in ("step_ranges", "step"):
        times = []
        for i in range(steps + 1):
            k.copy_(k0)
            v.copy_(v0)
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            if name == "step_ranges":
                B.skipkv_step_ranges(cache, ranges, params, q, None, sent_score, sent_lambda, None, sent_keep, kept_idx,
                                     new_len, new_off, new_cnt, kept_stride, ws)
            else:
                B.skipkv_step(cache, params, q, None, sent_score, sent_lambda, None, sent_keep, kept_idx, new_len,
                              new_off, new_cnt, kept_stride, ws)
            e1.record()
            torch.cuda.synchronize()
            if i:
                times.append(e0.elapsed_time(e1))
        out[name] = sum(times) / len(times)
        out[name + "_kernels"] = {n: round(t, 4) for n, t in B.skipkv_profile_read(prof)}  # of the last call
    assert int(status.item()) == 0, "device status %d" % int(status.item())
    B.skipkv_profile_destroy(prof)
    print(json.dumps({"op": "step_ranges", "workload": "config %d: %s" % (cfg.config_id, cfg.name),
                      "ms_per_step_per_head_ranges": out["step_ranges"], "ms_per_step_shared_ranges": out["step"],
                      "kernel_ms_per_head_ranges": out["step_ranges_kernels"], "kernel_ms_shared_ranges": out["step_kernels"],
                      "steps": steps}))
    return 0


def time_paged(config_id: int, block_size: int = 16, heads_first: bool = False, steps: int = 5) -> int:
    """Times skipkv_step_paged (and skipkv_step_ranges_paged on the same cache described per head) on the workload scattered into a pool of blocks of `block_size` token
    slots ([layers, blocks, slots, KV heads, 128], or [layers, blocks, KV heads, slots, 128] with
    heads_first; blocks in random order), next to skipkv_step on the contiguous cache."""
    import numpy as np
    import torch

    from paper_2512_07993_amd import binding as B
    from paper_2512_07993_amd import workloads as W

    torch.cuda.set_device(0)
    dev = "cuda:0"
    cfg = W.CONFIGS[config_id]
    st = W.make_structure(cfg)
    k0, v0, q = W.fill_cache(cfg, st, device=dev)
    L, H, Bn, S, T = cfg.n_layers, cfg.n_kv_heads, cfg.batch, st.total_sentences, st.total_tokens
    so, sp, sf = (torch.from_numpy(x).to(dev) for x in (st.seq_off, st.sent_ptr, st.sent_off))
    # placement: the blocks of all sequences in one random permutation
    nblk = [(int(n) + block_size - 1) // block_size for n in st.seq_len]
    n_blocks = sum(nblk)
    perm = np.random.default_rng(cfg.seed).permutation(n_blocks)
    table = np.full((Bn, max(nblk)), -1, dtype=np.int32)
    blk, slot, pos = np.empty(T, dtype=np.int64), np.empty(T, dtype=np.int64), 0
    for b in range(Bn):
        table[b, :nblk[b]] = perm[pos:pos + nblk[b]]
        pos += nblk[b]
        t = np.arange(int(st.seq_len[b]))
        blk[int(st.seq_off[b]):int(st.seq_off[b + 1])] = table[b, t // block_size]
        slot[int(st.seq_off[b]):int(st.seq_off[b + 1])] = t % block_size
    blk, slot = torch.from_numpy(blk).to(dev), torch.from_numpy(slot).to(dev)
    if heads_first:
        kp0 = torch.zeros((L, n_blocks, H, block_size, cfg.head_dim), dtype=k0.dtype, device=dev).permute(0, 1, 3, 2, 4)
        vp0 = torch.zeros((L, n_blocks, H, block_size, cfg.head_dim), dtype=k0.dtype, device=dev).permute(0, 1, 3, 2, 4)
    else:
        kp0 = torch.zeros((L, n_blocks, block_size, H, cfg.head_dim), dtype=k0.dtype, device=dev)
        vp0 = torch.zeros_like(kp0)
    kp0[:, blk, slot] = k0.permute(0, 2, 1, 3)
    vp0[:, blk, slot] = v0.permute(0, 2, 1, 3)
    kp, vp = torch.empty_like(kp0), torch.empty_like(vp0)  # (keeps the strides of a permuted pool)
    assert kp.stride() == kp0.stride()
    k, v = torch.empty_like(k0), torch.empty_like(v0)
    paged = B.PagedCache(kp, vp, torch.from_numpy(table).to(dev), cfg.n_q_heads, so, sp, sf, T, S)
    cache = B.Cache(k, v, cfg.n_q_heads, so, sp, sf, T, S)
    status = torch.zeros(1, dtype=torch.int32, device=dev)
    prof = B.skipkv_profile_create()
    params = B.Params(cfg.obs_window, cfg.protect_window, cfg.budget, dev_status=status, profile=prof)
    ws = torch.empty(B.skipkv_paged_workspace_bytes(paged, params), dtype=torch.uint8, device=dev)
    # the same cache described head by head (the form every step after the first takes)
    ranges = B.Ranges(torch.from_numpy(st.seq_len.astype(np.int32)).to(dev).expand(L, H, Bn).contiguous(),
                      torch.from_numpy(st.n_sent.astype(np.int32)).to(dev).expand(L, H, Bn).contiguous(),
                      sf.expand(L, H, sf.numel()).contiguous())
    ws_rp = torch.empty(B.skipkv_ranges_paged_workspace_bytes(paged, params), dtype=torch.uint8, device=dev)
    kept_stride = min(cfg.budget, T)
    sent_score = torch.empty((L, H, S), dtype=torch.float32, device=dev)
    sent_lambda = torch.empty_like(sent_score)
    sent_keep = torch.empty((L, H, S), dtype=torch.uint8, device=dev)
    kept_idx = torch.empty((L, H, Bn, kept_stride), dtype=torch.int32, device=dev)
    new_len = torch.empty((L, H, Bn), dtype=torch.int32, device=dev)
    new_off = torch.empty((L, H, S + Bn), dtype=torch.int32, device=dev)
    new_cnt = torch.empty((L, H, Bn), dtype=torch.int32, device=dev)
    out = {}
    for name in ("step_paged", "step_ranges_paged", "step"):
        times = []
        for i in range(steps + 1):
            if name != "step":
                kp.copy_(kp0)
                vp.copy_(vp0)
            else:
                k.copy_(k0)
                v.copy_(v0)
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            if name == "step_paged":
                B.skipkv_step_paged(paged, params, q, None, sent_score, sent_lambda, None, sent_keep, kept_idx, new_len,
                                    new_off, new_cnt, kept_stride, ws)
            elif name == "step_ranges_paged":
                B.skipkv_step_ranges_paged(paged, ranges, params, q, None, sent_score, sent_lambda, None, sent_keep,
                                           kept_idx, new_len, new_off, new_cnt, kept_stride, ws_rp)
            else:
                B.skipkv_step(cache, params, q, None, sent_score, sent_lambda, None, sent_keep, kept_idx, new_len,
                              new_off, new_cnt, kept_stride, ws)
            e1.record()
            torch.cuda.synchronize()
            if i:
                times.append(e0.elapsed_time(e1))
        out[name] = sum(times) / len(times)
        out[name + "_kernels"] = {n: round(t, 4) for n, t in B.skipkv_profile_read(prof)}  # of the last call
    assert int(status.item()) == 0, "device status %d" % int(status.item())
    B.skipkv_profile_destroy(prof)
    print(json.dumps({"op": "step_paged", "workload": "config %d: %s" % (cfg.config_id, cfg.name), "block_size": block_size,
                      "layout": "[blocks, heads, slots, 128]" if heads_first else "[blocks, slots, heads, 128]", "blocks": n_blocks, "ms_per_step_paged": out["step_paged"], "ms_per_step_ranges_paged": out["step_ranges_paged"], "ms_per_step_contiguous": out["step"],
                      "kernel_ms_paged": out["step_paged_kernels"], "kernel_ms_ranges_paged": out["step_ranges_paged_kernels"],
                      "kernel_ms_contiguous": out["step_kernels"],
                      "steps": steps}))
    return 0


def time_shared_lambda(config_id: int, d_model: int = 4096, steps: int = 5) -> int:
    """Times the paper-literal variant of the step: sentence similarity from hidden states once per
    sequence (Eq. 1-3), then scores with that shared lambda, selection and compaction."""
    import torch

    from paper_2512_07993_amd import binding as B
    from paper_2512_07993_amd import workloads as W

    torch.cuda.set_device(0)
    dev = "cuda:0"
    cfg = W.CONFIGS[config_id]
    st = W.make_structure(cfg)
    k0, v0, q = W.fill_cache(cfg, st, device=dev)
    L, H, Bn, S, T = cfg.n_layers, cfg.n_kv_heads, cfg.batch, st.total_sentences, st.total_tokens
    so, sp, sf = (torch.from_numpy(x).to(dev) for x in (st.seq_off, st.sent_ptr, st.sent_off))
    k, v = torch.empty_like(k0), torch.empty_like(v0)
    cache = B.Cache(k, v, cfg.n_q_heads, so, sp, sf, T, S)
    g = torch.Generator(device=dev)
    g.manual_seed(cfg.seed)
    hidden = torch.randn((T, d_model), generator=g, device=dev).to(k0.dtype)
    status = torch.zeros(1, dtype=torch.int32, device=dev)
    prof = B.skipkv_profile_create()
    params = B.Params(cfg.obs_window, cfg.protect_window, cfg.budget, dev_status=status, profile=prof)
    ws = torch.empty(B.skipkv_workspace_bytes(cache, params), dtype=torch.uint8, device=dev)
    ws_sim = torch.empty(B.skipkv_similarity_workspace_bytes(cache, d_model), dtype=torch.uint8, device=dev)
    kept_stride = min(cfg.budget, T)
    shared = torch.empty((S,), dtype=torch.float32, device=dev)
    sent_score = torch.empty((L, H, S), dtype=torch.float32, device=dev)
    sent_keep = torch.empty((L, H, S), dtype=torch.uint8, device=dev)
    kept_idx = torch.empty((L, H, Bn, kept_stride), dtype=torch.int32, device=dev)
    new_len = torch.empty((L, H, Bn), dtype=torch.int32, device=dev)
    t_sim, t_rest = [], []
    for i in range(steps + 1):
        k.copy_(k0)
        v.copy_(v0)
        ev = [torch.cuda.Event(enable_timing=True) for _ in range(3)]
        ev[0].record()
        B.skipkv_sentence_similarity(cache, hidden, shared, ws_sim)
        ev[1].record()
        B.skipkv_score_shared(cache, params, q, None, shared, sent_score, None, None, ws)
        B.skipkv_select(cache, params, sent_score, sent_keep, kept_idx, new_len, None, None, kept_stride)
        B.skipkv_compact(cache, kept_idx, new_len, kept_stride)
        ev[2].record()
        torch.cuda.synchronize()
        if i:
            t_sim.append(ev[0].elapsed_time(ev[1]))
            t_rest.append(ev[1].elapsed_time(ev[2]))
    assert int(status.item()) == 0, "device status %d" % int(status.item())
    kern = {n: round(t, 4) for n, t in B.skipkv_profile_read(prof)}  # of the last skipkv_score_shared
    B.skipkv_profile_destroy(prof)
    print(json.dumps({"op": "step_shared_lambda", "workload": "config %d: %s" % (cfg.config_id, cfg.name),
                      "d_model": d_model, "sentence_similarity_ms": sum(t_sim) / len(t_sim),
                      "score_select_compact_ms": sum(t_rest) / len(t_rest), "score_kernel_ms": kern, "steps": steps}))
    return 0


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=2)
    ap.add_argument("--config", type=int, default=3, help="workload: index into BASELINE.json configs (1-based)")
    ap.add_argument("--copies", type=int, default=5, help="pristine-copy working buffers (HBM: 2 x cache each)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--calib-copy", action="store_true", help="run only the counter-calibration copy (see profiles/)")
    ap.add_argument("--redundancy", action="store_true", help="time only skipkv_token_redundancy on the workload's keys")
    ap.add_argument("--shared-lambda", action="store_true", help="time the variant with hidden-state sentence similarity shared by all heads")
    ap.add_argument("--ranges", action="store_true", help="time skipkv_step_ranges (per-head sentence ranges) next to skipkv_step")
    ap.add_argument("--paged", type=int, default=0, metavar="BLOCK", help="time skipkv_step_paged with blocks of BLOCK token slots next to skipkv_step")
    ap.add_argument("--paged-heads-first", action="store_true", help="with --paged: pools laid out [blocks, heads, slots, 128] instead of [blocks, slots, heads, 128]")
    args = ap.parse_args()
    if args.calib_copy:
        return calib_copy()
    if args.redundancy:
        return time_redundancy(args.config)
    if args.paged:
        return time_paged(args.config, args.paged, args.paged_heads_first)
    if args.ranges:
        return time_ranges(args.config)
    if args.shared_lambda:
        return time_shared_lambda(args.config)
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU (heads are independent: more GPUs would only shard them); "
              "--gpus %d is not supported" % args.gpus, file=sys.stderr)
        return 2

    import torch

    from paper_2512_07993_amd import binding as B
    from paper_2512_07993_amd import workloads as W

    torch.cuda.set_device(0)
    dev = "cuda:0"
    cfg = W.CONFIGS[args.config]
    st = W.make_structure(cfg)
    k0, v0, q = W.fill_cache(cfg, st, device=dev)
    L, H, Bn, S, T = cfg.n_layers, cfg.n_kv_heads, cfg.batch, st.total_sentences, st.total_tokens
    esz = k0.element_size()

    so = torch.from_numpy(st.seq_off).to(dev)
    sp = torch.from_numpy(st.sent_ptr).to(dev)
    sf = torch.from_numpy(st.sent_off).to(dev)
    n_copies = max(1, min(args.copies, max(args.steps, args.warmup)))
    # working copies of K and V (restored from the pristine pair before each group of steps): as many as fit
    free_bytes, _ = torch.cuda.mem_get_info()
    pair_bytes = 2 * k0.numel() * esz
    n_copies = max(1, min(n_copies, int(0.8 * free_bytes // pair_bytes)))
    bufs = [(torch.empty_like(k0), torch.empty_like(v0)) for _ in range(n_copies)]
    caches = [B.Cache(k, v, cfg.n_q_heads, so, sp, sf, T, S) for (k, v) in bufs]
    status = torch.zeros(1, dtype=torch.int32, device=dev)
    prof = B.skipkv_profile_create()
    params = B.Params(cfg.obs_window, cfg.protect_window, cfg.budget, dev_status=status, profile=prof)
    ws = torch.empty(B.skipkv_workspace_bytes(caches[0], params), dtype=torch.uint8, device=dev)
    kept_stride = min(cfg.budget, T)
    sent_score = torch.empty((L, H, S), dtype=torch.float32, device=dev)
    sent_lambda = torch.empty_like(sent_score)
    sent_keep = torch.empty((L, H, S), dtype=torch.uint8, device=dev)
    kept_idx = torch.empty((L, H, Bn, kept_stride), dtype=torch.int32, device=dev)
    new_len = torch.empty((L, H, Bn), dtype=torch.int32, device=dev)

    def restore(n):
        for i in range(n):
            bufs[i][0].copy_(k0)
            bufs[i][1].copy_(v0)

    params_plain = B.Params(cfg.obs_window, cfg.protect_window, cfg.budget, dev_status=status)

    def step(i, with_events=True):
        B.skipkv_step(caches[i], params if with_events else params_plain, q, None, sent_score, sent_lambda, None,
                      sent_keep, kept_idx, new_len, None, None, kept_stride, ws)

    def run_group(n, timed, with_events=True):
        restore(n)
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        per_kernel = {}
        total = 0.0
        for i in range(n):
            e0.record()
            step(i, with_events)
            e1.record()
            torch.cuda.synchronize()
            if timed:
                total += e0.elapsed_time(e1)
                if with_events:
                    for name, ms in B.skipkv_profile_read(prof):
                        per_kernel.setdefault(name, []).append(ms)
        return total, per_kernel

    done = 0
    while done < args.warmup:
        n = min(n_copies, args.warmup - done)
        run_group(n, False)
        done += n
    total_ms, kernels = 0.0, {}
    done = 0
    while done < args.steps:
        n = min(n_copies, args.steps - done)
        t, pk = run_group(n, True)
        total_ms += t
        for name, v in pk.items():
            kernels.setdefault(name, []).extend(v)
        done += n
    assert int(status.item()) == 0, "device status %d" % int(status.item())
    ms_per_step = total_ms / args.steps
    # The timed steps above carry the library's per-kernel HIP events (two event records per kernel: they are
    # what the roofline figure is computed from).  The same number of steps again without them, for comparison.
    plain_ms, done = 0.0, 0
    while done < args.steps:
        n = min(n_copies, args.steps - done)
        plain_ms += run_group(n, True, with_events=False)[0]
        done += n
    ms_per_step_plain = plain_ms / args.steps

    # ---- algorithmic bytes of one step (what the method must move, not what the kernels do)
    ar = torch.arange(kept_stride, device=dev, dtype=torch.int32)
    valid = ar[None, None, None, :] < new_len[..., None]
    moved_rows = int(((kept_idx != ar) & valid).sum().item())
    k_scan_bytes = L * H * T * 128 * esz
    q_bytes = q.numel() * esz
    off_bytes = L * H * (S + Bn) * 4
    move_bytes = 4 * moved_rows * 128 * esz   # K and V rows that change place: read + write
    step_bytes = k_scan_bytes + move_bytes + q_bytes + off_bytes
    kernel_bytes = {
        "scan_fused": k_scan_bytes + q_bytes + off_bytes,
        "scan_stats": k_scan_bytes + q_bytes + off_bytes,
        "scan_scores": k_scan_bytes + q_bytes + off_bytes,
        "compact": move_bytes,
    }
    avg = {name: sum(v) / len(v) for name, v in kernels.items()}
    dominant = max((n for n in avg if n in kernel_bytes), key=lambda n: avg[n])
    achieved = kernel_bytes[dominant] / (avg[dominant] * 1e-3) / 1e9
    traffic = stored_traffic(args.config, dominant)
    result = {
        "metric": "compressed KV tokens/sec per compression step; achieved HBM GB/s vs peak",
        "value": T / (ms_per_step * 1e-3),
        "unit": "tokens/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": ms_per_step,
        "ms_per_step_without_kernel_events": ms_per_step_plain,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": cfg.dtype,
        "data": "synthetic",
        "config": {
            "workload": "config %d: %s" % (cfg.config_id, cfg.name),
            "batch": Bn, "layers": L, "kv_heads": H, "q_heads": cfg.n_q_heads, "head_dim": 128,
            "tokens": T, "sentences": S, "budget": cfg.budget, "obs_window": cfg.obs_window,
            "protect_window": cfg.protect_window, "heads": L * H * Bn,
            "token_heads_per_s": T * L * H / (ms_per_step * 1e-3),
            "kept_tokens_mean": float(new_len.float().mean().item()),
            "moved_rows": moved_rows,
        },
        "step_algorithmic_bytes": step_bytes,
        "step_algorithmic_gbps": step_bytes / (ms_per_step * 1e-3) / 1e9,
        "step_frac_of_hbm_peak": step_bytes / (ms_per_step * 1e-3) / 1e9 / HBM_PEAK_GBPS,
        "kernel_ms": {n: round(t, 4) for n, t in avg.items()},
        "roofline": {
            "kernel": dominant, "bound": "hbm", "achieved": achieved, "peak": HBM_PEAK_GBPS, "unit": "GB/s",
            "frac": achieved / HBM_PEAK_GBPS, "traffic": traffic,
            "traffic_source": ("stored rocprofv3 FETCH_SIZE + WRITE_SIZE counters, " + TRAFFIC_PROFILE) if traffic else None,
            "algorithmic_bytes_per_launch": kernel_bytes[dominant],
        },
    }
    if not args.no_cpu_baseline:
        result["cpu_baseline"] = cpu_baseline(cfg, st, k0, v0, q)
    B.skipkv_profile_destroy(prof)
    print(json.dumps(result))
    return 0


if __name__ == "__main__":
    sys.exit(main())

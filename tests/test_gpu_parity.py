"""GPU parity: the HIP path through the C ABI against the CPU oracle, head by head, on the
same seeded bits.  Sizes are chosen so that the oracle finishes in seconds while the work
still spans several chunks, tiles and a ragged tail."""
import numpy as np
import pytest
import torch

from paper_2512_07993_amd import workloads as W

from helpers import compare_head, oracle_head, run_step, sample_heads

pytestmark = pytest.mark.gpu


def _run_and_compare(cfg, n_heads, fused=True, seed=0):
    st = W.make_structure(cfg)
    k0, v0, q = W.fill_cache(cfg, st, device="cuda")
    k, v = k0.clone(), v0.clone()
    print("running", cfg.name, "tokens", st.total_tokens, "sentences", st.total_sentences, flush=True)
    out = run_step(cfg, st, k, v, q, fused=fused)
    assert int(out.dev_status.item()) == 0
    stats = {}
    for (l, h, b) in sample_heads(cfg, st, n_heads, seed):
        ora = oracle_head(cfg, st, k0, v0, q, l, h, b)
        compare_head(cfg, st, out, k, v, k0, v0, ora, l, h, b, stats)
    print(cfg.name, stats, flush=True)
    assert stats.get("near_tie_heads", 0) <= max(1, stats["heads"] // 20)
    return stats


def test_config1_tiny_fp32_all_heads():
    _run_and_compare(W.CONFIGS[1], 8)


def test_config1_separate_calls_match_fused():
    _run_and_compare(W.CONFIGS[1], 8, fused=False)


def test_config2_llama8b_single_two_layers():
    _run_and_compare(W.CONFIGS[2].scaled(n_layers=2), 16)


def test_config3_ragged_batch_one_layer():
    _run_and_compare(W.CONFIGS[3].scaled(n_layers=1, batch=6), 12)


def test_config4_qwen7b_gqa7_one_layer():
    _run_and_compare(W.CONFIGS[4].scaled(n_layers=1, batch=5), 10)


def test_config5_longcot_one_layer():
    _run_and_compare(W.CONFIGS[5].scaled(n_layers=1, batch=1), 3)


def test_two_pass_scan_matches_oracle(monkeypatch):
    """The fallback scan (K read twice, no cross-workgroup wait), forced for every sequence."""
    monkeypatch.setenv("SKIPKV_FORCE_TWO_PASS", "1")
    _run_and_compare(W.CONFIGS[3].scaled(n_layers=1, batch=4), 8)
    _run_and_compare(W.CONFIGS[1], 4)


def test_bounded_wait_reports_timeout_and_returns(monkeypatch):
    """With a poll limit of zero a workgroup that finds its head's normalisers not ready gives up
    at once: the step must still run to completion, raise the time-out bit, and leave the
    library usable (the next call, with the default limit, is correct again)."""
    from paper_2512_07993_amd import binding as B
    cfg = W.CONFIGS[3].scaled(n_layers=1, batch=4)
    st = W.make_structure(cfg)
    k0, v0, q = W.fill_cache(cfg, st, device="cuda")
    monkeypatch.setenv("SKIPKV_SPIN_LIMIT", "0")
    out = run_step(cfg, st, k0.clone(), v0.clone(), q)
    assert int(out.dev_status.item()) & B.DEV_TIMEOUT
    new_len = out.new_len.cpu().numpy()
    assert (new_len >= 0).all() and (new_len <= cfg.budget).all()
    monkeypatch.delenv("SKIPKV_SPIN_LIMIT")
    _run_and_compare(cfg, 6)


def test_config3_full_size_sampled_heads():
    """The benchmark workload itself (all 32 layers, batch 16: the grid, plan and workspace sizes
    that bench.py times), checked on heads sampled across layers, heads and sequences."""
    stats = _run_and_compare(W.CONFIGS[3], 16, seed=3)
    assert stats["heads"] == 16


def test_config4_full_size_sampled_heads():
    """Qwen-7B shape at full size (64 sequences, 28 layers, GQA 7, alpha 8) on sampled heads."""
    stats = _run_and_compare(W.CONFIGS[4], 12, seed=4)
    assert stats["heads"] == 12


def test_config5_full_size_sampled_heads():
    """Long-CoT shape at full size (8 sequences of 32896 tokens, 48 layers, 160 query rows per head:
    the two-pass scan) on sampled heads."""
    stats = _run_and_compare(W.CONFIGS[5], 6, seed=5)
    assert stats["heads"] == 6


def test_long_sequences_counter_protocol_next_to_short_ones():
    """Sequences of more than 128 scan items (here 75 K and 99 K tokens: 160 and 211 items) exchange
    their row statistics through the arrive counter and one merging workgroup, shorter ones (55 K
    tokens: 118 items) have every workgroup merge the records itself; one launch holds both."""
    cfg = W.CONFIGS[3].scaled(n_layers=1, batch=3, n_kv_heads=2, n_q_heads=8, len_lo=30000, len_hi=100000,
                              sent_mean=40.0)
    stats = _run_and_compare(cfg, 6, seed=7)
    assert stats["heads"] == 6


@pytest.mark.parametrize("group,alpha,dtype", [
    (1, 1, "bf16"), (1, 32, "bf16"), (2, 16, "bf16"), (3, 8, "bf16"), (4, 4, "f32"), (5, 8, "bf16"), (6, 10, "bf16"),
    (7, 8, "bf16"), (8, 8, "bf16"), (8, 4, "f32"), (4, 32, "bf16"), (8, 32, "bf16"), (5, 32, "f32"),
])
def test_group_sizes_and_observation_windows(group, alpha, dtype):
    """Every shape of the query block: group sizes 1-8, windows 1-32; up to 64 query rows the
    single-pass scan runs, beyond that the two-pass one.  All heads against the oracle."""
    cfg = W.Config("rows-%dx%d" % (group, alpha), 40 + group * 33 + alpha, 3, 1, 2, 2 * group, dtype, 150, 900, 256,
                   alpha, max(alpha, 40), 12.0, 0.2)
    stats = _run_and_compare(cfg, 6)
    assert stats["heads"] == 6

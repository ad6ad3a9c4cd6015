"""Seeded synthetic inputs shaped like the paper's workloads.

The paper evaluates on chain-of-thought traces of DeepSeek-R1-distilled models (Sec. 5.1);
neither those traces nor the weights are available, so this module only reproduces their
SHAPES and statistics: head counts of the three model families, cache length = budget +
128 newly decoded tokens (compression interval, Appendix "Hyper-parameters"), sentence
lengths, and a planted fraction of near-duplicate sentences (the redundancy the method
is built to find, Sec. 4 Observation 4).

This module holds NO arithmetic of the method: it only draws lengths, sentence
boundaries and N(0,1) tensors.  Both the GPU path and the CPU oracle are fed from it.
"""
from __future__ import annotations

import dataclasses
import math
from dataclasses import dataclass
from typing import Optional

import numpy as np
import torch


@dataclass(frozen=True)
class Config:
    name: str
    config_id: int
    batch: int
    n_layers: int
    n_kv_heads: int
    n_q_heads: int
    dtype: str                # "f32" | "bf16"
    len_lo: int               # per-sequence cache length, integer-uniform in [len_lo, len_hi]
    len_hi: int
    budget: int
    obs_window: int
    protect_window: int
    sent_mean: float          # mean of the log-normal sentence length
    dup_frac: float           # probability that a sentence (s >= 1) copies an earlier one
    head_dim: int = 128
    sent_sigma: float = 0.5   # shape of the log-normal
    sent_min: int = 4
    sent_max: int = 64
    dup_noise: float = 0.05
    steer_d_model: int = 0    # > 0: also build a steering-add problem [batch, d_model]
    steer_coef: float = 0.0

    @property
    def seed(self) -> int:
        return 20260000 + self.config_id

    @property
    def group(self) -> int:
        return self.n_q_heads // self.n_kv_heads

    def scaled(self, **kw) -> "Config":
        """Same recipe with some fields replaced (smaller layer count, batch, ...)."""
        return dataclasses.replace(self, **kw)


CONFIGS = {
    1: Config("tiny-fp32", 1, 1, 1, 8, 32, "f32", 1152, 1152, 1024, 8, 32, 16.0, 0.10),
    2: Config("llama8b-single", 2, 1, 32, 8, 32, "bf16", 4224, 4224, 4096, 16, 64, 20.0, 0.15),
    3: Config("llama8b-ragged16", 3, 16, 32, 8, 32, "bf16", 2048, 16384, 2048, 16, 64, 20.0, 0.20),
    4: Config("qwen7b-batch64", 4, 64, 28, 4, 28, "bf16", 4096, 8192, 1024, 8, 32, 24.0, 0.25,
              steer_d_model=3584, steer_coef=0.5),
    5: Config("qwen14b-longcot8", 5, 8, 48, 8, 40, "bf16", 32896, 32896, 4096, 32, 128, 20.0, 0.30),
}


@dataclass
class Structure:
    """Host-side ragged structure shared by all layers and heads of a batch."""
    seq_len: np.ndarray    # [B]   int32
    seq_off: np.ndarray    # [B+1] int32 token CSR
    sent_ptr: np.ndarray   # [B+1] int32 index into sent_off of each sequence's first entry
    sent_off: np.ndarray   # [sum(S_b + 1)] int32, per sequence ascending, first 0, last N_b
    dup_src: list          # per sequence: int array [S_b], source sentence or -1

    @property
    def total_tokens(self) -> int:
        return int(self.seq_off[-1])

    @property
    def n_sent(self) -> np.ndarray:
        return np.diff(self.sent_ptr) - 1

    @property
    def total_sentences(self) -> int:
        return int(self.n_sent.sum())

    def offsets(self, b: int) -> np.ndarray:
        return self.sent_off[self.sent_ptr[b]: self.sent_ptr[b + 1]]

    def sent_base(self, b: int) -> int:
        """Index of sequence b's first sentence in arrays laid out [.., S_total]."""
        return int(self.sent_ptr[b]) - b


def make_structure(cfg: Config) -> Structure:
    lens, offs_all, dups = [], [], []
    for b in range(cfg.batch):
        rng = np.random.Generator(np.random.Philox(key=cfg.seed, counter=[b, 0, 0, 0]))
        n_tok = int(rng.integers(cfg.len_lo, cfg.len_hi + 1))
        mu = math.log(cfg.sent_mean) - 0.5 * cfg.sent_sigma ** 2
        off, slen, src = [0], [], []
        while off[-1] < n_tok:
            s = len(slen)
            j = -1
            if s >= 1 and rng.random() < cfg.dup_frac:
                j = int(rng.integers(0, s))
                ln = slen[j]
            else:
                ln = int(np.clip(round(rng.lognormal(mu, cfg.sent_sigma)), cfg.sent_min, cfg.sent_max))
            ln = min(ln, n_tok - off[-1])       # the last sentence is truncated at N
            slen.append(ln)
            src.append(j)
            off.append(off[-1] + ln)
        lens.append(n_tok)
        offs_all.append(np.asarray(off, dtype=np.int32))
        dups.append(np.asarray(src, dtype=np.int64))
    seq_len = np.asarray(lens, dtype=np.int32)
    seq_off = np.concatenate([[0], np.cumsum(seq_len)]).astype(np.int32)
    sent_ptr = np.concatenate([[0], np.cumsum([len(o) for o in offs_all])]).astype(np.int32)
    return Structure(seq_len, seq_off, sent_ptr, np.concatenate(offs_all).astype(np.int32), dups)


def torch_dtype(cfg: Config):
    return torch.float32 if cfg.dtype == "f32" else torch.bfloat16


def fill_cache(cfg: Config, st: Structure, device="cpu", dup_noise: Optional[float] = None):
    """K, V : [L, Hk, T, D]; Q : [L, B, Hq, alpha, D] in the config's storage dtype.

    Planted near-duplicates: for a sentence s with source j the keys of s are the (stored)
    keys of j plus dup_noise * N(0,1), computed in fp32 and rounded to the storage dtype,
    for every layer and head; sources are resolved in sentence order, so chains compound.
    """
    noise = cfg.dup_noise if dup_noise is None else dup_noise
    dt = torch_dtype(cfg)
    L, H, T, D = cfg.n_layers, cfg.n_kv_heads, st.total_tokens, cfg.head_dim
    k = torch.empty((L, H, T, D), dtype=dt, device=device)
    v = torch.empty((L, H, T, D), dtype=dt, device=device)
    q = torch.empty((L, cfg.batch, cfg.n_q_heads, cfg.obs_window, D), dtype=dt, device=device)
    for l in range(L):
        g = torch.Generator(device=device)
        g.manual_seed(cfg.seed * 1000 + l)
        k[l] = torch.randn((H, T, D), generator=g, device=device, dtype=torch.float32).to(dt)
        v[l] = torch.randn((H, T, D), generator=g, device=device, dtype=torch.float32).to(dt)
        q[l] = torch.randn(q.shape[1:], generator=g, device=device, dtype=torch.float32).to(dt)
    g = torch.Generator(device=device)
    g.manual_seed(cfg.seed * 1000 + 999)
    for b in range(cfg.batch):
        off = st.offsets(b)
        t0 = int(st.seq_off[b])
        for s, j in enumerate(st.dup_src[b]):
            if j < 0:
                continue
            ln = int(off[s + 1] - off[s])
            src = k[:, :, t0 + int(off[j]): t0 + int(off[j]) + ln, :].to(torch.float32)
            eps = torch.randn(src.shape, generator=g, device=device, dtype=torch.float32)
            k[:, :, t0 + int(off[s]): t0 + int(off[s + 1]), :] = (src + noise * eps).to(dt)
    return k, v, q


def fill_steer(cfg: Config, device="cpu"):
    """Hidden state [B, d_model], steering vector [d_model] (storage dtype), coefficient."""
    assert cfg.steer_d_model > 0
    dt = torch_dtype(cfg)
    g = torch.Generator(device=device)
    g.manual_seed(cfg.seed * 1000 + 998)
    h = torch.randn((cfg.batch, cfg.steer_d_model), generator=g, device=device, dtype=torch.float32).to(dt)
    vec = torch.randn((cfg.steer_d_model,), generator=g, device=device, dtype=torch.float32).to(dt)
    return h, vec, cfg.steer_coef


def head_arrays(cfg: Config, st: Structure, k, v, q, l: int, h: int, b: int):
    """Float64 numpy copies of one head's inputs, exactly the stored values.

    Returns (q_group [n, alpha, D], k [N, D], v [N, D], off [S+1])."""
    t0, t1 = int(st.seq_off[b]), int(st.seq_off[b + 1])
    n = cfg.group
    kk = k[l, h, t0:t1].to(torch.float64).cpu().numpy()
    vv = v[l, h, t0:t1].to(torch.float64).cpu().numpy()
    qq = q[l, b, h * n:(h + 1) * n].to(torch.float64).cpu().numpy()
    return qq, kk, vv, st.offsets(b).astype(np.int64)

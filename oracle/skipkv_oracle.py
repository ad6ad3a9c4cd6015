"""Plain float64 reference of one SkipKV compression step for ONE (sequence, layer, KV head).

TEST INFRASTRUCTURE ONLY: imported by the tests, the smoke check and the benchmark's
cpu_baseline leg, never by the product path.  No blocking, fusion or reordering: each
function is the step of the method written out so it can be checked against the paper
by eye.  Inputs are float64 arrays holding exactly the values of the stored bf16/fp32
bits; everything is computed in float64.

Sections cited: Sec. 4.1 ("Skipping KV Storage with Sentence-level Scoring") with its
un-numbered equations counted in order of appearance: Eq.1 PSS, Eq.2 sentence embedding,
Eq.3 redundant set, Eq.4 attention importance, Eq.6 cumulative score, Eq.11 range remap;
Sec. 4.2 (steering injection); Alg.1 (eviction step); Appendix "Hyper-parameters".

Readings taken where the paper is silent or ambiguous (each is also listed in the design
notes of the repository):
  * query heads are 0-based, the group of KV head h is {h*n .. h*n+n-1};
  * "softmax(maxpool(.))" is the max over the group's heads of the softmax probabilities;
  * "normalise on the observation window" is the arithmetic mean over the alpha queries;
  * the mask M keeps only its causal part (ragged layout has no padding);
  * PSS is a cosine: embeddings are L2-normalised (eps = 1e-12 added to the norm);
  * embeddings are mean-pooled KEYS of the head (not the last-layer hidden state);
  * a sentence s is redundant when some LATER sentence j > s has cosine > tau (strict);
    its penalty is the largest such cosine;
  * token scores are aggregated to a sentence by the arithmetic mean over its
    unprotected span; the token-redundancy term R is an optional input (0 if absent);
  * token redundancy (Eq.5): softmax of the cosine matrix along each row, then the mean over
    the rows: R[t] is the average share of softmax mass the head's keys give to key t;
    the diagonal is kept, there is no causal mask and no padding (ragged layout), eps = 1e-12;
  * eviction is by whole sentences: rank by (score desc, index desc), keep the longest
    prefix that fits the budget left after the protected recent window;
  * the token-level form of the same step (Eq.6 as printed: every token of a redundant sentence
    carries the sentence's penalty): the protected recent window is always kept, the other
    tokens are ranked by (score desc, index desc) and exactly budget - window of them survive;
    sentence ranges follow Eq.11;
  * across steps (Eq.9-10) ranges are kept in CACHE positions per head: the shift by the number
    of evicted tokens that Eq.10 writes out is contained in the head's cache length; a token
    that follows a delimiter starts a new sentence, any other appended token continues the
    head's last sentence;
  * with the similarity taken from hidden states (one lambda per sentence of the text), a head
    finds the lambda of a sentence it still holds by the number that sentence has in the
    sequence's own list: numbers survive an eviction with their sentences (Eq.11) and continue
    after an append (Eq.10).

Parity pins: every function below is pinned by tests/test_oracle_*.py against library
routines, closed forms, brute force or invariants.  The whole-step result has no
paper-printed numeric example to compare against ("parity unpinned" against the paper's
own numbers: it prints none); only the per-step pins hold it.
"""
from __future__ import annotations

import math

import numpy as np

__all__ = [
    "token_importance",
    "sentence_embeddings",
    "sentence_redundancy",
    "token_redundancy",
    "sentence_scores",
    "select_sentences",
    "token_scores",
    "select_tokens",
    "remap_ranges",
    "append_ranges",
    "compact",
    "compress_head",
    "steer_add",
    "steer_strength",
    "round_to_bf16",
]


# --------------------------------------------------------------------------------------
# Sec. 4.1 "Token Importance Score" (Eq.4 and the sentence after it)
# --------------------------------------------------------------------------------------
def token_importance(q: np.ndarray, k: np.ndarray) -> np.ndarray:
    """I[t] for one KV head.

    q : [n, alpha, D]  queries of the n query heads that share this KV head, for the
        last alpha cache positions (the observation window).
    k : [N, D]         cached keys of the head.
    Returns I : [N] float64.

    Eq.4: A^i = softmax(Q^i K^T / sqrt(d) + M) over the N keys, one row per (head i,
    window query a).  Query a sits at cache position N-alpha+a and, by the causal part
    of M, sees keys t <= N-alpha+a.  Then the probabilities are max-pooled over the n
    heads of the group and averaged over the alpha window queries.
    """
    q = np.asarray(q, dtype=np.float64)
    k = np.asarray(k, dtype=np.float64)
    n, alpha, d = q.shape
    n_tok = k.shape[0]
    probs = np.zeros((n, alpha, n_tok), dtype=np.float64)
    for i in range(n):
        for a in range(alpha):
            last_visible = n_tok - alpha + a
            if last_visible < 0:
                continue  # this window query precedes the cache: it sees nothing
            logits = (k[: last_visible + 1] @ q[i, a]) / math.sqrt(d)
            e = np.exp(logits - logits.max())
            probs[i, a, : last_visible + 1] = e / e.sum()
    group_max = probs.max(axis=0)          # [alpha, N]  max over the GQA group
    return group_max.sum(axis=0) / alpha   # [N]         mean over the window


# --------------------------------------------------------------------------------------
# Sec. 4.1 "Sentence Similarity Score" (Eq.1 - Eq.3)
# --------------------------------------------------------------------------------------
def sentence_embeddings(k: np.ndarray, off: np.ndarray) -> np.ndarray:
    """Eq.2: v_s = mean of the vectors of sentence s (here: the head's keys).

    off : [S+1] ascending token offsets, off[0] = 0, off[S] = N; sentence s is
          the half-open span [off[s], off[s+1]).
    """
    k = np.asarray(k, dtype=np.float64)
    n_sent = len(off) - 1
    v = np.zeros((n_sent, k.shape[1]), dtype=np.float64)
    for s in range(n_sent):
        v[s] = k[off[s]: off[s + 1]].mean(axis=0)
    return v


def sentence_redundancy(v: np.ndarray, eps: float = 1e-12) -> np.ndarray:
    """lambda_s = max over later sentences j > s of the cosine PSS(v_s, v_j)  (Eq.1, Eq.3).

    The last sentence has no later one: lambda = -inf (never redundant).
    """
    v = np.asarray(v, dtype=np.float64)
    n_sent = v.shape[0]
    norm = np.sqrt((v * v).sum(axis=1))
    vhat = v / (norm + eps)[:, None]
    lam = np.full(n_sent, -np.inf, dtype=np.float64)
    for s in range(n_sent - 1):
        lam[s] = (vhat[s + 1:] @ vhat[s]).max()
    return lam


# --------------------------------------------------------------------------------------
# Sec. 4.1 "Sentence Redundancy Driven Cumulative Score" (Eq.6), lifted to sentences
# --------------------------------------------------------------------------------------
# --------------------------------------------------------------------------------------
# Sec. 4.1 "Token Redundancy Score" (Eq.5)
# --------------------------------------------------------------------------------------
def token_redundancy(k: np.ndarray, eps: float = 1e-12) -> np.ndarray:
    """R[t] for one KV head: mean over the rows of the row-wise softmax of Kbar Kbar^T.

    k : [N, D] keys of the head.  Kbar = k / (||k||_2 + eps) row by row.  Returns R : [N]
    (R sums to 1).  The cosine matrix is symmetric, so "softmax along rows, mean along columns"
    would give the same vector; a mean along the softmax axis would be the constant 1/N and is
    not what a per-token score can mean.
    """
    k = np.asarray(k, dtype=np.float64)
    n_tok = k.shape[0]
    if n_tok == 0:
        return np.zeros(0)
    kbar = k / (np.sqrt((k * k).sum(axis=1, keepdims=True)) + eps)
    cos = kbar @ kbar.T
    e = np.exp(cos - cos.max(axis=1, keepdims=True))
    p = e / e.sum(axis=1, keepdims=True)
    return p.mean(axis=0)


def sentence_scores(imp, lam, off, protect, sigma=0.1, tau=0.95, red=None):
    """Per-sentence eviction score and the number of unprotected tokens of each sentence.

    imp : [N] token importance, lam : [S] sentence redundancy, off : [S+1] offsets,
    protect : size w of the recent window that is never evicted, red : optional [N]
    token-redundancy term R of Eq.6.

    The protected window is the last min(w, N) tokens, starting at p.  A sentence is a
    candidate when it begins before p; its candidate span is [off[s], min(off[s+1], p)).
    score_s = sigma * mean(I) - (1 - sigma) * mean(R) - (lambda_s if lambda_s > tau).
    Non-candidates get score +inf and candidate length 0.
    """
    imp = np.asarray(imp, dtype=np.float64)
    n_tok = imp.shape[0]
    n_sent = len(off) - 1
    p = n_tok - min(protect, n_tok)
    score = np.full(n_sent, np.inf, dtype=np.float64)
    candlen = np.zeros(n_sent, dtype=np.int64)
    for s in range(n_sent):
        b = int(off[s])
        if b >= p:
            continue
        e = min(int(off[s + 1]), p)
        val = sigma * imp[b:e].mean()
        if red is not None:
            val -= (1.0 - sigma) * np.asarray(red, dtype=np.float64)[b:e].mean()
        if lam[s] > tau:
            val -= lam[s]
        score[s] = val
        candlen[s] = e - b
    return score, candlen


# --------------------------------------------------------------------------------------
# Sec. 4.1 last paragraph of Eq.6 ("evict in increasing order of the final score"),
# Alg.1 eviction line, and the surviving index set P of the range-remap paragraph
# --------------------------------------------------------------------------------------
def select_sentences(score, candlen, off, budget, protect):
    """Whole-sentence selection under a token budget.

    Returns dict(keep [S] bool, kept_idx ascending int64, new_len, new_off).
    keep[s] says whether the candidate span of s survives (True for non-candidates).
    new_off are the offsets of the surviving sentences in the compacted cache; a
    sentence none of whose tokens survive is dropped (cf. Eq.11).
    """
    off = np.asarray(off, dtype=np.int64)
    n_sent = len(off) - 1
    n_tok = int(off[-1])
    p = n_tok - min(protect, n_tok)
    keep = np.ones(n_sent, dtype=bool)
    if n_tok > budget:
        cands = [s for s in range(n_sent) if off[s] < p]
        # evict lowest score first  <=>  keep from the top; ties: the later sentence wins
        order = sorted(cands, key=lambda s: (-score[s], -s))
        room = budget - (n_tok - p)
        keep[cands] = False
        used = 0
        for s in order:
            if used + candlen[s] > room:
                break
            used += candlen[s]
            keep[s] = True
    kept = []
    new_off = [0]
    for s in range(n_sent):
        b, e = int(off[s]), int(off[s + 1])
        if b < p:
            surv = list(range(b, min(e, p))) if keep[s] else []
            surv += list(range(max(b, p), e)) if e > p else []
        else:
            surv = list(range(b, e))
        if surv:
            kept += surv
            new_off.append(new_off[-1] + len(surv))
    return {
        "keep": keep,
        "kept_idx": np.asarray(kept, dtype=np.int64),
        "new_len": len(kept),
        "new_off": np.asarray(new_off, dtype=np.int64),
    }


# --------------------------------------------------------------------------------------
# Token-level form of Eq.6 and of the eviction rule that follows it
# --------------------------------------------------------------------------------------
def token_scores(imp, red, lam, off, sigma=0.1, tau=0.95):
    """Eq.6 per token: sigma * I[t] - (1 - sigma) * R[t], minus lambda_s for every token of a
    sentence s in the redundant set (lambda_s > tau).  red may be None (R = 0)."""
    imp = np.asarray(imp, dtype=np.float64)
    score = sigma * imp
    if red is not None:
        score = score - (1.0 - sigma) * np.asarray(red, dtype=np.float64)
    score = score.copy()
    for s in range(len(off) - 1):
        if lam[s] > tau:
            score[int(off[s]):int(off[s + 1])] -= lam[s]
    return score


def select_tokens(score, off, budget, protect):
    """Token-level selection under a budget ("evict tokens in increasing order of the final score").

    The last min(protect, N) tokens are kept.  If N <= budget everything is kept; otherwise the
    remaining tokens are ranked by (score desc, index desc) and the first budget - window of them
    are kept, so exactly `budget` tokens survive.  Returns dict(keep [N] bool, kept_idx
    ascending, new_len, new_off): new_off are the offsets of the sentences that still have a
    token, in the compacted cache (Eq.11; a sentence with no survivor is dropped).
    """
    score = np.asarray(score, dtype=np.float64)
    off = np.asarray(off, dtype=np.int64)
    n_tok = int(off[-1])
    p = n_tok - min(protect, n_tok)
    keep = np.ones(n_tok, dtype=bool)
    if n_tok > budget:
        room = budget - (n_tok - p)
        order = sorted(range(p), key=lambda t: (-score[t], -t))
        keep[:p] = False
        for t in order[:room]:
            keep[t] = True
    kept = np.nonzero(keep)[0].astype(np.int64)
    new_off = [0]
    for s in range(len(off) - 1):
        cnt = int(keep[int(off[s]):int(off[s + 1])].sum())
        if cnt:
            new_off.append(new_off[-1] + cnt)
    return {"keep": keep, "kept_idx": kept, "new_len": len(kept), "new_off": np.asarray(new_off, dtype=np.int64)}


def remap_ranges(off, kept_idx):
    """Eq.11: b <- min{k : p_k >= b},  e <- max{k : p_k <= e} on inclusive ranges (b, e);
    a range with no surviving token is discarded.  Returns a list of inclusive (b, e)."""
    out = []
    for s in range(len(off) - 1):
        b, e = int(off[s]), int(off[s + 1]) - 1
        ks_b = [k for k, pk in enumerate(kept_idx) if pk >= b]
        ks_e = [k for k, pk in enumerate(kept_idx) if pk <= e]
        if not ks_b or not ks_e or min(ks_b) > max(ks_e):
            continue
        out.append((min(ks_b), max(ks_e)))
    return out


def surviving_sentence_ids(off, kept_idx, ids=None):
    """Numbers of the sentences that still hold a token after an eviction (cf. Eq.11: a range with
    no surviving token is discarded, every other range stays), in order.  ids : [S] the numbers the
    sentences had before (default: their positions).  Written from the kept tokens alone: sentence
    s survives when some kept token lies in [off[s], off[s+1])."""
    off = np.asarray(off, dtype=np.int64)
    kept = set(int(t) for t in kept_idx)
    out = []
    for s in range(len(off) - 1):
        if any(t in kept for t in range(int(off[s]), int(off[s + 1]))):
            out.append(int(ids[s]) if ids is not None else s)
    return np.asarray(out, dtype=np.int64)


def append_sentence_ids(ids, n_added):
    """Numbers after an append (Eq.10): the new sentences continue after the last old one (which
    an eviction never removes: the tail of the cache is protected); from 0 for an empty list."""
    ids = np.asarray(ids, dtype=np.int64)
    nxt = int(ids[-1]) + 1 if ids.size else 0
    return np.concatenate([ids, nxt + np.arange(int(n_added), dtype=np.int64)])


def append_ranges(off, n_new, starts):
    """Eq.10 in cache positions: n_new tokens are appended to a cache of N = off[-1] tokens;
    `starts` are the positions 0 <= p < n_new inside the appended run at which a new sentence
    starts.  A sentence is the run of tokens from one start to the next: the starts of the new
    cache are the old ones, the new ones shifted by N, and N itself if the cache was empty.
    Returns the new offsets (starts, then the new length)."""
    off = [int(x) for x in off]
    n_old = off[-1]
    begin = set(off[:-1])
    begin |= {n_old + int(p) for p in starts}
    if len(off) == 1:
        begin.add(0)
    return np.array(sorted(begin) + [n_old + int(n_new)], dtype=np.int64)


def compact(k, v, kept_idx):
    """Alg.1 eviction line: the cache keeps exactly the surviving rows, in order."""
    kept_idx = np.asarray(kept_idx, dtype=np.int64)
    return np.asarray(k)[kept_idx].copy(), np.asarray(v)[kept_idx].copy()


def compress_head(q, k, v, off, budget, protect, sigma=0.1, tau=0.95, red=None):
    """One full step for one head: score -> select -> compact.  q:[n,alpha,D], k,v:[N,D]."""
    imp = token_importance(q, k)
    emb = sentence_embeddings(k, off)
    lam = sentence_redundancy(emb)
    score, candlen = sentence_scores(imp, lam, off, protect, sigma, tau, red)
    sel = select_sentences(score, candlen, off, budget, protect)
    k_new, v_new = compact(k, v, sel["kept_idx"])
    out = dict(sel)
    out.update(imp=imp, emb=emb, lam=lam, score=score, candlen=candlen, k=k_new, v=v_new)
    return out


# --------------------------------------------------------------------------------------
# Sec. 4.2 steering injection  H <- H + alpha_t * v
# --------------------------------------------------------------------------------------
def round_to_bf16(x):
    """Round float64 values to the nearest bfloat16 (ties to even) in ONE rounding.

    Returns (values as float64, bit patterns as uint16).  Finite inputs below the
    bfloat16 overflow threshold only.
    """
    x = np.asarray(x, dtype=np.float64)
    a = np.abs(x)
    base = (a.astype(np.float32).view(np.uint32).astype(np.int64)) & 0xFFFF0000
    best_bits = None
    best_dist = None
    for delta in (-0x10000, 0, 0x10000):
        cb = np.maximum(base + delta, 0)
        cv = cb.astype(np.uint32).view(np.float32).astype(np.float64)
        dist = np.abs(a - cv)
        if best_bits is None:
            best_bits, best_dist = cb, dist
            continue
        even = ((cb >> 16) & 1) == 0
        better = (dist < best_dist) | ((dist == best_dist) & even & (cb != best_bits))
        best_bits = np.where(better, cb, best_bits)
        best_dist = np.where(better, dist, best_dist)
    sign = np.signbit(x).astype(np.int64) << 31
    bits32 = (best_bits | sign).astype(np.uint32)
    vals = bits32.view(np.float32).astype(np.float64)
    return vals, (bits32 >> 16).astype(np.uint16)


def steer_strength(n_nonexec, alpha0, gamma):
    """Sec. 4.2: alpha_t = alpha_0 + gamma * N_o per sample (float64)."""
    return float(alpha0) + float(gamma) * np.asarray(n_nonexec, dtype=np.float64)


def steer_add(h, vec, coef, row_mask=None, dtype="bf16"):
    """H[b, :] <- H[b, :] + coef[b] * vec for the rows selected by row_mask.

    Computed in float64 and rounded once to the storage dtype ("bf16" or "f32").
    Returns the new values as float64.
    """
    h = np.asarray(h, dtype=np.float64)
    vec = np.asarray(vec, dtype=np.float64)
    coef = np.broadcast_to(np.asarray(coef, dtype=np.float64), (h.shape[0],))
    out = h + coef[:, None] * vec[None, :]
    if dtype == "bf16":
        out = round_to_bf16(out)[0]
    elif dtype == "f32":
        out = out.astype(np.float32).astype(np.float64)
    else:
        raise ValueError(dtype)
    if row_mask is not None:
        m = np.asarray(row_mask).astype(bool)
        out = np.where(m[:, None], out, h)
    return out

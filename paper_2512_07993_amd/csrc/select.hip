// Budgeted whole-sentence selection (Sec. 4.1, text after Eq. 6: tokens are evicted in
// increasing order of the score until the budget is met; here the unit of eviction is a
// sentence) and the surviving index set P with the remapped sentence ranges (Eq. 11).
//
// Candidates are ranked by the key (score descending, sentence index descending).  Keys are
// distinct and every candidate has length >= 1, so the kept set - the longest ranked prefix whose
// lengths fit the room - is {key > K0}, where K0 is the largest key value for which the total
// length of {key >= K0} exceeds the room.  K0 is found bit by bit (32 score bits, then 12 index
// bits); every step is one masked sum over the candidates.  Nothing is sorted.
//
// A head with at most 1024 sentences is handled by ONE wave, 16 sentences per lane in registers,
// without any workgroup barrier; four such heads share a workgroup.  A head with more sentences
// (up to 4096) is handled afterwards by the four waves together, with the same code.
#include <type_traits>

#include "common.h"

namespace skipkv {

namespace {

constexpr int kEPL = 16;                  // sentences per lane
constexpr int kWaveSent = 64 * kEPL;      // sentences one wave can rank
static_assert(4 * kWaveSent >= SKIPKV_MAX_SENTENCES, "a workgroup ranks any admissible head");
static_assert(SKIPKV_MAX_SENTENCES <= (1 << 12), "the index part of the key is searched over 12 bits");

// Sum over the wave in a scalar register: one DPP add per step (rotations inside the rows of 16
// lanes, then row 0 -> 1 and 2 -> 3, then the lower half -> the upper half; lane 63 has the total).
__device__ __forceinline__ int wave_sum_i(int v) {
#define SKIPKV_ROR(N) \
  asm volatile("s_nop 1\n\tv_add_u32_dpp %0, %1, %1 row_ror:" #N " row_mask:0xf bank_mask:0xf" : "=v"(v) : "v"(v))
  SKIPKV_ROR(8);
  SKIPKV_ROR(4);
  SKIPKV_ROR(2);
  SKIPKV_ROR(1);
#undef SKIPKV_ROR
  // rows that are masked off keep their value, so the operand is read-write (same register)
  asm volatile("s_nop 1\n\tv_add_u32_dpp %0, %0, %0 row_bcast:15 row_mask:0xa bank_mask:0xf" : "+v"(v));
  asm volatile("s_nop 1\n\tv_add_u32_dpp %0, %0, %0 row_bcast:31 row_mask:0xc bank_mask:0xf" : "+v"(v));
  return __builtin_amdgcn_readlane(v, 63);
}

__device__ __forceinline__ int wave_scan_incl(int v, int lane) {
#pragma unroll
  for (int d = 1; d < 64; d <<= 1) {
    const int up = __shfl_up(v, d);
    if (lane >= d) v += up;
  }
  return v;
}

// Cross-wave exchange slots of a workgroup (used only when four waves share a head).  Calls
// alternate between two sets of slots, so one barrier per call is enough.
struct Exchange {
  int *slots;  // [2][4]
  int call;
};

template <int NW>
__device__ __forceinline__ int group_sum(int v, int gw, Exchange &x) {
  const int s = wave_sum_i(v);
  if constexpr (NW == 1) {
    return s;
  } else {
    int *slot = x.slots + 4 * (x.call & 1);
    ++x.call;
    if ((threadIdx.x & 63) == 0) slot[gw] = s;
    __syncthreads();
    return slot[0] + slot[1] + slot[2] + slot[3];
  }
}

// Exclusive prefix of v over the group's threads in thread order; `total` gets the group's sum.
template <int NW>
__device__ __forceinline__ int group_scan_excl(int v, int gw, int lane, Exchange &x, int &total) {
  const int incl = wave_scan_incl(v, lane);
  const int wtot = __builtin_amdgcn_readlane(incl, 63);
  if constexpr (NW == 1) {
    total = wtot;
    return incl - v;
  } else {
    int *slot = x.slots + 4 * (x.call & 1);
    ++x.call;
    if (lane == 0) slot[gw] = wtot;
    __syncthreads();
    int before = 0;
#pragma unroll
    for (int w = 0; w < 4; ++w)
      if (w < gw) before += slot[w];
    total = slot[0] + slot[1] + slot[2] + slot[3];
    return before + incl - v;
  }
}

// What a head's inputs say about its size, clamped to the room that the CSR arrays describe, and
// whether they can be trusted.  A head with a problem keeps its whole cache (keep_everything).
struct HeadShape {
  int n_tok, n_sent, sp, budget;
  int problem;  // SKIPKV_DEV_* bits, 0: fine so far
};
__device__ __forceinline__ HeadShape head_shape(const SelectArgs &a, int lhb) {
  const int b = lhb % a.batch;
  HeadShape h;
  const int room_tok = a.seq_off[b + 1] - a.seq_off[b];
  const int n_tok_raw = seq_tokens(a.seq_off, a.len, b);
  h.sp = a.sent_ptr[b];
  const int room_sent = a.sent_ptr[b + 1] - h.sp - 1;
  const int n_sent_raw = seq_sentences(a.sent_ptr, a.cnt, b);
  h.n_tok = max(0, min(n_tok_raw, room_tok));
  h.n_sent = max(0, min(n_sent_raw, room_sent));
  h.budget = a.budget ? a.budget[b] : a.budget_scalar;
  h.problem = 0;
  if (h.n_tok != n_tok_raw || h.n_sent != n_sent_raw || (h.n_sent == 0 && h.n_tok != 0)) h.problem |= SKIPKV_DEV_BAD_OFFSETS;
  if (h.n_sent > SKIPKV_MAX_SENTENCES) h.problem |= SKIPKV_DEV_TOO_MANY_SENT;
  // the kept indices must fit their row, and the protected window must fit the budget
  const int protect = min(a.protect, h.n_tok);
  if (h.budget < 0 || min(h.budget, h.n_tok) > a.kept_stride || (h.n_tok > h.budget && h.budget < protect)) h.problem |= SKIPKV_DEV_BAD_BUDGET;
  return h;
}

// A head whose inputs cannot be trusted (offsets, counts, budget, a NaN score) keeps everything:
// new_len = N, the identity as far as the row of kept indices reaches, every sentence flagged
// kept, ranges copied.  The compaction leaves a head with new_len > kept_stride alone and moves
// nothing where the indices are the identity, so the cache of such a head is not touched.
__device__ __forceinline__ void keep_everything(const SelectArgs &a, int lhb, const HeadShape &h, int gt, int G, int problem) {
  const int lh = lhb / a.batch, b = lhb % a.batch;
  int32_t *kept = a.kept_idx + (int64_t)lhb * a.kept_stride;
  const int64_t col0 = (int64_t)lh * a.total_sentences + (h.sp - b);
  const int n_sent = min(h.n_sent, SKIPKV_MAX_SENTENCES);
  for (int t = gt; t < min(h.n_tok, a.kept_stride); t += G) kept[t] = t;
  if (a.sent_keep)
    for (int s = gt; s < n_sent; s += G) a.sent_keep[col0 + s] = 1;
  if (a.new_sent_off) {
    int32_t *noff = a.new_sent_off + (int64_t)lh * (a.total_sentences + a.batch) + h.sp;
    const int32_t *off = a.sent_off + h.sp;
    for (int s = gt; s <= n_sent; s += G) noff[s] = off[s];
  }
  if (gt == 0) {
    a.new_len[lhb] = h.n_tok;
    if (a.new_sent_cnt) a.new_sent_cnt[lhb] = n_sent;
    if (problem && a.dev_status) atomicOr(a.dev_status, problem);
  }
}

// One head, handled by NW waves; gt = thread index inside the group, gw = wave inside the group.
// keep_l: 1024 * NW bytes of LDS, 16-byte aligned.
template <int NW>
__device__ __forceinline__ void select_head(const SelectArgs &a, int lhb, const HeadShape &hs, int gt, int gw, uint8_t *keep_l, Exchange &x) {
  constexpr int G = 64 * NW;
  const int lane = gt & 63;
  const int lh = lhb / a.batch, b = lhb % a.batch;
  const int n_tok = hs.n_tok, sp = hs.sp, n_sent = hs.n_sent, budget = hs.budget;
  const int32_t *off = a.sent_off + sp;
  const int64_t col0 = (int64_t)lh * a.total_sentences + (sp - b);
  int32_t *kept = a.kept_idx + (int64_t)lhb * a.kept_stride;
  int32_t *noff = a.new_sent_off ? a.new_sent_off + (int64_t)lh * (a.total_sentences + a.batch) + sp : nullptr;

  if (hs.problem || n_tok <= budget) {  // nothing can be evicted, or the cache already fits
    keep_everything(a, lhb, hs, gt, G, hs.problem);
    return;
  }

  const int p_start = n_tok - min(a.protect, n_tok);
  const int room = budget - (n_tok - p_start);

  // ---- candidates, sentence s = r * G + gt: order-preserving image of the score, unprotected length
  uint32_t hi[kEPL];
  int len[kEPL];
  int bad = 0;  // low half: offsets out of order, high half: NaN scores
#pragma unroll
  for (int r = 0; r < kEPL; ++r) {
    const int s = r * G + gt;
    hi[r] = 0;
    len[r] = 0;  // not a candidate: protected, or past the end
    if (s < n_sent) {
      const int o0 = off[s], o1 = off[s + 1];
      // the ranges must run from 0 to N, strictly ascending (the scores of a head whose ranges the
      // plan rejected were never written)
      if (o1 <= o0 || (s == 0 && o0 != 0) || (s == n_sent - 1 && o1 != n_tok)) bad += 1;
      if (o0 < p_start) {
        const float sc = a.sent_score[col0 + s];
        if (sc != sc) bad += 1 << 16;  // a NaN cannot be ranked (the scan marks scores it could not finish this way)
        uint32_t u = __float_as_uint(sc);
        if (u == 0x80000000u) u = 0;  // -0.0 ties with 0.0
        hi[r] = (u & 0x80000000u) ? ~u : (u | 0x80000000u);
        len[r] = max(0, min(o1, p_start) - o0);
      }
    }
  }
  bad = group_sum<NW>(bad, gw, x);
  if (bad) {
    keep_everything(a, lhb, hs, gt, G, (bad & 0xFFFF) ? SKIPKV_DEV_BAD_OFFSETS : SKIPKV_DEV_BAD_SCORES);  // scores under bad ranges were never written
    return;
  }

  // ---- score part of K0: the largest H such that the candidates with hi >= H do not fit.
  // (All candidates together are p_start > room tokens, so H = 0 qualifies.)
  uint32_t H = 0;
  for (int bit = 31; bit >= 0; --bit) {
    const uint32_t th = H | (1u << bit);
    int part = 0;
#pragma unroll
    for (int r = 0; r < kEPL; ++r) part += hi[r] >= th ? len[r] : 0;
    if (group_sum<NW>(part, gw, x) > room) H = th;
  }
  // ---- index part: among the candidates with hi == H, the largest index bound L such that those
  // with index >= L, together with everything above H (which fits), do not fit
  int above = 0;
  int se[kEPL];
#pragma unroll
  for (int r = 0; r < kEPL; ++r) {
    above += hi[r] > H ? len[r] : 0;
    se[r] = (hi[r] == H && len[r] > 0) ? r * G + gt : -1;
  }
  above = group_sum<NW>(above, gw, x);
  int L = 0;
  for (int bit = 11; bit >= 0; --bit) {
    const int tl = L | (1 << bit);
    int part = 0;
#pragma unroll
    for (int r = 0; r < kEPL; ++r) part += se[r] >= tl ? len[r] : 0;
    if (above + group_sum<NW>(part, gw, x) > room) L = tl;
  }
  // ---- keep flags: key > (H, L); sentences that are not candidates keep their (protected) tokens
#pragma unroll
  for (int r = 0; r < kEPL; ++r) {
    const int s = r * G + gt;
    if (s < n_sent) {
      const uint8_t k = len[r] == 0 || hi[r] > H || (hi[r] == H && s > L);
      keep_l[s] = k;
      if (a.sent_keep) a.sent_keep[col0 + s] = k;
    }
  }
  if constexpr (NW > 1) __syncthreads();

  // ---- sentences in index order, 16 consecutive ones per thread: every sentence keeps one
  // contiguous run of tokens (its unprotected part if kept, followed by its protected part)
  const int s0 = gt * kEPL;
  const uint4 kb4 = *reinterpret_cast<const uint4 *>(keep_l + s0);
  const uint32_t kb[4] = {kb4.x, kb4.y, kb4.z, kb4.w};
  int run_bgn[kEPL], run_len[kEPL], run_dst[kEPL];
  int o_prev = off[min(s0, n_sent)];
  int tok = 0, sent = 0;
#pragma unroll
  for (int r = 0; r < kEPL; ++r) {
    const int s = s0 + r;
    const int end = off[min(s + 1, n_sent)];
    const bool kp = (kb[r >> 2] >> (8 * (r & 3))) & 0xFF;
    const int bgn = kp ? o_prev : max(o_prev, p_start);
    const int n = s < n_sent ? max(0, end - bgn) : 0;
    run_bgn[r] = bgn;
    run_len[r] = n;
    tok += n;
    sent += n > 0;
    o_prev = end;
  }
  int total_tok, total_sent;
  int tok_run = group_scan_excl<NW>(tok, gw, lane, x, total_tok);
  int sent_run = group_scan_excl<NW>(sent, gw, lane, x, total_sent);
#pragma unroll
  for (int r = 0; r < kEPL; ++r) {
    run_dst[r] = tok_run;
    if (run_len[r] > 0) {
      if (noff) noff[sent_run] = tok_run;
      tok_run += run_len[r];
      ++sent_run;
    }
  }
  if (gt == 0) {
    a.new_len[lhb] = total_tok;
    if (a.new_sent_cnt) a.new_sent_cnt[lhb] = total_sent;
    if (noff) noff[total_sent] = total_tok;
  }
  // ---- ascending surviving token indices: the wave writes the runs of its lanes one after the other
#pragma unroll
  for (int r = 0; r < kEPL; ++r) {
    unsigned long long todo = __ballot(run_len[r] > 0);
    while (todo) {
      const int l = __builtin_ctzll(todo);
      todo &= todo - 1;
      const int bgn = __builtin_amdgcn_readlane(run_bgn[r], l);
      const int n = __builtin_amdgcn_readlane(run_len[r], l);
      const int d = __builtin_amdgcn_readlane(run_dst[r], l);
      for (int i = lane; i < n; i += 64) kept[d + i] = bgn + i;
    }
  }
}

__global__ void __launch_bounds__(256, 4) k_select(SelectArgs a) {
  __shared__ __align__(16) uint8_t keep_l[4 * kWaveSent];
  __shared__ int slots[8];
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int n_heads = a.n_lh * a.batch;
  Exchange x{slots, 0};

  {  // every wave takes one head of its own if the head is small enough
    const int lhb = blockIdx.x * 4 + wave;
    if (lhb < n_heads) {
      const HeadShape hs = head_shape(a, lhb);
      if (hs.n_sent <= kWaveSent) select_head<1>(a, lhb, hs, lane, 0, keep_l + wave * kWaveSent, x);
    }
  }
  for (int w = 0; w < 4; ++w) {  // the larger heads, one after the other, by the whole workgroup
    const int lhb = blockIdx.x * 4 + w;
    if (lhb >= n_heads) break;
    const HeadShape hs = head_shape(a, lhb);
    if (hs.n_sent <= kWaveSent) continue;
    __syncthreads();  // the flag buffer is free: every wave is done with its own head (or the previous large one)
    select_head<4>(a, lhb, hs, tid, wave, keep_l, x);  // more than SKIPKV_MAX_SENTENCES: flagged by head_shape, keeps everything
  }
}

// ---------------------------------------------------------------------------------------------
// Token-level form (Eq. 6 as printed, then "evict tokens in increasing order of the final score"):
// every token carries sigma * I - (1 - sigma) * R, minus its sentence's lambda when the sentence
// is in the redundant set; the protected recent window is kept and exactly budget - window of the
// other tokens survive, ranked by (score descending, index descending).  Same search for the cut
// key as above, with counts in place of lengths.  One workgroup per head.
constexpr int kMaxTokens = SKIPKV_MAX_TOKENS_TOKEN_SELECT;

__device__ __forceinline__ int block_sum(int v, int *slots /*[2][4]*/, int &call, int wave, int lane) {
  const int s = wave_sum_i(v);
  int *slot = slots + 4 * (call & 1);
  ++call;
  if (lane == 0) slot[wave] = s;
  __syncthreads();
  return slot[0] + slot[1] + slot[2] + slot[3];
}
__device__ __forceinline__ int block_scan_excl(int v, int *slots, int &call, int wave, int lane, int &total) {
  const int incl = wave_scan_incl(v, lane);
  const int wtot = __builtin_amdgcn_readlane(incl, 63);
  int *slot = slots + 4 * (call & 1);
  ++call;
  if (lane == 0) slot[wave] = wtot;
  __syncthreads();
  int before = 0;
#pragma unroll
  for (int w = 0; w < 4; ++w)
    if (w < wave) before += slot[w];
  total = slot[0] + slot[1] + slot[2] + slot[3];
  return before + incl - v;
}
__device__ __forceinline__ uint32_t score_order(float f) {  // order-preserving image; -0.0 ties with 0.0
  uint32_t u = __float_as_uint(f);
  if (u == 0x80000000u) u = 0;
  return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}

__global__ void __launch_bounds__(256) k_select_tokens(TokSelectArgs a) {
  __shared__ uint32_t keep_bits[kMaxTokens / 32];
  __shared__ int off_l[SKIPKV_MAX_SENTENCES + 1];
  __shared__ int slots[8];
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
  const int lhb = blockIdx.x, lh = lhb / a.batch, b = lhb % a.batch;
  const int tok0 = a.seq_off[b];
  const int n_tok_raw = seq_tokens(a.seq_off, a.len, b);
  const int n_tok = max(0, min(n_tok_raw, a.seq_off[b + 1] - tok0));  // per-head ranges: the head's own length, within its room
  const int sp = a.sent_ptr[b];
  const int n_sent_raw = seq_sentences(a.sent_ptr, a.cnt, b);
  const int n_sent = max(0, min(n_sent_raw, a.sent_ptr[b + 1] - sp - 1));
  const int32_t *off = a.sent_off + sp;
  const int64_t tcol = (int64_t)lh * a.total_tokens + tok0;
  const int64_t scol = (int64_t)lh * a.total_sentences + (sp - b);
  int32_t *kept = a.kept_idx + (int64_t)lhb * a.kept_stride;
  int32_t *noff = a.new_sent_off ? a.new_sent_off + (int64_t)lh * (a.total_sentences + a.batch) + sp : nullptr;
  const int budget = a.budget ? a.budget[b] : a.budget_scalar;
  int call = 0;

  // A head whose inputs cannot be trusted keeps everything (see keep_everything above): sizes outside
  // the room or the kernel's limits, a budget that the row of kept indices or the protected window
  // does not fit, ranges that do not run strictly ascending from 0 to N.
  int problem = 0;
  if (n_tok > kMaxTokens) problem |= SKIPKV_DEV_TOO_MANY_TOK;
  if (n_sent > SKIPKV_MAX_SENTENCES) problem |= SKIPKV_DEV_TOO_MANY_SENT;
  if (n_tok != n_tok_raw || n_sent != n_sent_raw || (n_sent == 0 && n_tok != 0)) problem |= SKIPKV_DEV_BAD_OFFSETS;
  if (budget < 0 || min(budget, n_tok) > a.kept_stride || (n_tok > budget && budget < min(a.protect, n_tok))) problem |= SKIPKV_DEV_BAD_BUDGET;
  if (!problem) {
    int bad = 0;
    for (int s = tid; s < n_sent; s += 256) {
      const int o0 = off[s], o1 = off[s + 1];
      bad |= o1 <= o0 || (s == 0 && o0 != 0) || (s == n_sent - 1 && o1 != n_tok);
    }
    if (block_sum(bad, slots, call, wave, lane)) problem |= SKIPKV_DEV_BAD_OFFSETS;
  }
  if (problem) {
    const int ns = min(n_sent, SKIPKV_MAX_SENTENCES);
    for (int t = tid; t < min(n_tok, a.kept_stride); t += 256) kept[t] = t;
    if (a.tok_keep)
      for (int t = tid; t < n_tok; t += 256) a.tok_keep[tcol + t] = 1;
    if (noff)
      for (int s = tid; s <= ns; s += 256) noff[s] = off[s];
    if (tid == 0) {
      if (a.dev_status) atomicOr(a.dev_status, problem);
      a.new_len[lhb] = n_tok;
      if (a.new_sent_cnt) a.new_sent_cnt[lhb] = ns;
    }
    return;
  }

  // ---- token scores (Eq. 6): thread t takes tokens t, t+256, ... (coalesced); the sentence of a
  // token is found by bisection in the offsets, which sit in LDS
  float *score = a.tok_score + tcol;
  for (int s = tid; s <= n_sent; s += 256) off_l[s] = off[s];
  __syncthreads();
  for (int t = tid; t < n_tok; t += 256) {
    int lo = 0, hi = n_sent - 1;  // invariant: off_l[lo] <= t < off_l[hi + 1]
    while (lo < hi) {
      const int mid = (lo + hi + 1) >> 1;
      if (off_l[mid] <= t) lo = mid; else hi = mid - 1;
    }
    const float lam = a.sent_lambda[scol + lo];
    float v = a.sigma * a.tok_imp[tcol + t];
    if (a.tok_red) v -= (1.f - a.sigma) * a.tok_red[tcol + t];
    score[t] = v - (lam > a.tau ? lam : 0.f);
  }
  __syncthreads();  // the scores are read back by other threads of this workgroup

  const int p_start = n_tok - min(a.protect, n_tok);
  uint32_t H = 0;
  int L = -1;  // keep = key > (H, L); (0, -1) keeps everything
  if (n_tok > budget) {
    const int room = budget - (n_tok - p_start);
    // The order images of the unprotected tokens t = tid + 256 r stay in registers when the
    // sequence is short enough (EPL per thread); longer sequences re-read the scores from L2.
    auto search = [&](auto epl_tag) {
      constexpr int EPL = decltype(epl_tag)::value;
      uint32_t key[EPL > 0 ? EPL : 1];
      if constexpr (EPL > 0) {
#pragma unroll
        for (int r = 0; r < EPL; ++r) {
          const int t = tid + 256 * r;
          key[r] = t < p_start ? score_order(score[t]) : 0u;
        }
      }
      auto count = [&](auto pred) -> int {  // number of unprotected tokens with pred(order, index)
        int cnt = 0;
        if constexpr (EPL > 0) {
#pragma unroll
          for (int r = 0; r < EPL; ++r) cnt += (tid + 256 * r < p_start) && pred(key[r], tid + 256 * r);
        } else {
          for (int t = tid; t < p_start; t += 256) cnt += pred(score_order(score[t]), t);
        }
        return block_sum(cnt, slots, call, wave, lane);
      };
      // score part: the largest H such that more than `room` unprotected tokens have order >= H
      for (int bit = 31; bit >= 0; --bit) {
        const uint32_t th = H | (1u << bit);
        if (count([&](uint32_t o, int) { return o >= th; }) > room) H = th;
      }
      const int above = count([&](uint32_t o, int) { return o > H; });
      // index part: the largest L such that, among the tokens with order == H, those with index >= L do not fit
      L = 0;
      for (int bit = 31 - __builtin_clz(max(p_start, 1)); bit >= 0; --bit) {
        const int tl = L | (1 << bit);
        if (above + count([&](uint32_t o, int t) { return o == H && t >= tl; }) > room) L = tl;
      }
    };
    if (p_start <= 256 * 16)
      search(std::integral_constant<int, 16>{});
    else if (p_start <= 256 * 64)
      search(std::integral_constant<int, 64>{});
    else
      search(std::integral_constant<int, 0>{});
  }

  // ---- keep flags as a bit map in LDS, set token by token in the coalesced order; then every
  // thread owns a run of whole 32-token words of it
  const int words = (n_tok + 31) / 32;
  const int per_w = (words + 255) / 256;
  for (int w = tid; w < words; w += 256) keep_bits[w] = 0;
  __syncthreads();
  for (int t = tid; t < n_tok; t += 256) {
    bool k = t >= p_start;
    if (!k) {
      const uint32_t o = score_order(score[t]);
      k = o > H || (o == H && t > L);
    }
    if (k) atomicOr(&keep_bits[t >> 5], 1u << (t & 31));
    if (a.tok_keep) a.tok_keep[tcol + t] = k;
  }
  __syncthreads();
  int mine = 0;
  for (int w = tid * per_w; w < min((tid + 1) * per_w, words); ++w) mine += __popc(keep_bits[w]);
  int total_tok;
  int dst = block_scan_excl(mine, slots, call, wave, lane, total_tok);  // also makes the bit map visible
  for (int w = tid * per_w; w < min((tid + 1) * per_w, words); ++w) {
    uint32_t bits = keep_bits[w];
    while (bits) {
      const int i = __builtin_ctz(bits);
      bits &= bits - 1;
      kept[dst++] = 32 * w + i;
    }
  }

  // ---- sentences that still have a token, and where they now start (Eq. 11)
  const int per_s = (n_sent + 255) / 256;
  const int s_lo = tid * per_s, s_hi = min(s_lo + per_s, n_sent);
  auto survivors = [&](int s) -> int {
    int cnt = 0;
    const int bgn = off[s], end = off[s + 1];
    for (int w = bgn >> 5; w <= (end - 1) >> 5; ++w) {
      uint32_t m = keep_bits[w];
      if (w == (bgn >> 5)) m &= 0xFFFFFFFFu << (bgn & 31);
      if (w == ((end - 1) >> 5) && (end & 31)) m &= 0xFFFFFFFFu >> (32 - (end & 31));
      cnt += __popc(m);
    }
    return cnt;
  };
  int sent_cnt = 0;
  for (int s = s_lo; s < s_hi; ++s) sent_cnt += survivors(s) > 0;
  int my_tok = 0;
  for (int s = s_lo; s < s_hi; ++s) my_tok += survivors(s);
  int tot_t, tot_s;
  int tok_before = block_scan_excl(my_tok, slots, call, wave, lane, tot_t);  // kept tokens before this thread's first sentence
  int sent_before = block_scan_excl(sent_cnt, slots, call, wave, lane, tot_s);
  for (int s = s_lo; s < s_hi; ++s) {
    const int c = survivors(s);
    if (c > 0) {
      if (noff) noff[sent_before] = tok_before;
      ++sent_before;
      tok_before += c;
    }
  }
  if (tid == 0) {
    a.new_len[lhb] = total_tok;
    if (a.new_sent_cnt) a.new_sent_cnt[lhb] = tot_s;
    if (noff) noff[tot_s] = total_tok;
  }
}

}  // namespace

hipError_t launch_select_tokens(const TokSelectArgs &a, hipStream_t st) {
  const int heads = a.n_lh * a.batch;
  if (heads == 0) return hipSuccess;
  hipLaunchKernelGGL(k_select_tokens, dim3(heads), dim3(256), 0, st, a);
  return hipGetLastError();
}

hipError_t launch_select(const SelectArgs &a, hipStream_t st) {
  const int heads = a.n_lh * a.batch;
  if (heads == 0) return hipSuccess;
  hipLaunchKernelGGL(k_select, dim3((heads + 3) / 4), dim3(256), 0, st, a);
  return hipGetLastError();
}

}  // namespace skipkv

// Budgeted whole-sentence selection (Sec. 4.1, text after Eq. 6: tokens are evicted in
// increasing order of the score until the budget is met; here the unit of eviction is a
// sentence) and the surviving index set P with the remapped sentence ranges (Eq. 11).
//
// One workgroup per head.  Candidates are ranked by (score descending, index descending) with
// a bitonic sort of 64-bit keys in LDS; since every candidate has length >= 1 the prefix sums
// of the ranked lengths are strictly increasing, so "longest prefix that fits" is simply
// "inclusive prefix <= room" for each rank independently.
#include "common.h"

namespace skipkv {

namespace {

constexpr int kMaxS = SKIPKV_MAX_SENTENCES;

// Inclusive scan of one int per thread over the 256 threads of the block.
__device__ __forceinline__ int block_scan_incl(int v, int *tmp /*[256]*/, int tid) {
  tmp[tid] = v;
  __syncthreads();
  for (int d = 1; d < 256; d <<= 1) {
    const int add = tid >= d ? tmp[tid - d] : 0;
    __syncthreads();
    tmp[tid] += add;
    __syncthreads();
  }
  return tmp[tid];
}

__global__ void __launch_bounds__(256) k_select(SelectArgs a) {
  __shared__ unsigned long long keys[kMaxS];
  __shared__ int dst[kMaxS + 1];       // first: ranked candidate lengths, then destination offsets by sentence
  __shared__ uint8_t keep[kMaxS];
  __shared__ int tmp[256];
  __shared__ int s_total, s_nsurv;

  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
  const int lhb = blockIdx.x, lh = lhb / a.batch, b = lhb % a.batch;
  const int n_tok = a.seq_off[b + 1] - a.seq_off[b];
  const int sp = a.sent_ptr[b];
  const int n_sent = a.sent_ptr[b + 1] - sp - 1;
  const int32_t *off = a.sent_off + sp;
  const int64_t col0 = (int64_t)lh * a.total_sentences + (sp - b);
  int32_t *kept = a.kept_idx + (int64_t)lhb * a.kept_stride;
  int32_t *noff = a.new_sent_off ? a.new_sent_off + (int64_t)lh * (a.total_sentences + a.batch) + sp : nullptr;
  const int budget = a.budget ? a.budget[b] : a.budget_scalar;

  if (n_sent > kMaxS || n_sent < 0) {
    if (tid == 0) {
      if (a.dev_status) atomicOr(a.dev_status, SKIPKV_DEV_TOO_MANY_SENT);
      a.new_len[lhb] = 0;
      if (a.new_sent_cnt) a.new_sent_cnt[lhb] = 0;
    }
    return;
  }

  if (n_tok <= budget) {  // the cache already fits: nothing is evicted
    for (int t = tid; t < n_tok; t += 256) kept[t] = t;
    for (int s = tid; s < n_sent; s += 256)
      if (a.sent_keep) a.sent_keep[col0 + s] = 1;
    if (noff)
      for (int s = tid; s <= n_sent; s += 256) noff[s] = off[s];
    if (tid == 0) {
      a.new_len[lhb] = n_tok;
      if (a.new_sent_cnt) a.new_sent_cnt[lhb] = n_sent;
    }
    return;
  }

  const int p_start = n_tok - min(a.protect, n_tok);
  const int room = budget - (n_tok - p_start);
  int p2 = 256;
  while (p2 < n_sent) p2 <<= 1;

  // ---- keys: order-preserving image of the score in the high word, sentence index in the low
  for (int s = tid; s < p2; s += 256) {
    unsigned long long key = 0;  // padding and non-candidates rank last
    if (s < n_sent && off[s] < p_start) {
      const uint32_t u = __float_as_uint(a.sent_score[col0 + s] + 0.f);  // +0: -0.0 ties with 0.0
      const uint32_t ord = (u & 0x80000000u) ? ~u : (u | 0x80000000u);
      key = ((unsigned long long)ord << 32) | (uint32_t)s;
    }
    keys[s] = key;
    if (s < n_sent) keep[s] = 1;
  }
  __syncthreads();

  // ---- bitonic sort, descending
  for (int k = 2; k <= p2; k <<= 1) {
    for (int j = k >> 1; j > 0; j >>= 1) {
      for (int i = tid; i < p2; i += 256) {
        const int ixj = i ^ j;
        if (ixj > i) {
          const unsigned long long x = keys[i], y = keys[ixj];
          const bool desc = (i & k) == 0;
          if (desc ? (x < y) : (x > y)) {
            keys[i] = y;
            keys[ixj] = x;
          }
        }
      }
      __syncthreads();
    }
  }

  // ---- inclusive prefix of the ranked candidate lengths; keep while it fits
  const int per = p2 / 256;
  int local = 0;
  for (int i = tid * per; i < (tid + 1) * per; ++i) {
    const unsigned long long key = keys[i];
    int len = 0;
    if (key != 0) {
      const int s = (int)(uint32_t)key;
      len = min(off[s + 1], p_start) - off[s];
    }
    dst[i] = len;
    local += len;
  }
  int run = block_scan_incl(local, tmp, tid) - local;
  for (int i = tid * per; i < (tid + 1) * per; ++i) {
    run += dst[i];
    const unsigned long long key = keys[i];
    if (key != 0) keep[(int)(uint32_t)key] = run <= room;
  }
  __syncthreads();

  // ---- surviving tokens of every sentence in index order -> destination offsets
  const int per_s = (n_sent + 255) / 256;
  const int s_lo = tid * per_s, s_hi = min(s_lo + per_s, n_sent);
  int tok_cnt = 0, sent_cnt = 0;
  for (int s = s_lo; s < s_hi; ++s) {
    const int bgn = off[s], end = off[s + 1];
    const int cand = keep[s] ? max(0, min(end, p_start) - bgn) : 0;
    const int prot = max(0, end - max(bgn, p_start));
    tok_cnt += cand + prot;
    sent_cnt += (cand + prot) > 0;
  }
  int tok_run = block_scan_incl(tok_cnt, tmp, tid) - tok_cnt;
  if (tid == 255) s_total = tok_run + tok_cnt;
  __syncthreads();
  int sent_run = block_scan_incl(sent_cnt, tmp, tid) - sent_cnt;
  if (tid == 255) s_nsurv = sent_run + sent_cnt;
  for (int s = s_lo; s < s_hi; ++s) {
    const int bgn = off[s], end = off[s + 1];
    const int cand = keep[s] ? max(0, min(end, p_start) - bgn) : 0;
    const int prot = max(0, end - max(bgn, p_start));
    dst[s] = tok_run;
    if (cand + prot > 0 && noff) noff[sent_run] = tok_run;
    tok_run += cand + prot;
    sent_run += (cand + prot) > 0;
    if (a.sent_keep) a.sent_keep[col0 + s] = keep[s];
  }
  __syncthreads();
  if (tid == 0) {
    a.new_len[lhb] = s_total;
    if (a.new_sent_cnt) a.new_sent_cnt[lhb] = s_nsurv;
    if (noff) noff[s_nsurv] = s_total;
  }

  // ---- ascending surviving token indices, one wave per sentence
  for (int s = wave; s < n_sent; s += 4) {
    const int bgn = off[s], end = off[s + 1];
    const int c_end = keep[s] ? min(end, p_start) : bgn;  // kept candidate part [bgn, c_end)
    const int p_bgn = max(bgn, p_start);                   // protected part [p_bgn, end)
    const int n_c = max(0, c_end - bgn), n_p = max(0, end - p_bgn);
    const int d0 = dst[s];
    for (int i = lane; i < n_c + n_p; i += 64) kept[d0 + i] = i < n_c ? bgn + i : p_bgn + (i - n_c);
  }
}

}  // namespace

hipError_t launch_select(const SelectArgs &a, hipStream_t st) {
  const int blocks = a.n_lh * a.batch;
  if (blocks == 0) return hipSuccess;
  hipLaunchKernelGGL(k_select, dim3(blocks), dim3(256), 0, st, a);
  return hipGetLastError();
}

}  // namespace skipkv

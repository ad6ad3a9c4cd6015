// Per-head sentence ranges across compression steps (Sec. 4.1 "Sentence-level eviction", Eq. 9-11).
// After the first step every (layer, KV head, sequence) has evicted its own sentences, so cache
// lengths and sentence ranges are per head.  Eq. 11 (remapping the surviving ranges onto the
// compacted cache) is part of the selection kernel; here are the append rule of Eq. 10 and the
// bookkeeping that lets the kernels of the step see each head as a sequence of its own.
#include "common.h"

namespace skipkv {

namespace {

// Positions are cache positions: the shift by the number of evicted tokens that Eq. 10 writes
// out is already contained in the per-head cache length.
__global__ void __launch_bounds__(256) k_ranges_append(RangesAppendArgs a) {
  const int v = blockIdx.x * 256 + threadIdx.x;
  if (v >= a.n_lh * a.batch) return;
  const int lh = v / a.batch, b = v % a.batch;
  const int n = a.n_new[b];
  if (n <= 0) return;
  const int sp = a.sent_ptr[b];
  const int cap_s = a.sent_ptr[b + 1] - sp - 1, cap_t = a.seq_off[b + 1] - a.seq_off[b];
  int32_t *off = a.off + (int64_t)lh * (a.total_sentences + a.batch) + sp;
  const int N = a.len[v], S = a.cnt[v];
  const int32_t *bnd = a.bnd_off + a.bnd_ptr[b];
  const int m = a.bnd_ptr[b + 1] - a.bnd_ptr[b];
  // boundaries: strictly ascending positions inside the appended run
  bool bad = N < 0 || S < 0 || S > cap_s || n > cap_t - N || (S == 0 && N != 0);
  int inner = 0, prev = -1;
  for (int j = 0; j < m; ++j) {
    const int p = bnd[j];
    bad |= (p <= prev) | (p >= n);
    prev = p;
    inner += p > 0;
  }
  // the first appended token opens a sentence if the cache is empty or a boundary says so;
  // otherwise it continues the last sentence, whose end moves
  const bool starts_new = S == 0 || (m > 0 && bnd[0] == 0);
  const int S_new = S + inner + (starts_new ? 1 : 0);
  if (bad || S_new > cap_s) {
    if (a.dev_status) atomicOr(a.dev_status, bad ? SKIPKV_DEV_BAD_OFFSETS : SKIPKV_DEV_TOO_MANY_SENT);
    return;
  }
  int w;  // index of the offset written next
  if (S == 0) {
    off[0] = 0;
    w = 1;
  } else {
    w = starts_new ? S + 1 : S;  // o[S] = N stays (sentence closed) or is overwritten (sentence grows)
  }
  for (int j = 0; j < m; ++j)
    if (bnd[j] > 0) off[w++] = N + bnd[j];
  off[w] = N + n;  // w == S_new
  a.cnt[v] = w;
  a.len[v] = N + n;
}

__global__ void __launch_bounds__(256) k_virtual_layout(const int32_t *seq_off, const int32_t *sent_ptr, int batch, int n_lh,
                                                        int total_tokens, int total_sentences, int32_t *v_seq_off,
                                                        int32_t *v_sent_ptr) {
  const int v = blockIdx.x * 256 + threadIdx.x;
  const int n = n_lh * batch;
  if (v > n) return;
  if (v == n) {
    v_seq_off[v] = n_lh * total_tokens;
    v_sent_ptr[v] = n_lh * (total_sentences + batch);
    return;
  }
  const int lh = v / batch, b = v % batch;
  v_seq_off[v] = lh * total_tokens + seq_off[b];
  v_sent_ptr[v] = lh * (total_sentences + batch) + sent_ptr[b];
}

}  // namespace

hipError_t launch_ranges_append(const RangesAppendArgs &a, hipStream_t st) {
  const int n = a.n_lh * a.batch;
  if (n == 0) return hipSuccess;
  hipLaunchKernelGGL(k_ranges_append, dim3((n + 255) / 256), dim3(256), 0, st, a);
  return hipGetLastError();
}

hipError_t launch_virtual_layout(const int32_t *seq_off, const int32_t *sent_ptr, int32_t batch, int32_t n_lh, int32_t total_tokens,
                                 int32_t total_sentences, int32_t *v_seq_off, int32_t *v_sent_ptr, hipStream_t st) {
  const int n = n_lh * batch + 1;
  hipLaunchKernelGGL(k_virtual_layout, dim3((n + 255) / 256), dim3(256), 0, st, seq_off, sent_ptr, batch, n_lh, total_tokens,
                     total_sentences, v_seq_off, v_sent_ptr);
  return hipGetLastError();
}

}  // namespace skipkv

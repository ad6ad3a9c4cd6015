// Per-head sentence ranges across compression steps (Sec. 4.1 "KV Cache Sentence Range Monitoring Logic", Eq. 9-11).
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

// One wave per (layer, head, sequence): stream compaction of the sentence numbers, 64 at a time.
// Every chunk is read before anything of it is written and writes never run ahead of the reads,
// so id_out may be id_in.
__global__ void __launch_bounds__(256) k_ranges_ids_select(RangesIdsArgs a) {
  const int v = blockIdx.x * 4 + (threadIdx.x >> 6), lane = threadIdx.x & 63;
  if (v >= a.n_lh * a.batch) return;
  const int lh = v / a.batch, b = v % a.batch;
  const int sp = a.sent_ptr[b];
  const int room = a.sent_ptr[b + 1] - sp - 1, room_t = a.seq_off[b + 1] - a.seq_off[b];
  const int n = a.old_cnt ? min(max(a.old_cnt[v], 0), room) : room;
  const int n_tok = a.len ? min(max(a.len[v], 0), room_t) : room_t;
  const int p_start = n_tok - min(a.protect, n_tok);  // first protected token
  const int32_t *off = a.off ? a.off + (int64_t)lh * (a.total_sentences + a.batch) + sp : a.sent_off + sp;
  const int64_t col = (int64_t)lh * a.total_sentences + (sp - b);
  int k = 0;
  for (int s0 = 0; s0 < n; s0 += 64) {
    const int s = s0 + lane;
    const bool stays = s < n && (a.keep[col + s] != 0 || off[s + 1] > p_start);
    const int id = stays ? (a.id_in ? a.id_in[col + s] : s) : 0;
    const unsigned long long m = __ballot(stays);
    if (stays) a.id_out[col + k + __popcll(m & ((1ull << lane) - 1ull))] = id;
    k += __popcll(m);
  }
}

__global__ void __launch_bounds__(256) k_ranges_ids_append(RangesIdsArgs a) {
  const int v = blockIdx.x * 4 + (threadIdx.x >> 6), lane = threadIdx.x & 63;
  if (v >= a.n_lh * a.batch) return;
  const int lh = v / a.batch, b = v % a.batch;
  const int room = a.sent_ptr[b + 1] - a.sent_ptr[b] - 1;
  const int co = min(max(a.old_cnt[v], 0), room), cn = min(a.new_cnt[v], room);
  const int64_t col = (int64_t)lh * a.total_sentences + (a.sent_ptr[b] - b);
  const int next = co > 0 ? a.id_out[col + co - 1] + 1 : 0;
  for (int s = co + lane; s < cn; s += 64) a.id_out[col + s] = next + (s - co);
}

}  // namespace

hipError_t launch_ranges_ids_select(const RangesIdsArgs &a, hipStream_t st) {
  const int n = a.n_lh * a.batch;
  if (n == 0) return hipSuccess;
  hipLaunchKernelGGL(k_ranges_ids_select, dim3((n + 3) / 4), dim3(256), 0, st, a);
  return hipGetLastError();
}

hipError_t launch_ranges_ids_append(const RangesIdsArgs &a, hipStream_t st) {
  const int n = a.n_lh * a.batch;
  if (n == 0) return hipSuccess;
  hipLaunchKernelGGL(k_ranges_ids_append, dim3((n + 3) / 4), dim3(256), 0, st, a);
  return hipGetLastError();
}

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

// Work decomposition for one compression step: cuts every sequence's sentence list into
// chunks (units of the key scan) and row blocks (units of the redundancy kernel), and checks
// the sentence offsets.  Shared by all layers and heads of the batch, so it is tiny.
#include "common.h"

namespace skipkv {

__global__ void k_plan_reset(PlanHeader *hdr) {
  if (threadIdx.x == 0) {
    hdr->n_chunks = 0;
    hdr->n_rowblocks = 0;
  }
}

// One block per sequence.  A sentence s begins a new chunk when it starts in a different
// window of kChunkWindow tokens than sentence s-1, or when it is the (k*kChunkMaxSent)-th
// sentence starting in its window.  Chunks therefore hold whole sentences, at most
// kChunkMaxSent of them, and about kChunkWindow tokens.
__global__ void __launch_bounds__(256) k_plan(PlanArgs a) {
  const int b = blockIdx.x;
  const int tid = threadIdx.x;
  const int n_tok = a.seq_off[b + 1] - a.seq_off[b];
  const int sp = a.sent_ptr[b];
  const int n_sent = a.sent_ptr[b + 1] - sp - 1;
  const int32_t *off = a.sent_off + sp;

  __shared__ int s_cnt[256];
  __shared__ int s_base;
  __shared__ int s_bad;
  if (tid == 0) s_bad = 0;
  __syncthreads();

  if (n_sent > SKIPKV_MAX_SENTENCES || n_sent < 0) {
    if (tid == 0) {
      if (a.dev_status) atomicOr(a.dev_status, SKIPKV_DEV_TOO_MANY_SENT);
      a.ws.chunk_base[b] = 0;
      a.ws.chunk_cnt[b] = 0;
      a.ws.rb_base[b] = 0;
      a.ws.rb_cnt[b] = 0;
    }
    return;
  }

  // validation: o[0] = 0, o[S] = N, strictly ascending
  int bad = 0;
  for (int s = tid; s < n_sent; s += 256) bad |= (off[s + 1] <= off[s]);
  if (tid == 0) bad |= (off[0] != 0) | (off[n_sent] != n_tok) | (n_sent == 0 && n_tok != 0);
  if (bad) s_bad = 1;

  // each thread owns up to 16 consecutive sentences
  const int per = (n_sent + 255) / 256;
  const int lo = tid * per, hi = min(lo + per, n_sent);
  auto begins = [&](int s) -> bool {
    const int w = off[s] / kChunkWindow;
    if (s == 0 || off[s - 1] / kChunkWindow != w) return true;
    int first = s - 1;
    while (first > 0 && off[first - 1] / kChunkWindow == w) --first;
    return ((s - first) % kChunkMaxSent) == 0;
  };
  int cnt = 0;
  for (int s = lo; s < hi; ++s) cnt += begins(s);
  s_cnt[tid] = cnt;
  __syncthreads();
  if (tid == 0) {
    int run = 0;
    for (int i = 0; i < 256; ++i) {
      const int c = s_cnt[i];
      s_cnt[i] = run;
      run += c;
    }
    const int nrb = (n_sent + kRowBlock - 1) / kRowBlock;
    const bool ok = !s_bad;
    const int nchunks = ok ? run : 0;
    s_base = atomicAdd(&a.ws.hdr->n_chunks, nchunks);
    a.ws.chunk_base[b] = s_base;
    a.ws.chunk_cnt[b] = nchunks;
    const int rb0 = atomicAdd(&a.ws.hdr->n_rowblocks, ok ? nrb : 0);
    a.ws.rb_base[b] = rb0;
    a.ws.rb_cnt[b] = ok ? nrb : 0;
    for (int i = 0; ok && i < nrb; ++i) a.ws.rowblocks[rb0 + i] = RowBlock{b, i * kRowBlock};
    if (!ok && a.dev_status) atomicOr(a.dev_status, SKIPKV_DEV_BAD_OFFSETS);
  }
  __syncthreads();
  if (s_bad) return;
  int idx = s_base + s_cnt[tid];
  for (int s = lo; s < hi; ++s) {
    if (!begins(s)) continue;
    int e = s + 1;
    while (e < n_sent && !begins(e)) ++e;
    a.ws.chunks[idx++] = Chunk{b, s, e, 0};
  }
}

hipError_t launch_plan(const PlanArgs &a, hipStream_t st) {
  hipLaunchKernelGGL(k_plan_reset, dim3(1), dim3(64), 0, st, a.ws.hdr);
  if (a.batch > 0) hipLaunchKernelGGL(k_plan, dim3(a.batch), dim3(256), 0, st, a);
  return hipGetLastError();
}

}  // namespace skipkv

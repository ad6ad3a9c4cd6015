// Work decomposition for one compression step: cuts every sequence's sentence list into
// chunks (units of the key scan) and row blocks (units of the redundancy kernel), checks the
// sentence offsets, and decides per sequence which scan variant handles it.  Shared by all
// layers and heads of the batch, so it is tiny.
#include "common.h"

#include <algorithm>

namespace skipkv {

__global__ void k_plan_reset(PlanHeader *hdr) {
  if (threadIdx.x == 0) {
    hdr->ranges = 0;
    hdr->n_unfused = 0;
    hdr->abort = 0;
  }
}

// End (exclusive sentence index) of the run of whole sentences that starts at sentence `start` and
// holds at most `cap` tokens and `max_sent` sentences: the largest e in (start, start + max_sent]
// with off[e] - off[start] <= cap, at least start + 1.
__device__ __forceinline__ int run_end(const int *off, int start, int n_sent, int cap, int max_sent) {
  int lo = start + 1, hi = min(n_sent, start + max_sent);
  const int limit = off[start] + cap;
  while (lo < hi) {  // invariant: the answer lies in [lo, hi]
    const int mid = (lo + hi + 1) >> 1;
    if (off[mid] <= limit) lo = mid; else hi = mid - 1;
  }
  return lo;
}

// One block per sequence.  Chunks (two-pass scan) and spans (single-pass scan) are packed greedily:
// the longest run of whole sentences within the unit's token and sentence limits; a sentence longer
// than the token limit is a unit of its own (a span like that sends its sequence to the two-pass scan).
__global__ void __launch_bounds__(256) k_plan(PlanArgs a) {
  const int b = blockIdx.x;
  const int tid = threadIdx.x;
  const int tok0 = a.seq_off[b];
  const int n_tok = seq_tokens(a.seq_off, a.len, b);
  const int sp = a.sent_ptr[b];
  const int n_sent = seq_sentences(a.sent_ptr, a.cnt, b);
  const int32_t *off = a.sent_off + sp;

  __shared__ int s_off[SKIPKV_MAX_SENTENCES + 1];
  __shared__ int s_bad;
  if (tid == 0) s_bad = 0;
  __syncthreads();

  bool reject = n_sent > SKIPKV_MAX_SENTENCES || n_sent < 0;
  // explicit lengths and counts must fit the room that the CSR arrays describe
  const bool overflow = !reject && (n_tok < 0 || n_tok > a.seq_off[b + 1] - tok0 || n_sent > a.sent_ptr[b + 1] - sp - 1);
  if (overflow) {
    if (tid == 0) s_bad = 1;
  } else if (!reject) {
    // validation: o[0] = 0, o[S] = N, strictly ascending
    int bad = 0;
    for (int s = tid; s <= n_sent; s += 256) {
      const int o = off[s];
      s_off[s] = o;
      if (s < n_sent) bad |= (off[s + 1] <= o);
    }
    if (tid == 0) bad |= (off[0] != 0) | (off[n_sent] != n_tok) | (n_sent == 0 && n_tok != 0);
    if (bad) s_bad = 1;
  }
  __syncthreads();
  __shared__ int s_base, s_nchunks, s_ibase, s_nspans, s_fused;
  static_assert(SKIPKV_MAX_SENTENCES <= 65535, "sentence indices are kept in 16 bits here");
  __shared__ uint16_t s_next[SKIPKV_MAX_SENTENCES];    // end of the chunk that would start at each sentence
  __shared__ uint16_t s_first[SKIPKV_MAX_SENTENCES];   // first sentence of every chunk
  __shared__ uint16_t s_snext[SKIPKV_MAX_SENTENCES];   // the same for spans
  __shared__ uint16_t s_sfirst[SKIPKV_MAX_SENTENCES + 1];
  const bool ok = !reject && !s_bad;
  for (int lh = tid; lh < a.n_lh; lh += 256) a.ws.head_redo[(int64_t)lh * a.batch + b] = 0;
  // the greedy packing is a walk along s -> chunk_end(s); the ends are found for all sentences at
  // once, so that the (serial) walk is one LDS read per chunk
  if (ok)
    for (int s = tid; s < n_sent; s += 256) {
      s_next[s] = (uint16_t)run_end(s_off, s, n_sent, kChunkCap, kChunkMaxSent);
      s_snext[s] = (uint16_t)run_end(s_off, s, n_sent, kSpanCap, kSpanMaxSent);
    }
  __syncthreads();
  if (tid == 0) {
    s_nchunks = -1;
    if (!ok) {
      if (a.dev_status) atomicOr(a.dev_status, reject ? SKIPKV_DEV_TOO_MANY_SENT : SKIPKV_DEV_BAD_OFFSETS);
      a.ws.chunk_base[b] = 0;
      a.ws.chunk_cnt[b] = 0;
      a.ws.rb_base[b] = 0;
      a.ws.rb_cnt[b] = 0;
      a.ws.seq_fused[b] = 1;  // nothing to scan either way
    } else {
      int n_chunks = 0, longest = 0;
      for (int start = 0; start < n_sent;) {
        const int e = s_next[start];
        longest = max(longest, s_off[e] - s_off[start]);
        s_first[n_chunks++] = (uint16_t)start;
        start = e;
      }
      int n_spans = 0, longest_span = 0;
      for (int start = 0; start < n_sent;) {
        const int e = s_snext[start];
        longest_span = max(longest_span, s_off[e] - s_off[start]);
        s_sfirst[n_spans++] = (uint16_t)start;
        start = e;
      }
      s_sfirst[n_spans] = (uint16_t)n_sent;
      // one atomic draws the block's ranges of chunks, items and row blocks
      const int n_items = (n_spans + kItemSpans - 1) / kItemSpans;
      const int nrb = (n_sent + kRowBlock - 1) / kRowBlock;
      const unsigned long long old = atomicAdd(&a.ws.hdr->ranges, (unsigned long long)n_chunks | ((unsigned long long)n_items << kHdrItemShift) |
                                                                      ((unsigned long long)nrb << kHdrRbShift));
      const int base = hdr_chunks(old), ibase = hdr_items(old), rb0 = hdr_rowblocks(old);
      a.ws.chunk_base[b] = base;
      a.ws.chunk_cnt[b] = n_chunks;
      (void)longest;
      const bool fused = longest_span <= kSpanCap && n_items <= kFuseMaxItems;
      a.ws.seq_fused[b] = fused;
      if (!fused && n_chunks > 0) atomicAdd(&a.ws.hdr->n_unfused, 1);
      a.ws.rb_base[b] = rb0;
      a.ws.rb_cnt[b] = nrb;
      for (int i = 0; i < nrb; ++i) a.ws.rowblocks[rb0 + i] = RowBlock{b, i * kRowBlock};
      s_base = base;
      s_nchunks = n_chunks;
      s_ibase = ibase;
      s_nspans = n_spans;
      s_fused = fused;
    }
  }
  __syncthreads();
  if (s_nchunks < 0) return;
  const int base = s_base, n_chunks = s_nchunks, n_spans = s_nspans, n_items = (n_spans + kItemSpans - 1) / kItemSpans;
  for (int j = tid; j < n_chunks; j += 256) {  // one record per chunk
    const int s0 = s_first[j], e = s_next[s0];
    a.ws.chunks[base + j] = Chunk{b, s0, e - s0, s_off[s0], s_off[e] - s_off[s0], sp + s0, tok0, n_tok};
  }
  for (int j = tid; j < n_items; j += 256) {  // one record per item: up to kItemSpans consecutive spans
    const int nsp = min(kItemSpans, n_spans - kItemSpans * j);
    int32_t *r = a.ws.item_rec + (int64_t)(s_ibase + j) * kItemRecInts;
    const int s0 = s_sfirst[kItemSpans * j];
    r[kIrB] = b;
    r[kIrNsp] = s_fused ? nsp : 0;
    r[kIrRec] = s_ibase + j;
    r[kIrTok0] = tok0;
    r[kIrNTok] = n_tok;
    r[kIrNItems] = n_items;
    r[kIrFirst] = s_ibase;
    r[kIrSoffIdx] = sp + s0;
    uint32_t ns = 0;
    for (int w = 0; w <= kItemSpans; ++w) {
      const int sw = s_sfirst[kItemSpans * j + min(w, nsp)];
      r[kIrT0 + w] = s_off[sw];
      if (w < nsp) ns |= (uint32_t)(s_sfirst[kItemSpans * j + w + 1] - sw) << (8 * w);
    }
    r[kIrNs] = (int32_t)ns;
  }
}

// Marks the statistics records of all items of this step as "not written yet": the single-pass
// scan polls them.  The number of items is only known on the device, so the grid covers the
// capacity and the surplus exits.  grid = (x, LH); one thread writes two rows of a record at a time.
__global__ void __launch_bounds__(256) k_plan_preset(Workspace ws) {
  const int64_t n16 = (int64_t)hdr_items(ws.hdr->ranges) * ws.rows / 2;  // 16-byte pieces per head
  uint4 *dst = reinterpret_cast<uint4 *>(ws.item_stat + (int64_t)blockIdx.y * ws.ni_max * ws.rows);
  for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < n16; i += (int64_t)gridDim.x * 256)
    dst[i] = make_uint4(kRowNormUnset, 0u, kRowNormUnset, 0u);
}

hipError_t launch_plan(const PlanArgs &a, hipStream_t st) {
  hipLaunchKernelGGL(k_plan_reset, dim3(1), dim3(64), 0, st, a.ws.hdr);
  if (a.batch > 0) {
    hipLaunchKernelGGL(k_plan, dim3(a.batch), dim3(256), 0, st, a);
    const int64_t cap16 = (int64_t)a.ws.ni_max * a.ws.rows / 2;
    const int gx = (int)std::min<int64_t>((cap16 + 255) / 256, std::max(32, 8192 / std::max(1, a.n_lh)));  // ~8192 workgroups in all
    if (a.n_lh > 0 && cap16 > 0) hipLaunchKernelGGL(k_plan_preset, dim3(gx, a.n_lh), dim3(256), 0, st, a.ws);
  }
  return hipGetLastError();
}

}  // namespace skipkv

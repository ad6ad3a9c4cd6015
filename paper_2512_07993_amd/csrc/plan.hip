// Work decomposition for one compression step: cuts every sequence's sentence list into
// chunks (units of the key scan) and row blocks (units of the redundancy kernel), checks the
// sentence offsets, and decides per sequence which scan variant handles it.  Shared by all
// layers and heads of the batch, so it is tiny.
#include "common.h"

#include <algorithm>

namespace skipkv {

__global__ void k_plan_reset(PlanHeader *hdr, int32_t *flags, int n_flags, uint32_t *row_norm_bits, int n_norm) {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i == 0) {
    hdr->ranges = 0;
    hdr->n_unfused = 0;
    hdr->abort = 0;
  }
  for (int j = i; j < n_flags; j += gridDim.x * blockDim.x) flags[j] = 0;
  for (int j = i; j < n_norm; j += gridDim.x * blockDim.x) row_norm_bits[j] = kRowNormUnset;
}

// End (exclusive sentence index) of the chunk that starts at sentence `start`: the largest e in
// (start, start + kChunkMaxSent] with off[e] - off[start] <= kChunkCap, at least start + 1.
__device__ __forceinline__ int chunk_end(const int *off, int start, int n_sent) {
  int lo = start + 1, hi = min(n_sent, start + kChunkMaxSent);
  const int limit = off[start] + kChunkCap;
  while (lo < hi) {  // invariant: the answer lies in [lo, hi]
    const int mid = (lo + hi + 1) >> 1;
    if (off[mid] <= limit) lo = mid; else hi = mid - 1;
  }
  return lo;
}

// One block per sequence.  Chunks are packed greedily: a chunk is the longest run of whole
// sentences with at most kChunkCap tokens and kChunkMaxSent sentences (a sentence longer than
// kChunkCap is a chunk of its own, and sends its sequence to the two-pass scan).
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
  __shared__ int s_base, s_nchunks, s_pbase, s_fused;
  static_assert(SKIPKV_MAX_SENTENCES <= 65535, "sentence indices are kept in 16 bits here");
  __shared__ uint16_t s_next[SKIPKV_MAX_SENTENCES];    // end of the chunk that would start at each sentence
  __shared__ uint16_t s_first[SKIPKV_MAX_SENTENCES];   // first sentence of every chunk
  const bool ok = !reject && !s_bad;
  // the greedy packing is a walk along s -> chunk_end(s); the ends are found for all sentences at
  // once, so that the (serial) walk is one LDS read per chunk
  if (ok)
    for (int s = tid; s < n_sent; s += 256) s_next[s] = (uint16_t)chunk_end(s_off, s, n_sent);
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
      a.ws.pair_cnt[b] = 0;
    } else {
      int n_chunks = 0, longest = 0;
      for (int start = 0; start < n_sent;) {
        const int e = s_next[start];
        longest = max(longest, s_off[e] - s_off[start]);
        s_first[n_chunks++] = (uint16_t)start;
        start = e;
      }
      // one atomic draws the block's ranges of chunks, pairs and row blocks
      const int n_pairs = (n_chunks + 1) / 2;
      const int nrb = (n_sent + kRowBlock - 1) / kRowBlock;
      const unsigned long long old = atomicAdd(&a.ws.hdr->ranges, (unsigned long long)n_chunks | ((unsigned long long)n_pairs << kHdrPairShift) |
                                                                      ((unsigned long long)nrb << kHdrRbShift));
      const int base = hdr_chunks(old), pbase = hdr_pairs(old), rb0 = hdr_rowblocks(old);
      a.ws.chunk_base[b] = base;
      a.ws.chunk_cnt[b] = n_chunks;
      const bool fused = longest <= kChunkCap && n_chunks <= kFuseMaxChunks;
      a.ws.seq_fused[b] = fused;
      if (!fused && n_chunks > 0) atomicAdd(&a.ws.hdr->n_unfused, 1);
      // the single-pass scan works on pairs of consecutive chunks of a sequence
      a.ws.pair_cnt[b] = n_pairs;
      a.ws.rb_base[b] = rb0;
      a.ws.rb_cnt[b] = nrb;
      for (int i = 0; i < nrb; ++i) a.ws.rowblocks[rb0 + i] = RowBlock{b, i * kRowBlock};
      s_base = base;
      s_nchunks = n_chunks;
      s_pbase = pbase;
      s_fused = fused;
    }
  }
  __syncthreads();
  if (s_nchunks < 0) return;
  const int base = s_base, n_chunks = s_nchunks, n_pairs = (n_chunks + 1) / 2;
  for (int j = tid; j < n_chunks; j += 256) {  // one record per chunk
    const int s0 = s_first[j], e = s_next[s0];
    a.ws.chunks[base + j] = Chunk{b, s0, e - s0, s_off[s0], s_off[e] - s_off[s0], sp + s0, tok0, n_tok};
  }
  for (int j = tid; j < n_pairs; j += 256) {  // one record per pair
    const int s0 = s_first[2 * j], e0 = s_next[s0];
    const bool two = 2 * j + 1 < n_chunks;
    const int e1 = two ? s_next[e0] : e0;
    int32_t *r = a.ws.pair_rec + (int64_t)(s_pbase + j) * kPairRecInts;
    r[kPrB] = b;
    r[kPrNch] = s_fused ? (two ? 2 : 1) : 0;
    r[kPrC0] = base + 2 * j;
    r[kPrTok0] = tok0;
    r[kPrNTok] = n_tok;
    r[kPrTBegin] = s_off[s0];
    r[kPrLen0] = s_off[e0] - s_off[s0];
    r[kPrNs0] = e0 - s0;
    r[kPrSoffIdx] = sp + s0;
    r[kPrLen1] = s_off[e1] - s_off[e0];
    r[kPrNs1] = e1 - e0;
    r[kPrNPairs] = n_pairs;
    r[kPrCFirst] = base;
  }
}

// Marks the statistics records of all chunks of this step as "not written yet": the single-pass
// scan polls them.  The number of chunks is only known on the device, so the grid covers the
// capacity and the surplus exits.  grid = (x, LH); one thread writes two rows of a record at a time.
__global__ void __launch_bounds__(256) k_plan_preset(Workspace ws) {
  const int64_t n16 = (int64_t)hdr_chunks(ws.hdr->ranges) * ws.rows / 2;  // 16-byte pieces per head
  uint4 *dst = reinterpret_cast<uint4 *>(ws.stat_part + (int64_t)blockIdx.y * ws.nc_max * ws.rows);
  for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < n16; i += (int64_t)gridDim.x * 256)
    dst[i] = make_uint4(kRowNormUnset, 0u, kRowNormUnset, 0u);
}

hipError_t launch_plan(const PlanArgs &a, hipStream_t st) {
  const int n_flags = a.n_lh * a.batch;  // arrive counters
  hipLaunchKernelGGL(k_plan_reset, dim3(64), dim3(256), 0, st, a.ws.hdr, a.ws.arrive, n_flags,
                     reinterpret_cast<uint32_t *>(a.ws.row_norm), a.n_lh * a.batch * a.ws.rows);
  if (a.batch > 0) {
    hipLaunchKernelGGL(k_plan, dim3(a.batch), dim3(256), 0, st, a);
    const int64_t cap16 = (int64_t)a.ws.nc_max * a.ws.rows / 2;
    const int gx = (int)std::min<int64_t>((cap16 + 255) / 256, std::max(32, 8192 / std::max(1, a.n_lh)));  // ~8192 workgroups in all
    if (a.n_lh > 0 && cap16 > 0) hipLaunchKernelGGL(k_plan_preset, dim3(gx, a.n_lh), dim3(256), 0, st, a.ws);
  }
  return hipGetLastError();
}

}  // namespace skipkv

// In-place compaction of K and V (Alg. 1, eviction line): row k of every head becomes the
// row kept_idx[k] it had before.  Pure byte movement.
//
// Because kept_idx is strictly ascending, kept_idx[k] >= k: a row is only ever moved towards
// the front.  One wave owns one (head, K-or-V) stream and walks it front to back in tiles; all
// loads of a tile are complete before its first store, and everything a later tile reads lies
// behind everything already written, so no row is overwritten before it has been read.  The
// leading rows with kept_idx[k] == k are not touched at all.
#include "common.h"

namespace skipkv {

namespace {

template <int ROWB>
__global__ void __launch_bounds__(256) k_compact(CompactArgs a) {
  constexpr int PPR = ROWB / 16;   // 16-byte pieces per row
  constexpr int RPI = 64 / PPR;    // rows moved by one wave-wide instruction
  constexpr int U = 8;             // instructions in flight per tile
  constexpr int ESZ = ROWB / kD;
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int64_t sid = (int64_t)blockIdx.x * 4 + wave;
  const int64_t n_lhb = (int64_t)a.n_layers * a.n_kv_heads * a.batch;
  if (sid >= 2 * n_lhb) return;
  const int64_t lhb = sid >> 1;
  const int b = (int)(lhb % a.batch);
  const int lh = (int)(lhb / a.batch), l = lh / a.n_kv_heads, h = lh % a.n_kv_heads;
  char *base = static_cast<char *>((sid & 1) ? a.v : a.k) +
               ((int64_t)l * a.stride_layer + (int64_t)h * a.stride_head + (int64_t)a.seq_off[b] * a.stride_tok) * ESZ;
  const int64_t pitch = a.stride_tok * ESZ;
  const int32_t *kept = a.kept_idx + lhb * a.kept_stride;
  const int nl = a.new_len[lhb];

  // first row that actually moves
  int first = nl;
  for (int k0 = 0; k0 < nl; k0 += 64) {
    const int k = k0 + lane;
    const unsigned long long moved = __ballot(k < nl && kept[k] != k);
    if (moved) {
      first = k0 + __ffsll((long long)moved) - 1;
      break;
    }
  }

  const int sub = lane / PPR, piece = lane % PPR;
  for (int k0 = first; k0 < nl; k0 += U * RPI) {
    uint4 regs[U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int k = k0 + u * RPI + sub;
      if (k < nl) regs[u] = *reinterpret_cast<const uint4 *>(base + (int64_t)kept[k] * pitch + piece * 16);
    }
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");  // every load of the tile has landed before any store is issued
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int k = k0 + u * RPI + sub;
      if (k < nl) *reinterpret_cast<uint4 *>(base + (int64_t)k * pitch + piece * 16) = regs[u];
    }
  }
}

}  // namespace

hipError_t launch_compact(const CompactArgs &a, hipStream_t st) {
  const int64_t streams = 2LL * a.n_layers * a.n_kv_heads * a.batch;
  if (streams == 0) return hipSuccess;
  const unsigned grid = (unsigned)((streams + 3) / 4);
  if (a.dtype == SKIPKV_BF16)
    hipLaunchKernelGGL(k_compact<256>, dim3(grid), dim3(256), 0, st, a);
  else
    hipLaunchKernelGGL(k_compact<512>, dim3(grid), dim3(256), 0, st, a);
  return hipGetLastError();
}

}  // namespace skipkv

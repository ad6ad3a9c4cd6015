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

// Paged cache (PAGED): rows live in block slots.  Sources come pre-translated (src_rows: slot row of
// kept_idx[k], written by k_kept_rows below), destinations are read from the row map one coalesced
// load per tile, issued right before the tile's row loads.  Logical positions still only move
// forward and distinct logical rows are distinct slots, so the order argument above holds.
template <int ROWB, bool PAGED>
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
  if (PAGED && a.seq_bad[b]) return;  // invalid block table: leave the sequence alone
  const int lh = (int)(lhb / a.batch), l = lh / a.n_kv_heads, h = lh % a.n_kv_heads;
  char *base = static_cast<char *>((sid & 1) ? a.v : a.k) +
               ((int64_t)l * a.stride_layer + (int64_t)h * a.stride_head + (PAGED ? 0 : (int64_t)a.seq_off[b] * a.stride_tok)) * ESZ;
  const int64_t pitch = (PAGED ? a.map_stride : a.stride_tok) * ESZ;  // paged: rows are addressed in units of the row map
  const int32_t *kept = a.kept_idx + lhb * a.kept_stride;
  const int32_t *srcs = PAGED ? a.src_rows + lhb * a.src_stride : kept;  // what the row loads are addressed with
  const int32_t *rmap = PAGED ? a.row_map + a.seq_off[b] : nullptr;
  const int nl = a.new_len[lhb];
  // A head that kept everything because its inputs could not be trusted reports its full length,
  // which its row of indices may not even hold: nothing to move, and nothing to read past the row.
  if (nl > a.kept_stride || (PAGED && nl > a.src_stride)) return;
  const int room = a.seq_off[b + 1] - a.seq_off[b];  // contiguous cache: a source index is a row of the sequence

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

  // Software pipeline, two tiles deep.  Tile i's loads may be issued before tile i-1's stores
  // (a tile only reads rows at or behind its own first row, a tile's stores only write rows of
  // that tile), so the wave always has one tile of loads and one tile of stores in flight; the
  // only ordering kept is that a tile's own loads have landed before its stores.  Vector memory
  // operations complete in issue order, which lets a counted wait express exactly that.  The
  // tile's source indices come in with one coalesced load, a tile ahead of their use.
  const int sub = lane / PPR, piece = lane % PPR;
  constexpr int TR = U * RPI;  // rows per tile
  static_assert(TR <= 64, "one lane per row index of a tile");
  auto load_idx = [&](int k0) -> int {  // unconditional (clamped), so that it always counts as one outstanding load
    const int i = srcs[min(k0 + lane, nl - 1)];
    return PAGED ? i : max(0, min(i, room - 1));  // never address a row outside the sequence, whatever the indices say
  };
  auto load_dst = [&](int k0) -> int {  // paged: slot rows of the tile's destinations (same rule)
    return PAGED ? rmap[min(k0 + lane, nl - 1)] : 0;
  };
  if (first >= nl) return;
  // The two tiles are written out as named registers (A0..A7, B0..B7): arrays carried around the
  // loop end up in scratch memory with this compiler.
  static_assert(U == 8, "the tiles below are spelled out for 8 instructions");
#define SKIPKV_EACH(X, T) X(T, 0) X(T, 1) X(T, 2) X(T, 3) X(T, 4) X(T, 5) X(T, 6) X(T, 7)
#define SKIPKV_DECL(T, u) uint4 T##u;
  // always U loads per tile: rows past the end re-read the last kept row (index loads are clamped)
#define SKIPKV_LOAD(T, u) \
  T##u = *reinterpret_cast<const uint4 *>(base + (int64_t)__shfl(idx_##T, u * RPI + sub) * pitch + piece * 16);
  // destination row of the lane's piece: position in the sequence, or (paged) its slot row; the shuffle
  // is taken by all lanes, outside any condition
#define SKIPKV_DROW(T, u) const int64_t dr_##u = PAGED ? (int64_t)__shfl(dst_##T, u * RPI + sub) : (int64_t)(ks + u * RPI + sub);
#define SKIPKV_STORE(T, u) *reinterpret_cast<uint4 *>(base + dr_##u * pitch + piece * 16) = T##u;
#define SKIPKV_STORE_TAIL(T, u) \
  if (ks + u * RPI + sub < nl) *reinterpret_cast<uint4 *>(base + dr_##u * pitch + piece * 16) = T##u;
#define SKIPKV_STORE_TILE(T, K0)        \
  {                                     \
    const int ks = (K0);                \
    SKIPKV_EACH(SKIPKV_DROW, T)         \
    if (ks + TR <= nl) {                \
      SKIPKV_EACH(SKIPKV_STORE, T)      \
    } else {                            \
      SKIPKV_EACH(SKIPKV_STORE_TAIL, T) \
    }                                   \
  }
  // Wait until the loads of the tile about to be stored have landed.  Behind them in the queue
  // are the previous tile's U stores (none for the first tile), one index load and the next
  // tile's U loads (paged: plus the load of the next tile's destination rows, NX = 1).  The next tile is always loaded, also past the end (clamped, one tile of
  // wasted reads per stream): unconditional loads keep the counts exact and the registers in place.
  SKIPKV_EACH(SKIPKV_DECL, A)
  SKIPKV_EACH(SKIPKV_DECL, B)
  constexpr int NX = PAGED ? 1 : 0;
  int idx_A = load_idx(first);
  int idx_B = load_idx(first + TR);
  int dst_A = load_dst(first), dst_B = 0;
  SKIPKV_EACH(SKIPKV_LOAD, A)
  for (int k0 = first;; k0 += 2 * TR) {
    idx_A = load_idx(k0 + 2 * TR);
    dst_B = load_dst(k0 + TR);
    SKIPKV_EACH(SKIPKV_LOAD, B)
    if (k0 != first)
      asm volatile("s_waitcnt vmcnt(%0)" ::"n"(2 * U + 1 + NX) : "memory");
    else
      asm volatile("s_waitcnt vmcnt(%0)" ::"n"(U + 1 + NX) : "memory");
    SKIPKV_STORE_TILE(A, k0)
    if (k0 + TR >= nl) break;
    idx_B = load_idx(k0 + 3 * TR);
    dst_A = load_dst(k0 + 2 * TR);
    SKIPKV_EACH(SKIPKV_LOAD, A)
    asm volatile("s_waitcnt vmcnt(%0)" ::"n"(2 * U + 1 + NX) : "memory");
    SKIPKV_STORE_TILE(B, k0 + TR)
    if (k0 + 2 * TR >= nl) break;
  }
#undef SKIPKV_EACH
#undef SKIPKV_DECL
#undef SKIPKV_LOAD
#undef SKIPKV_STORE
#undef SKIPKV_DROW
#undef SKIPKV_STORE_TAIL
#undef SKIPKV_STORE_TILE
}

// Paged cache: src_rows[head, k] = slot row of the head's kept token k, for k < new_len (one wave
// per head; shared by the K and the V stream of the head).
__global__ void __launch_bounds__(256) k_kept_rows(CompactArgs a) {
  const int64_t lhb = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
  if (lhb >= (int64_t)a.n_layers * a.n_kv_heads * a.batch) return;
  const int b = (int)(lhb % a.batch), lane = threadIdx.x & 63;
  if (a.seq_bad[b]) return;
  const int32_t *kept = a.kept_idx + lhb * a.kept_stride;
  const int32_t *rmap = a.row_map + a.seq_off[b];
  int32_t *out = a.src_rows + lhb * a.src_stride;
  const int nl = min(min(a.new_len[lhb], a.src_stride), a.kept_stride);
  const int room = a.seq_off[b + 1] - a.seq_off[b];
  for (int k = lane; k < nl; k += 64) out[k] = rmap[max(0, min(kept[k], room - 1))];
}

}  // namespace

hipError_t launch_compact(const CompactArgs &a, hipStream_t st) {
  const int64_t heads = (int64_t)a.n_layers * a.n_kv_heads * a.batch, streams = 2 * heads;
  if (streams == 0) return hipSuccess;
  const unsigned grid = (unsigned)((streams + 3) / 4);
  if (a.row_map) {
    hipLaunchKernelGGL(k_kept_rows, dim3((unsigned)((heads + 3) / 4)), dim3(256), 0, st, a);
    if (a.dtype == SKIPKV_BF16)
      hipLaunchKernelGGL((k_compact<256, true>), dim3(grid), dim3(256), 0, st, a);
    else
      hipLaunchKernelGGL((k_compact<512, true>), dim3(grid), dim3(256), 0, st, a);
    return hipGetLastError();
  }
  if (a.dtype == SKIPKV_BF16)
    hipLaunchKernelGGL((k_compact<256, false>), dim3(grid), dim3(256), 0, st, a);
  else
    hipLaunchKernelGGL((k_compact<512, false>), dim3(grid), dim3(256), 0, st, a);
  return hipGetLastError();
}

}  // namespace skipkv

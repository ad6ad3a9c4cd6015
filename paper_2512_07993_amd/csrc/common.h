// Shared definitions of the libskipkv kernels (gfx950, wave64).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "skipkv.h"

namespace skipkv {

constexpr int kD = SKIPKV_HEAD_DIM;  // head dimension
constexpr int kChunkCap = 256;       // a chunk of scan work = a maximal run of whole sentences of at most this many tokens
constexpr int kChunkMaxSent = 32;    // ... and at most this many sentences (a single longer sentence is a chunk of its own)
// Units of the single-pass scan (scan_fused.hip): a span is a maximal run of whole sentences of at most
// kSpanCap tokens and kSpanMaxSent sentences, the share of ONE wave; an item is up to kItemSpans
// consecutive spans of one sequence, the share of one workgroup.  A sequence with a sentence longer than
// kSpanCap tokens, or with more than kFuseMaxItems items, takes the two-pass scan.
constexpr int kSpanCap = 128;
constexpr int kSpanMaxSent = 16;
constexpr int kItemSpans = 4;
constexpr int kItemMaxSent = kItemSpans * kSpanMaxSent;
constexpr int kFuseMaxItems = 256;
constexpr uint32_t kRowNormUnset = 0xFFFFFFFFu;  // bit pattern no computed normaliser has (a NaN with full payload)
constexpr float kRefInit = -3.0e38f;  // "no key seen yet" softmax reference, finite so that -inf - ref stays -inf
constexpr int kRowBlock = 128;       // sentences per row block of the redundancy kernel

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(4 * sizeof(float)))) float f32x4;

// One unit of scan work: sentences [s0, s0 + ns) of sequence b, tokens [t_begin, t_begin + len)
// relative to the sequence.  Carries what a kernel needs to start without further lookups.
struct Chunk {
  int32_t b, s0, ns, t_begin, len;
  int32_t soff_idx;  // index into sent_off of the chunk's first offset
  int32_t tok0;      // packed index of the sequence's first token
  int32_t n_tok;     // length of the sequence
};
// One unit of redundancy work: rows [r0, r0 + kRowBlock) of sequence b.
struct RowBlock {
  int32_t b, r0;
};

// Record of one work item of the single-pass scan, written by the plan so that a workgroup learns
// everything about an item from one 64-byte read.
constexpr int kItemRecInts = 16;
enum ItemRec : int {
  kIrB = 0,        // sequence
  kIrNsp,          // spans in the item: 1..kItemSpans; 0 = the sequence takes the two-pass scan
  kIrRec,          // index of the item (its statistics record is filed there)
  kIrTok0,         // first token of the sequence in the packed cache
  kIrNTok,         // tokens of the sequence
  kIrNItems,       // items of the sequence
  kIrFirst,        // index of the sequence's first item
  kIrSoffIdx,      // index of the item's first sentence offset in sent_off
  kIrT0,           // kIrT0 + w: first token of span w, relative to the sequence; kIrT0 + nsp: end of the item
  kIrNs = kIrT0 + kItemSpans + 1,  // sentences of the four spans, one byte each
};
static_assert(kIrNs < kItemRecInts && kSpanMaxSent < 256, "the record holds the spans' bounds and sentence counts");

// Device scalars at the head of the workspace.

struct PlanHeader {
  // The three range counters that every plan block draws from, packed into one word so that a
  // block needs ONE atomic (with thousands of blocks the same-address atomics are what the plan
  // costs): chunks (units of the two-pass scan) in bits 0..21, items (units of the single-pass scan)
  // in bits 22..42, row blocks in bits 43..63.
  unsigned long long ranges;
  int32_t n_unfused;  // number of sequences that take the two-pass scan
  int32_t abort;      // set by the first cross-workgroup wait of the single-pass scan that runs out: every later wait gives up at once
  int32_t pad[60];
};
constexpr int kHdrItemShift = 22, kHdrRbShift = 43;
constexpr int64_t kHdrMaxChunks = (1ll << 22) - 1, kHdrMaxItems = (1ll << 21) - 1, kHdrMaxRowBlocks = (1ll << 21) - 1;
__host__ __device__ inline int32_t hdr_chunks(unsigned long long r) { return (int32_t)(r & ((1ull << kHdrItemShift) - 1)); }
__host__ __device__ inline int32_t hdr_items(unsigned long long r) { return (int32_t)((r >> kHdrItemShift) & ((1ull << (kHdrRbShift - kHdrItemShift)) - 1)); }
__host__ __device__ inline int32_t hdr_rowblocks(unsigned long long r) { return (int32_t)(r >> kHdrRbShift); }

// Carved-up view of the caller's workspace.  All sections 256-byte aligned.
struct Workspace {
  PlanHeader *hdr;
  int32_t *chunk_base;   // [B] first chunk of each sequence (ranges are handed out by an atomic counter)
  int32_t *chunk_cnt;    // [B] number of chunks of each sequence
  int32_t *rb_base;      // [B] first row block of each sequence
  int32_t *rb_cnt;       // [B]
  int32_t *seq_fused;    // [B] 1: the sequence goes through the single-pass scan
  int32_t *head_redo;    // [LH, B] 1: a wait of the single-pass scan ran out for this head: the two-pass scan does it again
  int32_t *item_rec;     // [ni_max][kItemRecInts] one record per item of the single-pass scan (ItemRec)
  Chunk *chunks;         // [nc_max]
  RowBlock *rowblocks;   // [nrb_max]
  float2 *stat_part;     // [LH, nc_max, R]  two-pass scan: per-chunk (max, sum) of every query row, log2 domain
  float2 *item_stat;     // [LH, ni_max, R]  single-pass scan: per-item (reference, sum) of every query row; the plan presets .x of the used records to kRowNormUnset
  float *row_norm;       // [LH, B, R]       two-pass scan: log2 of the softmax normaliser of every query row
  uint16_t *vhat_hi;     // [LH, S_total, 128] bf16 high part of the unit sentence embedding
  uint16_t *vhat_lo;     // [LH, S_total, 128] bf16 low part (residual)
  float *sent_imp;       // [LH, S_total]    mean token importance over the candidate span
  float *sent_red;       // [LH, S_total]    mean token redundancy over the candidate span
  int32_t nc_max, ni_max, nrb_max, rows;  // rows = R, padded query rows per head
  bool fits;                      // the counts fit the packed range counters of the plan header
  size_t bytes;
};

// How the n*alpha query rows of a head are laid over MFMA row tiles.
// Lane group g = lane/16 of a 16x16 tile owns output rows 4g..4g+3 of every row tile; we give
// it the window queries a = g, g+4, g+8, ... and, for each, the NP (>= n) heads of the group,
// so that the max over the group's heads is a max over registers of one lane.
struct RowLayout {
  int np;    // padded group size
  int al;    // window queries per lane group = ceil(alpha / 4)
  int nt;    // row tiles of 16 rows
  int rows;  // nt * 16
};

inline bool make_row_layout(int n, int alpha, RowLayout *out) {
  // the scan kernels are instantiated for NP in {4, 8} x AL in {2, 4, 8}, plus the exact
  // shapes (NP, AL) = (5, 8) and (7, 2) of the two Qwen-distill configurations
  int al = alpha <= 8 ? 2 : (alpha <= 16 ? 4 : 8);
  int np = n <= 4 ? 4 : ((n == 5 && al == 8) ? 5 : ((n == 7 && al == 2) ? 7 : 8));
  if (n < 1 || n > SKIPKV_MAX_GROUP || alpha < 1 || alpha > SKIPKV_MAX_OBS_WINDOW) return false;
  out->np = np;
  out->al = al;
  out->nt = (np * al + 3) / 4;
  out->rows = out->nt * 16;
  return true;
}

struct Profile;  // api.hip

// ---- kernel launchers (one per .hip file) -------------------------------------------------
// Eq. 10 on per-head ranges: n_new[b] tokens are appended to sequence b of every head; bnd_off
// (CSR over sequences, bnd_ptr) lists the positions inside the appended run at which a new
// sentence starts.
struct RangesAppendArgs {
  int32_t n_lh, batch, total_sentences;
  const int32_t *seq_off, *sent_ptr;  // capacities
  int32_t *len, *cnt, *off;           // [n_lh, batch], [n_lh, batch], [n_lh, total_sentences + batch], updated in place
  const int32_t *n_new, *bnd_ptr, *bnd_off;
  int32_t *dev_status;
};
hipError_t launch_ranges_append(const RangesAppendArgs &a, hipStream_t st);
// Sentence numbers of per-head ranges (layout [n_lh, total_sentences], sentence s of (lh, b) at column
// sent_ptr[b] - b + s).  select: numbers of the sentences that survive a sentence-level selection, in
// order: those with keep != 0 and those that reach into the protected window (their tail stays, so the
// sentence stays); the ranges are those the selection ran on (len / cnt / off null: the shared ones);
// id_in null: a sentence's number is its position; may run in place.  append: sentences
// old_cnt .. new_cnt-1 continue the numbering after the head's last old sentence.
struct RangesIdsArgs {
  int32_t n_lh, batch, total_sentences, protect;
  const int32_t *seq_off, *sent_ptr, *sent_off;  // shared structure (capacities)
  const int32_t *len, *old_cnt, *off;            // per head: [n_lh, batch], [n_lh, batch], [n_lh, total_sentences + batch]
  const int32_t *new_cnt;                        // append only
  const uint8_t *keep;                           // select only
  const int32_t *id_in;
  int32_t *id_out;
};
hipError_t launch_ranges_ids_select(const RangesIdsArgs &a, hipStream_t st);
hipError_t launch_ranges_ids_append(const RangesIdsArgs &a, hipStream_t st);
hipError_t launch_virtual_layout(const int32_t *seq_off, const int32_t *sent_ptr, int32_t batch, int32_t n_lh, int32_t total_tokens,
                                 int32_t total_sentences, int32_t *v_seq_off, int32_t *v_sent_ptr, hipStream_t st);

// Length and sentence count of sequence b: explicit where given, else from the CSR arrays.
__device__ __forceinline__ int seq_tokens(const int32_t *seq_off, const int32_t *len, int b) {
  return len ? len[b] : seq_off[b + 1] - seq_off[b];
}
__device__ __forceinline__ int seq_sentences(const int32_t *sent_ptr, const int32_t *cnt, int b) {
  return cnt ? cnt[b] : sent_ptr[b + 1] - sent_ptr[b] - 1;
}

struct PlanArgs {
  const int32_t *seq_off, *sent_ptr, *sent_off;
  int32_t batch, n_lh;
  Workspace ws;
  int32_t *dev_status;
  const int32_t *len, *cnt;  // nullable [batch]: explicit lengths and sentence counts (then seq_off / sent_ptr only give capacities)
};
hipError_t launch_plan(const PlanArgs &a, hipStream_t st);

struct ScanArgs {
  const void *k;
  const void *q;
  int64_t stride_layer, stride_head, stride_tok;
  int32_t dtype, n_layers, n_kv_heads, n_q_heads, batch, total_tokens, total_sentences;
  int32_t alpha, protect;
  const int32_t *seq_off, *sent_ptr, *sent_off;
  const float *tok_red;  // nullable
  float *tok_imp;        // nullable
  Workspace ws;
  RowLayout rl;
  int32_t force_two_pass;  // debugging aid: send every sequence through the two-pass scan
  int32_t spin_limit;      // bound on the polls of a cross-workgroup wait in the single-pass scan
  int32_t *dev_status;
  // Per-head ranges: every (layer, KV head, sequence) triple is presented to the kernels as a
  // sequence of its own of ONE layer with ONE KV head (v = (l * H_k + h) * B + b); only the query
  // rows are still laid out by the real (l, b, h).  virt_hk = real H_k (0: off), virt_b = real B.
  int32_t virt_hk, virt_b;
  int32_t no_pool;  // 1: sentence embeddings are not needed (lambda comes from elsewhere): skip the key pooling
  // Paged cache: row_map[seq_off[b] + t] = slot row of logical token t, in units of map_stride elements
  // from the head's base (consecutive slots of a block are still stride_tok apart); null for a
  // contiguous cache.
  const int32_t *row_map;
  int32_t page_size;   // token slots per block of a paged cache (the single-pass scan needs a power of two >= 16)
  int64_t map_stride;  // stride_tok, or one head row when every (layer, head) has a map of its own
};
bool scan_fused_supported(const RowLayout &rl, int64_t row_pitch_bytes);
hipError_t launch_scan_fused(const ScanArgs &a, hipStream_t st);    // single pass over K (sequences the plan marked fused)
int scan_two_pass_rows(const RowLayout &rl, int dtype);  // rows of the statistics arrays that the two-pass scan of this shape needs (>= rl.rows)
hipError_t launch_scan_stats(const ScanArgs &a, hipStream_t st);    // pass A: row statistics + sentence embeddings
hipError_t launch_row_norm(const ScanArgs &a, hipStream_t st);      // combine the per-chunk statistics
hipError_t launch_scan_scores(const ScanArgs &a, hipStream_t st);   // pass B: token importance, sentence means

struct CosineArgs {
  int32_t n_lh, batch, total_sentences, protect;
  float sigma, tau;
  bool has_red;
  const int32_t *seq_off, *sent_ptr, *sent_off;
  Workspace ws;
  float *sent_score, *sent_lambda;
  const int32_t *len, *cnt;  // nullable, see PlanArgs
};
hipError_t launch_cosine(const CosineArgs &a, hipStream_t st);

struct SelectArgs {
  int32_t n_lh, batch, total_sentences, protect, budget_scalar, kept_stride;
  const int32_t *budget;
  const int32_t *seq_off, *sent_ptr, *sent_off;
  const float *sent_score;
  uint8_t *sent_keep;
  int32_t *kept_idx, *new_len, *new_sent_off, *new_sent_cnt;
  int32_t *dev_status;
  const int32_t *len, *cnt;  // nullable, see PlanArgs
};
hipError_t launch_select(const SelectArgs &a, hipStream_t st);

struct TokSelectArgs {
  int32_t n_lh, batch, total_tokens, total_sentences, protect, budget_scalar, kept_stride;
  float sigma, tau;
  const int32_t *budget;
  const int32_t *seq_off, *sent_ptr, *sent_off;
  const float *tok_imp, *tok_red, *sent_lambda;
  float *tok_score;
  uint8_t *tok_keep;
  int32_t *kept_idx, *new_len, *new_sent_off, *new_sent_cnt;
  int32_t *dev_status;
  const int32_t *len, *cnt;  // per-head ranges (virtual view): tokens and sentences of every sequence; null: from the offsets
};
hipError_t launch_select_tokens(const TokSelectArgs &a, hipStream_t st);

struct CompactArgs {
  void *k, *v;
  int64_t stride_layer, stride_head, stride_tok;
  int32_t dtype, n_layers, n_kv_heads, batch, kept_stride;
  const int32_t *seq_off, *kept_idx, *new_len;
  const int32_t *row_map;  // paged cache: logical token -> slot row (see ScanArgs); null: contiguous
  const int32_t *seq_bad;  // paged cache, [batch]: nonzero = invalid block table, leave the sequence alone
  int32_t *src_rows;       // paged cache, workspace [heads, src_stride]: slot row of every kept token
  int32_t src_stride;      // >= every new_len
  int64_t map_stride;      // paged cache: elements per unit of the row map (stride_tok unless the map is per head)
};
hipError_t launch_compact(const CompactArgs &a, hipStream_t st);

// Paged cache: for every logical token the row of its slot, in units of the map's row pitch:
//   row_map[lh * total_tokens + seq_off[b] + t] = l * unit_layer + h * unit_head
//       + block_table[b][t / block_size] * unit_block + (t % block_size) * unit_tok.
// One map serves all heads when the unit is the token pitch (n_lh = 1, unit_layer = unit_head = 0,
// unit_tok = 1); with per-head ranges every (layer, head) gets its own map in units of one head row.
// Block ids outside [0, n_blocks) are flagged (dev_status, seq_bad[lh * batch + b]) and read as 0.
struct RowMapArgs {
  const int32_t *seq_off, *block_table;
  int32_t batch, table_stride, block_size, n_blocks;
  int32_t n_lh, n_kv_heads, total_tokens;
  int64_t unit_layer, unit_head, unit_block, unit_tok;
  int32_t *row_map, *seq_bad, *dev_status;
};
hipError_t launch_row_map(const RowMapArgs &a, hipStream_t st);

constexpr int kTokredRows = 256;  // key rows per workgroup of the token-redundancy sweeps

struct TokRedArgs {
  const void *k;
  int64_t stride_layer, stride_head, stride_tok;
  int32_t dtype, n_layers, n_kv_heads, batch, total_tokens;
  int32_t nrb_max;           // upper bound on the kTokredRows-row blocks of all sequences
  const int32_t *seq_off;
  float *scale;              // [LH, T] workspace: sqrt(log2 e) / (||k|| + eps)
  float *inv_l;              // [LH, T] workspace: 1 / row sums
  unsigned long long *acc;   // [LH, T] workspace: fixed-point totals of the sweep that is running
  float *out;                // [LH, T] token redundancy
  const int32_t *row_map;    // paged cache: logical token -> slot row in units of stride_tok (see ScanArgs); null: contiguous
  const int32_t *len;        // per-head ranges, [LH, batch]: tokens of every head's sequence (within its room); null: from seq_off
};
hipError_t launch_token_redundancy(const TokRedArgs &a, hipStream_t st);

// Sentence similarity from hidden states (Eq. 1-3 as printed), shared by all layers and heads.
struct HiddenSimArgs {
  int32_t batch, total_sentences, d_model, dtype;
  const int32_t *seq_off, *sent_ptr, *sent_off;
  const void *hidden;    // [total_tokens, d_model]
  float *sum_scratch;    // [total_sentences, d_model]
  uint16_t *vhat_hi, *vhat_lo;  // [total_sentences, d_model] unit embeddings, bf16 high part and residual
  float *sent_lambda;    // out [total_sentences]
};
hipError_t launch_hidden_similarity(const HiddenSimArgs &a, hipStream_t st);

// Eq. 6 with a lambda that is given per sequence instead of computed per head.
struct FuseSharedArgs {
  int32_t n_lh, batch, total_sentences, protect;
  float sigma, tau;
  bool has_red;
  const int32_t *seq_off, *sent_ptr, *sent_off;
  const float *sent_imp, *sent_red, *shared_lambda;
  float *sent_score, *sent_lambda;  // sent_lambda nullable
  // Per-head ranges (virtual view, sequence v = lh * virt_b + b): tokens and sentences of every head, and
  // the number each of its sentences has in the sequence's own list: lambda of sentence s of v is
  // shared_lambda[lam_ptr[b] + sent_id[column of s]].  All null / 0 for shared ranges.
  const int32_t *len, *cnt, *sent_id, *lam_ptr;
  int32_t virt_b;
  int32_t *dev_status;
};
hipError_t launch_fuse_shared(const FuseSharedArgs &a, hipStream_t st);

struct SteerArgs {
  void *hidden;
  const void *vec;
  const float *coef;
  float coef_scalar;
  const uint8_t *row_mask;
  int32_t rows, d_model, dtype;
};
hipError_t launch_steer(const SteerArgs &a, hipStream_t st);
hipError_t launch_steer_strength(const int32_t *n_nonexec, float alpha0, float gamma, float *coef, int32_t rows, hipStream_t st);

// ---- device helpers -----------------------------------------------------------------------
#if defined(__HIPCC__)
__device__ __forceinline__ float bf16_bits_to_f32(uint32_t b) { return __uint_as_float(b << 16); }

// fp32 -> bf16 bits, round to nearest even (finite inputs).
__device__ __forceinline__ uint32_t f32_to_bf16_bits(float f) {
  uint32_t u = __float_as_uint(f);
  u += 0x7FFFu + ((u >> 16) & 1u);
  return u >> 16;
}

// Rotate within each row of 16 lanes by N lanes (DPP row_ror).
template <int N>
__device__ __forceinline__ float row_ror(float v) {
  return __builtin_amdgcn_update_dpp(0.f, v, 0x120 + N, 0xf, 0xf, false);
}
// All 16 lanes of a row end up with the sum / max over the row.
__device__ __forceinline__ float row16_sum(float v) {
  v += row_ror<8>(v);
  v += row_ror<4>(v);
  v += row_ror<2>(v);
  v += row_ror<1>(v);
  return v;
}
__device__ __forceinline__ float row16_max(float v) {
  v = fmaxf(v, row_ror<8>(v));
  v = fmaxf(v, row_ror<4>(v));
  v = fmaxf(v, row_ror<2>(v));
  v = fmaxf(v, row_ror<1>(v));
  return v;
}
__device__ __forceinline__ float wave_sum(float v) {
  v = row16_sum(v);
  v += __shfl_xor(v, 16);
  v += __shfl_xor(v, 32);
  return v;
}

// Blocks are dealt round-robin to the 8 XCDs, each with its own L2.  Remap the block index so
// that every XCD works on one contiguous range of work items (neighbouring items share the
// head's queries and sentence offsets).
__device__ __forceinline__ uint32_t xcd_contiguous_item(uint32_t block, uint32_t n_blocks) {
  const uint32_t per = (n_blocks + 7u) / 8u;
  return (block % 8u) * per + block / 8u;
}
#endif

}  // namespace skipkv

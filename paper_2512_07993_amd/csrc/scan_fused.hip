// Single-pass key scan (Sec. 4.1 "Token Importance Score", Eq. 4; sentence embedding of Eq. 2
// over the head's keys): K is read from HBM exactly once.
//
// The softmax normaliser of a query row needs all N keys of the head, which are spread over many
// workgroups.  Instead of a second pass over K, every workgroup keeps the logits of its share in
// registers (they are MFMA accumulators anyway), publishes one (reference, sum exp) record per
// query row over its share, merges the records of ALL shares of the head itself (loading them
// again while any still holds the marker that the plan preset it to), and then finishes I[t]
// from its registers.
//
// Work decomposition.  The plan cuts every sequence into SPANS: maximal runs of whole sentences of at
// most 128 tokens and 16 sentences.  A span is the share of ONE wave: 8 stages of 16 tokens, 128
// accumulator registers of logits, and - because no sentence crosses a span - a complete set of
// sentence key sums, so waves never exchange partial sentences.  An item is up to four consecutive
// spans of one sequence, the share of one workgroup; workgroup w of the persistent grid takes items
// w, w + G, ...  The four waves only meet at two barriers per item: statistics ready -> the
// head's normalisers ready.
//
// Per stage a wave issues, besides the loads, three blocks of work:
//   logits      16 v_mfma_f32_16x16x32_bf16 of the stage's key rows against the query tile in LDS;
//   statistics  one exponential per logit relative to ONE reference per lane group, fixed after the
//               span's first stage (its largest logit): no running maximum, no rescaling.  Should a
//               later logit outgrow the reference by more than the exponent range, or a row's sum
//               vanish against it, the wave recomputes its rows exactly from the logits it still
//               holds (the slow path below); results do not depend on which path ran beyond rounding;
//   key sums    [16 sentences x 16 tokens] 0/1 indicator times [16 tokens x 128 dims] keys on the
//               matrix cores (8 v_mfma_f32_16x16x16_bf16); the token-major operand comes straight
//               from the stage buffer with transposing LDS reads (ds_read_b64_tr_b16).  All sentences
//               of the span accumulate in 32 registers and are normalised and written together at
//               the end of the span, 16 bytes per lane, a sentence's 256 bytes contiguous.  The
//               embedding's dimensions are stored in a permuted order (position 8c + j holds dimension
//               16j + c); every embedding of a head uses the same order, so cosines are unaffected.
//
// Forward progress.  The grid is persistent and no larger than what is co-resident on the chip
// (occupancy query on the host): the launch must have the GPU's compute units to itself for the
// argument below to hold; other work on the GPU at the same time can only be waited out by the bound.
// A workgroup only ever waits for the head of the item it has just published.  A head has at most
// kFuseMaxItems <= G items, on distinct workgroups, each of which reaches its item of that head
// without waiting on that head first; by induction over heads in item order every wait ends.
// The wait is bounded anyway (spin_limit polls): on expiry SKIPKV_DEV_TIMEOUT is raised, every
// later wait of the launch gives up at once, the item's sentence means become NaN (the selection
// then keeps that head whole) and the kernel runs to completion.
//
// Data movement.  Rows go HBM -> LDS directly (global_load_lds, 16 bytes per lane, no staging
// registers) into a ring of NBUF stage buffers private to the wave, which keeps NBUF-1 stages in
// flight ahead of the one it is computing on - also across the end of an item.  A direct load
// writes LDS at base + lane*16, so rows are stored unpadded; bank conflicts are avoided by an XOR
// swizzle: the 16-byte piece p of row r is kept at piece position p ^ swz(r), which each lane
// arranges by choosing which global piece it fetches.  For 256-byte rows swz is a permutation of the
// bits of r & 15 under which the 16 lanes of a 16-byte-per-lane read that walk 16 consecutive rows
// run at about 225 bytes per cycle on this chip (measured), against about 135 with swz(r) = r & 15;
// the query tile uses the same arrangement.
//
// Paged cache.  With a row map (logical token -> block slot) and blocks of a power of two >= 16
// slots, a stage spans at most two blocks: two scalar reads of the map give two bases per stage.
#include "scan_dev.h"

#ifndef SKIPKV_FRAG_AHEAD
#define SKIPKV_FRAG_AHEAD 3  // query fragments are read this many matrix instructions ahead of their use
#endif
#ifndef SKIPKV_SCAN_NBUF
#define SKIPKV_SCAN_NBUF 2   // stage buffers per wave
#endif

namespace skipkv {

namespace {

constexpr int kStageRows = 16;                      // rows per pipeline stage = one MFMA sub-tile of tokens
constexpr int kSpanStages = kSpanCap / kStageRows;  // stages per span
constexpr int kMergeDepth = 8;                      // records a lane has in flight while merging

typedef __attribute__((__vector_size__(4 * sizeof(short)))) short i16x4;

struct Item {  // one item as seen by one wave
  uint32_t item;  // >= n_items: none
  int lh, b, nsp, rec, n_tok, tok0, np, first, soff_idx, ns_item;
  const char *kbase;
  int w0, w1, nst;  // the wave's span: token range (relative to the sequence) and number of stages
  int ns, sb;       // ... its sentences: count, and index of the first one among the item's sentences
};

// Swizzle of 256-byte rows (see "Data movement" above): bits (r0, r1, r2, r3) of the row number go to
// bits (1, 2, 0, 3) of the piece number.  A permutation of bits, hence linear over XOR:
// swz(a ^ b) = swz(a) ^ swz(b).
__host__ __device__ constexpr int swz16(int r) { return ((r & 3) << 1) | ((r >> 2) & 1) | (r & 8); }

// Transposing LDS read: the 16 lanes of a group hand in 16 addresses of 4 consecutive 16-bit
// elements each, read as a 4 x 16 matrix (lanes 4i .. 4i+3 hold row i); lane n gets column n.
__device__ __forceinline__ i16x4 lds_read_tr16(uint32_t addr) {
  return __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) i16x4 *)(uintptr_t)addr);
}

// A uniform 64-bit address as a scalar register pair (the compiler may hold it in vector registers).
__device__ __forceinline__ uint64_t scalar64(const void *p_) {
  const uint64_t p = (uint64_t)(uintptr_t)p_;
  return ((uint64_t)(uint32_t)__builtin_amdgcn_readfirstlane((int)(p >> 32)) << 32) | (uint32_t)__builtin_amdgcn_readfirstlane((int)p);
}
// Direct HBM -> LDS load with a scalar base and a 32-bit offset per lane.
__device__ __forceinline__ void load_to_lds_16_sbase(uint64_t sbase, uint32_t voff, void *wave_lds_base) {
  const uint32_t l = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) char *)wave_lds_base;
  asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2" ::"s"(l), "v"(voff), "s"(sbase) : "memory");
}

template <int DT, int NP, int AL>
__global__ void __launch_bounds__(256, (DT == SKIPKV_BF16 ? 2 : 1)) k_scan_fused(ScanArgs a) {
  constexpr int SL = NP * AL;
  constexpr int NT = (SL + 3) / 4;
  constexpr int SLP = 4 * NT;
  constexpr int R = 16 * NT;
  constexpr int SUBS = kSpanStages;
  constexpr int LSTR = Tr<DT>::LSTR, ROWB = Tr<DT>::ROWB, ESZ = Tr<DT>::ESZ;
  constexpr int PPR = ROWB / 16;                      // 16-byte pieces per row
  constexpr int GL = kStageRows * PPR / 64;           // direct loads per stage
  constexpr int RPL = 64 / PPR;                       // rows covered by one direct load
  constexpr int NBUF = SKIPKV_SCAN_NBUF;
  constexpr int STAGEB = kStageRows * ROWB;
  // bf16 keys are pooled with an indicator whose ones are written as 2.0 (a single bit, cheap to
  // build from a row mask): all key sums of that path carry this factor, which the normalisation
  // to a unit vector removes.
  constexpr float kPoolScale = (DT == SKIPKV_BF16) ? 2.f : 1.f;
  constexpr int QSTR = (DT == SKIPKV_BF16) ? ROWB : LSTR;  // row pitch of the query tile: swizzled (bf16) or padded (fp32)
  auto swz = [](int r) { return DT == SKIPKV_BF16 ? swz16(r) : (r & 15); };
  static_assert(R <= 64, "one wave merges the head's records, one lane per query row");

  __shared__ __align__(256) char kt[4][NBUF][STAGEB];  // 256-byte aligned: the row swizzle is applied as an XOR on address bits
  __shared__ __align__(256) char qt[R * QSTR];
  __shared__ int soff_buf[2][kItemMaxSent + 2];  // [item parity]: offsets of the item's sentences
  __shared__ float wstat[4][R][2];               // (reference, sum) of every row over each wave's span
  __shared__ float mstat[4][R][2];               // (reference, sum) of every row over each wave's quarter of the head's records
  __shared__ float imp[4][kSpanCap];             // token importance of each wave's span (private to the wave)
  __shared__ float row_norm_l[4][R];             // every wave's own copy of the head's normalisers
  __shared__ int s_timeout[2];  // [item parity] a wait of the item ran out: its sentences get NaN means

  const int tid = threadIdx.x, lane = tid & 63, c16 = lane & 15, g = lane >> 4;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);  // in a scalar register: everything derived from it is uniform control flow
  const int n_lh = a.n_layers * a.n_kv_heads;
  const int n_per_lh = hdr_items(a.ws.hdr->ranges);
  const uint32_t n_items = (uint32_t)n_lh * (uint32_t)n_per_lh;
  const int n = a.n_q_heads / a.n_kv_heads;
  const int64_t tok_pitch = a.stride_tok * ESZ;
  const float inv_alpha = 1.f / (float)a.alpha;
  if (a.force_two_pass) return;
  // The plan is constant while this kernel runs: reading it through the constant address space
  // lets the compiler use scalar loads, which do not queue behind the key loads in flight.
  typedef const __attribute__((address_space(4))) int32_t *ConstIntPtr;
  const ConstIntPtr item_rec_c = (ConstIntPtr)a.ws.item_rec;
  const ConstIntPtr row_map_c = (ConstIntPtr)a.row_map;  // written by an earlier kernel, constant here

  // ---- item descriptors: one 64-byte record per item, written by the plan ----------------------
  auto load_item = [&](uint32_t item) -> Item {  // first fused item at or after `item` in this workgroup's sequence
    Item it{};
    for (; item < n_items; item += gridDim.x) {
      const ConstIntPtr r = item_rec_c + (int64_t)(item % n_per_lh) * kItemRecInts;
      const int nsp = r[kIrNsp];
      if (nsp == 0) continue;  // the sequence takes the two-pass scan
      it.lh = item / n_per_lh;
      it.b = r[kIrB];
      it.nsp = nsp;
      it.rec = r[kIrRec];
      it.tok0 = r[kIrTok0];
      it.n_tok = r[kIrNTok];
      it.np = r[kIrNItems];
      it.first = r[kIrFirst];
      it.soff_idx = r[kIrSoffIdx];
      const uint32_t nsw = (uint32_t)r[kIrNs];
      it.ns_item = (int)((nsw & 0xFF) + ((nsw >> 8) & 0xFF) + ((nsw >> 16) & 0xFF) + (nsw >> 24));
      const uint32_t below = nsw & ((1u << (8 * wave)) - 1u);  // the spans before this wave's
      it.sb = (int)((below & 0xFF) + ((below >> 8) & 0xFF) + ((below >> 16) & 0xFF));
      it.ns = wave < nsp ? (int)((nsw >> (8 * wave)) & 0xFF) : 0;
      it.w0 = r[kIrT0 + min(wave, nsp)];
      it.w1 = r[kIrT0 + min(wave + 1, nsp)];
      it.nst = (it.w1 - it.w0 + kStageRows - 1) / kStageRows;
      const int l = it.lh / a.n_kv_heads, h = it.lh % a.n_kv_heads;
      // contiguous cache: first row of the sequence; paged cache: the head's base, rows come from the row map
      it.kbase = static_cast<const char *>(a.k) +
                 ((int64_t)l * a.stride_layer + (int64_t)h * a.stride_head + (a.row_map ? 0 : (int64_t)it.tok0 * a.stride_tok)) * ESZ;
      break;
    }
    it.item = item;
    return it;
  };
  // Queries of the group and the sentence offsets of an item, in two steps so that the global
  // latency can hide behind other work: fetch into registers, later commit to LDS (padded rows).
  constexpr int NQ = R * PPR / 256;  // 16-byte pieces of the query tile per thread
  struct QFetch {
    uint4 q[NQ];
    int so;
  };
  auto q_fetch = [&](const Item &it) -> QFetch {
    QFetch f;
    const int t = opaque(tid);
    f.so = 0;
    if (t <= it.ns_item) f.so = a.sent_off[it.soff_idx + t];
    const char *qbase = static_cast<const char *>(a.q);
    // layer, KV head and sequence that address the query rows (the real ones under per-head ranges)
    int l = it.lh / a.n_kv_heads, h = it.lh % a.n_kv_heads, qb = it.b, q_batch = a.batch, q_heads = a.n_q_heads;
    if (a.virt_hk > 0) {
      const int lh_r = it.b / a.virt_b;
      qb = it.b % a.virt_b;
      l = lh_r / a.virt_hk;
      h = lh_r % a.virt_hk;
      q_batch = a.virt_b;
      q_heads = a.virt_hk * n;
    }
#pragma unroll
    for (int u = 0; u < NQ; ++u) {
      const int r = u * (256 / PPR) + t / PPR, piece = t % PPR;
      const int slot = 4 * (r >> 4) + (r & 3), gq = (r >> 2) & 3;
      const int al = slot / NP, i = slot % NP, aq = gq + 4 * al;
      f.q[u] = make_uint4(0, 0, 0, 0);
      if (slot < SL && i < n && aq < a.alpha) {
        const int64_t row = (((int64_t)l * q_batch + qb) * q_heads + (h * n + i)) * a.alpha + aq;
        f.q[u] = *reinterpret_cast<const uint4 *>(qbase + row * ROWB + piece * 16);
      }
    }
    return f;
  };
  auto q_commit = [&](const Item &it, const QFetch &f, int par) {
    const int t = opaque(tid);
    if (t <= it.ns_item) soff_buf[par][t] = f.so;
#pragma unroll
    for (int u = 0; u < NQ; ++u) {
      const int r = u * (256 / PPR) + t / PPR, piece = t % PPR;
      *reinterpret_cast<uint4 *>(qt + r * QSTR + (DT == SKIPKV_BF16 ? (piece ^ swz16(r & 15)) : piece) * 16) = f.q[u];
    }
  };

  // ---- the wave's load stream: stages of consecutive items, NBUF-1 ahead of the compute --------
  // Direct load j of a stage brings rows j*RPL .. j*RPL+RPL-1: lane -> row j*RPL + lane/PPR, global piece
  // (lane % PPR) ^ swz(row).  j*RPL and lane/PPR occupy different bits of the row number and swz is linear, so
  // the lane's part is (lane/PPR) * pitch + (((lane % PPR) ^ swz(lane/PPR)) ^ swz(j*RPL)) * 16 and the rest
  // goes into the scalar base.  The lane's part is formed where it is used, from an opaque copy of
  // the lane id: kept in registers across an item it gets spilled, and a reload from scratch in the
  // stage loop would wait for every key load in flight.
  const uint32_t pitch32 = (uint32_t)tok_pitch;
  // The stage of 16 tokens from token `ts` of a span that ends at `w1` goes into ring slot `slot`
  // (kbase, tok0, n_tok: of the span's item).
  auto issue_stage = [&](const char *kbase, int ts, int w1, int tok0, int n_tok, uint32_t slot) {
    char *dst = kt[wave][slot % NBUF];
    const int last = w1 - 1 - ts;  // rows past the span re-read its last row (they only meet zero weights)
    if (a.row_map == nullptr) {
      // scalar 64-bit base of the stage + a 32-bit offset per lane (the launcher only takes this
      // kernel for row pitches below 2^24 bytes)
      const uint64_t sbase = scalar64(kbase + (int64_t)ts * tok_pitch);
      const uint32_t ln = (uint32_t)opaque(lane);
      const uint32_t vp0 = ((ln % PPR) ^ (uint32_t)swz((int)(ln / PPR))) << 4;
#pragma unroll
      for (int j = 0; j < GL; ++j) {
        const int row = j * RPL + (int)(ln / PPR);
        load_to_lds_16_sbase(sbase, __umul24((uint32_t)min(row, last), pitch32) + (vp0 ^ (uint32_t)(swz(j * RPL) << 4)), dst + j * 1024);
      }
    } else {
      // Paged cache, blocks of a power of two >= 16 slots: the stage's 16 tokens lie in at most two
      // blocks, in consecutive slots within each.  Two scalar reads of the row map give the slot
      // row of the stage's first token and of the first token of the next block.  Map entries count
      // units of map_stride elements (the token pitch, or one head row when every (layer, head) has a
      // map of its own); consecutive slots of a block are one token pitch apart either way.
      const int ln = opaque(lane);
      const int jb = a.page_size - (ts & (a.page_size - 1));  // rows of the stage before the next block begins (may be >= 16)
      const int r0 = row_map_c[tok0 + ts];
      const int r1 = row_map_c[tok0 + min(ts + jb, n_tok - 1)];
      const int64_t map_pitch = a.map_stride * ESZ;  // bytes per unit of the row map
      const char *base0 = kbase + (int64_t)r0 * map_pitch;
      const char *base1 = kbase + (int64_t)r1 * map_pitch - (int64_t)jb * tok_pitch;
#pragma unroll
      for (int j = 0; j < GL; ++j) {
        const int row = j * RPL + ln / PPR;
        const int piece = (ln % PPR) ^ swz(row);
        const int jr = min(row, last);
        const uint32_t off = __umul24((uint32_t)jr, pitch32) + (uint32_t)piece * 16u;
        load_to_lds_16((jr >= jb ? base1 : base0) + off, dst + j * 1024);
      }
    }
  };
  // A wait has run out when it has used up its polls, or when any wait of this launch did before
  // (looked up every 256 polls): the first time-out is reported and raises the launch's abort word.
  auto wait_expired = [&](int polls) -> bool {
    if (polls < a.spin_limit && ((polls & 255) != 255 || __hip_atomic_load(&a.ws.hdr->abort, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) == 0)) return false;
    if (lane == 0) {
      if (a.dev_status) atomicOr(a.dev_status, SKIPKV_DEV_TIMEOUT);
      __hip_atomic_store(&a.ws.hdr->abort, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
    return true;
  };

  Item cur = load_item(blockIdx.x);
  if (cur.item >= n_items) return;
  static_assert(NBUF == 2, "the load stream runs exactly one stage ahead of the compute");
  uint32_t ring = 0;   // ring slot of the stage to be computed next
  bool primed = false;  // that stage's loads are already in flight
  int par = 0;           // which soff buffer holds the current item's offsets
  q_commit(cur, q_fetch(cur), par);
  if (tid < 2) s_timeout[tid] = 0;
  lds_barrier();

  // per-lane constants of the LDS addressing (offsets inside a stage buffer)
  // key fragment of the logits: row c16, piece (4g + kk) ^ swz(c16) (the slice index kk is an XOR on bits 4..5);
  // the query fragments sit in the query tile in the same way
  const uint32_t b_off = c16 * ROWB + (((4 * g) ^ swz(c16)) << 4);
  // transposed key fragment of the pooling: row 4g + c16/4, elements 4 (c16 % 4) .. +3 of the 16 dimensions of
  // slice j, i.e. piece (2j + (c16 >> 1 & 1)) ^ swz(row), byte 8 (c16 & 1) in it (the slice index j is an XOR on bits 5..7)
  const int tr_row = 4 * g + (c16 >> 2);
  const uint32_t tr_off = tr_row * ROWB + (((((c16 >> 1) & 1) ^ swz(tr_row)) & 15) << 4) + ((c16 & 1) << 3);

  while (cur.item < n_items) {
    const int lh = cur.lh, b = cur.b;
    const int n_tok = cur.n_tok;
    const int last_free = n_tok - a.alpha;  // keys t <= last_free are visible to every window query
    const int *soff = soff_buf[par];
    const int w0 = cur.w0, w1 = cur.w1, ns = cur.ns;
    // The next item of this workgroup, known from the start: its first stage is prefetched behind this
    // item's last one, its queries and offsets are fetched at the end of the first phase.  After the
    // last item the descriptor is all zero (the fetch then reads valid memory that nobody uses).
    const Item nxt = load_item(cur.item + gridDim.x);
    if (cur.nst > 0 && !primed) issue_stage(cur.kbase, cur.w0, cur.w1, cur.tok0, cur.n_tok, ring);  // this wave had no span in the previous item

    f32x4 acc[SUBS][NT];
    f32x4 pool[8];      // key sums: register r of pool[j] = sentence 4g + r of the span, dimension 16j + c16
    float lsum[SLP];
    float ref1 = kRefInit;
#pragma unroll
    for (int q = 0; q < SLP; ++q) lsum[q] = 0.f;
#pragma unroll
    for (int j = 0; j < 8; ++j) pool[j] = f32x4{0.f, 0.f, 0.f, 0.f};
    // the lane's sentence of the span (slot c16): token range, empty for unused slots
    const int s_mine = cur.sb + min(c16, max(ns - 1, 0));
    const int s_lo = soff[s_mine];
    const int s_hi = c16 < ns ? soff[s_mine + 1] : s_lo;

    // =============== first phase: logits, row statistics and sentence key sums =================
#pragma unroll
    for (int st = 0; st < SUBS; ++st) {
#pragma unroll
      for (int T = 0; T < NT; ++T) acc[st][T] = f32x4{0.f, 0.f, 0.f, 0.f};
      if (st < cur.nst) {
        const int ts = w0 + st * kStageRows, te = min(ts + kStageRows, w1);
        // keep the load stream one stage ahead (into the next item behind this item's last stage),
        // then wait for this stage's rows to land
        const bool more = st + 1 < cur.nst;
        if (more || nxt.nst > 0) {
          issue_stage(more ? cur.kbase : nxt.kbase, more ? ts + kStageRows : nxt.w0, more ? w1 : nxt.w1, more ? cur.tok0 : nxt.tok0,
                      more ? n_tok : nxt.n_tok, ring + 1);
          wait_vm<GL>();
        } else {
          wait_all();
        }
        const char *stage = kt[wave][ring % NBUF];
        ++ring;
        const uint32_t stage_a = lds_addr(stage);

        // ---- operands of the sentence key sums, fetched first so that they land behind the logits block:
        // the indicator of the lane's sentence (slot c16) over the stage's 16 tokens as a bit mask
        // (tokens past the span belong to no sentence), and the transposed key fragments
        const int ra = min(max(s_lo - ts, 0), kStageRows), rb = min(max(s_hi - ts, 0), kStageRows);
        const uint32_t rows = (1u << rb) - (1u << ra);
        i16x4 trv[8];
        if constexpr (DT == SKIPKV_BF16) {
          if (!a.no_pool) {
            const uint32_t taddr = stage_a + tr_off;
#pragma unroll
            for (int j = 0; j < 8; ++j) trv[j] = lds_read_tr16(taddr ^ (j << 5));
          }
        }

        // ---- logits of this stage's 16 tokens against all query rows
        if constexpr (DT == SKIPKV_BF16) {
          // Fragment reads run AHEAD matrix instructions ahead of their use (the order is pinned:
          // the compiler would otherwise read each fragment right before its use and pay the LDS
          // latency every time, or read all of them first and run out of registers).
          // Step i multiplies slice i / NT of the head dimension into row tile i % NT.
          constexpr int AHEAD = SKIPKV_FRAG_AHEAD, NSTEP = 4 * NT;
          const uint32_t baddr = stage_a + b_off;
          const uint32_t aaddr = lds_addr(qt) + b_off;  // row 16 T + c16 of the query tile: same lane pattern as the key fragment
          auto rd_a = [&](int i) {
            return *reinterpret_cast<const __attribute__((address_space(3))) bf16x8 *>((uintptr_t)((aaddr ^ ((i / NT) << 4)) + 16 * (i % NT) * ROWB));
          };
          auto rd_b = [&](int kk) {
            return *reinterpret_cast<const __attribute__((address_space(3))) bf16x8 *>((uintptr_t)(baddr ^ (kk << 4)));
          };
          bf16x8 bfr[4], afr[NSTEP];
          bfr[0] = rd_b(0);
#pragma unroll
          for (int i = 0; i < AHEAD && i < NSTEP; ++i) afr[i] = rd_a(i);
          __builtin_amdgcn_sched_barrier(0);
#pragma unroll
          for (int i = 0; i < NSTEP; ++i) {
            if (i + AHEAD < NSTEP) afr[i + AHEAD] = rd_a(i + AHEAD);
            if (i % NT == 0 && i / NT + 1 < 4) bfr[i / NT + 1] = rd_b(i / NT + 1);
            __builtin_amdgcn_sched_barrier(0);
            acc[st][i % NT] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(afr[i], bfr[i / NT], acc[st][i % NT], 0, 0, 0);
            __builtin_amdgcn_sched_barrier(0);
          }
        } else {
#pragma unroll
          for (int cc = 0; cc < 8; ++cc) {
            const float4 bfrag = *reinterpret_cast<const float4 *>(stage + c16 * ROWB + (((4 * cc + g) ^ c16) * 16));
#pragma unroll
            for (int T = 0; T < NT; ++T) {
              const float4 afrag = *reinterpret_cast<const float4 *>(qt + (16 * T + c16) * LSTR + cc * 64 + g * 16);
              acc[st][T] = __builtin_amdgcn_mfma_f32_16x16x4f32(afrag.x, bfrag.x, acc[st][T], 0, 0, 0);
              acc[st][T] = __builtin_amdgcn_mfma_f32_16x16x4f32(afrag.y, bfrag.y, acc[st][T], 0, 0, 0);
              acc[st][T] = __builtin_amdgcn_mfma_f32_16x16x4f32(afrag.z, bfrag.z, acc[st][T], 0, 0, 0);
              acc[st][T] = __builtin_amdgcn_mfma_f32_16x16x4f32(afrag.w, bfrag.w, acc[st][T], 0, 0, 0);
            }
          }
        }

        // ---- sentence key sums over the stage's tokens (they keep the matrix cores busy while the
        // logits drain into the statistics below)
        if (!a.no_pool) {
          if constexpr (DT == SKIPKV_BF16) {
            // the lane's operand: tokens 4g .. 4g+3 as bf16 values 2.0 (= bit 14 alone) or 0; row bits
            // 4g, 4g+1 go to bits 14 and 30 of the first word, 4g+2, 4g+3 of the second one
            const uint32_t x = rows >> (4 * g);
            const uint2 ind = make_uint2(((x << 14) | (x << 29)) & 0x40004000u, ((x << 12) | (x << 27)) & 0x40004000u);
            const i16x4 av = __builtin_bit_cast(i16x4, ind);
#pragma unroll
            for (int j = 0; j < 8; ++j) pool[j] = __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(av, trv[j], pool[j], 0, 0, 0);
          } else {
            // fp32 keys: 16x16x4 products, token 4 ks + g against dimension 16 j + c16
#pragma unroll
            for (int ks = 0; ks < 4; ++ks) {
              const int row = 4 * ks + g;
              const float av = ((rows >> row) & 1u) ? 1.f : 0.f;
              const uint32_t raddr = stage_a + row * ROWB + (c16 & 3) * 4;
#pragma unroll
              for (int j = 0; j < 8; ++j) {
                const float bv = lds_read_f32(raddr + ((((4 * j + (c16 >> 2)) ^ row) & 31) << 4));
                pool[j] = __builtin_amdgcn_mfma_f32_16x16x4f32(av, bv, pool[j], 0, 0, 0);
              }
            }
          }
        }
        __builtin_amdgcn_sched_barrier(0);

        // ---- softmax statistics of every query row (accumulators stay unscaled)
        {
          const int t = ts + c16;
          const bool edge = (ts + 15 >= te) || (ts + 15 > last_free);
          if (edge) {
#pragma unroll
            for (int q = 0; q < SLP; ++q) {
              const int aq = g + 4 * (q / NP);
              if (!(t < te && t <= last_free + aq)) acc[st][q >> 2][q & 3] = -INFINITY;
            }
          }
          if (st == 0) {
            // the reference of the lane group's rows for the whole span: the largest logit of the first stage
            float mx = acc[0][0][0];
#pragma unroll
            for (int q = 1; q < SLP; ++q) mx = fmaxf(mx, acc[0][q >> 2][q & 3]);
            ref1 = fmaxf(row16_max_fast(mx) * kScale2, kRefInit);
          }
          // all arguments, then all exponentials, then all sums: independent instructions back to back
          float e[SLP];
#pragma unroll
          for (int q = 0; q < SLP; ++q) e[q] = fmaf(acc[st][q >> 2][q & 3], kScale2, -ref1);
          __builtin_amdgcn_sched_barrier(0);
#pragma unroll
          for (int q = 0; q < SLP; ++q) e[q] = __builtin_amdgcn_exp2f(e[q]);
          __builtin_amdgcn_sched_barrier(0);
#pragma unroll
          for (int q = 0; q < SLP; ++q) lsum[q] += e[q];
        }
      }
    }

    // ---- the span's row statistics: (reference, sum) per row, exact if the fast path is in doubt
    {
      float tot[SLP];
      bool doubt = false;
      // From here until the head's records are folded the wave runs at raised priority: what it does now is
      // what the other workgroups of its head wait for, while the other wave of the SIMD is mostly in its first phase.
      __builtin_amdgcn_s_setprio(3);
#pragma unroll
      for (int q = 0; q < SLP; ++q) tot[q] = lsum[q];
#pragma unroll
      for (int q = 0; q < SLP; ++q) tot[q] = row16_sum_fast(tot[q]);
#pragma unroll
      for (int q = 0; q < SLP; ++q) {
        const bool used = q < SL && (q % NP) < n && (g + 4 * (q / NP)) < a.alpha;  // padding rows hold zero queries: whatever they sum to is never used
        doubt = doubt || (used && !(tot[q] > 1e-30f && tot[q] < 3e38f));  // also catches NaN and infinity
      }
      float refq[SLP];
#pragma unroll
      for (int q = 0; q < SLP; ++q) refq[q] = ref1;
      if (cur.nst > 0 && __any(doubt)) {
        // slow path (a logit far above the first stage's, a row far below its group's, rows that see
        // no key of the span): every row gets its own reference, its true maximum over the span
#pragma unroll
        for (int q = 0; q < SLP; ++q) {
          float m = -INFINITY;
#pragma unroll
          for (int st = 0; st < SUBS; ++st)
            if (st < cur.nst) m = fmaxf(m, acc[st][q >> 2][q & 3]);
          m = fmaxf(row16_max_fast(m) * kScale2, kRefInit);
          float s = 0.f;
#pragma unroll
          for (int st = 0; st < SUBS; ++st)
            if (st < cur.nst) s += __builtin_amdgcn_exp2f(fmaf(acc[st][q >> 2][q & 3], kScale2, -m));
          tot[q] = row16_sum_fast(s);
          refq[q] = m;
        }
      }
      if (c16 == 0) {
#pragma unroll
        for (int q = 0; q < SLP; ++q) {
          const int r = 16 * (q >> 2) + 4 * g + (q & 3);
          wstat[wave][r][0] = cur.nst > 0 ? refq[q] : kRefInit;
          wstat[wave][r][1] = cur.nst > 0 ? tot[q] : 0.f;
        }
      }
    }
    primed = cur.nst > 0 && nxt.nst > 0;
    // the next item's queries and offsets: fetched now, committed before the second barrier below
    const QFetch nq = q_fetch(nxt);
    lds_barrier();  // B1: every wave is done with the query tile and has left its statistics

    // ---- publish the item's row statistics: one (reference, sum) record per row, lane = query row.
    // The last wave does it: items with fewer than four spans leave it idle first.
    if (wave == 3 && lane < R) {
      if (lane == 0) s_timeout[par ^ 1] = 0;  // the other item's flag: read for the last time before the barrier above
      float m = kRefInit;
#pragma unroll
      for (int w = 0; w < 4; ++w) m = fmaxf(m, wstat[w][lane][0]);
      float s = 0.f;
#pragma unroll
      for (int w = 0; w < 4; ++w) s += wstat[w][lane][1] * __builtin_amdgcn_exp2f(wstat[w][lane][0] - m);
      coherent_store2(&a.ws.item_stat[((int64_t)lh * a.ws.ni_max + cur.rec) * R + lane], make_float2(m, s));
    }
    // ---- the head's normalisers, first half: every wave loads a quarter of the records of the head's items
    // (wave w: items w, w + 4, ...; lane = query row), kMergeDepth coherent loads in flight per lane, and
    // lets them travel while it commits the next item's queries and writes its embeddings.
    // (The queries are committed first: they arrived long ago, and a wait for them placed behind the
    // record loads would wait for those as well.  Always kMergeDepth loads, surplus ones on the head's last
    // record, so that the number of loads in flight is known where later code waits for older ones.)
    q_commit(nxt, nq, par ^ 1);
    const int np = cur.np;
    const float2 *recs = a.ws.item_stat + ((int64_t)lh * a.ws.ni_max + cur.first) * R + min(opaque(lane), R - 1);
    float2 pv[kMergeDepth];
    auto load_records = [&](int pp) {
#pragma unroll
      for (int u = 0; u < kMergeDepth; ++u) pv[u] = coherent_load2(recs + (int64_t)min(pp + 4 * u, np - 1) * R);
    };
    load_records(wave);

    // ---- sentence embeddings of the span: unit vectors as bf16 hi + lo, four sentences at a time
    if (!a.no_pool && ns > 0) {
      // (addresses are formed here, from an opaque copy: formed early they are spilled, and a reload from
      // scratch waits for every load in flight, the record loads above included)
      const int64_t col0 = (int64_t)lh * a.total_sentences + opaque(cur.soff_idx - b + cur.sb);
      const int g4 = 4 * opaque(g);
      float ssq[4] = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
      for (int j = 0; j < 8; ++j)
#pragma unroll
        for (int r = 0; r < 4; ++r) ssq[r] = fmaf(pool[j][r], pool[j][r], ssq[r]);
#pragma unroll
      for (int r = 0; r < 4; ++r) ssq[r] = row16_sum_fast(ssq[r]);  // the 16 lanes of the group hold a sentence's 128 dimensions
#pragma unroll
      for (int r = 0; r < 4; ++r) {
        if (r == 2) load_records(wave);  // a second look, timed to land when the embeddings are out
        const float ss = ssq[r];
        const int slot = g4 + r, sl = cur.sb + min(slot, ns - 1);
        const int len = soff[sl + 1] - soff[sl];
        // mean / (|mean| + eps) = sum / (|sum| + eps * len): no division by the length.  1-ulp
        // reciprocal and square root: a common scale error of ~1e-7 on the unit vector
        // (bf16 keys: the sums arrive scaled by kPoolScale, and so does the epsilon)
        const float inv = __builtin_amdgcn_rcpf(__builtin_amdgcn_sqrtf(ss) + (1e-12f * kPoolScale) * (float)len);
        uint32_t hi[4], lo[4];
#pragma unroll
        for (int j = 0; j < 4; ++j) {
          const float u0 = pool[2 * j][r] * inv, u1 = pool[2 * j + 1][r] * inv;
          hi[j] = pack_bf16x2(u0, u1);  // round to nearest even, both halves in one instruction
          lo[j] = pack_bf16x2(u0 - __uint_as_float(hi[j] << 16), u1 - __uint_as_float(hi[j] & 0xFFFF0000u));
        }
        if (slot < ns) {
          const int64_t o = (col0 + slot) * (kD / 8) + opaque(c16);  // in 16-byte units
          reinterpret_cast<uint4 *>(a.ws.vhat_hi)[o] = make_uint4(hi[0], hi[1], hi[2], hi[3]);
          reinterpret_cast<uint4 *>(a.ws.vhat_lo)[o] = make_uint4(lo[0], lo[1], lo[2], lo[3]);
        }
      }
    }

    // ---- the head's normalisers, second half: fold the quarter's records.  A record that has not been
    // written yet still holds the plan's marker: load again.
    {
      float m = kRefInit, s = 0.f;
      for (int pp = wave; pp < np; pp += 4 * kMergeDepth) {
        if (pp != wave) load_records(pp);
        for (int polls = 0;; ++polls) {
          bool ok = true;
#pragma unroll
          for (int u = 0; u < kMergeDepth; ++u) ok = ok && __float_as_uint(pv[u].x) != kRowNormUnset;  // surplus loads hold a real record too
          if (__all(ok)) break;
          if (wait_expired(polls)) {
            if (lane == 0) {
              s_timeout[par] = 1;
              // the head is done again by the two-pass kernels that follow this one in the stream
              a.ws.head_redo[(int64_t)lh * a.batch + b] = 1;
              atomicAdd(&a.ws.hdr->n_unfused, 1);
            }
            break;
          }
          __builtin_amdgcn_s_sleep(1);
          load_records(pp);
        }
#pragma unroll
        for (int u = 0; u < kMergeDepth; ++u) {
          if (pp + 4 * u < np) {  // uniform
            const float nm = fmaxf(m, pv[u].x);
            s = s * __builtin_amdgcn_exp2f(m - nm) + pv[u].y * __builtin_amdgcn_exp2f(pv[u].x - nm);
            m = nm;
          }
        }
      }
      if (lane < R) {
        mstat[wave][lane][0] = m;
        mstat[wave][lane][1] = s;
      }
    }
    __builtin_amdgcn_s_setprio(0);
    lds_barrier();  // B2: the quarters are there; the next item's queries and offsets are committed
    if (lane < R) {  // every wave folds the four quarters into its own copy of the normalisers
      float m = kRefInit;
#pragma unroll
      for (int w = 0; w < 4; ++w) m = fmaxf(m, mstat[w][lane][0]);
      float s = 0.f;
#pragma unroll
      for (int w = 0; w < 4; ++w) s += mstat[w][lane][1] * __builtin_amdgcn_exp2f(mstat[w][lane][0] - m);
      row_norm_l[wave][lane] = s > 0.f ? m + __builtin_amdgcn_logf(s) : INFINITY;  // log2 of the softmax normaliser
    }

    // =============== second phase: token importance from the logits still in registers =========
    if (cur.nst > 0) {
      float cn[SLP];
#pragma unroll
      for (int q = 0; q < SLP; ++q) {
        const int al = q / NP, i = q % NP;
        const bool used = q < SL && i < n && (g + 4 * al) < a.alpha;
        cn[q] = used ? row_norm_l[wave][16 * (q >> 2) + 4 * g + (q & 3)] : INFINITY;
      }
      float part[SUBS];  // per stage: the lane's token, summed over the lane group's window queries
#pragma unroll
      for (int st = 0; st < SUBS; ++st) {
        part[st] = 0.f;
        if (st < cur.nst) {
#pragma unroll
          for (int al = 0; al < AL; ++al) {
            float gm = -INFINITY;
#pragma unroll
            for (int i = 0; i < NP; ++i) {
              const int q = al * NP + i;
              gm = fmaxf(gm, fmaf(acc[st][q >> 2][q & 3], kScale2, -cn[q]));  // masked logits are -inf already
            }
            part[st] += __builtin_amdgcn_exp2f(gm);
          }
        }
      }
      // the four lane groups hold the four quarters of the window: all stages' exchanges back to back
      float other[SUBS];
#pragma unroll
      for (int st = 0; st < SUBS; ++st) other[st] = __shfl_xor(part[st], 16);
#pragma unroll
      for (int st = 0; st < SUBS; ++st) part[st] += other[st];
#pragma unroll
      for (int st = 0; st < SUBS; ++st) other[st] = __shfl_xor(part[st], 32);
#pragma unroll
      for (int st = 0; st < SUBS; ++st) {
        const int t = w0 + 16 * st + c16;
        if (g == 0 && st < cur.nst) imp[wave][16 * st + c16] = (t < w1) ? (part[st] + other[st]) * inv_alpha : 0.f;
      }
    }
    // imp[wave] is written and read by this wave only: no barrier
    const int p_start = n_tok - min(a.protect, n_tok);
    const int64_t tok_col = (int64_t)lh * a.total_tokens + cur.tok0;
    {  // sentence means: 4 lanes per sentence, wave w takes the sentences of span w
      static_assert(kSpanMaxSent * 4 <= 64, "4 lanes per sentence of a span");
      const int tl = opaque(lane);
      const int s_idx = tl >> 2, part = tl & 3;
      const bool valid = s_idx < ns;
      float sum_i = 0.f, sum_r = 0.f;
      int lo = 0, hi = 0;
      if (valid) {
        lo = soff[cur.sb + s_idx];
        hi = min(soff[cur.sb + s_idx + 1], p_start);
        for (int t = lo + part; t < hi; t += 4) {
          sum_i += imp[wave][t - w0];
          if (a.tok_red) sum_r += a.tok_red[tok_col + t];
        }
      }
      sum_i += __shfl_xor(sum_i, 1);
      sum_r += __shfl_xor(sum_r, 1);
      sum_i += __shfl_xor(sum_i, 2);
      sum_r += __shfl_xor(sum_r, 2);
      if (valid && part == 0) {
        const int64_t o = (int64_t)lh * a.total_sentences + (cur.soff_idx - b) + cur.sb + s_idx;
        const float inv = hi > lo ? 1.f / (float)(hi - lo) : 0.f;
        if (s_timeout[par]) sum_i = __builtin_nanf("");
        a.ws.sent_imp[o] = sum_i * inv;
        a.ws.sent_red[o] = sum_r * inv;
      }
    }
    if (a.tok_imp) {
      const int tl = opaque(lane);
      for (int i = tl; i < w1 - w0; i += 64) a.tok_imp[tok_col + w0 + i] = imp[wave][i];
    }
    // No barrier here: every buffer shared between waves is written next only after at least one
    // of the next item's barriers, which no wave passes before all have finished reading above.
    cur = nxt;
    par ^= 1;
  }
}

template <int DT, int NP, int AL>
hipError_t launch_one(const ScanArgs &a, hipStream_t st) {
  int dev = 0, cus = 0, per_cu = 0;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return e;
  e = hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev);
  if (e != hipSuccess) return e;
  e = hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, k_scan_fused<DT, NP, AL>, 256, 0);
  if (e != hipSuccess) return e;
  const int grid = cus * per_cu;  // persistent: every workgroup is resident at once
  if (grid < kFuseMaxItems) return hipErrorInvalidConfiguration;
  hipLaunchKernelGGL((k_scan_fused<DT, NP, AL>), dim3(grid), dim3(256), 0, st, a);
  return hipGetLastError();
}

}  // namespace

bool scan_fused_supported(const RowLayout &rl, int64_t row_pitch_bytes) {
  return rl.nt <= 4 && row_pitch_bytes > 0 && row_pitch_bytes < (1 << 24);  // the key loads form lane offsets with a 24-bit multiply
}

hipError_t launch_scan_fused(const ScanArgs &a, hipStream_t st) {
  if ((int64_t)a.n_layers * a.n_kv_heads * a.batch == 0 || a.force_two_pass) return hipSuccess;
#define SKIPKV_CASE(NP_, AL_)                                                \
  if (a.rl.np == NP_ && a.rl.al == AL_)                                      \
    return a.dtype == SKIPKV_BF16 ? launch_one<SKIPKV_BF16, NP_, AL_>(a, st) \
                                  : launch_one<SKIPKV_F32, NP_, AL_>(a, st);
  SKIPKV_CASE(4, 2)
  SKIPKV_CASE(4, 4)
  SKIPKV_CASE(7, 2)
  SKIPKV_CASE(8, 2)
#undef SKIPKV_CASE
  return hipErrorInvalidValue;
}

}  // namespace skipkv

// Single-pass key scan (Sec. 4.1 "Token Importance Score", Eq. 4; sentence embedding of Eq. 2
// over the head's keys): K is read from HBM exactly once.
//
// The softmax normaliser of a query row needs all N keys of the head, which are spread over many
// chunks, i.e. many workgroups.  Instead of a second pass over K, every workgroup keeps the
// logits of its share in registers (they are MFMA accumulators anyway: per wave 64 tokens x all
// query rows of the GQA group, for each of two consecutive chunks), publishes the (max, sum exp)
// of every row over its share as one record, and then merges the records of ALL shares of the
// head itself, loading them again while any still holds the marker that the plan preset it to.
// (Heads of more than kAllMergeMax items keep an older protocol: an arrive counter, the last share
// to arrive merges and writes the normalisers over their marker, the others poll those.)  Then
// each workgroup finishes I[t] from its registers.  A unit of work ("item") is a PAIR of
// consecutive chunks of one head, so that the exchange is paid once per 512 tokens.
//
// Forward progress.  The grid is persistent and no larger than what is co-resident on the chip
// (occupancy query on the host).  Workgroup w takes items w, w+G, w+2G, ... in increasing order,
// a head's items being consecutive.  A workgroup only ever waits for the head of the item it has
// just published.  Since a head has at most kFuseMaxChunks/2 <= G items, they belong to distinct
// workgroups, each of which reaches its item of that head without waiting on that head first;
// by induction over heads in item order every wait ends.  The wait is bounded anyway
// (spin_limit polls): on expiry SKIPKV_DEV_TIMEOUT is raised and the kernel runs to completion
// with invalid scores rather than hanging.
//
// Data movement.  Inside a workgroup the 4 waves are independent streams: wave w owns tokens
// [64w, 64w+64) of each chunk, in stages of 16 rows.  Rows go HBM -> LDS directly
// (global_load_lds, 16 bytes per lane, no staging registers) into a ring of NBUF stage buffers
// private to the wave, and the wave always keeps NBUF-1 stages in flight ahead of the one it is
// computing on - also across the end of an item, so the synchronisation at the end of an item
// overlaps with the first loads of the next one.  A direct load writes LDS at base + lane*16, so
// rows are stored unpadded; bank conflicts are avoided by an XOR swizzle instead: the 16-byte
// piece p of row r is kept at piece position p ^ (r & 15), which each lane arranges by choosing
// which global piece it fetches.
//
// Paged cache.  With a row map (logical token -> block slot) and blocks of a power of two >= 16
// slots, a stage spans at most two blocks: two scalar reads of the map give two bases per stage.
//
// Pooling.  Key sums per sentence come from 4x4x4 matrix products of a 0/1 indicator with the
// stage's rows.  A sentence that lies inside one wave's range is normalised and written straight from
// registers; the (at most 3 per chunk) sentences that cross wave boundaries are pieced together
// through LDS in a fixed order, so results are reproducible.
#include "scan_dev.h"

#ifndef SKIPKV_FRAG_AHEAD
#define SKIPKV_FRAG_AHEAD 3  // query fragments are read this many matrix instructions ahead of their use
#endif

namespace skipkv {

namespace {

constexpr int kCapW = kChunkCap / 4;  // tokens per wave per chunk
constexpr int kStageRows = 16;        // rows per pipeline stage = one MFMA sub-tile of tokens
constexpr int kStagesPerWave = kCapW / kStageRows;

struct ChunkD {  // one chunk as seen by one wave
  int ns, t_begin, t_end, soff_idx;
  int w0, w1, nst;  // the wave's token range and its number of stages
};
struct Pair {  // one item
  uint32_t item;  // >= n_items: none
  int lh, b, c0, nch, n_tok, tok0, np, c_first;
  const char *kbase;
  ChunkD ch[2];
};

template <int DT, int NP, int AL>
__global__ void __launch_bounds__(256, (DT == SKIPKV_BF16 ? 2 : 1)) k_scan_fused(ScanArgs a) {
  constexpr int SL = NP * AL;
  constexpr int NT = (SL + 3) / 4;
  constexpr int SLP = 4 * NT;
  constexpr int R = 16 * NT;
  constexpr int SUBS = kStagesPerWave;
  constexpr int LSTR = Tr<DT>::LSTR, ROWB = Tr<DT>::ROWB, ESZ = Tr<DT>::ESZ;
  constexpr int PPR = ROWB / 16;                      // 16-byte pieces per row
  constexpr int GL = kStageRows * PPR / 64;           // direct loads per stage
  constexpr int RPL = 64 / PPR;                       // rows covered by one direct load
  constexpr int NBUF = 2;                             // stage buffers per wave (a third one gains nothing: memory latency does not pace the waves)
  constexpr int STAGEB = kStageRows * ROWB;
  // bf16 keys are pooled by matrix products with an indicator whose ones are written as 2.0 (a
  // single bit, cheap to build from a row mask): all key sums of that path carry this factor,
  // which the normalisation to a unit vector removes.
  constexpr float kPoolScale = (DT == SKIPKV_BF16) ? 2.f : 1.f;

  __shared__ __align__(256) char kt[4][NBUF][STAGEB];  // 256-byte aligned: the row swizzle is applied as an XOR on address bits
  __shared__ __align__(16) char qt[R * LSTR];
  __shared__ int soff_buf[2][2][kChunkMaxSent + 2];  // [item parity][chunk of the pair]
  __shared__ float part_first[2][4][kD];  // key sum, over a wave's range, of the sentence already running at its start
  __shared__ float part_last[2][4][kD];   // key sum of the sentence that starts in a wave's range and runs past its end
  __shared__ float wstat[4][R][2];
  __shared__ float imp[2][kChunkCap];
  __shared__ int s_flag;
  __shared__ int s_timeout;  // a wait of the current item ran out: its sentences get NaN means, so that the selection keeps the head whole
  __shared__ float row_norm_l[R];

  const int tid = threadIdx.x, lane = tid & 63, c16 = lane & 15, g = lane >> 4;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);  // in a scalar register: everything derived from it is uniform control flow
  const int n_lh = a.n_layers * a.n_kv_heads;
  const int n_pairs = hdr_pairs(a.ws.hdr->ranges);
  const uint32_t n_items = (uint32_t)n_lh * (uint32_t)n_pairs;
  const int n = a.n_q_heads / a.n_kv_heads;
  const int64_t tok_pitch = a.stride_tok * ESZ;
  const float inv_alpha = 1.f / (float)a.alpha;
  if (a.force_two_pass) return;
  // The plan is constant while this kernel runs: reading it through the constant address space
  // lets the compiler use scalar loads, which do not queue behind the key loads in flight.
  typedef const __attribute__((address_space(4))) int32_t *ConstIntPtr;
  const ConstIntPtr pair_rec_c = (ConstIntPtr)a.ws.pair_rec;
  const ConstIntPtr row_map_c = (ConstIntPtr)a.row_map;  // written by an earlier kernel, constant here

  // ---- item descriptors: one 64-byte record per pair of chunks, written by the plan ----------
  auto make_chunk = [&](int t_begin, int len, int ns, int soff_idx) -> ChunkD {
    ChunkD d;
    d.ns = ns;
    d.t_begin = t_begin;
    d.t_end = t_begin + len;
    d.soff_idx = soff_idx;
    d.w0 = d.t_begin + wave * kCapW;
    d.w1 = min(d.w0 + kCapW, d.t_end);
    d.nst = d.w1 > d.w0 ? (d.w1 - d.w0 + kStageRows - 1) / kStageRows : 0;
    return d;
  };
  auto load_pair = [&](uint32_t item) -> Pair {  // first fused item at or after `item` in this workgroup's sequence
    Pair it{};
    for (; item < n_items; item += gridDim.x) {
      const ConstIntPtr r = pair_rec_c + (int64_t)(item % n_pairs) * kPairRecInts;
      const int nch = r[kPrNch];
      if (nch == 0) continue;  // the sequence takes the two-pass scan
      it.lh = item / n_pairs;
      it.b = r[kPrB];
      it.c0 = r[kPrC0];
      it.nch = nch;
      it.tok0 = r[kPrTok0];
      it.n_tok = r[kPrNTok];
      it.np = r[kPrNPairs];
      it.c_first = r[kPrCFirst];
      it.ch[0] = make_chunk(r[kPrTBegin], r[kPrLen0], r[kPrNs0], r[kPrSoffIdx]);
      it.ch[1] = nch == 2 ? make_chunk(r[kPrTBegin] + r[kPrLen0], r[kPrLen1], r[kPrNs1], r[kPrSoffIdx] + r[kPrNs0]) : ChunkD{};
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
  auto q_fetch = [&](const Pair &it) -> QFetch {
    QFetch f;
    const int t = opaque(tid);
    f.so = 0;
    if (t <= it.ch[0].ns) f.so = a.sent_off[it.ch[0].soff_idx + t];
    if (it.nch == 2 && t >= 64 && t - 64 <= it.ch[1].ns) f.so = a.sent_off[it.ch[1].soff_idx + t - 64];
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
  auto q_commit = [&](const Pair &it, const QFetch &f, int par) {
    const int t = opaque(tid);
    if (t <= it.ch[0].ns) soff_buf[par][0][t] = f.so;
    if (it.nch == 2 && t >= 64 && t - 64 <= it.ch[1].ns) soff_buf[par][1][t - 64] = f.so;
#pragma unroll
    for (int u = 0; u < NQ; ++u) {
      const int r = u * (256 / PPR) + t / PPR, piece = t % PPR;
      *reinterpret_cast<uint4 *>(qt + r * LSTR + piece * 16) = f.q[u];
    }
  };

  // ---- the wave's load stream: stages of consecutive chunks, NBUF-1 ahead of the compute ------
  Pair iss = load_pair(blockIdx.x);  // item whose stages are being issued
  int iss_k = 0;                     // ... chunk of that item
  int iss_st = 0;                    // ... next stage of that chunk
  uint32_t iss_cnt = 0;              // stages issued so far (ring position)
  uint32_t iss_from = 0xFFFFFFFFu;   // the item the stream was on before it moved to `iss`
  auto issue_next = [&]() -> bool {
    while (iss.item < n_items && iss_st >= (iss_k ? iss.ch[1].nst : iss.ch[0].nst)) {
      if (iss_k + 1 < iss.nch) {
        ++iss_k;
      } else {
        iss_from = iss.item;
        iss = load_pair(iss.item + gridDim.x);
        iss_k = 0;
      }
      iss_st = 0;
    }
    if (iss.item >= n_items) return false;
    char *dst = kt[wave][iss_cnt % NBUF];
    const int ts = (iss_k ? iss.ch[1].w0 : iss.ch[0].w0) + iss_st * kStageRows;
    const int w1 = iss_k ? iss.ch[1].w1 : iss.ch[0].w1;
    int ln = lane;
    asm volatile("" : "+v"(ln));  // opaque copy: the per-load address parts are recomputed here rather than kept live across the item
    // scalar 64-bit base of the stage + a 32-bit offset per lane (one 24-bit multiply; the launcher
    // only takes this kernel for row pitches below 2^24 bytes): no 64-bit multiplies per load
    const int last = w1 - 1 - ts;  // rows past the range re-read its last row (masked later)
    const uint32_t pitch32 = (uint32_t)tok_pitch;
    if (a.row_map == nullptr) {
      const char *sbase = iss.kbase + (int64_t)ts * tok_pitch;
#pragma unroll
      for (int j = 0; j < GL; ++j) {
        const int row = j * RPL + ln / PPR;         // row of the stage this lane's 16 bytes belong to
        const int piece = (ln % PPR) ^ (row & 15);    // swizzle: LDS position (lane % PPR) holds this global piece
        const uint32_t off = __umul24((uint32_t)min(row, last), pitch32) + (uint32_t)piece * 16u;
        load_to_lds_16(sbase + off, dst + j * 1024);
      }
    } else {
      // Paged cache, blocks of a power of two >= 16 slots: the stage's 16 tokens lie in at most two
      // blocks, in consecutive slots within each.  Two scalar reads of the row map give the slot
      // row of the stage's first token and of the first token of the next block.  Map entries count
      // units of map_stride elements (the token pitch, or one head row when every (layer, head) has a
      // map of its own); consecutive slots of a block are one token pitch apart either way.
      const int jb = a.page_size - (ts & (a.page_size - 1));  // rows of the stage before the next block begins (may be >= 16)
      const int r0 = row_map_c[iss.tok0 + ts];
      const int r1 = row_map_c[iss.tok0 + min(ts + jb, iss.n_tok - 1)];
      const int64_t map_pitch = a.map_stride * ESZ;  // bytes per unit of the row map
      const char *base0 = iss.kbase + (int64_t)r0 * map_pitch;
      const char *base1 = iss.kbase + (int64_t)r1 * map_pitch - (int64_t)jb * tok_pitch;
#pragma unroll
      for (int j = 0; j < GL; ++j) {
        const int row = j * RPL + ln / PPR;
        const int piece = (ln % PPR) ^ (row & 15);
        const int jr = min(row, last);
        const uint32_t off = __umul24((uint32_t)jr, pitch32) + (uint32_t)piece * 16u;
        load_to_lds_16((jr >= jb ? base1 : base0) + off, dst + j * 1024);
      }
    }
    ++iss_st;
    ++iss_cnt;
    return true;
  };

  // A wait has run out when it has used up its polls, or when any wait of this launch did before
  // (looked up every 256 polls): the first time-out is reported and raises the launch's abort word.
  auto wait_expired = [](const ScanArgs &a, int polls) -> bool {
    if (polls < a.spin_limit && ((polls & 255) != 255 || __hip_atomic_load(&a.ws.hdr->abort, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) == 0)) return false;
    if ((threadIdx.x & 63) == 0) {
      if (a.dev_status) atomicOr(a.dev_status, SKIPKV_DEV_TIMEOUT);
      __hip_atomic_store(&a.ws.hdr->abort, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
    return true;
  };
  Pair cur = load_pair(blockIdx.x);
  if (cur.item >= n_items) return;
#pragma unroll
  for (int i = 0; i < NBUF - 1; ++i) issue_next();
  uint32_t cmp_cnt = 0;  // stages computed so far (ring position)
  int par = 0;           // which soff buffers hold the current item's offsets
  q_commit(cur, q_fetch(cur), par);
  lds_barrier();

  while (cur.item < n_items) {
    const int lh = cur.lh, b = cur.b;
    const int n_tok = cur.n_tok;
    const int lhb = lh * a.batch + b;
    const int last_free = n_tok - a.alpha;  // keys t <= last_free are visible to every window query

    f32x4 acc[2][SUBS][NT];
    float ref[SLP], lsum[SLP];
#pragma unroll
    for (int q = 0; q < SLP; ++q) {
      ref[q] = kRefInit;
      lsum[q] = 0.f;
    }

    auto emit_sentence = [&](int len, int sent_col0, int s_idx, float k0, float k1) {  // unit embedding, bf16 hi + lo
      // mean / (|mean| + eps) = sum / (|sum| + eps * len): no division by the length.  1-ulp
      // reciprocal and square root: a common scale error of ~1e-7 on the unit vector
      // (bf16 keys: the sums arrive scaled by kPoolScale, and so does the epsilon)
      const float inv = __builtin_amdgcn_rcpf(__builtin_amdgcn_sqrtf(wave_sum_fast(k0 * k0 + k1 * k1)) + (1e-12f * kPoolScale) * (float)len);
      const float u0 = k0 * inv, u1 = k1 * inv;
      const uint32_t hi = pack_bf16x2(u0, u1);  // round to nearest even, both halves in one instruction
      const uint32_t lo = pack_bf16x2(u0 - __uint_as_float(hi << 16), u1 - __uint_as_float(hi & 0xFFFF0000u));
      // the lane's part of the address is formed here, from an opaque copy: kept across the item it
      // could be spilled, and its reload would wait for every key load in flight
      const int64_t o = ((int64_t)lh * a.total_sentences + sent_col0 + s_idx) * (kD / 2) + opaque(lane);
      reinterpret_cast<uint32_t *>(a.ws.vhat_hi)[o] = hi;
      reinterpret_cast<uint32_t *>(a.ws.vhat_lo)[o] = lo;
    };

    // =============== first phase: logits, row statistics and sentence key sums =================
#pragma unroll
    for (int k = 0; k < 2; ++k) {
#pragma unroll
      for (int s = 0; s < SUBS; ++s)
#pragma unroll
        for (int T = 0; T < NT; ++T) acc[k][s][T] = f32x4{0.f, 0.f, 0.f, 0.f};
      if (k < cur.nch) {
        const ChunkD &cd = cur.ch[k];
        const int *soff = soff_buf[par][k];
        const int ns = cd.ns, w0 = cd.w0, w1 = cd.w1;
        const int sent_col0 = cd.soff_idx - b;
        // sentence pooling state: current sentence si and the running key sums of sentences si .. si+3
        // (lane = 2 head-dim columns: pk0 the even one, pk1 the odd one; component j belongs to sentence
        // si + j; the fp32 path only uses component 0); lane i keeps offset i of the chunk, so that
        // boundaries are fetched with v_readlane
        const int soff_v = soff[min(lane, ns)];
        int si = 0;
        f32x4 pk0 = {0.f, 0.f, 0.f, 0.f}, pk1 = {0.f, 0.f, 0.f, 0.f};
        if (w0 < w1) si = __popcll(__ballot(lane >= 1 && lane <= ns && soff_v <= w0));
        int s_bgn = __builtin_amdgcn_readlane(soff_v, si), s_end = __builtin_amdgcn_readlane(soff_v, min(si + 1, ns));

#pragma unroll
        for (int st = 0; st < SUBS; ++st) {
          if (st < cd.nst) {
            const int ts = w0 + st * kStageRows, te = min(ts + kStageRows, w1);
            // keep the load stream NBUF-1 stages ahead, then wait for this stage's rows to land
            if (issue_next())
              wait_vm<GL *(NBUF - 1)>();
            else
              wait_all();
            const char *stage = kt[wave][cmp_cnt % NBUF];
            ++cmp_cnt;

            // ---- logits of this stage's 16 tokens against all query rows
            if constexpr (DT == SKIPKV_BF16) {
              // Fragment reads run AHEAD matrix instructions ahead of their use (the order is
              // pinned: the compiler would otherwise read each fragment right before its use and pay
              // the LDS latency every time, or read all of them first and run out of registers).
              // Step i multiplies slice i / NT of the head dimension into row tile i % NT.
              constexpr int AHEAD = SKIPKV_FRAG_AHEAD, NSTEP = 4 * NT;
              // key row c16, piece (4g + kk) ^ c16: the stage buffers are 256-byte aligned, so the slice
              // index is an XOR on bits 4..5 of one address per lane (no address register per slice)
              const uint32_t baddr = lds_addr(stage) + c16 * ROWB + (((4 * g) ^ c16) << 4);
              const char *arow = qt + c16 * LSTR + g * 64;
              auto rd_a = [&](int i) { return *reinterpret_cast<const bf16x8 *>(arow + 16 * (i % NT) * LSTR + (i / NT) * 16); };
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
                acc[k][st][i % NT] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(afr[i], bfr[i / NT], acc[k][st][i % NT], 0, 0, 0);
                __builtin_amdgcn_sched_barrier(0);
              }
            } else {
#pragma unroll
              for (int cc = 0; cc < 8; ++cc) {
                const float4 bfrag = *reinterpret_cast<const float4 *>(stage + c16 * ROWB + (((4 * cc + g) ^ c16) * 16));
#pragma unroll
                for (int T = 0; T < NT; ++T) {
                  const float4 afrag = *reinterpret_cast<const float4 *>(qt + (16 * T + c16) * LSTR + cc * 64 + g * 16);
                  acc[k][st][T] = __builtin_amdgcn_mfma_f32_16x16x4f32(afrag.x, bfrag.x, acc[k][st][T], 0, 0, 0);
                  acc[k][st][T] = __builtin_amdgcn_mfma_f32_16x16x4f32(afrag.y, bfrag.y, acc[k][st][T], 0, 0, 0);
                  acc[k][st][T] = __builtin_amdgcn_mfma_f32_16x16x4f32(afrag.z, bfrag.z, acc[k][st][T], 0, 0, 0);
                  acc[k][st][T] = __builtin_amdgcn_mfma_f32_16x16x4f32(afrag.w, bfrag.w, acc[k][st][T], 0, 0, 0);
                }
              }
            }

            // ---- running softmax statistics of every query row (accumulators stay unscaled)
            {
              const int t = ts + c16;
              const bool edge = (ts + 15 >= te) || (ts + 15 > last_free);
              if (edge) {
#pragma unroll
                for (int q = 0; q < SLP; ++q) {
                  const int aq = g + 4 * (q / NP);
                  if (!(t < te && t <= last_free + aq)) acc[k][st][q >> 2][q & 3] = -INFINITY;
                }
              }
              // exponent arguments relative to the running references; one test tells whether any of
              // them has outgrown its reference (then the references are refreshed, rarely)
              float e[SLP];
              float emax = -INFINITY;
#pragma unroll
              for (int q = 0; q < SLP; ++q) {
                e[q] = fmaf(acc[k][st][q >> 2][q & 3], kScale2, -ref[q]);
                emax = fmaxf(emax, e[q]);
              }
              if (__any(emax > kRescaleSlack)) {
#pragma unroll
                for (int q = 0; q < SLP; ++q) {
                  const float nr = fmaxf(ref[q], row16_max_fast(acc[k][st][q >> 2][q & 3]) * kScale2);
                  lsum[q] *= __builtin_amdgcn_exp2f(ref[q] - nr);
                  ref[q] = nr;
                  e[q] = fmaf(acc[k][st][q >> 2][q & 3], kScale2, -nr);
                }
              }
#pragma unroll
              for (int q = 0; q < SLP; ++q) lsum[q] += __builtin_amdgcn_exp2f(e[q]);
            }

            // ---- sentence key sums over tokens [ts, te).  All rows of the stage come into registers
            // with one LDS round trip (lane = 2 head-dim columns of every row).
            if (!a.no_pool) {
              float x0[kStageRows], x1[kStageRows];
              uint32_t xw[kStageRows];
              // the stage buffers are 256-byte aligned, so the swizzle (piece ^ row) is an XOR on bits
              // 4..7 of the address: one VALU op per row, the row's base goes into the offset field
              if constexpr (DT == SKIPKV_BF16) {
                const uint32_t la = lds_addr(stage) + ((lane >> 2) << 4) + (lane & 3) * 4;
#pragma unroll
                for (int i = 0; i < kStageRows; ++i) xw[i] = lds_read_u32((la ^ (i << 4)) + i * ROWB);
              } else {
                const uint32_t la = lds_addr(stage) + ((lane >> 1) << 4) + (lane & 1) * 8;
#pragma unroll
                for (int i = 0; i < kStageRows; ++i) {
                  x0[i] = lds_read_f32((la ^ (i << 4)) + i * ROWB);
                  x1[i] = lds_read_f32((la ^ (i << 4)) + i * ROWB + 4);
                }
              }
              auto sentence_done = [&]() {  // sentence si ends: emit it (or leave its part), move the sums up one place
                if (s_bgn >= w0) {
                  emit_sentence(s_end - s_bgn, sent_col0, si, pk0[0], pk1[0]);
                } else {
                  part_first[k][wave][2 * lane] = pk0[0];
                  part_first[k][wave][2 * lane + 1] = pk1[0];
                }
                pk0 = f32x4{pk0[1], pk0[2], pk0[3], 0.f};
                pk1 = f32x4{pk1[1], pk1[2], pk1[3], 0.f};
                ++si;
                s_bgn = s_end;
                s_end = __builtin_amdgcn_readlane(soff_v, min(si + 1, ns));
              };
              int t = ts;
              if constexpr (DT == SKIPKV_BF16) {
                // Segment sums on the matrix cores: [4 sentences x 16 tokens] 0/1 indicator times
                // [16 tokens x 128 columns] keys, as 4x4x4 products in 16 independent blocks.  Every
                // block gets the same indicator rows (lane % 4 = sentence si + lane % 4) and four
                // columns of its own; a lane's B operand is its own column, so the result comes back
                // in the lane that pools that column: register j = sentence si + j.  One product per
                // 4 tokens and column parity, whatever the number of sentence ends in the stage; the
                // loop below runs again only when more than 4 sentences meet in one stage.
                while (t < te) {
                  const int g_end = min(__builtin_amdgcn_readlane(soff_v, min(si + 4, ns)), te);
                  if (g_end <= t) break;  // cannot happen with validated offsets; never spin on bad ones
                  const int c = min(si + (lane & 3), ns), c1 = min(c + 1, ns);
                  const int lo_t = max(soff[c], t), hi_t = min(soff[c1], g_end);
                  uint32_t rows = 0;  // rows of the stage that belong to this lane's sentence
                  if (hi_t > lo_t) rows = ((1u << (hi_t - ts)) - 1u) & ~((1u << (lo_t - ts)) - 1u);
#pragma unroll
                  for (int q = 0; q < kStageRows / 4; ++q) {
                    // indicator of rows 4q .. 4q+3 as four bf16 values 2.0 (= bit 14 alone) or 0: row bits
                    // 4q, 4q+1 go to bits 14 and 30 of the first word, 4q+2, 4q+3 of the second one, by
                    // shifts and one mask each (every other bit that the shifts bring along is masked off)
                    const uint2 ind = make_uint2(((rows << (14 - 4 * q)) | (rows << (29 - 4 * q))) & 0x40004000u,
                                                 ((rows << (12 - 4 * q)) | (rows << (27 - 4 * q))) & 0x40004000u);
                    const bf16x4_t av = __builtin_bit_cast(bf16x4_t, ind);
                    // tokens 4q .. 4q+3 of the even column (low halves) and of the odd column (high halves)
                    const uint2 be = make_uint2(__builtin_amdgcn_perm(xw[4 * q + 1], xw[4 * q], 0x05040100u),
                                                __builtin_amdgcn_perm(xw[4 * q + 3], xw[4 * q + 2], 0x05040100u));
                    const uint2 bo = make_uint2(__builtin_amdgcn_perm(xw[4 * q + 1], xw[4 * q], 0x07060302u),
                                                __builtin_amdgcn_perm(xw[4 * q + 3], xw[4 * q + 2], 0x07060302u));
                    pk0 = __builtin_amdgcn_mfma_f32_4x4x4bf16_1k(av, __builtin_bit_cast(bf16x4_t, be), pk0, 0, 0, 0);
                    pk1 = __builtin_amdgcn_mfma_f32_4x4x4bf16_1k(av, __builtin_bit_cast(bf16x4_t, bo), pk1, 0, 0, 0);
                  }
                  t = g_end;
                  while (si < ns && s_end <= t) sentence_done();
                }
              } else {
                // fp32 keys: every run of rows that belongs to one sentence is added with a 0/1 weight
                // per row taken from a scalar bit mask, so there is no branch per row
                while (t < te) {
                  const int run_end = min(s_end, te);
                  if (run_end <= t) break;  // cannot happen with validated offsets; never spin on bad ones
                  const uint32_t rows = ((1u << (run_end - ts)) - 1u) & ~((1u << (t - ts)) - 1u);  // rows of this run
#pragma unroll
                  for (int i = 0; i < kStageRows; ++i) {
                    const float m = ((rows >> i) & 1u) ? 1.f : 0.f;
                    pk0[0] = fmaf(x0[i], m, pk0[0]);
                    pk1[0] = fmaf(x1[i], m, pk1[0]);
                  }
                  t = run_end;
                  if (t == s_end) sentence_done();
                }
              }
            }
          }
        }
        if (!a.no_pool && w0 < w1 && si < ns && s_bgn < w1 && w1 < s_end) {  // a sentence is still running at the end of this wave's range
          float *dst = (s_bgn >= w0) ? part_last[k][wave] : part_first[k][wave];
          dst[2 * lane] = pk0[0];
          dst[2 * lane + 1] = pk1[0];
        }
      }
    }
    // The next item is usually known already (the load stream has just moved on to it; after very
    // short items it may be further ahead, then the descriptor is read again).  Its queries and
    // offsets are fetched now and committed before the second barrier below, so that their latency
    // and the sentences pieced together below overlap with the round trips of the exchange.  After
    // the last item the descriptor is all zero: the fetch then reads valid memory that nobody uses,
    // which keeps fetch and commit free of conditions (a fetch that may stay uncommitted would
    // make the compiler drain the load queue at the next fetch).
    const Pair nxt = (iss_from == cur.item) ? iss : load_pair(cur.item + gridDim.x);
    const QFetch nq = q_fetch(nxt);
#pragma unroll
    for (int q = 0; q < SLP; ++q) {
      const float tot = row16_sum_fast(lsum[q]);
      if (c16 == 0) {
        const int r = 16 * (q >> 2) + 4 * g + (q & 3);
        wstat[wave][r][0] = ref[q];
        wstat[wave][r][1] = tot;
      }
    }
    lds_barrier();  // every wave is done with the query tile and has left its partials

    // ---- publish the share's row statistics (one record per item, filed under its first chunk).
    // The last wave does it, lane = query row: no sentence that crosses a wave boundary starts in
    // its range, so it has nothing else to do while the other waves piece those together.
    static_assert(R <= 64, "the record is written by one wave: only that wave waits for the acknowledgement");
    // Heads of at most kAllMergeMax items: no arrive counter and no merging workgroup.  Every
    // workgroup of the head polls the head's records (the plan has preset them to a marker) and
    // merges them itself, so nobody waits for one workgroup's merge and there is no
    // acknowledgement + counter + publication chain between the last record and the readers.
    const bool all_merge = cur.np <= kAllMergeMax;
    int arrived = 0;
    if (wave == 3) {
      if (lane < R) {
        float m = kRefInit;
#pragma unroll
        for (int w = 0; w < 4; ++w) m = fmaxf(m, wstat[w][lane][0]);
        float s = 0.f;
#pragma unroll
        for (int w = 0; w < 4; ++w) s += wstat[w][lane][1] * __builtin_amdgcn_exp2f(wstat[w][lane][0] - m);
        coherent_store2(&a.ws.stat_part[((int64_t)lh * a.ws.nc_max + cur.c0) * R + lane], make_float2(m, s));
      }
      if (!all_merge) {
        wait_all();  // the statistics are acknowledged (the other waves keep their key loads in flight)
        if (lane == 0) arrived = __hip_atomic_fetch_add(&a.ws.arrive[lhb], 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      }
    }
    // ---- sentences that cross wave boundaries: the wave in whose range one starts pieces it together
#pragma unroll
    for (int k = 0; k < 2; ++k) {
      if (k < cur.nch) {
        const ChunkD &cd = cur.ch[k];
        const int *soff = soff_buf[par][k];
        if (cd.w0 < cd.w1 && wave < 3 && !a.no_pool) {
          const int sl = __popcll(__ballot(lane < cd.ns && soff[lane + 1] <= cd.w1 - 1));  // sentence holding the wave's last token
          if (soff[sl] >= cd.w0 && soff[sl + 1] > cd.w1) {
            const int ln = opaque(lane);
            float k0 = part_last[k][wave][2 * ln], k1 = part_last[k][wave][2 * ln + 1];
            for (int w = wave + 1; w < 4 && cd.t_begin + w * kCapW < soff[sl + 1]; ++w) {
              k0 += part_first[k][w][2 * ln];
              k1 += part_first[k][w][2 * ln + 1];
            }
            emit_sentence(soff[sl + 1] - soff[sl], cd.soff_idx - b, sl, k0, k1);
          }
        }
      }
    }
    q_commit(nxt, nq, par ^ 1);
    if (tid == 192) {
      s_flag = all_merge || (arrived == cur.np - 1);
      s_timeout = 0;
    }
    lds_barrier();
    float *rn = a.ws.row_norm + (int64_t)lhb * R;
    if (s_flag) {  // merge the head's partials into the normalisers (every share, or the last one to arrive)
      // lane = query row, wave w takes items w, w+4, ...; 8 independent loads in flight per lane.
      // A record that has not been written yet still holds the plan's marker: load again.
      const int c_first = cur.c_first, np = cur.np;
      for (int r = opaque(lane); r < R; r += 64) {
        float m = kRefInit, s = 0.f;
        for (int pp = wave; pp < np; pp += 32) {
          float2 pv[8];
          for (int polls = 0;; ++polls) {
            bool ok = true;
#pragma unroll
            for (int u = 0; u < 8; ++u) {
              pv[u] = make_float2(kRefInit, 0.f);
              if (pp + 4 * u < np)
                pv[u] = coherent_load2(&a.ws.stat_part[((int64_t)lh * a.ws.nc_max + c_first + 2 * (pp + 4 * u)) * R + r]);
              ok = ok && __float_as_uint(pv[u].x) != kRowNormUnset;
            }
            if (__all(ok)) break;
            if (wait_expired(a, polls)) {
              if (lane == 0) s_timeout = 1;
              break;
            }
            __builtin_amdgcn_s_sleep(1);
          }
#pragma unroll
          for (int u = 0; u < 8; ++u) {
            const float nm = fmaxf(m, pv[u].x);
            s = s * __builtin_amdgcn_exp2f(m - nm) + pv[u].y * __builtin_amdgcn_exp2f(pv[u].x - nm);
            m = nm;
          }
        }
        wstat[wave][r][0] = m;
        wstat[wave][r][1] = s;
      }
      lds_barrier();
      for (int r = opaque(tid); r < R; r += 256) {
        float mm = kRefInit;
#pragma unroll
        for (int w = 0; w < 4; ++w) mm = fmaxf(mm, wstat[w][r][0]);
        float ss = 0.f;
#pragma unroll
        for (int w = 0; w < 4; ++w) ss += wstat[w][r][1] * __builtin_amdgcn_exp2f(wstat[w][r][0] - mm);
        const float v = ss > 0.f ? mm + __builtin_amdgcn_logf(ss) : INFINITY;  // log2 of the softmax normaliser
        if (!all_merge) coherent_store(&rn[r], v);  // for the workgroups that poll
        row_norm_l[r] = v;  // this workgroup uses its own copy
      }
      // no flag: the readers poll the rows themselves, which the plan has preset to a marker
    } else if (wave == 0) {
      // wait for the head's normalisers: one coherent load per row and poll, all rows at once;
      // they go round the workgroup through LDS
      const uint32_t *rn_bits = reinterpret_cast<const uint32_t *>(rn);
      for (int polls = 0;; ++polls) {
        const uint32_t u = lane < R ? __hip_atomic_load(&rn_bits[lane], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) : 0u;
        const bool done = __all(u != kRowNormUnset);
        if (done || wait_expired(a, polls)) {
          if (!done && lane == 0) s_timeout = 1;
          if (lane < R) row_norm_l[opaque(lane)] = __uint_as_float(u);
          break;
        }
        __builtin_amdgcn_s_sleep(2);
      }
    }
    lds_barrier();

    // =============== second phase: token importance from the logits still in registers =========
    float cn[SLP];
#pragma unroll
    for (int q = 0; q < SLP; ++q) {
      const int al = q / NP, i = q % NP;
      const bool used = q < SL && i < n && (g + 4 * al) < a.alpha;
      cn[q] = used ? row_norm_l[16 * (q >> 2) + 4 * g + (q & 3)] : INFINITY;
    }
#pragma unroll
    for (int k = 0; k < 2; ++k) {
      if (k < cur.nch) {
#pragma unroll
        for (int s = 0; s < SUBS; ++s) {
          const int t = cur.ch[k].w0 + 16 * s + c16;
          float sum = 0.f;
#pragma unroll
          for (int al = 0; al < AL; ++al) {
            float gm = -INFINITY;
#pragma unroll
            for (int i = 0; i < NP; ++i) {
              const int q = al * NP + i;
              gm = fmaxf(gm, fmaf(acc[k][s][q >> 2][q & 3], kScale2, -cn[q]));  // masked logits are -inf already
            }
            sum += __builtin_amdgcn_exp2f(gm);
          }
          sum += __shfl_xor(sum, 16);
          sum += __shfl_xor(sum, 32);
          if (g == 0) imp[k][wave * kCapW + 16 * s + c16] = (t < cur.ch[k].w1) ? sum * inv_alpha : 0.f;
        }
      }
    }
    lds_barrier();
    const int p_start = n_tok - min(a.protect, n_tok);
    const int64_t tok_col = (int64_t)lh * a.total_tokens + cur.tok0;
    {  // sentence means: 4 lanes per sentence; threads 0..127 take the first chunk, 128..255 the second
      static_assert(kChunkMaxSent * 4 <= 128, "4 lanes per sentence of a chunk");
      const int tl = opaque(tid);
      const int k = tl >> 7, s_idx = (tl & 127) >> 2, part = tl & 3;
      const bool valid = k < cur.nch && s_idx < (k ? cur.ch[1].ns : cur.ch[0].ns);
      float sum_i = 0.f, sum_r = 0.f;
      int lo = 0, hi = 0;
      if (valid) {
        const int *soff = soff_buf[par][k];
        const int t_begin = k ? cur.ch[1].t_begin : cur.ch[0].t_begin;
        lo = soff[s_idx];
        hi = min(soff[s_idx + 1], p_start);
        for (int t = lo + part; t < hi; t += 4) {
          sum_i += imp[k][t - t_begin];
          if (a.tok_red) sum_r += a.tok_red[tok_col + t];
        }
      }
      sum_i += __shfl_xor(sum_i, 1);
      sum_r += __shfl_xor(sum_r, 1);
      sum_i += __shfl_xor(sum_i, 2);
      sum_r += __shfl_xor(sum_r, 2);
      if (valid && part == 0) {
        const int sent_col0 = (k ? cur.ch[1].soff_idx : cur.ch[0].soff_idx) - b;
        const int64_t o = (int64_t)lh * a.total_sentences + sent_col0 + s_idx;
        const float inv = hi > lo ? 1.f / (float)(hi - lo) : 0.f;
        if (s_timeout) sum_i = __builtin_nanf("");
        a.ws.sent_imp[o] = sum_i * inv;
        a.ws.sent_red[o] = sum_r * inv;
      }
    }
    if (a.tok_imp) {
      const int tl = opaque(tid);
#pragma unroll
      for (int k = 0; k < 2; ++k)
        if (k < cur.nch)
          for (int i = tl; i < cur.ch[k].t_end - cur.ch[k].t_begin; i += 256)
            a.tok_imp[tok_col + cur.ch[k].t_begin + i] = imp[k][i];
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
  if (grid < kFuseMaxChunks / 2) return hipErrorInvalidConfiguration;
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

// The key scan of the compression step (Sec. 4.1 "Token Importance Score", Eq. 4, and the
// sentence embedding of Eq. 2 taken over the head's keys).
//
// One workgroup (4 waves) handles one chunk of one head: a run of whole sentences of up to
// kChunkCap tokens (longer only when a single sentence is).  Keys stream HBM -> LDS in tiles of TT tokens with 16-byte-per-lane
// coalesced loads; each wave multiplies its 16*NSUB tokens against all query rows of the GQA
// group on the matrix cores (16x16 MFMA tiles, fp32 accumulate), so a lane ends up holding, for
// ONE token, the logits of every (window query a, group head i) pair assigned to its lane group.
//
// The softmax of Eq. 4 runs over all N keys of the head, which span many chunks, so it takes
// two passes over K:
//   pass A (PASSB = false): per chunk, the running (max, sum of exp) of every query row, and the
//       mean-pooled, L2-normalised key of every sentence of the chunk (split into bf16 hi + lo);
//   k_row_norm: merges the per-chunk statistics into log2 of each row's normaliser;
//   pass B (PASSB = true): recomputes the logits, forms I[t] = (1/alpha) sum_a max_i softmax and
//       its mean over the unprotected part of every sentence.
// exp() is evaluated in base 2: logits are scaled by log2(e)/sqrt(d).
#include "scan_common.h"

#include <algorithm>

namespace skipkv {

namespace {

template <int DT, int NP, int AL, int NSUB, bool PASSB>
// (two workgroups per CU are asked for where the query tile leaves room for them in LDS: bf16, up to 160 rows)
__global__ void __launch_bounds__(256, ((DT == SKIPKV_BF16 && NP * AL <= 40) ? 2 : 1)) k_scan(ScanArgs a) {
  constexpr int SL = NP * AL;        // used (a, i) slots per lane group
  constexpr int NT = (SL + 3) / 4;   // row tiles
  constexpr int SLP = 4 * NT;        // slots incl. padding
  constexpr int R = 16 * NT;         // padded query rows
  constexpr int WT = 16 * NSUB;      // tokens per wave per tile
  constexpr int TT = 4 * WT;         // tokens per tile
  constexpr int LSTR = Tr<DT>::LSTR, ROWB = Tr<DT>::ROWB, ESZ = Tr<DT>::ESZ;
  constexpr int PPR = ROWB / 16;     // 16-byte pieces per row
  constexpr int LOADS = TT * PPR / 256;

  __shared__ __align__(16) char kt[TT * LSTR];
  __shared__ __align__(16) char qt[R * LSTR];
  __shared__ int soff[kChunkMaxSent + 1];
  // pass A: sentence key sums [kChunkMaxSent][128] then per-wave row statistics [4][R][2]
  // pass B: token importance of the tile [TT], sentence sums of I and of R [2][kChunkMaxSent]
  constexpr int SBUF = PASSB ? (TT + 2 * kChunkMaxSent) : (kChunkMaxSent * kD);
  __shared__ float sbuf[SBUF];

  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63, c16 = lane & 15, g = lane >> 4;
  // Fallback path: only sequences that the single-pass scan cannot take (a sentence longer than
  // a chunk, or too many chunks), unless the caller forces this path for everything.
  if (!a.force_two_pass && a.ws.hdr->n_unfused == 0) return;
  const int n_lh = a.n_layers * a.n_kv_heads;
  const int n_chunks = hdr_chunks(a.ws.hdr->ranges);
  const uint32_t n_items = (uint32_t)n_lh * (uint32_t)n_chunks;
  const int n = a.n_q_heads / a.n_kv_heads;
  for (uint32_t item = blockIdx.x; item < n_items; item += gridDim.x) {
  const int lh = item / n_chunks, c = item % n_chunks;
  const Chunk ch = a.ws.chunks[c];
  const int b = ch.b, ns = ch.ns;
  if (!a.force_two_pass && a.ws.seq_fused[b] && !a.ws.head_redo[(int64_t)lh * a.batch + b]) continue;  // done by the single-pass scan
  const int l = lh / a.n_kv_heads, h = lh % a.n_kv_heads;
  const int tok0 = ch.tok0;
  const int n_tok = ch.n_tok;
  const int sent_col0 = ch.soff_idx - b;  // column of the chunk's first sentence in [.., S_total] arrays
  __syncthreads();  // the previous item's readers of LDS are done

  if (tid <= ns) soff[tid] = a.sent_off[ch.soff_idx + tid];
  for (int i = tid; i < SBUF; i += 256) sbuf[i] = 0.f;

  // ---- queries of the group -> LDS, one padded row per (lane group, slot)
  {
    const char *qbase = static_cast<const char *>(a.q);
    // layer, KV head and sequence that address the query rows (the real ones under per-head ranges)
    int ql = l, qh = h, qb = b, q_batch = a.batch, q_heads = a.n_q_heads;
    if (a.virt_hk > 0) {
      const int lh_r = b / a.virt_b;
      qb = b % a.virt_b;
      ql = lh_r / a.virt_hk;
      qh = lh_r % a.virt_hk;
      q_batch = a.virt_b;
      q_heads = a.virt_hk * n;
    }
    for (int r0 = 0; r0 < R; r0 += 256 / PPR) {
      const int r = r0 + tid / PPR, piece = tid % PPR;
      const int slot = 4 * (r >> 4) + (r & 3), gq = (r >> 2) & 3;
      const int al = slot / NP, i = slot % NP, aq = gq + 4 * al;
      uint4 val = make_uint4(0, 0, 0, 0);
      if (slot < SL && i < n && aq < a.alpha) {
        const int64_t row = (((int64_t)ql * q_batch + qb) * q_heads + (qh * n + i)) * a.alpha + aq;
        val = *reinterpret_cast<const uint4 *>(qbase + row * ROWB + piece * 16);
      }
      *reinterpret_cast<uint4 *>(qt + r * LSTR + piece * 16) = val;
    }
  }
  __syncthreads();

  const int t_begin = soff[0], t_end = soff[ns];
  // contiguous cache: row t of the sequence is row tok0 + t of the head; paged cache: the row map says where it is
  const int32_t *rmap = a.row_map ? a.row_map + tok0 : nullptr;
  const char *kbase = static_cast<const char *>(a.k) +
                      ((int64_t)l * a.stride_layer + (int64_t)h * a.stride_head + (rmap ? 0 : (int64_t)tok0 * a.stride_tok)) * ESZ;
  const int64_t tok_pitch = (a.row_map ? a.map_stride : a.stride_tok) * ESZ;  // paged: bytes per unit of the row map
  const int last_free = n_tok - a.alpha;  // keys t <= last_free are visible to every window query

  // per-lane state
  float ref[SLP], lsum[SLP];  // pass A: reference (uniform over the 16 lanes of a row) and sum of exp2(x - ref)
  float cn[SLP];              // pass B: log2 normaliser of the slot's query row (+inf: unused slot)
  if constexpr (!PASSB) {
#pragma unroll
    for (int q = 0; q < SLP; ++q) {
      ref[q] = kRefInit;
      lsum[q] = 0.f;
    }
  } else {
    const float *rn = a.ws.row_norm + ((int64_t)lh * a.batch + b) * R;
#pragma unroll
    for (int q = 0; q < SLP; ++q) {
      const int al = q / NP, i = q % NP;
      const bool used = q < SL && i < n && (g + 4 * al) < a.alpha;
      cn[q] = used ? rn[16 * (q >> 2) + 4 * g + (q & 3)] : INFINITY;
    }
  }
  const int p_start = n_tok - min(a.protect, n_tok);  // first protected token

  for (int tile_t = t_begin; tile_t < t_end; tile_t += TT) {
    // ---- stream the tile into LDS
    {
      uint4 regs[LOADS];
      int rows[LOADS];
#pragma unroll
      for (int it = 0; it < LOADS; ++it) {
        const int t = tile_t + (it * 256 + tid) / PPR;
        rows[it] = t;
        if (rmap && t < t_end) rows[it] = rmap[t];
      }
#pragma unroll
      for (int it = 0; it < LOADS; ++it) {
        const int idx = it * 256 + tid, row = idx / PPR, piece = idx % PPR, t = tile_t + row;
        regs[it] = make_uint4(0, 0, 0, 0);
        if (t < t_end) regs[it] = *reinterpret_cast<const uint4 *>(kbase + (int64_t)rows[it] * tok_pitch + piece * 16);
      }
#pragma unroll
      for (int it = 0; it < LOADS; ++it) {
        const int idx = it * 256 + tid, row = idx / PPR, piece = idx % PPR;
        *reinterpret_cast<uint4 *>(kt + row * LSTR + piece * 16) = regs[it];
      }
    }
    __syncthreads();

    const int wt0 = tile_t + wave * WT;  // first token of this wave's share
    f32x4 acc[NSUB][NT];
#pragma unroll
    for (int s = 0; s < NSUB; ++s) {
#pragma unroll
      for (int T = 0; T < NT; ++T) acc[s][T] = f32x4{0.f, 0.f, 0.f, 0.f};
      if (wt0 + 16 * s < t_end)
        tile_logits<DT, NT>(qt, kt + (wave * WT + 16 * s + c16) * LSTR, c16, g, acc[s]);
    }

    if constexpr (!PASSB) {
      // ---- running softmax statistics of every query row over this wave's tokens
      float tmax[SLP];
#pragma unroll
      for (int q = 0; q < SLP; ++q) tmax[q] = -INFINITY;
#pragma unroll
      for (int s = 0; s < NSUB; ++s) {
        const int t = wt0 + 16 * s + c16;
        const bool edge = (wt0 + 16 * s + 15 >= t_end) || (wt0 + 16 * s + 15 > last_free);
#pragma unroll
        for (int q = 0; q < SLP; ++q) {
          float x = acc[s][q >> 2][q & 3] * kScale2;
          if (edge) {
            const int aq = g + 4 * (q / NP);
            if (!(t < t_end && t <= last_free + aq)) x = -INFINITY;
          }
          acc[s][q >> 2][q & 3] = x;
          tmax[q] = fmaxf(tmax[q], x);
        }
      }
      bool need = false;
#pragma unroll
      for (int q = 0; q < SLP; ++q) need |= tmax[q] > ref[q] + kRescaleSlack;
      if (__any(need)) {
#pragma unroll
        for (int q = 0; q < SLP; ++q) {
          const float nr = fmaxf(ref[q], row16_max(tmax[q]));
          lsum[q] *= __builtin_amdgcn_exp2f(ref[q] - nr);
          ref[q] = nr;
        }
      }
#pragma unroll
      for (int s = 0; s < NSUB; ++s)
#pragma unroll
        for (int q = 0; q < SLP; ++q) lsum[q] += __builtin_amdgcn_exp2f(acc[s][q >> 2][q & 3] - ref[q]);

      // ---- sentence key sums: wave w takes sentences w, w + 4, ... of the chunk, lane = 2 head-dim
      // columns.  A sentence's rows are added in token order by one wave only (also across the tiles
      // of the chunk), so the sums are the same bits on every run.
      {
        const int t_hi = min(tile_t + TT, t_end);
        for (int si = __popcll(__ballot(lane < ns && soff[lane + 1] <= tile_t)); si < ns && soff[si] < t_hi; ++si) {
          if ((si & 3) != wave) continue;
          const int lo = max(soff[si], tile_t), hi = min(soff[si + 1], t_hi);
          float s0 = 0.f, s1 = 0.f;
          for (int t = lo; t < hi; ++t) {
            const char *rowp = kt + (t - tile_t) * LSTR;
            if constexpr (DT == SKIPKV_BF16) {
              const uint32_t w = *reinterpret_cast<const uint32_t *>(rowp + lane * 4);
              s0 += __uint_as_float(w << 16);
              s1 += __uint_as_float(w & 0xFFFF0000u);
            } else {
              const float2 w = *reinterpret_cast<const float2 *>(rowp + lane * 8);
              s0 += w.x;
              s1 += w.y;
            }
          }
          sbuf[si * kD + 2 * lane] += s0;
          sbuf[si * kD + 2 * lane + 1] += s1;
        }
      }
    } else {
      // ---- token importance: max over the group's heads in registers, exp2, sum over window queries
      float *imp = sbuf;
#pragma unroll
      for (int s = 0; s < NSUB; ++s) {
        const int t = wt0 + 16 * s + c16;
        const bool edge = (wt0 + 16 * s + 15 > last_free);
        float sum = 0.f;
#pragma unroll
        for (int al = 0; al < AL; ++al) {
          float gm = -INFINITY;
#pragma unroll
          for (int i = 0; i < NP; ++i) {
            const int q = al * NP + i;
            gm = fmaxf(gm, fmaf(acc[s][q >> 2][q & 3], kScale2, -cn[q]));
          }
          if (edge && t > last_free + g + 4 * al) gm = -INFINITY;
          sum += __builtin_amdgcn_exp2f(gm);
        }
        sum += __shfl_xor(sum, 16);
        sum += __shfl_xor(sum, 32);
        if (g == 0) imp[wave * WT + 16 * s + c16] = (t < t_end) ? sum / (float)a.alpha : 0.f;
      }
      __syncthreads();
      // sentence sums over the unprotected part, and the optional per-token outputs / inputs
      const int64_t tok_col = (int64_t)lh * a.total_tokens + tok0;
      if (tid < ns) {
        const int lo = max(soff[tid], tile_t), hi = min(min(soff[tid + 1], p_start), tile_t + TT);
        float si = 0.f, sr = 0.f;
        for (int t = lo; t < hi; ++t) {
          si += imp[t - tile_t];
          if (a.tok_red) sr += a.tok_red[tok_col + t];
        }
        sbuf[TT + tid] += si;
        sbuf[TT + kChunkMaxSent + tid] += sr;
      }
      if (a.tok_imp) {
        for (int i = tid; i < TT && tile_t + i < t_end; i += 256) a.tok_imp[tok_col + tile_t + i] = imp[i];
      }
    }
    __syncthreads();  // the next tile overwrites kt / imp
  }

  if constexpr (!PASSB) {
    // ---- unit sentence embeddings, split into bf16 hi + lo, one wave per sentence
    for (int si = wave; si < ns && !a.no_pool; si += 4) {
      const float inv_len = 1.f / (float)(soff[si + 1] - soff[si]);
      const float m0 = sbuf[si * kD + 2 * lane] * inv_len, m1 = sbuf[si * kD + 2 * lane + 1] * inv_len;
      const float nrm = sqrtf(wave_sum(m0 * m0 + m1 * m1));
      const float inv = 1.f / (nrm + 1e-12f);
      const float u0 = m0 * inv, u1 = m1 * inv;
      const uint32_t h0 = f32_to_bf16_bits(u0), h1 = f32_to_bf16_bits(u1);
      const uint32_t l0 = f32_to_bf16_bits(u0 - bf16_bits_to_f32(h0)), l1 = f32_to_bf16_bits(u1 - bf16_bits_to_f32(h1));
      const int64_t o = ((int64_t)lh * a.total_sentences + sent_col0 + si) * (kD / 2) + lane;
      reinterpret_cast<uint32_t *>(a.ws.vhat_hi)[o] = h0 | (h1 << 16);
      reinterpret_cast<uint32_t *>(a.ws.vhat_lo)[o] = l0 | (l1 << 16);
    }
    // ---- merge the row statistics of the 4 waves and publish the chunk's partial
    // (in the key tile's buffer, which nobody reads after the last tile: with 160 query rows this keeps
    // the workgroup under half of the CU's LDS)
    static_assert(8 * R * sizeof(float) <= sizeof(kt), "the statistics of the 4 waves fit the key tile");
    float *wstat = reinterpret_cast<float *>(kt);
#pragma unroll
    for (int q = 0; q < SLP; ++q) {
      const float tot = row16_sum(lsum[q]);
      if (c16 == 0) {
        const int r = 16 * (q >> 2) + 4 * g + (q & 3);
        wstat[(wave * R + r) * 2] = ref[q];
        wstat[(wave * R + r) * 2 + 1] = tot;
      }
    }
    __syncthreads();
    for (int r = tid; r < R; r += 256) {
      float m = kRefInit;
#pragma unroll
      for (int w = 0; w < 4; ++w) m = fmaxf(m, wstat[(w * R + r) * 2]);
      float s = 0.f;
#pragma unroll
      for (int w = 0; w < 4; ++w) s += wstat[(w * R + r) * 2 + 1] * __builtin_amdgcn_exp2f(wstat[(w * R + r) * 2] - m);
      a.ws.stat_part[((int64_t)lh * a.ws.nc_max + c) * R + r] = make_float2(m, s);
    }
  } else {
    if (tid < ns) {
      const int len = min(soff[tid + 1], p_start) - soff[tid];
      const int64_t o = (int64_t)lh * a.total_sentences + sent_col0 + tid;
      a.ws.sent_imp[o] = len > 0 ? sbuf[TT + tid] / (float)len : 0.f;
      a.ws.sent_red[o] = len > 0 ? sbuf[TT + kChunkMaxSent + tid] / (float)len : 0.f;
    }
  }
  }  // item loop
}

// ---- many query rows (more than four row tiles; bf16) ------------------------------------------
// With n * alpha > 64 query rows the kernel above reads every query fragment from LDS again for
// every 16 tokens, and that LDS traffic is what bounds it.  Here the rows are split over the
// waves instead of the tokens: wave w owns the window queries al = w*APW .. w*APW+APW-1 of every
// lane group (all NP heads of each, so that the maximum over the group's heads stays inside a
// lane), keeps their query fragments in registers for the whole chunk (loaded straight from
// global memory: no query tile in LDS), and multiplies them with all 64 tokens of a key tile.
// Row statistics need no merge across waves (a row belongs to one wave); token importance does
// (a token's window queries are spread over the waves) and goes through a small LDS array.
// Row ids: r = wave * RW + 16 * T + 4 * g + j for local row tile T, lane group g, register j.
template <int NP, int AL>
struct WideShape {
  static constexpr int APW = AL / 4;            // window-query slots per wave and lane group
  static constexpr int SPW = APW * NP;          // used (a, i) slots per wave
  static constexpr int TPW = (SPW + 3) / 4;     // row tiles per wave
  static constexpr int SLW = 4 * TPW;           // slots per wave incl. padding
  static constexpr int RW = 16 * TPW;           // query rows per wave
  static constexpr int R = 4 * RW;              // rows of the statistics arrays
};

template <int NP, int AL, bool PASSB>
__global__ void __launch_bounds__(256, PASSB ? 4 : 3) k_scan_wide(ScanArgs a) {
  using WS = WideShape<NP, AL>;
  constexpr int APW = WS::APW, SPW = WS::SPW, TPW = WS::TPW, SLW = WS::SLW, RW = WS::RW;
  constexpr int TT = 64;             // tokens per key tile: four sub-tiles of 16
  constexpr int LSTR = Tr<SKIPKV_BF16>::LSTR, ROWB = Tr<SKIPKV_BF16>::ROWB, ESZ = 2;
  constexpr int PPR = ROWB / 16, LOADS = TT * PPR / 256;
  static_assert(AL % 4 == 0, "the window-query slots are dealt out to four waves");

  __shared__ __align__(16) char kt[TT * LSTR];
  __shared__ int soff[kChunkMaxSent + 1];
  // pass A: sentence key sums [kChunkMaxSent][128]
  // pass B, per group of GT tokens (four tiles): token importance [GT], sentence sums of I and of R
  // [2][kChunkMaxSent], per-wave parts [4][GT]
  constexpr int GT = 4 * TT;
  constexpr int SBUF = PASSB ? (GT + 2 * kChunkMaxSent + 4 * GT) : (kChunkMaxSent * kD);
  __shared__ float sbuf[SBUF];

  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63, c16 = lane & 15, g = lane >> 4;
  if (!a.force_two_pass && a.ws.hdr->n_unfused == 0) return;
  const int R = a.ws.rows;  // stride of the statistics arrays (>= WS::R)
  const int n_lh = a.n_layers * a.n_kv_heads;
  const int n_chunks = hdr_chunks(a.ws.hdr->ranges);
  const uint32_t n_items = (uint32_t)n_lh * (uint32_t)n_chunks;
  const int n = a.n_q_heads / a.n_kv_heads;
  for (uint32_t item = blockIdx.x; item < n_items; item += gridDim.x) {
  const int lh = item / n_chunks, c = item % n_chunks;
  const Chunk ch = a.ws.chunks[c];
  const int b = ch.b, ns = ch.ns;
  if (!a.force_two_pass && a.ws.seq_fused[b] && !a.ws.head_redo[(int64_t)lh * a.batch + b]) continue;  // done by the single-pass scan
  const int l = lh / a.n_kv_heads, h = lh % a.n_kv_heads;
  const int tok0 = ch.tok0;
  const int n_tok = ch.n_tok;
  const int sent_col0 = ch.soff_idx - b;
  __syncthreads();  // the previous item's readers of LDS are done

  if (tid <= ns) soff[tid] = a.sent_off[ch.soff_idx + tid];
  for (int i = tid; i < SBUF; i += 256) sbuf[i] = 0.f;

  // ---- the wave's query fragments: lane (row c16 of a tile, head-dim slice g), as the A operand wants them
  bf16x8 afr[TPW][4];
  {
    const char *qbase = static_cast<const char *>(a.q);
    // layer, KV head and sequence that address the query rows (the real ones under per-head ranges)
    int ql = l, qh = h, qb = b, q_batch = a.batch, q_heads = a.n_q_heads;
    if (a.virt_hk > 0) {
      const int lh_r = b / a.virt_b;
      qb = b % a.virt_b;
      ql = lh_r / a.virt_hk;
      qh = lh_r % a.virt_hk;
      q_batch = a.virt_b;
      q_heads = a.virt_hk * n;
    }
#pragma unroll
    for (int T = 0; T < TPW; ++T) {
      // row c16 of a tile is register (c16 & 3) of lane group c16 / 4 in the output
      const int slot = 4 * T + (c16 & 3), gq = c16 >> 2;
      const int al = wave * APW + slot / NP, i = slot % NP, aq = gq + 4 * al;
      const bool used = slot < SPW && i < n && aq < a.alpha;
      const int64_t row = (((int64_t)ql * q_batch + qb) * q_heads + (qh * n + (used ? i : 0))) * a.alpha + (used ? aq : 0);
#pragma unroll
      for (int kk = 0; kk < 4; ++kk) {
        uint4 v = make_uint4(0, 0, 0, 0);
        if (used) v = *reinterpret_cast<const uint4 *>(qbase + row * ROWB + g * 64 + kk * 16);
        afr[T][kk] = __builtin_bit_cast(bf16x8, v);
      }
    }
  }
  __syncthreads();

  const int t_begin = soff[0], t_end = soff[ns];
  // contiguous cache: row t of the sequence is row tok0 + t of the head; paged cache: the row map says where it is
  const int32_t *rmap = a.row_map ? a.row_map + tok0 : nullptr;
  const char *kbase = static_cast<const char *>(a.k) +
                      ((int64_t)l * a.stride_layer + (int64_t)h * a.stride_head + (rmap ? 0 : (int64_t)tok0 * a.stride_tok)) * ESZ;
  const int64_t tok_pitch = (a.row_map ? a.map_stride : a.stride_tok) * ESZ;  // paged: bytes per unit of the row map
  const int last_free = n_tok - a.alpha;  // keys t <= last_free are visible to every window query

  // per-lane state; slot q = 4 * T + j of this wave: window query g + 4 * (wave * APW + q / NP), head q % NP
  float ref[SLW], lsum[SLW], cn[SLW];
  const int64_t lhb = (int64_t)lh * a.batch + b;
#pragma unroll
  for (int q = 0; q < SLW; ++q) {
    ref[q] = kRefInit;
    lsum[q] = 0.f;
    cn[q] = INFINITY;  // pass B: log2 normaliser of the slot's query row (+inf: unused slot)
    if constexpr (PASSB) {
      const int i = q % NP, aq = g + 4 * (wave * APW + q / NP);
      const bool used = q < SPW && i < n && aq < a.alpha;
      if (used) cn[q] = a.ws.row_norm[lhb * R + wave * RW + 16 * (q >> 2) + 4 * g + (q & 3)];
    }
  }
  const int p_start = n_tok - min(a.protect, n_tok);  // first protected token

  // Pass A keeps the softmax statistics of a row relative to a reference that is fixed by the chunk's first
  // 16 tokens (one fma, one exponential, one add per logit).  Should a row's sum then lie outside what fp32
  // holds comfortably (a later logit far above the first ones, or all of them far below), the whole chunk is
  // done again with a running reference per row, as exactly as before; results agree up to rounding.
  [[maybe_unused]] bool exact = false;
  for (int attempt = 0; attempt < (PASSB ? 1 : 2); ++attempt) {
  if (attempt == 1) {
    exact = true;
#pragma unroll
    for (int q = 0; q < SLW; ++q) {
      ref[q] = kRefInit;
      lsum[q] = 0.f;
    }
    __syncthreads();
    for (int i = tid; i < SBUF; i += 256) sbuf[i] = 0.f;
    __syncthreads();
  }
  for (int tile_t = t_begin; tile_t < t_end; tile_t += TT) {
    // ---- stream the tile into LDS
    {
      uint4 regs[LOADS];
      int rows[LOADS];
#pragma unroll
      for (int it = 0; it < LOADS; ++it) {
        const int t = tile_t + (it * 256 + tid) / PPR;
        rows[it] = t;
        if (rmap && t < t_end) rows[it] = rmap[t];
      }
#pragma unroll
      for (int it = 0; it < LOADS; ++it) {
        const int idx = it * 256 + tid, row = idx / PPR, piece = idx % PPR, t = tile_t + row;
        regs[it] = make_uint4(0, 0, 0, 0);
        if (t < t_end) regs[it] = *reinterpret_cast<const uint4 *>(kbase + (int64_t)rows[it] * tok_pitch + piece * 16);
      }
#pragma unroll
      for (int it = 0; it < LOADS; ++it) {
        const int idx = it * 256 + tid, row = idx / PPR, piece = idx % PPR;
        *reinterpret_cast<uint4 *>(kt + row * LSTR + piece * 16) = regs[it];
      }
    }
    __syncthreads();

    // ---- per sub-tile of 16 tokens: logits of the wave's rows (acc[T][j] = row 4g+j of tile T, token 16s + c16),
    // then straight away what the pass needs from them, so that only one sub-tile's logits are live
    [[maybe_unused]] float *part = sbuf + GT + 2 * kChunkMaxSent + ((tile_t - t_begin) % GT);  // this tile's slice of the group
#pragma unroll
    for (int s = 0; s < 4; ++s) {
      if (tile_t + 16 * s >= t_end) {
        if constexpr (PASSB)
          if (g == 0) part[wave * GT + 16 * s + c16] = 0.f;
        continue;
      }
      f32x4 acc[TPW];
#pragma unroll
      for (int T = 0; T < TPW; ++T) acc[T] = f32x4{0.f, 0.f, 0.f, 0.f};
      const char *krow = kt + (16 * s + c16) * LSTR + g * 64;
#pragma unroll
      for (int kk = 0; kk < 4; ++kk) {
        const bf16x8 bfrag = *reinterpret_cast<const bf16x8 *>(krow + kk * 16);
#pragma unroll
        for (int T = 0; T < TPW; ++T) acc[T] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(afr[T][kk], bfrag, acc[T], 0, 0, 0);
      }
      const int t = tile_t + 16 * s + c16;
      if constexpr (!PASSB) {
        const bool edge = (tile_t + 16 * s + 15 >= t_end) || (tile_t + 16 * s + 15 > last_free);
        if (!exact) {
          if (s == 0 && tile_t == t_begin) {  // the chunk's first 16 tokens fix the references
#pragma unroll
            for (int q = 0; q < SLW; ++q) {
              float x = acc[q >> 2][q & 3] * kScale2;
              if (edge) {
                const int aq = g + 4 * (wave * APW + q / NP);
                if (!(t < t_end && t <= last_free + aq)) x = -INFINITY;
              }
              ref[q] = fmaxf(row16_max(x), kRefInit);
            }
          }
#pragma unroll
          for (int q = 0; q < SLW; ++q) {
            float x = fmaf(acc[q >> 2][q & 3], kScale2, -ref[q]);
            if (edge) {
              const int aq = g + 4 * (wave * APW + q / NP);
              if (!(t < t_end && t <= last_free + aq)) x = -INFINITY;
            }
            lsum[q] += __builtin_amdgcn_exp2f(x);
          }
          continue;
        }
        // running softmax statistics of the wave's query rows
        bool need = false;
#pragma unroll
        for (int q = 0; q < SLW; ++q) {
          float x = acc[q >> 2][q & 3] * kScale2;
          if (edge) {
            const int aq = g + 4 * (wave * APW + q / NP);
            if (!(t < t_end && t <= last_free + aq)) x = -INFINITY;
          }
          acc[q >> 2][q & 3] = x;
          need |= x > ref[q] + kRescaleSlack;
        }
        if (__any(need)) {
#pragma unroll
          for (int q = 0; q < SLW; ++q) {
            const float nr = fmaxf(ref[q], row16_max(acc[q >> 2][q & 3]));
            lsum[q] *= __builtin_amdgcn_exp2f(ref[q] - nr);
            ref[q] = nr;
          }
        }
#pragma unroll
        for (int q = 0; q < SLW; ++q) lsum[q] += __builtin_amdgcn_exp2f(acc[q >> 2][q & 3] - ref[q]);
      } else {
        // token importance: max over the group's heads in registers, exp2, sum over the wave's window queries
        const bool edge = (tile_t + 16 * s + 15 > last_free);
        float sum = 0.f;
#pragma unroll
        for (int al = 0; al < APW; ++al) {
          float gm = -INFINITY;
#pragma unroll
          for (int i = 0; i < NP; ++i) {
            const int q = al * NP + i;
            gm = fmaxf(gm, fmaf(acc[q >> 2][q & 3], kScale2, -cn[q]));
          }
          if (edge && t > last_free + g + 4 * (wave * APW + al)) gm = -INFINITY;
          sum += __builtin_amdgcn_exp2f(gm);
        }
        sum += __shfl_xor(sum, 16);
        sum += __shfl_xor(sum, 32);
        if (g == 0) part[wave * GT + 16 * s + c16] = sum;
      }
    }

    if constexpr (!PASSB) {
      // ---- sentence key sums: wave w takes sentences w, w + 4, ... of the chunk, lane = 2 head-dim
      // columns.  A sentence's rows are added in token order by one wave only (also across the tiles
      // of the chunk), so the sums are the same bits on every run.
      {
        const int t_hi = min(tile_t + TT, t_end);
        for (int si = __popcll(__ballot(lane < ns && soff[lane + 1] <= tile_t)); si < ns && soff[si] < t_hi; ++si) {
          if ((si & 3) != wave) continue;
          const int lo = max(soff[si], tile_t), hi = min(soff[si + 1], t_hi);
          float s0 = 0.f, s1 = 0.f;
          for (int t = lo; t < hi; ++t) {
            const uint32_t w = *reinterpret_cast<const uint32_t *>(kt + (t - tile_t) * LSTR + lane * 4);
            s0 += __uint_as_float(w << 16);
            s1 += __uint_as_float(w & 0xFFFF0000u);
          }
          sbuf[si * kD + 2 * lane] += s0;
          sbuf[si * kD + 2 * lane + 1] += s1;
        }
      }
    } else {
      // ---- at the end of a group of four tiles (or of the chunk): the four waves' parts of the token
      // importance are added in a fixed order, then the sentences' sums over their unprotected part
      const int g0 = t_begin + (tile_t - t_begin) / GT * GT;  // first token of the group
      if (tile_t + TT >= t_end || tile_t + TT >= g0 + GT) {
        float *imp = sbuf;
        const float *parts = sbuf + GT + 2 * kChunkMaxSent;
        const int g1 = min(min(t_end, tile_t + TT), g0 + GT);
        __syncthreads();
        {
          const float tot = ((parts[tid] + parts[GT + tid]) + parts[2 * GT + tid]) + parts[3 * GT + tid];
          imp[tid] = (g0 + tid < g1) ? tot / (float)a.alpha : 0.f;
        }
        __syncthreads();
        const int64_t tok_col = (int64_t)lh * a.total_tokens + tok0;
        {  // eight lanes per sentence
          static_assert(kChunkMaxSent * 8 <= 256, "eight lanes per sentence of a chunk");
          const int si = tid >> 3, sub = tid & 7;
          float sum_i = 0.f, sum_r = 0.f;
          if (si < ns) {
            const int lo = max(soff[si], g0), hi = min(min(soff[si + 1], p_start), g1);
            for (int t = lo + sub; t < hi; t += 8) {
              sum_i += imp[t - g0];
              if (a.tok_red) sum_r += a.tok_red[tok_col + t];
            }
          }
#pragma unroll
          for (int m = 1; m < 8; m <<= 1) {
            sum_i += __shfl_xor(sum_i, m);
            sum_r += __shfl_xor(sum_r, m);
          }
          if (si < ns && sub == 0) {
            sbuf[GT + si] += sum_i;
            sbuf[GT + kChunkMaxSent + si] += sum_r;
          }
        }
        if (a.tok_imp && g0 + tid < g1) a.tok_imp[tok_col + g0 + tid] = imp[tid];
      }
    }
    __syncthreads();  // the next tile overwrites kt; the next group imp and the parts
  }

  if constexpr (!PASSB) {
    if (attempt == 0) {
      bool doubt = false;
#pragma unroll
      for (int q = 0; q < SLW; ++q) {
        const int i = q % NP, aq = g + 4 * (wave * APW + q / NP);
        // rows of padding hold zero queries, and a window query that does not even see the chunk's first token sees none of it
        const bool used = q < SPW && i < n && aq < a.alpha && t_begin <= last_free + aq && t_begin < t_end;
        const float tot = row16_sum(lsum[q]);
        doubt = doubt || (used && !(tot > 1e-30f && tot < 3e38f));  // also catches NaN and infinity
      }
      if (!__syncthreads_or(doubt)) break;
    }
  }
  }  // attempts
  if constexpr (!PASSB) {
    // ---- unit sentence embeddings, split into bf16 hi + lo, one wave per sentence
    for (int si = wave; si < ns && !a.no_pool; si += 4) {
      const float inv_len = 1.f / (float)(soff[si + 1] - soff[si]);
      const float m0 = sbuf[si * kD + 2 * lane] * inv_len, m1 = sbuf[si * kD + 2 * lane + 1] * inv_len;
      const float nrm = sqrtf(wave_sum(m0 * m0 + m1 * m1));
      const float inv = 1.f / (nrm + 1e-12f);
      const float u0 = m0 * inv, u1 = m1 * inv;
      const uint32_t h0 = f32_to_bf16_bits(u0), h1 = f32_to_bf16_bits(u1);
      const uint32_t l0 = f32_to_bf16_bits(u0 - bf16_bits_to_f32(h0)), l1 = f32_to_bf16_bits(u1 - bf16_bits_to_f32(h1));
      const int64_t o = ((int64_t)lh * a.total_sentences + sent_col0 + si) * (kD / 2) + lane;
      reinterpret_cast<uint32_t *>(a.ws.vhat_hi)[o] = h0 | (h1 << 16);
      reinterpret_cast<uint32_t *>(a.ws.vhat_lo)[o] = l0 | (l1 << 16);
    }
    // ---- the chunk's partial statistics: every row belongs to one wave, nothing to merge
#pragma unroll
    for (int q = 0; q < SLW; ++q) {
      const float tot = row16_sum(lsum[q]);
      if (c16 == 0)
        a.ws.stat_part[((int64_t)lh * a.ws.nc_max + c) * R + wave * RW + 16 * (q >> 2) + 4 * g + (q & 3)] = make_float2(ref[q], tot);
    }
  } else {
    if (tid < ns) {
      const int len = min(soff[tid + 1], p_start) - soff[tid];
      const int64_t o = (int64_t)lh * a.total_sentences + sent_col0 + tid;
      a.ws.sent_imp[o] = len > 0 ? sbuf[GT + tid] / (float)len : 0.f;
      a.ws.sent_red[o] = len > 0 ? sbuf[GT + kChunkMaxSent + tid] / (float)len : 0.f;
    }
  }
  }  // item loop
}

// log2 of the softmax normaliser of every query row: merge the chunk partials of a head.
__global__ void k_row_norm(ScanArgs a, int R) {
  const int lhb = blockIdx.x, lh = lhb / a.batch, b = lhb % a.batch;
  if (!a.force_two_pass && a.ws.seq_fused[b] && !a.ws.head_redo[lhb]) return;  // the single-pass scan computed these itself
  const int c0 = a.ws.chunk_base[b], nc = a.ws.chunk_cnt[b];
  for (int r = threadIdx.x; r < R; r += blockDim.x) {
    float m = kRefInit, s = 0.f;
    for (int c = c0; c < c0 + nc; ++c) {
      const float2 p = a.ws.stat_part[((int64_t)lh * a.ws.nc_max + c) * R + r];
      const float nm = fmaxf(m, p.x);
      s = s * __builtin_amdgcn_exp2f(m - nm) + p.y * __builtin_amdgcn_exp2f(p.x - nm);
      m = nm;
    }
    a.ws.row_norm[(int64_t)lhb * R + r] = s > 0.f ? m + __builtin_amdgcn_logf(s) : INFINITY;
  }
}

template <int DT, int NP, int AL, bool PASSB>
hipError_t launch_one(const ScanArgs &a, hipStream_t st) {
  constexpr int NT = (NP * AL + 3) / 4;
  constexpr int NSUB = (DT == SKIPKV_F32) ? 1 : (NT <= 4 ? 2 : 1);
  const int64_t items = (int64_t)a.n_layers * a.n_kv_heads * a.ws.nc_max;
  if (items == 0) return hipSuccess;
  const int64_t grid = items < 4096 ? items : 4096;  // grid-stride over the items
  hipLaunchKernelGGL((k_scan<DT, NP, AL, NSUB, PASSB>), dim3((unsigned)grid), dim3(256), 0, st, a);
  return hipGetLastError();
}

template <int NP, int AL, bool PASSB>
hipError_t launch_wide(const ScanArgs &a, hipStream_t st) {
  if (a.ws.rows < WideShape<NP, AL>::R) return hipErrorInvalidValue;
  const int64_t items = (int64_t)a.n_layers * a.n_kv_heads * a.ws.nc_max;
  if (items == 0) return hipSuccess;
  const int64_t grid = items < 4096 ? items : 4096;  // grid-stride over the items
  hipLaunchKernelGGL((k_scan_wide<NP, AL, PASSB>), dim3((unsigned)grid), dim3(256), 0, st, a);
  return hipGetLastError();
}

template <bool PASSB>
hipError_t dispatch(const ScanArgs &a, hipStream_t st) {
  if (a.dtype == SKIPKV_BF16 && a.rl.nt > 4) {  // many query rows: rows split over the waves
    if (a.rl.np == 4 && a.rl.al == 8) return launch_wide<4, 8, PASSB>(a, st);
    if (a.rl.np == 8 && a.rl.al == 4) return launch_wide<8, 4, PASSB>(a, st);
    if (a.rl.np == 8 && a.rl.al == 8) return launch_wide<8, 8, PASSB>(a, st);
    if (a.rl.np == 5 && a.rl.al == 8) return launch_wide<5, 8, PASSB>(a, st);
  }
#define SKIPKV_CASE(NP_, AL_)                                                       \
  if (a.rl.np == NP_ && a.rl.al == AL_)                                             \
    return a.dtype == SKIPKV_BF16 ? launch_one<SKIPKV_BF16, NP_, AL_, PASSB>(a, st) \
                                  : launch_one<SKIPKV_F32, NP_, AL_, PASSB>(a, st);
  SKIPKV_CASE(4, 2)
  SKIPKV_CASE(4, 4)
  SKIPKV_CASE(4, 8)
  SKIPKV_CASE(8, 2)
  SKIPKV_CASE(8, 4)
  if (a.rl.np == 8 && a.rl.al == 8)  // 256 fp32 query rows do not fit in LDS: bf16 only
    return a.dtype == SKIPKV_BF16 ? launch_one<SKIPKV_BF16, 8, 8, PASSB>(a, st) : hipErrorInvalidValue;
  SKIPKV_CASE(5, 8)
  SKIPKV_CASE(7, 2)
#undef SKIPKV_CASE
  return hipErrorInvalidValue;
}

}  // namespace

int scan_two_pass_rows(const RowLayout &rl, int dtype) {
  if (dtype == SKIPKV_BF16 && rl.nt > 4 && rl.al % 4 == 0) {
    const int tiles_per_wave = ((rl.al / 4) * rl.np + 3) / 4;
    return std::max(rl.rows, 64 * tiles_per_wave);
  }
  return rl.rows;
}

hipError_t launch_scan_stats(const ScanArgs &a, hipStream_t st) { return dispatch<false>(a, st); }
hipError_t launch_scan_scores(const ScanArgs &a, hipStream_t st) { return dispatch<true>(a, st); }

hipError_t launch_row_norm(const ScanArgs &a, hipStream_t st) {
  const int blocks = a.n_layers * a.n_kv_heads * a.batch;
  if (blocks == 0) return hipSuccess;
  hipLaunchKernelGGL(k_row_norm, dim3(blocks), dim3(64), 0, st, a, a.rl.rows);
  return hipGetLastError();
}

}  // namespace skipkv

// Sentence-by-sentence redundancy (Sec. 4.1 "Sentence Similarity Score", Eq. 1 and Eq. 3) and
// the fused per-sentence score (Eq. 6).
//
// Per head the unit sentence embeddings form an S x 128 matrix; lambda_s is the row maximum of
// the strictly upper triangle of its Gram matrix.  The Gram tiles run on the bf16 matrix cores;
// to keep fp32-grade cosines (the ranking among near-duplicates depends on differences of
// ~1e-3) each embedding is carried as bf16 hi + bf16 lo and a tile is the product
// (hi + lo)(hi + lo)^T without its lo*lo term (below 2^-16 of a unit cosine, i.e. fp32-grade
// for the comparison with tau and for the ranking): three bf16 MFMAs, small terms first.
// One workgroup owns kRowBlock = 128 rows (32 per wave, A operands in registers) and walks the
// 64-column blocks at and to the right of the diagonal, staged through LDS and shared by the 4
// waves; the next column block is fetched into registers while the current one is multiplied.
#include "common.h"

namespace skipkv {

namespace {

constexpr int LSTR = 272;    // bytes per staged embedding row (256 + 16 so that 16-byte reads of 8 rows hit distinct banks)
constexpr int kColBlock = 64;
constexpr int kRowTiles = kRowBlock / 64;  // 16-row tiles per wave
static_assert(kRowBlock % 64 == 0, "four waves, whole tiles");

__global__ void __launch_bounds__(256, 3) k_cosine(CosineArgs a) {
  __shared__ __align__(16) char col_hi[kColBlock * LSTR];
  __shared__ __align__(16) char col_lo[kColBlock * LSTR];

  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63, c16 = lane & 15, g = lane >> 4;
  // the grid is sized for the largest possible number of row blocks; the work items that exist
  // are numbered densely (head-major) and dealt to the XCDs in contiguous ranges
  const uint32_t n_rb = (uint32_t)hdr_rowblocks(a.ws.hdr->ranges);
  const uint32_t n_items = (uint32_t)a.n_lh * n_rb;
  const uint32_t per_xcd = (n_items + 7u) / 8u;
  if (blockIdx.x >= 8u * per_xcd) return;
  const uint32_t item = xcd_contiguous_item(blockIdx.x, 8u * per_xcd);
  if (item >= n_items) return;
  const int lh = item / n_rb, rb = item % n_rb;
  const RowBlock blk = a.ws.rowblocks[rb];
  const int b = blk.b, r0 = blk.r0;
  const int sp = a.sent_ptr[b];
  const int n_sent = seq_sentences(a.sent_ptr, a.cnt, b);
  const int64_t col0 = (int64_t)lh * a.total_sentences + (sp - b);
  const char *hi = reinterpret_cast<const char *>(a.ws.vhat_hi) + col0 * 256;
  const char *lo = reinterpret_cast<const char *>(a.ws.vhat_lo) + col0 * 256;

  // A operands: this wave's rows, lane (row c16 of a tile, head-dim slice g)
  const int rw0 = r0 + 16 * kRowTiles * wave;
  bf16x8 a_hi[kRowTiles][4], a_lo[kRowTiles][4];
#pragma unroll
  for (int t = 0; t < kRowTiles; ++t) {
    const int row = rw0 + 16 * t + c16;
#pragma unroll
    for (int kk = 0; kk < 4; ++kk) {
      uint4 vh = make_uint4(0, 0, 0, 0), vl = make_uint4(0, 0, 0, 0);
      if (row < n_sent) {
        vh = *reinterpret_cast<const uint4 *>(hi + (int64_t)row * 256 + g * 64 + kk * 16);
        vl = *reinterpret_cast<const uint4 *>(lo + (int64_t)row * 256 + g * 64 + kk * 16);
      }
      a_hi[t][kk] = __builtin_bit_cast(bf16x8, vh);
      a_lo[t][kk] = __builtin_bit_cast(bf16x8, vl);
    }
  }
  // inputs of the epilogue, one row per lane (lanes c16 < 4 * kRowTiles), fetched now so that their
  // latency is hidden behind the products
  static_assert(4 * kRowTiles <= 16, "one epilogue row per lane of a 16-lane group");
  const int my_row = rw0 + 16 * (c16 >> 2) + 4 * g + (c16 & 3);
  const int n_tok = seq_tokens(a.seq_off, a.len, b);
  const int p_start = n_tok - min(a.protect, n_tok);
  float my_imp = 0.f, my_red = 0.f;
  int my_off = 0;
  if (c16 < 4 * kRowTiles && my_row < n_sent) {
    my_off = a.sent_off[sp + my_row];
    my_imp = a.ws.sent_imp[col0 + my_row];
    if (a.has_red) my_red = a.ws.sent_red[col0 + my_row];
  }
  float rmax[kRowTiles][4];
#pragma unroll
  for (int t = 0; t < kRowTiles; ++t)
#pragma unroll
    for (int j = 0; j < 4; ++j) rmax[t][j] = -INFINITY;

  // a column block is 2 x 64 rows x 16 pieces of 16 bytes: 8 pieces per thread
  uint4 pre[8];
  auto fetch = [&](int jb) {
#pragma unroll
    for (int it = 0; it < 8; ++it) {
      const int idx = it * 256 + tid, half = idx >> 10, rem = idx & 1023, row = rem >> 4, piece = rem & 15;
      pre[it] = make_uint4(0, 0, 0, 0);
      if (jb + row < n_sent) pre[it] = *reinterpret_cast<const uint4 *>((half ? lo : hi) + (int64_t)(jb + row) * 256 + piece * 16);
    }
  };
  auto commit = [&]() {
#pragma unroll
    for (int it = 0; it < 8; ++it) {
      const int idx = it * 256 + tid, half = idx >> 10, rem = idx & 1023, row = rem >> 4, piece = rem & 15;
      *reinterpret_cast<uint4 *>((half ? col_lo : col_hi) + row * LSTR + piece * 16) = pre[it];
    }
  };

  if (r0 < n_sent) fetch(r0);
  for (int jb = r0; jb < n_sent; jb += kColBlock) {
    commit();
    __syncthreads();
    if (jb + kColBlock < n_sent) fetch(jb + kColBlock);  // lands while this block is multiplied
#pragma unroll
    for (int ct = 0; ct < kColBlock / 16; ++ct) {
      const int cbase = jb + 16 * ct;
      if (cbase >= n_sent) continue;
      // both row tiles of the wave share the column fragments (one LDS read serves two products)
      bool live[kRowTiles];
      bool any_live = false;
#pragma unroll
      for (int t = 0; t < kRowTiles; ++t) {
        const int rt0 = rw0 + 16 * t;
        live[t] = !(cbase + 15 <= rt0 || rt0 >= n_sent);  // something right of the diagonal in this tile
        any_live |= live[t];
      }
      if (!any_live) continue;
      f32x4 acc[kRowTiles];
#pragma unroll
      for (int t = 0; t < kRowTiles; ++t) acc[t] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
      for (int kk = 0; kk < 4; ++kk) {
        const bf16x8 b_hi = *reinterpret_cast<const bf16x8 *>(col_hi + (16 * ct + c16) * LSTR + g * 64 + kk * 16);
        const bf16x8 b_lo = *reinterpret_cast<const bf16x8 *>(col_lo + (16 * ct + c16) * LSTR + g * 64 + kk * 16);
#pragma unroll
        for (int t = 0; t < kRowTiles; ++t) {
          acc[t] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a_lo[t][kk], b_hi, acc[t], 0, 0, 0);
          acc[t] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a_hi[t][kk], b_lo, acc[t], 0, 0, 0);
          acc[t] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a_hi[t][kk], b_hi, acc[t], 0, 0, 0);
        }
      }
      const int col = cbase + c16;
#pragma unroll
      for (int t = 0; t < kRowTiles; ++t) {
        if (!live[t]) continue;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
          const int row = rw0 + 16 * t + 4 * g + j;
          if (col > row && col < n_sent) rmax[t][j] = fmaxf(rmax[t][j], acc[t][j]);
        }
      }
    }
    __syncthreads();
  }

  // row maxima across the 16 column lanes, then the fused score of Eq. 6: lane c16 = 4t + j of
  // a lane group finishes row (tile t, register j), with the inputs it fetched at the start
#pragma unroll
  for (int t = 0; t < kRowTiles; ++t) {
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const float lam = row16_max(rmax[t][j]);
      if (c16 == 4 * t + j && my_row < n_sent) {
        float score = INFINITY;
        if (my_off < p_start) {
          score = a.sigma * my_imp;
          if (a.has_red) score -= (1.f - a.sigma) * my_red;
          if (lam > a.tau) score -= lam;
        }
        a.sent_lambda[col0 + my_row] = lam;
        a.sent_score[col0 + my_row] = score;
      }
    }
  }
}

}  // namespace

hipError_t launch_cosine(const CosineArgs &a, hipStream_t st) {
  const int64_t items = (int64_t)a.n_lh * a.ws.nrb_max;
  if (items == 0) return hipSuccess;
  const int64_t grid = (items + 7) / 8 * 8;
  hipLaunchKernelGGL(k_cosine, dim3((unsigned)grid), dim3(256), 0, st, a);
  return hipGetLastError();
}

}  // namespace skipkv

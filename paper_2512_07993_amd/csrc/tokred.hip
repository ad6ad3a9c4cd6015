// Token redundancy (Sec. 4.1 "Token Redundancy Score", Eq. 5): per head, with Kbar the rows of K
// scaled to unit length, R[t] = mean over rows i of softmax_j(Kbar Kbar^T)[i, t].
//
// The cosine matrix is symmetric and its entries lie in [-1, 1], so no running maximum is
// needed: with E = exp(Kbar Kbar^T), l = E 1 (row sums) and R = (1/N) E (1 / l).  Both are sums
// over the same symmetric N x N matrix, which is never stored:
//   sweep 1:  l_i = sum_j e_ij
//   sweep 2:  R_i = (1/N) sum_j e_ij / l_j
// with e_ij = exp2(<k_i, k_j> * c_i * c_j), where c = sqrt(log2 e) / (||k|| + eps) carries both the
// normalisation and the change of base.  The dot products run on the bf16 matrix cores with the
// RAW keys (exact products, fp32 accumulation; fp32 caches are rounded to bf16 first) and the
// scale factors are applied to the accumulators.
//
// Only the blocks at and right of the diagonal are computed.  One workgroup owns 256 rows (64 per
// wave: the A operands stay in registers) and walks the 64-column blocks from its own rows to the
// end of the sequence, staged through LDS and shared by the 4 waves; the next block is fetched
// into registers while the current one is multiplied.  The 256 x 256 square on the diagonal is
// computed in full and gives row sums only; every block right of it gives e_ij both to row i
// (weighted with column j's factor) and, by symmetry, to row j (weighted with row i's factor):
// the column sums of a block are reduced over the workgroup's rows and added to the row's total.
// Totals are accumulated across workgroups as 64-bit FIXED-POINT integers (integer addition is
// associative: the result does not depend on the order in which workgroups arrive, and the
// conversion of an fp32 partial sum is exact at the chosen scale for all but negligible terms),
// then turned back into fp32 by a small kernel after each sweep.
#include <algorithm>
#include <type_traits>

#include "common.h"

namespace skipkv {

namespace {

constexpr int kRows = kTokredRows;  // rows per workgroup
constexpr int kTW = kRows / 64;      // 16-row tiles per wave
constexpr int kCols = 64;      // columns per staged block
constexpr int LSTR = 272;      // bytes per staged key row (256 + 16: 16-byte reads of 8 rows hit distinct banks)
constexpr float kSqrtLog2e = 1.2011224087864498f;
// fixed-point scales of the two accumulations: row sums l <= e * N (2^40: room for N up to 2^21 tokens,
// resolution 1e-12 against terms >= 0.37), and R <= e^2 / N... <= 8 (2^50: resolution 1e-15 against R ~ 1/N)
constexpr float kFix1 = 1099511627776.f, kFix2 = 1125899906842624.f;

__device__ __forceinline__ void add_fixed(unsigned long long *dst, float x, float scale) {
  atomicAdd(dst, (unsigned long long)__float2ll_rn(x * scale));  // x >= 0
}

__device__ __forceinline__ uint32_t pack2(float lo, float hi) {  // two fp32 -> packed bf16, nearest even
  typedef __attribute__((__vector_size__(2 * sizeof(__bf16)))) __bf16 bf16x2_t;
  bf16x2_t v;
  v[0] = (__bf16)lo;
  v[1] = (__bf16)hi;
  return __builtin_bit_cast(uint32_t, v);
}

// 16 bytes of a key row as bf16: piece p (8 elements) of the row at `row_ptr`.
template <int DT>
__device__ __forceinline__ uint4 load_piece_bf16(const char *row_ptr, int piece) {
  if constexpr (DT == SKIPKV_BF16) {
    return *reinterpret_cast<const uint4 *>(row_ptr + piece * 16);
  } else {
    const float4 x = *reinterpret_cast<const float4 *>(row_ptr + piece * 32);
    const float4 y = *reinterpret_cast<const float4 *>(row_ptr + piece * 32 + 16);
    return make_uint4(pack2(x.x, x.y), pack2(x.z, x.w), pack2(y.x, y.y), pack2(y.z, y.w));
  }
}

// c[t] = sqrt(log2 e) / (||k_t|| + eps) for every key row; 16 lanes per row.
template <int DT>
__global__ void __launch_bounds__(256) k_key_scale(TokRedArgs a) {
  constexpr int ESZ = DT == SKIPKV_BF16 ? 2 : 4;
  const int lane16 = threadIdx.x & 15;
  const int64_t n_rows = (int64_t)a.n_layers * a.n_kv_heads * a.total_tokens;
  for (int64_t row = ((int64_t)blockIdx.x * 256 + threadIdx.x) >> 4; row < n_rows; row += ((int64_t)gridDim.x * 256) >> 4) {
    const int64_t lh = row / a.total_tokens, t = row % a.total_tokens;
    const int l = (int)(lh / a.n_kv_heads), h = (int)(lh % a.n_kv_heads);
    const int64_t slot = a.row_map ? (int64_t)a.row_map[t] : t;  // paged cache: the token's slot row
    const char *p = static_cast<const char *>(a.k) + ((int64_t)l * a.stride_layer + (int64_t)h * a.stride_head + slot * a.stride_tok) * ESZ;
    float ss = 0.f;
    if constexpr (DT == SKIPKV_BF16) {
      const uint4 v = *reinterpret_cast<const uint4 *>(p + lane16 * 16);
      const uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const float x = __uint_as_float(w[i] << 16), y = __uint_as_float(w[i] & 0xFFFF0000u);
        ss += x * x + y * y;
      }
    } else {
      // the dot products use the keys rounded to bf16: the norm is taken of the same values
      const uint4 v = load_piece_bf16<DT>(p, lane16);
      const uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const float x = __uint_as_float(w[i] << 16), y = __uint_as_float(w[i] & 0xFFFF0000u);
        ss += x * x + y * y;
      }
    }
    ss = row16_sum(ss);
    if (lane16 == 0) {
      a.scale[row] = kSqrtLog2e / (sqrtf(ss) + 1e-12f);
      a.acc[row] = 0ull;  // the first sweep's accumulator
    }
  }
}

// SWEEP 1: adds every row's sum of e_ij into acc (scale kFix1).  SWEEP 2: adds R (scale kFix2).
template <int DT, int SWEEP>
__global__ void __launch_bounds__(256, kTW == 4 ? 2 : 3) k_tokred_sweep(TokRedArgs a) {
  constexpr int ESZ = DT == SKIPKV_BF16 ? 2 : 4;
  constexpr float kFix = SWEEP == 1 ? kFix1 : kFix2;
  __shared__ __align__(16) char cols[kCols * LSTR];
  __shared__ float col_c[kCols];     // scale factor of each staged column
  __shared__ float col_w[kCols];     // weight of each staged column in a row's sum: 1 (sweep 1), 1 / l (sweep 2)
  __shared__ float cpart[2][4][kCols];  // [block parity]: column sums of a block over each wave's rows

  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63, c16 = lane & 15, g = lane >> 4;
  // ---- which (head, sequence, row block) is this?
  const uint32_t item = xcd_contiguous_item(blockIdx.x, gridDim.x);
  if (item >= (uint32_t)a.n_layers * a.n_kv_heads * (uint32_t)a.nrb_max) return;
  const int lh = item / a.nrb_max;
  int j = item % a.nrb_max, b = 0, n_tok = 0, tok0 = 0;
  for (; b < a.batch; ++b) {
    tok0 = a.seq_off[b];
    n_tok = a.seq_off[b + 1] - tok0;
    const int cnt = (n_tok + kRows - 1) / kRows;
    if (j < cnt) break;
    j -= cnt;
  }
  if (b >= a.batch) return;
  const int r0 = j * kRows;
  if (a.len) n_tok = min(n_tok, a.len[lh * a.batch + b]);  // per-head ranges: the head's own length within the sequence's room
  if (r0 >= n_tok) return;
  const int l = lh / a.n_kv_heads, h = lh % a.n_kv_heads;
  // paged cache: rows are looked up in the row map (slot rows from the head's base), else they follow tok0
  const int32_t *rmap = a.row_map ? a.row_map + tok0 : nullptr;
  const char *kbase = static_cast<const char *>(a.k) + ((int64_t)l * a.stride_layer + (int64_t)h * a.stride_head + (rmap ? 0 : (int64_t)tok0 * a.stride_tok)) * ESZ;
  const int64_t pitch = a.stride_tok * ESZ;
  auto slot_of = [&](int row) -> int64_t { return rmap ? (int64_t)rmap[row] : (int64_t)row; };
  const int64_t col0 = (int64_t)lh * a.total_tokens + tok0;  // index of the sequence's first token in the per-token arrays

  // ---- A operands: this wave's 64 rows (4 tiles), lane (row c16 of a tile, head-dim slice g)
  const int rw0 = r0 + 16 * kTW * wave;
  bf16x8 af[kTW][4];
  float row_c[kTW][4];  // scale factors of the lane's output rows (rows 4g+j of every tile)
  float row_w[kTW][4];  // their weights in a column's sum (0 for rows past the end)
#pragma unroll
  for (int t = 0; t < kTW; ++t) {
    const int row = min(rw0 + 16 * t + c16, n_tok - 1);
    const int64_t srow = slot_of(row);
#pragma unroll
    for (int kk = 0; kk < 4; ++kk) af[t][kk] = __builtin_bit_cast(bf16x8, load_piece_bf16<DT>(kbase + srow * pitch, 4 * g + kk));
#pragma unroll
    for (int jj = 0; jj < 4; ++jj) {
      const int r = rw0 + 16 * t + 4 * g + jj;
      row_c[t][jj] = a.scale[col0 + min(r, n_tok - 1)];
      row_w[t][jj] = r < n_tok ? (SWEEP == 1 ? 1.f : a.inv_l[col0 + r]) : 0.f;
    }
  }
  float rsum[kTW][4];
#pragma unroll
  for (int t = 0; t < kTW; ++t)
#pragma unroll
    for (int jj = 0; jj < 4; ++jj) rsum[t][jj] = 0.f;
  const float inv_n = SWEEP == 1 ? 1.f : 1.f / (float)n_tok;

  // a column block is 64 rows x 16 pieces of 16 bytes: 4 pieces per thread
  uint4 pre[4];
  float pre_c = 0.f, pre_w = 0.f;
  auto fetch = [&](int jb) {
#pragma unroll
    for (int it = 0; it < 4; ++it) {
      const int idx = it * 256 + tid, row = min(jb + (idx >> 4), n_tok - 1), piece = idx & 15;
      pre[it] = load_piece_bf16<DT>(kbase + slot_of(row) * pitch, piece);
    }
    if (tid < kCols) {
      const int col = jb + tid;
      pre_c = a.scale[col0 + min(col, n_tok - 1)];
      pre_w = col < n_tok ? (SWEEP == 1 ? 1.f : a.inv_l[col0 + col]) : 0.f;  // weight 0 drops columns past the end
    }
  };
  auto commit = [&]() {
#pragma unroll
    for (int it = 0; it < 4; ++it) {
      const int idx = it * 256 + tid, row = idx >> 4, piece = idx & 15;
      *reinterpret_cast<uint4 *>(cols + row * LSTR + piece * 16) = pre[it];
    }
    if (tid < kCols) {
      col_c[tid] = pre_c;
      col_w[tid] = pre_w;
    }
  };

  // The column sums of block jb are added to the totals one block later, right after the next fetch has
  // been issued: the atomics then travel during that block's products, and the wait for the fetched
  // columns (which waits for everything this thread has in flight) finds them done.
  auto emit = [&](int jb, int buf) {
    if (jb >= r0 + kRows && tid < kCols && jb + tid < n_tok) {
      const float tot = ((cpart[buf][0][tid] + cpart[buf][1][tid]) + cpart[buf][2][tid]) + cpart[buf][3][tid];
      add_fixed(a.acc + col0 + jb + tid, tot * inv_n, kFix);
    }
  };
  fetch(r0);
  int buf = 0;
  for (int jb = r0; jb < n_tok; jb += kCols, buf ^= 1) {
    commit();
    __syncthreads();
    if (jb + kCols < n_tok) fetch(jb + kCols);  // lands while this block is multiplied
    if (jb > r0) emit(jb - kCols, buf ^ 1);
    const bool mirror = jb >= r0 + kRows;       // right of the diagonal square: the block also stands for its transpose
    auto products = [&](auto mirror_c) {
      constexpr bool MIRROR = decltype(mirror_c)::value;
#pragma unroll
      for (int ct = 0; ct < kCols / 16; ++ct) {
        const int cbase = jb + 16 * ct;
        if (cbase >= n_tok) continue;
        bf16x8 bfr[4];
#pragma unroll
        for (int kk = 0; kk < 4; ++kk) bfr[kk] = *reinterpret_cast<const bf16x8 *>(cols + (16 * ct + c16) * LSTR + (4 * g + kk) * 16);
        const float cc = col_c[16 * ct + c16];
        const float cw = col_w[16 * ct + c16];
        float csum[4] = {0.f, 0.f, 0.f, 0.f};  // the lane's column over the wave's rows: four independent chains
#pragma unroll
        for (int t = 0; t < kTW; ++t) {
          f32x4 acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
          for (int kk = 0; kk < 4; ++kk) acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(af[t][kk], bfr[kk], acc, 0, 0, 0);
#pragma unroll
          for (int jj = 0; jj < 4; ++jj) {
            const float e = __builtin_amdgcn_exp2f(acc[jj] * (row_c[t][jj] * cc));
            rsum[t][jj] = fmaf(e, cw, rsum[t][jj]);
            if constexpr (MIRROR) csum[jj] = fmaf(e, row_w[t][jj], csum[jj]);
          }
        }
        if constexpr (MIRROR) {
          // the four lane groups hold different rows of the same column
          float v = (csum[0] + csum[1]) + (csum[2] + csum[3]);
          v += __shfl_xor(v, 16);
          v += __shfl_xor(v, 32);
          if (g == 0) cpart[buf][wave][16 * ct + c16] = v;
        }
      }
    };
    if (rw0 < n_tok) {
      if (mirror) products(std::true_type{});
      else products(std::false_type{});
    } else if (mirror && g == 0) {  // a wave without rows adds nothing to the columns
#pragma unroll
      for (int ct = 0; ct < kCols / 16; ++ct) cpart[buf][wave][16 * ct + c16] = 0.f;
    }
    __syncthreads();  // (a cpart buffer is written again two blocks later, behind two more barriers)
  }
  {
    const int last = r0 + (n_tok - 1 - r0) / kCols * kCols;
    emit(last, ((last - r0) / kCols) & 1);
  }

  // ---- sums across the 16 column lanes, then the rows' share of their totals
#pragma unroll
  for (int t = 0; t < kTW; ++t) {
#pragma unroll
    for (int jj = 0; jj < 4; ++jj) {
      const float s = row16_sum(rsum[t][jj]);
      const int row = rw0 + 16 * t + 4 * g + jj;
      if (c16 == 0 && row < n_tok) add_fixed(a.acc + col0 + row, s * inv_n, kFix);
    }
  }
}

// After sweep 1: inv_l = 1 / l, accumulator cleared for sweep 2.  After sweep 2: R.  Entries that no row
// contributed to (beyond a head's own length) stay as they are.
template <int SWEEP>
__global__ void __launch_bounds__(256) k_tokred_finish(TokRedArgs a) {
  const int64_t n = (int64_t)a.n_layers * a.n_kv_heads * a.total_tokens;
  for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < n; i += (int64_t)gridDim.x * 256) {
    const unsigned long long v = a.acc[i];
    if (v == 0ull) continue;
    if (SWEEP == 1) {
      a.inv_l[i] = 1.f / ((float)v * (1.f / kFix1));
      a.acc[i] = 0ull;
    } else {
      a.out[i] = (float)v * (1.f / kFix2);
    }
  }
}

}  // namespace

hipError_t launch_token_redundancy(const TokRedArgs &a, hipStream_t st) {
  const int64_t n_lh = (int64_t)a.n_layers * a.n_kv_heads;
  if (n_lh == 0 || a.total_tokens == 0 || a.batch == 0) return hipSuccess;
  const int64_t rows = n_lh * a.total_tokens;
  const unsigned g0 = (unsigned)std::min<int64_t>((rows + 15) / 16, 1 << 16);
  const int64_t items = n_lh * a.nrb_max;
  const unsigned g1 = (unsigned)((items + 7) / 8 * 8);
  const unsigned g2 = (unsigned)std::min<int64_t>((rows + 255) / 256, 1 << 16);
  if (a.dtype == SKIPKV_BF16) {
    hipLaunchKernelGGL(k_key_scale<SKIPKV_BF16>, dim3(g0), dim3(256), 0, st, a);
    hipLaunchKernelGGL((k_tokred_sweep<SKIPKV_BF16, 1>), dim3(g1), dim3(256), 0, st, a);
    hipLaunchKernelGGL(k_tokred_finish<1>, dim3(g2), dim3(256), 0, st, a);
    hipLaunchKernelGGL((k_tokred_sweep<SKIPKV_BF16, 2>), dim3(g1), dim3(256), 0, st, a);
    hipLaunchKernelGGL(k_tokred_finish<2>, dim3(g2), dim3(256), 0, st, a);
  } else {
    hipLaunchKernelGGL(k_key_scale<SKIPKV_F32>, dim3(g0), dim3(256), 0, st, a);
    hipLaunchKernelGGL((k_tokred_sweep<SKIPKV_F32, 1>), dim3(g1), dim3(256), 0, st, a);
    hipLaunchKernelGGL(k_tokred_finish<1>, dim3(g2), dim3(256), 0, st, a);
    hipLaunchKernelGGL((k_tokred_sweep<SKIPKV_F32, 2>), dim3(g1), dim3(256), 0, st, a);
    hipLaunchKernelGGL(k_tokred_finish<2>, dim3(g2), dim3(256), 0, st, a);
  }
  return hipGetLastError();
}

}  // namespace skipkv

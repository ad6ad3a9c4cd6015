// Sentence similarity from the last layer's hidden states (Sec. 4.1 "Sentence Similarity Score",
// Eq. 1-3 as printed): v_s = mean of H over the tokens of sentence s, lambda_s = largest cosine
// with a later sentence, computed once per sequence and shared by all layers and heads - and
// the scores of Eq. 6 with that shared lambda, so that the per-head key pooling and Gram
// matrices drop out of the step.
#include <algorithm>

#include "common.h"

namespace skipkv {

namespace {

constexpr int LSTR = 272;  // bytes per staged 128-dim slice of an embedding (256 + 16: 16-byte reads of 8 rows hit distinct banks)

// sequence of sentence column c (columns of sequence b are [sent_ptr[b] - b, sent_ptr[b+1] - (b+1)))
__device__ __forceinline__ int seq_of_column(const int32_t *sent_ptr, int batch, int c) {
  int lo = 0, hi = batch - 1;  // invariant: first column of lo <= c
  while (lo < hi) {
    const int mid = (lo + hi + 1) >> 1;
    if (sent_ptr[mid] - mid <= c) lo = mid; else hi = mid - 1;
  }
  return lo;
}

// One workgroup per sentence: mean of the hidden-state rows, unit vector as bf16 hi + lo.
// d_model is a multiple of 8; the mean is scale-free under the normalisation, so the sum is
// normalised with eps scaled by the length.
template <int DT>
__global__ void __launch_bounds__(256) k_hidden_pool(HiddenSimArgs a) {
  constexpr int ESZ = DT == SKIPKV_BF16 ? 2 : 4;
  __shared__ float red[4];
  const int c = blockIdx.x, tid = threadIdx.x;
  const int b = seq_of_column(a.sent_ptr, a.batch, c);
  const int s = c - (a.sent_ptr[b] - b);
  const int32_t *off = a.sent_off + a.sent_ptr[b];
  // offsets are clamped to the sequence: this entry point does not run the plan's validation
  const int n_tok = a.seq_off[b + 1] - a.seq_off[b];
  const int o0 = min(max(off[s], 0), n_tok), o1 = min(max(off[s + 1], o0), n_tok);
  const int t0 = a.seq_off[b] + o0, t1 = a.seq_off[b] + o1;
  const char *h = static_cast<const char *>(a.hidden);
  const int64_t pitch = (int64_t)a.d_model * ESZ;
  float ssq = 0.f;
  // every thread owns groups of 8 columns: tid, tid + 256, ...; sums are kept in the output row (fp32 scratch) between the two passes
  float *sum_row = a.sum_scratch + (int64_t)c * a.d_model;
  for (int g8 = tid; g8 * 8 < a.d_model; g8 += 256) {
    float acc[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
#pragma unroll 4
    for (int t = t0; t < t1; ++t) {
      const char *p = h + t * pitch + (int64_t)g8 * 8 * ESZ;
      if constexpr (DT == SKIPKV_BF16) {
        const uint4 v = *reinterpret_cast<const uint4 *>(p);
        const uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          acc[2 * i] += __uint_as_float(w[i] << 16);
          acc[2 * i + 1] += __uint_as_float(w[i] & 0xFFFF0000u);
        }
      } else {
        const float4 v0 = *reinterpret_cast<const float4 *>(p), v1 = *reinterpret_cast<const float4 *>(p + 16);
        acc[0] += v0.x; acc[1] += v0.y; acc[2] += v0.z; acc[3] += v0.w;
        acc[4] += v1.x; acc[5] += v1.y; acc[6] += v1.z; acc[7] += v1.w;
      }
    }
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      ssq = fmaf(acc[i], acc[i], ssq);
      sum_row[g8 * 8 + i] = acc[i];
    }
  }
  ssq = wave_sum(ssq);
  if ((tid & 63) == 0) red[tid >> 6] = ssq;
  __syncthreads();
  const float inv = 1.f / (sqrtf(red[0] + red[1] + red[2] + red[3]) + 1e-12f * (float)(t1 - t0));
  if (tid == 0) a.sent_lambda[c] = -INFINITY;  // the Gram kernel folds its row maxima into this
  uint16_t *hi = a.vhat_hi + (int64_t)c * a.d_model, *lo = a.vhat_lo + (int64_t)c * a.d_model;
  for (int g8 = tid; g8 * 8 < a.d_model; g8 += 256) {
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      const float u = sum_row[g8 * 8 + i] * inv;  // written by this thread above
      const uint32_t hb = f32_to_bf16_bits(u);
      hi[g8 * 8 + i] = (uint16_t)hb;
      lo[g8 * 8 + i] = (uint16_t)f32_to_bf16_bits(u - bf16_bits_to_f32(hb));
    }
  }
}

// atomic max on a float that may be negative (order of the bit patterns: ints for >= 0, reversed uints for < 0)
__device__ __forceinline__ void atomic_max_float(float *addr, float v) {
  if (v >= 0.f)
    atomicMax(reinterpret_cast<int *>(addr), __float_as_int(v));
  else
    atomicMin(reinterpret_cast<unsigned int *>(addr), __float_as_uint(v));
}

// One 64 x 64 block of a sequence's Gram matrix at or right of the diagonal: accumulated over the
// 128-dim slices of the embedding (A and B slices staged through LDS, bf16 hi + lo, three products
// per slice step as in the per-head kernel), then folded into the row maxima (lambda, preset to
// -inf by the pooling kernel) with atomics, so that all blocks of a sequence run side by side.
__global__ void __launch_bounds__(256) k_cosine_wide(HiddenSimArgs a) {
  __shared__ __align__(16) char sa_hi[64 * LSTR], sa_lo[64 * LSTR], sb_hi[64 * LSTR], sb_lo[64 * LSTR];
  const int b = blockIdx.x;
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63, c16 = lane & 15, g = lane >> 4;
  const int sp = a.sent_ptr[b];
  const int n_sent = min(a.sent_ptr[b + 1] - sp - 1, SKIPKV_MAX_SENTENCES);
  const int nb = (n_sent + 63) / 64;
  // blockIdx.y enumerates the pairs (rb, cb), cb >= rb, row by row
  int rb = 0, rest = blockIdx.y;
  while (rb < nb && rest >= nb - rb) {
    rest -= nb - rb;
    ++rb;
  }
  if (rb >= nb) return;
  const int r0 = 64 * rb, jb = 64 * (rb + rest);
  const int64_t col0 = sp - b;
  const char *hi = reinterpret_cast<const char *>(a.vhat_hi + col0 * a.d_model);
  const char *lo = reinterpret_cast<const char *>(a.vhat_lo + col0 * a.d_model);
  const int64_t pitch = (int64_t)a.d_model * 2;
  auto stage = [&](char *dst_hi, char *dst_lo, int row0, int d0) {  // 64 rows x 128 dims, hi and lo: 8 pieces of 16 bytes per thread
#pragma unroll
    for (int it = 0; it < 8; ++it) {
      const int idx = it * 256 + tid, half = idx >> 10, rem = idx & 1023, row = rem >> 4, piece = rem & 15;
      uint4 v = make_uint4(0, 0, 0, 0);
      if (row0 + row < n_sent) v = *reinterpret_cast<const uint4 *>((half ? lo : hi) + (row0 + row) * pitch + (int64_t)d0 * 2 + piece * 16);
      *reinterpret_cast<uint4 *>((half ? dst_lo : dst_hi) + row * LSTR + piece * 16) = v;
    }
  };
  f32x4 acc[4];
#pragma unroll
  for (int ct = 0; ct < 4; ++ct) acc[ct] = f32x4{0.f, 0.f, 0.f, 0.f};
  for (int d0 = 0; d0 < a.d_model; d0 += 128) {
    __syncthreads();  // the previous slice is consumed
    stage(sa_hi, sa_lo, r0, d0);
    stage(sb_hi, sb_lo, jb, d0);
    __syncthreads();
#pragma unroll
    for (int kk = 0; kk < 4; ++kk) {
      const bf16x8 a_hi = *reinterpret_cast<const bf16x8 *>(sa_hi + (16 * wave + c16) * LSTR + g * 64 + kk * 16);
      const bf16x8 a_lo = *reinterpret_cast<const bf16x8 *>(sa_lo + (16 * wave + c16) * LSTR + g * 64 + kk * 16);
#pragma unroll
      for (int ct = 0; ct < 4; ++ct) {
        const bf16x8 b_hi = *reinterpret_cast<const bf16x8 *>(sb_hi + (16 * ct + c16) * LSTR + g * 64 + kk * 16);
        const bf16x8 b_lo = *reinterpret_cast<const bf16x8 *>(sb_lo + (16 * ct + c16) * LSTR + g * 64 + kk * 16);
        acc[ct] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a_lo, b_hi, acc[ct], 0, 0, 0);
        acc[ct] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a_hi, b_lo, acc[ct], 0, 0, 0);
        acc[ct] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a_hi, b_hi, acc[ct], 0, 0, 0);
      }
    }
  }
  float rmax[4] = {-INFINITY, -INFINITY, -INFINITY, -INFINITY};
#pragma unroll
  for (int ct = 0; ct < 4; ++ct) {
    const int col = jb + 16 * ct + c16;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const int row = r0 + 16 * wave + 4 * g + j;
      if (col > row && col < n_sent) rmax[j] = fmaxf(rmax[j], acc[ct][j]);
    }
  }
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    const float lam = row16_max(rmax[j]);
    const int row = r0 + 16 * wave + 4 * g + j;
    if (c16 == 0 && row < n_sent && lam > -INFINITY) atomic_max_float(&a.sent_lambda[col0 + row], lam);
  }
}

// Eq. 6 per (layer, head, sentence) with the sequence's shared lambda.
__global__ void __launch_bounds__(256) k_fuse_shared(FuseSharedArgs a) {
  const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (i >= (int64_t)a.n_lh * a.total_sentences) return;
  const int c = (int)(i % a.total_sentences);
  const int b = seq_of_column(a.sent_ptr, a.batch, c);
  const int sp = a.sent_ptr[b];
  const int s = c - (sp - b);
  if (s >= min(seq_sentences(a.sent_ptr, a.cnt, b), a.sent_ptr[b + 1] - sp - 1)) return;  // per-head ranges: beyond the head's sentences
  const int n_tok = min(seq_tokens(a.seq_off, a.len, b), a.seq_off[b + 1] - a.seq_off[b]);
  const int p_start = n_tok - min(a.protect, n_tok);
  float lam;
  if (a.sent_id) {  // the sentence's number in its sequence's own list
    const int rb = b % a.virt_b, id = a.sent_id[c];
    const int lp = a.lam_ptr[rb], ln = a.lam_ptr[rb + 1] - lp;
    if (id >= 0 && id < ln) {
      lam = a.shared_lambda[lp + id];
    } else {
      lam = -INFINITY;
      if (a.dev_status) atomicOr(a.dev_status, SKIPKV_DEV_BAD_OFFSETS);
    }
  } else {
    lam = a.shared_lambda[c];
  }
  float score = INFINITY;
  if (a.sent_off[sp + s] < p_start) {
    score = a.sigma * a.sent_imp[i];
    if (a.has_red) score -= (1.f - a.sigma) * a.sent_red[i];
    if (lam > a.tau) score -= lam;
  }
  a.sent_score[i] = score;
  if (a.sent_lambda) a.sent_lambda[i] = lam;
}

}  // namespace

hipError_t launch_hidden_similarity(const HiddenSimArgs &a, hipStream_t st) {
  if (a.total_sentences == 0 || a.batch == 0) return hipSuccess;
  if (a.dtype == SKIPKV_BF16)
    hipLaunchKernelGGL(k_hidden_pool<SKIPKV_BF16>, dim3(a.total_sentences), dim3(256), 0, st, a);
  else
    hipLaunchKernelGGL(k_hidden_pool<SKIPKV_F32>, dim3(a.total_sentences), dim3(256), 0, st, a);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  // a sequence has at most min(total_sentences, SKIPKV_MAX_SENTENCES) sentences: that many 64-row blocks, all pairs of them
  const int nb = (std::min(a.total_sentences, SKIPKV_MAX_SENTENCES) + 63) / 64;
  hipLaunchKernelGGL(k_cosine_wide, dim3(a.batch, nb * (nb + 1) / 2), dim3(256), 0, st, a);
  return hipGetLastError();
}

hipError_t launch_fuse_shared(const FuseSharedArgs &a, hipStream_t st) {
  const int64_t n = (int64_t)a.n_lh * a.total_sentences;
  if (n == 0) return hipSuccess;
  hipLaunchKernelGGL(k_fuse_shared, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, st, a);
  return hipGetLastError();
}

}  // namespace skipkv

// Paged KV cache (Appendix, "System-Level Evaluation on vLLM"): the translation from logical
// tokens to block slots, done once per step for the whole batch.  The kernels that touch K and V
// then address rows through this map instead of through the block table.
#include "common.h"

namespace skipkv {

__global__ void k_row_map_reset(int32_t *seq_bad, int n) {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) seq_bad[i] = 0;
}

// grid = (x, batch, n_lh): the blocks of column (b, lh) walk the tokens of sequence b.
__global__ void __launch_bounds__(256) k_row_map(RowMapArgs a) {
  const int b = blockIdx.y, lh = blockIdx.z;
  const int tok0 = a.seq_off[b], n_tok = a.seq_off[b + 1] - tok0;
  const int32_t *table = a.block_table + (int64_t)b * a.table_stride;
  const int64_t head_row = (int64_t)(lh / a.n_kv_heads) * a.unit_layer + (int64_t)(lh % a.n_kv_heads) * a.unit_head;
  int32_t *out = a.row_map + (int64_t)lh * a.total_tokens + tok0;
  bool bad = false;
  for (int t = blockIdx.x * 256 + threadIdx.x; t < n_tok; t += gridDim.x * 256) {
    const int bi = t / a.block_size;
    int p = bi < a.table_stride ? table[bi] : -1;
    if (p < 0 || p >= a.n_blocks) {
      bad = true;
      p = 0;
    }
    out[t] = (int32_t)(head_row + p * a.unit_block + (t - bi * a.block_size) * a.unit_tok);
  }
  if (__any(bad) && (threadIdx.x & 63) == 0) {
    a.seq_bad[lh * a.batch + b] = 1;  // every writer stores the same value
    if (a.dev_status) atomicOr(a.dev_status, SKIPKV_DEV_BAD_BLOCK_TABLE);
  }
}

hipError_t launch_row_map(const RowMapArgs &a, hipStream_t st) {
  if (a.batch == 0 || a.n_lh == 0) return hipSuccess;
  const int n_flags = a.n_lh * a.batch;
  hipLaunchKernelGGL(k_row_map_reset, dim3((n_flags + 255) / 256), dim3(256), 0, st, a.seq_bad, n_flags);
  hipLaunchKernelGGL(k_row_map, dim3(a.n_lh > 1 ? 8 : 64, a.batch, a.n_lh), dim3(256), 0, st, a);
  return hipGetLastError();
}

}  // namespace skipkv

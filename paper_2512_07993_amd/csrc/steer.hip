// Steering injection (Sec. 4.2): H_k <- H_k + alpha_t * v on the rows whose current token is a
// sentence delimiter.  The sum is formed in fp64 (exact for bf16/fp32 inputs up to the final
// addition) and rounded once, to nearest even, to the storage type.
#include "common.h"

namespace skipkv {

namespace {

// double -> bf16 bits with a single round-to-nearest-even (finite inputs).
__device__ __forceinline__ uint32_t f64_to_bf16_bits(double y) {
  const double ay = fabs(y);
  double r;
  if (ay < 1.1754943508222875e-38) {  // below the smallest normal: bf16 subnormals are multiples of 2^-133
    r = rint(y * 0x1p133) * 0x1p-133;
  } else {
    unsigned long long u = (unsigned long long)__double_as_longlong(y);
    const unsigned long long lsb = (u >> 45) & 1ull;  // bf16 keeps 7 of the 52 fraction bits
    u += ((1ull << 44) - 1ull) + lsb;
    u &= ~((1ull << 45) - 1ull);
    r = __longlong_as_double((long long)u);
  }
  return __float_as_uint((float)r) >> 16;  // r is exactly representable: the conversion is exact
}

template <int DT>
__global__ void __launch_bounds__(256) k_steer(SteerArgs a) {
  const int row = blockIdx.y;
  if (a.row_mask && !a.row_mask[row]) return;
  const double c = (double)(a.coef ? a.coef[row] : a.coef_scalar);
  const int col = blockIdx.x * 256 + threadIdx.x;
  if (col >= a.d_model) return;
  const int64_t o = (int64_t)row * a.d_model + col;
  if constexpr (DT == SKIPKV_BF16) {
    uint16_t *h = static_cast<uint16_t *>(a.hidden);
    const uint16_t *v = static_cast<const uint16_t *>(a.vec);
    const double y = (double)bf16_bits_to_f32(h[o]) + c * (double)bf16_bits_to_f32(v[col]);
    h[o] = (uint16_t)f64_to_bf16_bits(y);
  } else {
    float *h = static_cast<float *>(a.hidden);
    const float *v = static_cast<const float *>(a.vec);
    h[o] = (float)((double)h[o] + c * (double)v[col]);
  }
}

// Adaptive strength (Sec. 4.2): alpha_t = alpha_0 + gamma * N_o per sample, N_o the running
// count of non-execution thoughts.  One rounding (fused multiply-add).
__global__ void __launch_bounds__(256) k_steer_strength(const int32_t *n_nonexec, float alpha0, float gamma, float *coef, int rows) {
  const int i = blockIdx.x * 256 + threadIdx.x;
  if (i < rows) coef[i] = fmaf(gamma, (float)n_nonexec[i], alpha0);
}

}  // namespace

hipError_t launch_steer_strength(const int32_t *n_nonexec, float alpha0, float gamma, float *coef, int32_t rows, hipStream_t st) {
  if (rows == 0) return hipSuccess;
  hipLaunchKernelGGL(k_steer_strength, dim3((rows + 255) / 256), dim3(256), 0, st, n_nonexec, alpha0, gamma, coef, rows);
  return hipGetLastError();
}

hipError_t launch_steer(const SteerArgs &a, hipStream_t st) {
  if (a.rows == 0 || a.d_model == 0) return hipSuccess;
  const dim3 grid((a.d_model + 255) / 256, a.rows);
  if (a.dtype == SKIPKV_BF16)
    hipLaunchKernelGGL(k_steer<SKIPKV_BF16>, grid, dim3(256), 0, st, a);
  else
    hipLaunchKernelGGL(k_steer<SKIPKV_F32>, grid, dim3(256), 0, st, a);
  return hipGetLastError();
}

}  // namespace skipkv

// Device-side helpers shared by the single-pass scan kernels: coherent cross-workgroup
// accesses, counted waits, direct HBM -> LDS loads, DPP reductions.
#pragma once

#include "scan_common.h"

namespace skipkv {

typedef __attribute__((__vector_size__(2 * sizeof(__bf16)))) __bf16 bf16x2_t;

// Cross-workgroup communication (the workgroups may sit on different XCDs, whose L2 caches are not
// coherent with each other).  Everything that is communicated - the statistics records of the items, the
// abort word - is accessed ONLY with device-scope relaxed atomics, which are coherent by themselves.
// A record is ONE 8-byte store and carries its own validity (its first word holds a marker until it is
// written), so readers need no ordering between words and writers need no fence or flag.  No device-scope
// fence is used: on this chip such a fence writes back and invalidates a whole L2, which is ruinous when
// thousands of workgroups do it.
__device__ __forceinline__ void coherent_store2(float2 *p, float2 v) {
  unsigned long long u = (unsigned long long)__float_as_uint(v.x) | ((unsigned long long)__float_as_uint(v.y) << 32);
  __hip_atomic_store(reinterpret_cast<unsigned long long *>(p), u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ float2 coherent_load2(const float2 *p) {
  const unsigned long long u =
      __hip_atomic_load(reinterpret_cast<const unsigned long long *>(p), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  return make_float2(__uint_as_float((uint32_t)u), __uint_as_float((uint32_t)(u >> 32)));
}

// s_waitcnt immediates (gfx9 encoding: vmcnt[3:0] | expcnt[6:4] | lgkmcnt[11:8] | vmcnt[5:4] << 14)
// A copy of a per-thread value that the compiler cannot trace back to its source: address parts
// derived from it are computed where they are used instead of being kept in registers (or in
// scratch, whose reloads would wait for every key load in flight) across a whole item.
__device__ __forceinline__ int opaque(int x) {
  asm volatile("" : "+v"(x));
  return x;
}

template <int N>
__device__ __forceinline__ void wait_vm() {  // at most N vector-memory operations still outstanding
  __builtin_amdgcn_s_waitcnt((N & 0xF) | (0x7 << 4) | (0xF << 8) | ((N >> 4) << 14));
}
__device__ __forceinline__ void wait_all() { __builtin_amdgcn_s_waitcnt(0); }
// Workgroup barrier for data exchanged through LDS: waits for this wave's LDS operations only, so
// that key loads already in flight for later stages are not drained (a __syncthreads() would).
__device__ __forceinline__ void lds_barrier() {
  __builtin_amdgcn_s_waitcnt(0xC07F);  // lgkmcnt(0)
  __builtin_amdgcn_s_barrier();
}

// Direct HBM -> LDS load: every lane fetches 16 bytes from its own global address; the wave's 64
// pieces land at wave_lds_base + lane * 16 (the base travels in M0).  Issued through inline
// assembly on purpose: the compiler orders LDS reads against direct loads it knows about by
// waiting for ALL of them, which would drain the ring of stages on every read; here the stages
// are ordered by hand with wait_vm<>() (loads complete in issue order).  Nothing else in this
// kernel uses M0.
__device__ __forceinline__ void load_to_lds_16(const void *gsrc, void *wave_lds_base) {
  const uint32_t l = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) char *)wave_lds_base;
  asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, off" ::"s"(l), "v"(gsrc) : "memory");
}

// (lo, hi) fp32 -> packed bf16 pair, round to nearest even (v_cvt_pk_bf16_f32).
__device__ __forceinline__ uint32_t pack_bf16x2(float lo, float hi) {
  bf16x2_t v;
  v[0] = (__bf16)lo;
  v[1] = (__bf16)hi;
  return __builtin_bit_cast(uint32_t, v);
}

__device__ __forceinline__ uint32_t lds_addr(const void *p) {
  return (uint32_t)(uintptr_t)(const __attribute__((address_space(3))) char *)p;
}
__device__ __forceinline__ float lds_read_f32(uint32_t addr) {
  return *(const __attribute__((address_space(3))) float *)(uintptr_t)addr;
}

// Row (16-lane) reductions with the DPP modifier on the arithmetic instruction itself: one
// instruction per step.  The s_nop covers the two wait states a DPP read needs after a VALU write.
#define SKIPKV_DPP_STEP(OP, N)                                                                          \
  asm volatile("s_nop 1\n\t" OP " %0, %1, %1 row_ror:" #N " row_mask:0xf bank_mask:0xf" : "=v"(v) : "v"(v))
__device__ __forceinline__ float row16_max_fast(float v) {
  SKIPKV_DPP_STEP("v_max_f32_dpp", 8);
  SKIPKV_DPP_STEP("v_max_f32_dpp", 4);
  SKIPKV_DPP_STEP("v_max_f32_dpp", 2);
  SKIPKV_DPP_STEP("v_max_f32_dpp", 1);
  return v;
}
__device__ __forceinline__ float row16_sum_fast(float v) {
  SKIPKV_DPP_STEP("v_add_f32_dpp", 8);
  SKIPKV_DPP_STEP("v_add_f32_dpp", 4);
  SKIPKV_DPP_STEP("v_add_f32_dpp", 2);
  SKIPKV_DPP_STEP("v_add_f32_dpp", 1);
  return v;
}
#undef SKIPKV_DPP_STEP

}  // namespace skipkv

// Single-pass key scan (Sec. 4.1 "Token Importance Score", Eq. 4; sentence embedding of Eq. 2
// over the head's keys): K is read from HBM exactly once.
//
// The softmax normaliser of a query row needs all N keys of the head, which are spread over many
// chunks, i.e. many workgroups.  Instead of a second pass over K, every workgroup keeps the
// logits of its chunk in registers (they are MFMA accumulators anyway: 64 tokens per wave x all
// query rows of the GQA group), publishes its chunk's (max, sum exp) per row, and waits until the
// head's normalisers are final; the last chunk of a head to arrive merges the partials and
// raises the head's ready flag.  Then each workgroup finishes I[t] from its registers.
//
// Forward progress.  The grid is persistent and no larger than what is co-resident on the chip
// (occupancy query on the host).  Workgroup w takes items w, w+G, w+2G, ... in increasing order,
// items being (head, chunk) pairs with a head's chunks consecutive.  A workgroup only ever waits
// for the head of the item it has just published.  Since a head has at most kFuseMaxChunks <= G
// chunks, its chunks belong to distinct workgroups, each of which reaches its chunk of that head
// without waiting on that head first; by induction over heads in item order every wait ends.
// The wait is bounded anyway (spin_limit polls): on expiry SKIPKV_DEV_TIMEOUT is raised and the
// kernel runs to completion with invalid scores rather than hanging.
//
// Inside a workgroup the 4 waves are independent streams: wave w owns tokens [64w, 64w+64) of the
// chunk, stages its own rows HBM -> registers -> its private LDS region (no workgroup barrier per
// tile), multiplies them against the query tile on the matrix cores, updates the running row
// statistics and pools keys per sentence.  A sentence that lies inside one wave's range is
// normalised and written straight from registers; the (at most 3) sentences that cross wave
// boundaries are pieced together through LDS in a fixed order, so results are reproducible.
#include "scan_common.h"

namespace skipkv {

namespace {

constexpr int kCapW = kChunkCap / 4;  // tokens per wave

// Cross-workgroup communication (the workgroups may sit on different XCDs, whose L2 caches are not
// coherent with each other).  Everything that is communicated - chunk statistics, row normalisers,
// the arrive counter and the ready flag - is accessed ONLY with device-scope relaxed atomics, which
// are coherent by themselves; ordering comes from waiting until the data stores have been
// acknowledged before the counter or flag is touched, and from program order plus a workgroup
// barrier on the reading side.  No device-scope fence is used: on this chip such a fence writes
// back and invalidates a whole L2, which is ruinous when thousands of workgroups do it.
__device__ __forceinline__ void coherent_store(float *p, float v) {
  __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ float coherent_load(const float *p) {
  return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ void coherent_store2(float2 *p, float2 v) {
  unsigned long long u = (unsigned long long)__float_as_uint(v.x) | ((unsigned long long)__float_as_uint(v.y) << 32);
  __hip_atomic_store(reinterpret_cast<unsigned long long *>(p), u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ float2 coherent_load2(const float2 *p) {
  const unsigned long long u =
      __hip_atomic_load(reinterpret_cast<const unsigned long long *>(p), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  return make_float2(__uint_as_float((uint32_t)u), __uint_as_float((uint32_t)(u >> 32)));
}
__device__ __forceinline__ void stores_done() { __builtin_amdgcn_s_waitcnt(0); }  // vmcnt(0): every earlier store is acknowledged

template <int DT, int NP, int AL>
__global__ void __launch_bounds__(256) k_scan_fused(ScanArgs a) {
  constexpr int SL = NP * AL;
  constexpr int NT = (SL + 3) / 4;
  constexpr int SLP = 4 * NT;
  constexpr int R = 16 * NT;
  constexpr int SUBS = kCapW / 16;                       // 16-token sub-tiles per wave
  constexpr int NSUB = (DT == SKIPKV_BF16) ? 2 : 1;      // sub-tiles staged and multiplied per step
  constexpr int STEPS = SUBS / NSUB;
  constexpr int WT = 16 * NSUB;                          // tokens per step
  constexpr int LSTR = Tr<DT>::LSTR, ROWB = Tr<DT>::ROWB, ESZ = Tr<DT>::ESZ;
  constexpr int PPR = ROWB / 16;
  constexpr int LOADS = WT * PPR / 64;                   // 16-byte loads per lane per step

  __shared__ __align__(16) char kt[4][WT * LSTR];
  __shared__ __align__(16) char qt[R * LSTR];
  __shared__ int soff[kChunkMaxSent + 2];
  __shared__ float part_first[4][kD];  // key sum, over this wave's range, of the sentence already running at its start
  __shared__ float part_last[4][kD];   // key sum of the sentence that starts in this wave's range and runs past its end
  __shared__ float wstat[4][R][2];
  __shared__ float imp[kChunkCap];
  __shared__ int s_flag;

  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63, c16 = lane & 15, g = lane >> 4;
  const int n_lh = a.n_layers * a.n_kv_heads;
  const int n_chunks = a.ws.hdr->n_chunks;
  const uint32_t n_items = (uint32_t)n_lh * (uint32_t)n_chunks;
  const int n = a.n_q_heads / a.n_kv_heads;
  const int64_t tok_pitch = a.stride_tok * ESZ;
  const float inv_alpha = 1.f / (float)a.alpha;

  for (uint32_t item = blockIdx.x; item < n_items; item += gridDim.x) {
    const int lh = item / n_chunks, c = item % n_chunks;
    const Chunk ch = a.ws.chunks[c];
    const int b = ch.b, ns = ch.ns;
    if (a.force_two_pass || !a.ws.seq_fused[b]) continue;
    const int l = lh / a.n_kv_heads, h = lh % a.n_kv_heads;
    const int n_tok = ch.n_tok;
    const int t_begin = ch.t_begin, t_end = ch.t_begin + ch.len;
    const int sent_col0 = ch.soff_idx - b;
    const int lhb = lh * a.batch + b;
    __syncthreads();  // the previous item's readers of LDS are done

    if (tid <= ns) soff[tid] = a.sent_off[ch.soff_idx + tid];
    {  // queries of the group -> LDS, one padded row per (lane group, slot)
      const char *qbase = static_cast<const char *>(a.q);
      for (int r0 = 0; r0 < R; r0 += 256 / PPR) {
        const int r = r0 + tid / PPR, piece = tid % PPR;
        const int slot = 4 * (r >> 4) + (r & 3), gq = (r >> 2) & 3;
        const int al = slot / NP, i = slot % NP, aq = gq + 4 * al;
        uint4 val = make_uint4(0, 0, 0, 0);
        if (slot < SL && i < n && aq < a.alpha) {
          const int64_t row = (((int64_t)l * a.batch + b) * a.n_q_heads + (h * n + i)) * a.alpha + aq;
          val = *reinterpret_cast<const uint4 *>(qbase + row * ROWB + piece * 16);
        }
        *reinterpret_cast<uint4 *>(qt + r * LSTR + piece * 16) = val;
      }
    }
    __syncthreads();

    const char *kbase = static_cast<const char *>(a.k) +
                        ((int64_t)l * a.stride_layer + (int64_t)h * a.stride_head + (int64_t)ch.tok0 * a.stride_tok) * ESZ;
    const int last_free = n_tok - a.alpha;  // keys t <= last_free are visible to every window query
    const int w0 = t_begin + wave * kCapW, w1 = min(w0 + kCapW, t_end);  // this wave's tokens

    f32x4 acc[SUBS][NT];
    float ref[SLP], lsum[SLP];
#pragma unroll
    for (int q = 0; q < SLP; ++q) {
      ref[q] = kRefInit;
      lsum[q] = 0.f;
    }
#pragma unroll
    for (int s = 0; s < SUBS; ++s)
#pragma unroll
      for (int T = 0; T < NT; ++T) acc[s][T] = f32x4{0.f, 0.f, 0.f, 0.f};

    // sentence pooling state: current sentence, its running key sum (lane = 2 head-dim columns)
    int si = 0;
    float ps0 = 0.f, ps1 = 0.f;
    if (w0 < w1) si = __popcll(__ballot(lane < ns && soff[lane + 1] <= w0));

    auto emit_sentence = [&](int s_idx, float k0, float k1) {  // unit embedding, bf16 hi + lo
      const float inv_len = 1.f / (float)(soff[s_idx + 1] - soff[s_idx]);
      const float m0 = k0 * inv_len, m1 = k1 * inv_len;
      const float inv = 1.f / (sqrtf(wave_sum(m0 * m0 + m1 * m1)) + 1e-12f);
      const float u0 = m0 * inv, u1 = m1 * inv;
      const uint32_t h0 = f32_to_bf16_bits(u0), h1 = f32_to_bf16_bits(u1);
      const uint32_t l0 = f32_to_bf16_bits(u0 - bf16_bits_to_f32(h0)), l1 = f32_to_bf16_bits(u1 - bf16_bits_to_f32(h1));
      const int64_t o = ((int64_t)lh * a.total_sentences + sent_col0 + s_idx) * (kD / 2) + lane;
      reinterpret_cast<uint32_t *>(a.ws.vhat_hi)[o] = h0 | (h1 << 16);
      reinterpret_cast<uint32_t *>(a.ws.vhat_lo)[o] = l0 | (l1 << 16);
    };

#pragma unroll
    for (int step = 0; step < STEPS; ++step) {
      const int ts = w0 + step * WT;
      if (ts < w1) {
        const int te = min(ts + WT, w1);
        char *ktw = kt[wave];
        {  // stage this wave's rows: HBM -> registers -> private LDS region
          uint4 regs[LOADS];
#pragma unroll
          for (int it = 0; it < LOADS; ++it) {
            const int idx = it * 64 + lane, row = idx / PPR, piece = idx % PPR, t = ts + row;
            regs[it] = make_uint4(0, 0, 0, 0);
            if (t < te) regs[it] = *reinterpret_cast<const uint4 *>(kbase + (int64_t)t * tok_pitch + piece * 16);
          }
#pragma unroll
          for (int it = 0; it < LOADS; ++it) {
            const int idx = it * 64 + lane, row = idx / PPR, piece = idx % PPR;
            *reinterpret_cast<uint4 *>(ktw + row * LSTR + piece * 16) = regs[it];
          }
        }
        __builtin_amdgcn_wave_barrier();  // LDS operations of one wave execute in order: later reads see these writes

#pragma unroll
        for (int s = 0; s < NSUB; ++s)
          if (ts + 16 * s < te) tile_logits<DT, NT>(qt, ktw + (16 * s + c16) * LSTR, c16, g, acc[step * NSUB + s]);

        // ---- running softmax statistics of every query row over these tokens
        float tmax[SLP];
#pragma unroll
        for (int q = 0; q < SLP; ++q) tmax[q] = -INFINITY;
#pragma unroll
        for (int s = 0; s < NSUB; ++s) {
          const int t = ts + 16 * s + c16;
          const bool edge = (ts + 16 * s + 15 >= te) || (ts + 16 * s + 15 > last_free);
#pragma unroll
          for (int q = 0; q < SLP; ++q) {
            float x = acc[step * NSUB + s][q >> 2][q & 3] * kScale2;
            if (edge) {
              const int aq = g + 4 * (q / NP);
              if (!(t < te && t <= last_free + aq)) x = -INFINITY;
            }
            acc[step * NSUB + s][q >> 2][q & 3] = x;
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
          for (int q = 0; q < SLP; ++q) lsum[q] += __builtin_amdgcn_exp2f(acc[step * NSUB + s][q >> 2][q & 3] - ref[q]);

        // ---- sentence key sums over tokens [ts, te), walked in order
        int t = ts;
        while (t < te) {
          const int run_end = min(soff[si + 1], te);
          const char *rowp = ktw + (t - ts) * LSTR;
          float q0 = 0.f, q1 = 0.f, r0 = 0.f, r1 = 0.f;  // two independent chains
          int cnt = run_end - t;
          if constexpr (DT == SKIPKV_BF16) {
            for (; cnt >= 2; cnt -= 2, rowp += 2 * LSTR) {
              const uint32_t wa = *reinterpret_cast<const uint32_t *>(rowp + lane * 4);
              const uint32_t wb = *reinterpret_cast<const uint32_t *>(rowp + LSTR + lane * 4);
              q0 += __uint_as_float(wa << 16);
              q1 += __uint_as_float(wa & 0xFFFF0000u);
              r0 += __uint_as_float(wb << 16);
              r1 += __uint_as_float(wb & 0xFFFF0000u);
            }
            if (cnt) {
              const uint32_t wa = *reinterpret_cast<const uint32_t *>(rowp + lane * 4);
              q0 += __uint_as_float(wa << 16);
              q1 += __uint_as_float(wa & 0xFFFF0000u);
            }
          } else {
            for (; cnt >= 2; cnt -= 2, rowp += 2 * LSTR) {
              const float2 wa = *reinterpret_cast<const float2 *>(rowp + lane * 8);
              const float2 wb = *reinterpret_cast<const float2 *>(rowp + LSTR + lane * 8);
              q0 += wa.x;
              q1 += wa.y;
              r0 += wb.x;
              r1 += wb.y;
            }
            if (cnt) {
              const float2 wa = *reinterpret_cast<const float2 *>(rowp + lane * 8);
              q0 += wa.x;
              q1 += wa.y;
            }
          }
          ps0 += q0 + r0;
          ps1 += q1 + r1;
          t = run_end;
          if (t == soff[si + 1]) {  // the sentence ends here
            if (soff[si] >= w0) {
              emit_sentence(si, ps0, ps1);
            } else {
              part_first[wave][2 * lane] = ps0;
              part_first[wave][2 * lane + 1] = ps1;
            }
            ps0 = ps1 = 0.f;
            ++si;
          }
        }
      }
    }
    if (w0 < w1 && si < ns && soff[si] < w1 && w1 < soff[si + 1]) {  // a sentence is still running at the end of this wave's range
      float *dst = (soff[si] >= w0) ? part_last[wave] : part_first[wave];
      dst[2 * lane] = ps0;
      dst[2 * lane + 1] = ps1;
    }
#pragma unroll
    for (int q = 0; q < SLP; ++q) {
      const float tot = row16_sum(lsum[q]);
      if (c16 == 0) {
        const int r = 16 * (q >> 2) + 4 * g + (q & 3);
        wstat[wave][r][0] = ref[q];
        wstat[wave][r][1] = tot;
      }
    }
    __syncthreads();

    // ---- sentences that cross wave boundaries: the wave in whose range one starts pieces it together
    if (w0 < w1) {
      const int sl = __popcll(__ballot(lane < ns && soff[lane + 1] <= w1 - 1));  // sentence holding the wave's last token
      if (soff[sl] >= w0 && soff[sl + 1] > w1) {
        float k0 = part_last[wave][2 * lane], k1 = part_last[wave][2 * lane + 1];
        for (int w = wave + 1; w < 4 && t_begin + w * kCapW < soff[sl + 1]; ++w) {
          k0 += part_first[w][2 * lane];
          k1 += part_first[w][2 * lane + 1];
        }
        emit_sentence(sl, k0, k1);
      }
    }
    // ---- publish the chunk's row statistics
    for (int r = tid; r < R; r += 256) {
      float m = kRefInit;
#pragma unroll
      for (int w = 0; w < 4; ++w) m = fmaxf(m, wstat[w][r][0]);
      float s = 0.f;
#pragma unroll
      for (int w = 0; w < 4; ++w) s += wstat[w][r][1] * __builtin_amdgcn_exp2f(wstat[w][r][0] - m);
      coherent_store2(&a.ws.stat_part[((int64_t)lh * a.ws.nc_max + c) * R + r], make_float2(m, s));
    }
    stores_done();
    __syncthreads();
    if (tid == 0) {
      const int old = __hip_atomic_fetch_add(&a.ws.arrive[lhb], 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      s_flag = (old == a.ws.chunk_cnt[b] - 1);
    }
    __syncthreads();
    float *rn = a.ws.row_norm + (int64_t)lhb * R;
    if (s_flag) {  // last chunk of the head to arrive: merge the partials into the normalisers
      // lane = query row, wave w takes chunks c0+w, c0+w+4, ...; 8 independent loads in flight per lane
      const int c0 = a.ws.chunk_base[b], nc = a.ws.chunk_cnt[b];
      float m = kRefInit, s = 0.f;
      for (int r = lane; r < R; r += 64) {
        m = kRefInit;
        s = 0.f;
        for (int cc = wave; cc < nc; cc += 32) {
          float2 pv[8];
#pragma unroll
          for (int u = 0; u < 8; ++u) {
            pv[u] = make_float2(kRefInit, 0.f);
            if (cc + 4 * u < nc) pv[u] = coherent_load2(&a.ws.stat_part[((int64_t)lh * a.ws.nc_max + c0 + cc + 4 * u) * R + r]);
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
      __syncthreads();
      for (int r = tid; r < R; r += 256) {
        float mm = kRefInit;
#pragma unroll
        for (int w = 0; w < 4; ++w) mm = fmaxf(mm, wstat[w][r][0]);
        float ss = 0.f;
#pragma unroll
        for (int w = 0; w < 4; ++w) ss += wstat[w][r][1] * __builtin_amdgcn_exp2f(wstat[w][r][0] - mm);
        coherent_store(&rn[r], ss > 0.f ? mm + __builtin_amdgcn_logf(ss) : INFINITY);
      }
      stores_done();
      __syncthreads();
      if (tid == 0) __hip_atomic_store(&a.ws.ready[lhb], 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    } else {
      if (tid == 0) {
        int polls = 0;
        while (__hip_atomic_load(&a.ws.ready[lhb], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) == 0) {
          __builtin_amdgcn_s_sleep(4);
          if (++polls > a.spin_limit) {
            if (a.dev_status) atomicOr(a.dev_status, SKIPKV_DEV_TIMEOUT);
            break;
          }
        }
      }
      __syncthreads();
    }

    // ---- token importance from the logits still in registers
    float cn[SLP];
#pragma unroll
    for (int q = 0; q < SLP; ++q) {
      const int al = q / NP, i = q % NP;
      const bool used = q < SL && i < n && (g + 4 * al) < a.alpha;
      cn[q] = used ? coherent_load(&rn[16 * (q >> 2) + 4 * g + (q & 3)]) : INFINITY;
    }
#pragma unroll
    for (int s = 0; s < SUBS; ++s) {
      const int t = w0 + 16 * s + c16;
      float sum = 0.f;
#pragma unroll
      for (int al = 0; al < AL; ++al) {
        float gm = -INFINITY;
#pragma unroll
        for (int i = 0; i < NP; ++i) {
          const int q = al * NP + i;
          gm = fmaxf(gm, acc[s][q >> 2][q & 3] - cn[q]);  // logits were scaled and masked in the first phase
        }
        sum += __builtin_amdgcn_exp2f(gm);
      }
      sum += __shfl_xor(sum, 16);
      sum += __shfl_xor(sum, 32);
      if (g == 0) imp[wave * kCapW + 16 * s + c16] = (t < w1) ? sum * inv_alpha : 0.f;
    }
    __syncthreads();
    const int p_start = n_tok - min(a.protect, n_tok);
    const int64_t tok_col = (int64_t)lh * a.total_tokens + ch.tok0;
    if (tid < ns) {
      const int lo = soff[tid], hi = min(soff[tid + 1], p_start);
      float sum_i = 0.f, sum_r = 0.f;
      for (int t = lo; t < hi; ++t) {
        sum_i += imp[t - t_begin];
        if (a.tok_red) sum_r += a.tok_red[tok_col + t];
      }
      const int64_t o = (int64_t)lh * a.total_sentences + sent_col0 + tid;
      a.ws.sent_imp[o] = hi > lo ? sum_i / (float)(hi - lo) : 0.f;
      a.ws.sent_red[o] = hi > lo ? sum_r / (float)(hi - lo) : 0.f;
    }
    if (a.tok_imp)
      for (int i = tid; i < t_end - t_begin; i += 256) a.tok_imp[tok_col + t_begin + i] = imp[i];
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
  if (grid < kFuseMaxChunks) return hipErrorInvalidConfiguration;
  hipLaunchKernelGGL((k_scan_fused<DT, NP, AL>), dim3(grid), dim3(256), 0, st, a);
  return hipGetLastError();
}

}  // namespace

bool scan_fused_supported(const RowLayout &rl) { return rl.nt <= 4; }

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

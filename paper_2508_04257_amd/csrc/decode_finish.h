// Last step of decode attention for one (sequence, query head): log-sum-exp merge of the parts a
// token stream was cut into, the kept (sink) tokens' fp16 rows folded into the same running
// softmax, normalise, store fp16 (paper, Section 4.2: the attention sum split into sink and
// non-sink tokens; here the non-sink sum itself arrives in several parts).
//
// One wave, lane = channels 2 lane and 2 lane + 1.  Used by the stream kernel's last-arriving
// workgroup (decode_mfma_impl.h) and by the stand-alone combine kernel (decode.hip).
#pragma once

#include "kvs_device.h"

namespace kvs {

constexpr int kPartRow = KVS_HEAD_DIM + 2;          // unnormalised output row, running max (natural log), running sum
constexpr float kRsqrtHeadDim = 0.08838834764831845f;   // 1 / sqrt(128)

// Device-coherent accesses (they go through to memory instead of living in the compute die's own
// L2): how workgroups on different dies hand each other their parts inside one kernel without a
// cache-wide write-back / invalidate, which costs microseconds per workgroup.
__device__ inline void store_coherent(float* p, float v) {
  __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ inline void store_coherent(float2* p, float2 v) {
  __hip_atomic_store(reinterpret_cast<unsigned long long*>(p), __builtin_bit_cast(unsigned long long, v), __ATOMIC_RELAXED,
                     __HIP_MEMORY_SCOPE_AGENT);
}
template <bool COHERENT>
__device__ inline float load_part(const float* p) {
  if (COHERENT) return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  return *p;
}
template <bool COHERENT>
__device__ inline float2 load_part(const float2* p) {
  if (COHERENT)
    return __builtin_bit_cast(float2, __hip_atomic_load(reinterpret_cast<const unsigned long long*>(p), __ATOMIC_RELAXED,
                                                        __HIP_MEMORY_SCOPE_AGENT));
  return *p;
}

//   COHERENT the parts were written by other workgroups of the running kernel (store_coherent)
//   q2      the lane's two query values (packed fp16 pair of the row b * Hq + hq)
//   parts   `splits` rows of kPartRow floats; xrow one more such row or null
//   kk, kv  the lane's words of the (b, kv head) keep rows (row j at word offset 64 j); cnt rows
template <bool COHERENT>
__device__ inline void finish_row(uint32_t q2, const float* __restrict__ parts, int splits,
                                  const float* __restrict__ xrow, const uint32_t* __restrict__ kk,
                                  const uint32_t* __restrict__ kv, int cnt, uint32_t* __restrict__ out_word,
                                  float* __restrict__ lse_ptr, int lane) {
  const float q0 = half_bits_to_float(static_cast<uint16_t>(q2 & 0xFFFFu));
  const float q1 = half_bits_to_float(static_cast<uint16_t>(q2 >> 16));

  // The first kept rows are requested before anything else is read.
  constexpr int kKeepBatch = 8;
  uint32_t kw_next[kKeepBatch], vw_next[kKeepBatch];
#pragma unroll
  for (int u = 0; u < kKeepBatch; ++u) {
    kw_next[u] = 0;  vw_next[u] = 0;
    if (cnt > 0) {
      const int j = min(u, cnt - 1);
      kw_next[u] = kk[j * 64];
      vw_next[u] = kv[j * 64];
    }
  }

  float M = -INFINITY;
  for (int s = lane; s < splits; s += KVS_WAVE) M = fmaxf(M, load_part<COHERENT>(parts + s * kPartRow + 128));
  M = wave_max(M);
  if (xrow) M = fmaxf(M, xrow[128]);
  float L = 0.0f, O0 = 0.0f, O1 = 0.0f;
  if (xrow) {
    const float ms = xrow[128];
    const float f = ms == -INFINITY ? 0.0f : __expf(ms - M);
    const float2 o = reinterpret_cast<const float2*>(xrow)[lane];
    L = xrow[129] * f;
    O0 = o.x * f;
    O1 = o.y * f;
  }
#pragma unroll 4
  for (int s = 0; s < splits; ++s) {
    const float ms = load_part<COHERENT>(parts + s * kPartRow + 128);
    const float f = ms == -INFINITY ? 0.0f : __expf(ms - M);
    const float2 o = load_part<COHERENT>(reinterpret_cast<const float2*>(parts + s * kPartRow) + lane);
    L += load_part<COHERENT>(parts + s * kPartRow + 129) * f;
    O0 += o.x * f;
    O1 += o.y * f;
  }

  // Kept tokens: exact fp16 rows, eight per step; the step after next is requested before this
  // one is folded in.
  for (int j0 = 0; j0 < cnt; j0 += kKeepBatch) {
    uint32_t kw[kKeepBatch], vw[kKeepBatch];
#pragma unroll
    for (int u = 0; u < kKeepBatch; ++u) { kw[u] = kw_next[u]; vw[u] = vw_next[u]; }
    if (j0 + kKeepBatch < cnt) {
#pragma unroll
      for (int u = 0; u < kKeepBatch; ++u) {
        const int j = min(j0 + kKeepBatch + u, cnt - 1);
        kw_next[u] = kk[j * 64];
        vw_next[u] = kv[j * 64];
      }
    }
    float sc[kKeepBatch];
#pragma unroll
    for (int u = 0; u < kKeepBatch; ++u)               // the reductions of one step are independent of each other
      sc[u] = wave_sum(q0 * half_bits_to_float(static_cast<uint16_t>(kw[u] & 0xFFFFu)) +
                       q1 * half_bits_to_float(static_cast<uint16_t>(kw[u] >> 16))) * kRsqrtHeadDim;
#pragma unroll
    for (int u = 0; u < kKeepBatch; ++u) {
      if (j0 + u < cnt) {
        const float m_new = fmaxf(M, sc[u]);
        const float alpha = M == -INFINITY ? 0.0f : __expf(M - m_new);
        const float p = __expf(sc[u] - m_new);
        L = L * alpha + p;
        O0 = O0 * alpha + p * half_bits_to_float(static_cast<uint16_t>(vw[u] & 0xFFFFu));
        O1 = O1 * alpha + p * half_bits_to_float(static_cast<uint16_t>(vw[u] >> 16));
        M = m_new;
      }
    }
  }
  const float inv = L > 0.0f ? 1.0f / L : 0.0f;
  out_word[lane] = static_cast<uint32_t>(float_to_half_bits_rn(O0 * inv)) |
                   (static_cast<uint32_t>(float_to_half_bits_rn(O1 * inv)) << 16);
  if (lse_ptr && lane == 0) *lse_ptr = L > 0.0f ? M + __logf(L) : -INFINITY;
}

}  // namespace kvs

// Where a quantise workgroup parks its isolated entries until the row pointers are known
// (dense-and-sparse variant; paper, Section 5.1).  The staging list of one tensor is cut into
// kEmitSegments segments, each with a counter of its own, plus one overflow region as large as the
// CSR capacity: a workgroup claims room for its whole run with one atomic on the counter of
// segment (workgroup index mod kEmitSegments), and only if the run does not fit there any more
// with a second atomic on the overflow counter.  One counter for everything serialised the claims
// of tens of thousands of workgroups on a single address and bounded the whole kernel.  Whatever
// the distribution, a tensor with no more than `cap` isolated entries fits: the overflow region
// alone could hold them all.
#pragma once

#include "kvs_device.h"

namespace kvs {

constexpr int kEmitSegments = 64;

// Positions are 32-bit: with a capacity too large for two regions of that size there is one
// segment and no overflow region (the behaviour of a single counter).
__host__ __device__ inline int emit_segments(long long cap) {
  return cap <= (1ll << 30) - kEmitSegments ? kEmitSegments : 1;
}
__host__ __device__ inline long long emit_segment_cap(long long cap) {
  const int s = emit_segments(cap);
  return s == 1 ? cap : (cap + s - 1) / s;
}
// Words of one tensor's staging list.
__host__ __device__ inline long long emit_list_words(long long cap) {
  const int s = emit_segments(cap);
  return s == 1 ? cap : s * emit_segment_cap(cap) + cap;
}
// Counters per tensor: one per segment, then the overflow counter.
constexpr int kEmitCounters = kEmitSegments + 1;

#ifdef __HIPCC__
// Which halves of a register pair hold a magnitude at or above a threshold, with packed 16-bit
// arithmetic (used by the quantise kernels to mark isolated entries and by the histogram pass to
// find the few entries above its bound).
typedef unsigned short ushort2v __attribute__((ext_vector_type(2)));
typedef short short2v __attribute__((ext_vector_type(2)));
// 0xFFFF in every half of w whose magnitude pattern is below tau (tau2 = tau in both halves,
// tau <= 0x8000), 0 in the others.
__device__ inline uint32_t below_mask(uint32_t w, uint32_t tau2) {
  const ushort2v d = __builtin_bit_cast(ushort2v, w & 0x7FFF7FFFu) - __builtin_bit_cast(ushort2v, tau2);
  uint32_t m = __builtin_bit_cast(uint32_t, __builtin_bit_cast(short2v, d) >> 15);
  // The empty statement hides where the mask comes from: knowing that it is a sign, the compiler
  // turns every (a & m) | (b & ~m) that follows into two 16-bit compares, selects and a byte
  // permute - eight instructions where one bit-field insert does it.
  asm volatile("" : "+v"(m));
  return m;
}
// Bit j = element j of the uint4 (eight halves) is at or above tau.  Each mask contributes the
// two bits of its pair: the low half's at bit 2 k, the high half's at bit 16 + 2 k + 1.
__device__ inline uint32_t isolated8(const uint32_t m[4]) {
  uint32_t x = m[0] & 0x00020001u;
  x |= m[1] & 0x00080004u;
  x |= m[2] & 0x00200010u;
  x |= m[3] & 0x00800040u;
  return ((x | (x >> 16)) & 0xFFu) ^ 0xFFu;
}
// Start of a run of `count` entries for this workgroup (called by one lane).
__device__ inline int claim_run(const SparseEmit& emit, int count) {
  const int segs = emit_segments(emit.cap);
  if (segs == 1) return atomicAdd(emit.counter, count);
  const int seg_cap = static_cast<int>(emit_segment_cap(emit.cap));
  const int seg = static_cast<int>(blockIdx.x % kEmitSegments);
  const int base = atomicAdd(emit.counter + seg, count);
  if (base <= seg_cap - count) return seg * seg_cap + base;
  return segs * seg_cap + atomicAdd(emit.counter + kEmitSegments, count);
}
#endif

}  // namespace kvs

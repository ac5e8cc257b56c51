// Internal helpers shared by the gfx950 kernels: packed-word format, wave64 reductions,
// fp16 bit handling.  Not part of the C ABI.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "kvs.h"

#define KVS_WAVE 64

namespace kvs {

// Packed-word format of one bit width (the layout comment of kvs.h).
template <int BITS>
struct Fmt;
template <>
struct Fmt<2> {
  static constexpr int cpw = 16, W = 8, qmax = 3;
  __host__ __device__ static constexpr int shift(int j) { return 2 * j; }
};
template <>
struct Fmt<3> {
  static constexpr int cpw = 10, W = 13, qmax = 7;
  __host__ __device__ static constexpr int shift(int j) { return 3 * (j % 5) + 16 * (j / 5); }
};
template <>
struct Fmt<4> {
  static constexpr int cpw = 8, W = 16, qmax = 15;
  __host__ __device__ static constexpr int shift(int j) { return 4 * j; }
};
template <>
struct Fmt<8> {
  static constexpr int cpw = 4, W = 32, qmax = 255;
  __host__ __device__ static constexpr int shift(int j) { return 8 * j; }
};

// Host-side checks and launch geometry shared by the entry points (kvs_api.hip).
kvs_status validate_desc(const kvs_desc* d);
struct DecodeGeometry {
  int splits;        // workgroups (token ranges) per (sequence, KV head)
  int split_tokens;  // tokens per split, a multiple of 128
};
DecodeGeometry decode_geometry(const kvs_desc* d);
DecodeGeometry decode_geometry(const kvs_desc* d, int n_used);
int decode_max_splits(const kvs_desc* d);
size_t decode_workspace_bytes(const kvs_desc* d);   // the part of kvs_workspace_bytes the decode calls use
// Host-side argument checks of the two prefill calls (what they refuse before launching anything).
kvs_status check_predict_call(const void* hidden, int32_t B, int32_t n, int32_t d, const int32_t* channels,
                              int32_t n_channels, int32_t k, int32_t first_n, const int32_t* sink_idx,
                              const uint8_t* keep_mask);
kvs_status check_quantize_call(const kvs_desc* desc, const void* K, const void* V, const uint8_t* keep_mask,
                               const kvs_cache* out, const void* workspace);
// Matrix-core decode kernel (decode_mfma.hip); dense-and-sparse caches included (the isolated
// outliers' corrections are applied inside it).
void launch_decode_mfma(const kvs_desc* d, const DecodeGeometry& geo, const void* q, const kvs_cache* c,
                        void* out, float* lse, float* ws, int* arrive, int n_used, const float* extra, hipStream_t s);
// The workspace starts with the stream kernel's arrival counters, one 32-bit word per (sequence,
// KV head), rounded up to 256 bytes: zero before a call, put back to zero by the call.  What the
// calls keep in the workspace otherwise follows them.
inline size_t workspace_counter_words(const kvs_desc* d) {
  return (static_cast<size_t>(d->B) * d->Hkv + 63) & ~static_cast<size_t>(63);
}
// The CSR column / value arrays are four entries longer than the capacity: the decode kernel
// reads aligned groups of four entries, and the last group may start just below the capacity.
constexpr int kCsrPadEntries = 4;

// Which tokens a quantise launch reads and where they go.  A plain call quantises the whole
// tensor in place (every field = desc->n, offsets 0); a growing cache quantises the whole blocks of
// a prompt, or one block out of the residual window, into buffers laid out for the capacity.
struct QuantSpan {
  int n_in;         // tokens per (b, h) in the input tensors (their row stride)
  int n_tokens;     // tokens to quantise per (b, h), from input token 0 on; a multiple of 128
  int n_cap;        // tokens per (b, h) the cache buffers are laid out for
  int t_out;        // cache token index of input token 0; a multiple of 128
  int mask_stride;  // tokens per sequence in the keep mask that is passed along
  int mask_t0;      // mask index of input token 0
};
inline QuantSpan whole_span(const kvs_desc* d) { return QuantSpan{d->n, d->n, d->n, 0, d->n, 0}; }

// Lean quantisation kernels (quantize_fast.hip), every bit width; with `plan` (dense-and-sparse)
// they also mark the isolated entries and park them in the plan's staging lists.  own_keep: also
// build the keep index and copy the kept rows (a plain call); otherwise the caller does both.
struct SparsePlan;
void launch_quantize_fast(const kvs_desc* d, const QuantSpan& sp, bool own_keep, const void* K, const void* V,
                          const uint8_t* mask, const kvs_cache* out, const uint32_t* static_k, const uint32_t* static_v,
                          const SparsePlan* plan, hipStream_t s);
// Static quantisation: calibration state [4][Hkv][128] uint32 (order-preserving float encoding).
void launch_calibrate_reset(const kvs_desc* d, uint32_t* calib, hipStream_t s);
void launch_calibrate(const kvs_desc* d, const void* K, const void* V, const uint8_t* mask, uint32_t* calib, hipStream_t s);
void launch_static_params(const kvs_desc* d, const uint32_t* calib, uint32_t* static_k, uint32_t* static_v, hipStream_t s);

// Dense-and-sparse helpers (sparse.hip): where the scratch lives and the launch sequences.
// Where a quantise kernel leaves the isolated entries of one tensor: every workgroup claims one
// run of the staging list (counter), notes where it starts (block_base, one per workgroup) and
// writes its entries there in their final relative order as  index | fp16 value << 16.
struct SparseEmit {
  uint32_t* list;     // [cap]
  int* counter;       // entries claimed so far
  int* block_base;    // [workgroups of the quantise kernel]
  long long cap;
};
struct SparsePlan {
  size_t rows;      // B * Hkv * n, the row count of both CSR structures
  int nblk;         // scan workgroups
  uint32_t* hist;   // histograms of K and V: [2][32768] sample, [2][32768] full, [2][4096] bracket
  uint32_t* tau;    // [2] thresholds as fp16 magnitude patterns (0x8000 = isolate nothing)
  int* sums_k;      // [nblk + 1] scan scratch
  int* sums_v;
  SparseEmit emit_k, emit_v;
  int rows_per_block_k;   // CSR rows per quantise workgroup: max(G, 64) for Keys, 128 for Values
};
size_t sparse_workspace_words(const kvs_desc* d);
SparsePlan sparse_plan(const kvs_desc* d, void* workspace);
void sparse_thresholds(const kvs_desc* d, const SparsePlan& p, const void* K, const void* V,
                       const uint8_t* mask, const kvs_cache* out, hipStream_t s);
void sparse_given_thresholds(const SparsePlan& p, const uint32_t* given, const kvs_cache* out, hipStream_t s);
void sparse_export_thresholds(const SparsePlan& p, uint32_t* tau_out, hipStream_t s);
void sparse_build_csr(const kvs_desc* d, const SparsePlan& p, const kvs_cache* out, hipStream_t s);

__host__ __device__ inline int words_per_128(int bits) { return bits == 2 ? 8 : (bits == 3 ? 13 : (bits == 4 ? 16 : 32)); }

__device__ inline float half_bits_to_float(uint16_t h) {
  return static_cast<float>(__builtin_bit_cast(_Float16, h));
}
__device__ inline uint16_t float_to_half_bits_rn(float f) {
  return __builtin_bit_cast(uint16_t, static_cast<_Float16>(f));
}

// Parameter word: fp16 scale in the low half, int16 zero in the high half.
__device__ inline void unpack_param(uint32_t p, float& scale, int& zero) {
  scale = half_bits_to_float(static_cast<uint16_t>(p & 0xFFFFu));
  zero = static_cast<int>(static_cast<int16_t>(p >> 16));
}

// Wave-wide reductions whose result every lane receives.  Inside a row of 16 lanes the partners
// come through data-parallel-primitive moves (lane ^ 1, lane ^ 2, mirrored half row, mirrored
// row), which cost one vector instruction each; the four row results are then read as scalars.
// (A butterfly of lane shuffles would send all six steps through the LDS crossbar.)
template <int CTRL>
__device__ inline int dpp_move(int v) {
  return __builtin_amdgcn_update_dpp(0, v, CTRL, 0xF, 0xF, true);
}
constexpr int kDppXor1 = 0xB1, kDppXor2 = 0x4E, kDppHalfMirror = 0x141, kDppMirror = 0x140;

__device__ inline float wave_max(float v) {
  v = fmaxf(v, __builtin_bit_cast(float, dpp_move<kDppXor1>(__builtin_bit_cast(int, v))));
  v = fmaxf(v, __builtin_bit_cast(float, dpp_move<kDppXor2>(__builtin_bit_cast(int, v))));
  v = fmaxf(v, __builtin_bit_cast(float, dpp_move<kDppHalfMirror>(__builtin_bit_cast(int, v))));
  v = fmaxf(v, __builtin_bit_cast(float, dpp_move<kDppMirror>(__builtin_bit_cast(int, v))));
  const int i = __builtin_bit_cast(int, v);
  const float r0 = __builtin_bit_cast(float, __builtin_amdgcn_readlane(i, 0));
  const float r1 = __builtin_bit_cast(float, __builtin_amdgcn_readlane(i, 16));
  const float r2 = __builtin_bit_cast(float, __builtin_amdgcn_readlane(i, 32));
  const float r3 = __builtin_bit_cast(float, __builtin_amdgcn_readlane(i, 48));
  return fmaxf(fmaxf(r0, r1), fmaxf(r2, r3));
}
__device__ inline float wave_sum(float v) {
  v += __builtin_bit_cast(float, dpp_move<kDppXor1>(__builtin_bit_cast(int, v)));
  v += __builtin_bit_cast(float, dpp_move<kDppXor2>(__builtin_bit_cast(int, v)));
  v += __builtin_bit_cast(float, dpp_move<kDppHalfMirror>(__builtin_bit_cast(int, v)));
  v += __builtin_bit_cast(float, dpp_move<kDppMirror>(__builtin_bit_cast(int, v)));
  const int i = __builtin_bit_cast(int, v);
  const float r0 = __builtin_bit_cast(float, __builtin_amdgcn_readlane(i, 0));
  const float r1 = __builtin_bit_cast(float, __builtin_amdgcn_readlane(i, 16));
  const float r2 = __builtin_bit_cast(float, __builtin_amdgcn_readlane(i, 32));
  const float r3 = __builtin_bit_cast(float, __builtin_amdgcn_readlane(i, 48));
  return (r0 + r1) + (r2 + r3);
}
__device__ inline uint32_t wave_max_u32(uint32_t v) {
  auto mx = [](uint32_t x, uint32_t y) { return x > y ? x : y; };
  v = mx(v, static_cast<uint32_t>(dpp_move<kDppXor1>(static_cast<int>(v))));
  v = mx(v, static_cast<uint32_t>(dpp_move<kDppXor2>(static_cast<int>(v))));
  v = mx(v, static_cast<uint32_t>(dpp_move<kDppHalfMirror>(static_cast<int>(v))));
  v = mx(v, static_cast<uint32_t>(dpp_move<kDppMirror>(static_cast<int>(v))));
  const int i = static_cast<int>(v);
  const uint32_t r0 = static_cast<uint32_t>(__builtin_amdgcn_readlane(i, 0));
  const uint32_t r1 = static_cast<uint32_t>(__builtin_amdgcn_readlane(i, 16));
  const uint32_t r2 = static_cast<uint32_t>(__builtin_amdgcn_readlane(i, 32));
  const uint32_t r3 = static_cast<uint32_t>(__builtin_amdgcn_readlane(i, 48));
  return mx(mx(r0, r1), mx(r2, r3));
}

}  // namespace kvs

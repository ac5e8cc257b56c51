// kvs_predict_sinks: sink-token prediction from the extreme activation outliers of the
// emergence layer's hidden state (paper, Algorithm 1 - the "l = l_E" branch - and Section 4.3).
//
// One workgroup of 16 waves per sequence.  Token i lives in lane i % 1024; each lane keeps the
// ordering keys of its tokens in registers, so the strided column of H is read exactly once.
// Key = (15-bit fp16 magnitude pattern, lower index first): monotone in |x| for finite inputs
// and independent of how tokens map to lanes, so the result is unique.
// Selection, k <= 64: every wave extracts the top k of its own tokens with wave-level arg-max
// rounds (no workgroup barrier), then wave 0 extracts the top k of the 16 k candidates.
// Larger k: k rounds of a workgroup-wide arg-max.
// Long sequences (n > 4096, k <= 64, workspace given): the strided gather would be bound by what
// one compute unit can pull, so each 4096-token slice gets its own workgroup, which leaves its
// top-k keys in the workspace, and a one-wave kernel per sequence merges the slices.
#include "kvs_device.h"

namespace {

constexpr int kPredictThreads = 1024;
constexpr int kPredictWaves = kPredictThreads / KVS_WAVE;
constexpr int kMaxChannels = 8;
constexpr int kFastK = 64;

struct ChannelList {
  int32_t c[kMaxChannels];
  int32_t count;
};

// KPL = keys per lane: a workgroup covers 1024 * KPL tokens.  SLICE: the workgroup is one of
// `slices` per sequence and writes its top-k keys to slice_keys instead of the final result.
template <int KPL, bool SLICE>
__global__ __launch_bounds__(kPredictThreads) void predict_sinks_kernel(
    const uint16_t* __restrict__ hidden, int n, int d, ChannelList channels, int k, int first_n,
    int32_t* __restrict__ sink_idx, uint8_t* __restrict__ keep_mask, int slices,
    uint32_t* __restrict__ slice_keys) {
  __shared__ uint32_t cand[kPredictWaves * kFastK];   // per-wave winners (fast path) / wave maxima
  __shared__ int32_t chosen[KVS_MAX_TOPK];
  __shared__ uint32_t round_best;

  const int b = SLICE ? blockIdx.x / slices : blockIdx.x;
  const int tok0 = SLICE ? (blockIdx.x % slices) * (kPredictThreads * KPL) : 0;
  const int tid = threadIdx.x, lane = tid & (KVS_WAVE - 1), wave = tid / KVS_WAVE;
  const uint16_t* Hb = hidden + static_cast<size_t>(b) * n * d;
  uint8_t* mask_b = keep_mask + static_cast<size_t>(b) * n;

  // key = (magnitude + 1) << 16 | (65535 - index); 0 = no token / already taken.
  uint32_t key[KPL];
#pragma unroll
  for (int j = 0; j < KPL; ++j) {
    const int i = tok0 + tid + j * kPredictThreads;
    key[j] = 0;
    if (i < n) {
      uint32_t m = 0;
      for (int c = 0; c < channels.count; ++c) {
        const uint32_t v = Hb[static_cast<size_t>(i) * d + channels.c[c]] & 0x7FFFu;
        m = v > m ? v : m;
      }
      key[j] = ((m + 1) << 16) | static_cast<uint32_t>(65535 - i);
      mask_b[i] = i < first_n ? 1 : 0;
    }
  }

  if (k <= kFastK) {
    for (int r = 0; r < k; ++r) {                       // top k of this wave's tokens
      uint32_t best = 0;
#pragma unroll
      for (int j = 0; j < KPL; ++j) best = key[j] > best ? key[j] : best;
      best = kvs::wave_max_u32(best);
#pragma unroll
      for (int j = 0; j < KPL; ++j) key[j] = key[j] == best ? 0u : key[j];   // keys are unique
      if (lane == 0) cand[wave * k + r] = best;         // 0 once the wave has run out of tokens
    }
    __syncthreads();
    if (wave == 0) {                                    // top k of the 16 k candidates
      constexpr int CPL = kPredictWaves * kFastK / KVS_WAVE;   // 16 candidates per lane at most
      uint32_t c[CPL];
#pragma unroll
      for (int j = 0; j < CPL; ++j) {
        const int idx = lane + j * KVS_WAVE;
        c[j] = idx < kPredictWaves * k ? cand[idx] : 0u;
      }
      for (int r = 0; r < k; ++r) {
        uint32_t best = 0;
#pragma unroll
        for (int j = 0; j < CPL; ++j) best = c[j] > best ? c[j] : best;
        best = kvs::wave_max_u32(best);
#pragma unroll
        for (int j = 0; j < CPL; ++j) c[j] = c[j] == best ? 0u : c[j];
        if (lane == 0) {
          if (SLICE) slice_keys[static_cast<size_t>(blockIdx.x) * k + r] = best;
          else chosen[r] = 65535 - static_cast<int>(best & 0xFFFFu);
        }
      }
    }
    if (SLICE) return;
    __syncthreads();
  } else {
    for (int r = 0; r < k; ++r) {
      uint32_t best = 0;
#pragma unroll
      for (int j = 0; j < KPL; ++j) best = key[j] > best ? key[j] : best;
      best = kvs::wave_max_u32(best);
      if (lane == 0) cand[wave] = best;
      __syncthreads();
      if (tid < KVS_WAVE) {
        uint32_t v = tid < kPredictWaves ? cand[tid] : 0u;
        v = kvs::wave_max_u32(v);
        if (tid == 0) {
          round_best = v;
          chosen[r] = 65535 - static_cast<int>(v & 0xFFFFu);
        }
      }
      __syncthreads();
      const uint32_t win = round_best;
#pragma unroll
      for (int j = 0; j < KPL; ++j) key[j] = key[j] == win ? 0u : key[j];
    }
    __syncthreads();
  }

  // Ascending output by rank (k is small), and the mask bits of the chosen tokens.
  for (int j = tid; j < k; j += kPredictThreads) {
    const int mine = chosen[j];
    int rank = 0;
    for (int i = 0; i < k; ++i) rank += chosen[i] < mine ? 1 : 0;
    sink_idx[static_cast<size_t>(b) * k + rank] = mine;
    mask_b[mine] = 1;
  }
}

// One wave per sequence: top k of the slices' candidates, ascending output, mask bits.
__global__ __launch_bounds__(KVS_WAVE) void predict_merge_kernel(
    const uint32_t* __restrict__ slice_keys, int slices, int n, int k, int32_t* __restrict__ sink_idx,
    uint8_t* __restrict__ keep_mask) {
  __shared__ int32_t chosen[kFastK];
  constexpr int CPL = 16 * kFastK / KVS_WAVE;          // at most 16 slices of at most 64 keys
  const int b = blockIdx.x, lane = threadIdx.x;
  const uint32_t* src = slice_keys + static_cast<size_t>(b) * slices * k;
  uint32_t c[CPL];
#pragma unroll
  for (int j = 0; j < CPL; ++j) {
    const int idx = lane + j * KVS_WAVE;
    c[j] = idx < slices * k ? src[idx] : 0u;
  }
  for (int r = 0; r < k; ++r) {
    uint32_t best = 0;
#pragma unroll
    for (int j = 0; j < CPL; ++j) best = c[j] > best ? c[j] : best;
    best = kvs::wave_max_u32(best);
#pragma unroll
    for (int j = 0; j < CPL; ++j) c[j] = c[j] == best ? 0u : c[j];
    if (lane == 0) chosen[r] = 65535 - static_cast<int>(best & 0xFFFFu);
  }
  __syncthreads();
  for (int j = lane; j < k; j += KVS_WAVE) {
    const int mine = chosen[j];
    int rank = 0;
    for (int i = 0; i < k; ++i) rank += chosen[i] < mine ? 1 : 0;
    sink_idx[static_cast<size_t>(b) * k + rank] = mine;
    keep_mask[static_cast<size_t>(b) * n + mine] = 1;
  }
}

template <int KPL>
void launch_predict(int B, hipStream_t s, const uint16_t* hidden, int n, int d, const ChannelList& list, int k,
                    int first_n, int32_t* sink_idx, uint8_t* keep_mask) {
  hipLaunchKernelGGL((predict_sinks_kernel<KPL, false>), dim3(B), dim3(kPredictThreads), 0, s, hidden, n, d, list,
                     k, first_n, sink_idx, keep_mask, 1, static_cast<uint32_t*>(nullptr));
}

constexpr int kSliceTokens = 4 * kPredictThreads;

bool sliced(int n, int k) { return n > kSliceTokens && k >= 1 && k <= kFastK; }

}  // namespace

extern "C" size_t kvs_predict_workspace_bytes(int32_t B, int32_t n, int32_t k) {
  if (B < 1 || n < 1 || k < 0 || !sliced(n, k)) return 0;
  const size_t slices = (static_cast<size_t>(n) + kSliceTokens - 1) / kSliceTokens;
  return ((static_cast<size_t>(B) * slices * k * sizeof(uint32_t)) + 15) & ~static_cast<size_t>(15);
}

// Everything kvs_predict_sinks can refuse on the host, without launching anything.
kvs_status kvs::check_predict_call(const void* hidden, int32_t B, int32_t n, int32_t d, const int32_t* channels,
                                   int32_t n_channels, int32_t k, int32_t first_n, const int32_t* sink_idx,
                                   const uint8_t* keep_mask) {
  if (!hidden || !channels || !keep_mask) return KVS_ERR_INVALID;
  if (B < 1 || n < 1 || d < 1 || n_channels < 1 || k < 0 || first_n < 0) return KVS_ERR_INVALID;
  if (k > n || first_n > n) return KVS_ERR_INVALID;
  if (k > 0 && !sink_idx) return KVS_ERR_INVALID;
  for (int j = 0; j < n_channels && j < kMaxChannels; ++j)
    if (channels[j] < 0 || channels[j] >= d) return KVS_ERR_INVALID;
  if (n_channels > kMaxChannels || k > KVS_MAX_TOPK || n > KVS_MAX_PREDICT_TOKENS)
    return KVS_ERR_UNSUPPORTED;
  return KVS_OK;
}

extern "C" kvs_status kvs_predict_sinks(const void* hidden, int32_t B, int32_t n, int32_t d,
                                         const int32_t* channels, int32_t n_channels, int32_t k,
                                         int32_t first_n, int32_t* sink_idx, uint8_t* keep_mask,
                                         void* workspace, void* stream) {
  const kvs_status st = kvs::check_predict_call(hidden, B, n, d, channels, n_channels, k, first_n, sink_idx, keep_mask);
  if (st != KVS_OK) return st;

  ChannelList list{};
  list.count = n_channels;
  for (int j = 0; j < n_channels; ++j) list.c[j] = channels[j];

  hipStream_t s = static_cast<hipStream_t>(stream);
  const uint16_t* Hp = static_cast<const uint16_t*>(hidden);
  if (sliced(n, k) && workspace) {
    const int slices = (n + kSliceTokens - 1) / kSliceTokens;
    uint32_t* keys = static_cast<uint32_t*>(workspace);
    hipLaunchKernelGGL((predict_sinks_kernel<4, true>), dim3(B * slices), dim3(kPredictThreads), 0, s, Hp, n, d, list,
                       k, first_n, sink_idx, keep_mask, slices, keys);
    hipLaunchKernelGGL(predict_merge_kernel, dim3(B), dim3(KVS_WAVE), 0, s, keys, slices, n, k, sink_idx, keep_mask);
    return hipGetLastError() == hipSuccess ? KVS_OK : KVS_ERR_DEVICE;
  }
  if (n <= 4 * kPredictThreads) launch_predict<4>(B, s, Hp, n, d, list, k, first_n, sink_idx, keep_mask);
  else if (n <= 16 * kPredictThreads) launch_predict<16>(B, s, Hp, n, d, list, k, first_n, sink_idx, keep_mask);
  else launch_predict<64>(B, s, Hp, n, d, list, k, first_n, sink_idx, keep_mask);
  return hipGetLastError() == hipSuccess ? KVS_OK : KVS_ERR_DEVICE;
}

// kvs_decode_attn: decode attention that streams the packed low-bit KV cache and merges the
// fp16 rows of the kept (sink) tokens (paper, Section 2 attention equation; the split of the
// attention sum into sink and non-sink tokens is the equation of Section 4.2).
//
// This file holds the entry points and the small kernels around the stream kernel
// (decode_mfma_impl.h, which every cache goes through):
//   decode_combine_kernel  one wave per (b, hq): log-sum-exp merge of the parts a stream was cut
//       into, then the kept tokens' fp16 rows are folded into the same online softmax,
//       normalise, store fp16.  Not needed when one workgroup covered the whole sequence.
//   residual_part_kernel   the fp16 residual rows of a growing cache as one more part.
// Caches with isolated outliers go the same way: their corrections are part of the stream kernel.
#include <atomic>

#include "decode_finish.h"
#include "kvs_device.h"

namespace {

// Scratch of kvs_decode_attn_noalloc: what the other decode calls take as `workspace`, held by the
// library so that the call needs no allocation.  Every GPU the library runs on holds its own copy
// (at its own address) until the process ends.  In host code the array's name is only a handle
// for hipGetSymbolAddress; the address that kernels, copies and fills take is looked up once per
// device (scratch_of_current_device) and kept.
constexpr size_t kScratchBytes = size_t{KVS_NOALLOC_SCRATCH_BYTES};
static __device__ __align__(256) unsigned char scratch[kScratchBytes];
constexpr int kMaxDevices = 64;
std::atomic<void*> scratch_addr[kMaxDevices];      // device address of `scratch` on each device, null until asked

kvs_status scratch_of_current_device(void** ptr) {
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return KVS_ERR_DEVICE;
  void* p = scratch_addr[dev].load(std::memory_order_acquire);
  if (!p) {                                          // two threads may both ask: they get the same answer
    if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) return KVS_ERR_DEVICE;
    scratch_addr[dev].store(p, std::memory_order_release);
  }
  *ptr = p;
  return KVS_OK;
}

__global__ void clear_words_kernel(uint32_t* __restrict__ p, int n) {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) p[i] = 0;
}

constexpr int kWaves = 4;
constexpr int kThreads = kWaves * KVS_WAVE;
constexpr float kRsqrtD = 0.08838834764831845f;   // 1 / sqrt(128)
constexpr int kWsRow = KVS_HEAD_DIM + 2;          // output row, running max, running sum

// One wave per (b, hq): the parts a stream kernel left in the workspace, the extra part and the
// kept rows into one output row (finish_row).  Only needed when no stream kernel ran at all (a
// growing cache that still holds fewer than 128 tokens: splits == 0); a stream cut into parts is
// finished by its own last-arriving workgroup.
__global__ __launch_bounds__(KVS_WAVE) void decode_combine_kernel(
    const uint16_t* __restrict__ q, const float* __restrict__ ws, const float* __restrict__ extra, int splits, int Hq, int Hkv,
    int cap, const uint16_t* __restrict__ keep_k, const uint16_t* __restrict__ keep_v,
    const int32_t* __restrict__ keep_cnt, uint16_t* __restrict__ out, float* __restrict__ lse) {
  const int lane = threadIdx.x;
  const size_t bq = blockIdx.x;                       // b * Hq + hq
  const int b = static_cast<int>(bq / Hq), hq = static_cast<int>(bq % Hq);
  const int h = hq / (Hq / Hkv);
  const int cnt = min(keep_cnt[b], cap);
  const uint32_t q2 = reinterpret_cast<const uint32_t*>(q + bq * 128)[lane];
  const uint32_t* kk = reinterpret_cast<const uint32_t*>(keep_k) + (static_cast<size_t>(b) * Hkv + h) * cap * 64 + lane;
  const uint32_t* kv = reinterpret_cast<const uint32_t*>(keep_v) + (static_cast<size_t>(b) * Hkv + h) * cap * 64 + lane;
  kvs::finish_row<false>(q2, ws + bq * splits * kWsRow, splits, extra ? extra + bq * kWsRow : nullptr, kk, kv, cnt,
                  reinterpret_cast<uint32_t*>(out + bq * 128), lse ? lse + bq : nullptr, lane);
}

}  // namespace

// The residual window of a growing cache as one more part: softmax state of `rows` fp16 rows of one
// (b, hq), unnormalised.  One workgroup of four waves per (b, hq); wave w takes rows w, w + 4, ...
// eight at a time (their loads in flight together); lane = channels 2 lane, 2 lane + 1.
__global__ __launch_bounds__(kThreads) void residual_part_kernel(
    const uint16_t* __restrict__ q, const uint16_t* __restrict__ res_k, const uint16_t* __restrict__ res_v,
    int rows, int Hq, int Hkv, float* __restrict__ extra) {
  __shared__ float part_o[kWaves][128];
  __shared__ float part_m[kWaves], part_l[kWaves];
  const int lane = threadIdx.x & (KVS_WAVE - 1), wave = threadIdx.x / KVS_WAVE;
  const size_t bq = blockIdx.x;
  const int b = static_cast<int>(bq / Hq), hq = static_cast<int>(bq % Hq);
  const size_t bh = static_cast<size_t>(b) * Hkv + hq / (Hq / Hkv);
  const uint32_t q2 = reinterpret_cast<const uint32_t*>(q + bq * 128)[lane];
  const float q0 = kvs::half_bits_to_float(static_cast<uint16_t>(q2 & 0xFFFFu)) * kRsqrtD;
  const float q1 = kvs::half_bits_to_float(static_cast<uint16_t>(q2 >> 16)) * kRsqrtD;
  const uint32_t* kk = reinterpret_cast<const uint32_t*>(res_k) + bh * KVS_V_TILE * 64 + lane;
  const uint32_t* kv = reinterpret_cast<const uint32_t*>(res_v) + bh * KVS_V_TILE * 64 + lane;
  constexpr int kBatch = 8;
  float M = -INFINITY, L = 0.0f, O0 = 0.0f, O1 = 0.0f;
  for (int r0 = wave; r0 < rows; r0 += kWaves * kBatch) {
    uint32_t kw[kBatch], vw[kBatch];
#pragma unroll
    for (int u = 0; u < kBatch; ++u) {
      const int r = min(r0 + u * kWaves, rows - 1);
      kw[u] = kk[r * 64];
      vw[u] = kv[r * 64];
    }
#pragma unroll
    for (int u = 0; u < kBatch; ++u) {
      if (r0 + u * kWaves < rows) {                   // wave-uniform
        const float s = kvs::wave_sum(q0 * kvs::half_bits_to_float(static_cast<uint16_t>(kw[u] & 0xFFFFu)) +
                                      q1 * kvs::half_bits_to_float(static_cast<uint16_t>(kw[u] >> 16)));
        const float m_new = fmaxf(M, s);
        const float alpha = M == -INFINITY ? 0.0f : __expf(M - m_new);
        const float p = __expf(s - m_new);
        L = L * alpha + p;
        O0 = O0 * alpha + p * kvs::half_bits_to_float(static_cast<uint16_t>(vw[u] & 0xFFFFu));
        O1 = O1 * alpha + p * kvs::half_bits_to_float(static_cast<uint16_t>(vw[u] >> 16));
        M = m_new;
      }
    }
  }
  reinterpret_cast<float2*>(&part_o[wave][0])[lane] = float2{O0, O1};
  if (lane == 0) { part_m[wave] = M; part_l[wave] = L; }
  __syncthreads();
  if (wave == 0) {
    float Mx = -INFINITY;
#pragma unroll
    for (int w = 0; w < kWaves; ++w) Mx = fmaxf(Mx, part_m[w]);
    float Ls = 0.0f, A0 = 0.0f, A1 = 0.0f;
#pragma unroll
    for (int w = 0; w < kWaves; ++w) {
      const float f = part_m[w] == -INFINITY ? 0.0f : __expf(part_m[w] - Mx);
      const float2 o = reinterpret_cast<const float2*>(&part_o[w][0])[lane];
      Ls += part_l[w] * f;
      A0 += o.x * f;
      A1 += o.y * f;
    }
    float* dst = extra + bq * kWsRow;
    reinterpret_cast<float2*>(dst)[lane] = float2{A0, A1};
    if (lane == 0) { dst[128] = Mx; dst[129] = Ls; }
  }
}

static kvs_status check_decode_args(const kvs_desc* desc, const void* q, const kvs_cache* cache, const void* out) {
  const kvs_status st = kvs::validate_desc(desc);
  if (st != KVS_OK) return st;
  if (!q || !cache || !out) return KVS_ERR_INVALID;
  if (!cache->k_codes || !cache->v_codes || !cache->k_params || !cache->v_params ||
      !cache->keep_cnt || !cache->keep_mask)
    return KVS_ERR_INVALID;
  if (desc->keep_cap > 0 && (!cache->keep_k || !cache->keep_v)) return KVS_ERR_INVALID;
  if (desc->sparse_frac > 0.0f && (!cache->k_rowptr || !cache->k_col || !cache->k_val ||
                                   !cache->v_rowptr || !cache->v_col || !cache->v_val))
    return KVS_ERR_INVALID;
  // The stream is read 16 bytes a lane, CSR entries four (8 bytes) at a time.
  const auto misaligned = [](const void* p, uintptr_t to) { return (reinterpret_cast<uintptr_t>(p) & (to - 1)) != 0; };
  if (misaligned(cache->k_codes, 16) || misaligned(cache->v_codes, 16) || misaligned(cache->keep_k, 16) ||
      misaligned(cache->keep_v, 16) || misaligned(cache->k_params, 8) || misaligned(cache->v_params, 4))
    return KVS_ERR_INVALID;
  if (desc->sparse_frac > 0.0f && (misaligned(cache->k_col, 8) || misaligned(cache->k_val, 8) ||
                                   misaligned(cache->v_col, 8) || misaligned(cache->v_val, 8)))
    return KVS_ERR_INVALID;
  return KVS_OK;
}

// Dense caches: the first n_used tokens (whole blocks) through the stream kernel, which also
// finishes the rows (kept rows, the residual rows' part when there is one) whether one workgroup
// or several cover a head.  Only a cache without a single whole block takes the combine kernel.
static void decode_dense(const kvs_desc* desc, const void* q, const kvs_cache* cache, int n_used, const float* extra,
                         void* out, float* lse, float* ws, int* arrive, hipStream_t s) {
  if (n_used > 0) {
    const kvs::DecodeGeometry geo = kvs::decode_geometry(desc, n_used);
    kvs::launch_decode_mfma(desc, geo, q, cache, out, lse, ws, arrive, n_used, extra, s);
    return;
  }
  hipLaunchKernelGGL(decode_combine_kernel, dim3(desc->B * desc->Hq), dim3(KVS_WAVE), 0, s,
                     static_cast<const uint16_t*>(q), ws, extra, 0, desc->Hq, desc->Hkv, desc->keep_cap,
                     static_cast<const uint16_t*>(cache->keep_k), static_cast<const uint16_t*>(cache->keep_v),
                     cache->keep_cnt, static_cast<uint16_t*>(out), lse);
}

extern "C" kvs_status kvs_decode_attn(const kvs_desc* desc, const void* q, const kvs_cache* cache,
                                       void* out, float* lse, void* workspace, void* stream) {
  const kvs_status st = check_decode_args(desc, q, cache, out);
  if (st != KVS_OK) return st;
  if (!workspace) return KVS_ERR_INVALID;
  hipStream_t s = static_cast<hipStream_t>(stream);
  int* arrive = static_cast<int*>(workspace);
  float* ws = static_cast<float*>(workspace) + kvs::workspace_counter_words(desc);
  decode_dense(desc, q, cache, desc->n, nullptr, out, lse, ws, arrive, s);
  return hipGetLastError() == hipSuccess ? KVS_OK : KVS_ERR_DEVICE;
}

// kvs_decode_attn for callers that cannot allocate: the same kernels, with the library's own
// scratch array in place of the caller's workspace.
extern "C" kvs_status kvs_decode_attn_noalloc(const kvs_desc* desc, const void* q, const kvs_cache* cache,
                                               void* out, float* lse, void* stream) {
  const kvs_status st = check_decode_args(desc, q, cache, out);
  if (st != KVS_OK) return st;
  if (kvs::decode_workspace_bytes(desc) > kScratchBytes) return KVS_ERR_SCRATCH;
  void* ws = nullptr;
  const kvs_status sp = scratch_of_current_device(&ws);
  if (sp != KVS_OK) return sp;
  // The array keeps what the last call on this GPU left.  A finished call leaves the arrival
  // counters at its head zero; an interrupted one may not have, so they are cleared first - by a
  // kernel, which a graph capture records like any other launch.
  const int words = static_cast<int>(kvs::workspace_counter_words(desc));
  hipLaunchKernelGGL(clear_words_kernel, dim3((words + 255) / 256), dim3(256), 0, static_cast<hipStream_t>(stream),
                     static_cast<uint32_t*>(ws), words);
  return kvs_decode_attn(desc, q, cache, out, lse, ws, stream);
}

extern "C" kvs_status kvs_decode_attn_n(const kvs_desc* desc, const void* q, const kvs_cache* cache, int32_t n_tokens,
                                         void* out, float* lse, void* workspace, void* stream) {
  const kvs_status st = check_decode_args(desc, q, cache, out);
  if (st != KVS_OK) return st;
  if (!workspace) return KVS_ERR_INVALID;
  if (desc->sparse_frac > 0.0f) return KVS_ERR_UNSUPPORTED;
  if (n_tokens < 1 || n_tokens > desc->n) return KVS_ERR_INVALID;
  hipStream_t s = static_cast<hipStream_t>(stream);
  int* arrive = static_cast<int*>(workspace);
  float* ws = static_cast<float*>(workspace) + kvs::workspace_counter_words(desc);
  const int n_used = (n_tokens / KVS_V_TILE) * KVS_V_TILE;
  const int rows = n_tokens - n_used;
  float* extra = nullptr;
  if (rows > 0) {
    if (!cache->res_k || !cache->res_v) return KVS_ERR_INVALID;
    // behind the parts of the stream kernels (sized for the most splits any token count can get)
    extra = ws + static_cast<size_t>(desc->B) * desc->Hq * kvs::decode_max_splits(desc) * kWsRow;
    hipLaunchKernelGGL(residual_part_kernel, dim3(desc->B * desc->Hq), dim3(kThreads), 0, s,
                       static_cast<const uint16_t*>(q), static_cast<const uint16_t*>(cache->res_k),
                       static_cast<const uint16_t*>(cache->res_v), rows, desc->Hq, desc->Hkv, extra);
  }
  decode_dense(desc, q, cache, n_used, extra, out, lse, ws, arrive, s);
  return hipGetLastError() == hipSuccess ? KVS_OK : KVS_ERR_DEVICE;
}

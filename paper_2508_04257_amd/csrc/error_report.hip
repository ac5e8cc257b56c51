// kvs_quant_error: quantisation-error report with the structure of the paper's Table 1
// (Section 4.1): the squared error of every cache entry of a non-kept token, summed separately
// over the quantisation groups that contain a flagged (sink) token and those that do not, for
// Keys and for Values.  A per-channel Key group is G consecutive tokens of one channel; a
// per-token group (Values, and Keys under the per-token scheme) is G channels of one token.
//
// One workgroup per (sequence, KV head, 128-token tile) and tensor.  A lane owns 8 channels of
// rows rslot, rslot + 16, ...: it reads the fp16 row once (the only large traffic, 2 bytes per
// element), takes the codes and parameter words from the cache (a quarter of that or less, and
// mostly cache hits: neighbouring lanes share words), forms x - scale (code - zero) with the
// product in fp32 - the value the decode step sees - and the difference and its square in fp64.
// Sums go through LDS into one double atomic per workgroup and class.
#include "kvs_device.h"

namespace {

using kvs::Fmt;

constexpr int kThreads = 256;

struct Report {            // the 64-byte report the caller reads
  double sse[2][2];        // [tensor: 0 Keys, 1 Values][class: 0 without, 1 with a flagged token]
  unsigned long long count[2][2];
};

__global__ void report_reset_kernel(Report* r) {
  if (threadIdx.x < 4) {
    (&r->sse[0][0])[threadIdx.x] = 0.0;
    (&r->count[0][0])[threadIdx.x] = 0ull;
  }
}

template <int BITS>
__global__ __launch_bounds__(kThreads) void quant_error_kernel(
    const uint16_t* __restrict__ K, const uint16_t* __restrict__ V, const uint32_t* __restrict__ k_codes,
    const uint32_t* __restrict__ v_codes, const uint32_t* __restrict__ k_params, const uint32_t* __restrict__ v_params,
    const uint8_t* __restrict__ keep_mask, const uint8_t* __restrict__ sink_mask, int n, int Hkv, int G,
    int key_per_token, Report* __restrict__ report) {
  constexpr int W = Fmt<BITS>::W, cpw = Fmt<BITS>::cpw;
  constexpr uint32_t qmask = static_cast<uint32_t>(Fmt<BITS>::qmax);
  __shared__ uint8_t flag_s[128], kept_s[128], group_s[4];
  __shared__ double red_sse[kThreads / KVS_WAVE][2];
  __shared__ unsigned int red_cnt[kThreads / KVS_WAVE][2];

  const int tid = threadIdx.x, chunk = tid & 15, rslot = tid >> 4;
  const int tiles = n / KVS_V_TILE;
  const int tile = blockIdx.x % tiles;
  const size_t bh = blockIdx.x / tiles;
  const int b = static_cast<int>(bh / Hkv);
  const int tensor = blockIdx.y;                       // 0: Keys, 1: Values
  const int t0 = tile * KVS_V_TILE;
  const int NGC = 128 / G;

  if (tid < 128) {
    flag_s[tid] = sink_mask[static_cast<size_t>(b) * n + t0 + tid] != 0;
    kept_s[tid] = keep_mask[static_cast<size_t>(b) * n + t0 + tid] != 0;
  }
  __syncthreads();
  if (tid < 128 / G) {                                 // does the token group hold a flagged token?
    uint8_t any = 0;
    for (int i = 0; i < G; ++i) any |= flag_s[tid * G + i];
    group_s[tid] = any;
  }
  __syncthreads();

  const bool per_token = tensor == 1 || key_per_token != 0;
  const uint16_t* X = (tensor == 0 ? K : V) + (bh * n + t0) * 128;
  const uint32_t* params = tensor == 0 ? k_params : v_params;
  double sse[2] = {0.0, 0.0};
  unsigned int cnt[2] = {0u, 0u};
  for (int i = 0; i < 8; ++i) {
    const int r = rslot + 16 * i;                      // token of the tile
    if (kept_s[r]) continue;                           // stored exactly: not part of the report
    const int cls = per_token ? flag_s[r] : group_s[r / G];
    const uint4 raw = *reinterpret_cast<const uint4*>(X + r * 128 + 8 * chunk);
    const uint32_t w4[4] = {raw.x, raw.y, raw.z, raw.w};
    double acc = 0.0;
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      const int c = 8 * chunk + j;
      uint32_t word;
      int slot;
      if (tensor == 0) {                               // Key word (T, w, t): channels cpw w .. of token 64 T + t
        const int t = t0 + r;
        word = k_codes[(bh * (n / KVS_K_TILE) + t / KVS_K_TILE) * (W * KVS_K_TILE) + (c / cpw) * KVS_K_TILE + t % KVS_K_TILE];
        slot = c % cpw;
      } else {                                         // Value word (T, u, c): tokens 128 T + cpw u .. of channel c
        word = v_codes[(bh * tiles + tile) * (W * 128) + (r / cpw) * 128 + c];
        slot = r % cpw;
      }
      const int code = static_cast<int>((word >> Fmt<BITS>::shift(slot)) & qmask);
      const uint32_t pw = per_token ? params[(bh * n + t0 + r) * NGC + c / G]
                                    : params[(bh * (n / G) + (t0 + r) / G) * 128 + c];
      float scale;
      int zero;
      kvs::unpack_param(pw, scale, zero);
      const float deq = scale * static_cast<float>(code - zero);
      const uint16_t hbits = static_cast<uint16_t>(j & 1 ? w4[j >> 1] >> 16 : w4[j >> 1] & 0xFFFFu);
      const double e = static_cast<double>(kvs::half_bits_to_float(hbits)) - static_cast<double>(deq);
      acc += e * e;
    }
    sse[cls] += acc;
    cnt[cls] += 8;
  }

  // wave sums (plain shuffles: this is not a hot loop), then one atomic per workgroup and class
  for (int c = 0; c < 2; ++c) {
    double s = sse[c];
    unsigned int k = cnt[c];
    for (int o = KVS_WAVE / 2; o > 0; o >>= 1) {
      s += __shfl_xor(s, o, KVS_WAVE);
      k += __shfl_xor(k, o, KVS_WAVE);
    }
    if ((tid & (KVS_WAVE - 1)) == 0) { red_sse[tid / KVS_WAVE][c] = s; red_cnt[tid / KVS_WAVE][c] = k; }
  }
  __syncthreads();
  if (tid < 2) {
    double s = 0.0;
    unsigned long long k = 0;
    for (int w = 0; w < kThreads / KVS_WAVE; ++w) { s += red_sse[w][tid]; k += red_cnt[w][tid]; }
    if (k) {
      atomicAdd(&report->sse[tensor][tid], s);
      atomicAdd(&report->count[tensor][tid], k);
    }
  }
}

}  // namespace

extern "C" kvs_status kvs_quant_error(const kvs_desc* desc, const void* K, const void* V, const kvs_cache* cache,
                                       const uint8_t* sink_mask, void* report, void* stream) {
  const kvs_status st = kvs::validate_desc(desc);
  if (st != KVS_OK) return st;
  if (desc->sparse_frac > 0.0f) return KVS_ERR_UNSUPPORTED;
  if (!K || !V || !cache || !sink_mask || !report) return KVS_ERR_INVALID;
  if (!cache->k_codes || !cache->v_codes || !cache->k_params || !cache->v_params || !cache->keep_mask)
    return KVS_ERR_INVALID;
  hipStream_t s = static_cast<hipStream_t>(stream);
  Report* r = static_cast<Report*>(report);
  hipLaunchKernelGGL(report_reset_kernel, dim3(1), dim3(64), 0, s, r);
  const dim3 grid(desc->B * desc->Hkv * (desc->n / KVS_V_TILE), 2), block(kThreads);
  const uint16_t* Kp = static_cast<const uint16_t*>(K);
  const uint16_t* Vp = static_cast<const uint16_t*>(V);
#define KVS_LAUNCH_REPORT(BITS)                                                                                  \
  hipLaunchKernelGGL(quant_error_kernel<BITS>, grid, block, 0, s, Kp, Vp, cache->k_codes, cache->v_codes,       \
                     cache->k_params, cache->v_params, cache->keep_mask, sink_mask, desc->n, desc->Hkv, desc->group, \
                     desc->key_per_token, r)
  if (desc->bits == 2) KVS_LAUNCH_REPORT(2);
  else if (desc->bits == 3) KVS_LAUNCH_REPORT(3);
  else KVS_LAUNCH_REPORT(4);
#undef KVS_LAUNCH_REPORT
  return hipGetLastError() == hipSuccess ? KVS_OK : KVS_ERR_DEVICE;
}

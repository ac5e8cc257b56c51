// kvs_quant_error: quantisation-error report with the structure of the paper's Table 1
// (Section 4.1): the squared error of every cache entry of a non-kept token, summed separately
// over the quantisation groups that contain a flagged (sink) token and those that do not, for
// Keys and for Values.  A per-channel Key group is G consecutive tokens of one channel; a
// per-token group (Values, and Keys under the per-token scheme) is G channels of one token.
//
// Workgroups walk (sequence, KV head, 128-token tile) blocks of one tensor.  A lane owns 8
// channels of rows rslot, rslot + 16, ...: it reads the fp16 row once (the only large traffic,
// 2 bytes per element), takes the words that hold its eight codes and its parameter words from the
// cache, forms x - scale (code - zero) with the product in fp32 - the value the decode step sees -
// and the difference and its square in fp64.  Sums go through LDS into one double atomic per
// workgroup and class.
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
    int key_per_token, int total_tiles, Report* __restrict__ report) {
  constexpr int W = Fmt<BITS>::W, cpw = Fmt<BITS>::cpw;
  constexpr uint32_t qmask = static_cast<uint32_t>(Fmt<BITS>::qmax);
  __shared__ uint8_t flag_s[128], kept_s[128], group_s[4];
  __shared__ double red_sse[kThreads / KVS_WAVE][2];
  __shared__ unsigned int red_cnt[kThreads / KVS_WAVE][2];

  const int tid = threadIdx.x, chunk = tid & 15, rslot = tid >> 4;
  const int tiles = n / KVS_V_TILE;
  const int tensor = blockIdx.y;                       // 0: Keys, 1: Values
  const int NGC = 128 / G;
  const bool per_token = tensor == 1 || key_per_token != 0;
  const uint32_t* params = tensor == 0 ? k_params : v_params;
  double sse[2] = {0.0, 0.0};
  unsigned int cnt[2] = {0u, 0u};

  // A workgroup walks several (sequence, KV head, tile) blocks: one pair of atomics per workgroup
  // and class at the end, not per block (thousands of atomics on one address serialise).
  for (int blk = blockIdx.x; blk < total_tiles; blk += gridDim.x) {
    const int tile = blk % tiles;
    const size_t bh = blk / tiles;
    const int b = static_cast<int>(bh / Hkv);
    const int t0 = tile * KVS_V_TILE;
    __syncthreads();                                   // the flags of the previous block are no longer read
    if (tid < 128) {
      flag_s[tid] = sink_mask[static_cast<size_t>(b) * n + t0 + tid] != 0;
      kept_s[tid] = keep_mask[static_cast<size_t>(b) * n + t0 + tid] != 0;
    }
    __syncthreads();
    if (tid < 128 / G) {                               // does the token group hold a flagged token?
      uint8_t any = 0;
      for (int i = 0; i < G; ++i) any |= flag_s[tid * G + i];
      group_s[tid] = any;
    }
    __syncthreads();

    const uint16_t* X = (tensor == 0 ? K : V) + (bh * n + t0) * 128;
#pragma unroll 2
    for (int i = 0; i < 8; ++i) {
      const int r = rslot + 16 * i;                    // token of the tile
      if (kept_s[r]) continue;                         // stored exactly: not part of the report
      const int cls = per_token ? flag_s[r] : group_s[r / G];
      const uint4 raw = *reinterpret_cast<const uint4*>(X + r * 128 + 8 * chunk);
      const uint32_t w4[4] = {raw.x, raw.y, raw.z, raw.w};
      // The lane's eight codes: for Keys they sit in one or two words of the token's row (channels
      // cpw w ..), for Values in one word per channel (tokens cpw u ..).
      uint32_t cw[8];
      int slot[8];
      if (tensor == 0) {
        const int t = t0 + r;
        const uint32_t* row = k_codes + (bh * (n / KVS_K_TILE) + t / KVS_K_TILE) * (W * KVS_K_TILE) + t % KVS_K_TILE;
        const int w_lo = (8 * chunk) / cpw, w_hi = (8 * chunk + 7) / cpw;
        const uint32_t lo = row[w_lo * KVS_K_TILE], hi = w_hi != w_lo ? row[w_hi * KVS_K_TILE] : lo;
#pragma unroll
        for (int j = 0; j < 8; ++j) {
          const int c = 8 * chunk + j;
          cw[j] = c / cpw == w_lo ? lo : hi;
          slot[j] = c % cpw;
        }
      } else {
        const uint4* words = reinterpret_cast<const uint4*>(v_codes + (bh * tiles + tile) * (W * 128) + (r / cpw) * 128 + 8 * chunk);
        const uint4 a = words[0], c2 = words[1];
        cw[0] = a.x; cw[1] = a.y; cw[2] = a.z; cw[3] = a.w; cw[4] = c2.x; cw[5] = c2.y; cw[6] = c2.z; cw[7] = c2.w;
#pragma unroll
        for (int j = 0; j < 8; ++j) slot[j] = r % cpw;
      }
      uint32_t pw[8];
      if (per_token) {                                 // one word for the lane's eight channels (G >= 32)
        const uint32_t p = params[(bh * n + t0 + r) * NGC + (8 * chunk) / G];
#pragma unroll
        for (int j = 0; j < 8; ++j) pw[j] = p;
      } else {
        const uint4* pp = reinterpret_cast<const uint4*>(params + (bh * (n / G) + (t0 + r) / G) * 128 + 8 * chunk);
        const uint4 a = pp[0], c2 = pp[1];
        pw[0] = a.x; pw[1] = a.y; pw[2] = a.z; pw[3] = a.w; pw[4] = c2.x; pw[5] = c2.y; pw[6] = c2.z; pw[7] = c2.w;
      }
      double acc = 0.0;
#pragma unroll
      for (int j = 0; j < 8; ++j) {
        const int code = static_cast<int>((cw[j] >> Fmt<BITS>::shift(slot[j])) & qmask);
        float scale;
        int zero;
        kvs::unpack_param(pw[j], scale, zero);
        const float deq = scale * static_cast<float>(code - zero);
        const uint16_t hbits = static_cast<uint16_t>(j & 1 ? w4[j >> 1] >> 16 : w4[j >> 1] & 0xFFFFu);
        const double e = static_cast<double>(kvs::half_bits_to_float(hbits)) - static_cast<double>(deq);
        acc += e * e;
      }
      sse[cls] += acc;
      cnt[cls] += 8;
    }
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
  const int total_tiles = desc->B * desc->Hkv * (desc->n / KVS_V_TILE);
  const dim3 grid(total_tiles < 2048 ? total_tiles : 2048, 2), block(kThreads);
  const uint16_t* Kp = static_cast<const uint16_t*>(K);
  const uint16_t* Vp = static_cast<const uint16_t*>(V);
#define KVS_LAUNCH_REPORT(BITS)                                                                                  \
  hipLaunchKernelGGL(quant_error_kernel<BITS>, grid, block, 0, s, Kp, Vp, cache->k_codes, cache->v_codes,       \
                     cache->k_params, cache->v_params, cache->keep_mask, sink_mask, desc->n, desc->Hkv, desc->group, \
                     desc->key_per_token, total_tiles, r)
  if (desc->bits == 2) KVS_LAUNCH_REPORT(2);
  else if (desc->bits == 3) KVS_LAUNCH_REPORT(3);
  else if (desc->bits == 4) KVS_LAUNCH_REPORT(4);
  else KVS_LAUNCH_REPORT(8);
#undef KVS_LAUNCH_REPORT
  return hipGetLastError() == hipSuccess ? KVS_OK : KVS_ERR_DEVICE;
}

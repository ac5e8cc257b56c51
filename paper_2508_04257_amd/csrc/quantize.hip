// kvs_quantize_kv: sink-preserving low-bit KV-cache quantisation (paper, Appendix C equations
// for Q(X), scale and zero; Algorithm 1's two quantise steps; Section 4.1 for the per-channel
// Key / per-token Value grouping).
//
// Every kernel here is bound by the fp16 read of K and V (2 bytes per element in, bits/8 out).
// A workgroup of 256 lanes owns one token block of one (sequence, KV head): each lane loads
// 8 consecutive channels (one 128-bit load) of 8 or 4 rows, statistics are reduced along the
// group axis (LDS for the Key's token axis, cross-lane for the Value's channel axis), codes are
// staged as bytes in LDS and packed into words whose global order is contiguous per workgroup.
//
// The quantiser arithmetic is the exact fp32 sequence the ABI header documents; this file is
// compiled with floating-point contraction off so that no multiply-add fuses across it.
#include "kvs_device.h"

namespace {

using kvs::Fmt;

constexpr int kThreads = 256;
constexpr int kRowStride = 132;   // bytes per staged code row: 128 + 4 keeps LDS banks spread

struct GroupParam {
  float inv;    // 1 / scale, fp32
  int zero;
  uint32_t word;
};

// scale / zero of one group from its unmasked minimum and maximum (count == 0: empty group).
template <int BITS>
__device__ inline GroupParam make_param(float mn, float mx, bool any) {
  constexpr float qmax = static_cast<float>(Fmt<BITS>::qmax);
  if (!any) { mn = 0.0f; mx = 0.0f; }
  uint16_t hbits;
  if (mx == mn) {
    const float a = mn != 0.0f ? fabsf(mn) : 1.0f;    // exactly representable in fp16
    hbits = kvs::float_to_half_bits_rn(a);
  } else {
    const float s32 = (mx - mn) / qmax;
    hbits = kvs::float_to_half_bits_rn(s32);
    if (kvs::half_bits_to_float(hbits) < s32) hbits += 1;   // next fp16 up (positive values)
  }
  const float s = kvs::half_bits_to_float(hbits);
  GroupParam p;
  p.inv = 1.0f / s;
  p.zero = -static_cast<int>(rintf(mn * p.inv));
  p.word = static_cast<uint32_t>(hbits) | (static_cast<uint32_t>(p.zero & 0xFFFF) << 16);
  return p;
}

template <int BITS>
__device__ inline uint32_t quantize_one(float x, float inv, int zero, bool masked) {
  int c = static_cast<int>(rintf(x * inv)) + zero;
  c = c < 0 ? 0 : (c > Fmt<BITS>::qmax ? Fmt<BITS>::qmax : c);
  return masked ? 0u : static_cast<uint32_t>(c);
}

__device__ inline void unpack8(const uint4& raw, uint16_t h[8]) {
  h[0] = raw.x & 0xFFFF; h[1] = raw.x >> 16; h[2] = raw.y & 0xFFFF; h[3] = raw.y >> 16;
  h[4] = raw.z & 0xFFFF; h[5] = raw.z >> 16; h[6] = raw.w & 0xFFFF; h[7] = raw.w >> 16;
}

// ---------------------------------------------------------------------------------------------
// Keys: per channel, groups of G consecutive tokens.  Block = TB = max(G, 64) tokens.
// ---------------------------------------------------------------------------------------------
template <int BITS, int G>
__global__ __launch_bounds__(kThreads) void quantize_k_kernel(
    const uint4* __restrict__ K, const uint8_t* __restrict__ keep_mask, kvs::QuantSpan sp, int Hkv,
    const uint32_t* __restrict__ tau_ptr, uint32_t* __restrict__ k_codes, uint32_t* __restrict__ k_params,
    int32_t* __restrict__ row_count, kvs::SparseEmit emit) {
  constexpr int TB = G > 64 ? G : 64;
  constexpr int NG = TB / G;             // groups per block: 1 or 2
  constexpr int ROWS = TB / 16;          // rows per lane
  constexpr int W = Fmt<BITS>::W, cpw = Fmt<BITS>::cpw;

  __shared__ float red_min[NG][16][128];
  __shared__ float red_max[NG][16][128];
  __shared__ float inv_s[NG][128];
  __shared__ int zero_s[NG][128];
  __shared__ __align__(16) uint8_t code_s[TB * kRowStride];
  // Dense-and-sparse only: which entries of each row are isolated (128 bits per row), where the
  // row's entries start inside the block's run, and where that run starts in the staging list.
  __shared__ uint32_t iso_s[TB][4];
  __shared__ int row_off_s[TB];
  __shared__ int run_base_s;

  const int tid = threadIdx.x;
  const int chunk = tid & 15;            // channels 8*chunk .. 8*chunk+7
  const int rslot = tid >> 4;            // rows rslot, rslot+16, ...
  const uint32_t tau = tau_ptr ? *tau_ptr : 0x8000u;   // 0x8000: no magnitude pattern reaches it
  if (row_count) {
    for (int i = tid; i < TB * 4; i += kThreads) (&iso_s[0][0])[i] = 0;
    __syncthreads();
  }
  const int blocks_per_head = sp.n_tokens / TB;
  const int blk = blockIdx.x % blocks_per_head;
  const size_t bh = blockIdx.x / blocks_per_head;       // b * Hkv + h
  const int b = static_cast<int>(bh / Hkv);
  const int n = sp.n_cap;                               // layout of everything written
  const int t0 = sp.t_out + blk * TB;                   // cache token of the block's first row

  const uint4* src = K + (bh * sp.n_in + blk * TB) * 16;   // 16 uint4 per 128-channel row
  const uint8_t* mask_b = keep_mask + static_cast<size_t>(b) * sp.mask_stride + sp.mask_t0 + blk * TB;

  uint4 raw[ROWS];
  bool kept[ROWS];
#pragma unroll
  for (int i = 0; i < ROWS; ++i) {
    const int r = rslot + 16 * i;
    raw[i] = src[r * 16 + chunk];
    kept[i] = mask_b[r] != 0;
  }

  // Lane-local min / max per channel and per group, over the unmasked entries.
  float mn[NG][8], mx[NG][8];
#pragma unroll
  for (int g = 0; g < NG; ++g)
#pragma unroll
    for (int j = 0; j < 8; ++j) { mn[g][j] = INFINITY; mx[g][j] = -INFINITY; }
#pragma unroll
  for (int i = 0; i < ROWS; ++i) {
    constexpr int rows_per_group = G / 16;
    const int g = i / rows_per_group;     // compile-time after unrolling
    uint16_t h[8];
    unpack8(raw[i], h);
    uint32_t bits = 0;                    // isolated entries of this row piece
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      const bool iso = !kept[i] && (h[j] & 0x7FFFu) >= tau;
      const bool masked = kept[i] || iso;
      const float x = kvs::half_bits_to_float(h[j]);
      mn[g][j] = masked ? mn[g][j] : fminf(mn[g][j], x);
      mx[g][j] = masked ? mx[g][j] : fmaxf(mx[g][j], x);
      bits |= iso ? 1u << j : 0u;
    }
    if (row_count && bits) atomicOr(&iso_s[rslot + 16 * i][chunk >> 2], bits << (8 * (chunk & 3)));
  }
#pragma unroll
  for (int g = 0; g < NG; ++g)
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      red_min[g][rslot][8 * chunk + j] = mn[g][j];
      red_max[g][rslot][8 * chunk + j] = mx[g][j];
    }
  __syncthreads();

  // One lane per (group, channel): finish the reduction, derive scale / zero, publish.
  if (tid < NG * 128) {
    const int g = tid >> 7, c = tid & 127;
    float a = INFINITY, z = -INFINITY;
#pragma unroll
    for (int s = 0; s < 16; ++s) {
      a = fminf(a, red_min[g][s][c]);
      z = fmaxf(z, red_max[g][s][c]);
    }
    const GroupParam p = make_param<BITS>(a, z, a <= z);
    inv_s[g][c] = p.inv;
    zero_s[g][c] = p.zero;
    k_params[(bh * (n / G) + static_cast<size_t>(t0 / G + g)) * 128 + c] = p.word;
  }
  if (row_count && tid >= kThreads - KVS_WAVE) {
    // Meanwhile the last wave: row counts (CSR row = token), their exclusive scan over the block,
    // and one claim in the staging list for the block's whole run.
    const int lane = tid - (kThreads - KVS_WAVE);
    int cnt[TB / KVS_WAVE], mine = 0;
#pragma unroll
    for (int k = 0; k < TB / KVS_WAVE; ++k) {
      const int r = lane * (TB / KVS_WAVE) + k;
      cnt[k] = __popc(iso_s[r][0]) + __popc(iso_s[r][1]) + __popc(iso_s[r][2]) + __popc(iso_s[r][3]);
      row_count[bh * n + t0 + r] = cnt[k];
      mine += cnt[k];
    }
    int incl = mine;
#pragma unroll
    for (int o = 1; o < KVS_WAVE; o <<= 1) {
      const int up = __shfl_up(incl, o, KVS_WAVE);
      if (lane >= o) incl += up;
    }
    int run = incl - mine;
#pragma unroll
    for (int k = 0; k < TB / KVS_WAVE; ++k) { row_off_s[lane * (TB / KVS_WAVE) + k] = run; run += cnt[k]; }
    if (lane == KVS_WAVE - 1) {
      const int base = incl > 0 ? atomicAdd(emit.counter, incl) : 0;
      emit.block_base[blockIdx.x] = base;
      run_base_s = base;
    }
  }
  __syncthreads();

  // Codes of the lane's entries -> bytes in LDS.
#pragma unroll
  for (int i = 0; i < ROWS; ++i) {
    constexpr int rows_per_group = G / 16;
    const int g = i / rows_per_group;
    const int r = rslot + 16 * i;
    uint16_t h[8];
    unpack8(raw[i], h);
    uint32_t lo = 0, hi = 0;
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      const bool masked = kept[i] || (h[j] & 0x7FFFu) >= tau;
      const uint32_t c = quantize_one<BITS>(kvs::half_bits_to_float(h[j]), inv_s[g][8 * chunk + j],
                                            zero_s[g][8 * chunk + j], masked);
      if (j < 4) lo |= c << (8 * j); else hi |= c << (8 * (j - 4));
    }
    uint32_t* dst = reinterpret_cast<uint32_t*>(code_s + r * kRowStride + 8 * chunk);
    dst[0] = lo;
    dst[1] = hi;
  }
  __syncthreads();

  if (row_count) {
    // Isolated entries to the block's run of the staging list, in final order (rows ascending,
    // channels ascending inside a row).  Driven by the mask words, one or two per lane, so the
    // work is proportional to the number of entries; their fp16 values are read again from
    // memory (two bytes each, just read by this workgroup).
    const uint16_t* src16 = reinterpret_cast<const uint16_t*>(src);
    for (int wi = tid; wi < TB * 4; wi += kThreads) {
      uint32_t m = (&iso_s[0][0])[wi];
      if (m == 0) continue;
      const int r = wi >> 2, q4 = wi & 3;
      long long pos = static_cast<long long>(run_base_s) + row_off_s[r];
      for (int k = 0; k < q4; ++k) pos += __popc(iso_s[r][k]);
      while (m) {
        const int c = 32 * q4 + __builtin_ctz(m);
        m &= m - 1;
        if (pos < emit.cap) emit.list[pos] = static_cast<uint32_t>(c) | (static_cast<uint32_t>(src16[r * 128 + c]) << 16);
        ++pos;
      }
    }
  }

  // Pack: the block's words are contiguous in global memory in (tile, w, t) order.
  uint32_t* out = k_codes + (bh * (n / KVS_K_TILE) + static_cast<size_t>(t0 / KVS_K_TILE)) * (W * KVS_K_TILE);
  constexpr int words = (TB / KVS_K_TILE) * W * KVS_K_TILE;
  for (int widx = tid; widx < words; widx += kThreads) {
    const int t = widx % KVS_K_TILE;
    const int w = (widx / KVS_K_TILE) % W;
    const int tile = widx / (KVS_K_TILE * W);
    const uint8_t* row = code_s + (tile * KVS_K_TILE + t) * kRowStride + cpw * w;
    uint32_t word = 0;
#pragma unroll
    for (int j = 0; j < cpw; ++j)
      if (cpw * w + j < 128) word |= static_cast<uint32_t>(row[j]) << Fmt<BITS>::shift(j);
    out[widx] = word;
  }
}

// ---------------------------------------------------------------------------------------------
// Values: per token, groups of G consecutive channels.  Block = one 128-token code tile.
// ---------------------------------------------------------------------------------------------
template <int BITS, int G>
__global__ __launch_bounds__(kThreads) void quantize_v_kernel(
    const uint4* __restrict__ V, const uint8_t* __restrict__ keep_mask, kvs::QuantSpan sp, int Hkv,
    const uint32_t* __restrict__ tau_ptr, uint32_t* __restrict__ v_codes, uint32_t* __restrict__ v_params,
    int32_t* __restrict__ row_count, kvs::SparseEmit emit) {
  constexpr int ROWS = KVS_V_TILE / 16;  // 8 rows per lane
  constexpr int W = Fmt<BITS>::W, cpw = Fmt<BITS>::cpw;
  constexpr int LANES_PER_GROUP = G / 8;
  constexpr int NGC = 128 / G;

  __shared__ __align__(16) uint8_t code_s[KVS_V_TILE * kRowStride];
  // Dense-and-sparse only: which tokens of each channel are isolated (128 bits per channel = one
  // CSR row), where the channel's entries start inside the tile's run, where the run starts.
  __shared__ uint32_t iso_s[128][4];
  __shared__ int chan_off_s[128];
  __shared__ int run_base_s;

  const int tid = threadIdx.x;
  const int chunk = tid & 15;
  const int rslot = tid >> 4;
  const uint32_t tau = tau_ptr ? *tau_ptr : 0x8000u;
  if (row_count) {
    for (int i = tid; i < 128 * 4; i += kThreads) (&iso_s[0][0])[i] = 0;
    __syncthreads();
  }
  const int tiles_in = sp.n_tokens / KVS_V_TILE;
  const int tile_in = blockIdx.x % tiles_in;
  const size_t bh = blockIdx.x / tiles_in;
  const int b = static_cast<int>(bh / Hkv);
  const int n = sp.n_cap;                               // layout of everything written
  const int tiles_per_head = n / KVS_V_TILE;
  const int tile = sp.t_out / KVS_V_TILE + tile_in;
  const int t0 = tile * KVS_V_TILE;                     // cache token of the tile's first row

  const uint4* src = V + (bh * sp.n_in + tile_in * KVS_V_TILE) * 16;
  const uint8_t* mask_b = keep_mask + static_cast<size_t>(b) * sp.mask_stride + sp.mask_t0 + tile_in * KVS_V_TILE;

  // Load; with isolated outliers, first mark them (per channel: which tokens), so that the counts
  // and the tile's place in the staging list are known while the codes are being computed.
  uint4 raw[ROWS];
  bool kept[ROWS];
  uint32_t iso_bits[ROWS];               // bit j of row i = channel 8 chunk + j is isolated
#pragma unroll
  for (int i = 0; i < ROWS; ++i) {
    const int r = rslot + 16 * i;
    raw[i] = src[r * 16 + chunk];
    kept[i] = mask_b[r] != 0;
    iso_bits[i] = 0;
  }
  if (row_count) {
#pragma unroll
    for (int i = 0; i < ROWS; ++i) {
      const int r = rslot + 16 * i;
      uint16_t h[8];
      unpack8(raw[i], h);
#pragma unroll
      for (int j = 0; j < 8; ++j) {
        if (!kept[i] && (h[j] & 0x7FFFu) >= tau) {
          iso_bits[i] |= 1u << j;
          atomicOr(&iso_s[8 * chunk + j][r >> 5], 1u << (r & 31));
        }
      }
    }
    __syncthreads();
    if (tid >= kThreads - KVS_WAVE) {
      // The last wave: channel counts (CSR row = (tile, channel)), their exclusive scan over the
      // tile, one claim in the staging list for the tile's whole run.
      const int lane = tid - (kThreads - KVS_WAVE);
      int cnt[2], mine = 0;
#pragma unroll
      for (int k = 0; k < 2; ++k) {
        const int c = 2 * lane + k;
        cnt[k] = __popc(iso_s[c][0]) + __popc(iso_s[c][1]) + __popc(iso_s[c][2]) + __popc(iso_s[c][3]);
        row_count[(bh * tiles_per_head + static_cast<size_t>(tile)) * 128 + c] = cnt[k];
        mine += cnt[k];
      }
      int incl = mine;
#pragma unroll
      for (int o = 1; o < KVS_WAVE; o <<= 1) {
        const int up = __shfl_up(incl, o, KVS_WAVE);
        if (lane >= o) incl += up;
      }
      chan_off_s[2 * lane] = incl - mine;
      chan_off_s[2 * lane + 1] = incl - mine + cnt[0];
      if (lane == KVS_WAVE - 1) {
        const int base = incl > 0 ? atomicAdd(emit.counter, incl) : 0;
        emit.block_base[blockIdx.x] = base;
        run_base_s = base;
      }
    }
  }

#pragma unroll
  for (int i = 0; i < ROWS; ++i) {
    const int r = rslot + 16 * i;
    uint16_t h[8];
    unpack8(raw[i], h);
    float mn = INFINITY, mx = -INFINITY;
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      const bool masked = kept[i] || ((iso_bits[i] >> j) & 1u);
      const float x = kvs::half_bits_to_float(h[j]);
      mn = masked ? mn : fminf(mn, x);
      mx = masked ? mx : fmaxf(mx, x);
    }
    // The lanes of one channel group are LANES_PER_GROUP consecutive lanes of the same row.
#pragma unroll
    for (int o = 1; o < LANES_PER_GROUP; o <<= 1) {
      mn = fminf(mn, __shfl_xor(mn, o, KVS_WAVE));
      mx = fmaxf(mx, __shfl_xor(mx, o, KVS_WAVE));
    }
    const GroupParam p = make_param<BITS>(mn, mx, mn <= mx);
    if ((chunk % LANES_PER_GROUP) == 0)
      v_params[(bh * n + static_cast<size_t>(t0 + r)) * NGC + chunk / LANES_PER_GROUP] = p.word;
    uint32_t lo = 0, hi = 0;
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      const bool masked = kept[i] || ((iso_bits[i] >> j) & 1u);
      const uint32_t c = quantize_one<BITS>(kvs::half_bits_to_float(h[j]), p.inv, p.zero, masked);
      if (j < 4) lo |= c << (8 * j); else hi |= c << (8 * (j - 4));
    }
    uint32_t* dst = reinterpret_cast<uint32_t*>(code_s + r * kRowStride + 8 * chunk);
    dst[0] = lo;
    dst[1] = hi;
  }
  __syncthreads();

  if (row_count) {
    // Isolated entries to the tile's run of the staging list in final order (channels ascending,
    // tokens ascending inside a channel), driven by the mask words; values read again from memory.
    const uint16_t* src16 = reinterpret_cast<const uint16_t*>(src);
    for (int wi = tid; wi < 128 * 4; wi += kThreads) {
      uint32_t m = (&iso_s[0][0])[wi];
      if (m == 0) continue;
      const int c = wi >> 2, q4 = wi & 3;
      long long pos = static_cast<long long>(run_base_s) + chan_off_s[c];
      for (int k = 0; k < q4; ++k) pos += __popc(iso_s[c][k]);
      while (m) {
        const int t = 32 * q4 + __builtin_ctz(m);
        m &= m - 1;
        if (pos < emit.cap) emit.list[pos] = static_cast<uint32_t>(t) | (static_cast<uint32_t>(src16[t * 128 + c]) << 16);
        ++pos;
      }
    }
  }

  // Pack along tokens: word (u, c) holds tokens cpw*u .. of channel c; contiguous per block.
  uint32_t* out = v_codes + (bh * tiles_per_head + static_cast<size_t>(tile)) * (W * 128);
  for (int widx = tid; widx < W * 128; widx += kThreads) {
    const int c = widx & 127;
    const int u = widx >> 7;
    uint32_t word = 0;
#pragma unroll
    for (int j = 0; j < cpw; ++j)
      if (cpw * u + j < 128)
        word |= static_cast<uint32_t>(code_s[(cpw * u + j) * kRowStride + c]) << Fmt<BITS>::shift(j);
    out[widx] = word;
  }
}

// ---------------------------------------------------------------------------------------------
// Keep rows: index list of the kept tokens (ascending) and bit-exact copies of their rows.
// ---------------------------------------------------------------------------------------------
constexpr int kIndexThreads = 1024;

// n tokens are indexed; both masks have `stride` bytes per sequence (they may be the same array).
__global__ __launch_bounds__(kIndexThreads) void keep_index_kernel(
    const uint8_t* __restrict__ keep_mask, int n, int stride, int cap, int32_t* __restrict__ keep_idx,
    int32_t* __restrict__ keep_cnt, uint8_t* __restrict__ mask_copy, int32_t* __restrict__ status) {
  __shared__ int wave_count[kIndexThreads / KVS_WAVE];
  __shared__ int base_s;
  const int b = blockIdx.x, tid = threadIdx.x;
  const int lane = tid & (KVS_WAVE - 1), wave = tid / KVS_WAVE;
  const uint8_t* m = keep_mask + static_cast<size_t>(b) * stride;
  if (tid == 0) base_s = 0;
  __syncthreads();
  for (int i0 = 0; i0 < n; i0 += kIndexThreads) {
    const int i = i0 + tid;
    const bool flag = i < n && m[i] != 0;
    if (i < n) mask_copy[static_cast<size_t>(b) * stride + i] = flag ? 1 : 0;
    const unsigned long long ballot = __ballot(flag);
    const int before = __popcll(ballot & ((1ull << lane) - 1ull));
    if (lane == 0) wave_count[wave] = __popcll(ballot);
    __syncthreads();
    int offset = base_s;
    for (int w = 0; w < wave; ++w) offset += wave_count[w];
    const int pos = offset + before;
    if (flag && pos < cap) keep_idx[static_cast<size_t>(b) * cap + pos] = i;
    __syncthreads();
    if (tid == 0) {
      int total = 0;
      for (int w = 0; w < kIndexThreads / KVS_WAVE; ++w) total += wave_count[w];
      base_s += total;
    }
    __syncthreads();
  }
  const int total = base_s;
  for (int j = total + tid; j < cap; j += kIndexThreads) keep_idx[static_cast<size_t>(b) * cap + j] = -1;
  if (tid == 0) {
    keep_cnt[b] = total;
    if (total > cap) atomicCAS(status, 0, static_cast<int>(KVS_ERR_CAPACITY));
  }
}

// One wave per (b, h, j): copies the 256-byte K row and V row of kept token j if it lies in the
// span the input tensors hold (cache tokens t_out .. t_out + n_tokens), zeros past the count;
// rows of other kept tokens, written by an earlier call, are left alone.
__global__ __launch_bounds__(KVS_WAVE) void keep_gather_kernel(
    const uint32_t* __restrict__ K, const uint32_t* __restrict__ V, kvs::QuantSpan sp, int Hkv, int cap,
    const int32_t* __restrict__ keep_idx, uint32_t* __restrict__ keep_k, uint32_t* __restrict__ keep_v) {
  const int j = blockIdx.x % cap;
  const size_t bh = blockIdx.x / cap;
  const int b = static_cast<int>(bh / Hkv);
  const int t = keep_idx[static_cast<size_t>(b) * cap + j];
  const int lane = threadIdx.x;
  const size_t dst = (bh * cap + j) * 64 + lane;       // 64 uint32 per row
  if (t >= sp.t_out && t < sp.t_out + sp.n_tokens) {
    const size_t srcw = (bh * sp.n_in + (t - sp.t_out)) * 64 + lane;
    keep_k[dst] = K[srcw];
    keep_v[dst] = V[srcw];
  } else if (t < 0) {
    keep_k[dst] = 0;
    keep_v[dst] = 0;
  }
}

template <int BITS, int G>
void launch_dense(const kvs_desc* d, const void* K, const void* V, const uint8_t* mask,
                  const kvs_cache* out, const uint32_t* tau, const kvs::SparsePlan& plan, const kvs::QuantSpan& sp,
                  hipStream_t stream) {
  constexpr int TB = G > 64 ? G : 64;
  const int bh = d->B * d->Hkv;
  if (sp.n_tokens == 0) return;
  hipLaunchKernelGGL((quantize_k_kernel<BITS, G>), dim3(bh * (sp.n_tokens / TB)), dim3(kThreads), 0, stream,
                     static_cast<const uint4*>(K), mask, sp, d->Hkv, tau, out->k_codes, out->k_params,
                     tau ? out->k_rowptr + 1 : nullptr, plan.emit_k);
  hipLaunchKernelGGL((quantize_v_kernel<BITS, G>), dim3(bh * (sp.n_tokens / KVS_V_TILE)), dim3(kThreads), 0,
                     stream, static_cast<const uint4*>(V), mask, sp, d->Hkv, tau ? tau + 1 : nullptr,
                     out->v_codes, out->v_params, tau ? out->v_rowptr + 1 : nullptr, plan.emit_v);
}

template <int BITS>
void launch_dense_g(const kvs_desc* d, const void* K, const void* V, const uint8_t* mask,
                    const kvs_cache* out, const uint32_t* tau, const kvs::SparsePlan& plan, const kvs::QuantSpan& sp,
                    hipStream_t s) {
  switch (d->group) {
    case 32: launch_dense<BITS, 32>(d, K, V, mask, out, tau, plan, sp, s); break;
    case 64: launch_dense<BITS, 64>(d, K, V, mask, out, tau, plan, sp, s); break;
    default: launch_dense<BITS, 128>(d, K, V, mask, out, tau, plan, sp, s); break;
  }
}

}  // namespace

// Shared by the three quantising entry points: the quantise kernels over one span, then - unless
// the lean kernels did it themselves - the keep index over the first n_index cache tokens and the
// kept rows that lie in the span.
static void quantize_span(const kvs_desc* desc, const kvs::QuantSpan& sp, bool whole, const void* K, const void* V,
                          const uint8_t* mask, const uint8_t* index_mask, int n_index, const kvs_cache* out,
                          void* workspace, hipStream_t s, const uint32_t* static_k = nullptr,
                          const uint32_t* static_v = nullptr) {
  const bool sparse = desc->sparse_frac > 0.0f;
  if (kvs::quantize_fast_supported(desc)) {            // 2 / 4 bit without isolated outliers
    kvs::launch_quantize_fast(desc, sp, whole, K, V, mask, out, static_k, static_v, s);
    if (whole) return;
  } else {
    kvs::SparsePlan plan{};
    const uint32_t* tau = nullptr;       // device [2]: thresholds of K and V
    if (sparse) {
      plan = kvs::sparse_plan(desc, workspace);
      kvs::sparse_thresholds(desc, plan, K, V, mask, out, s);
      tau = plan.tau;
    }
    switch (desc->bits) {
      case 2: launch_dense_g<2>(desc, K, V, mask, out, tau, plan, sp, s); break;
      case 3: launch_dense_g<3>(desc, K, V, mask, out, tau, plan, sp, s); break;
      default: launch_dense_g<4>(desc, K, V, mask, out, tau, plan, sp, s); break;
    }
    if (sparse) kvs::sparse_build_csr(desc, plan, out, s);
  }
  hipLaunchKernelGGL(keep_index_kernel, dim3(desc->B), dim3(kIndexThreads), 0, s, index_mask, n_index,
                     whole ? desc->n : sp.n_cap, desc->keep_cap, out->keep_idx, out->keep_cnt, out->keep_mask,
                     out->status);
  if (desc->keep_cap > 0)
    hipLaunchKernelGGL(keep_gather_kernel, dim3(desc->B * desc->Hkv * desc->keep_cap), dim3(KVS_WAVE), 0, s,
                       static_cast<const uint32_t*>(K), static_cast<const uint32_t*>(V), sp, desc->Hkv,
                       desc->keep_cap, out->keep_idx, static_cast<uint32_t*>(out->keep_k),
                       static_cast<uint32_t*>(out->keep_v));
}

static kvs_status check_quantize_args(const kvs_desc* desc, const kvs_cache* out) {
  const kvs_status st = kvs::validate_desc(desc);
  if (st != KVS_OK) return st;
  if (!out) return KVS_ERR_INVALID;
  if (!out->k_codes || !out->v_codes || !out->k_params || !out->v_params || !out->keep_idx ||
      !out->keep_cnt || !out->keep_mask || !out->status)
    return KVS_ERR_INVALID;
  if (desc->keep_cap > 0 && (!out->keep_k || !out->keep_v)) return KVS_ERR_INVALID;
  return KVS_OK;
}

extern "C" kvs_status kvs_quantize_kv(const kvs_desc* desc, const void* K, const void* V,
                                       const uint8_t* keep_mask, const kvs_cache* out,
                                       void* workspace, void* stream) {
  const kvs_status st = check_quantize_args(desc, out);
  if (st != KVS_OK) return st;
  if (!K || !V || !keep_mask) return KVS_ERR_INVALID;
  const bool sparse = desc->sparse_frac > 0.0f;
  if (sparse && (!workspace || !out->k_rowptr || !out->k_col || !out->k_val || !out->v_rowptr ||
                 !out->v_col || !out->v_val))
    return KVS_ERR_INVALID;
  hipStream_t s = static_cast<hipStream_t>(stream);
  quantize_span(desc, kvs::whole_span(desc), true, K, V, keep_mask, keep_mask, desc->n, out, workspace, s);
  return hipGetLastError() == hipSuccess ? KVS_OK : KVS_ERR_DEVICE;
}

// ---------------------------------------------------------------------------------------------
// Growing caches (paper, Section 2 "KV cache": the decoding phase appends the new token's K, V).
// Whole 128-token blocks are quantised; the tokens after the last whole block wait in fp16 rows
// (res_k / res_v) until their block is complete.
// ---------------------------------------------------------------------------------------------
namespace {

// Keep mask of a prompt into the cache's capacity-wide mask: flags normalised to 0 / 1, zeros
// from the prompt's end to the capacity.
__global__ void grow_mask_kernel(const uint8_t* __restrict__ mask, int n_tokens, int n_cap, uint8_t* __restrict__ dst) {
  const int b = blockIdx.y;
  for (int i = blockIdx.x * blockDim.x + threadIdx.x; i < n_cap; i += gridDim.x * blockDim.x)
    dst[static_cast<size_t>(b) * n_cap + i] = i < n_tokens && mask[static_cast<size_t>(b) * n_tokens + i] != 0 ? 1 : 0;
}

// rows tokens of each (b, h), starting at input token t_in of a [B*Hkv, n_in, 128] tensor pair, to
// residual rows r_out .. of the [B*Hkv, 128, 128] windows.  One wave per (b, h, row).
__global__ __launch_bounds__(KVS_WAVE) void residual_copy_kernel(
    const uint32_t* __restrict__ K, const uint32_t* __restrict__ V, int n_in, int t_in, int rows, int r_out,
    uint32_t* __restrict__ res_k, uint32_t* __restrict__ res_v) {
  const int r = blockIdx.x % rows;
  const size_t bh = blockIdx.x / rows;
  const size_t src = (bh * n_in + t_in + r) * 64 + threadIdx.x;
  const size_t dst = (bh * KVS_V_TILE + r_out + r) * 64 + threadIdx.x;
  res_k[dst] = K[src];
  res_v[dst] = V[src];
}

}  // namespace

extern "C" kvs_status kvs_quantize_prefix(const kvs_desc* desc, const void* K, const void* V,
                                           const uint8_t* keep_mask, int32_t n_tokens, const kvs_cache* out,
                                           void* workspace, void* stream) {
  const kvs_status st = check_quantize_args(desc, out);
  if (st != KVS_OK) return st;
  if (desc->sparse_frac > 0.0f) return KVS_ERR_UNSUPPORTED;
  if (n_tokens < 0 || n_tokens > desc->n) return KVS_ERR_INVALID;
  if (!out->res_k || !out->res_v) return KVS_ERR_INVALID;
  if (n_tokens > 0 && (!K || !V || !keep_mask)) return KVS_ERR_INVALID;
  hipStream_t s = static_cast<hipStream_t>(stream);
  const int nq = (n_tokens / KVS_V_TILE) * KVS_V_TILE;
  hipLaunchKernelGGL(grow_mask_kernel, dim3((desc->n + 255) / 256, desc->B), dim3(256), 0, s, keep_mask, n_tokens,
                     desc->n, out->keep_mask);
  const kvs::QuantSpan sp{n_tokens, nq, desc->n, 0, n_tokens, 0};
  quantize_span(desc, sp, false, K, V, keep_mask, out->keep_mask, nq, out, workspace, s);
  if (n_tokens > nq)
    hipLaunchKernelGGL(residual_copy_kernel, dim3(desc->B * desc->Hkv * (n_tokens - nq)), dim3(KVS_WAVE), 0, s,
                       static_cast<const uint32_t*>(K), static_cast<const uint32_t*>(V), n_tokens, nq, n_tokens - nq,
                       0, static_cast<uint32_t*>(out->res_k), static_cast<uint32_t*>(out->res_v));
  return hipGetLastError() == hipSuccess ? KVS_OK : KVS_ERR_DEVICE;
}

extern "C" kvs_status kvs_append_kv(const kvs_desc* desc, const void* k_new, const void* v_new, int32_t n_tokens,
                                     const kvs_cache* cache, void* workspace, void* stream) {
  const kvs_status st = check_quantize_args(desc, cache);
  if (st != KVS_OK) return st;
  if (desc->sparse_frac > 0.0f) return KVS_ERR_UNSUPPORTED;
  if (n_tokens < 0 || n_tokens >= desc->n) return KVS_ERR_INVALID;     // no room for one more token
  if (!k_new || !v_new || !cache->res_k || !cache->res_v) return KVS_ERR_INVALID;
  hipStream_t s = static_cast<hipStream_t>(stream);
  const int nq = (n_tokens / KVS_V_TILE) * KVS_V_TILE;
  const int r = n_tokens - nq;
  hipLaunchKernelGGL(residual_copy_kernel, dim3(desc->B * desc->Hkv), dim3(KVS_WAVE), 0, s,
                     static_cast<const uint32_t*>(k_new), static_cast<const uint32_t*>(v_new), 1, 0, 1, r,
                     static_cast<uint32_t*>(cache->res_k), static_cast<uint32_t*>(cache->res_v));
  if (r == KVS_V_TILE - 1) {                           // the window is a whole block now
    const kvs::QuantSpan sp{KVS_V_TILE, KVS_V_TILE, desc->n, nq, desc->n, nq};
    quantize_span(desc, sp, false, cache->res_k, cache->res_v, cache->keep_mask, cache->keep_mask,
                  nq + KVS_V_TILE, cache, workspace, s);
  }
  return hipGetLastError() == hipSuccess ? KVS_OK : KVS_ERR_DEVICE;
}

// ---------------------------------------------------------------------------------------------
// Static quantisation (paper, Appendix C "Dynamic and static quantization"): calibrate, derive
// fixed parameters, quantise with them.
// ---------------------------------------------------------------------------------------------
extern "C" size_t kvs_calibration_bytes(const kvs_desc* desc) {
  if (kvs::validate_desc(desc) != KVS_OK) return 0;
  return static_cast<size_t>(4) * desc->Hkv * KVS_HEAD_DIM * sizeof(uint32_t);
}

extern "C" kvs_status kvs_calibrate_reset(const kvs_desc* desc, void* calib, void* stream) {
  const kvs_status st = kvs::validate_desc(desc);
  if (st != KVS_OK) return st;
  if (!calib) return KVS_ERR_INVALID;
  kvs::launch_calibrate_reset(desc, static_cast<uint32_t*>(calib), static_cast<hipStream_t>(stream));
  return hipGetLastError() == hipSuccess ? KVS_OK : KVS_ERR_DEVICE;
}

extern "C" kvs_status kvs_calibrate(const kvs_desc* desc, const void* K, const void* V, const uint8_t* keep_mask,
                                     void* calib, void* stream) {
  const kvs_status st = kvs::validate_desc(desc);
  if (st != KVS_OK) return st;
  if (!K || !V || !keep_mask || !calib) return KVS_ERR_INVALID;
  kvs::launch_calibrate(desc, K, V, keep_mask, static_cast<uint32_t*>(calib), static_cast<hipStream_t>(stream));
  return hipGetLastError() == hipSuccess ? KVS_OK : KVS_ERR_DEVICE;
}

extern "C" kvs_status kvs_static_params(const kvs_desc* desc, const void* calib, uint32_t* k_static,
                                         uint32_t* v_static, void* stream) {
  const kvs_status st = kvs::validate_desc(desc);
  if (st != KVS_OK) return st;
  if (!calib || !k_static || !v_static) return KVS_ERR_INVALID;
  kvs::launch_static_params(desc, static_cast<const uint32_t*>(calib), k_static, v_static,
                            static_cast<hipStream_t>(stream));
  return hipGetLastError() == hipSuccess ? KVS_OK : KVS_ERR_DEVICE;
}

extern "C" kvs_status kvs_quantize_kv_static(const kvs_desc* desc, const void* K, const void* V,
                                              const uint8_t* keep_mask, const uint32_t* k_static,
                                              const uint32_t* v_static, const kvs_cache* out, void* workspace,
                                              void* stream) {
  const kvs_status st = check_quantize_args(desc, out);
  if (st != KVS_OK) return st;
  if (desc->sparse_frac > 0.0f) return KVS_ERR_UNSUPPORTED;
  if (!K || !V || !keep_mask || !k_static || !v_static) return KVS_ERR_INVALID;
  hipStream_t s = static_cast<hipStream_t>(stream);
  quantize_span(desc, kvs::whole_span(desc), true, K, V, keep_mask, keep_mask, desc->n, out, workspace, s,
                k_static, v_static);
  return hipGetLastError() == hipSuccess ? KVS_OK : KVS_ERR_DEVICE;
}

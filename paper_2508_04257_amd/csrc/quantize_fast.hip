// The quantisation kernels of kvs_quantize_kv and the calls built on it (paper, Appendix C
// equations for Q(X), scale and zero; Algorithm 1's two quantise steps; Section 4.1 for the
// per-channel Key / per-token Value grouping; Section 5.1 for the per-token Key scheme and the
// dense-and-sparse variant).  One pass over the fp16 tensors, bound by that 2-byte-per-element
// read; the quantiser arithmetic is the exact fp32 sequence the ABI header documents.
//
// How the work is laid out:
//   * group minima / maxima are taken on the raw fp16 pairs (v_pk_min_f16 / v_pk_max_f16): the
//     minimum of the fp16 values converted to fp32 is the converted fp16 minimum;
//   * one lane per group derives scale / zero (two IEEE divisions) and the others receive them;
//   * codes are clamped in fp32 and inserted into the word with one shift-or each;
//   * Values: a lane owns 8 consecutive tokens x 8 channels, which is exactly eight 4-bit words of
//     the token-packed layout, so nothing is staged in LDS; Keys: one word per (token, lane), moved
//     through a padded LDS tile so that the global stores are contiguous.
//   * 3 bit: ten codes per word do not line up with eight-element lanes, so a lane first makes a
//     24-bit piece (eight codes) and the words are cut out of the row's sixteen pieces in LDS;
//   * rows of kept tokens go straight from registers to the fp16 side buffer;
//   * SPARSE variants: entries at or above the threshold are marked with packed 16-bit
//     arithmetic, leave the statistics, get code 0, and are written - by the lane that holds them,
//     in final order - to the workgroup's run of a staging list (see the helpers below).
// Compiled with floating-point contraction off and correctly rounded division, so that no
// multiply-add fuses across the quantiser's operations.
#include "kvs_device.h"
#include "sparse_emit.h"

namespace {

using kvs::Fmt;
typedef _Float16 half2v __attribute__((ext_vector_type(2)));

constexpr int kThreads = 256;
constexpr uint32_t kPosMax2 = 0x7BFF7BFFu;   // (+65504, +65504)
constexpr uint32_t kNegMax2 = 0xFBFFFBFFu;   // (-65504, -65504)

// Packed fp16 minimum / maximum of two register pairs.  Written as the instruction itself: the
// generic elementwise builtins first canonicalise each operand (one more instruction per
// operand) in case it holds a signalling NaN, and the inputs here are finite by contract.
__device__ inline uint32_t pk_min(uint32_t a, uint32_t b) {
  uint32_t r;
  asm("v_pk_min_f16 %0, %1, %2" : "=v"(r) : "v"(a), "v"(b));
  return r;
}
__device__ inline uint32_t pk_max(uint32_t a, uint32_t b) {
  uint32_t r;
  asm("v_pk_max_f16 %0, %1, %2" : "=v"(r) : "v"(a), "v"(b));
  return r;
}
// Streaming store of 16 bytes: the packed cache is written once and read much later, so it
// should not linger as dirty lines in the last-level cache (whoever streams next would pay for
// its write-back).
typedef uint32_t uint4v __attribute__((ext_vector_type(4)));
__device__ inline void store_stream(uint4* dst, const uint4& v) {
  __builtin_nontemporal_store(uint4v{v.x, v.y, v.z, v.w}, reinterpret_cast<uint4v*>(dst));
}
__device__ inline uint4 load_stream(const uint4* src) {
  const uint4v v = __builtin_nontemporal_load(reinterpret_cast<const uint4v*>(src));
  return uint4{v.x, v.y, v.z, v.w};
}

__device__ inline float lo_half(uint32_t v) { return kvs::half_bits_to_float(static_cast<uint16_t>(v & 0xFFFFu)); }
__device__ inline float hi_half(uint32_t v) { return kvs::half_bits_to_float(static_cast<uint16_t>(v >> 16)); }

struct Param {
  float inv;     // 1 / scale
  float zero;    // zero point as an exact float
  uint32_t word; // fp16 scale | int16 zero << 16
};

// scale / zero of one group from its minimum and maximum (any == false: no unmasked entry).
template <int BITS>
__device__ inline Param make_param(float mn, float mx, bool any) {
  constexpr float qmax = static_cast<float>(Fmt<BITS>::qmax);
  if (!any) { mn = 0.0f; mx = 0.0f; }
  uint16_t hbits;
  if (mx == mn) {
    hbits = kvs::float_to_half_bits_rn(mn != 0.0f ? fabsf(mn) : 1.0f);
  } else {
    float s32 = (mx - mn) / qmax;
    // 8 bit: the zero point must still fit its int16 half.  (Up to 4 bit it always does for fp16
    // data: max - min is at least |min| / 2048.)
    if constexpr (BITS == 8) s32 = fmaxf(s32, fabsf(mn) / 32766.0f);
    hbits = kvs::float_to_half_bits_rn(s32);
    if (kvs::half_bits_to_float(hbits) < s32) hbits += 1;   // next fp16 up (positive values)
  }
  Param p;
  p.inv = 1.0f / kvs::half_bits_to_float(hbits);
  const int z = -static_cast<int>(rintf(mn * p.inv));
  p.zero = static_cast<float>(z);
  p.word = static_cast<uint32_t>(hbits) | (static_cast<uint32_t>(z & 0xFFFF) << 16);
  return p;
}

// The same from a stored parameter word (static quantisation: the parameters are given).
__device__ inline Param param_of_word(uint32_t word) {
  Param p;
  p.inv = 1.0f / kvs::half_bits_to_float(static_cast<uint16_t>(word & 0xFFFFu));
  p.zero = static_cast<float>(static_cast<int>(static_cast<int16_t>(word >> 16)));
  p.word = word;
  return p;
}

// clamp(rne(x / scale) + zero, 0, qmax) as an unsigned integer; every intermediate is an exact
// integer in fp32, so clamping before the conversion gives the same code as clamping after it.
template <int BITS>
__device__ inline uint32_t code_of(float x, float inv, float zero) {
  const float v = rintf(x * inv) + zero;
  return static_cast<uint32_t>(__builtin_amdgcn_fmed3f(v, 0.0f, static_cast<float>(Fmt<BITS>::qmax)));
}

// The eight codes of one uint4 of fp16 values (channels 8 chunk .. + 7), code j at bits BITS * j.
template <int BITS>
__device__ inline uint32_t codes8(const uint4& raw, const float inv[8], const float zero[8]) {
  const uint32_t w[4] = {raw.x, raw.y, raw.z, raw.w};
  uint32_t out = 0;
#pragma unroll
  for (int k = 0; k < 4; ++k) {
    out |= code_of<BITS>(lo_half(w[k]), inv[2 * k], zero[2 * k]) << (BITS * 2 * k);
    out |= code_of<BITS>(hi_half(w[k]), inv[2 * k + 1], zero[2 * k + 1]) << (BITS * (2 * k + 1));
  }
  return out;
}

// 8 bit: the same eight codes fill two words (channels 8 chunk .. + 3, then + 4 .. + 7).
__device__ inline void codes8_bytes(const uint4& raw, const float inv[8], const float zero[8], uint32_t& lo, uint32_t& hi) {
  const uint32_t w[4] = {raw.x, raw.y, raw.z, raw.w};
  lo = code_of<8>(lo_half(w[0]), inv[0], zero[0]) | (code_of<8>(hi_half(w[0]), inv[1], zero[1]) << 8) |
       (code_of<8>(lo_half(w[1]), inv[2], zero[2]) << 16) | (code_of<8>(hi_half(w[1]), inv[3], zero[3]) << 24);
  hi = code_of<8>(lo_half(w[2]), inv[4], zero[4]) | (code_of<8>(hi_half(w[2]), inv[5], zero[5]) << 8) |
       (code_of<8>(lo_half(w[3]), inv[6], zero[6]) << 16) | (code_of<8>(hi_half(w[3]), inv[7], zero[7]) << 24);
}

// 3 bit: a row of 128 codes is first held as sixteen 24-bit pieces (eight codes each, 3 bits per
// code); word w of the packed layout is codes 10 w .. 10 w + 9 of that 384-bit string, five in bits
// 0-14 and five in bits 16-30 (the last word holds eight codes).
constexpr int kPieceStride = 17;                // 16 pieces per row + 1: keeps the LDS banks spread
__device__ inline uint32_t compose3(const uint32_t* pieces, int w) {
  const int o = 30 * w, p0 = o / 24, sh = o % 24;
  unsigned long long x = pieces[p0];
  if (p0 + 1 < 16) x |= static_cast<unsigned long long>(pieces[p0 + 1]) << 24;
  if (p0 + 2 < 16) x |= static_cast<unsigned long long>(pieces[p0 + 2]) << 48;
  x >>= sh;
  return static_cast<uint32_t>(x & 0x7FFFu) | (static_cast<uint32_t>((x >> 15) & 0x7FFFu) << 16);
}

// Dense-and-sparse support (paper, Section 5.1: the largest-magnitude entries are isolated in
// 16 bit).  An entry whose fp16 magnitude pattern reaches tau leaves the statistics, gets code 0
// and is recorded in a bit mask per CSR row; the masks then drive the emission.
__device__ inline uint32_t select_halves(uint32_t m, uint32_t a, uint32_t b) { return (a & m) | (b & ~m); }
// Field mask of a lane's eight codes: bit j of `bits` -> the BITS-wide field of code j.
template <int BITS>
__device__ inline void fill_spread_table(uint32_t* table, int tid) {
  if (tid < 256) {
    uint32_t m = 0;
#pragma unroll
    for (int j = 0; j < 8; ++j) m |= ((tid >> j) & 1) ? static_cast<uint32_t>(Fmt<BITS>::qmax) << (BITS * j) : 0u;
    table[tid] = m;
  }
}
// Transpose of an 8 x 8 bit matrix held as row i = byte i (lo: rows 0-3, hi: rows 4-7), bit j = column j.
__device__ inline void transpose8x8(uint32_t& lo, uint32_t& hi) {
  unsigned long long x = static_cast<unsigned long long>(lo) | (static_cast<unsigned long long>(hi) << 32);
  unsigned long long t;
  t = 0x0F0F0F0F00000000ull & (x ^ (x << 28)); x ^= t ^ (t >> 28);
  t = 0x3333000033330000ull & (x ^ (x << 14)); x ^= t ^ (t >> 14);
  t = 0x5500550055005500ull & (x ^ (x << 7));  x ^= t ^ (t >> 7);
  lo = static_cast<uint32_t>(x);
  hi = static_cast<uint32_t>(x >> 32);
}

// Number of set bits of a 128-bit mask row (four words) below byte `byte` (0 .. 15).
__device__ inline int bits_below_byte(const uint32_t* row, int byte) {
  const uint4 m = *reinterpret_cast<const uint4*>(row);
  const int q = byte >> 2;
  int pre = (q > 0 ? __popc(m.x) : 0) + (q > 1 ? __popc(m.y) : 0) + (q > 2 ? __popc(m.z) : 0);
  const uint32_t wq = q == 0 ? m.x : (q == 1 ? m.y : (q == 2 ? m.z : m.w));
  return pre + __popc(wq & ((1u << (8 * (byte & 3))) - 1u));
}
// Half j (0 .. 7) of a uint4 of fp16 values, j known only at run time.
__device__ inline uint32_t half_of(const uint4& v, int j) {
  const int k = j >> 1;
  const uint32_t w = k == 0 ? v.x : (k == 1 ? v.y : (k == 2 ? v.z : v.w));
  return (j & 1) ? w >> 16 : w & 0xFFFFu;
}

// Slot of token t in the ascending keep list of its sequence, or -1 (binary search: the list can
// be long when a first-N policy keeps many tokens).
__device__ inline int keep_slot(const int32_t* __restrict__ keep_idx, int cnt, int t) {
  int lo = 0, hi = cnt;                          // first index whose token is >= t
  while (lo < hi) {
    const int mid = (lo + hi) >> 1;
    if (keep_idx[mid] < t) lo = mid + 1; else hi = mid;
  }
  return lo < cnt && keep_idx[lo] == t ? lo : -1;
}

// ---------------------------------------------------------------------------------------------
// Keys: per channel, groups of G consecutive tokens.  Block = TB = max(G, 64) tokens.
// ---------------------------------------------------------------------------------------------
template <int BITS, int G, bool SPARSE>
__global__ __launch_bounds__(kThreads) void quantize_k_fast_kernel(
    const uint4* __restrict__ K, const uint8_t* __restrict__ keep_mask, kvs::QuantSpan sp, int Hkv,
    uint32_t* __restrict__ k_codes, uint32_t* __restrict__ k_params, const int32_t* __restrict__ keep_idx,
    const int32_t* __restrict__ keep_cnt, int cap, uint4* __restrict__ keep_k,
    const uint32_t* __restrict__ static_k,            // [Hkv, 128] fixed parameter words, or null
    const uint32_t* __restrict__ tau_ptr, int32_t* __restrict__ row_count, kvs::SparseEmit emit) {   // SPARSE only
  constexpr int TB = G > 64 ? G : 64;
  constexpr int NG = TB / G;
  constexpr int ROWS = TB / 16;
  constexpr int RPG = G / 16;                   // rows of one lane that fall into one group
  constexpr int W = Fmt<BITS>::W;
  constexpr int TILE_STRIDE = 68;               // padded token stride of the staged word tile
  constexpr int LANES_PER_WORD = BITS == 2 ? 2 : 1;    // 2 bit: two lanes share a word
  constexpr int kStage = BITS == 3 ? TB * kPieceStride : (TB / KVS_K_TILE) * W * TILE_STRIDE;

  __shared__ uint32_t red_mn[NG][16][64];       // [group][row slot][channel pair] packed fp16 minima
  __shared__ uint32_t red_mx[NG][16][64];
  __shared__ float inv_s[NG][128];
  __shared__ float zero_s[NG][128];
  __shared__ __align__(16) uint32_t tile_s[kStage];     // words as [tile][w][token]; 3 bit: pieces [token][16]
  // SPARSE: which entries of each row are isolated (128 bits per row = CSR row (b, h, token)),
  // where the row's entries start inside the block's run, where that run starts in the staging
  // list, and the field masks that clear the codes of isolated entries.
  __shared__ uint32_t iso_s[SPARSE ? TB : 1][4];
  __shared__ int row_off_s[SPARSE ? TB : 1];
  __shared__ int run_base_s;
  __shared__ uint32_t spread_s[SPARSE ? 256 : 1];

  const int tid = threadIdx.x;
  const int chunk = tid & 15;
  const int rslot = tid >> 4;
  uint32_t tau2 = 0;
  if (SPARSE) {
    const uint32_t tau = *tau_ptr;                 // 0x8000: no magnitude pattern reaches it
    tau2 = tau | (tau << 16);
    if constexpr (BITS != 8) fill_spread_table<BITS>(spread_s, tid);
  }
  const int blocks_per_head = sp.n_tokens / TB;
  const int blk = blockIdx.x % blocks_per_head;
  const size_t bh = blockIdx.x / blocks_per_head;
  const int b = static_cast<int>(bh / Hkv);
  const int t0 = blk * TB;                      // input token; the cache token is sp.t_out + t0
  const int n = sp.n_cap;                       // layout of everything written
  const int tc0 = sp.t_out + t0;
  const uint4* src = K + (bh * sp.n_in + t0) * 16;
  const uint8_t* mask_b = keep_mask + static_cast<size_t>(b) * sp.mask_stride + sp.mask_t0 + t0;

  uint4 raw[ROWS];
  bool kept[ROWS];
#pragma unroll
  for (int i = 0; i < ROWS; ++i) {
    const int r = rslot + 16 * i;
    raw[i] = load_stream(src + r * 16 + chunk);
    kept[i] = mask_b[r] != 0;
  }

  // Lane-local packed minima / maxima per group over the rows that are not kept.
  bool any_g[NG];                               // does any token of the group survive?
  uint32_t iso8[SPARSE ? ROWS : 1];             // SPARSE: isolated entries of the lane's piece of each row
  int run_claim = 0;                            // SPARSE, last lane: start of the block's run in the staging list
#pragma unroll
  for (int g = 0; g < NG; ++g) {
    uint32_t mn[4] = {kPosMax2, kPosMax2, kPosMax2, kPosMax2};
    uint32_t mx[4] = {kNegMax2, kNegMax2, kNegMax2, kNegMax2};
    bool any = false;
#pragma unroll
    for (int i = g * RPG; i < (g + 1) * RPG; ++i) {
      if (SPARSE) {
        const uint32_t w4[4] = {raw[i].x, raw[i].y, raw[i].z, raw[i].w};
        uint32_t m[4];
#pragma unroll
        for (int k = 0; k < 4; ++k) m[k] = kvs::below_mask(w4[k], tau2);
        iso8[i] = kept[i] ? 0u : kvs::isolated8(m);
        if (!kept[i]) {
#pragma unroll
          for (int k = 0; k < 4; ++k) {
            mn[k] = pk_min(mn[k], select_halves(m[k], w4[k], kPosMax2));
            mx[k] = pk_max(mx[k], select_halves(m[k], w4[k], kNegMax2));
          }
          any = true;
        }
        reinterpret_cast<uint8_t*>(&iso_s[0][0])[(rslot + 16 * i) * 16 + chunk] = static_cast<uint8_t>(iso8[i]);
      } else if (!kept[i]) {
        mn[0] = pk_min(mn[0], raw[i].x); mn[1] = pk_min(mn[1], raw[i].y);
        mn[2] = pk_min(mn[2], raw[i].z); mn[3] = pk_min(mn[3], raw[i].w);
        mx[0] = pk_max(mx[0], raw[i].x); mx[1] = pk_max(mx[1], raw[i].y);
        mx[2] = pk_max(mx[2], raw[i].z); mx[3] = pk_max(mx[3], raw[i].w);
        any = true;
      }
    }
    *reinterpret_cast<uint4*>(&red_mn[g][rslot][4 * chunk]) = uint4{mn[0], mn[1], mn[2], mn[3]};
    *reinterpret_cast<uint4*>(&red_mx[g][rslot][4 * chunk]) = uint4{mx[0], mx[1], mx[2], mx[3]};
    any_g[g] = __syncthreads_or(any ? 1 : 0) != 0;     // also orders the LDS writes before the reads
  }

  // One lane per (group, channel pair): finish the reduction, derive both parameters.
  if (tid < NG * 64) {
    const int g = tid >> 6, cp = tid & 63;
    uint32_t a = kPosMax2, z = kNegMax2;
#pragma unroll
    for (int s = 0; s < 16; ++s) { a = pk_min(a, red_mn[g][s][cp]); z = pk_max(z, red_mx[g][s][cp]); }
    const bool any = any_g[g];
    Param p0, p1;
    if (static_k) {
      const uint2 w = reinterpret_cast<const uint2*>(static_k + (bh % Hkv) * 128)[cp];
      p0 = param_of_word(w.x);
      p1 = param_of_word(w.y);
    } else if (SPARSE) {                          // a channel can lose every entry of the group to the CSR
      p0 = make_param<BITS>(lo_half(a), lo_half(z), any && lo_half(a) <= lo_half(z));
      p1 = make_param<BITS>(hi_half(a), hi_half(z), any && hi_half(a) <= hi_half(z));
    } else {
      p0 = make_param<BITS>(lo_half(a), lo_half(z), any);
      p1 = make_param<BITS>(hi_half(a), hi_half(z), any);
    }
    inv_s[g][2 * cp] = p0.inv;  inv_s[g][2 * cp + 1] = p1.inv;
    zero_s[g][2 * cp] = p0.zero;  zero_s[g][2 * cp + 1] = p1.zero;
    __builtin_nontemporal_store(__builtin_bit_cast(unsigned long long, uint2{p0.word, p1.word}),
                                reinterpret_cast<unsigned long long*>(k_params + (bh * (n / G) + static_cast<size_t>(tc0 / G + g)) * 128) + cp);
  }
  if (SPARSE && tid >= kThreads - KVS_WAVE) {
    // Meanwhile the last wave: row counts (CSR row = token), their exclusive scan over the block,
    // and one claim in the staging list for the block's whole run.
    const int lane = tid - (kThreads - KVS_WAVE);
    int cnt[TB / KVS_WAVE], mine = 0;
#pragma unroll
    for (int k = 0; k < TB / KVS_WAVE; ++k) {
      const int r = lane * (TB / KVS_WAVE) + k;
      cnt[k] = __popc(iso_s[r][0]) + __popc(iso_s[r][1]) + __popc(iso_s[r][2]) + __popc(iso_s[r][3]);
      row_count[bh * n + tc0 + r] = cnt[k];
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
    // requested now, needed only when the entries are written out
    if (lane == KVS_WAVE - 1 && incl > 0) run_claim = kvs::claim_run(emit, incl);
  }
  __syncthreads();

  // Codes: one word (4 bit) or half a word (2 bit) per row and lane, staged as [tile][w][token].
  const int cnt = min(keep_cnt[b], cap);
#pragma unroll
  for (int g = 0; g < NG; ++g) {
    float inv[8], zero[8];
#pragma unroll
    for (int j = 0; j < 8; ++j) { inv[j] = inv_s[g][8 * chunk + j]; zero[j] = zero_s[g][8 * chunk + j]; }
#pragma unroll
    for (int i = g * RPG; i < (g + 1) * RPG; ++i) {
      const int r = rslot + 16 * i;
      if constexpr (BITS == 8) {                  // two words per row and lane
        uint32_t lo = 0, hi = 0;
        if (!kept[i]) codes8_bytes(raw[i], inv, zero, lo, hi);
        tile_s[((r / KVS_K_TILE) * W + 2 * chunk) * TILE_STRIDE + (r % KVS_K_TILE)] = lo;
        tile_s[((r / KVS_K_TILE) * W + 2 * chunk + 1) * TILE_STRIDE + (r % KVS_K_TILE)] = hi;
      } else {
        uint32_t word = kept[i] ? 0u : codes8<BITS>(raw[i], inv, zero);
        if (SPARSE) word &= ~spread_s[iso8[i]];     // isolated entries hold code 0
        if (LANES_PER_WORD == 2) {                  // 2 bit: lanes (even, odd) share a word
          const uint32_t other = static_cast<uint32_t>(__shfl_xor(static_cast<int>(word), 1, KVS_WAVE));
          word = word | (other << 16);
        }
        if (BITS == 3)
          tile_s[r * kPieceStride + chunk] = word;
        else if (LANES_PER_WORD == 1 || (chunk & 1) == 0)
          tile_s[((r / KVS_K_TILE) * W + chunk / LANES_PER_WORD) * TILE_STRIDE + (r % KVS_K_TILE)] = word;
      }
      if (kept[i]) {                              // exact copy of the row into the fp16 side buffer
        const int j = keep_slot(keep_idx + static_cast<size_t>(b) * cap, cnt, tc0 + r);
        if (j >= 0) keep_k[(bh * cap + j) * 16 + chunk] = raw[i];
      }
    }
  }
  if (SPARSE && tid == kThreads - 1) {            // the claim has had the whole code phase to return
    emit.block_base[blockIdx.x] = run_claim;
    run_base_s = run_claim;
  }
  __syncthreads();

  if (SPARSE) {
    // Isolated entries to the block's run of the staging list, in final order (rows ascending,
    // channels ascending inside a row): the lane that holds an entry writes it from its
    // registers; its place is the row's start plus the entries of the row to its left.
    // The run's start is the same for the whole workgroup: the list is addressed from there with
    // 32-bit positions, and `room` is what is left of the list behind it.
    const int run_base = __builtin_amdgcn_readfirstlane(run_base_s);
    const long long left = kvs::emit_list_words(emit.cap) - run_base;
    const int room = left < 0 ? 0 : (left > 0x7FFFFFFF ? 0x7FFFFFFF : static_cast<int>(left));
    uint32_t* run = emit.list + run_base;
#pragma unroll
    for (int i = 0; i < ROWS; ++i) {
      // Entries of the row to the lane's left: the sixteen lanes of a row are one 16-lane row of the
      // wave, so a shift-and-add scan of the lanes' counts gives it without a look at the row's mask.
      const int own = __popc(iso8[i]);
      int upto = own;
      upto += __builtin_amdgcn_update_dpp(0, upto, 0x111, 0xF, 0xF, true);
      upto += __builtin_amdgcn_update_dpp(0, upto, 0x112, 0xF, 0xF, true);
      upto += __builtin_amdgcn_update_dpp(0, upto, 0x114, 0xF, 0xF, true);
      upto += __builtin_amdgcn_update_dpp(0, upto, 0x118, 0xF, 0xF, true);
      uint32_t bits = iso8[i];
      if (bits == 0) continue;
      const int r = rslot + 16 * i;
      int pos = row_off_s[r] + upto - own;
      while (bits) {
        const int j = __builtin_ctz(bits);
        bits &= bits - 1;
        if (pos < room)                            // channel | token inside its 128-token tile << 7 | fp16 value << 16
          run[pos] = static_cast<uint32_t>(8 * chunk + j) | (static_cast<uint32_t>((tc0 + r) & 127) << 7) | (half_of(raw[i], j) << 16);
        ++pos;
      }
    }
  }

  // The block's words are contiguous in global memory in (tile, w, t) order: 128-bit stores.
  uint4* out = reinterpret_cast<uint4*>(k_codes + (bh * (n / KVS_K_TILE) + static_cast<size_t>(tc0 / KVS_K_TILE)) * (W * KVS_K_TILE));
  constexpr int quads = (TB / KVS_K_TILE) * W * (KVS_K_TILE / 4);
  for (int qi = tid; qi < quads; qi += kThreads) {
    const int row = qi / (KVS_K_TILE / 4), t4 = qi % (KVS_K_TILE / 4);
    if (BITS == 3) {
      const int tile = row / W, w = row % W;
      const uint32_t* p = &tile_s[(tile * KVS_K_TILE + 4 * t4) * kPieceStride];
      store_stream(out + qi, uint4{compose3(p, w), compose3(p + kPieceStride, w), compose3(p + 2 * kPieceStride, w),
                                   compose3(p + 3 * kPieceStride, w)});
    } else {
      store_stream(out + qi, *reinterpret_cast<const uint4*>(&tile_s[row * TILE_STRIDE + 4 * t4]));
    }
  }
}

// ---------------------------------------------------------------------------------------------
// Keys of the per-token scheme (paper, Section 5.1): a Key row is quantised like a Value row,
// groups of G consecutive channels of one token; the packed words keep the Key layout.  Block =
// two 64-token code tiles; a lane owns channels 8 chunk .. + 7 of rows rslot, rslot + 16, ...
// ---------------------------------------------------------------------------------------------
template <int BITS, int G>
__global__ __launch_bounds__(kThreads) void quantize_k_token_fast_kernel(
    const uint4* __restrict__ K, const uint8_t* __restrict__ keep_mask, kvs::QuantSpan sp, int Hkv,
    uint32_t* __restrict__ k_codes, uint32_t* __restrict__ k_params, const int32_t* __restrict__ keep_idx,
    const int32_t* __restrict__ keep_cnt, int cap, uint4* __restrict__ keep_k,
    const uint32_t* __restrict__ static_k) {          // [Hkv, 128 / G] fixed parameter words, or null
  constexpr int TB = 2 * KVS_K_TILE;            // two code tiles per block
  constexpr int ROWS = TB / 16;                 // 8 rows per lane
  constexpr int LPG = G / 8;                    // lanes per channel group: 4, 8, 16
  constexpr int NGC = 128 / G;
  constexpr int ROWS_PER_LANE = LPG >= ROWS ? 1 : ROWS / LPG;   // rows whose parameters one lane derives
  constexpr int W = Fmt<BITS>::W;
  constexpr int TILE_STRIDE = 68;
  constexpr int LANES_PER_WORD = BITS == 2 ? 2 : 1;
  constexpr int kStage = BITS == 3 ? TB * kPieceStride : (TB / KVS_K_TILE) * W * TILE_STRIDE;

  __shared__ __align__(16) uint32_t tile_s[kStage];     // words as [tile][w][token]; 3 bit: pieces [token][16]

  const int tid = threadIdx.x;
  const int lane = tid & (KVS_WAVE - 1);
  const int chunk = tid & 15;
  const int rslot = tid >> 4;
  const int blocks_per_head = sp.n_tokens / TB;
  const int blk = blockIdx.x % blocks_per_head;
  const size_t bh = blockIdx.x / blocks_per_head;
  const int b = static_cast<int>(bh / Hkv);
  const int t0 = blk * TB;                      // input token; the cache token is sp.t_out + t0
  const int n = sp.n_cap;
  const int tc0 = sp.t_out + t0;
  const uint4* src = K + (bh * sp.n_in + t0) * 16;
  const uint8_t* mask_b = keep_mask + static_cast<size_t>(b) * sp.mask_stride + sp.mask_t0 + t0;

  uint4 raw[ROWS];
  bool kept[ROWS];
#pragma unroll
  for (int i = 0; i < ROWS; ++i) {
    const int r = rslot + 16 * i;
    raw[i] = load_stream(src + r * 16 + chunk);
    kept[i] = mask_b[r] != 0;
  }

  // (min, -max) of each row's group as one packed pair, reduced across the group's lanes.
  uint32_t stat[ROWS];
#pragma unroll
  for (int i = 0; i < ROWS; ++i) {
    const uint32_t mn2 = pk_min(pk_min(raw[i].x, raw[i].y), pk_min(raw[i].z, raw[i].w));
    const uint32_t mx2 = pk_max(pk_max(raw[i].x, raw[i].y), pk_max(raw[i].z, raw[i].w));
    const uint32_t mn1 = pk_min(mn2, mn2 >> 16) & 0xFFFFu;
    const uint32_t mx1 = pk_max(mx2, mx2 >> 16) & 0xFFFFu;
    uint32_t s = mn1 | ((mx1 ^ 0x8000u) << 16);
#pragma unroll
    for (int o = 1; o < LPG; o <<= 1) s = pk_min(s, static_cast<uint32_t>(__shfl_xor(static_cast<int>(s), o, KVS_WAVE)));
    stat[i] = s;
  }

  // Lane p of a group derives the parameters of the lane's rows p, p + LPG, ...; the others fetch them.
  const int p = chunk % LPG;
  const int group_base = lane - p;
  float inv_mine[ROWS_PER_LANE], zero_mine[ROWS_PER_LANE];
#pragma unroll
  for (int k = 0; k < ROWS_PER_LANE; ++k) {
    const int row = p + k * LPG;                // may exceed ROWS - 1 for idle lanes of wide groups
    uint32_t s = stat[0];
    bool kp = kept[0];
#pragma unroll
    for (int i = 1; i < ROWS; ++i) { s = row == i ? stat[i] : s; kp = row == i ? kept[i] : kp; }
    const Param prm = static_k ? param_of_word(static_k[(bh % Hkv) * NGC + chunk / LPG])
                               : make_param<BITS>(lo_half(s), -hi_half(s), !kp);
    inv_mine[k] = prm.inv;
    zero_mine[k] = prm.zero;
    if (row < ROWS) __builtin_nontemporal_store(prm.word, &k_params[(bh * n + static_cast<size_t>(tc0 + rslot + 16 * row)) * NGC + chunk / LPG]);
  }

  const int cnt = min(keep_cnt[b], cap);
#pragma unroll
  for (int i = 0; i < ROWS; ++i) {
    const int r = rslot + 16 * i;
    const int owner = group_base + (i % LPG);
    const int k = i / LPG;                      // compile-time after unrolling
    const float inv1 = __shfl(inv_mine[k < ROWS_PER_LANE ? k : 0], owner, KVS_WAVE);
    const float zero1 = __shfl(zero_mine[k < ROWS_PER_LANE ? k : 0], owner, KVS_WAVE);
    float inv[8], zero[8];
#pragma unroll
    for (int j = 0; j < 8; ++j) { inv[j] = inv1; zero[j] = zero1; }
    if constexpr (BITS == 8) {                  // two words per row and lane
      uint32_t lo = 0, hi = 0;
      if (!kept[i]) codes8_bytes(raw[i], inv, zero, lo, hi);
      tile_s[((r / KVS_K_TILE) * W + 2 * chunk) * TILE_STRIDE + (r % KVS_K_TILE)] = lo;
      tile_s[((r / KVS_K_TILE) * W + 2 * chunk + 1) * TILE_STRIDE + (r % KVS_K_TILE)] = hi;
    } else {
      uint32_t word = kept[i] ? 0u : codes8<BITS>(raw[i], inv, zero);
      if (LANES_PER_WORD == 2) {                  // 2 bit: lanes (even, odd) share a word
        const uint32_t other = static_cast<uint32_t>(__shfl_xor(static_cast<int>(word), 1, KVS_WAVE));
        word = word | (other << 16);
      }
      if (BITS == 3)
        tile_s[r * kPieceStride + chunk] = word;
      else if (LANES_PER_WORD == 1 || (chunk & 1) == 0)
        tile_s[((r / KVS_K_TILE) * W + chunk / LANES_PER_WORD) * TILE_STRIDE + (r % KVS_K_TILE)] = word;
    }
    if (kept[i]) {                              // exact copy of the row into the fp16 side buffer
      const int j = keep_slot(keep_idx + static_cast<size_t>(b) * cap, cnt, tc0 + r);
      if (j >= 0) keep_k[(bh * cap + j) * 16 + chunk] = raw[i];
    }
  }
  __syncthreads();

  // The block's words are contiguous in global memory in (tile, w, t) order: 128-bit stores.
  uint4* out = reinterpret_cast<uint4*>(k_codes + (bh * (n / KVS_K_TILE) + static_cast<size_t>(tc0 / KVS_K_TILE)) * (W * KVS_K_TILE));
  constexpr int quads = (TB / KVS_K_TILE) * W * (KVS_K_TILE / 4);
  for (int qi = tid; qi < quads; qi += kThreads) {
    const int row = qi / (KVS_K_TILE / 4), t4 = qi % (KVS_K_TILE / 4);
    if (BITS == 3) {
      const int tile = row / W, w = row % W;
      const uint32_t* pc = &tile_s[(tile * KVS_K_TILE + 4 * t4) * kPieceStride];
      store_stream(out + qi, uint4{compose3(pc, w), compose3(pc + kPieceStride, w), compose3(pc + 2 * kPieceStride, w),
                                   compose3(pc + 3 * kPieceStride, w)});
    } else {
      store_stream(out + qi, *reinterpret_cast<const uint4*>(&tile_s[row * TILE_STRIDE + 4 * t4]));
    }
  }
}

// ---------------------------------------------------------------------------------------------
// Values: per token, groups of G consecutive channels.  Block = one 128-token tile; a lane owns
// tokens 8 rs .. 8 rs + 7 and channels 8 chunk .. 8 chunk + 7.
// ---------------------------------------------------------------------------------------------
template <int BITS, int G, bool SPARSE>
__global__ __launch_bounds__(kThreads) void quantize_v_fast_kernel(
    const uint4* __restrict__ V, const uint8_t* __restrict__ keep_mask, kvs::QuantSpan sp, int Hkv,
    uint32_t* __restrict__ v_codes, uint32_t* __restrict__ v_params, const int32_t* __restrict__ keep_idx,
    const int32_t* __restrict__ keep_cnt, int cap, uint4* __restrict__ keep_v,
    const uint32_t* __restrict__ static_v,            // [Hkv, 128 / G] fixed parameter words, or null
    const uint32_t* __restrict__ tau_ptr, int32_t* __restrict__ row_count, kvs::SparseEmit emit) {   // SPARSE only
  constexpr int W = Fmt<BITS>::W;
  // SPARSE: which tokens of each channel are isolated (128 bits per channel = CSR row (b, h, tile,
  // channel)), where the channel's entries start inside the tile's run, where the run starts.
  __shared__ uint32_t iso_s[SPARSE ? 128 : 1][4];
  __shared__ int chan_off_s[SPARSE ? 128 : 1];
  __shared__ int run_base_s;
  __shared__ uint32_t spread_s[SPARSE ? 256 : 1];
  constexpr int LPG = G / 8;                    // lanes per channel group: 4, 8, 16
  constexpr int NGC = 128 / G;
  constexpr int ROWS_PER_LANE = LPG >= 8 ? 1 : 8 / LPG;   // rows whose parameters one lane derives

  const int tid = threadIdx.x;
  const int lane = tid & (KVS_WAVE - 1);
  const int chunk = tid & 15;
  const int rs = tid >> 4;                      // token word: tokens 8 rs .. 8 rs + 7
  const int tiles_in = sp.n_tokens / KVS_V_TILE;
  const int tile_in = blockIdx.x % tiles_in;
  const size_t bh = blockIdx.x / tiles_in;
  const int b = static_cast<int>(bh / Hkv);
  const int n = sp.n_cap;                       // layout of everything written
  const int tiles_per_head = n / KVS_V_TILE;
  const int tile = sp.t_out / KVS_V_TILE + tile_in;
  const int t0 = tile * KVS_V_TILE;             // cache token of the tile's first row
  const uint4* src = V + (bh * sp.n_in + tile_in * KVS_V_TILE + 8 * rs) * 16 + chunk;
  // (a prompt's mask rows may start at any byte)
  const uint8_t* mrow = keep_mask + static_cast<size_t>(b) * sp.mask_stride + sp.mask_t0 + tile_in * KVS_V_TILE + 8 * rs;
  uint2 mask8;
  if (((sp.mask_stride | sp.mask_t0) & 7) == 0) {
    mask8 = *reinterpret_cast<const uint2*>(mrow);
  } else {
    mask8.x = mrow[0] | (mrow[1] << 8) | (mrow[2] << 16) | (static_cast<uint32_t>(mrow[3]) << 24);
    mask8.y = mrow[4] | (mrow[5] << 8) | (mrow[6] << 16) | (static_cast<uint32_t>(mrow[7]) << 24);
  }

  uint4 raw[8];
#pragma unroll
  for (int i = 0; i < 8; ++i) raw[i] = load_stream(src + i * 16);

  uint32_t tau2 = 0;
  if (SPARSE) {
    const uint32_t tau = *tau_ptr;                 // 0x8000: no magnitude pattern reaches it
    tau2 = tau | (tau << 16);
    if constexpr (BITS != 8) fill_spread_table<BITS>(spread_s, tid);
  }
  uint32_t iso_lo = 0, iso_hi = 0;                // SPARSE: byte i = isolated channels of the lane's token i;
  uint32_t row_lo = 0, row_hi = 0;                // after the transposition byte j = isolated tokens of channel j
  int run_claim = 0;                              // SPARSE, last lane: start of the tile's run in the staging list

  // (min, -max) of the lane's 8 values of each row as one packed pair, then across the group's
  // lanes: one packed minimum per step does both.
  uint32_t stat[8];
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    uint32_t a4[4] = {raw[i].x, raw[i].y, raw[i].z, raw[i].w};   // operands of the minimum
    uint32_t z4[4] = {raw[i].x, raw[i].y, raw[i].z, raw[i].w};   // operands of the maximum
    if (SPARSE) {
      uint32_t m[4];
#pragma unroll
      for (int k = 0; k < 4; ++k) {
        m[k] = kvs::below_mask(a4[k], tau2);
        z4[k] = select_halves(m[k], a4[k], kNegMax2);
        a4[k] = select_halves(m[k], a4[k], kPosMax2);
      }
      const bool kept_i = ((i < 4 ? mask8.x >> (8 * i) : mask8.y >> (8 * (i - 4))) & 0xFFu) != 0;
      const uint32_t bits = kept_i ? 0u : kvs::isolated8(m);
      if (i < 4) iso_lo |= bits << (8 * i); else iso_hi |= bits << (8 * (i - 4));
    }
    const uint32_t mn2 = pk_min(pk_min(a4[0], a4[1]), pk_min(a4[2], a4[3]));
    const uint32_t mx2 = pk_max(pk_max(z4[0], z4[1]), pk_max(z4[2], z4[3]));
    const uint32_t mn1 = pk_min(mn2, mn2 >> 16) & 0xFFFFu;
    const uint32_t mx1 = pk_max(mx2, mx2 >> 16) & 0xFFFFu;
    uint32_t s = mn1 | ((mx1 ^ 0x8000u) << 16);
#pragma unroll
    for (int o = 1; o < LPG; o <<= 1) s = pk_min(s, static_cast<uint32_t>(__shfl_xor(static_cast<int>(s), o, KVS_WAVE)));
    stat[i] = s;
  }

  if (SPARSE) {
    // Channel-major masks: byte rs of channel 8 chunk + j = which of the lane's eight tokens are
    // isolated in that channel.  Then the last wave turns them into channel counts (CSR row =
    // (tile, channel)), scans them over the tile and claims the tile's run in the staging list.
    row_lo = iso_lo;  row_hi = iso_hi;
    transpose8x8(iso_lo, iso_hi);
    uint8_t* iso_b = reinterpret_cast<uint8_t*>(&iso_s[0][0]);
#pragma unroll
    for (int j = 0; j < 8; ++j)
      iso_b[(8 * chunk + j) * 16 + rs] = static_cast<uint8_t>((j < 4 ? iso_lo >> (8 * j) : iso_hi >> (8 * (j - 4))) & 0xFFu);
    __syncthreads();
    if (tid >= kThreads - KVS_WAVE) {
      const int sl = tid - (kThreads - KVS_WAVE);
      int cnt[2], mine = 0;
#pragma unroll
      for (int k = 0; k < 2; ++k) {
        const int c = 2 * sl + k;
        cnt[k] = __popc(iso_s[c][0]) + __popc(iso_s[c][1]) + __popc(iso_s[c][2]) + __popc(iso_s[c][3]);
        row_count[(bh * tiles_per_head + static_cast<size_t>(tile)) * 128 + c] = cnt[k];
        mine += cnt[k];
      }
      int incl = mine;
#pragma unroll
      for (int o = 1; o < KVS_WAVE; o <<= 1) {
        const int up = __shfl_up(incl, o, KVS_WAVE);
        if (sl >= o) incl += up;
      }
      chan_off_s[2 * sl] = incl - mine;
      chan_off_s[2 * sl + 1] = incl - mine + cnt[0];
      // requested now, needed only when the entries are written out
      if (sl == KVS_WAVE - 1 && incl > 0) run_claim = kvs::claim_run(emit, incl);
    }
  }

  // Lane p of a group derives the parameters of rows p, p + LPG, ...; the others fetch them.
  const int p = chunk % LPG;
  const int group_base = lane - p;
  float inv_mine[ROWS_PER_LANE], zero_mine[ROWS_PER_LANE];
#pragma unroll
  for (int k = 0; k < ROWS_PER_LANE; ++k) {
    const int row = p + k * LPG;                // may exceed 7 for idle lanes of wide groups
    uint32_t s = stat[0];
#pragma unroll
    for (int i = 1; i < 8; ++i) s = row == i ? stat[i] : s;
    const bool kept = row < 8 && ((row < 4 ? mask8.x >> (8 * row) : mask8.y >> (8 * (row - 4))) & 0xFFu) != 0;
    // SPARSE: a group can lose every entry to the CSR
    const bool any = !kept && (!SPARSE || lo_half(s) <= -hi_half(s));
    const Param prm = static_v ? param_of_word(static_v[(bh % Hkv) * NGC + chunk / LPG])
                               : make_param<BITS>(lo_half(s), -hi_half(s), any);
    inv_mine[k] = prm.inv;
    zero_mine[k] = prm.zero;
    if (row < 8) __builtin_nontemporal_store(prm.word, &v_params[(bh * n + static_cast<size_t>(t0 + 8 * rs + row)) * NGC + chunk / LPG]);
  }

  const int cnt = min(keep_cnt[b], cap);
  uint32_t words[8];                            // word j: channel 8 chunk + j, tokens 8 rs .. + 7
  uint32_t words_hi[BITS == 8 ? 8 : 1];         // 8 bit: tokens 8 rs + 4 .. + 7 fill a second word
#pragma unroll
  for (int j = 0; j < 8; ++j) words[j] = 0;
#pragma unroll
  for (int j = 0; j < (BITS == 8 ? 8 : 1); ++j) words_hi[j] = 0;
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    const int owner = group_base + (i % LPG);
    const int k = i / LPG;                      // compile-time after unrolling
    const float inv = __shfl(inv_mine[k < ROWS_PER_LANE ? k : 0], owner, KVS_WAVE);
    const float zero = __shfl(zero_mine[k < ROWS_PER_LANE ? k : 0], owner, KVS_WAVE);
    const bool kept = ((i < 4 ? mask8.x >> (8 * i) : mask8.y >> (8 * (i - 4))) & 0xFFu) != 0;
    if (!kept) {
      const uint32_t w4[4] = {raw[i].x, raw[i].y, raw[i].z, raw[i].w};
#pragma unroll
      for (int c = 0; c < 4; ++c) {
        if constexpr (BITS == 8) {
          uint32_t* dst = i < 4 ? words : words_hi;
          dst[2 * c] |= code_of<8>(lo_half(w4[c]), inv, zero) << (8 * (i & 3));
          dst[2 * c + 1] |= code_of<8>(hi_half(w4[c]), inv, zero) << (8 * (i & 3));
        } else {
          words[2 * c] |= code_of<BITS>(lo_half(w4[c]), inv, zero) << (BITS * i);
          words[2 * c + 1] |= code_of<BITS>(hi_half(w4[c]), inv, zero) << (BITS * i);
        }
      }
    } else {
      const int j = keep_slot(keep_idx + static_cast<size_t>(b) * cap, cnt, t0 + 8 * rs + i);
      if (j >= 0) keep_v[(bh * cap + j) * 16 + chunk] = raw[i];
    }
  }
  if (SPARSE) {
#pragma unroll
    for (int j = 0; j < 8; ++j)                   // isolated entries hold code 0
      words[j] &= ~spread_s[(j < 4 ? iso_lo >> (8 * j) : iso_hi >> (8 * (j - 4))) & 0xFFu];
    // Isolated entries to the tile's run of the staging list in final order (channels ascending,
    // tokens ascending inside a channel): the lane that holds an entry writes it from its
    // registers; its place is the channel's start plus the channel's entries at earlier tokens.
    if (tid == kThreads - 1) {                    // the claim has had the whole code phase to return
      emit.block_base[blockIdx.x] = run_claim;
      run_base_s = run_claim;
    }
    __syncthreads();
    // (the list is addressed from the run's start, the same for the whole workgroup, with 32-bit
    // positions; `room` is what is left of the list behind it)
    const int run_base = __builtin_amdgcn_readfirstlane(run_base_s);
    const long long left = kvs::emit_list_words(emit.cap) - run_base;
    const int room = left < 0 ? 0 : (left > 0x7FFFFFFF ? 0x7FFFFFFF : static_cast<int>(left));
    uint32_t* run = emit.list + run_base;
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      uint32_t bits = (i < 4 ? row_lo >> (8 * i) : row_hi >> (8 * (i - 4))) & 0xFFu;   // channels of token 8 rs + i
      while (bits) {
        const int j = __builtin_ctz(bits);
        bits &= bits - 1;
        const int c = 8 * chunk + j;
        const uint32_t tokens = (j < 4 ? iso_lo >> (8 * j) : iso_hi >> (8 * (j - 4))) & 0xFFu;   // the lane's tokens of channel c
        const int pos = chan_off_s[c] + bits_below_byte(&iso_s[c][0], rs) + __popc(tokens & ((1u << i) - 1u));
        if (pos < room)                            // token inside the tile | channel << 7 | fp16 value << 16
          run[pos] = static_cast<uint32_t>(8 * rs + i) | (static_cast<uint32_t>(c) << 7) | (half_of(raw[i], j) << 16);
      }
    }
  }
  if (BITS == 3) {                              // pieces [channel][token octet] -> 13 words per channel
    __shared__ uint32_t piece_s[128 * kPieceStride];
#pragma unroll
    for (int j = 0; j < 8; ++j) piece_s[(8 * chunk + j) * kPieceStride + rs] = words[j];
    __syncthreads();
    uint4* out = reinterpret_cast<uint4*>(v_codes + (bh * tiles_per_head + static_cast<size_t>(tile)) * (W * 128));
    for (int qi = tid; qi < W * 32; qi += kThreads) {      // four channels of one word row per step
      const int u = qi / 32, c4 = qi % 32;
      const uint32_t* p = &piece_s[4 * c4 * kPieceStride];
      store_stream(out + qi, uint4{compose3(p, u), compose3(p + kPieceStride, u), compose3(p + 2 * kPieceStride, u),
                                   compose3(p + 3 * kPieceStride, u)});
    }
    return;
  }
  if constexpr (BITS == 8) {                    // four tokens per word: word rows 2 rs and 2 rs + 1
    uint4* out = reinterpret_cast<uint4*>(v_codes + (bh * tiles_per_head + static_cast<size_t>(tile)) * (W * 128) + 2 * rs * 128 + 8 * chunk);
    store_stream(out, uint4{words[0], words[1], words[2], words[3]});
    store_stream(out + 1, uint4{words[4], words[5], words[6], words[7]});
    store_stream(out + 32, uint4{words_hi[0], words_hi[1], words_hi[2], words_hi[3]});
    store_stream(out + 33, uint4{words_hi[4], words_hi[5], words_hi[6], words_hi[7]});
    return;
  }
  if (BITS == 2) {                              // 16 tokens per word: row slots (even, odd) share it
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      const uint32_t other = static_cast<uint32_t>(__shfl_xor(static_cast<int>(words[j]), 16, KVS_WAVE));
      words[j] |= other << 16;
    }
  }
  if (BITS == 4 || (rs & 1) == 0) {
    const int u = BITS == 4 ? rs : rs / 2;
    uint4* out = reinterpret_cast<uint4*>(v_codes + (bh * tiles_per_head + static_cast<size_t>(tile)) * (W * 128) + u * 128 + 8 * chunk);
    store_stream(out, uint4{words[0], words[1], words[2], words[3]});
    store_stream(out + 1, uint4{words[4], words[5], words[6], words[7]});
  }
}

// Index list of the kept tokens (ascending), count, mask copy, overflow status, and zero padding
// of the unused rows of the fp16 side buffers.  One workgroup of 16 waves per sequence: wave w
// owns one contiguous segment of the mask (a multiple of 1024 bytes: 16 per lane and step), first
// counts its kept tokens, then - knowing how many lie before its segment - writes their indices.
constexpr int kIndexWaves = 16;
__global__ __launch_bounds__(kIndexWaves * KVS_WAVE) void keep_index_fast_kernel(
    const uint8_t* __restrict__ keep_mask, int n, int Hkv, int cap, int32_t* __restrict__ keep_idx,
    int32_t* __restrict__ keep_cnt, uint8_t* __restrict__ mask_copy, int32_t* __restrict__ status,
    uint4* __restrict__ keep_k, uint4* __restrict__ keep_v) {
  __shared__ int wave_count[kIndexWaves];
  const int b = blockIdx.x, tid = threadIdx.x;
  const int lane = tid & (KVS_WAVE - 1), wave = tid / KVS_WAVE;
  const uint8_t* m = keep_mask + static_cast<size_t>(b) * n;
  uint8_t* mc = mask_copy + static_cast<size_t>(b) * n;
  constexpr int kStep = KVS_WAVE * 16;                   // bytes one wave takes per step
  const int seg = ((n + kIndexWaves * kStep - 1) / (kIndexWaves * kStep)) * kStep;   // bytes per wave
  const int seg_begin = min(n, wave * seg), seg_end = min(n, seg_begin + seg);

  // bit 0 of each byte of the result = the mask byte is nonzero (n is a multiple of 128, so a
  // lane's 16 bytes are either all inside the sequence or all outside)
  auto load_norm = [&](int i, uint32_t (&norm)[4]) -> int {
    uint4 v = {0, 0, 0, 0};
    if (i < seg_end) v = *reinterpret_cast<const uint4*>(m + i);
    const uint32_t w[4] = {v.x, v.y, v.z, v.w};
    int mine = 0;
#pragma unroll
    for (int k = 0; k < 4; ++k) {
      uint32_t nz = w[k] | (w[k] >> 4);
      nz |= nz >> 2;  nz |= nz >> 1;
      norm[k] = nz & 0x01010101u;
      mine += __popc(norm[k]);
    }
    return mine;
  };

  int count = 0;
  for (int i0 = seg_begin; i0 < seg_end; i0 += kStep) {
    uint32_t norm[4];
    count += load_norm(i0 + lane * 16, norm);
  }
#pragma unroll
  for (int o = KVS_WAVE / 2; o > 0; o >>= 1) count += __shfl_xor(count, o, KVS_WAVE);
  if (lane == 0) wave_count[wave] = count;
  __syncthreads();
  int base = 0, total = 0;
#pragma unroll
  for (int w = 0; w < kIndexWaves; ++w) {
    base += w < wave ? wave_count[w] : 0;
    total += wave_count[w];
  }

  for (int i0 = seg_begin; i0 < seg_end; i0 += kStep) {  // the segment again (cache hits)
    const int i = i0 + lane * 16;
    uint32_t norm[4];
    const int mine = load_norm(i, norm);
    if (i < seg_end) *reinterpret_cast<uint4*>(mc + i) = uint4{norm[0], norm[1], norm[2], norm[3]};
    int incl = mine;
#pragma unroll
    for (int o = 1; o < KVS_WAVE; o <<= 1) {
      const int up = __shfl_up(incl, o, KVS_WAVE);
      if (lane >= o) incl += up;
    }
    int pos = base + incl - mine;
#pragma unroll
    for (int k = 0; k < 4; ++k)
#pragma unroll
      for (int j = 0; j < 4; ++j)
        if ((norm[k] >> (8 * j)) & 1u) {
          if (pos < cap) keep_idx[static_cast<size_t>(b) * cap + pos] = i + 4 * k + j;
          ++pos;
        }
    base += __shfl(incl, KVS_WAVE - 1, KVS_WAVE);
  }

  for (int j = total + tid; j < cap; j += kIndexWaves * KVS_WAVE) keep_idx[static_cast<size_t>(b) * cap + j] = -1;
  if (tid == 0) {
    keep_cnt[b] = total;
    if (total > cap) atomicCAS(status, 0, static_cast<int>(KVS_ERR_CAPACITY));
  }
  // zero the rows past the count, for every head of this sequence (16 uint4 per row)
  const int first = min(total, cap);
  const int per_head = (cap - first) * 16;
  for (int h = 0; h < Hkv; ++h) {
    const size_t row0 = ((static_cast<size_t>(b) * Hkv + h) * cap + first) * 16;
    for (int e = tid; e < per_head; e += kIndexWaves * KVS_WAVE) {
      keep_k[row0 + e] = uint4{0, 0, 0, 0};
      keep_v[row0 + e] = uint4{0, 0, 0, 0};
    }
  }
}

// ---------------------------------------------------------------------------------------------
// Static quantisation (paper, Appendix C "Dynamic and static quantization"; Table 1's setting:
// global min-max, kept tokens left out of the calibration).  The calibration state is four
// arrays [Hkv, 128] - Key minimum, Key maximum, Value minimum, Value maximum per channel - of
// floats in an order-preserving unsigned encoding, so that they can be lowered / raised with
// integer atomics by any number of calls.
// ---------------------------------------------------------------------------------------------
constexpr int kCalibTokens = 1024;              // tokens of one (b, h) per workgroup
__device__ inline uint32_t order_key(float f) {
  const uint32_t u = __builtin_bit_cast(uint32_t, f);
  return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}
__device__ inline float order_value(uint32_t k) {
  return __builtin_bit_cast(float, (k & 0x80000000u) ? (k & 0x7FFFFFFFu) : ~k);
}

__global__ void calibrate_reset_kernel(uint32_t* __restrict__ calib, int Hkv) {
  const int i = blockIdx.x * 128 + threadIdx.x;
  const int plane = Hkv * 128;
  calib[i] = order_key(INFINITY);                // Key minimum
  calib[plane + i] = order_key(-INFINITY);       // Key maximum
  calib[2 * plane + i] = order_key(INFINITY);    // Value minimum
  calib[3 * plane + i] = order_key(-INFINITY);   // Value maximum
}

// blockIdx.y: 0 = Keys, 1 = Values.  Lane = 8 channels of every 16th row of the segment.
__global__ __launch_bounds__(kThreads) void calibrate_kernel(
    const uint4* __restrict__ K, const uint4* __restrict__ V, const uint8_t* __restrict__ keep_mask, int n, int Hkv,
    uint32_t* __restrict__ calib) {
  __shared__ uint32_t red_mn[16][64], red_mx[16][64];
  const int tid = threadIdx.x, chunk = tid & 15, rslot = tid >> 4;
  const int segs = (n + kCalibTokens - 1) / kCalibTokens;
  const int seg = blockIdx.x % segs;
  const size_t bh = blockIdx.x / segs;
  const int b = static_cast<int>(bh / Hkv), h = static_cast<int>(bh % Hkv);
  const uint4* X = (blockIdx.y == 0 ? K : V) + bh * n * 16;
  const uint8_t* mask_b = keep_mask + static_cast<size_t>(b) * n;
  const int t_end = min(n, (seg + 1) * kCalibTokens);
  uint32_t mn[4] = {kPosMax2, kPosMax2, kPosMax2, kPosMax2};
  uint32_t mx[4] = {kNegMax2, kNegMax2, kNegMax2, kNegMax2};
  bool any = false;
  for (int t = seg * kCalibTokens + rslot; t < t_end; t += 16) {
    if (mask_b[t]) continue;
    const uint4 raw = load_stream(X + static_cast<size_t>(t) * 16 + chunk);
    mn[0] = pk_min(mn[0], raw.x); mn[1] = pk_min(mn[1], raw.y); mn[2] = pk_min(mn[2], raw.z); mn[3] = pk_min(mn[3], raw.w);
    mx[0] = pk_max(mx[0], raw.x); mx[1] = pk_max(mx[1], raw.y); mx[2] = pk_max(mx[2], raw.z); mx[3] = pk_max(mx[3], raw.w);
    any = true;
  }
  *reinterpret_cast<uint4*>(&red_mn[rslot][4 * chunk]) = uint4{mn[0], mn[1], mn[2], mn[3]};
  *reinterpret_cast<uint4*>(&red_mx[rslot][4 * chunk]) = uint4{mx[0], mx[1], mx[2], mx[3]};
  const bool any_wg = __syncthreads_or(any ? 1 : 0) != 0;
  if (any_wg && tid < 64) {                       // channel pair tid
    uint32_t a = kPosMax2, z = kNegMax2;
#pragma unroll
    for (int s = 0; s < 16; ++s) { a = pk_min(a, red_mn[s][tid]); z = pk_max(z, red_mx[s][tid]); }
    const int plane = Hkv * 128;
    uint32_t* base = calib + (blockIdx.y == 0 ? 0 : 2 * plane) + h * 128 + 2 * tid;
    atomicMin(base, order_key(lo_half(a)));
    atomicMin(base + 1, order_key(hi_half(a)));
    atomicMax(base + plane, order_key(lo_half(z)));
    atomicMax(base + plane + 1, order_key(hi_half(z)));
  }
}

// One workgroup per KV head: the parameter word of every Key channel and Value channel group.
template <int BITS>
__global__ void static_params_kernel(const uint32_t* __restrict__ calib, int Hkv, int group, int key_per_token,
                                     uint32_t* __restrict__ static_k, uint32_t* __restrict__ static_v) {
  const int h = blockIdx.x, c = threadIdx.x;
  const int plane = Hkv * 128;
  if (!key_per_token) {
    const float kmn = order_value(calib[h * 128 + c]), kmx = order_value(calib[plane + h * 128 + c]);
    static_k[h * 128 + c] = make_param<BITS>(kmn, kmx, kmn <= kmx).word;
  } else if (c < 128 / group) {                  // one word per Key channel group, as for Values
    float kmn = INFINITY, kmx = -INFINITY;
    for (int j = 0; j < group; ++j) {
      kmn = fminf(kmn, order_value(calib[h * 128 + c * group + j]));
      kmx = fmaxf(kmx, order_value(calib[plane + h * 128 + c * group + j]));
    }
    static_k[h * (128 / group) + c] = make_param<BITS>(kmn, kmx, kmn <= kmx).word;
  }
  if (c < 128 / group) {
    float vmn = INFINITY, vmx = -INFINITY;
    for (int j = 0; j < group; ++j) {
      vmn = fminf(vmn, order_value(calib[2 * plane + h * 128 + c * group + j]));
      vmx = fmaxf(vmx, order_value(calib[3 * plane + h * 128 + c * group + j]));
    }
    static_v[h * (128 / group) + c] = make_param<BITS>(vmn, vmx, vmn <= vmx).word;
  }
}

template <int BITS, int G>
void launch_fast(const kvs_desc* d, const kvs::QuantSpan& sp, bool own_keep, const void* K, const void* V,
                 const uint8_t* mask, const kvs_cache* out, const uint32_t* static_k, const uint32_t* static_v,
                 const kvs::SparsePlan* plan, hipStream_t s) {
  constexpr int TB = G > 64 ? G : 64;
  const int bh = d->B * d->Hkv;
  const int cap = own_keep ? d->keep_cap : 0;            // 0: the kernels copy no kept rows themselves
  if (own_keep)
    hipLaunchKernelGGL(keep_index_fast_kernel, dim3(d->B), dim3(kIndexWaves * KVS_WAVE), 0, s, mask, d->n, d->Hkv, d->keep_cap,
                       out->keep_idx, out->keep_cnt, out->keep_mask, out->status, static_cast<uint4*>(out->keep_k),
                       static_cast<uint4*>(out->keep_v));
  if (sp.n_tokens == 0) return;
  if (d->key_per_token)
    hipLaunchKernelGGL((quantize_k_token_fast_kernel<BITS, G>), dim3(bh * (sp.n_tokens / (2 * KVS_K_TILE))), dim3(kThreads), 0, s,
                       static_cast<const uint4*>(K), mask, sp, d->Hkv, out->k_codes, out->k_params, out->keep_idx,
                       out->keep_cnt, cap, static_cast<uint4*>(out->keep_k), static_k);
  else if (plan) {    // isolated outliers: thresholds plan->tau[0 / 1], row counts behind the row pointers' first word
    if constexpr (BITS != 8)                     // (never asked for at 8 bit: the descriptor check refuses it)
      hipLaunchKernelGGL((quantize_k_fast_kernel<BITS, G, true>), dim3(bh * (sp.n_tokens / TB)), dim3(kThreads), 0, s,
                         static_cast<const uint4*>(K), mask, sp, d->Hkv, out->k_codes, out->k_params, out->keep_idx,
                         out->keep_cnt, cap, static_cast<uint4*>(out->keep_k), static_k, plan->tau, out->k_rowptr + 1,
                         plan->emit_k);
  } else
    hipLaunchKernelGGL((quantize_k_fast_kernel<BITS, G, false>), dim3(bh * (sp.n_tokens / TB)), dim3(kThreads), 0, s,
                       static_cast<const uint4*>(K), mask, sp, d->Hkv, out->k_codes, out->k_params, out->keep_idx,
                       out->keep_cnt, cap, static_cast<uint4*>(out->keep_k), static_k, nullptr, nullptr,
                       kvs::SparseEmit{});
  if (plan) {
    if constexpr (BITS != 8)
      hipLaunchKernelGGL((quantize_v_fast_kernel<BITS, G, true>), dim3(bh * (sp.n_tokens / KVS_V_TILE)), dim3(kThreads), 0, s,
                         static_cast<const uint4*>(V), mask, sp, d->Hkv, out->v_codes, out->v_params, out->keep_idx,
                         out->keep_cnt, cap, static_cast<uint4*>(out->keep_v), static_v, plan->tau + 1, out->v_rowptr + 1,
                         plan->emit_v);
  } else
    hipLaunchKernelGGL((quantize_v_fast_kernel<BITS, G, false>), dim3(bh * (sp.n_tokens / KVS_V_TILE)), dim3(kThreads), 0, s,
                       static_cast<const uint4*>(V), mask, sp, d->Hkv, out->v_codes, out->v_params, out->keep_idx,
                       out->keep_cnt, cap, static_cast<uint4*>(out->keep_v), static_v, nullptr, nullptr,
                       kvs::SparseEmit{});
}

template <int BITS>
void launch_fast_g(const kvs_desc* d, const kvs::QuantSpan& sp, bool own_keep, const void* K, const void* V,
                   const uint8_t* mask, const kvs_cache* out, const uint32_t* static_k, const uint32_t* static_v,
                   const kvs::SparsePlan* plan, hipStream_t s) {
  switch (d->group) {
    case 32: launch_fast<BITS, 32>(d, sp, own_keep, K, V, mask, out, static_k, static_v, plan, s); break;
    case 64: launch_fast<BITS, 64>(d, sp, own_keep, K, V, mask, out, static_k, static_v, plan, s); break;
    default: launch_fast<BITS, 128>(d, sp, own_keep, K, V, mask, out, static_k, static_v, plan, s); break;
  }
}

}  // namespace

namespace kvs {

void launch_quantize_fast(const kvs_desc* d, const QuantSpan& sp, bool own_keep, const void* K, const void* V,
                          const uint8_t* mask, const kvs_cache* out, const uint32_t* static_k, const uint32_t* static_v,
                          const SparsePlan* plan, hipStream_t s) {
  if (d->bits == 2) launch_fast_g<2>(d, sp, own_keep, K, V, mask, out, static_k, static_v, plan, s);
  else if (d->bits == 3) launch_fast_g<3>(d, sp, own_keep, K, V, mask, out, static_k, static_v, plan, s);
  else if (d->bits == 4) launch_fast_g<4>(d, sp, own_keep, K, V, mask, out, static_k, static_v, plan, s);
  else launch_fast_g<8>(d, sp, own_keep, K, V, mask, out, static_k, static_v, plan, s);
}

void launch_calibrate_reset(const kvs_desc* d, uint32_t* calib, hipStream_t s) {
  hipLaunchKernelGGL(calibrate_reset_kernel, dim3(d->Hkv), dim3(128), 0, s, calib, d->Hkv);
}
void launch_calibrate(const kvs_desc* d, const void* K, const void* V, const uint8_t* mask, uint32_t* calib,
                      hipStream_t s) {
  const int segs = (d->n + kCalibTokens - 1) / kCalibTokens;
  hipLaunchKernelGGL(calibrate_kernel, dim3(d->B * d->Hkv * segs, 2), dim3(kThreads), 0, s,
                     static_cast<const uint4*>(K), static_cast<const uint4*>(V), mask, d->n, d->Hkv, calib);
}
void launch_static_params(const kvs_desc* d, const uint32_t* calib, uint32_t* static_k, uint32_t* static_v,
                          hipStream_t s) {
  if (d->bits == 2) hipLaunchKernelGGL(static_params_kernel<2>, dim3(d->Hkv), dim3(128), 0, s, calib, d->Hkv, d->group, d->key_per_token, static_k, static_v);
  else if (d->bits == 3) hipLaunchKernelGGL(static_params_kernel<3>, dim3(d->Hkv), dim3(128), 0, s, calib, d->Hkv, d->group, d->key_per_token, static_k, static_v);
  else if (d->bits == 4) hipLaunchKernelGGL(static_params_kernel<4>, dim3(d->Hkv), dim3(128), 0, s, calib, d->Hkv, d->group, d->key_per_token, static_k, static_v);
  else hipLaunchKernelGGL(static_params_kernel<8>, dim3(d->Hkv), dim3(128), 0, s, calib, d->Hkv, d->group, d->key_per_token, static_k, static_v);
}

}  // namespace kvs

// Matrix-core decode-attention kernel over the packed low-bit KV cache, all bit widths and group
// sizes (paper, Section 2 attention equation over the quantised cache; the sink / non-sink split
// of Section 4.2).  Included by decode_mfma_b{2,3,4,8}.hip and decode_mfma_kpt_b{2,3,4,8}.hip,
// one bit width each.
//
// Dequantised values are never formed.  With x' = scale (code - zero) (Appendix C):
//   score[t]  = sum_c q_c scale_c (code[t, c] - zero_c)        per-channel Keys, one (scale, zero)
//             = sum_c (q scale)_c code[t, c] - sum_c (q scale)_c zero_c     per channel and token group:
//     the scale goes into the query once per token group, the zero points into one bias per group;
//   out[c]    = sum_t p_t scale_t (code[t, c] - zero_t)        per-token Values, one (scale, zero)
//             = sum_t (p scale)_t code[t, c] - sum_t (p scale)_t zero_t     per token and channel group:
//     the scale goes into the softmax weight, the zero points into one running scalar per channel
//     group.  Kept tokens get weight zero here (their fp16 rows are merged separately).
//
// Why matrix cores even for a one-row query: at ~0.5 byte per cached element the HBM stream
// delivers ~1e13 codes/s, and unpack + convert + multiply-add on the vector ALU costs 3+
// instructions per code, which is what bounded a vector-ALU version of this kernel.  Here a code becomes an fp16
// operand with ~0.6 instruction: a b-bit field sitting in mantissa bits [p, p+b) of a half whose
// exponent field is set to 25 - p reads as 2^(10-p) + code, so (w & mask) | magic yields two
// operands at once and most fields need no shift.  The additive offsets leave with the zero
// points.  The products run on v_mfma_f32_16x16x32_f16; spare columns of the 16-wide tile carry
// the low half of an fp16 hi/lo split of the other operand (query x scale, weight x scale), so
// the fp16 rounding of that operand does not reach the result, and - for group size 32 - the
// second quantisation group that a 64-row tile spans.
//
// A workgroup of 8 waves (4 for the register-hungry variants, see waves_for) owns one part of the
// token range of one (sequence, KV head); its
// 128-token chunks are handed to the waves on demand (a counter in LDS), each wave keeping the
// next chunk's codes in flight, and the waves meet once, at the end, to merge their running
// softmax states in LDS.  (Which wave gets which chunk depends on timing, so the fp32 summation
// order - not the result beyond rounding - can differ between two runs.)  When a single
// workgroup covers the whole sequence the kept (sink) tokens' fp16 rows are folded in - wave w
// takes rows w, w + waves, ... as one more softmax state - and the output row is written right
// there; otherwise the part's state goes to the workspace, the workgroup counts itself in on the
// (sequence, KV head)'s arrival counter, and the workgroup that arrives last merges all parts,
// folds the kept rows in and writes the output rows (the counter block heads the workspace; it
// is zero before the call and the last arriver leaves it zero).  Per 128-token chunk:
//   scores  S^T[token, col] = sum_c code[token, c] * B[c, col]     tokens are the M rows
//   softmax with lane = token (scores pass through LDS once)
//   output  O^T[chan, col] = sum_t code[t, chan] * W[t, col]       channels are the M rows
// Operand layouts follow the instruction: lane l holds row (l % 16) and the 8 contraction
// indices of chunk (l / 16); the result holds rows 4 (l / 16) + i of column (l % 16).
#pragma once

#include "decode_finish.h"
#include "kvs_device.h"

namespace kvs_mfma {

typedef _Float16 half8 __attribute__((ext_vector_type(8)));
typedef float float4v __attribute__((ext_vector_type(4)));

// Waves per workgroup: 8, two per SIMD with up to 256 registers each, or 4 with up to 512.  At
// 8 bit the stream registers of a wave double, and the variants that also carry several (head,
// group) columns spill with 256 (1.3 - 2.3 times the run time); so do a few low-bit variants.
// The table is by measurement: four waves where that was faster, eight elsewhere (a variant that
// spills a few dozen bytes can still be faster with eight).
__host__ __device__ constexpr int waves_for(int bits, int G, int R, bool kpt, bool sparse = false) {
  if (sparse && (R == 8 || (G == 32 && R == 4))) return 4;   // the outlier tables of eight waves would not fit the LDS
  if (bits == 8) return R * (128 / G) * (kpt ? 2 : 1) >= 4 ? 4 : 8;
  if (!kpt) return ((bits >= 3 && G == 32 && R == 4) || (G == 64 && R == 8)) ? 4 : 8;   // (64, 8): the tables of 8 waves exceed the LDS
  if (bits >= 3 && G == 128 && R == 8) return 4;
  return 8;
}
constexpr float kLog2eRsqrtD = 1.4426950408889634f * 0.08838834764831845f;   // log2(e) / sqrt(128)
constexpr float kLn2 = 0.6931471805599453f;
constexpr int kWsRow = KVS_HEAD_DIM + 2;

// Exponent patterns (both halves) under which a field at mantissa bit p reads 2^(10-p) + code.
// They live in vector registers so that (x & mask) | magic is one v_and_or_b32; the empty asm
// emits nothing and only hides the constants from the compiler, which would otherwise split
// the operation in two.
struct Magic {
  uint32_t m0, m2, m3, m4, m6, m8;   // fields at mantissa bit 0, 2, 3, 4, 6, 8
};
__device__ inline Magic make_magic() {
  Magic m{0x64006400u, 0x5C005C00u, 0x58005800u, 0x54005400u, 0x4C004C00u, 0x44004400u};
  asm volatile("" : "+v"(m.m0), "+v"(m.m2), "+v"(m.m3), "+v"(m.m4), "+v"(m.m6), "+v"(m.m8));
  return m;
}

// Register-level format of one packed word: it unpacks into RPW registers, register rho holding
// slots (rho, rho + RPW) of the word as two halves; offset(rho) is the additive constant.
template <int BITS>
struct Pack;
template <>
struct Pack<4> {
  static constexpr int CPW = 8, RPW = 4, W = 16;
  __device__ static constexpr float offset(int rho) { return (rho & 1) ? 64.0f : 1024.0f; }
  __device__ static inline void unpack(uint32_t w, uint32_t* r, const Magic& m) {
    const uint32_t t = w >> 8;
    r[0] = (w & 0x000F000Fu) | m.m0;
    r[1] = (w & 0x00F000F0u) | m.m4;
    r[2] = (t & 0x000F000Fu) | m.m0;
    r[3] = (t & 0x00F000F0u) | m.m4;
  }
};
template <>
struct Pack<3> {   // five codes in bits 0-14, five in bits 16-30
  static constexpr int CPW = 10, RPW = 5, W = 13;
  __device__ static constexpr float offset(int rho) { return (rho == 0 || rho == 3) ? 1024.0f : ((rho == 2) ? 16.0f : 128.0f); }
  __device__ static inline void unpack(uint32_t w, uint32_t* r, const Magic& m) {
    const uint32_t t = w >> 9;
    r[0] = (w & 0x00070007u) | m.m0;
    r[1] = (w & 0x00380038u) | m.m3;
    r[2] = (w & 0x01C001C0u) | m.m6;
    r[3] = (t & 0x00070007u) | m.m0;
    r[4] = (t & 0x00380038u) | m.m3;
  }
};
template <>
struct Pack<2> {
  static constexpr int CPW = 16, RPW = 8, W = 8;
  __device__ static constexpr float offset(int rho) {
    return (rho == 0 || rho == 5) ? 1024.0f : ((rho == 1 || rho == 6) ? 256.0f : ((rho == 2 || rho == 7) ? 64.0f : (rho == 3 ? 16.0f : 4.0f)));
  }
  __device__ static inline void unpack(uint32_t w, uint32_t* r, const Magic& m) {
    const uint32_t t = w >> 10;
    r[0] = (w & 0x00030003u) | m.m0;
    r[1] = (w & 0x000C000Cu) | m.m2;
    r[2] = (w & 0x00300030u) | m.m4;
    r[3] = (w & 0x00C000C0u) | m.m6;
    r[4] = (w & 0x03000300u) | m.m8;
    r[5] = (t & 0x00030003u) | m.m0;
    r[6] = (t & 0x000C000Cu) | m.m2;
    r[7] = (t & 0x00300030u) | m.m4;
  }
};

template <>
struct Pack<8> {   // bytes 0 and 2 already sit at mantissa bit 0 of their halves; bytes 1 and 3 after one shift
  static constexpr int CPW = 4, RPW = 2, W = 32;
  __device__ static constexpr float offset(int) { return 1024.0f; }
  __device__ static inline void unpack(uint32_t w, uint32_t* r, const Magic& m) {
    r[0] = (w & 0x00FF00FFu) | m.m0;
    r[1] = ((w >> 8) & 0x00FF00FFu) | m.m0;
  }
};

// Lane group g (= lane / 16) streams word rows g, 4 + g, 8 + g, ... of a tile; its unpacked
// registers, in that order, are cut into operands of 4 registers (8 contraction slots).
template <int BITS>
struct Shape {
  static constexpr int CPW = Pack<BITS>::CPW, RPW = Pack<BITS>::RPW, W = Pack<BITS>::W;
  static constexpr int KW = (W + 3) / 4;            // word rows per lane group (the last may be missing)
  static constexpr int NREG = KW * RPW;             // registers per lane and row: 16, 20, 16, 16
  static constexpr int NOPS = NREG / 4;             // matrix instructions per 16 rows: 4, 5, 4, 4
  static constexpr int TBL = NOPS * 32;             // halves of one operand-table column
  static_assert(NREG % 4 == 0, "operands must be whole");
  // Position in a table column of element e (a channel for Keys, a token of the tile for Values).
  __device__ static inline int table_pos(int e) {
    const int w = e / CPW, j = e % CPW;
    const int lin = (w >> 2) * RPW + (j % RPW);
    return ((lin >> 2) * 4 + (w & 3)) * 8 + 2 * (lin & 3) + j / RPW;
  }
  __device__ static inline float elem_offset(int e) {
    const int rho = (e % CPW) % RPW;
    float f = Pack<BITS>::offset(0);
#pragma unroll
    for (int i = 1; i < RPW; ++i) f = rho == i ? Pack<BITS>::offset(i) : f;
    return f;
  }
};

// Streaming (read-once) 16-byte load: the code stream should not displace anything in the caches.
typedef uint32_t uint4v __attribute__((ext_vector_type(4)));
__device__ inline uint4 load_stream(const uint32_t* src) {
  const uint4v v = __builtin_nontemporal_load(reinterpret_cast<const uint4v*>(src));
  return uint4{v.x, v.y, v.z, v.w};
}

__device__ inline uint32_t word_of(const uint4& v, int r) { return r == 0 ? v.x : (r == 1 ? v.y : (r == 2 ? v.z : v.w)); }

// lane n of each 16-lane row receives the value of lane n + S of the same row (0 past the row end).
template <int S>
__device__ inline float row_shift_down(float v) {
  static_assert(S >= 1 && S <= 15, "row shift");
  return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), 0x100 + S, 0xF, 0xF, true));
}

// A value that is the same in every lane (the result of a wave reduction), moved to a scalar
// register: the per-head running state then costs no vector registers.
__device__ inline float uniform(float v) {
  return __builtin_bit_cast(float, __builtin_amdgcn_readfirstlane(__builtin_bit_cast(int, v)));
}

__device__ inline void wave_lds_sync() {
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
  __builtin_amdgcn_wave_barrier();
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

// Lane n of each 16-lane row receives the value of lane n - S of the same row (0 before the row start).
template <int S>
__device__ inline float row_shift_up(float v) {
  static_assert(S >= 1 && S <= 15, "row shift");
  return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), 0x110 + S, 0xF, 0xF, true));
}
// Exclusive prefix sums over the 256 values of a wave, four consecutive ones per lane (value i sits
// in f[i & 3] of lane i / 4): out[i] = sum of the values before i, out[256] = the total.  Per 16-lane
// row a shift-and-add scan of the lanes' totals, the three row totals read as scalars.
constexpr int kPrefixStride = 260;                 // 257 entries, padded to a multiple of four floats
__device__ inline void wave_prefix_256(const float f[4], float* out, int lane) {
  const float p0 = f[0], p1 = p0 + f[1], p2 = p1 + f[2], p3 = p2 + f[3];
  float v = p3;
  v += row_shift_up<1>(v);
  v += row_shift_up<2>(v);
  v += row_shift_up<4>(v);
  v += row_shift_up<8>(v);
  const int vi = __builtin_bit_cast(int, v);
  const float t0 = __builtin_bit_cast(float, __builtin_amdgcn_readlane(vi, 15));
  const float t1 = __builtin_bit_cast(float, __builtin_amdgcn_readlane(vi, 31));
  const float t2 = __builtin_bit_cast(float, __builtin_amdgcn_readlane(vi, 47));
  const int row = lane >> 4;
  const float rows_before = row == 0 ? 0.0f : (row == 1 ? t0 : (row == 2 ? t0 + t1 : (t0 + t1) + t2));
  const float excl = row_shift_up<1>(v) + rows_before;
  *reinterpret_cast<float4v*>(out + 4 * lane) = float4v{excl, excl + p0, excl + p1, excl + p2};
  if (lane == KVS_WAVE - 1) out[256] = excl + p3;
}

struct MfmaArgs {
  const uint16_t* q;
  const uint32_t* k_codes; const uint32_t* v_codes; const uint32_t* k_params; const uint32_t* v_params;
  const uint8_t* keep_mask;
  const uint16_t* keep_k; const uint16_t* keep_v; const int32_t* keep_cnt;
  uint16_t* out; float* lse; float* ws;
  int* arrive;       // one arrival counter per (b, kv head): zero on entry, zero again on exit
  // dense-and-sparse only: the CSR arrays of the isolated outliers (rows (b, h, token) for Keys,
  // (b, h, tile, channel) for Values - the same row numbering) and their capacity in entries
  const int32_t* k_rowptr; const uint16_t* k_col; const uint16_t* k_val;
  const int32_t* v_rowptr; const uint16_t* v_col; const uint16_t* v_val;
  int sparse_cap;
  int n, Hkv, cap;   // n: tokens per (b, h) the buffers are laid out for
  int n_used;        // tokens to attend to (the first n_used; a multiple of 128)
  const float* extra;   // one more softmax state per (b, hq) to merge (a growing cache's residual rows), or null
  int parts;         // workgroups per (b, h)
  int part_tokens;   // tokens per workgroup
  int rep;           // query heads per KV head (Hq / Hkv)
  int head_off;      // first of them that this launch takes; it takes R
};

// SPARSE (caches with isolated fp16 outliers, Section 5.1): an isolated slot holds code 0, i.e.
// it dequantises to -scale * zero; replacing it by its fp16 value v adds
//     q_c (v + scale zero)   to the score of its token         (Keys,   CSR row = token,   column = channel)
//     w_t (v + scale zero)   to the output channel it sits in  (Values, CSR row = channel of the tile, column = token)
// Both are done here, per chunk.  A chunk is one 128-row tile of either structure, so its entries
// are one contiguous run of the column / value arrays, [rowptr[tile start], rowptr[tile end]): the
// wave reads the run with aligned 8-byte loads (four consecutive entries per lane, 253 or more per
// round; a tile at 1% holds about 164, longer runs take more rounds, on demand), requested at the
// start of the stage before the one that uses them.  Each lane turns its four entries into
// products - Key entries with the chunk's q and scale * zero tables in LDS, Value entries with the
// chunk's softmax weights, which replace the scores in LDS once those have been read; an entry's
// column word names its row inside the tile (bits 7-13), which says which quantisation group's
// scale * zero applies - and the wave leaves the exclusive prefix sums of the 256 products in LDS
// (a shift-and-add scan per 16-lane row, row totals as scalars).  A row's sum is then the
// difference of two prefix sums at the row's own pointers, which travel with the Value parameters:
// the lane that owns the row (lane = tokens lane, lane + 64 in the softmax stage; lane = channels
// lane, lane + 64 after the Value product) reads them, adds the Key sums to its scores and
// keeps the Value sums in two registers per head that follow the accumulators' rescaling.  No
// loop over a row's entries, no scatter, no atomic; every load is aligned and coalesced.
// (Measured against it on 32 x 32 heads x 4096 tokens at 1%: each lane gathering its own row's
// entries, 8 bytes at 2-byte alignment, +11%; LDS float atomics +35%; a staging row in LDS walked by
// the rows' owners +26%.)  Every index read from the cache is clamped (positions to the run, the run
// to the arrays and to the 16384 entries a tile can hold, rows and columns to 7 bits), so a cache
// with garbage in its CSR arrays yields garbage, not a fault.
//
// KPT (per-token Keys, the other Key scheme of the paper's Section 5.1): a Key row carries one
// parameter pair per group of G channels, like a Value row.  The scale then depends on the token
// - the M row of the score product - and cannot be folded into the query; instead the B operand
// is the bare query, cut into one pair of (hi, lo) columns per channel group, built once per
// workgroup, and the softmax stage combines the per-group sums with the token's parameters:
//   score[t] = sum_g scale[t, g] (raw_g[t] - C_g - zero[t, g] Q_g),
// C_g = what the product holds for the operand offsets, Q_g = the query's sum over the group.
template <int BITS, int G, int R, bool SPARSE, bool KPT = false>
__global__ __launch_bounds__(waves_for(BITS, G, R, KPT, SPARSE) * KVS_WAVE) void decode_mfma_kernel(MfmaArgs a) {
  static_assert(!(KPT && SPARSE), "per-token Keys are dense only");
  constexpr int kWaves = waves_for(BITS, G, R, KPT, SPARSE);
  constexpr int HPW = (R + kWaves - 1) / kWaves;   // heads whose states one wave merges at the end
  using S = Shape<BITS>;
  constexpr int W = S::W, KW = S::KW, RPW = S::RPW, NOPS = S::NOPS, TBL = S::TBL;
  constexpr int NGK = 128 / G;                     // Key token groups per chunk
  constexpr int NGT = G < 64 ? 2 : 1;              // Key token groups per 64-token tile
  constexpr int NGC = 128 / G;                     // Value channel groups
  constexpr int NTAB = G == 128 ? 1 : 2;           // Value operand tables (one per channel half)
  constexpr int KCOLS = KPT ? 2 * R * NGC : 2 * R * NGT;   // [hi | lo] per token group of the tile (KPT: per channel group)
  constexpr int NSC = KPT ? R * NGC : R;           // score rows a chunk leaves in LDS
  constexpr int KTABS = KPT ? 1 : kWaves;          // KPT: one table for the workgroup, built by wave 0
  constexpr int VCOLS = G == 32 ? 4 * R : 2 * R;   // [hi | lo] per channel group of the half
  static_assert(KCOLS <= 16 && VCOLS <= 16, "tile columns");
  constexpr int LOG2G = G == 32 ? 5 : (G == 64 ? 6 : 7);

  // Per-wave LDS: operand tables in the instruction's slot order (column *COLS stays zero: the
  // lanes of the unused tile columns read it, and so do padded slots), and the score exchange.
  __shared__ __align__(16) _Float16 bq[KTABS][KCOLS + 1][TBL];           // query x Key scale (KPT: the query)
  __shared__ __align__(16) float sc[kWaves][NSC][128];                   // scores, token order
  __shared__ __align__(16) _Float16 wh[kWaves][NTAB][VCOLS + 1][TBL];    // weight x Value scale
  // At the end each wave leaves its unnormalised output rows (R x 128 floats) in its own table.
  static_assert(sizeof(wh[0]) >= R * 128 * sizeof(float), "output rows must fit the weight table");
  auto part_o = [&](int w, int r) -> float* { return reinterpret_cast<float*>(&wh[w][0][0][0]) + r * 128; };
  __shared__ float part_m[2 * kWaves][R], part_l[2 * kWaves][R];         // [kWaves + w]: wave w's kept rows
  __shared__ int next_chunk;                                             // chunk hand-out counter
  // SPARSE: the query (log2 units) by channel; scale x zero of the chunk's Key groups by channel
  // and of its Value groups by token
  __shared__ __align__(16) float qtab[SPARSE ? R : 1][SPARSE ? 128 : 1];
  __shared__ __align__(16) float sz_k[SPARSE ? kWaves : 1][SPARSE ? NGK : 1][SPARSE ? 128 : 1];
  __shared__ __align__(16) float sz_v[SPARSE ? kWaves : 1][SPARSE ? NGC : 1][SPARSE ? 128 : 1];
  // SPARSE: exclusive prefix sums of one round's 256 products, per head (0 .. 256)
  __shared__ __align__(16) float psum[SPARSE ? kWaves : 1][SPARSE ? R : 1][SPARSE ? kPrefixStride : 4];
  __shared__ int arrived_last;                                           // this workgroup completes its (b, h)

  const int lane = threadIdx.x & (KVS_WAVE - 1), wave = threadIdx.x / KVS_WAVE;
  const int col = lane & 15, grp = lane >> 4;
  const Magic magic = make_magic();
  const int kcol = col < KCOLS ? col : KCOLS;      // table columns this lane's tile column reads
  const int vcol = col < VCOLS ? col : VCOLS;
  const int n = a.n;
  const size_t bh = blockIdx.x / a.parts;
  const int part = blockIdx.x % a.parts;
  const int b = static_cast<int>(bh / a.Hkv), h = static_cast<int>(bh % a.Hkv);
  const int Hq = a.Hkv * a.rep;
  const int hq0 = h * a.rep + a.head_off;        // the launch's R heads of KV head h
  const int keep_cnt_b = a.keep_cnt[b];            // uniform: a scalar load, issued first
  // The wave's first kept row (rows past the count are zero padding), requested before the
  // stream starts so that it has long arrived when it is needed.
  const uint32_t* keep_rows_k = reinterpret_cast<const uint32_t*>(a.keep_k) + bh * a.cap * 64 + lane;
  const uint32_t* keep_rows_v = reinterpret_cast<const uint32_t*>(a.keep_v) + bh * a.cap * 64 + lane;
  uint32_t keep_first_k = 0, keep_first_v = 0;
  // The finishing wave of head r also requests the extra state now, if there is one.
  float2 extra_o[HPW];
  float extra_m[HPW], extra_l[HPW];
#pragma unroll
  for (int k = 0; k < HPW; ++k) {
    extra_o[k] = float2{0.0f, 0.0f};  extra_m[k] = -INFINITY;  extra_l[k] = 0.0f;
    const int r = wave + k * kWaves;
    if (a.extra && a.parts == 1 && r < R) {
      const float* x = a.extra + (static_cast<size_t>(b) * Hq + hq0 + r) * kWsRow;
      extra_o[k] = reinterpret_cast<const float2*>(x)[lane];
      extra_m[k] = x[128];
      extra_l[k] = x[129];
    }
  }
  if (a.parts == 1 && wave < a.cap) {
    keep_first_k = keep_rows_k[wave * 64];
    keep_first_v = keep_rows_v[wave * 64];
  }

  const int part_begin = min(a.n_used, part * a.part_tokens);
  const int part_end = min(a.n_used, part_begin + a.part_tokens);
  const int nchunks = (part_end - part_begin) / 128;       // chunks of this workgroup
  const uint8_t* mask_b = a.keep_mask + static_cast<size_t>(b) * n;
  const uint32_t* kcodes = a.k_codes + bh * (n / 64) * (W * 64);
  const uint32_t* vcodes = a.v_codes + bh * (n / 128) * (W * 128);
  const uint32_t* kparams = a.k_params + bh * (n / G) * 128;     // KPT: bh * n * NGC, the same number
  const uint32_t* vparams = a.v_params + bh * n * NGC;

  float m_run[R], l_run[R], z_run[R][NGC];         // running max (log2 units), lane-partial sums
  float4v acc[2][4];                               // [channel half][r]: rows = channels 64 half + 16 grp + 4 i + r
#pragma unroll
  for (int r = 0; r < R; ++r) {
    m_run[r] = -INFINITY; l_run[r] = 0.0f;
#pragma unroll
    for (int g = 0; g < NGC; ++g) z_run[r][g] = 0.0f;
  }
#pragma unroll
  for (int hf = 0; hf < 2; ++hf)
#pragma unroll
    for (int r = 0; r < 4; ++r) acc[hf][r] = float4v{0.0f, 0.0f, 0.0f, 0.0f};

  // The entries of one tile as the cache gives them, made safe: 0 <= begin <= end <= capacity and
  // at most 16384 entries (128 rows of 128 columns).  Wave-uniform.
  struct TileRun { int begin, end; };
  auto tile_run = [&](int lo, int hi) -> TileRun {
    const int b0 = __builtin_amdgcn_readfirstlane(max(0, min(lo, a.sparse_cap)));
    const int e0 = __builtin_amdgcn_readfirstlane(min(max(min(hi, a.sparse_cap), b0), b0 + 128 * 128));
    return TileRun{b0, e0};
  };
  // Round k of a run: lane l takes the four entries from (begin & ~3) + 256 k + 4 l on, one aligned
  // 8-byte load per array (the arrays hold four entries more than the capacity, so the last
  // aligned group can be read whole); the entries outside [begin, end) are there and not used.
  auto entry_pos = [&](const TileRun& run, int k) -> int { return (run.begin & ~3) + 256 * k + 4 * lane; };
  auto load_entries = [&](const uint16_t* arr, int pos) -> uint64_t {
    return *reinterpret_cast<const uint64_t*>(arr + min(pos, a.sparse_cap & ~3));
  };
  auto entry_of = [](uint64_t four, int j) -> uint32_t { return static_cast<uint32_t>(four >> (16 * j)) & 0xFFFFu; };
  // The rows lane and lane + 64 of a tile, from their pointers (rp[0], rp[1]) and the pointer behind
  // the tile's last row (rp[2]): [lo, hi) of each, clamped into the run.
  struct RowPair { int lo[2], hi[2]; };
  auto rows_of = [&](int rp0, int rp1, int rp_end, const TileRun& run) __attribute__((always_inline)) -> RowPair {
    const int first_hi = __builtin_amdgcn_readfirstlane(rp1);          // row 64 starts where row 63 ends
    const int nxt0 = __shfl_down(rp0, 1, KVS_WAVE), nxt1 = __shfl_down(rp1, 1, KVS_WAVE);
    const int end0 = lane == KVS_WAVE - 1 ? first_hi : nxt0, end1 = lane == KVS_WAVE - 1 ? rp_end : nxt1;
    RowPair p;
    p.lo[0] = min(max(rp0, run.begin), run.end);  p.hi[0] = min(max(end0, p.lo[0]), run.end);
    p.lo[1] = min(max(rp1, run.begin), run.end);  p.hi[1] = min(max(end1, p.lo[1]), run.end);
    return p;
  };
  // The stream of one chunk lives in registers, and every piece of it (a 64-token Key tile, the
  // parameters, a 64-channel half of the Value tile) is requested again - for the wave's next
  // chunk - as soon as its last use is over, so that about one chunk per wave is always in
  // flight.  A wave takes its next chunk from the workgroup's counter when it starts one: waves
  // that the memory system serves late end up with fewer chunks, and all of them stream until
  // the workgroup's range is used up.  Past the last chunk the same loads are still issued
  // (every path issues the same number of loads, which keeps the waits exact) but every lane
  // then reads the head of the range: a few cache lines.
  struct KeyRegs {
    uint4 kx[2][KW];       // [64-token tile][word row 4 k + grp], tokens 4 col .. 4 col + 3
    uint2 kp[NGK];         // parameters of channels 2 lane, 2 lane + 1, per token group
  };
  struct ValueRegs {
    uint4 vx[KW][2];       // [token word row 4 k + grp][channel half], channels 4 col .. + 3
    uint32_t vp0[NGC], vp1[NGC];   // parameters of tokens lane, lane + 64
    uint32_t kq0[KPT ? NGC : 1], kq1[KPT ? NGC : 1];   // KPT: Key parameters of the same tokens
    int krp[SPARSE ? 3 : 1], vrp[SPARSE ? 3 : 1];   // CSR row pointers of rows lane, lane + 64 and of the row behind the tile's last
    uint8_t mask0, mask1;  // keep-mask bytes of the same tokens
  };
  KeyRegs keys;
  ValueRegs vals;
  // SPARSE: the current chunk's runs of both CSR structures, the first round of their entries, the
  // lane's Value rows, and the Value corrections so far (same scale as the accumulators).
  TileRun krun = {0, 0}, vrun = {0, 0};
  uint64_t kcol0 = 0, kval0 = 0, vcol0 = 0, vval0 = 0;
  RowPair vrows = {{0, 0}, {0, 0}};
  float vcorr[R][2];
#pragma unroll
  for (int r = 0; r < R; ++r) { vcorr[r][0] = 0.0f; vcorr[r][1] = 0.0f; }
  auto take_chunk = [&]() -> int {
    int c = 0;
    if (lane == 0) c = atomicAdd(&next_chunk, 1);
    return __builtin_amdgcn_readfirstlane(c);
  };
  // Loaders, one piece at a time so that a piece can be requested again the moment it has been
  // consumed.  A chunk index past the end (wave-uniform) turns the piece into a few cache lines.
  auto load_key_tile = [&](KeyRegs& s, int ci, int kt) {        // 64 tokens x W words
    const bool real = ci < nchunks;
    const int t0 = real ? part_begin + ci * 128 : 0;
    const int lane_words = real ? grp * 64 + 4 * col : 0;
    const uint32_t* ktile = kcodes + static_cast<size_t>(t0 / 64 + kt) * (W * 64) + lane_words;
#pragma unroll
    for (int k = 0; k < KW; ++k) {
      s.kx[kt][k] = uint4{0, 0, 0, 0};
      if (4 * k + 3 < W || 4 * k + grp < W)        // only the last word row of a 13-row tile can be missing
        s.kx[kt][k] = load_stream(ktile + 4 * k * 64);
    }
  };
  auto load_key_params = [&](KeyRegs& s, int ci, int kt) {      // the token groups that tile kt uses first
    const bool real = ci < nchunks;
    const int t0 = real ? part_begin + ci * 128 : 0;
    const int lane_pair = real ? lane : 0;
    if (KPT || (G == 128 && kt == 1)) return;
#pragma unroll
    for (int ga = 0; ga < NGT; ++ga) {
      const int g = G == 128 ? 0 : kt * NGT + ga;
      s.kp[g] = reinterpret_cast<const uint2*>(kparams + static_cast<size_t>(t0 / G + g) * 128)[lane_pair];
    }
  };
  auto load_value_params = [&](ValueRegs& s, int ci) {
    const bool real = ci < nchunks;
    const int t0 = real ? part_begin + ci * 128 : 0;
    const int lane_tok = real ? lane : 0;
#pragma unroll
    for (int g = 0; g < NGC; ++g) {
      s.vp0[g] = vparams[static_cast<size_t>(t0 + lane_tok) * NGC + g];
      s.vp1[g] = vparams[static_cast<size_t>(t0 + 64 + lane_tok) * NGC + g];
      if (KPT) {
        s.kq0[g] = kparams[static_cast<size_t>(t0 + lane_tok) * NGC + g];
        s.kq1[g] = kparams[static_cast<size_t>(t0 + 64 + lane_tok) * NGC + g];
      }
    }
    s.mask0 = mask_b[t0 + lane_tok];
    s.mask1 = mask_b[t0 + 64 + lane_tok];
    if (SPARSE) {                                  // Key rows are tokens, Value rows the channels of the tile:
      const size_t row = bh * n + t0;              // the same numbers
      s.krp[0] = a.k_rowptr[row + lane_tok];  s.krp[1] = a.k_rowptr[row + 64 + lane_tok];  s.krp[2] = a.k_rowptr[row + 128];
      s.vrp[0] = a.v_rowptr[row + lane_tok];  s.vrp[1] = a.v_rowptr[row + 64 + lane_tok];  s.vrp[2] = a.v_rowptr[row + 128];
    }
  };
  auto load_value_half = [&](ValueRegs& s, int ci, int hf) {    // 128 tokens x 64 channels
    const bool real = ci < nchunks;
    const int t0 = real ? part_begin + ci * 128 : 0;
    const int lane_words = real ? grp * 128 + 4 * col : 0;
    const uint32_t* vtile = vcodes + static_cast<size_t>(t0 / 128) * (W * 128) + lane_words + 64 * hf;
#pragma unroll
    for (int k = 0; k < KW; ++k) {
      s.vx[k][hf] = uint4{0, 0, 0, 0};
      if (4 * k + 3 < W || 4 * k + grp < W)
        s.vx[k][hf] = load_stream(vtile + 4 * k * 128);
    }
  };
  auto load_keys = [&](KeyRegs& s, int ci) {
    load_key_tile(s, ci, 0);  load_key_params(s, ci, 0);     // the order in which they are requested again
    load_key_tile(s, ci, 1);  load_key_params(s, ci, 1);
  };
  auto load_values = [&](ValueRegs& s, int ci) {
    load_value_params(s, ci);
    load_value_half(s, ci, 0);  load_value_half(s, ci, 1);
  };
  // The wave's first chunk is its own index: request it before anything else is set up.
  if (wave < nchunks) {
    load_keys(keys, wave);
    load_values(vals, wave);
  }
  if (threadIdx.x == 0) next_chunk = kWaves;               // chunks 0 .. kWaves - 1 are the waves' first
  {
    if (!KPT || wave == 0) {
      uint32_t* zq = reinterpret_cast<uint32_t*>(&bq[KPT ? 0 : wave][0][0]);
      for (int i = lane; i < (KCOLS + 1) * TBL / 2; i += KVS_WAVE) zq[i] = 0;
    }
    uint32_t* zw = reinterpret_cast<uint32_t*>(&wh[wave][0][0][0]);
    for (int i = lane; i < NTAB * (VCOLS + 1) * TBL / 2; i += KVS_WAVE) zw[i] = 0;
  }
  // Query of the lane's two channels (2 lane, 2 lane + 1), all R heads, scaled to log2 units;
  // where those channels and the lane's two tokens (lane, lane + 64) sit in a table column.
  float qf[R][2];
#pragma unroll
  for (int r = 0; r < R; ++r) {
    const uint32_t two = reinterpret_cast<const uint32_t*>(a.q + (static_cast<size_t>(b) * Hq + hq0 + r) * 128)[lane];
    qf[r][0] = kvs::half_bits_to_float(static_cast<uint16_t>(two & 0xFFFFu)) * kLog2eRsqrtD;
    qf[r][1] = kvs::half_bits_to_float(static_cast<uint16_t>(two >> 16)) * kLog2eRsqrtD;
  }
  if (SPARSE && wave == 0) {
#pragma unroll
    for (int r = 0; r < R; ++r) reinterpret_cast<float2*>(&qtab[r][0])[lane] = float2{qf[r][0], qf[r][1]};
  }
  const int cpos0 = S::table_pos(2 * lane), cpos1 = S::table_pos(2 * lane + 1);
  const float coff0 = S::elem_offset(2 * lane), coff1 = S::elem_offset(2 * lane + 1);
  const int tpos0 = S::table_pos(lane), tpos1 = S::table_pos(lane + 64);
  const float toff0 = S::elem_offset(lane), toff1 = S::elem_offset(lane + 64);

  // KPT: the score product's B operand is the query alone, in the columns of the lane's channel
  // group; kc / kqs are what the product holds for the operand offsets, and the query's sum.
  float kc[KPT ? NGC : 1][R], kqs[KPT ? NGC : 1][R];
  if (KPT) {
    const int gk = (2 * lane) >> LOG2G;                    // channel group of the lane's two channels
    if (wave == 0) wave_lds_sync();                        // the table is zeroed
#pragma unroll
    for (int r = 0; r < R; ++r) {
      const _Float16 h0 = static_cast<_Float16>(qf[r][0]), h1 = static_cast<_Float16>(qf[r][1]);
      const _Float16 e0 = static_cast<_Float16>(qf[r][0] - static_cast<float>(h0));
      const _Float16 e1 = static_cast<_Float16>(qf[r][1] - static_cast<float>(h1));
      if (wave == 0) {
        bq[0][gk * 2 * R + r][cpos0] = h0;  bq[0][gk * 2 * R + r][cpos1] = h1;
        bq[0][gk * 2 * R + R + r][cpos0] = e0;  bq[0][gk * 2 * R + R + r][cpos1] = e1;
      }
      const float q0 = static_cast<float>(h0) + static_cast<float>(e0), q1 = static_cast<float>(h1) + static_cast<float>(e1);
#pragma unroll
      for (int g = 0; g < NGC; ++g) {
        kc[g][r] = uniform(kvs::wave_sum(gk == g ? q0 * coff0 + q1 * coff1 : 0.0f));
        kqs[g][r] = uniform(kvs::wave_sum(gk == g ? q0 + q1 : 0.0f));
      }
    }
  }

  __syncthreads();                                         // the chunk counter (and the KPT table) is set

  half8 bq_fixed[NOPS];                            // KPT: the B operand never changes
  if (KPT) {
#pragma unroll
    for (int m = 0; m < NOPS; ++m) bq_fixed[m] = *reinterpret_cast<const half8*>(&bq[0][kcol][(4 * m + grp) * 8]);
  }

  float bias[NGK][R];                              // what the score product holds for offsets and zero points

  auto score_chunk = [&](KeyRegs& s, int refill) {
    if (SPARSE) {
      // The chunk's isolated entries, Keys for the softmax stage and Values for after the Value
      // product, are requested now: loads return in order, and behind this stage's refills they
      // would make their readers wait for the next chunk's stream as well.
      krun = tile_run(vals.krp[0], vals.krp[2]);       // lane 0 holds the tile's first row
      vrun = tile_run(vals.vrp[0], vals.vrp[2]);
      kcol0 = load_entries(a.k_col, entry_pos(krun, 0));
      kval0 = load_entries(a.k_val, entry_pos(krun, 0));
      vcol0 = load_entries(a.v_col, entry_pos(vrun, 0));
      vval0 = load_entries(a.v_val, entry_pos(vrun, 0));
    }
#pragma unroll
    for (int kt = 0; kt < 2; ++kt) {
      // ---- (1) B operand of the score product: q x scale as hi + lo halves, per token group ----
      if (!KPT && (G < 128 || kt == 0)) {
#pragma unroll
        for (int ga = 0; ga < NGT; ++ga) {
          const int gi = G == 128 ? 0 : kt * NGT + ga;       // group inside the chunk
          float s0, s1; int z0, z1;
          kvs::unpack_param(s.kp[gi].x, s0, z0);
          kvs::unpack_param(s.kp[gi].y, s1, z1);
          const float zf0 = static_cast<float>(z0) + coff0, zf1 = static_cast<float>(z1) + coff1;
          if (SPARSE)
            reinterpret_cast<float2*>(&sz_k[wave][gi][0])[lane] = float2{s0 * static_cast<float>(z0), s1 * static_cast<float>(z1)};
#pragma unroll
          for (int r = 0; r < R; ++r) {
            const float a0 = qf[r][0] * s0, a1 = qf[r][1] * s1;
            const _Float16 h0 = static_cast<_Float16>(a0), h1 = static_cast<_Float16>(a1);
            const _Float16 e0 = static_cast<_Float16>(a0 - static_cast<float>(h0));
            const _Float16 e1 = static_cast<_Float16>(a1 - static_cast<float>(h1));
            bq[wave][ga * 2 * R + r][cpos0] = h0;  bq[wave][ga * 2 * R + r][cpos1] = h1;
            bq[wave][ga * 2 * R + R + r][cpos0] = e0;  bq[wave][ga * 2 * R + R + r][cpos1] = e1;
            // offsets and zero points exactly as the rounded operands will multiply them
            bias[gi][r] = uniform(kvs::wave_sum((static_cast<float>(h0) + static_cast<float>(e0)) * zf0 +
                                                (static_cast<float>(h1) + static_cast<float>(e1)) * zf1));
          }
        }
        wave_lds_sync();
      }
      half8 bqr[NOPS];
#pragma unroll
      for (int m = 0; m < NOPS; ++m)
        bqr[m] = KPT ? bq_fixed[m] : *reinterpret_cast<const half8*>(&bq[KPT ? 0 : wave][kcol][(4 * m + grp) * 8]);

      // ---- (2) scores on the matrix cores; hi + lo columns merged; to LDS in token order -------
      float4v d[4];                                    // [r]: rows = tokens 64 kt + 4 m + r, m = 0..15
#pragma unroll
      for (int r = 0; r < 4; ++r) {
        d[r] = float4v{0.0f, 0.0f, 0.0f, 0.0f};
        uint32_t regs[S::NREG];
#pragma unroll
        for (int k = 0; k < KW; ++k) Pack<BITS>::unpack(word_of(s.kx[kt][k], r), regs + k * RPW, magic);
#pragma unroll
        for (int m = 0; m < NOPS; ++m) {
          const uint32_t op[4] = {regs[4 * m], regs[4 * m + 1], regs[4 * m + 2], regs[4 * m + 3]};
          d[r] = __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(half8, op), bqr[m], d[r], 0, 0, 0);
        }
        if (R > 1) __builtin_amdgcn_sched_barrier(0);   // keep one row set's operands live at a time
      }
      float4v out[4];                                  // [i]: tokens 64 kt + 16 grp + 4 i + (0..3)
#pragma unroll
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int r = 0; r < 4; ++r) {
          float v = d[r][i] + row_shift_down<R>(d[r][i]);            // hi + lo
          if (!KPT && NGT == 2) {                                    // rows of lane groups 2, 3 belong to the
            const float w2 = row_shift_down<(2 * R) % 16 == 0 ? 1 : (2 * R) % 16>(v);   // tile's second token group
            v = grp >= 2 ? w2 : v;
          }
          out[i][r] = v;
        }
      __builtin_amdgcn_sched_barrier(0);               // keeps the loads below the tile's last use
      load_key_tile(s, refill, kt);
      load_key_params(s, refill, kt);
      __builtin_amdgcn_sched_barrier(0);
      if (KPT) {                                       // column g 2R + r: head r, channel group g
        if (col < KCOLS && (col % (2 * R)) < R) {
          const int slot = (col / (2 * R)) * R + col % (2 * R);
#pragma unroll
          for (int i = 0; i < 4; ++i)
            *reinterpret_cast<float4v*>(&sc[wave][slot][64 * kt + 16 * grp + 4 * i]) = out[i];
        }
      } else if (col < R) {
#pragma unroll
        for (int i = 0; i < 4; ++i)
          *reinterpret_cast<float4v*>(&sc[wave][col][64 * kt + 16 * grp + 4 * i]) = out[i];
      }
      if (!KPT && G < 128 && kt == 0) wave_lds_sync(); // the table is rebuilt for the second tile
    }
    wave_lds_sync();
  };

  auto value_chunk = [&](ValueRegs& s, int refill, int cur, bool settle) {
    // ---- (3) online softmax, lane = tokens (lane, lane + 64); weights x Value scale to LDS -----
    float alpha[R];
    float kcorr[R][2];                                 // SPARSE: what the isolated Key entries add to the scores
#pragma unroll
    for (int r = 0; r < R; ++r) { kcorr[r][0] = 0.0f; kcorr[r][1] = 0.0f; }
    if (SPARSE) {
      // The lane's Value rows are worked out now (their pointers are about to be loaded again) ...
      vrows = rows_of(s.vrp[0], s.vrp[1], s.vrp[2], vrun);
      // ... and the Key entries of tokens lane, lane + 64: entry (channel c, value v) adds
      // q_c (v + scale zero) to the token's score, for every head.
      const RowPair krows = rows_of(s.krp[0], s.krp[1], s.krp[2], krun);
      for (int k = 0; ; ++k) {                           // rounds: wave-uniform, one unless the tile holds more than ~253 entries
        const int wbeg = (krun.begin & ~3) + 256 * k;    // the round's window of positions: [wbeg, wbeg + 256)
        const uint64_t cols = k == 0 ? kcol0 : load_entries(a.k_col, entry_pos(krun, k));
        const uint64_t vals4 = k == 0 ? kval0 : load_entries(a.k_val, entry_pos(krun, k));
        float f[R][4];                                   // the lane's four entries: what each adds to its token's score
#pragma unroll
        for (int j = 0; j < 4; ++j) {
          const uint32_t e = entry_of(cols, j);
          const int c = e & 127, t = (e >> 7) & 127;     // channel; the row's token inside the tile
          const int pos = wbeg + 4 * lane + j;
          const bool live = pos >= krun.begin && pos < krun.end;
          const int gi = G == 128 ? 0 : t / G;           // the token's Key group in the chunk
          const float base = kvs::half_bits_to_float(static_cast<uint16_t>(entry_of(vals4, j))) + sz_k[wave][gi][c];
#pragma unroll
          for (int r = 0; r < R; ++r) f[r][j] = live ? qtab[r][c] * base : 0.0f;
        }
        if (k > 0) wave_lds_sync();                      // the last round's sums have been read
#pragma unroll
        for (int r = 0; r < R; ++r) wave_prefix_256(f[r], &psum[wave][r][0], lane);
        wave_lds_sync();
#pragma unroll
        for (int h = 0; h < 2; ++h) {                    // the row's part inside the window, as a difference of prefix sums
          const int lo = min(max(krows.lo[h], wbeg), wbeg + 256) - wbeg;
          const int hi = min(max(krows.hi[h], wbeg), wbeg + 256) - wbeg;
#pragma unroll
          for (int r = 0; r < R; ++r) kcorr[r][h] += psum[wave][r][hi] - psum[wave][r][lo];
        }
        if (wbeg + 256 >= krun.end) break;
      }
    }
    {
      float sv0[NGC], sv1[NGC], zf0[NGC], zf1[NGC];
      float sk0[KPT ? NGC : 1], sk1[KPT ? NGC : 1], zk0[KPT ? NGC : 1], zk1[KPT ? NGC : 1];
#pragma unroll
      for (int g = 0; g < NGC; ++g) {
        int z0, z1;
        kvs::unpack_param(s.vp0[g], sv0[g], z0);
        kvs::unpack_param(s.vp1[g], sv1[g], z1);
        zf0[g] = static_cast<float>(z0) + toff0;
        zf1[g] = static_cast<float>(z1) + toff1;
        if (SPARSE) { sz_v[wave][g][lane] = sv0[g] * static_cast<float>(z0); sz_v[wave][g][64 + lane] = sv1[g] * static_cast<float>(z1); }
        // Convert here and now: the parameter registers are about to be loaded again, and a
        // conversion postponed past that load would keep them alive in a second set.
        asm volatile("" : "+v"(sv0[g]), "+v"(sv1[g]), "+v"(zf0[g]), "+v"(zf1[g]));
        if (KPT) {
          kvs::unpack_param(s.kq0[g], sk0[g], z0);
          kvs::unpack_param(s.kq1[g], sk1[g], z1);
          zk0[g] = static_cast<float>(z0);
          zk1[g] = static_cast<float>(z1);
          asm volatile("" : "+v"(sk0[g]), "+v"(sk1[g]), "+v"(zk0[g]), "+v"(zk1[g]));
        }
      }
#pragma unroll
      for (int r = 0; r < R; ++r) {
        float s0, s1;
        if (KPT) {
          s0 = 0.0f;  s1 = 0.0f;
#pragma unroll
          for (int g = 0; g < NGC; ++g) {
            s0 += sk0[g] * (sc[wave][g * R + r][lane] - kc[g][r] - zk0[g] * kqs[g][r]);
            s1 += sk1[g] * (sc[wave][g * R + r][64 + lane] - kc[g][r] - zk1[g] * kqs[g][r]);
          }
          s0 = s.mask0 ? -INFINITY : s0;
          s1 = s.mask1 ? -INFINITY : s1;
        } else {
          // token lane is in Key group lane / G of the chunk, token lane + 64 in group (lane + 64) / G
          float b0 = bias[0][r], b1 = bias[NGK - 1][r];
          if (NGK == 2) { b0 = bias[0][r]; b1 = bias[1][r]; }
          if (NGK == 4) { b0 = lane >= 32 ? bias[1][r] : bias[0][r]; b1 = lane >= 32 ? bias[3][r] : bias[2][r]; }
          s0 = s.mask0 ? -INFINITY : sc[wave][r][lane] - b0;
          s1 = s.mask1 ? -INFINITY : sc[wave][r][64 + lane] - b1;
        }
        if (SPARSE) { s0 += kcorr[r][0];  s1 += kcorr[r][1]; }
        const float mx = uniform(kvs::wave_max(fmaxf(s0, s1)));
        const float m_new = fmaxf(m_run[r], mx);
        const float m_use = m_new == -INFINITY ? 0.0f : m_new;
        alpha[r] = __builtin_amdgcn_exp2f(m_run[r] - m_use);
        const float e0 = __builtin_amdgcn_exp2f(s0 - m_use), e1 = __builtin_amdgcn_exp2f(s1 - m_use);
        m_run[r] = m_new;
        l_run[r] = l_run[r] * alpha[r] + (e0 + e1);
        if (SPARSE) { sc[wave][r][lane] = e0;  sc[wave][r][64 + lane] = e1; }   // the weights take the scores' place
#pragma unroll
        for (int g = 0; g < NGC; ++g) {
          const float w0 = e0 * sv0[g], w1 = e1 * sv1[g];
          const _Float16 h0 = static_cast<_Float16>(w0), h1 = static_cast<_Float16>(w1);
          const _Float16 g0 = static_cast<_Float16>(w0 - static_cast<float>(h0));
          const _Float16 g1 = static_cast<_Float16>(w1 - static_cast<float>(h1));
          const int tab = G == 128 ? 0 : (G == 64 ? g : g >> 1);
          const int cb = G == 32 ? (g & 1) * 2 * R : 0;
          wh[wave][tab][cb + r][tpos0] = h0;  wh[wave][tab][cb + r][tpos1] = h1;
          wh[wave][tab][cb + R + r][tpos0] = g0;  wh[wave][tab][cb + R + r][tpos1] = g1;
          z_run[r][g] = z_run[r][g] * alpha[r] + (static_cast<float>(h0) + static_cast<float>(g0)) * zf0[g] +
                        (static_cast<float>(h1) + static_cast<float>(g1)) * zf1[g];
        }
      }
    }
    __builtin_amdgcn_sched_barrier(0);
    load_value_params(s, refill);
    __builtin_amdgcn_sched_barrier(0);
    wave_lds_sync();

    // ---- (4) rescale the accumulators if a running max moved, then the Value product -----------
    {
      bool moved = false;
#pragma unroll
      for (int r = 0; r < R; ++r) moved = moved || alpha[r] != 1.0f;     // wave-uniform
      if (moved) {
        float f = 1.0f;
#pragma unroll
        for (int r = 0; r < R; ++r) f = (col % R) == r ? alpha[r] : f;
#pragma unroll
        for (int hf = 0; hf < 2; ++hf)
#pragma unroll
          for (int r = 0; r < 4; ++r) acc[hf][r] *= f;
      }
    }
    half8 bwr[NOPS];
#pragma unroll
    for (int hf = 0; hf < 2; ++hf) {
      if (NTAB == 2 || hf == 0) {
#pragma unroll
        for (int m = 0; m < NOPS; ++m)
          bwr[m] = *reinterpret_cast<const half8*>(&wh[wave][NTAB == 2 ? hf : 0][vcol][(4 * m + grp) * 8]);
      }
#pragma unroll
      for (int r = 0; r < 4; ++r) {
        uint32_t regs[S::NREG];
#pragma unroll
        for (int k = 0; k < KW; ++k) Pack<BITS>::unpack(word_of(s.vx[k][hf], r), regs + k * RPW, magic);
#pragma unroll
        for (int m = 0; m < NOPS; ++m) {
          const uint32_t op[4] = {regs[4 * m], regs[4 * m + 1], regs[4 * m + 2], regs[4 * m + 3]};
          acc[hf][r] = __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(half8, op), bwr[m], acc[hf][r], 0, 0, 0);
        }
        if (R > 1) __builtin_amdgcn_sched_barrier(0);
      }
      __builtin_amdgcn_sched_barrier(0);
      load_value_half(s, refill, hf);
      __builtin_amdgcn_sched_barrier(0);
    }
    if (SPARSE) {
      // ---- the chunk's isolated Value entries: lane = channels lane, lane + 64 of the tile -------
      // out[c] += sum over the row's entries (token t, value v) of  weight[t] (v + scale[t] zero[t]);
      // what earlier chunks added follows the accumulators' rescaling first.
#pragma unroll
      for (int r = 0; r < R; ++r) { vcorr[r][0] *= alpha[r];  vcorr[r][1] *= alpha[r]; }
      for (int k = 0; ; ++k) {                           // rounds, as for the Keys
        const int wbeg = (vrun.begin & ~3) + 256 * k;
        const uint64_t cols = k == 0 ? vcol0 : load_entries(a.v_col, entry_pos(vrun, k));
        const uint64_t vals4 = k == 0 ? vval0 : load_entries(a.v_val, entry_pos(vrun, k));
        float f[R][4];
#pragma unroll
        for (int j = 0; j < 4; ++j) {
          const uint32_t e = entry_of(cols, j);
          const int t = e & 127, c = (e >> 7) & 127;     // token inside the tile; the row's channel
          const int pos = wbeg + 4 * lane + j;
          const bool live = pos >= vrun.begin && pos < vrun.end;
          const int gc = G == 128 ? 0 : c / G;           // the channel's Value group
          const float base = kvs::half_bits_to_float(static_cast<uint16_t>(entry_of(vals4, j))) + sz_v[wave][gc][t];
#pragma unroll
          for (int r = 0; r < R; ++r) f[r][j] = live ? sc[wave][r][t] * base : 0.0f;
        }
        wave_lds_sync();                                 // the sums' last reader is done
#pragma unroll
        for (int r = 0; r < R; ++r) wave_prefix_256(f[r], &psum[wave][r][0], lane);
        wave_lds_sync();
#pragma unroll
        for (int h = 0; h < 2; ++h) {
          const int lo = min(max(vrows.lo[h], wbeg), wbeg + 256) - wbeg;
          const int hi = min(max(vrows.hi[h], wbeg), wbeg + 256) - wbeg;
#pragma unroll
          for (int r = 0; r < R; ++r) vcorr[r][h] += psum[wave][r][hi] - psum[wave][r][lo];
        }
        if (wbeg + 256 >= vrun.end) break;
      }
    }
    // ---- (5) every few chunks: take what the accumulators hold for offsets and zero points out ----
    // The accumulators carry sum_t w_t (offset + code) and z_run carries sum_t w_t (offset + zero):
    // two sums up to 2^10 times larger than their difference, the output.  Left to grow over a whole
    // token range their fp32 roundings reach a few 1e-5 of the Value scale, which a long sequence
    // with flat attention (small outputs) sees; subtracting the running zero-point sums every
    // fourth chunk keeps both sums short.
    if (settle) {
#pragma unroll
      for (int hf = 0; hf < 2; ++hf) {
        float sub = 0.0f;                              // for this lane's column and channel group
#pragma unroll
        for (int r = 0; r < R; ++r)
#pragma unroll
          for (int g = 0; g < NGC; ++g) {
            if (hf == 0) z_run[r][g] = uniform(kvs::wave_sum(z_run[r][g]));   // the lanes' partial sums, once
            bool mine;
            if (G == 128) mine = col == r && g == 0;
            else if (G == 64) mine = col == r && g == hf;
            else mine = grp < 2 ? (col == r && g == 2 * hf) : (col == 2 * R + r && g == 2 * hf + 1);
            sub = mine ? z_run[r][g] : sub;
          }
#pragma unroll
        for (int r = 0; r < 4; ++r) acc[hf][r] -= sub;
      }
#pragma unroll
      for (int r = 0; r < R; ++r)
#pragma unroll
        for (int g = 0; g < NGC; ++g) z_run[r][g] = 0.0f;
    }
    wave_lds_sync();                                   // tables are rewritten by the next chunk
  };

  wave_lds_sync();                                     // tables zeroed
  if (wave < nchunks) {
    int nxt = take_chunk();
    int cur = wave;
    int done = 0;
    while (true) {                                     // the registers hold chunk cur and are filled
      score_chunk(keys, nxt);                          // again, piece by piece, for chunk nxt
      value_chunk(vals, nxt, cur, (++done & 3) == 0);
      if (nxt >= nchunks) break;
      cur = nxt;
      nxt = take_chunk();
    }
  }

  // ---- kept (sink) rows: wave w folds rows w, w + kWaves, ... into a softmax state of its own ----
  // (only when this workgroup covers the whole sequence; otherwise the combine kernel does it).
  // Lane = channels 2 lane, 2 lane + 1; the wave's score exchange area is free by now and takes
  // the unnormalised row.  The first row was requested at kernel start.
  const bool fold_keep = a.parts == 1;
  if (fold_keep) {
    const int cnt = min(keep_cnt_b, a.cap);
    float ms[R], ls[R], o0[R], o1[R];
#pragma unroll
    for (int r = 0; r < R; ++r) { ms[r] = -INFINITY; ls[r] = 0.0f; o0[r] = 0.0f; o1[r] = 0.0f; }
    for (int j = wave; j < cnt; j += kWaves) {
      uint32_t kw = keep_first_k, vw = keep_first_v;
      if (j != wave) { kw = keep_rows_k[j * 64]; vw = keep_rows_v[j * 64]; }
      const float k0 = kvs::half_bits_to_float(static_cast<uint16_t>(kw & 0xFFFFu));
      const float k1 = kvs::half_bits_to_float(static_cast<uint16_t>(kw >> 16));
      const float v0 = kvs::half_bits_to_float(static_cast<uint16_t>(vw & 0xFFFFu));
      const float v1 = kvs::half_bits_to_float(static_cast<uint16_t>(vw >> 16));
#pragma unroll
      for (int r = 0; r < R; ++r) {
        const float s2 = uniform(kvs::wave_sum(qf[r][0] * k0 + qf[r][1] * k1));   // log2 units
        const float m_new = fmaxf(ms[r], s2);
        const float alpha = __builtin_amdgcn_exp2f(ms[r] - m_new);
        const float pj = __builtin_amdgcn_exp2f(s2 - m_new);
        ls[r] = ls[r] * alpha + pj;
        o0[r] = o0[r] * alpha + pj * v0;
        o1[r] = o1[r] * alpha + pj * v1;
        ms[r] = m_new;
      }
    }
#pragma unroll
    for (int r = 0; r < R; ++r) {
      reinterpret_cast<float2*>(&sc[wave][r][0])[lane] = float2{o0[r], o1[r]};
      if (lane == 0) { part_m[kWaves + wave][r] = ms[r] * kLn2; part_l[kWaves + wave][r] = ls[r]; }
    }
  }

  // ---- each wave's state to LDS: unnormalised row, max (natural-log units), sum ----------------
  {
    float lsum[R], zsum[R][NGC];
#pragma unroll
    for (int r = 0; r < R; ++r) {
      lsum[r] = kvs::wave_sum(l_run[r]);
#pragma unroll
      for (int g = 0; g < NGC; ++g) zsum[r][g] = kvs::wave_sum(z_run[r][g]);
    }
    float mmine = m_run[0], lmine = lsum[0];
#pragma unroll
    for (int r = 1; r < R; ++r) { mmine = col == r ? m_run[r] : mmine; lmine = col == r ? lsum[r] : lmine; }
    const int head = col < R ? col : 0;
#pragma unroll
    for (int hf = 0; hf < 2; ++hf) {
      // zero-point term of this lane's rows: channels 64 hf + 16 grp + ..., group (64 hf + 16 grp) / G
      const int gc = G == 128 ? 0 : (G == 64 ? hf : 2 * hf + (grp >> 1));
      float zmine = zsum[0][0];
#pragma unroll
      for (int r = 0; r < R; ++r)
#pragma unroll
        for (int g = 0; g < NGC; ++g) zmine = (head == r && gc == g) ? zsum[r][g] : zmine;
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        float4v o;
#pragma unroll
        for (int r = 0; r < 4; ++r) {
          float v = acc[hf][r][i] + row_shift_down<R>(acc[hf][r][i]);
          if (G == 32) {
            const float w2 = row_shift_down<(2 * R) % 16 == 0 ? 1 : (2 * R) % 16>(v);
            v = grp >= 2 ? w2 : v;
          }
          o[r] = v - zmine;
        }
        if (col < R) *reinterpret_cast<float4v*>(part_o(wave, head) + 64 * hf + 16 * grp + 4 * i) = o;
      }
    }
    if (col < R && grp == 0) { part_m[wave][head] = mmine * kLn2; part_l[wave][head] = lmine; }
  }
  if (SPARSE) {                                        // the Value corrections join the wave's rows
    wave_lds_sync();
#pragma unroll
    for (int r = 0; r < R; ++r) {
      part_o(wave, r)[lane] += vcorr[r][0];
      part_o(wave, r)[64 + lane] += vcorr[r][1];
    }
  }
  __syncthreads();

  // ---- merge the waves' states (and the kept rows' states) -----------------------------------
#pragma unroll
  for (int k = 0; k < HPW; ++k) {
    const int r = wave + k * kWaves;
    if (r >= R) break;
    const size_t bq_row = static_cast<size_t>(b) * Hq + hq0 + r;
    float M = -INFINITY;
#pragma unroll
    for (int w = 0; w < kWaves; ++w) M = fmaxf(M, part_m[w][r]);
    if (fold_keep) {
#pragma unroll
      for (int w = kWaves; w < 2 * kWaves; ++w) M = fmaxf(M, part_m[w][r]);
      M = fmaxf(M, extra_m[k]);
    }
    float L = 0.0f, O0 = 0.0f, O1 = 0.0f;
    if (fold_keep && extra_m[k] != -INFINITY) {
      const float f = __expf(extra_m[k] - M);
      L = extra_l[k] * f;
      O0 = extra_o[k].x * f;
      O1 = extra_o[k].y * f;
    }
#pragma unroll
    for (int w = 0; w < kWaves; ++w) {
      const float ms = part_m[w][r];
      const float f = ms == -INFINITY ? 0.0f : __expf(ms - M);
      const float2 o = reinterpret_cast<const float2*>(part_o(w, r))[lane];
      L += part_l[w][r] * f;
      O0 += o.x * f;
      O1 += o.y * f;
    }
    if (a.parts > 1) {                                 // the last workgroup to arrive finishes (below)
      float* dst = a.ws + (bq_row * a.parts + part) * kWsRow;
      kvs::store_coherent(reinterpret_cast<float2*>(dst) + lane, float2{O0, O1});
      if (lane == 0) { kvs::store_coherent(dst + 128, M); kvs::store_coherent(dst + 129, L); }
      continue;
    }
#pragma unroll
    for (int w = 0; w < kWaves; ++w) {
      const float ms = part_m[kWaves + w][r];
      const float f = ms == -INFINITY ? 0.0f : __expf(ms - M);
      const float2 o = reinterpret_cast<const float2*>(&sc[w][r][0])[lane];
      L += part_l[kWaves + w][r] * f;
      O0 += o.x * f;
      O1 += o.y * f;
    }
    const float inv = L > 0.0f ? 1.0f / L : 0.0f;
    const uint32_t packed = static_cast<uint32_t>(kvs::float_to_half_bits_rn(O0 * inv)) |
                            (static_cast<uint32_t>(kvs::float_to_half_bits_rn(O1 * inv)) << 16);
    reinterpret_cast<uint32_t*>(a.out + bq_row * 128)[lane] = packed;
    if (a.lse && lane == 0) a.lse[bq_row] = L > 0.0f ? M + __logf(L) : -INFINITY;
  }

  // ---- several workgroups per (b, h): the one that arrives last finishes the rows ---------------
  // Every part is in memory before its workgroup counts itself in: the parts are written with
  // device-coherent stores, every wave waits until its stores have been acknowledged, then the
  // barrier, then one atomic per workgroup.  The workgroup whose count completes the (b, h) reads
  // all parts with device-coherent loads.  (A device-scope fence pair would do the same by writing
  // back and invalidating the whole L2 of the die, once per workgroup: that more than doubled the
  // kernel's time.)  The last arriver also puts the counter back to zero: nobody else touches it
  // any more in this launch.
  if (a.parts > 1) {
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __syncthreads();
    if (threadIdx.x == 0)
      arrived_last = __hip_atomic_fetch_add(a.arrive + bh, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) == a.parts - 1 ? 1 : 0;
    __syncthreads();
    if (arrived_last) {
      const int cnt = min(keep_cnt_b, a.cap);
#pragma unroll
      for (int k = 0; k < HPW; ++k) {
        const int r = wave + k * kWaves;
        if (r >= R) break;
        const size_t bq_row = static_cast<size_t>(b) * Hq + hq0 + r;
        const uint32_t q2 = reinterpret_cast<const uint32_t*>(a.q + bq_row * 128)[lane];
        kvs::finish_row<true>(q2, a.ws + bq_row * a.parts * kWsRow, a.parts, a.extra ? a.extra + bq_row * kWsRow : nullptr,
                        keep_rows_k, keep_rows_v, cnt, reinterpret_cast<uint32_t*>(a.out + bq_row * 128),
                        a.lse ? a.lse + bq_row : nullptr, lane);
      }
      if (threadIdx.x == 0) __hip_atomic_store(a.arrive + bh, 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
  }
}

inline MfmaArgs make_args(const kvs_desc* d, const kvs::DecodeGeometry& geo, const void* q, const kvs_cache* c,
                          void* out, float* lse, float* ws, int* arrive, int n_used, const float* extra) {
  MfmaArgs a;
  a.q = static_cast<const uint16_t*>(q);
  a.k_codes = c->k_codes; a.v_codes = c->v_codes; a.k_params = c->k_params; a.v_params = c->v_params;
  a.keep_mask = c->keep_mask;
  a.keep_k = static_cast<const uint16_t*>(c->keep_k); a.keep_v = static_cast<const uint16_t*>(c->keep_v);
  a.keep_cnt = c->keep_cnt;
  a.out = static_cast<uint16_t*>(out); a.lse = lse; a.ws = ws; a.arrive = arrive;
  a.k_rowptr = c->k_rowptr; a.k_col = c->k_col; a.k_val = static_cast<const uint16_t*>(c->k_val);
  a.v_rowptr = c->v_rowptr; a.v_col = c->v_col; a.v_val = static_cast<const uint16_t*>(c->v_val);
  a.sparse_cap = static_cast<int>(d->sparse_cap);
  a.n = d->n; a.Hkv = d->Hkv; a.cap = d->keep_cap;
  a.n_used = n_used; a.extra = extra;
  a.parts = geo.splits; a.part_tokens = geo.split_tokens;
  a.rep = d->Hq / d->Hkv; a.head_off = 0;
  return a;
}

// One launch takes R query heads of every KV head, starting at head_off; a shape whose heads do
// not fit the 16 tile columns is served by several launches of a narrower variant, each of which
// streams the codes again.
template <int BITS, int G, int R, bool KPT>
void launch_heads(const kvs_desc* d, const kvs::DecodeGeometry& geo, MfmaArgs args, hipStream_t s) {
  const dim3 grid(d->B * d->Hkv * geo.splits);
  const bool sparse = d->sparse_frac > 0.0f;
  for (args.head_off = 0; args.head_off < args.rep; args.head_off += R) {
    if constexpr (BITS != 8 && !KPT) {
      if (sparse) {
        hipLaunchKernelGGL((decode_mfma_kernel<BITS, G, R, true, false>), grid, dim3(waves_for(BITS, G, R, false, true) * KVS_WAVE),
                           0, s, args);
        continue;
      }
    }
    hipLaunchKernelGGL((decode_mfma_kernel<BITS, G, R, false, KPT>), grid, dim3(waves_for(BITS, G, R, KPT) * KVS_WAVE), 0, s, args);
  }
}

// Per-token Keys: heads x channel groups x [hi | lo] must fit the 16 tile columns, i.e.
// R (128 / G) <= 8 per launch.
template <int BITS>
void launch_bits_kpt(const kvs_desc* d, const kvs::DecodeGeometry& geo, const void* q, const kvs_cache* c, void* out,
                     float* lse, float* ws, int* arrive, int n_used, const float* extra, hipStream_t s) {
  const MfmaArgs a = make_args(d, geo, q, c, out, lse, ws, arrive, n_used, extra);
  const int rep = a.rep;
  if (d->group == 128) {
    if (rep == 1) launch_heads<BITS, 128, 1, true>(d, geo, a, s);
    else if (rep == 2) launch_heads<BITS, 128, 2, true>(d, geo, a, s);
    else if (rep == 4) launch_heads<BITS, 128, 4, true>(d, geo, a, s);
    else launch_heads<BITS, 128, 8, true>(d, geo, a, s);
  } else if (d->group == 64) {
    if (rep == 1) launch_heads<BITS, 64, 1, true>(d, geo, a, s);
    else if (rep == 2) launch_heads<BITS, 64, 2, true>(d, geo, a, s);
    else launch_heads<BITS, 64, 4, true>(d, geo, a, s);             // 8 heads: two launches
  } else {
    if (rep == 1) launch_heads<BITS, 32, 1, true>(d, geo, a, s);
    else launch_heads<BITS, 32, 2, true>(d, geo, a, s);             // 4, 8 heads: two, four launches
  }
}

// Per-channel Keys: 2 R (token groups per tile) columns for the scores, 2 R or (G = 32) 4 R for the
// output: everything fits but 8 heads at G = 32, which takes two launches of 4.  The
// dense-and-sparse variant exists for one query head per KV head.
template <int BITS>
void launch_bits(const kvs_desc* d, const kvs::DecodeGeometry& geo, const void* q, const kvs_cache* c, void* out,
                 float* lse, float* ws, int* arrive, int n_used, const float* extra, hipStream_t s) {
  const MfmaArgs a = make_args(d, geo, q, c, out, lse, ws, arrive, n_used, extra);
  const int rep = a.rep;
  if (d->group == 128) {
    if (rep == 1) launch_heads<BITS, 128, 1, false>(d, geo, a, s);
    else if (rep == 2) launch_heads<BITS, 128, 2, false>(d, geo, a, s);
    else if (rep == 4) launch_heads<BITS, 128, 4, false>(d, geo, a, s);
    else launch_heads<BITS, 128, 8, false>(d, geo, a, s);
  } else if (d->group == 64) {
    if (rep == 1) launch_heads<BITS, 64, 1, false>(d, geo, a, s);
    else if (rep == 2) launch_heads<BITS, 64, 2, false>(d, geo, a, s);
    else if (rep == 4) launch_heads<BITS, 64, 4, false>(d, geo, a, s);
    else launch_heads<BITS, 64, 8, false>(d, geo, a, s);
  } else {
    if (rep == 1) launch_heads<BITS, 32, 1, false>(d, geo, a, s);
    else if (rep == 2) launch_heads<BITS, 32, 2, false>(d, geo, a, s);
    else launch_heads<BITS, 32, 4, false>(d, geo, a, s);             // 8 heads: two launches
  }
}

}  // namespace kvs_mfma

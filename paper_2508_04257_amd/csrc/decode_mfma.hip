// Matrix-core variant of the decode-attention partial kernel for 4-bit caches with group size
// 128 (paper, Section 2 attention equation over the quantised cache; same result as the generic
// kernel in decode.hip, which documents the folding of scales and zero points).
//
// Why matrix cores for a one-row query: at 0.53 bytes per cached element the HBM stream delivers
// ~1e13 codes/s, and unpack + convert + multiply-add on the vector ALU costs 3+ instructions per
// code, which is what bounds the generic kernel.  Here a code is turned into an fp16 operand with
// 7/8 of an instruction ((w >> 4j) & 0x000F000F | 0x64006400 yields two halves 1024 + code) and
// the products run on v_mfma_f32_16x16x32_f16.  The spare output columns of the 16-wide tile
// carry the low half of a hi/lo fp16 split of the other operand (query x scale, weight x scale),
// so the fp16 operand rounding does not reach the result.
//
// A workgroup of 8 waves owns one part of the token range of one (sequence, KV head); each wave
// walks its own run of 128-token chunks with the next chunk's codes already in flight, and the
// waves meet once, at the end, to merge their running softmax states in LDS.  When a single
// workgroup covers the whole sequence the kept (sink) tokens' fp16 rows are folded in and the
// output row is written right there; otherwise the part's state goes to the workspace and the
// combine kernel of decode.hip finishes.  Per 128-token chunk:
//   scores  S^T[token, col] = sum_c code[token, c] * B[c, col]     tokens are the M rows
//   softmax with lane = token (scores pass through LDS once)
//   output  O^T[chan, col] = sum_t code[t, chan] * W[t, col]       channels are the M rows
// Operand layouts follow the instruction: lane l holds row (l % 16) and the 8 contraction
// indices of chunk (l / 16); the result holds rows 4 (l / 16) + i of column (l % 16).
#include "kvs_device.h"

namespace {

typedef _Float16 half8 __attribute__((ext_vector_type(8)));
typedef float float4v __attribute__((ext_vector_type(4)));

#ifndef KVS_MFMA_WAVES
#define KVS_MFMA_WAVES 8
#endif
constexpr int kWaves = KVS_MFMA_WAVES;
constexpr int kThreads = kWaves * KVS_WAVE;
constexpr float kLog2eRsqrtD = 1.4426950408889634f * 0.08838834764831845f;   // log2(e) / sqrt(128)
constexpr float kRsqrtD = 0.08838834764831845f;
constexpr float kLn2 = 0.6931471805599453f;
constexpr int kWsRow = KVS_HEAD_DIM + 2;

// Position of slot j of a 4-bit word inside the 8-half operand built by unpack4().
__device__ __host__ constexpr int slot_of(int j) { return (j & 3) * 2 + (j >> 2); }

// The two exponent patterns live in vector registers (see Magic below) so that
// (x & mask) | magic becomes one v_and_or_b32: with both constants as literals the compiler
// emits two instructions.
struct Magic {
  uint32_t even, odd;   // 0x64006400 (1024 + code), 0x54005400 (64 + code)
};
__device__ inline Magic make_magic() {
  Magic m{0x64006400u, 0x54005400u};
  asm volatile("" : "+v"(m.even), "+v"(m.odd));   // no instruction; only hides the constants
  return m;
}

// Eight 4-bit codes -> eight halves in operand order (c0 c4 c1 c5 c2 c6 c3 c7), five
// instructions.  A nibble in mantissa bits 0-3 under exponent 0x64 reads 1024 + code; a nibble in
// mantissa bits 4-7 under exponent 0x54 reads 64 + code, so the odd codes need no shift.  The
// offsets (1024 for even slots of the word, 64 for odd ones) are removed with the zero points.
__device__ inline half8 unpack4(uint32_t w, const Magic& m) {
  uint32_t r[4];
  const uint32_t t = w >> 8;
  r[0] = (w & 0x000F000Fu) | m.even;
  r[1] = (w & 0x00F000F0u) | m.odd;
  r[2] = (t & 0x000F000Fu) | m.even;
  r[3] = (t & 0x00F000F0u) | m.odd;
  return __builtin_bit_cast(half8, r);
}
constexpr float kEvenOffset = 1024.0f, kOddOffset = 64.0f;

__device__ inline uint32_t word_of(const uint4& v, int r) { return r == 0 ? v.x : (r == 1 ? v.y : (r == 2 ? v.z : v.w)); }

// lane n of each 16-lane row receives the value of lane n + R of the same row (0 past the row end).
template <int R>
__device__ inline float row_shift_down(float v) {
  return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), 0x100 + R, 0xF, 0xF, true));
}

__device__ inline void wave_lds_sync() {
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
  __builtin_amdgcn_wave_barrier();
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

// One 128-token chunk of streamed data as the lanes hold it, Key part and Value part.
struct KeyRegs {
  uint4 kx[2][4];        // Key words: [64-token tile][word row 4 wb + grp], tokens 4 col .. 4 col + 3
  uint2 kp;              // Key parameters of channels 2 lane, 2 lane + 1
};
struct ValueRegs {
  uint4 vx[4][2];        // Value words: [token word 4 mm + grp][channel half], channels 4 col .. + 3
  uint32_t vp0, vp1;     // Value parameters of tokens lane, lane + 64
  uint8_t mask0, mask1;  // keep-mask bytes of the same tokens
};

struct MfmaArgs {
  const uint16_t* q;
  const uint32_t* k_codes; const uint32_t* v_codes; const uint32_t* k_params; const uint32_t* v_params;
  const uint8_t* keep_mask;
  const uint16_t* keep_k; const uint16_t* keep_v; const int32_t* keep_cnt;
  uint16_t* out; float* lse; float* ws;
  int n, Hkv, cap;
  int parts;         // workgroups per (b, h)
  int part_tokens;   // tokens per workgroup
  int wave_tokens;   // tokens per wave, a multiple of 128
};

template <int R>
__global__ __launch_bounds__(kThreads) void decode_mfma_int4_kernel(MfmaArgs a) {
  constexpr int COLS = 2 * R;                      // hi columns 0..R-1, lo columns R..2R-1
  // Per-wave LDS: operand tables in the instruction's slot order, and the score exchange.
  // Column COLS of each table stays zero: the lanes of the unused tile columns read it.
  __shared__ __align__(16) _Float16 bq[kWaves][COLS + 1][128];   // query x Key scale (hi | lo)
  __shared__ __align__(16) float sc[kWaves][R][128];             // scores, token order
  __shared__ __align__(16) _Float16 wh[kWaves][COLS + 1][128];   // weight x Value scale (hi | lo)
  __shared__ __align__(16) float part_o[kWaves][R][128];     // end of kernel: each wave's row, max, sum
  __shared__ float part_m[kWaves][R], part_l[kWaves][R];

  const int lane = threadIdx.x & (KVS_WAVE - 1), wave = threadIdx.x / KVS_WAVE;
  const int col = lane & 15, grp = lane >> 4;
  const Magic magic = make_magic();
  const int tcol = col < COLS ? col : COLS;        // table column this lane's tile column reads
  bq[wave][COLS][lane] = 0;  bq[wave][COLS][64 + lane] = 0;
  wh[wave][COLS][lane] = 0;  wh[wave][COLS][64 + lane] = 0;
  const int n = a.n;
  const size_t bh = blockIdx.x / a.parts;
  const int part = blockIdx.x % a.parts;
  const int b = static_cast<int>(bh / a.Hkv), h = static_cast<int>(bh % a.Hkv);
  const int Hq = a.Hkv * R;
  const int hq0 = h * R;
  const int keep_cnt_b = a.keep_cnt[b];            // uniform: a scalar load, issued first

  // Query of the lane's two channels (2 lane, 2 lane + 1), all R heads, scaled to log2 units.
  float qf[R][2];
#pragma unroll
  for (int r = 0; r < R; ++r) {
    const uint32_t two = reinterpret_cast<const uint32_t*>(a.q + (static_cast<size_t>(b) * Hq + hq0 + r) * 128)[lane];
    qf[r][0] = kvs::half_bits_to_float(static_cast<uint16_t>(two & 0xFFFFu)) * kLog2eRsqrtD;
    qf[r][1] = kvs::half_bits_to_float(static_cast<uint16_t>(two >> 16)) * kLog2eRsqrtD;
  }

  const int part_end = min(n, (part + 1) * a.part_tokens);
  const int tok_begin = min(part_end, part * a.part_tokens + wave * a.wave_tokens);
  const int tok_end = min(part_end, tok_begin + a.wave_tokens);
  const uint8_t* mask_b = a.keep_mask + static_cast<size_t>(b) * n;
  const uint32_t* kcodes = a.k_codes + bh * (n / 64) * (16 * 64);
  const uint32_t* vcodes = a.v_codes + bh * (n / 128) * (16 * 128);
  const uint32_t* kparams = a.k_params + bh * (n / 128) * 128;
  const uint32_t* vparams = a.v_params + bh * n;

  float m_run[R], l_run[R], z_run[R];              // running max (log2 units), lane-partial sums
  float4v acc[2][4];                               // [channel half][r]: rows = channels 64 half + 16 grp + 4 i + r
#pragma unroll
  for (int r = 0; r < R; ++r) { m_run[r] = -INFINITY; l_run[r] = 0.0f; z_run[r] = 0.0f; }
#pragma unroll
  for (int hf = 0; hf < 2; ++hf)
#pragma unroll
    for (int r = 0; r < 4; ++r) acc[hf][r] = float4v{0.0f, 0.0f, 0.0f, 0.0f};

  // Streamed data is double buffered in registers, Keys and Values on their own schedule: the
  // next chunk's Key loads are issued before the current chunk's score product and its Value
  // loads right after it (when the current Key registers have just died), so a chunk's stream is
  // in flight for about one whole chunk of math.  Addresses past the wave's last chunk are
  // clamped to it: every path issues the same number of loads, which keeps the waits exact.
  const int nchunks = (tok_end - tok_begin) / 128;
  KeyRegs key_a, key_b;
  ValueRegs val_a, val_b;
  auto load_keys = [&](KeyRegs& s, int ci) {
    const int t0 = tok_begin + min(ci, nchunks - 1) * 128;
    const uint32_t* ktile = kcodes + static_cast<size_t>(t0 / 64) * (16 * 64);
#pragma unroll
    for (int kt = 0; kt < 2; ++kt)
#pragma unroll
      for (int wb = 0; wb < 4; ++wb)            // word row 4 wb + grp, tokens 4 col .. 4 col + 3
        s.kx[kt][wb] = *reinterpret_cast<const uint4*>(ktile + kt * 1024 + (4 * wb + grp) * 64 + 4 * col);
    s.kp = reinterpret_cast<const uint2*>(kparams + static_cast<size_t>(t0 / 128) * 128)[lane];
  };
  auto load_values = [&](ValueRegs& s, int ci) {
    const int t0 = tok_begin + min(ci, nchunks - 1) * 128;
    const uint32_t* vtile = vcodes + static_cast<size_t>(t0 / 128) * (16 * 128);
    s.vp0 = vparams[t0 + lane];
    s.vp1 = vparams[t0 + 64 + lane];
    s.mask0 = mask_b[t0 + lane];
    s.mask1 = mask_b[t0 + 64 + lane];
#pragma unroll
    for (int mm = 0; mm < 4; ++mm)              // token word 4 mm + grp, channels 64 hf + 4 col .. + 3
#pragma unroll
      for (int hf = 0; hf < 2; ++hf)
        s.vx[mm][hf] = *reinterpret_cast<const uint4*>(vtile + (4 * mm + grp) * 128 + 64 * hf + 4 * col);
  };

  float bias[R];
  auto score_chunk = [&](const KeyRegs& s) {
    // ---- (1) B operand of the score product: q x scale as hi + lo halves; bias per head -------
    {
      float s0, s1; int z0, z1;
      kvs::unpack_param(s.kp.x, s0, z0);
      kvs::unpack_param(s.kp.y, s1, z1);
      const float zf0 = static_cast<float>(z0) + kEvenOffset, zf1 = static_cast<float>(z1) + kOddOffset;
      const int c0 = 2 * lane;                         // channels c0, c0 + 1: word c0 / 8, slots c0 % 8, + 1
      const int p0 = (c0 & ~7) + slot_of(c0 & 7), p1 = (c0 & ~7) + slot_of((c0 & 7) + 1);
#pragma unroll
      for (int r = 0; r < R; ++r) {
        const float a0 = qf[r][0] * s0, a1 = qf[r][1] * s1;
        const _Float16 h0 = static_cast<_Float16>(a0), h1 = static_cast<_Float16>(a1);
        const _Float16 e0 = static_cast<_Float16>(a0 - static_cast<float>(h0));
        const _Float16 e1 = static_cast<_Float16>(a1 - static_cast<float>(h1));
        bq[wave][r][p0] = h0;  bq[wave][r][p1] = h1;
        bq[wave][R + r][p0] = e0;  bq[wave][R + r][p1] = e1;
        // what the product will contain for the 1024 offset and the zero point, exactly as rounded
        bias[r] = kvs::wave_sum((static_cast<float>(h0) + static_cast<float>(e0)) * zf0 +
                                (static_cast<float>(h1) + static_cast<float>(e1)) * zf1);
      }
    }
    wave_lds_sync();
    half8 bqr[4];
#pragma unroll
    for (int wb = 0; wb < 4; ++wb) bqr[wb] = *reinterpret_cast<const half8*>(&bq[wave][tcol][(4 * wb + grp) * 8]);

    // ---- (2) scores on the matrix cores; hi + lo columns merged; to LDS in token order ---------
#pragma unroll
    for (int kt = 0; kt < 2; ++kt) {
      float4v d[4];                                    // [r]: rows = tokens 64 kt + 4 m + r, m = 0..15
#pragma unroll
      for (int r = 0; r < 4; ++r) d[r] = float4v{0.0f, 0.0f, 0.0f, 0.0f};
#pragma unroll
      for (int wb = 0; wb < 4; ++wb)
#pragma unroll
        for (int r = 0; r < 4; ++r)                    // four independent accumulation chains
          d[r] = __builtin_amdgcn_mfma_f32_16x16x32_f16(unpack4(word_of(s.kx[kt][wb], r), magic), bqr[wb], d[r], 0, 0, 0);
      float4v out[4];                                  // [i]: tokens 64 kt + 16 grp + 4 i + (0..3)
#pragma unroll
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int r = 0; r < 4; ++r) out[i][r] = d[r][i] + row_shift_down<R>(d[r][i]);
      if (col < R) {
#pragma unroll
        for (int i = 0; i < 4; ++i)
          *reinterpret_cast<float4v*>(&sc[wave][col][64 * kt + 16 * grp + 4 * i]) = out[i];
      }
    }
    wave_lds_sync();
  };

  auto value_chunk = [&](const ValueRegs& s) {
    // ---- (3) online softmax, lane = tokens (lane, lane + 64); weights x Value scale to LDS -----
    float alpha[R];
    {
      float sv0, sv1; int zv0, zv1;
      kvs::unpack_param(s.vp0, sv0, zv0);
      kvs::unpack_param(s.vp1, sv1, zv1);
      const float toff = (lane & 1) ? kOddOffset : kEvenOffset;   // tokens lane and lane + 64 share parity
      const float zf0 = static_cast<float>(zv0) + toff, zf1 = static_cast<float>(zv1) + toff;
      const int p0 = (lane & ~7) + slot_of(lane & 7);  // operand position of token lane (and + 64)
#pragma unroll
      for (int r = 0; r < R; ++r) {
        const float s0 = s.mask0 ? -INFINITY : sc[wave][r][lane] - bias[r];
        const float s1 = s.mask1 ? -INFINITY : sc[wave][r][64 + lane] - bias[r];
        const float mx = kvs::wave_max(fmaxf(s0, s1));
        const float m_new = fmaxf(m_run[r], mx);
        const float m_use = m_new == -INFINITY ? 0.0f : m_new;
        alpha[r] = __builtin_amdgcn_exp2f(m_run[r] - m_use);
        const float e0 = __builtin_amdgcn_exp2f(s0 - m_use), e1 = __builtin_amdgcn_exp2f(s1 - m_use);
        m_run[r] = m_new;
        const float w0 = e0 * sv0, w1 = e1 * sv1;
        const _Float16 h0 = static_cast<_Float16>(w0), h1 = static_cast<_Float16>(w1);
        const _Float16 g0 = static_cast<_Float16>(w0 - static_cast<float>(h0));
        const _Float16 g1 = static_cast<_Float16>(w1 - static_cast<float>(h1));
        wh[wave][r][p0] = h0;  wh[wave][r][64 + p0] = h1;
        wh[wave][R + r][p0] = g0;  wh[wave][R + r][64 + p0] = g1;
        l_run[r] = l_run[r] * alpha[r] + (e0 + e1);
        z_run[r] = z_run[r] * alpha[r] + (static_cast<float>(h0) + static_cast<float>(g0)) * zf0 +
                   (static_cast<float>(h1) + static_cast<float>(g1)) * zf1;
      }
    }
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
    half8 bwr[4];
#pragma unroll
    for (int mm = 0; mm < 4; ++mm) bwr[mm] = *reinterpret_cast<const half8*>(&wh[wave][tcol][(4 * mm + grp) * 8]);
#pragma unroll
    for (int mm = 0; mm < 4; ++mm)
#pragma unroll
      for (int hf = 0; hf < 2; ++hf)
#pragma unroll
        for (int r = 0; r < 4; ++r)                    // eight independent accumulation chains
          acc[hf][r] = __builtin_amdgcn_mfma_f32_16x16x32_f16(unpack4(word_of(s.vx[mm][hf], r), magic), bwr[mm], acc[hf][r], 0, 0, 0);
    wave_lds_sync();                                   // tables are rewritten by the next chunk
  };

  if (nchunks > 0) {
    load_keys(key_a, 0);
    load_values(val_a, 0);
    for (int ci = 0; ci < nchunks; ci += 2) {
      load_keys(key_b, ci + 1);
      score_chunk(key_a);
      load_values(val_b, ci + 1);
      value_chunk(val_a);
      if (ci + 1 >= nchunks) break;
      load_keys(key_a, ci + 2);
      score_chunk(key_b);
      load_values(val_a, ci + 2);
      value_chunk(val_b);
    }
  }

  // ---- kept (sink) rows: start their loads now so that they overlap the merge below -----------
  // Wave r finishes head r; lane = channels 2 lane, 2 lane + 1.  The first 8 rows are fetched in
  // one batch (the usual keep set is a handful of tokens).
  constexpr int kBatch = 8;
  const bool finisher = wave < R && a.parts == 1;
  const int cnt = min(keep_cnt_b, a.cap);
  const uint32_t* kk = reinterpret_cast<const uint32_t*>(a.keep_k) + bh * a.cap * 64 + lane;
  const uint32_t* kv = reinterpret_cast<const uint32_t*>(a.keep_v) + bh * a.cap * 64 + lane;
  uint32_t kw[kBatch], vw[kBatch];
#pragma unroll
  for (int u = 0; u < kBatch; ++u) { kw[u] = 0; vw[u] = 0; }
  if (finisher && cnt > 0) {
#pragma unroll
    for (int u = 0; u < kBatch; ++u) {
      const int j = min(u, cnt - 1);
      kw[u] = kk[j * 64];
      vw[u] = kv[j * 64];
    }
  }

  // ---- each wave's state to LDS: unnormalised row, max (natural-log units), sum ----------------
  {
    float zsum[R], lsum[R];
#pragma unroll
    for (int r = 0; r < R; ++r) { zsum[r] = kvs::wave_sum(z_run[r]); lsum[r] = kvs::wave_sum(l_run[r]); }
    float zmine = zsum[0], mmine = m_run[0], lmine = lsum[0];
#pragma unroll
    for (int r = 1; r < R; ++r) {
      zmine = col == r ? zsum[r] : zmine; mmine = col == r ? m_run[r] : mmine; lmine = col == r ? lsum[r] : lmine;
    }
    const int head = col < R ? col : 0;
#pragma unroll
    for (int hf = 0; hf < 2; ++hf)
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        float4v o;
#pragma unroll
        for (int r = 0; r < 4; ++r) o[r] = acc[hf][r][i] + row_shift_down<R>(acc[hf][r][i]) - zmine;
        if (col < R) *reinterpret_cast<float4v*>(&part_o[wave][head][64 * hf + 16 * grp + 4 * i]) = o;
      }
    if (col < R && grp == 0) { part_m[wave][head] = mmine * kLn2; part_l[wave][head] = lmine; }
  }
  __syncthreads();

  // ---- merge the waves' states ----------------------------------------------------------------
  if (wave < R) {
    const int r = wave;
    const size_t bq_row = static_cast<size_t>(b) * Hq + hq0 + r;
    float M = -INFINITY;
#pragma unroll
    for (int w = 0; w < kWaves; ++w) M = fmaxf(M, part_m[w][r]);
    float L = 0.0f, O0 = 0.0f, O1 = 0.0f;
#pragma unroll
    for (int w = 0; w < kWaves; ++w) {
      const float ms = part_m[w][r];
      const float f = ms == -INFINITY ? 0.0f : __expf(ms - M);
      const float2 o = reinterpret_cast<const float2*>(&part_o[w][r][0])[lane];
      L += part_l[w][r] * f;
      O0 += o.x * f;
      O1 += o.y * f;
    }
    if (a.parts > 1) {                                 // another kernel merges the parts
      float* dst = a.ws + (bq_row * a.parts + part) * kWsRow;
      reinterpret_cast<float2*>(dst)[lane] = float2{O0, O1};
      if (lane == 0) { dst[128] = M; dst[129] = L; }
      return;
    }
    // Kept tokens: exact fp16 rows join the same running softmax.
    const uint32_t q2 = reinterpret_cast<const uint32_t*>(a.q + bq_row * 128)[lane];
    const float q0 = kvs::half_bits_to_float(static_cast<uint16_t>(q2 & 0xFFFFu));
    const float q1 = kvs::half_bits_to_float(static_cast<uint16_t>(q2 >> 16));
    for (int j0 = 0; j0 < cnt; j0 += kBatch) {
      if (j0 > 0) {                                    // rare: more kept tokens than one batch
#pragma unroll
        for (int u = 0; u < kBatch; ++u) {
          const int j = min(j0 + u, cnt - 1);
          kw[u] = kk[j * 64];
          vw[u] = kv[j * 64];
        }
      }
      float sj[kBatch];
#pragma unroll
      for (int u = 0; u < kBatch; ++u)
        sj[u] = q0 * kvs::half_bits_to_float(static_cast<uint16_t>(kw[u] & 0xFFFFu)) +
                q1 * kvs::half_bits_to_float(static_cast<uint16_t>(kw[u] >> 16));
#pragma unroll
      for (int o = 32; o > 0; o >>= 1)                 // eight reductions in step
#pragma unroll
        for (int u = 0; u < kBatch; ++u) sj[u] += __shfl_xor(sj[u], o, KVS_WAVE);
#pragma unroll
      for (int u = 0; u < kBatch; ++u) {
        if (j0 + u < cnt) {
          const float sc_u = sj[u] * kRsqrtD;
          const float m_new = fmaxf(M, sc_u);
          const float alpha = M == -INFINITY ? 0.0f : __expf(M - m_new);
          const float p = __expf(sc_u - m_new);
          L = L * alpha + p;
          O0 = O0 * alpha + p * kvs::half_bits_to_float(static_cast<uint16_t>(vw[u] & 0xFFFFu));
          O1 = O1 * alpha + p * kvs::half_bits_to_float(static_cast<uint16_t>(vw[u] >> 16));
          M = m_new;
        }
      }
    }
    const float inv = L > 0.0f ? 1.0f / L : 0.0f;
    const uint32_t packed = static_cast<uint32_t>(kvs::float_to_half_bits_rn(O0 * inv)) |
                            (static_cast<uint32_t>(kvs::float_to_half_bits_rn(O1 * inv)) << 16);
    reinterpret_cast<uint32_t*>(a.out + bq_row * 128)[lane] = packed;
    if (a.lse && lane == 0) a.lse[bq_row] = L > 0.0f ? M + __logf(L) : -INFINITY;
  }
}

template <int R>
void launch(const kvs_desc* d, const kvs::DecodeGeometry& geo, const MfmaArgs& args, hipStream_t s) {
  hipLaunchKernelGGL((decode_mfma_int4_kernel<R>), dim3(d->B * d->Hkv * geo.splits), dim3(kThreads), 0, s, args);
}

}  // namespace

namespace kvs {

bool decode_mfma_supported(const kvs_desc* d) {
  return d->bits == 4 && d->group == 128 && d->sparse_frac == 0.0f;
}

int decode_mfma_waves() { return kWaves; }

void launch_decode_mfma(const kvs_desc* d, const DecodeGeometry& geo, const void* q, const kvs_cache* c,
                        void* out, float* lse, float* ws, hipStream_t s) {
  MfmaArgs a;
  a.q = static_cast<const uint16_t*>(q);
  a.k_codes = c->k_codes; a.v_codes = c->v_codes; a.k_params = c->k_params; a.v_params = c->v_params;
  a.keep_mask = c->keep_mask;
  a.keep_k = static_cast<const uint16_t*>(c->keep_k); a.keep_v = static_cast<const uint16_t*>(c->keep_v);
  a.keep_cnt = c->keep_cnt;
  a.out = static_cast<uint16_t*>(out); a.lse = lse; a.ws = ws;
  a.n = d->n; a.Hkv = d->Hkv; a.cap = d->keep_cap;
  a.parts = geo.splits; a.part_tokens = geo.split_tokens; a.wave_tokens = geo.wave_tokens;
  switch (d->Hq / d->Hkv) {
    case 1: launch<1>(d, geo, a, s); break;
    case 2: launch<2>(d, geo, a, s); break;
    case 4: launch<4>(d, geo, a, s); break;
    default: launch<8>(d, geo, a, s); break;
  }
}

}  // namespace kvs

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
// One wave is one independent split (no workgroup barriers).  Per 128-token chunk:
//   scores  S^T[token, col] = sum_c code[token, c] * B[c, col]     tokens are the M rows
//   softmax with lane = token (scores pass through LDS once)
//   output  O^T[chan, col] = sum_t code[t, chan] * W[t, col]       channels are the M rows
// Operand layouts follow the instruction: lane l holds row (l % 16) and the 8 contraction
// indices of chunk (l / 16); the result holds rows 4 (l / 16) + i of column (l % 16).
#include "kvs_device.h"

namespace {

typedef _Float16 half8 __attribute__((ext_vector_type(8)));
typedef float float4v __attribute__((ext_vector_type(4)));

constexpr int kWaves = 4;
constexpr int kThreads = kWaves * KVS_WAVE;
constexpr float kLog2eRsqrtD = 1.4426950408889634f * 0.08838834764831845f;   // log2(e) / sqrt(128)
constexpr float kLn2 = 0.6931471805599453f;
constexpr int kWsRow = KVS_HEAD_DIM + 2;

// Position of slot j of a 4-bit word inside the 8-half operand built by unpack4().
__device__ __host__ constexpr int slot_of(int j) { return (j & 3) * 2 + (j >> 2); }

// Eight 4-bit codes -> eight halves (1024 + code), operand order (c0 c4 c1 c5 c2 c6 c3 c7).
__device__ inline half8 unpack4(uint32_t w) {
  uint32_t r[4];
  r[0] = (w & 0x000F000Fu) | 0x64006400u;
  r[1] = ((w >> 4) & 0x000F000Fu) | 0x64006400u;
  r[2] = ((w >> 8) & 0x000F000Fu) | 0x64006400u;
  r[3] = ((w >> 12) & 0x000F000Fu) | 0x64006400u;
  return __builtin_bit_cast(half8, r);
}

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

template <int R>
__global__ __launch_bounds__(kThreads) void decode_mfma_int4_kernel(
    const uint16_t* __restrict__ q, const uint32_t* __restrict__ k_codes,
    const uint32_t* __restrict__ v_codes, const uint32_t* __restrict__ k_params,
    const uint32_t* __restrict__ v_params, const uint8_t* __restrict__ keep_mask, int n, int Hkv,
    int splits, int split_tokens, float* __restrict__ ws) {
  constexpr int COLS = 2 * R;                      // hi columns 0..R-1, lo columns R..2R-1
  // Per-wave LDS: operand tables in the instruction's slot order, and the score exchange.
  __shared__ __align__(16) _Float16 bq[kWaves][COLS][128];   // query x Key scale (hi | lo)
  __shared__ __align__(16) float sc[kWaves][R][128];         // scores, token order
  __shared__ __align__(16) _Float16 wh[kWaves][COLS][128];   // weight x Value scale (hi | lo)

  const int lane = threadIdx.x & (KVS_WAVE - 1), wave = threadIdx.x / KVS_WAVE;
  const int col = lane & 15, grp = lane >> 4;
  const int waves_per_head = (splits + kWaves - 1) / kWaves;   // workgroups per (b, h)
  const size_t bh = blockIdx.x / waves_per_head;
  const int split = (blockIdx.x % waves_per_head) * kWaves + wave;
  if (split >= splits) return;                     // whole wave leaves; no barriers are used
  const int b = static_cast<int>(bh / Hkv), h = static_cast<int>(bh % Hkv);
  const int Hq = Hkv * R;
  const int hq0 = h * R;

  // Query of the lane's two channels (2 lane, 2 lane + 1), all R heads, scaled to log2 units.
  float qf[R][2];
#pragma unroll
  for (int r = 0; r < R; ++r) {
    const uint32_t two = reinterpret_cast<const uint32_t*>(q + (static_cast<size_t>(b) * Hq + hq0 + r) * 128)[lane];
    qf[r][0] = kvs::half_bits_to_float(static_cast<uint16_t>(two & 0xFFFFu)) * kLog2eRsqrtD;
    qf[r][1] = kvs::half_bits_to_float(static_cast<uint16_t>(two >> 16)) * kLog2eRsqrtD;
  }

  const int tok_begin = split * split_tokens;
  const int tok_end = min(n, tok_begin + split_tokens);
  const uint8_t* mask_b = keep_mask + static_cast<size_t>(b) * n;

  float m_run[R], l_run[R], z_run[R];              // running max (log2 units), lane-partial sums
  float4v acc[2][4];                               // [channel half][r]: rows = channels 64 half + 16 grp + 4 i + r
#pragma unroll
  for (int r = 0; r < R; ++r) { m_run[r] = -INFINITY; l_run[r] = 0.0f; z_run[r] = 0.0f; }
#pragma unroll
  for (int hf = 0; hf < 2; ++hf)
#pragma unroll
    for (int r = 0; r < 4; ++r) acc[hf][r] = float4v{0.0f, 0.0f, 0.0f, 0.0f};

  for (int t0 = tok_begin; t0 < tok_end; t0 += 128) {
    // ---- issue the chunk's code loads early -------------------------------------------------
    const uint32_t* ktile = k_codes + (bh * (n / 64) + static_cast<size_t>(t0 / 64)) * (16 * 64);
    const uint32_t* vtile = v_codes + (bh * (n / 128) + static_cast<size_t>(t0 / 128)) * (16 * 128);
    uint4 kx[2][4], vx[4][2];
#pragma unroll
    for (int kt = 0; kt < 2; ++kt)
#pragma unroll
      for (int wb = 0; wb < 4; ++wb)            // word row 4 wb + grp, tokens 4 col .. 4 col + 3
        kx[kt][wb] = *reinterpret_cast<const uint4*>(ktile + kt * 1024 + (4 * wb + grp) * 64 + 4 * col);
#pragma unroll
    for (int mm = 0; mm < 4; ++mm)              // token word 4 mm + grp, channels 64 hf + 4 col .. + 3
#pragma unroll
      for (int hf = 0; hf < 2; ++hf)
        vx[mm][hf] = *reinterpret_cast<const uint4*>(vtile + (4 * mm + grp) * 128 + 64 * hf + 4 * col);
    const uint2 kp = reinterpret_cast<const uint2*>(k_params + (bh * (n / 128) + static_cast<size_t>(t0 / 128)) * 128)[lane];
    const uint32_t vp0 = v_params[bh * n + t0 + lane], vp1 = v_params[bh * n + t0 + 64 + lane];
    const bool kept0 = mask_b[t0 + lane] != 0, kept1 = mask_b[t0 + 64 + lane] != 0;

    // ---- (1) B operand of the score product: q x scale as hi + lo halves; bias per head -------
    float bias[R];
    {
      float s0, s1; int z0, z1;
      kvs::unpack_param(kp.x, s0, z0);
      kvs::unpack_param(kp.y, s1, z1);
      const float zf0 = static_cast<float>(z0 + 1024), zf1 = static_cast<float>(z1 + 1024);
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
    for (int wb = 0; wb < 4; ++wb) {
      bqr[wb] = half8{0, 0, 0, 0, 0, 0, 0, 0};
      if (col < COLS) bqr[wb] = *reinterpret_cast<const half8*>(&bq[wave][col][(4 * wb + grp) * 8]);
    }

    // ---- (2) scores on the matrix cores; hi + lo columns merged; to LDS in token order ---------
#pragma unroll
    for (int kt = 0; kt < 2; ++kt) {
#pragma unroll
      for (int r = 0; r < 4; ++r) {                    // rows = tokens 64 kt + 4 m + r, m = 0..15
        float4v d = {0.0f, 0.0f, 0.0f, 0.0f};
#pragma unroll
        for (int wb = 0; wb < 4; ++wb)
          d = __builtin_amdgcn_mfma_f32_16x16x32_f16(unpack4(word_of(kx[kt][wb], r)), bqr[wb], d, 0, 0, 0);
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          const float s = d[i] + row_shift_down<R>(d[i]);
          if (col < R) sc[wave][col][64 * kt + 16 * grp + 4 * i + r] = s;   // token of row 4 grp + i
        }
      }
    }
    wave_lds_sync();

    // ---- (3) online softmax, lane = tokens (lane, lane + 64); weights x Value scale to LDS -----
    float alpha[R];
    {
      float sv0, sv1; int zv0, zv1;
      kvs::unpack_param(vp0, sv0, zv0);
      kvs::unpack_param(vp1, sv1, zv1);
      const float zf0 = static_cast<float>(zv0 + 1024), zf1 = static_cast<float>(zv1 + 1024);
      const int p0 = (lane & ~7) + slot_of(lane & 7);  // operand position of token lane (and + 64)
#pragma unroll
      for (int r = 0; r < R; ++r) {
        const float s0 = kept0 ? -INFINITY : sc[wave][r][lane] - bias[r];
        const float s1 = kept1 ? -INFINITY : sc[wave][r][64 + lane] - bias[r];
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
        float a = 1.0f;
#pragma unroll
        for (int r = 0; r < R; ++r) a = (col % R) == r ? alpha[r] : a;
#pragma unroll
        for (int hf = 0; hf < 2; ++hf)
#pragma unroll
          for (int r = 0; r < 4; ++r) acc[hf][r] *= a;
      }
    }
    half8 bwr[4];
#pragma unroll
    for (int mm = 0; mm < 4; ++mm) {
      bwr[mm] = half8{0, 0, 0, 0, 0, 0, 0, 0};
      if (col < COLS) bwr[mm] = *reinterpret_cast<const half8*>(&wh[wave][col][(4 * mm + grp) * 8]);
    }
#pragma unroll
    for (int hf = 0; hf < 2; ++hf)
#pragma unroll
      for (int r = 0; r < 4; ++r)
#pragma unroll
        for (int mm = 0; mm < 4; ++mm)
          acc[hf][r] = __builtin_amdgcn_mfma_f32_16x16x32_f16(unpack4(word_of(vx[mm][hf], r)), bwr[mm], acc[hf][r], 0, 0, 0);
    wave_lds_sync();                                   // tables are rewritten by the next chunk
  }

  // ---- write the split's partial result: unnormalised row, max (natural-log units), sum --------
  float zsum[R], lsum[R];
#pragma unroll
  for (int r = 0; r < R; ++r) { zsum[r] = kvs::wave_sum(z_run[r]); lsum[r] = kvs::wave_sum(l_run[r]); }
  float zmine = zsum[0], mmine = m_run[0], lmine = lsum[0];
#pragma unroll
  for (int r = 1; r < R; ++r) {
    zmine = col == r ? zsum[r] : zmine; mmine = col == r ? m_run[r] : mmine; lmine = col == r ? lsum[r] : lmine;
  }
  float* dst = ws + ((static_cast<size_t>(b) * Hq + hq0 + (col < R ? col : 0)) * splits + split) * kWsRow;
#pragma unroll
  for (int hf = 0; hf < 2; ++hf)
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      float4v o;
#pragma unroll
      for (int r = 0; r < 4; ++r) o[r] = acc[hf][r][i] + row_shift_down<R>(acc[hf][r][i]) - zmine;
      if (col < R) *reinterpret_cast<float4v*>(dst + 64 * hf + 16 * grp + 4 * i) = o;
    }
  if (col < R && grp == 0) { dst[128] = mmine * kLn2; dst[129] = lmine; }
}

template <int R>
void launch(const kvs_desc* d, const kvs::DecodeGeometry& geo, const void* q, const kvs_cache* c, float* ws,
            hipStream_t s) {
  const int waves_per_head = (geo.splits + kWaves - 1) / kWaves;
  const int grid = d->B * d->Hkv * waves_per_head;
  hipLaunchKernelGGL((decode_mfma_int4_kernel<R>), dim3(grid), dim3(kThreads), 0, s,
                     static_cast<const uint16_t*>(q), c->k_codes, c->v_codes, c->k_params, c->v_params,
                     c->keep_mask, d->n, d->Hkv, geo.splits, geo.split_tokens, ws);
}

}  // namespace

namespace kvs {

bool decode_mfma_supported(const kvs_desc* d) {
  return d->bits == 4 && d->group == 128 && d->sparse_frac == 0.0f;
}

void launch_decode_mfma(const kvs_desc* d, const DecodeGeometry& geo, const void* q, const kvs_cache* c,
                        float* ws, hipStream_t s) {
  switch (d->Hq / d->Hkv) {
    case 1: launch<1>(d, geo, q, c, ws, s); break;
    case 2: launch<2>(d, geo, q, c, ws, s); break;
    case 4: launch<4>(d, geo, q, c, ws, s); break;
    default: launch<8>(d, geo, q, c, ws, s); break;
  }
}

}  // namespace kvs

// kvs_decode_attn: decode attention that streams the packed low-bit KV cache and merges the
// fp16 rows of the kept (sink) tokens (paper, Section 2 attention equation; the split of the
// attention sum into sink and non-sink tokens is the equation of Section 4.2).
//
// The entry points, the kernel that finishes a call whose stream was cut into parts, and the
// vector-ALU stream kernel.  Dense caches, and caches with isolated outliers and one query head
// per KV head, stream through the matrix-core kernel (decode_mfma_impl.h); the stream kernel here
// serves caches with isolated outliers and several query heads per KV head, and states the
// arithmetic (how scales and zero points are folded) in its plainest form.
//   decode_partial_kernel  one workgroup per (sequence, KV head, token split).  Each wave walks
//       128-token chunks: scores from the Key code tile (lane = token, the per-channel scale is
//       folded into the query once per token group, the zero points into one bias per group),
//       online softmax with wave reductions, then the Value code tile (lane = channel, the
//       per-token scale folded into the softmax weight, zero points into one scalar per channel
//       group).  Kept tokens are masked out of this stream.  Result: unnormalised output row,
//       running max and sum per (b, hq, split) in the workspace.
//   decode_combine_kernel  one workgroup per (b, hq): log-sum-exp merge of the splits, then the
//       kept tokens' fp16 rows are folded into the same online softmax, normalise, store fp16.
//
// The stream of codes and parameters is the only large traffic (HBM bound); dequantisation is
// never materialised.
#include "kvs_device.h"

namespace {

using kvs::Fmt;

constexpr int kWaves = 4;
constexpr int kThreads = kWaves * KVS_WAVE;
constexpr float kRsqrtD = 0.08838834764831845f;   // 1 / sqrt(128)
constexpr int kWsRow = KVS_HEAD_DIM + 2;          // output row, running max, running sum

template <int BITS>
__device__ inline float code_at(uint32_t word, int j) {
  return static_cast<float>((word >> Fmt<BITS>::shift(j)) & static_cast<uint32_t>(Fmt<BITS>::qmax));
}

// CSR arrays of the isolated fp16 outliers (dense-and-sparse caches only).
struct SparseView {
  const int32_t* k_rowptr; const uint16_t* k_col; const uint16_t* k_val;   // rows (b, h, token), col = channel
  const int32_t* v_rowptr; const uint16_t* v_col; const uint16_t* v_val;   // rows (b, h, tile, channel), col = token in tile
  int cap;   // entries the col / val arrays hold; row pointers past it (reported overflow) are not followed
};

template <int BITS, int G, int R, bool SPARSE>
__global__ __launch_bounds__(kThreads) void decode_partial_kernel(
    const uint16_t* __restrict__ q, const uint32_t* __restrict__ k_codes,
    const uint32_t* __restrict__ v_codes, const uint32_t* __restrict__ k_params,
    const uint32_t* __restrict__ v_params, const uint8_t* __restrict__ keep_mask, int n, int n_used, int Hkv,
    int rep, int splits, int split_tokens, float* __restrict__ ws, SparseView sp) {
  constexpr int W = Fmt<BITS>::W, cpw = Fmt<BITS>::cpw;
  constexpr int NGK = 128 / G;   // Key token groups per 128-token chunk
  constexpr int NGC = 128 / G;   // Value channel groups per row
  constexpr int LOG2G = G == 32 ? 5 : (G == 64 ? 6 : 7);
  __shared__ float qf[R][128];                       // query / sqrt(D)
  __shared__ float qs[kWaves][NGK][R][128];          // query x Key scale, per wave and group
  __shared__ float wl[kWaves][R][NGC][128];          // softmax weight x Value scale, per token
  __shared__ float red_m[kWaves][R], red_l[kWaves][R];
  // Dense-and-sparse only: an isolated slot holds code 0, i.e. it dequantises to -scale * zero.
  // Replacing it by its fp16 value adds  q (val + scale zero)  to a score and
  // p (val + scale zero)  to an output channel.
  __shared__ float kz[SPARSE ? kWaves : 1][NGK][SPARSE ? 128 : 1];      // Key zero points
  __shared__ float pl[SPARSE ? kWaves : 1][R][SPARSE ? 128 : 1];        // softmax weights
  __shared__ float wz[SPARSE ? kWaves : 1][R][NGC][SPARSE ? 128 : 1];   // weight x Value scale x zero

  const int tid = threadIdx.x, lane = tid & (KVS_WAVE - 1), wave = tid / KVS_WAVE;
  const int head_groups = rep / R;
  int bid = blockIdx.x;
  const int split = bid % splits;  bid /= splits;
  const int hg = bid % head_groups;  bid /= head_groups;
  const size_t bh = bid;                             // b * Hkv + h
  const int b = static_cast<int>(bh / Hkv), h = static_cast<int>(bh % Hkv);
  const int Hq = Hkv * rep;
  const int hq0 = h * rep + hg * R;

  for (int i = tid; i < R * 128; i += kThreads) {
    const int r = i >> 7, c = i & 127;
    qf[r][c] = kvs::half_bits_to_float(q[(static_cast<size_t>(b) * Hq + hq0 + r) * 128 + c]) * kRsqrtD;
  }
  __syncthreads();

  const int tok_begin = split * split_tokens;
  const int tok_end = min(n_used, tok_begin + split_tokens);   // n is the layout, n_used what is attended to
  const int chunks = (tok_end - tok_begin) / KVS_V_TILE;
  const int rounds = (chunks + kWaves - 1) / kWaves;
  const uint8_t* mask_b = keep_mask + static_cast<size_t>(b) * n;

  float m[R], l[R], acc[R][2], zacc[R][NGC];
#pragma unroll
  for (int r = 0; r < R; ++r) {
    m[r] = -INFINITY; l[r] = 0.0f; acc[r][0] = acc[r][1] = 0.0f;
#pragma unroll
    for (int g = 0; g < NGC; ++g) zacc[r][g] = 0.0f;
  }

  for (int round = 0; round < rounds; ++round) {
    const int ci = round * kWaves + wave;
    const bool active = ci < chunks;                 // wave-uniform
    const int t0 = tok_begin + (active ? ci : 0) * KVS_V_TILE;

    // (1) query x Key scale for the chunk's token groups; bias = sum_c (q s)_c zero_c.
    float kbias[NGK][R];
    if (active) {
#pragma unroll
      for (int gl = 0; gl < NGK; ++gl) {
        const uint32_t* kp = k_params + (bh * (n / G) + static_cast<size_t>(t0 / G + gl)) * 128;
        float part[R];
#pragma unroll
        for (int r = 0; r < R; ++r) part[r] = 0.0f;
#pragma unroll
        for (int half = 0; half < 2; ++half) {
          const int c = lane + 64 * half;
          float s; int z;
          kvs::unpack_param(kp[c], s, z);
#pragma unroll
          for (int r = 0; r < R; ++r) {
            const float v = qf[r][c] * s;
            qs[wave][gl][r][c] = v;
            part[r] += v * static_cast<float>(z);
          }
          if constexpr (SPARSE) kz[wave][gl][c] = static_cast<float>(z);
        }
#pragma unroll
        for (int r = 0; r < R; ++r) kbias[gl][r] = kvs::wave_sum(part[r]);
      }
    }
    __syncthreads();

    // (2) scores: lane = token, two Key tiles of 64 tokens.
    float sc[2][R];
    if (active) {
#pragma unroll
      for (int kt = 0; kt < 2; ++kt) {
        const int tl = 64 * kt + lane;
        const int gl = tl >> LOG2G;
        const uint32_t* tile = k_codes + (bh * (n / KVS_K_TILE) + static_cast<size_t>(t0 / KVS_K_TILE + kt)) * (W * KVS_K_TILE);
        float dot[R];
#pragma unroll
        for (int r = 0; r < R; ++r) dot[r] = 0.0f;
#pragma unroll
        for (int w = 0; w < W; ++w) {
          const uint32_t word = tile[w * KVS_K_TILE + lane];
#pragma unroll
          for (int j = 0; j < cpw; ++j) {
            const int c = cpw * w + j;
            if (c < 128) {
              const float f = code_at<BITS>(word, j);
#pragma unroll
              for (int r = 0; r < R; ++r) dot[r] += qs[wave][gl][r][c] * f;
            }
          }
        }
        if constexpr (SPARSE) {
          const size_t row = bh * n + static_cast<size_t>(t0 + tl);
          const int e1 = min(sp.k_rowptr[row + 1], sp.cap);
          for (int e = max(sp.k_rowptr[row], 0); e < e1; ++e) {   // (a never-quantised cache must not walk out of the arrays)
            const int c = sp.k_col[e] & 127;
            const float v = kvs::half_bits_to_float(sp.k_val[e]);
#pragma unroll
            for (int r = 0; r < R; ++r) dot[r] += qf[r][c] * v + qs[wave][gl][r][c] * kz[wave][gl][c];
          }
        }
        const bool kept = mask_b[t0 + tl] != 0;
#pragma unroll
        for (int r = 0; r < R; ++r) {
          float bias = kbias[0][r];
#pragma unroll
          for (int g = 1; g < NGK; ++g) bias = gl == g ? kbias[g][r] : bias;
          sc[kt][r] = kept ? -INFINITY : dot[r] - bias;
        }
      }

      // (3) online softmax, (4) weights x Value scale.
      uint32_t vp[2][NGC];
#pragma unroll
      for (int kt = 0; kt < 2; ++kt)
#pragma unroll
        for (int g = 0; g < NGC; ++g)
          vp[kt][g] = v_params[(bh * n + static_cast<size_t>(t0 + 64 * kt + lane)) * NGC + g];
#pragma unroll
      for (int r = 0; r < R; ++r) {
        const float mx = kvs::wave_max(fmaxf(sc[0][r], sc[1][r]));
        const float m_new = fmaxf(m[r], mx);
        const float m_use = m_new == -INFINITY ? 0.0f : m_new;
        const float alpha = __expf(m[r] - m_use);
        const float p0 = __expf(sc[0][r] - m_use), p1 = __expf(sc[1][r] - m_use);
        l[r] = l[r] * alpha + kvs::wave_sum(p0 + p1);
        acc[r][0] *= alpha; acc[r][1] *= alpha;
        m[r] = m_new;
#pragma unroll
        for (int g = 0; g < NGC; ++g) {
          float s0, s1; int z0, z1;
          kvs::unpack_param(vp[0][g], s0, z0);
          kvs::unpack_param(vp[1][g], s1, z1);
          const float w0 = p0 * s0, w1 = p1 * s1;
          wl[wave][r][g][lane] = w0;
          wl[wave][r][g][64 + lane] = w1;
          zacc[r][g] = zacc[r][g] * alpha + w0 * static_cast<float>(z0) + w1 * static_cast<float>(z1);
          if constexpr (SPARSE) {
            wz[wave][r][g][lane] = w0 * static_cast<float>(z0);
            wz[wave][r][g][64 + lane] = w1 * static_cast<float>(z1);
          }
        }
        if constexpr (SPARSE) { pl[wave][r][lane] = p0; pl[wave][r][64 + lane] = p1; }
      }
    }
    __syncthreads();

    // (5) weighted Value sum: lane = channels lane and lane + 64, words packed along tokens.
    if (active) {
      const uint32_t* tile = v_codes + (bh * (n / KVS_V_TILE) + static_cast<size_t>(t0 / KVS_V_TILE)) * (W * 128);
      const int g0 = lane >> LOG2G, g1 = (lane + 64) >> LOG2G;
#pragma unroll
      for (int u = 0; u < W; ++u) {
        const uint32_t w0 = tile[u * 128 + lane];
        const uint32_t w1 = tile[u * 128 + 64 + lane];
#pragma unroll
        for (int j = 0; j < cpw; ++j) {
          const int tl = cpw * u + j;
          if (tl < 128) {
            const float f0 = code_at<BITS>(w0, j), f1 = code_at<BITS>(w1, j);
#pragma unroll
            for (int r = 0; r < R; ++r) {
              acc[r][0] += wl[wave][r][g0][tl] * f0;
              acc[r][1] += wl[wave][r][g1][tl] * f1;
            }
          }
        }
      }
      if constexpr (SPARSE) {
#pragma unroll
        for (int half = 0; half < 2; ++half) {
          const int g = half ? g1 : g0;
          const size_t row = (bh * (n / KVS_V_TILE) + static_cast<size_t>(t0 / KVS_V_TILE)) * 128 + lane + 64 * half;
          const int e1 = min(sp.v_rowptr[row + 1], sp.cap);
          for (int e = max(sp.v_rowptr[row], 0); e < e1; ++e) {
            const int tl = sp.v_col[e] & 127;
            const float v = kvs::half_bits_to_float(sp.v_val[e]);
#pragma unroll
            for (int r = 0; r < R; ++r) acc[r][half] += pl[wave][r][tl] * v + wz[wave][r][g][tl];
          }
        }
      }
    }
    __syncthreads();
  }

  // Remove the zero-point term of each channel group, then merge the four waves.
  float* stage = &qs[0][0][0][0];                    // reuse: [kWaves][R][128] floats fit (NGK >= 1)
  const int g0 = lane >> LOG2G, g1 = (lane + 64) >> LOG2G;
#pragma unroll
  for (int r = 0; r < R; ++r) {
    float zs[NGC];
#pragma unroll
    for (int g = 0; g < NGC; ++g) zs[g] = kvs::wave_sum(zacc[r][g]);
    float z0 = zs[0], z1 = zs[0];
#pragma unroll
    for (int g = 1; g < NGC; ++g) { z0 = g0 == g ? zs[g] : z0; z1 = g1 == g ? zs[g] : z1; }
    stage[(wave * R + r) * 128 + lane] = acc[r][0] - z0;
    stage[(wave * R + r) * 128 + 64 + lane] = acc[r][1] - z1;
    if (lane == 0) { red_m[wave][r] = m[r]; red_l[wave][r] = l[r]; }
  }
  __syncthreads();
  for (int i = tid; i < R * 128; i += kThreads) {
    const int r = i >> 7, c = i & 127;
    float M = -INFINITY;
#pragma unroll
    for (int w = 0; w < kWaves; ++w) M = fmaxf(M, red_m[w][r]);
    float L = 0.0f, O = 0.0f;
#pragma unroll
    for (int w = 0; w < kWaves; ++w) {
      const float f = red_m[w][r] == -INFINITY ? 0.0f : __expf(red_m[w][r] - M);
      L += red_l[w][r] * f;
      O += stage[(w * R + r) * 128 + c] * f;
    }
    float* dst = ws + ((static_cast<size_t>(b) * Hq + hq0 + r) * splits + split) * kWsRow;
    dst[c] = O;
    if (c == 0) { dst[128] = M; dst[129] = L; }
  }
}

// One wave per (b, hq), lane = channels 2 lane and 2 lane + 1: log-sum-exp merge of the splits,
// then the kept tokens' fp16 rows join the same running softmax.
__global__ __launch_bounds__(KVS_WAVE) void decode_combine_kernel(
    const uint16_t* __restrict__ q, const float* __restrict__ ws, const float* __restrict__ extra, int splits, int Hq, int Hkv,
    int cap, const uint16_t* __restrict__ keep_k, const uint16_t* __restrict__ keep_v,
    const int32_t* __restrict__ keep_cnt, uint16_t* __restrict__ out, float* __restrict__ lse) {
  const int lane = threadIdx.x;
  const size_t bq = blockIdx.x;                       // b * Hq + hq
  const int b = static_cast<int>(bq / Hq), hq = static_cast<int>(bq % Hq);
  const int h = hq / (Hq / Hkv);
  const float* row = ws + bq * splits * kWsRow;
  const int cnt = min(keep_cnt[b], cap);
  const uint32_t q2 = reinterpret_cast<const uint32_t*>(q + bq * 128)[lane];
  const float q0 = kvs::half_bits_to_float(static_cast<uint16_t>(q2 & 0xFFFFu));
  const float q1 = kvs::half_bits_to_float(static_cast<uint16_t>(q2 >> 16));

  // The first kept rows are requested before anything else is read.
  constexpr int kKeepBatch = 8;
  const uint32_t* kk = reinterpret_cast<const uint32_t*>(keep_k) + (static_cast<size_t>(b) * Hkv + h) * cap * 64 + lane;
  const uint32_t* kv = reinterpret_cast<const uint32_t*>(keep_v) + (static_cast<size_t>(b) * Hkv + h) * cap * 64 + lane;
  uint32_t kw_next[kKeepBatch], vw_next[kKeepBatch];
#pragma unroll
  for (int u = 0; u < kKeepBatch; ++u) {
    kw_next[u] = 0;  vw_next[u] = 0;
    if (cnt > 0) {
      const int j = min(u, cnt - 1);
      kw_next[u] = kk[j * 64];
      vw_next[u] = kv[j * 64];
    }
  }

  // One more part, if given: the fp16 rows of a growing cache's residual window (the same triple
  // of unnormalised row, maximum and sum, one per (b, hq)).
  const float* xrow = extra ? extra + bq * kWsRow : nullptr;
  float M = -INFINITY;
  for (int s = lane; s < splits; s += KVS_WAVE) M = fmaxf(M, row[s * kWsRow + 128]);
  M = kvs::wave_max(M);
  if (xrow) M = fmaxf(M, xrow[128]);
  float L = 0.0f, O0 = 0.0f, O1 = 0.0f;
  if (xrow) {
    const float ms = xrow[128];
    const float f = ms == -INFINITY ? 0.0f : __expf(ms - M);
    const float2 o = reinterpret_cast<const float2*>(xrow)[lane];
    L = xrow[129] * f;
    O0 = o.x * f;
    O1 = o.y * f;
  }
#pragma unroll 4
  for (int s = 0; s < splits; ++s) {
    const float ms = row[s * kWsRow + 128];
    const float f = ms == -INFINITY ? 0.0f : __expf(ms - M);
    const float2 o = reinterpret_cast<const float2*>(row + s * kWsRow)[lane];
    L += row[s * kWsRow + 129] * f;
    O0 += o.x * f;
    O1 += o.y * f;
  }

  // Kept tokens: exact fp16 rows, eight per step; the step after next is requested before this
  // one is folded in (the first one was requested at the top of the kernel).
  for (int j0 = 0; j0 < cnt; j0 += kKeepBatch) {
    uint32_t kw[kKeepBatch], vw[kKeepBatch];
#pragma unroll
    for (int u = 0; u < kKeepBatch; ++u) { kw[u] = kw_next[u]; vw[u] = vw_next[u]; }
    if (j0 + kKeepBatch < cnt) {
#pragma unroll
      for (int u = 0; u < kKeepBatch; ++u) {
        const int j = min(j0 + kKeepBatch + u, cnt - 1);
        kw_next[u] = kk[j * 64];
        vw_next[u] = kv[j * 64];
      }
    }
    float sc[kKeepBatch];
#pragma unroll
    for (int u = 0; u < kKeepBatch; ++u)               // the reductions of one step are independent of each other
      sc[u] = kvs::wave_sum(q0 * kvs::half_bits_to_float(static_cast<uint16_t>(kw[u] & 0xFFFFu)) +
                            q1 * kvs::half_bits_to_float(static_cast<uint16_t>(kw[u] >> 16))) * kRsqrtD;
#pragma unroll
    for (int u = 0; u < kKeepBatch; ++u) {
      if (j0 + u < cnt) {
        const float m_new = fmaxf(M, sc[u]);
        const float alpha = M == -INFINITY ? 0.0f : __expf(M - m_new);
        const float p = __expf(sc[u] - m_new);
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
  reinterpret_cast<uint32_t*>(out + bq * 128)[lane] = packed;
  if (lse && lane == 0) lse[bq] = L > 0.0f ? M + __logf(L) : -INFINITY;
}

// The stream kernel serves what the matrix-core kernel does not: caches with isolated outliers
// and more than one query head per KV head (so only its SPARSE variant is launched).
template <int BITS, int G, int R>
void launch_partial(const kvs_desc* d, const kvs::DecodeGeometry& geo, const void* q, const kvs_cache* c,
                    float* ws, int n_used, hipStream_t s) {
  const int rep = d->Hq / d->Hkv;
  const int grid = d->B * d->Hkv * (rep / R) * geo.splits;
  SparseView sp{c->k_rowptr, c->k_col, static_cast<const uint16_t*>(c->k_val),
                c->v_rowptr, c->v_col, static_cast<const uint16_t*>(c->v_val),
                static_cast<int>(d->sparse_cap)};
  hipLaunchKernelGGL((decode_partial_kernel<BITS, G, R, true>), dim3(grid), dim3(kThreads), 0, s,
                     static_cast<const uint16_t*>(q), c->k_codes, c->v_codes, c->k_params, c->v_params,
                     c->keep_mask, d->n, n_used, d->Hkv, rep, geo.splits, geo.split_tokens, ws, sp);
}

template <int BITS, int G>
void launch_partial_r(const kvs_desc* d, const kvs::DecodeGeometry& geo, const void* q, const kvs_cache* c,
                      float* ws, int n_used, hipStream_t s) {
  switch (d->Hq / d->Hkv) {
    case 1: launch_partial<BITS, G, 1>(d, geo, q, c, ws, n_used, s); break;
    case 2: launch_partial<BITS, G, 2>(d, geo, q, c, ws, n_used, s); break;
    default: launch_partial<BITS, G, 4>(d, geo, q, c, ws, n_used, s); break;   // 8 = two groups of 4 heads
  }
}

template <int BITS>
void launch_partial_g(const kvs_desc* d, const kvs::DecodeGeometry& geo, const void* q, const kvs_cache* c,
                      float* ws, int n_used, hipStream_t s) {
  switch (d->group) {
    case 32: launch_partial_r<BITS, 32>(d, geo, q, c, ws, n_used, s); break;
    case 64: launch_partial_r<BITS, 64>(d, geo, q, c, ws, n_used, s); break;
    default: launch_partial_r<BITS, 128>(d, geo, q, c, ws, n_used, s); break;
  }
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

static kvs_status check_decode_args(const kvs_desc* desc, const void* q, const kvs_cache* cache, const void* out,
                                    const void* workspace) {
  const kvs_status st = kvs::validate_desc(desc);
  if (st != KVS_OK) return st;
  if (!q || !cache || !out || !workspace) return KVS_ERR_INVALID;
  if (!cache->k_codes || !cache->v_codes || !cache->k_params || !cache->v_params ||
      !cache->keep_cnt || !cache->keep_mask)
    return KVS_ERR_INVALID;
  if (desc->keep_cap > 0 && (!cache->keep_k || !cache->keep_v)) return KVS_ERR_INVALID;
  if (desc->sparse_frac > 0.0f && (!cache->k_rowptr || !cache->k_col || !cache->k_val ||
                                   !cache->v_rowptr || !cache->v_col || !cache->v_val))
    return KVS_ERR_INVALID;
  return KVS_OK;
}

// Dense caches: the first n_used tokens (whole blocks) through the stream kernels, then - unless
// one matrix-core workgroup per head has already finished the rows - the combine kernel, which
// also takes the residual rows' part when there is one.
static void decode_dense(const kvs_desc* desc, const void* q, const kvs_cache* cache, int n_used, const float* extra,
                         void* out, float* lse, float* ws, hipStream_t s) {
  int splits = 0;
  if (n_used > 0) {
    const kvs::DecodeGeometry geo = kvs::decode_geometry(desc, n_used);
    splits = geo.splits;
    if (geo.mfma) {
      kvs::launch_decode_mfma(desc, geo, q, cache, out, lse, ws, nullptr, n_used, extra, s);
      if (geo.splits == 1) return;                       // finished in one kernel, the extra part included
    } else {
      switch (desc->bits) {
        case 2: launch_partial_g<2>(desc, geo, q, cache, ws, n_used, s); break;
        case 3: launch_partial_g<3>(desc, geo, q, cache, ws, n_used, s); break;
        default: launch_partial_g<4>(desc, geo, q, cache, ws, n_used, s); break;   // (8 bit has no isolated outliers)
      }
    }
  }
  hipLaunchKernelGGL(decode_combine_kernel, dim3(desc->B * desc->Hq), dim3(KVS_WAVE), 0, s,
                     static_cast<const uint16_t*>(q), ws, extra, splits, desc->Hq, desc->Hkv, desc->keep_cap,
                     static_cast<const uint16_t*>(cache->keep_k), static_cast<const uint16_t*>(cache->keep_v),
                     cache->keep_cnt, static_cast<uint16_t*>(out), lse);
}

extern "C" kvs_status kvs_decode_attn(const kvs_desc* desc, const void* q, const kvs_cache* cache,
                                       void* out, float* lse, void* workspace, void* stream) {
  const kvs_status st = check_decode_args(desc, q, cache, out, workspace);
  if (st != KVS_OK) return st;
  hipStream_t s = static_cast<hipStream_t>(stream);
  float* ws = static_cast<float*>(workspace);
  const kvs::DecodeGeometry geo = kvs::decode_geometry(desc);
  if (geo.mfma && desc->sparse_frac > 0.0f) {        // Key corrections, matrix-core kernel, finish
    float* cs = ws + kvs::decode_parts_floats(desc, geo);
    kvs::launch_sparse_key_corr(desc, q, cache, cs, s);
    kvs::launch_decode_mfma(desc, geo, q, cache, out, lse, ws, cs, desc->n, nullptr, s);
    kvs::launch_decode_finish_sparse(desc, geo, q, cache, ws, cs, out, lse, s);
  } else {
    decode_dense(desc, q, cache, desc->n, nullptr, out, lse, ws, s);
  }
  return hipGetLastError() == hipSuccess ? KVS_OK : KVS_ERR_DEVICE;
}

extern "C" kvs_status kvs_decode_attn_n(const kvs_desc* desc, const void* q, const kvs_cache* cache, int32_t n_tokens,
                                         void* out, float* lse, void* workspace, void* stream) {
  const kvs_status st = check_decode_args(desc, q, cache, out, workspace);
  if (st != KVS_OK) return st;
  if (desc->sparse_frac > 0.0f) return KVS_ERR_UNSUPPORTED;
  if (n_tokens < 1 || n_tokens > desc->n) return KVS_ERR_INVALID;
  hipStream_t s = static_cast<hipStream_t>(stream);
  float* ws = static_cast<float*>(workspace);
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
  decode_dense(desc, q, cache, n_used, extra, out, lse, ws, s);
  return hipGetLastError() == hipSuccess ? KVS_OK : KVS_ERR_DEVICE;
}

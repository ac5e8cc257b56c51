// Dense-and-sparse decode attention around the matrix-core kernel (paper, Section 5.1: isolated
// fp16 outliers; Section 2 attention equation).  An isolated slot holds code 0 in the packed
// cache, i.e. it dequantises to  -scale * zero;  replacing it by its fp16 value v adds
//     q_c (v + scale zero)   to the score of its token        (Keys)
//     p_t (v + scale zero)   to the output channel it sits in (Values).
// The Key side is known before the softmax and the Value side only after it, so the call becomes
//   1. sparse_key_corr_kernel      per token, the sum of its Key corrections (log2 units)
//   2. decode_mfma_kernel<SPARSE>  adds them to the scores, leaves every corrected score behind
//   3. decode_finish_sparse_kernel Value corrections with the final softmax weights, merge of the
//                                  parts, kept rows, output.
// Any number of query heads per KV head: the corrections are per (sequence, query head, token).
#include "kvs_device.h"

namespace {

constexpr float kLog2eRsqrtD = 1.4426950408889634f * 0.08838834764831845f;   // log2(e) / sqrt(128)
constexpr float kRsqrtD = 0.08838834764831845f;
constexpr float kLn2 = 0.6931471805599453f;
constexpr int kWsRow = KVS_HEAD_DIM + 2;

// One thread per token, kKeyIlp tokens in flight per thread (the three dependent loads of a row -
// pointers, entries, parameters - are each issued for all of them before any is used).
constexpr int kKeyIlp = 4;
__global__ __launch_bounds__(128) void sparse_key_corr_kernel(
    const uint16_t* __restrict__ q, const uint32_t* __restrict__ k_params, const int32_t* __restrict__ k_rowptr,
    const uint16_t* __restrict__ k_col, const uint16_t* __restrict__ k_val, int cap, int n, int group,
    int Hq, int Hkv, float* __restrict__ cs) {
  __shared__ float qf[128];
  __shared__ uint32_t prm_s[(128 * kKeyIlp / 32) * 128];     // parameter rows of the block's token groups
  const int blocks = (n + 128 * kKeyIlp - 1) / (128 * kKeyIlp);
  const size_t bq = blockIdx.x / blocks;              // b * Hq + hq
  const size_t bh = (bq / Hq) * Hkv + (bq % Hq) / (Hq / Hkv);  // b * Hkv + h: the rows the head reads
  const int tb = (blockIdx.x % blocks) * (128 * kKeyIlp);     // first token of the block
  const int t0 = tb + threadIdx.x;
  // The row pointers head the chain of dependent loads: they are requested first, together with
  // the query and the parameter rows (before the barrier, which would otherwise hold them back).
  int e0[kKeyIlp], e1[kKeyIlp];
#pragma unroll
  for (int u = 0; u < kKeyIlp; ++u) {
    const int t = min(t0 + 128 * u, n - 1);
    // (clamped on both sides: a cache that was never quantised must not send the walk out of the arrays)
    e0[u] = max(0, min(k_rowptr[bh * n + t], cap));
    e1[u] = max(0, min(k_rowptr[bh * n + t + 1], cap));
  }
  // the first entry of every row likewise (most rows hold one or two)
  int c_first[kKeyIlp];
  float v_first[kKeyIlp];
#pragma unroll
  for (int u = 0; u < kKeyIlp; ++u) {
    const int e = min(e0[u], max(e1[u], 1) - 1);
    c_first[u] = k_col[e] & 127;
    v_first[u] = kvs::half_bits_to_float(k_val[e]);
  }
  qf[threadIdx.x] = kvs::half_bits_to_float(q[bq * 128 + threadIdx.x]) * kLog2eRsqrtD;
  const int groups = (min(n - tb, 128 * kKeyIlp) + group - 1) / group;
  for (int i = threadIdx.x; i < groups * 128; i += 128)
    prm_s[i] = k_params[(bh * (n / group) + static_cast<size_t>(tb / group)) * 128 + i];
  __syncthreads();
  float acc[kKeyIlp];
  int len = 0;
#pragma unroll
  for (int u = 0; u < kKeyIlp; ++u) { acc[u] = 0.0f; len = max(len, e1[u] - e0[u]); }
  for (int i = 0; i < len; ++i) {
    int c[kKeyIlp];
    float v[kKeyIlp];
    uint32_t prm[kKeyIlp];
#pragma unroll
    for (int u = 0; u < kKeyIlp; ++u) {
      if (i == 0) { c[u] = c_first[u]; v[u] = v_first[u]; continue; }
      const int e = min(e0[u] + i, max(e1[u], 1) - 1);      // clamped; unused when the row is shorter
      c[u] = k_col[e] & 127;
      v[u] = kvs::half_bits_to_float(k_val[e]);
    }
#pragma unroll
    for (int u = 0; u < kKeyIlp; ++u) {
      const int t = min(t0 + 128 * u, n - 1);
      prm[u] = prm_s[((t - tb) / group) * 128 + c[u]];
    }
#pragma unroll
    for (int u = 0; u < kKeyIlp; ++u) {
      float s; int z;
      kvs::unpack_param(prm[u], s, z);
      if (e0[u] + i < e1[u]) acc[u] += qf[c[u]] * (v[u] + s * static_cast<float>(z));
    }
  }
#pragma unroll
  for (int u = 0; u < kKeyIlp; ++u)
    if (t0 + 128 * u < n) cs[bq * n + t0 + 128 * u] = acc[u];
}

// One workgroup per (b, hq).  A thread owns one channel and every eighth 128-token tile, i.e. a
// set of CSR rows (tile, channel) of the Value outliers, and walks kValIlp of them at a time; the
// eight partial sums of a channel meet in LDS.  Then one wave merges the parts and the kept rows
// as the dense path's combine kernel does.
constexpr int kFinishThreads = 1024;
constexpr int kValIlp = 4;

__global__ __launch_bounds__(kFinishThreads) void decode_finish_sparse_kernel(
    const uint16_t* __restrict__ q, const float* __restrict__ ws, int splits, int Hq, int Hkv, int n, int group,
    int cap, const uint16_t* __restrict__ keep_k, const uint16_t* __restrict__ keep_v,
    const int32_t* __restrict__ keep_cnt, const uint32_t* __restrict__ v_params,
    const int32_t* __restrict__ v_rowptr, const uint16_t* __restrict__ v_col, const uint16_t* __restrict__ v_val,
    int sparse_cap, const float* __restrict__ cs, uint16_t* __restrict__ out, float* __restrict__ lse) {
  extern __shared__ uint32_t seg_s[];                 // [4096] scores, then [4096 * ngc] Value parameters
  __shared__ float red[kFinishThreads / 128][128];
  __shared__ float corr[128];

  const int tid = threadIdx.x, lane = tid & (KVS_WAVE - 1);
  const size_t bq = blockIdx.x;                       // b * Hq + hq
  const int b = static_cast<int>(bq / Hq), hq = static_cast<int>(bq % Hq);
  const int h = hq / (Hq / Hkv);
  const size_t bh = static_cast<size_t>(b) * Hkv + h;
  const float* part = ws + bq * splits * kWsRow;
  const int ngc = 128 / group;

  // Wave 0 finishes the row at the end; what it needs from memory is requested right away.
  const bool finisher = tid < KVS_WAVE;
  const int cnt = min(keep_cnt[b], cap);
  const uint32_t* kk = reinterpret_cast<const uint32_t*>(keep_k) + bh * cap * 64 + lane;
  const uint32_t* kv = reinterpret_cast<const uint32_t*>(keep_v) + bh * cap * 64 + lane;
  uint32_t q2 = 0, kw[4] = {0, 0, 0, 0}, vw[4] = {0, 0, 0, 0};
  float2 o_first = {0.0f, 0.0f};
  if (finisher) {
    q2 = reinterpret_cast<const uint32_t*>(q + bq * 128)[lane];
    o_first = reinterpret_cast<const float2*>(part)[lane];
    if (cnt > 0) {
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        const int j = min(u, cnt - 1);
        kw[u] = kk[j * 64];
        vw[u] = kv[j * 64];
      }
    }
  }
  float M = -INFINITY;                                // natural-log units
  for (int s = 0; s < splits; ++s) M = fmaxf(M, part[s * kWsRow + 128]);
  const float m2 = M == -INFINITY ? 0.0f : M / kLn2;  // the same maximum in log2 units

  const int c = tid & 127, tg = tid >> 7;
  constexpr int kStride = kFinishThreads / 128;       // tile groups
  constexpr int kSegTiles = kStride * kValIlp;        // tiles (of 128 tokens) per staged segment
  const int tiles = n / 128;
  float* sc_s = reinterpret_cast<float*>(seg_s);
  const uint32_t* pr_s = seg_s + kSegTiles * 128;
  float acc = 0.0f;
  for (int seg_tile = 0; seg_tile < tiles; seg_tile += kSegTiles) {
    const int seg_tokens = min(kSegTiles, tiles - seg_tile) * 128;
    int e0[kValIlp], e1[kValIlp], len = 0;
#pragma unroll
    for (int u = 0; u < kValIlp; ++u) {               // row pointers in flight while the segment is staged
      const int tile = min(seg_tile + tg + kStride * u, tiles - 1);
      const size_t row = bh * n + static_cast<size_t>(tile) * 128 + c;
      e0[u] = max(0, min(v_rowptr[row], sparse_cap));
      e1[u] = seg_tile + tg + kStride * u < tiles ? max(0, min(v_rowptr[row + 1], sparse_cap)) : e0[u];
    }
    // the first entry of every row is requested before the segment is staged (most rows hold one or two)
    int col_first[kValIlp];
    float val_first[kValIlp];
#pragma unroll
    for (int u = 0; u < kValIlp; ++u) {
      const int e = min(e0[u], max(e1[u], 1) - 1);
      col_first[u] = v_col[e] & 127;
      val_first[u] = kvs::half_bits_to_float(v_val[e]);
    }
    __syncthreads();
    for (int i = tid; i < seg_tokens; i += kFinishThreads) sc_s[i] = cs[bq * n + seg_tile * 128 + i];
    for (int i = tid; i < seg_tokens * ngc; i += kFinishThreads)
      seg_s[kSegTiles * 128 + i] = v_params[(bh * n + static_cast<size_t>(seg_tile) * 128) * ngc + i];
    __syncthreads();
#pragma unroll
    for (int u = 0; u < kValIlp; ++u) len = max(len, e1[u] - e0[u]);
    for (int i = 0; i < len; ++i) {
      int tok[kValIlp];
      float val[kValIlp];
#pragma unroll
      for (int u = 0; u < kValIlp; ++u) {
        if (i == 0) { tok[u] = (tg + kStride * u) * 128 + col_first[u]; val[u] = val_first[u]; continue; }
        const int e = min(e0[u] + i, max(e1[u], 1) - 1);    // clamped; unused when the row is shorter
        tok[u] = (tg + kStride * u) * 128 + (v_col[e] & 127);   // token inside the segment
        val[u] = kvs::half_bits_to_float(v_val[e]);
      }
#pragma unroll
      for (int u = 0; u < kValIlp; ++u) {
        if (e0[u] + i < e1[u]) {
          float s; int z;
          kvs::unpack_param(pr_s[tok[u] * ngc + c / group], s, z);
          acc += __builtin_amdgcn_exp2f(sc_s[tok[u]] - m2) * (val[u] + s * static_cast<float>(z));
        }
      }
    }
  }
  red[tg][c] = acc;
  __syncthreads();
  if (tid < 128) {
    float t = 0.0f;
#pragma unroll
    for (int g = 0; g < kStride; ++g) t += red[g][tid];
    corr[tid] = t;
  }
  __syncthreads();
  if (!finisher) return;

  // ---- one wave: merge the parts, add the corrections, fold the kept rows in, write ----------
  const float q0 = kvs::half_bits_to_float(static_cast<uint16_t>(q2 & 0xFFFFu));
  const float q1 = kvs::half_bits_to_float(static_cast<uint16_t>(q2 >> 16));
  float L = 0.0f, O0 = corr[2 * lane], O1 = corr[2 * lane + 1];
  for (int s = 0; s < splits; ++s) {
    const float ms = part[s * kWsRow + 128];
    const float f = ms == -INFINITY ? 0.0f : __expf(ms - M);
    const float2 o = s == 0 ? o_first : reinterpret_cast<const float2*>(part + s * kWsRow)[lane];
    L += part[s * kWsRow + 129] * f;
    O0 += o.x * f;
    O1 += o.y * f;
  }
  for (int j0 = 0; j0 < cnt; j0 += 4) {
    if (j0 > 0) {
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        const int j = min(j0 + u, cnt - 1);
        kw[u] = kk[j * 64];
        vw[u] = kv[j * 64];
      }
    }
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      if (j0 + u < cnt) {
        const float dot = q0 * kvs::half_bits_to_float(static_cast<uint16_t>(kw[u] & 0xFFFFu)) +
                          q1 * kvs::half_bits_to_float(static_cast<uint16_t>(kw[u] >> 16));
        const float s = kvs::wave_sum(dot) * kRsqrtD;
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
  const float inv = L > 0.0f ? 1.0f / L : 0.0f;
  const uint32_t packed = static_cast<uint32_t>(kvs::float_to_half_bits_rn(O0 * inv)) |
                          (static_cast<uint32_t>(kvs::float_to_half_bits_rn(O1 * inv)) << 16);
  reinterpret_cast<uint32_t*>(out + bq * 128)[lane] = packed;
  if (lse && lane == 0) lse[bq] = L > 0.0f ? M + __logf(L) : -INFINITY;
}

}  // namespace

namespace kvs {

// Floats of the per-token correction / score array that follows the parts in the workspace.
size_t decode_sparse_score_floats(const kvs_desc* d) {
  return static_cast<size_t>(d->B) * d->Hq * d->n;
}

void launch_sparse_key_corr(const kvs_desc* d, const void* q, const kvs_cache* c, float* cs, hipStream_t s) {
  hipLaunchKernelGGL(sparse_key_corr_kernel, dim3(d->B * d->Hq * ((d->n + 128 * kKeyIlp - 1) / (128 * kKeyIlp))), dim3(128), 0, s,
                     static_cast<const uint16_t*>(q), c->k_params, c->k_rowptr, c->k_col,
                     static_cast<const uint16_t*>(c->k_val), static_cast<int>(d->sparse_cap), d->n, d->group, d->Hq, d->Hkv, cs);
}

void launch_decode_finish_sparse(const kvs_desc* d, const DecodeGeometry& geo, const void* q, const kvs_cache* c,
                                 const float* ws, const float* cs, void* out, float* lse, hipStream_t s) {
  const size_t lds = static_cast<size_t>(kFinishThreads / 128 * kValIlp) * 128 * (1 + 128 / d->group) * 4;
  hipLaunchKernelGGL(decode_finish_sparse_kernel, dim3(d->B * d->Hq), dim3(kFinishThreads), lds, s,
                     static_cast<const uint16_t*>(q), ws, geo.splits, d->Hq, d->Hkv, d->n, d->group, d->keep_cap,
                     static_cast<const uint16_t*>(c->keep_k), static_cast<const uint16_t*>(c->keep_v), c->keep_cnt,
                     c->v_params, c->v_rowptr, c->v_col, static_cast<const uint16_t*>(c->v_val),
                     static_cast<int>(d->sparse_cap), cs, static_cast<uint16_t*>(out), lse);
}

}  // namespace kvs

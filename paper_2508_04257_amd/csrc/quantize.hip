// kvs_quantize_kv and the calls built on it: sink-preserving low-bit KV-cache quantisation
// (paper, Appendix C equations for Q(X), scale and zero; Algorithm 1's two quantise steps;
// Section 4.1 for the per-channel Key / per-token Value grouping).  The quantise kernels are in
// quantize_fast.hip, the threshold / CSR kernels of the dense-and-sparse variant in sparse.hip;
// this file holds the entry points, the driver they share, and the small kernels around a growing
// cache (keep index over a prefix, kept rows of a span, mask and residual-row copies).
#include "kvs_device.h"

namespace {

using kvs::Fmt;

// ---------------------------------------------------------------------------------------------
// Keep rows: index list of the kept tokens (ascending) and bit-exact copies of their rows.
// ---------------------------------------------------------------------------------------------
constexpr int kIndexThreads = 1024;

// n tokens are indexed; both masks have `stride` bytes per sequence.  They may be the same array
// (a growing cache normalises its own mask in place), hence no __restrict__ on the two.
__global__ __launch_bounds__(kIndexThreads) void keep_index_kernel(
    const uint8_t* keep_mask, int n, int stride, int cap, int32_t* __restrict__ keep_idx,
    int32_t* __restrict__ keep_cnt, uint8_t* mask_copy, int32_t* __restrict__ status) {
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

}  // namespace

// Shared by the three quantising entry points: the quantise kernels over one span, then - unless
// the lean kernels did it themselves - the keep index over the first n_index cache tokens and the
// kept rows that lie in the span.
static void quantize_span(const kvs_desc* desc, const kvs::QuantSpan& sp, bool whole, const void* K, const void* V,
                          const uint8_t* mask, const uint8_t* index_mask, int n_index, const kvs_cache* out,
                          void* workspace, hipStream_t s, const uint32_t* static_k = nullptr,
                          const uint32_t* static_v = nullptr, const uint32_t* given_tau = nullptr) {
  kvs::SparsePlan plan{};
  const bool sparse = desc->sparse_frac > 0.0f;
  if (sparse) {                                        // thresholds of K and V first (plan.tau): searched, or the caller's
    plan = kvs::sparse_plan(desc, static_cast<uint32_t*>(workspace) + kvs::workspace_counter_words(desc));   // behind decode's counters
    if (given_tau) kvs::sparse_given_thresholds(plan, given_tau, out, s);
    else kvs::sparse_thresholds(desc, plan, K, V, mask, out, s);
  }
  kvs::launch_quantize_fast(desc, sp, whole, K, V, mask, out, static_k, static_v, sparse ? &plan : nullptr, s);
  if (sparse) kvs::sparse_build_csr(desc, plan, out, s);
  if (whole) return;                                   // the quantise kernels wrote index and kept rows
  hipLaunchKernelGGL(keep_index_kernel, dim3(desc->B), dim3(kIndexThreads), 0, s, index_mask, n_index,
                     sp.n_cap, desc->keep_cap, out->keep_idx, out->keep_cnt, out->keep_mask,
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

// Everything kvs_quantize_kv can refuse on the host, without launching anything.
kvs_status kvs::check_quantize_call(const kvs_desc* desc, const void* K, const void* V, const uint8_t* keep_mask,
                                    const kvs_cache* out, const void* workspace) {
  const kvs_status st = check_quantize_args(desc, out);
  if (st != KVS_OK) return st;
  if (!K || !V || !keep_mask) return KVS_ERR_INVALID;
  const bool sparse = desc->sparse_frac > 0.0f;
  if (sparse && (!workspace || !out->k_rowptr || !out->k_col || !out->k_val || !out->v_rowptr ||
                 !out->v_col || !out->v_val))
    return KVS_ERR_INVALID;
  return KVS_OK;
}

extern "C" kvs_status kvs_quantize_kv(const kvs_desc* desc, const void* K, const void* V,
                                       const uint8_t* keep_mask, const kvs_cache* out,
                                       void* workspace, void* stream) {
  const kvs_status st = kvs::check_quantize_call(desc, K, V, keep_mask, out, workspace);
  if (st != KVS_OK) return st;
  hipStream_t s = static_cast<hipStream_t>(stream);
  quantize_span(desc, kvs::whole_span(desc), true, K, V, keep_mask, keep_mask, desc->n, out, workspace, s);
  return hipGetLastError() == hipSuccess ? KVS_OK : KVS_ERR_DEVICE;
}

// Outlier thresholds apart from the quantise call (the dense-and-sparse setting of the paper's
// Section 5.1 is KVQuant's, whose outlier thresholds are fixed on calibration data before
// inference): the search alone, and the quantise call with the thresholds given.
extern "C" kvs_status kvs_outlier_thresholds(const kvs_desc* desc, const void* K, const void* V,
                                              const uint8_t* keep_mask, uint32_t* tau, void* workspace,
                                              void* stream) {
  const kvs_status st = kvs::validate_desc(desc);
  if (st != KVS_OK) return st;
  if (!(desc->sparse_frac > 0.0f)) return KVS_ERR_INVALID;
  if (!K || !V || !keep_mask || !tau || !workspace) return KVS_ERR_INVALID;
  hipStream_t s = static_cast<hipStream_t>(stream);
  const kvs::SparsePlan plan =
      kvs::sparse_plan(desc, static_cast<uint32_t*>(workspace) + kvs::workspace_counter_words(desc));
  kvs::sparse_thresholds(desc, plan, K, V, keep_mask, nullptr, s);
  kvs::sparse_export_thresholds(plan, tau, s);
  return hipGetLastError() == hipSuccess ? KVS_OK : KVS_ERR_DEVICE;
}

extern "C" kvs_status kvs_quantize_kv_thresholds(const kvs_desc* desc, const void* K, const void* V,
                                                  const uint8_t* keep_mask, const uint32_t* tau,
                                                  const kvs_cache* out, void* workspace, void* stream) {
  const kvs_status st = kvs::check_quantize_call(desc, K, V, keep_mask, out, workspace);
  if (st != KVS_OK) return st;
  if (!(desc->sparse_frac > 0.0f) || !tau) return KVS_ERR_INVALID;
  hipStream_t s = static_cast<hipStream_t>(stream);
  quantize_span(desc, kvs::whole_span(desc), true, K, V, keep_mask, keep_mask, desc->n, out, workspace, s, nullptr,
                nullptr, tau);
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

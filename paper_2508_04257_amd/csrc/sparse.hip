// Dense-and-sparse support for kvs_quantize_kv (paper, Section 5.1: the largest-magnitude
// entries are isolated in 16 bit - 16-bit value + 16-bit index each, the cost the average-bits
// column of Table 2 shows - and only the rest is quantised).
//
// Threshold: an exact histogram of the 15-bit fp16 magnitude pattern over all entries on
// non-kept tokens (one workgroup per compute unit, the whole 32768-bin histogram in 128 KB of
// LDS), then a suffix scan picks the magnitude tau at which the descending cumulative count
// first reaches ceil(f * count).  Integer counting only, so the result is order-free.
// CSR: the quantise kernels count the isolated entries per row and park them, block by block and
// already in their final relative order, in a staging list; an in-place scan turns the counts
// into row pointers and one small kernel moves every block's run to its place.  K and V are
// read twice in all (histogram, quantise).
#include "kvs_device.h"
#include "sparse_emit.h"

namespace {

constexpr int kHistThreads = 1024;
constexpr int kBins = 32768;

__global__ void fill_u32_kernel(uint32_t* __restrict__ p, size_t count, uint32_t value) {
  for (size_t i = blockIdx.x * static_cast<size_t>(blockDim.x) + threadIdx.x; i < count;
       i += static_cast<size_t>(gridDim.x) * blockDim.x)
    p[i] = value;
}

// Division of a row index (below 2^31) by a run-time constant as a multiply and a shift; the
// general 64-bit division the index arithmetic would otherwise compile to costs over a hundred
// instructions per load and was what bounded the histogram pass.
struct FastDiv {
  uint32_t d, m;
  int l;
};
FastDiv make_fastdiv(uint32_t d) {
  int l = 0;
  while ((1u << l) < d) ++l;
  const unsigned long long m = ((1ull << 32) * ((1ull << l) - d)) / d + 1;
  return FastDiv{d, static_cast<uint32_t>(m), l};
}
__device__ inline uint32_t fastdiv(uint32_t x, const FastDiv& f) { return (__umulhi(f.m, x) + x) >> f.l; }

// X: fp16 [B*Hkv*n, 128] viewed as uint4 (8 values); entries on kept tokens are skipped.
//
// Only the top of the histogram decides tau, and one LDS atomic per element is what this pass
// costs, so the bulk of the elements is not counted at all: a workgroup counts everything in its
// first kSampleSteps grid-stride steps (a sample spread over the whole tensor), takes from that
// sample the magnitude l0 above which about kSampleMargin * frac of the entries lie, and from
// then on counts only magnitudes >= l0.  Bins >= the largest l0 of any workgroup are exact in
// the merged histogram; the number of entries is counted separately.  If the threshold turns out
// to lie below that (a sample that misjudged the tail), ctrl[kNeedFull] is raised and the full
// histogram - the same kernel with full != 0 - is taken after all; it returns at once otherwise.
constexpr int kSampleSteps = 8;
constexpr float kSampleMargin = 3.0f;
enum { kCtrlCount = 0, kCtrlL0 = 1, kNeedFull = 2, kCtrlWords = 4 };   // per tensor, in the control block

__global__ __launch_bounds__(kHistThreads) void sparse_hist_kernel(
    const uint4* __restrict__ X, const uint8_t* __restrict__ keep_mask, size_t rows, FastDiv by_n, FastDiv by_heads,
    float frac, int full, uint32_t* __restrict__ hist, uint32_t* __restrict__ ctrl) {
  __shared__ uint32_t h[kBins];
  __shared__ unsigned long long part[kHistThreads];
  __shared__ uint32_t l0_s, seen_s;
  if (full && ctrl[kNeedFull] == 0) return;             // the bounded histogram was enough
  for (int i = threadIdx.x; i < kBins; i += kHistThreads) h[i] = 0;
  if (threadIdx.x == 0) { l0_s = 0; seen_s = 0; }
  __syncthreads();
  const int tid = threadIdx.x;
  const size_t units = rows * 16;                       // 16-byte units
  const size_t stride = static_cast<size_t>(gridDim.x) * kHistThreads;
  uint32_t seen = 0;                                    // units of non-kept tokens this lane met
  uint32_t l0 = 0;
  constexpr int U = 4;                                  // 16-byte loads in flight per lane
  const int steps = static_cast<int>((units + stride * U - 1) / (stride * U));   // the same for every lane
  for (int step = 0; step < steps; ++step) {
    if (!full && step == kSampleSteps / U) {
      // ---- lower bound from the sample: suffix sums over 1024 runs of 32 bins -----------------
      __syncthreads();
      unsigned long long own = 0;
      for (int j = 0; j < 32; ++j) own += h[32 * tid + j];
      part[tid] = own;
      __syncthreads();
      for (int o = 1; o < kHistThreads; o <<= 1) {
        const unsigned long long add = tid + o < kHistThreads ? part[tid + o] : 0ull;
        __syncthreads();
        part[tid] += add;
        __syncthreads();
      }
      const unsigned long long total = part[0], above = part[tid] - own;
      const unsigned long long want = static_cast<unsigned long long>(
          fminf(kSampleMargin * frac, 1.0f) * static_cast<float>(total)) + 1;
      if (want > total) { if (tid == 0) l0_s = 0; }
      else if (above < want && above + own >= want) {
        unsigned long long cum = above;
        for (int j = 31; j >= 0; --j) {
          cum += h[32 * tid + j];
          if (cum >= want) { l0_s = static_cast<uint32_t>(32 * tid + j); break; }
        }
      }
      __syncthreads();
      l0 = l0_s;
    }
    uint4 v[U];
    bool use[U];
#pragma unroll
    for (int k = 0; k < U; ++k) {
      // step-major, then workgroup, then the U loads of a step: a workgroup's loads of one step are contiguous
      const size_t u = ((static_cast<size_t>(step) * gridDim.x + blockIdx.x) * U + k) * kHistThreads + tid;
      use[k] = u < units;
      const size_t uc = use[k] ? u : 0;
      const uint32_t row = static_cast<uint32_t>(uc >> 4);      // (b * Hkv + h) * n + t, below 2^30
      const uint32_t bh = fastdiv(row, by_n);
      const uint32_t t = row - bh * by_n.d;
      const uint32_t b = fastdiv(bh, by_heads);
      use[k] = use[k] && keep_mask[static_cast<size_t>(b) * by_n.d + t] == 0;
      v[k] = X[uc];
    }
    const uint32_t l0_2 = l0 | (l0 << 16);
#pragma unroll
    for (int k = 0; k < U; ++k) {
      if (!use[k]) continue;
      ++seen;
      const uint32_t w[4] = {v[k].x, v[k].y, v[k].z, v[k].w};
      if (l0 == 0) {                                   // (uniform) everything is counted
#pragma unroll
        for (int j = 0; j < 4; ++j) {
          atomicAdd(&h[w[j] & 0x7FFFu], 1u);
          atomicAdd(&h[(w[j] >> 16) & 0x7FFFu], 1u);
        }
      } else {
        // Few entries reach the bound: find them with packed arithmetic and walk only those.
        uint32_t m[4];
#pragma unroll
        for (int j = 0; j < 4; ++j) m[j] = kvs::below_mask(w[j], l0_2);
        uint32_t bits = kvs::isolated8(m);
        while (bits) {
          const int j = __builtin_ctz(bits);
          bits &= bits - 1;
          const int q = j >> 1;
          const uint32_t wq = q == 0 ? w[0] : (q == 1 ? w[1] : (q == 2 ? w[2] : w[3]));
          atomicAdd(&h[((j & 1) ? wq >> 16 : wq) & 0x7FFFu], 1u);
        }
      }
    }
  }
  atomicAdd(&seen_s, seen);
  __syncthreads();
  // Only bins at or above this workgroup's own bound can matter (the threshold kernel never looks
  // below the largest bound); the sample's counts in the bins below it are dropped, which spares
  // most of the global atomics.
  const int first_bin = full ? 0 : static_cast<int>(l0_s);
  for (int i = first_bin + tid; i < kBins; i += kHistThreads)
    if (h[i]) atomicAdd(&hist[i], h[i]);
  if (tid == 0) {
    if (!full) {
      atomicAdd(&ctrl[kCtrlCount], seen_s * 8u);
      atomicMax(&ctrl[kCtrlL0], l0_s);
    }
  }
}

// One workgroup per tensor: tau = largest bin t with sum_{bin >= t} hist >= ceil(f * count), where
// count is the number of entries on non-kept tokens.  pass 0 reads the bounded histogram, whose
// bins below ctrl[kCtrlL0] are incomplete: if the walk would have to go below it, nothing is
// written but ctrl[kNeedFull].  pass 1 does the same on the full histogram, if that was raised.
__global__ __launch_bounds__(1024) void sparse_threshold_kernel(const uint32_t* __restrict__ hist_base,
                                                                 uint32_t* __restrict__ ctrl_base, float frac, int pass,
                                                                 uint32_t* __restrict__ tau_out) {
  __shared__ unsigned long long part[1024];
  const uint32_t* hist = hist_base + static_cast<size_t>(blockIdx.x) * kBins;
  uint32_t* ctrl = ctrl_base + blockIdx.x * kCtrlWords;
  if (pass == 1 && ctrl[kNeedFull] == 0) return;
  const uint32_t l0 = pass == 0 ? ctrl[kCtrlL0] : 0u;
  const int tid = threadIdx.x;
  unsigned long long own = 0;
  for (int j = 0; j < 32; ++j) own += hist[32 * tid + j];
  part[tid] = own;
  __syncthreads();
  // suffix sums over threads (1024 values): simple log-step scan in LDS
  for (int o = 1; o < 1024; o <<= 1) {
    const unsigned long long add = tid + o < 1024 ? part[tid + o] : 0ull;
    __syncthreads();
    part[tid] += add;
    __syncthreads();
  }
  const unsigned long long count = ctrl[kCtrlCount];
  const unsigned long long above = part[tid] - own;     // entries in bins of higher threads
  const double md = ceil(static_cast<double>(frac) * static_cast<double>(count));
  const unsigned long long m = md <= 0.0 ? 0ull : static_cast<unsigned long long>(md);
  if (tid == 0 && m == 0) tau_out[blockIdx.x] = 0x8000u;
  if (m > 0 && above < m && above + own >= m) {         // exactly one thread
    unsigned long long cum = above;
    for (int j = 31; j >= 0; --j) {
      cum += hist[32 * tid + j];
      if (cum >= m) {
        const uint32_t bin = static_cast<uint32_t>(32 * tid + j);
        if (bin >= l0) tau_out[blockIdx.x] = bin; else ctrl[kNeedFull] = 1u;
        break;
      }
    }
  }
  if (m > 0 && tid == 0 && part[0] < m) ctrl[kNeedFull] = 1u;   // pass 0 only: the counted part is too small
}

// ---- in-place inclusive scan of int32 counts (three phases, 4096 items per workgroup) -------
constexpr int kScanThreads = 1024;
constexpr int kScanItems = 4;
constexpr int kScanBlock = kScanThreads * kScanItems;

__device__ inline int block_exclusive_scan(int v, int* total) {
  __shared__ int wave_tot[kScanThreads / KVS_WAVE];
  const int lane = threadIdx.x & (KVS_WAVE - 1), wave = threadIdx.x / KVS_WAVE;
  int incl = v;
#pragma unroll
  for (int o = 1; o < KVS_WAVE; o <<= 1) {
    const int up = __shfl_up(incl, o, KVS_WAVE);
    if (lane >= o) incl += up;
  }
  if (lane == KVS_WAVE - 1) wave_tot[wave] = incl;
  __syncthreads();
  int base = 0, all = 0;
  for (int w = 0; w < kScanThreads / KVS_WAVE; ++w) {
    const int t = wave_tot[w];
    base += w < wave ? t : 0;
    all += t;
  }
  __syncthreads();
  *total = all;
  return base + incl - v;
}

__global__ __launch_bounds__(kScanThreads) void scan_reduce_kernel(const int* __restrict__ x, size_t count,
                                                                    int* __restrict__ sums) {
  const size_t base = blockIdx.x * static_cast<size_t>(kScanBlock) + threadIdx.x * kScanItems;
  int v = 0;
  for (int j = 0; j < kScanItems; ++j) v += base + j < count ? x[base + j] : 0;
  int total;
  block_exclusive_scan(v, &total);
  if (threadIdx.x == 0) sums[blockIdx.x] = total;
}

// Exclusive scan of the block sums in place (one workgroup); the grand total is checked against
// the capacity and also left in sums[nblk].
__global__ __launch_bounds__(kScanThreads) void scan_sums_kernel(int* __restrict__ sums, int nblk, long long cap,
                                                                  int32_t* __restrict__ status) {
  __shared__ int carry_s;
  if (threadIdx.x == 0) carry_s = 0;
  __syncthreads();
  for (int i0 = 0; i0 < nblk; i0 += kScanThreads) {
    const int i = i0 + threadIdx.x;
    const int v = i < nblk ? sums[i] : 0;
    int total;
    const int excl = block_exclusive_scan(v, &total);
    const int carry = carry_s;
    if (i < nblk) sums[i] = carry + excl;
    __syncthreads();
    if (threadIdx.x == 0) carry_s = carry + total;
    __syncthreads();
  }
  if (threadIdx.x == 0) {
    sums[nblk] = carry_s;
    if (static_cast<long long>(carry_s) > cap) atomicCAS(status, 0, static_cast<int>(KVS_ERR_CAPACITY));
  }
}

__global__ __launch_bounds__(kScanThreads) void scan_apply_kernel(int* __restrict__ x, size_t count,
                                                                   const int* __restrict__ sums) {
  const size_t base = blockIdx.x * static_cast<size_t>(kScanBlock) + threadIdx.x * kScanItems;
  int item[kScanItems];
  int v = 0;
  for (int j = 0; j < kScanItems; ++j) { item[j] = base + j < count ? x[base + j] : 0; v += item[j]; }
  int total;
  int run = sums[blockIdx.x] + block_exclusive_scan(v, &total);
  for (int j = 0; j < kScanItems; ++j) {
    run += item[j];
    if (base + j < count) x[base + j] = run;
  }
}

// ---- staging list -> CSR ---------------------------------------------------------------------
// One wave per workgroup of the quantise kernel: its run of the staging list, already in final
// order, moves to where the scanned row pointers put the block's first row.  A run that did not
// fit the list (a reported overflow) is replaced by harmless entries.
__global__ __launch_bounds__(KVS_WAVE) void csr_move_kernel(
    const uint32_t* __restrict__ list, const int* __restrict__ block_base, int rows_per_block,
    const int32_t* __restrict__ rowptr, long long cap, long long list_words, uint16_t* __restrict__ col,
    uint16_t* __restrict__ val) {
  const size_t first_row = blockIdx.x * static_cast<size_t>(rows_per_block);
  const long long dst0 = rowptr[first_row];
  const int cnt = static_cast<int>(rowptr[first_row + rows_per_block] - dst0);
  const long long src0 = block_base[blockIdx.x];
  for (int e = threadIdx.x; e < cnt; e += KVS_WAVE) {
    if (dst0 + e < cap) {
      const uint32_t w = src0 + e < list_words ? list[src0 + e] : 0u;
      col[dst0 + e] = static_cast<uint16_t>(w & 0xFFFFu);
      val[dst0 + e] = static_cast<uint16_t>(w >> 16);
    }
  }
}

}  // namespace

namespace kvs {

// Workspace layout in uint32 words: histograms and the control block - thresholds, per-tensor
// control words, the staging counters of both tensors - (zeroed together), scan scratch, the
// per-workgroup run starts, the two staging lists.
constexpr int kCtrlBlock = 256;                  // words: 0-1 tau, 8-15 per-tensor control, 32.. / 128.. staging counters
static_assert(32 + kEmitCounters <= 128 && 128 + kEmitCounters <= kCtrlBlock, "control block layout");
static int key_block_rows(const kvs_desc* d) { return d->group > 64 ? d->group : 64; }

size_t sparse_workspace_words(const kvs_desc* d) {
  const size_t rows = static_cast<size_t>(d->B) * d->Hkv * d->n;
  const size_t nblk = (rows + kScanBlock - 1) / kScanBlock;
  const size_t bases = rows / key_block_rows(d) + rows / KVS_V_TILE;
  return 4 * kBins + kCtrlBlock + 2 * (nblk + 1) + bases + 2 * static_cast<size_t>(emit_list_words(d->sparse_cap));
}

SparsePlan sparse_plan(const kvs_desc* d, void* workspace) {
  SparsePlan p;
  uint32_t* w = static_cast<uint32_t*>(workspace);
  const size_t rows = static_cast<size_t>(d->B) * d->Hkv * d->n;
  p.rows = rows;
  p.nblk = static_cast<int>((rows + kScanBlock - 1) / kScanBlock);
  p.hist = w;                                              // [2][kBins] bounded, then [2][kBins] full
  uint32_t* block = w + 4 * kBins;                         // the control block, zeroed with the histograms
  p.tau = block;
  p.sums_k = reinterpret_cast<int*>(block + kCtrlBlock);
  p.sums_v = p.sums_k + p.nblk + 1;
  p.rows_per_block_k = key_block_rows(d);
  int* bases = p.sums_v + p.nblk + 1;
  uint32_t* lists = reinterpret_cast<uint32_t*>(bases + rows / p.rows_per_block_k + rows / KVS_V_TILE);
  p.emit_k = SparseEmit{lists, reinterpret_cast<int*>(block + 32), bases, d->sparse_cap};
  p.emit_v = SparseEmit{lists + emit_list_words(d->sparse_cap), reinterpret_cast<int*>(block + 128),
                        bases + rows / p.rows_per_block_k, d->sparse_cap};
  return p;
}

void sparse_thresholds(const kvs_desc* d, const SparsePlan& p, const void* K, const void* V,
                       const uint8_t* mask, const kvs_cache* out, hipStream_t s) {
  hipLaunchKernelGGL(fill_u32_kernel, dim3(64), dim3(1024), 0, s, p.hist, static_cast<size_t>(4 * kBins + kCtrlBlock), 0u);
  hipLaunchKernelGGL(fill_u32_kernel, dim3(1), dim3(64), 0, s, reinterpret_cast<uint32_t*>(out->k_rowptr), size_t{1}, 0u);
  hipLaunchKernelGGL(fill_u32_kernel, dim3(1), dim3(64), 0, s, reinterpret_cast<uint32_t*>(out->v_rowptr), size_t{1}, 0u);
  // Two workgroups per compute unit in turn; fewer on small inputs, so that every workgroup still
  // takes several times kSampleSteps grid-stride steps and the bounded count means something.
  const size_t want_grid = p.rows * 16 / (static_cast<size_t>(kHistThreads) * 4 * kSampleSteps);   // >= 4 x the sample
  const int grid = static_cast<int>(want_grid < 1 ? 1 : (want_grid > 512 ? 512 : want_grid));
  uint32_t* ctrl = p.tau + 8;                             // [2][kCtrlWords]
  const void* X[2] = {K, V};
  for (int full = 0; full < 2; ++full) {                  // the second round returns at once unless asked for
    uint32_t* hist = p.hist + full * 2 * kBins;
    for (int t = 0; t < 2; ++t)
      hipLaunchKernelGGL(sparse_hist_kernel, dim3(grid), dim3(kHistThreads), 0, s, static_cast<const uint4*>(X[t]),
                         mask, p.rows, make_fastdiv(static_cast<uint32_t>(d->n)), make_fastdiv(static_cast<uint32_t>(d->Hkv)),
                         d->sparse_frac, full, hist + t * kBins, ctrl + t * kCtrlWords);
    hipLaunchKernelGGL(sparse_threshold_kernel, dim3(2), dim3(1024), 0, s, hist, ctrl, d->sparse_frac, full, p.tau);
  }
}

void sparse_build_csr(const kvs_desc* d, const SparsePlan& p, const kvs_cache* out, hipStream_t s) {
  const long long cap = d->sparse_cap;
  int* xs[2] = {out->k_rowptr + 1, out->v_rowptr + 1};
  int* sums[2] = {p.sums_k, p.sums_v};
  for (int i = 0; i < 2; ++i) {
    hipLaunchKernelGGL(scan_reduce_kernel, dim3(p.nblk), dim3(kScanThreads), 0, s, xs[i], p.rows, sums[i]);
    hipLaunchKernelGGL(scan_sums_kernel, dim3(1), dim3(kScanThreads), 0, s, sums[i], p.nblk, cap, out->status);
    hipLaunchKernelGGL(scan_apply_kernel, dim3(p.nblk), dim3(kScanThreads), 0, s, xs[i], p.rows, sums[i]);
  }
  hipLaunchKernelGGL(csr_move_kernel, dim3(static_cast<unsigned>(p.rows / p.rows_per_block_k)), dim3(KVS_WAVE), 0, s,
                     p.emit_k.list, p.emit_k.block_base, p.rows_per_block_k, out->k_rowptr, cap, emit_list_words(cap), out->k_col,
                     static_cast<uint16_t*>(out->k_val));
  hipLaunchKernelGGL(csr_move_kernel, dim3(static_cast<unsigned>(p.rows / KVS_V_TILE)), dim3(KVS_WAVE), 0, s,
                     p.emit_v.list, p.emit_v.block_base, KVS_V_TILE, out->v_rowptr, cap, emit_list_words(cap), out->v_col,
                     static_cast<uint16_t*>(out->v_val));
}

}  // namespace kvs

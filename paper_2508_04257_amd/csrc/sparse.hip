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

namespace {

constexpr int kHistThreads = 1024;
constexpr int kBins = 32768;

__global__ void fill_u32_kernel(uint32_t* __restrict__ p, size_t count, uint32_t value) {
  for (size_t i = blockIdx.x * static_cast<size_t>(blockDim.x) + threadIdx.x; i < count;
       i += static_cast<size_t>(gridDim.x) * blockDim.x)
    p[i] = value;
}

// X: fp16 [B*Hkv*n, 128] viewed as uint4 (8 values); entries on kept tokens are skipped.
__global__ __launch_bounds__(kHistThreads) void sparse_hist_kernel(
    const uint4* __restrict__ X, const uint8_t* __restrict__ keep_mask, size_t rows, int n, int Hkv,
    uint32_t* __restrict__ hist) {
  __shared__ uint32_t h[kBins];
  for (int i = threadIdx.x; i < kBins; i += kHistThreads) h[i] = 0;
  __syncthreads();
  const size_t units = rows * 16;                       // 16-byte units
  for (size_t u = blockIdx.x * static_cast<size_t>(kHistThreads) + threadIdx.x; u < units;
       u += static_cast<size_t>(gridDim.x) * kHistThreads) {
    const size_t row = u >> 4;
    const size_t b = row / (static_cast<size_t>(Hkv) * n);
    const int t = static_cast<int>(row % n);
    if (keep_mask[b * n + t]) continue;
    const uint4 v = X[u];
    atomicAdd(&h[v.x & 0x7FFFu], 1u); atomicAdd(&h[(v.x >> 16) & 0x7FFFu], 1u);
    atomicAdd(&h[v.y & 0x7FFFu], 1u); atomicAdd(&h[(v.y >> 16) & 0x7FFFu], 1u);
    atomicAdd(&h[v.z & 0x7FFFu], 1u); atomicAdd(&h[(v.z >> 16) & 0x7FFFu], 1u);
    atomicAdd(&h[v.w & 0x7FFFu], 1u); atomicAdd(&h[(v.w >> 16) & 0x7FFFu], 1u);
  }
  __syncthreads();
  for (int i = threadIdx.x; i < kBins; i += kHistThreads)
    if (h[i]) atomicAdd(&hist[i], h[i]);
}

// One workgroup per tensor: tau = largest bin t with sum_{bin >= t} hist >= ceil(f * count).
__global__ __launch_bounds__(1024) void sparse_threshold_kernel(const uint32_t* __restrict__ hist_base,
                                                                 float frac, uint32_t* __restrict__ tau_out) {
  __shared__ unsigned long long part[1024];
  const uint32_t* hist = hist_base + static_cast<size_t>(blockIdx.x) * kBins;
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
  const unsigned long long count = part[0];
  const unsigned long long above = part[tid] - own;     // entries in bins of higher threads
  const double md = ceil(static_cast<double>(frac) * static_cast<double>(count));
  const unsigned long long m = md <= 0.0 ? 0ull : static_cast<unsigned long long>(md);
  if (tid == 0 && m == 0) tau_out[blockIdx.x] = 0x8000u;
  if (m > 0 && above < m && above + own >= m) {
    unsigned long long cum = above;
    for (int j = 31; j >= 0; --j) {
      cum += hist[32 * tid + j];
      if (cum >= m) { tau_out[blockIdx.x] = static_cast<uint32_t>(32 * tid + j); break; }
    }
  }
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
    const int32_t* __restrict__ rowptr, long long cap, uint16_t* __restrict__ col, uint16_t* __restrict__ val) {
  const size_t first_row = blockIdx.x * static_cast<size_t>(rows_per_block);
  const long long dst0 = rowptr[first_row];
  const int cnt = static_cast<int>(rowptr[first_row + rows_per_block] - dst0);
  const long long src0 = block_base[blockIdx.x];
  for (int e = threadIdx.x; e < cnt; e += KVS_WAVE) {
    if (dst0 + e < cap) {
      const uint32_t w = src0 + e < cap ? list[src0 + e] : 0u;
      col[dst0 + e] = static_cast<uint16_t>(w & 0xFFFFu);
      val[dst0 + e] = static_cast<uint16_t>(w >> 16);
    }
  }
}

}  // namespace

namespace kvs {

// Workspace layout in uint32 words: histograms, thresholds and the two staging counters (zeroed
// together), scan scratch, the per-workgroup run starts, the two staging lists.
static int key_block_rows(const kvs_desc* d) { return d->group > 64 ? d->group : 64; }

size_t sparse_workspace_words(const kvs_desc* d) {
  const size_t rows = static_cast<size_t>(d->B) * d->Hkv * d->n;
  const size_t nblk = (rows + kScanBlock - 1) / kScanBlock;
  const size_t bases = rows / key_block_rows(d) + rows / KVS_V_TILE;
  return 2 * kBins + 64 + 2 * (nblk + 1) + bases + 2 * static_cast<size_t>(d->sparse_cap);
}

SparsePlan sparse_plan(const kvs_desc* d, void* workspace) {
  SparsePlan p;
  uint32_t* w = static_cast<uint32_t*>(workspace);
  const size_t rows = static_cast<size_t>(d->B) * d->Hkv * d->n;
  p.rows = rows;
  p.nblk = static_cast<int>((rows + kScanBlock - 1) / kScanBlock);
  p.hist = w;
  p.tau = w + 2 * kBins;                                   // words 0, 1 of a 64-word block
  p.sums_k = reinterpret_cast<int*>(w + 2 * kBins + 64);
  p.sums_v = p.sums_k + p.nblk + 1;
  p.rows_per_block_k = key_block_rows(d);
  int* bases = p.sums_v + p.nblk + 1;
  uint32_t* lists = reinterpret_cast<uint32_t*>(bases + rows / p.rows_per_block_k + rows / KVS_V_TILE);
  p.emit_k = SparseEmit{lists, reinterpret_cast<int*>(w + 2 * kBins + 2), bases, d->sparse_cap};
  p.emit_v = SparseEmit{lists + d->sparse_cap, reinterpret_cast<int*>(w + 2 * kBins + 3),
                        bases + rows / p.rows_per_block_k, d->sparse_cap};
  return p;
}

void sparse_thresholds(const kvs_desc* d, const SparsePlan& p, const void* K, const void* V,
                       const uint8_t* mask, const kvs_cache* out, hipStream_t s) {
  hipLaunchKernelGGL(fill_u32_kernel, dim3(64), dim3(1024), 0, s, p.hist, static_cast<size_t>(2 * kBins + 64), 0u);
  hipLaunchKernelGGL(fill_u32_kernel, dim3(1), dim3(64), 0, s, reinterpret_cast<uint32_t*>(out->k_rowptr), size_t{1}, 0u);
  hipLaunchKernelGGL(fill_u32_kernel, dim3(1), dim3(64), 0, s, reinterpret_cast<uint32_t*>(out->v_rowptr), size_t{1}, 0u);
  const int grid = 512;                                   // two workgroups per compute unit in turn
  hipLaunchKernelGGL(sparse_hist_kernel, dim3(grid), dim3(kHistThreads), 0, s, static_cast<const uint4*>(K), mask,
                     p.rows, d->n, d->Hkv, p.hist);
  hipLaunchKernelGGL(sparse_hist_kernel, dim3(grid), dim3(kHistThreads), 0, s, static_cast<const uint4*>(V), mask,
                     p.rows, d->n, d->Hkv, p.hist + kBins);
  hipLaunchKernelGGL(sparse_threshold_kernel, dim3(2), dim3(1024), 0, s, p.hist, d->sparse_frac, p.tau);
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
                     p.emit_k.list, p.emit_k.block_base, p.rows_per_block_k, out->k_rowptr, cap, out->k_col,
                     static_cast<uint16_t*>(out->k_val));
  hipLaunchKernelGGL(csr_move_kernel, dim3(static_cast<unsigned>(p.rows / KVS_V_TILE)), dim3(KVS_WAVE), 0, s,
                     p.emit_v.list, p.emit_v.block_base, KVS_V_TILE, out->v_rowptr, cap, out->v_col,
                     static_cast<uint16_t*>(out->v_val));
}

}  // namespace kvs

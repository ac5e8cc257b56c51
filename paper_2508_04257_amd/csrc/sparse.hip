// Dense-and-sparse support for kvs_quantize_kv (paper, Section 5.1: the largest-magnitude
// entries are isolated in 16 bit - 16-bit value + 16-bit index each, the cost the average-bits
// column of Table 2 shows - and only the rest is quantised).
//
// Threshold: tau is the fp16 magnitude pattern at which the descending cumulative count over all
// entries on non-kept tokens first reaches ceil(f * count).  A strided sample brackets it, one pass
// over the tensor counts exactly what lies in and above the bracket, and a full 32768-bin
// histogram (128 KB of LDS per workgroup) is the fallback when the bracket missed.  Integer
// counting only, so the result is order-free and the same whichever way it was found.
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

// Threshold of one tensor, X: fp16 [B*Hkv*n, 128] viewed as 16-byte units (8 values); entries on
// kept tokens are skipped everywhere.
//
// Only the top of the histogram decides tau, and an LDS atomic per element is what a full
// histogram costs (besides 128 KB of LDS per workgroup, i.e. one workgroup per compute unit).  So:
//   1. sample:   a full histogram of a strided sample (every stride-th 16 KB block, the block
//                inside each stride picked by a hash so that no token position is favoured);
//   2. bracket:  from the sample, the magnitudes lo / hi that about kMargin * f and f / kMargin
//                of the entries reach; tau is expected in [lo, hi);
//   3. count:    one pass over the whole tensor that counts the entries at or above hi (one
//                number) and, per bin, those in [lo, hi): few entries take the slow path and the
//                fine histogram is small; the kept tokens' entries are taken out again afterwards;
//   4. threshold: the descending cumulative count from hi downwards; if it does not land inside
//                [lo, hi) - a sample that misjudged the tail - ctrl[kNeedFull] is raised, and
//   5. the full histogram of the whole tensor is taken after all (sparse_hist_kernel and pass 1
//      of the threshold kernel; both return at once otherwise).
// Every count is an integer and exact, so tau does not depend on which way it was found.
constexpr float kMargin = 1.25f;
constexpr int kFineBins = 4096;                   // most bins [lo, hi) may span
constexpr int kSampleBlocks = 2048;               // 16 KB blocks a sample aims at (32 MB)
constexpr int kCountThreads = 256;
constexpr int kCountLoads = 4;                    // 16-byte loads per lane and step of the count pass
enum { kCtrlCount = 0, kCtrlLo = 1, kNeedFull = 2, kCtrlHi = 3, kCtrlNHi = 4, kCtrlWords = 8 };   // per tensor

struct TensorPair {
  const uint4* x[2];                              // K, V
};

// Is the token of 16-byte unit u kept?  (row = (b * Hkv + h) * n + t, below 2^30)
__device__ inline bool unit_kept(size_t u, const uint8_t* __restrict__ keep_mask, const FastDiv& by_n, const FastDiv& by_heads) {
  const uint32_t row = static_cast<uint32_t>(u >> 4);
  const uint32_t bh = fastdiv(row, by_n);
  const uint32_t t = row - bh * by_n.d;
  const uint32_t b = fastdiv(bh, by_heads);
  return keep_mask[static_cast<size_t>(b) * by_n.d + t] != 0;
}

// Every element of the units a workgroup is given goes into its LDS histogram (32768 bins).
// grid.y = tensor.  mode 0: the sample (blocks s * stride + hash(s) % stride); mode 1: the whole
// tensor, only if ctrl[kNeedFull] was raised (it then also recounts nothing: the entry count of
// the count pass stands).
__global__ __launch_bounds__(kHistThreads) void sparse_hist_kernel(
    TensorPair X, const uint8_t* __restrict__ keep_mask, size_t rows, FastDiv by_n, FastDiv by_heads,
    int full, uint32_t stride, uint32_t* __restrict__ hist_base, const uint32_t* __restrict__ ctrl_base) {
  __shared__ uint32_t h[kBins];
  const int tensor = blockIdx.y;
  if (full && ctrl_base[tensor * kCtrlWords + kNeedFull] == 0) return;   // the bracket was enough
  const uint4* __restrict__ x = X.x[tensor];
  uint32_t* hist = hist_base + static_cast<size_t>(tensor) * kBins;
  const int tid = threadIdx.x;
  for (int i = tid; i < kBins; i += kHistThreads) h[i] = 0;
  __syncthreads();
  const size_t units = rows * 16;
  const size_t blocks = (units + kHistThreads - 1) / kHistThreads;        // 16 KB blocks of the tensor
  const size_t picks = full ? blocks : (blocks + stride - 1) / stride;    // blocks this launch looks at
  constexpr int U = 4;                                                     // 16-byte loads in flight per lane
  for (size_t s0 = static_cast<size_t>(blockIdx.x) * U; s0 < picks; s0 += static_cast<size_t>(gridDim.x) * U) {
    uint4 v[U];
    bool use[U];
#pragma unroll
    for (int k = 0; k < U; ++k) {
      const size_t pick = s0 + k;
      size_t blk = pick;
      if (!full) blk = pick * stride + (static_cast<uint32_t>(pick) * 2654435761u >> 16) % stride;
      const size_t u = blk * kHistThreads + tid;
      use[k] = pick < picks && u < units;
      const size_t uc = use[k] ? u : 0;
      use[k] = use[k] && !unit_kept(uc, keep_mask, by_n, by_heads);
      v[k] = x[uc];
    }
#pragma unroll
    for (int k = 0; k < U; ++k) {
      if (!use[k]) continue;
      const uint32_t w[4] = {v[k].x, v[k].y, v[k].z, v[k].w};
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        atomicAdd(&h[w[j] & 0x7FFFu], 1u);
        atomicAdd(&h[(w[j] >> 16) & 0x7FFFu], 1u);
      }
    }
  }
  __syncthreads();
  for (int i = tid; i < kBins; i += kHistThreads)
    if (h[i]) atomicAdd(&hist[i], h[i]);
}

// Suffix sums over the 1024 threads of a workgroup (in place), log-step in LDS.
__device__ inline void suffix_scan_1024(unsigned long long* part, int tid) {
  for (int o = 1; o < 1024; o <<= 1) {
    const unsigned long long add = tid + o < 1024 ? part[tid + o] : 0ull;
    __syncthreads();
    part[tid] += add;
    __syncthreads();
  }
}

// One workgroup per tensor: lo / hi from the sample histogram.  lo = the largest bin that at least
// min(1, kMargin f) of the sample reaches (0 if the sample is too small to say), hi = one above
// the largest bin that at least f / kMargin of it reaches; at most kFineBins apart.
__global__ __launch_bounds__(1024) void sparse_bracket_kernel(const uint32_t* __restrict__ hist_base, float frac,
                                                               uint32_t* __restrict__ ctrl_base) {
  __shared__ unsigned long long part[1024];
  __shared__ uint32_t lo_s, hi_s;
  const uint32_t* hist = hist_base + static_cast<size_t>(blockIdx.x) * kBins;
  uint32_t* ctrl = ctrl_base + blockIdx.x * kCtrlWords;
  const int tid = threadIdx.x;
  if (tid == 0) { lo_s = 0; hi_s = kBins; }
  unsigned long long own = 0;
  for (int j = 0; j < 32; ++j) own += hist[32 * tid + j];
  part[tid] = own;
  __syncthreads();
  suffix_scan_1024(part, tid);
  const unsigned long long total = part[0], above = part[tid] - own;
  const float share_lo = fminf(kMargin * frac, 1.0f), share_hi = frac / kMargin;
  const unsigned long long want_lo = static_cast<unsigned long long>(share_lo * static_cast<float>(total)) + 1;
  const unsigned long long want_hi = static_cast<unsigned long long>(share_hi * static_cast<float>(total)) + 1;
  if (want_lo <= total && above < want_lo && above + own >= want_lo) {       // exactly one thread
    unsigned long long cum = above;
    for (int j = 31; j >= 0; --j) {
      cum += hist[32 * tid + j];
      if (cum >= want_lo) { lo_s = static_cast<uint32_t>(32 * tid + j); break; }
    }
  }
  if (want_hi <= total && above < want_hi && above + own >= want_hi) {       // exactly one thread
    unsigned long long cum = above;
    for (int j = 31; j >= 0; --j) {
      cum += hist[32 * tid + j];
      if (cum >= want_hi) { hi_s = static_cast<uint32_t>(32 * tid + j) + 1; break; }
    }
  }
  __syncthreads();
  if (tid == 0) {
    uint32_t lo = lo_s, hi = hi_s;
    if (hi <= lo) hi = lo + 1;
    if (hi - lo > kFineBins) lo = hi - kFineBins;
    ctrl[kCtrlLo] = lo;
    ctrl[kCtrlHi] = hi;
  }
}

// The pass over the whole tensor.  grid.y = tensor.  A workgroup's loads of one step are
// contiguous (4 x 4 KB) and the next step's loads are in flight while a step is counted (every
// load is issued unconditionally, with a clamped address past the end: a load behind a branch
// makes the compiler wait for all of them).  It does not look at the keep mask at all - two
// divisions and a dependent load per 16 bytes - : kept tokens are counted like any other and
// taken out again by sparse_uncount_kept_kernel; integer counts, so the difference is exact.
// The pass then runs at the speed of the loads (5.1 - 5.4 TB/s on a 2 x 1 GB layer).
__global__ __launch_bounds__(kCountThreads) void sparse_count_kernel(
    TensorPair X, size_t rows, uint32_t* __restrict__ fine_base, uint32_t* __restrict__ ctrl_base) {
  __shared__ uint32_t fine[kFineBins];
  __shared__ uint32_t nhi_s;
  const int tensor = blockIdx.y;
  const uint4* __restrict__ x = X.x[tensor];
  uint32_t* ctrl = ctrl_base + tensor * kCtrlWords;
  const int tid = threadIdx.x;
  const uint32_t lo = ctrl[kCtrlLo], hi = ctrl[kCtrlHi];
  for (int i = tid; i < kFineBins; i += kCountThreads) fine[i] = 0;
  if (tid == 0) nhi_s = 0;
  __syncthreads();
  const size_t units = rows * 16;
  constexpr int U = kCountLoads;
  const size_t per_step = static_cast<size_t>(gridDim.x) * U * kCountThreads;
  const int steps = static_cast<int>((units + per_step - 1) / per_step);    // the same for every lane
  // lo == 0 (a sample that could not say anything: tiny inputs) sends every entry down the slow path.
  const uint32_t lo2 = lo | (lo << 16);
  uint32_t nhi = 0;
  uint4 cur[U], nxt[U];
  auto fetch = [&](int step, uint4* v) {
#pragma unroll
    for (int k = 0; k < U; ++k) {
      const size_t u = ((static_cast<size_t>(step) * gridDim.x + blockIdx.x) * U + k) * kCountThreads + tid;
      v[k] = x[u < units ? u : 0];                        // unconditional, so that the waits stay exact; past the end: the
                                                          // first unit again, counted by nobody (see below)
    }
  };
  if (steps > 0) fetch(0, cur);
  for (int step = 0; step < steps; ++step) {
    fetch(step + 1, nxt);                             // (past the last step: clamped addresses, nobody counts them)
#pragma unroll
    for (int k = 0; k < U; ++k) {
      const size_t u = ((static_cast<size_t>(step) * gridDim.x + blockIdx.x) * U + k) * kCountThreads + tid;
      const uint32_t w[4] = {cur[k].x, cur[k].y, cur[k].z, cur[k].w};
      uint32_t bits = 0xFFu;
      if (lo != 0) {
        uint32_t m[4];
#pragma unroll
        for (int j = 0; j < 4; ++j) m[j] = kvs::below_mask(w[j], lo2);
        bits = kvs::isolated8(m);
      }
      if (u >= units) bits = 0;
      while (bits) {                                  // the few entries at or above lo
        const int j = __builtin_ctz(bits);
        bits &= bits - 1;
        const int q = j >> 1;
        const uint32_t wq = q == 0 ? w[0] : (q == 1 ? w[1] : (q == 2 ? w[2] : w[3]));
        const uint32_t pat = ((j & 1) ? wq >> 16 : wq) & 0x7FFFu;
        if (pat >= hi) ++nhi;
        else if (pat >= lo) atomicAdd(&fine[pat - lo], 1u);
      }
    }
#pragma unroll
    for (int k = 0; k < U; ++k) cur[k] = nxt[k];
  }
  atomicAdd(&nhi_s, nhi);
  __syncthreads();
  uint32_t* out = fine_base + static_cast<size_t>(tensor) * kFineBins;
  const int span = static_cast<int>(hi - lo);        // at most kFineBins
  for (int i = tid; i < span; i += kCountThreads)
    if (fine[i]) atomicAdd(&out[i], fine[i]);
  if (tid == 0 && nhi_s) atomicAdd(&ctrl[kCtrlNHi], nhi_s);
}

// Takes the entries of kept tokens out of what sparse_count_kernel counted, and sets the number of
// entries on non-kept tokens.  grid = (B, tensor, groups of four KV heads); a wave scans 256 mask
// bytes at a time and, for every kept token it finds, reads the token's rows of the block's four
// heads (16 lanes per row).  Runs after the count pass on the same stream, so no count goes
// below zero.
__global__ __launch_bounds__(256) void sparse_uncount_kept_kernel(
    TensorPair X, const uint8_t* __restrict__ keep_mask, int n, int Hkv, uint32_t* __restrict__ fine_base,
    uint32_t* __restrict__ ctrl_base) {
  __shared__ uint32_t kept_s, nhi_s;
  const int b = blockIdx.x, tensor = blockIdx.y;
  const uint4* __restrict__ x = X.x[tensor];
  uint32_t* ctrl = ctrl_base + tensor * kCtrlWords;
  uint32_t* fine = fine_base + static_cast<size_t>(tensor) * kFineBins;
  const uint32_t lo = ctrl[kCtrlLo], hi = ctrl[kCtrlHi];
  const int tid = threadIdx.x, lane = tid & (KVS_WAVE - 1), wave = tid / KVS_WAVE;
  const int h = 4 * blockIdx.z + (lane >> 4);
  if (tid == 0) { kept_s = 0; nhi_s = 0; }
  __syncthreads();
  uint32_t kept = 0, nhi = 0;
  const uint8_t* mrow = keep_mask + static_cast<size_t>(b) * n;
  for (int t0 = wave * 256; t0 < n; t0 += 4 * 256) {
    bool k[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int t = t0 + 64 * i + lane;
      k[i] = mrow[t < n ? t : 0] != 0 && t < n;
    }
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      unsigned long long found = __ballot(k[i]);
      kept += static_cast<uint32_t>(__popcll(found));             // (the same in every lane)
      while (found) {                                             // wave-uniform
        const int tk = t0 + 64 * i + __builtin_ctzll(found);
        found &= found - 1;
        if (h >= Hkv) continue;
        const uint4 v = x[((static_cast<size_t>(b) * Hkv + h) * n + tk) * 16 + (lane & 15)];
        const uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
        for (int j = 0; j < 8; ++j) {
          const uint32_t pat = ((j & 1) ? w[j >> 1] >> 16 : w[j >> 1]) & 0x7FFFu;
          if (pat >= hi) ++nhi;
          else if (pat >= lo) atomicSub(&fine[pat - lo], 1u);
        }
      }
    }
  }
  if (lane == 0) atomicAdd(&kept_s, kept);
  atomicAdd(&nhi_s, nhi);
  __syncthreads();
  if (tid == 0) {
    if (blockIdx.z == 0)
      atomicAdd(&ctrl[kCtrlCount], (static_cast<uint32_t>(n) - kept_s) * static_cast<uint32_t>(Hkv) * 128u);
    if (nhi_s) atomicSub(&ctrl[kCtrlNHi], nhi_s);
  }
}

// One workgroup per tensor: tau = largest bin t with sum_{bin >= t} counts >= m = ceil(f * count),
// count = the number of entries on non-kept tokens.
// pass 0: from the count pass - entries at or above hi, then the fine bins downwards.  If m is
// already reached above hi, or not reached down to lo, only ctrl[kNeedFull] is written.
// pass 1: the same walk over the full histogram, if that was raised.
__global__ __launch_bounds__(1024) void sparse_threshold_kernel(const uint32_t* __restrict__ hist_base,
                                                                 const uint32_t* __restrict__ fine_base,
                                                                 uint32_t* __restrict__ ctrl_base, float frac, int pass,
                                                                 uint32_t* __restrict__ tau_out) {
  __shared__ unsigned long long part[1024];
  uint32_t* ctrl = ctrl_base + blockIdx.x * kCtrlWords;
  if (pass == 1 && ctrl[kNeedFull] == 0) return;
  const int tid = threadIdx.x;
  const unsigned long long count = ctrl[kCtrlCount];
  const double md = ceil(static_cast<double>(frac) * static_cast<double>(count));
  const unsigned long long m = md <= 0.0 ? 0ull : static_cast<unsigned long long>(md);
  if (m == 0) {                                        // nothing to isolate
    if (tid == 0) tau_out[blockIdx.x] = 0x8000u;
    return;
  }
  // the bins this pass walks: per thread `per` consecutive ones, `first` = pattern of bin 0
  const uint32_t* bins = pass == 0 ? fine_base + static_cast<size_t>(blockIdx.x) * kFineBins
                                   : hist_base + static_cast<size_t>(blockIdx.x) * kBins;
  const int per = pass == 0 ? kFineBins / 1024 : kBins / 1024;
  const uint32_t first = pass == 0 ? ctrl[kCtrlLo] : 0u;
  const unsigned long long top = pass == 0 ? ctrl[kCtrlNHi] : 0ull;     // entries above every walked bin
  if (pass == 0 && top >= m) {                         // tau lies at or above hi
    if (tid == 0) ctrl[kNeedFull] = 1u;
    return;
  }
  unsigned long long own = 0;
  for (int j = 0; j < per; ++j) own += bins[per * tid + j];
  part[tid] = own;
  __syncthreads();
  suffix_scan_1024(part, tid);
  const unsigned long long above = top + part[tid] - own;       // entries in higher bins
  if (above < m && above + own >= m) {                 // exactly one thread
    unsigned long long cum = above;
    for (int j = per - 1; j >= 0; --j) {
      cum += bins[per * tid + j];
      if (cum >= m) { tau_out[blockIdx.x] = first + static_cast<uint32_t>(per * tid + j); break; }
    }
  }
  if (tid == 0 && top + part[0] < m) ctrl[kNeedFull] = 1u;      // pass 0 only: tau lies below lo
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
    if (base + j < count) __builtin_nontemporal_store(run, &x[base + j]);   // read next by another kernel: not left dirty in the cache
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
      __builtin_nontemporal_store(static_cast<uint16_t>(w & 0xFFFFu), &col[dst0 + e]);
      __builtin_nontemporal_store(static_cast<uint16_t>(w >> 16), &val[dst0 + e]);
    }
  }
}

}  // namespace

namespace kvs {

// Workspace layout in uint32 words: histograms and the control block - thresholds, per-tensor
// control words, the staging counters of both tensors - (zeroed together), scan scratch, the
// per-workgroup run starts, the two staging lists.
constexpr int kCtrlBlock = 256;                  // words: 0-1 tau, 8-23 per-tensor control, 32.. / 128.. staging counters
static_assert(32 + kEmitCounters <= 128 && 128 + kEmitCounters <= kCtrlBlock, "control block layout");
constexpr size_t kHistWords = 4 * kBins + 2 * kFineBins;
static int key_block_rows(const kvs_desc* d) { return d->group > 64 ? d->group : 64; }

size_t sparse_workspace_words(const kvs_desc* d) {
  const size_t rows = static_cast<size_t>(d->B) * d->Hkv * d->n;
  const size_t nblk = (rows + kScanBlock - 1) / kScanBlock;
  const size_t bases = rows / key_block_rows(d) + rows / KVS_V_TILE;
  return kHistWords + kCtrlBlock + 2 * (nblk + 1) + bases + 2 * static_cast<size_t>(emit_list_words(d->sparse_cap));
}

SparsePlan sparse_plan(const kvs_desc* d, void* workspace) {
  SparsePlan p;
  uint32_t* w = static_cast<uint32_t*>(workspace);
  const size_t rows = static_cast<size_t>(d->B) * d->Hkv * d->n;
  p.rows = rows;
  p.nblk = static_cast<int>((rows + kScanBlock - 1) / kScanBlock);
  p.hist = w;                                              // [2][kBins] sample, [2][kBins] full, [2][kFineBins] fine
  uint32_t* block = w + kHistWords;                        // the control block, zeroed with the histograms
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

// Thresholds given by the caller (device words, e.g. what an earlier search left): the control
// block starts from zero as after a search, the two words are taken over, anything above 0x8000
// (the pattern no magnitude reaches) counts as 0x8000.
__global__ void take_thresholds_kernel(const uint32_t* __restrict__ given, uint32_t* __restrict__ tau) {
  if (threadIdx.x < 2) tau[threadIdx.x] = given[threadIdx.x] < 0x8000u ? given[threadIdx.x] : 0x8000u;
}
__global__ void copy_thresholds_kernel(const uint32_t* __restrict__ tau, uint32_t* __restrict__ out) {
  if (threadIdx.x < 2) out[threadIdx.x] = tau[threadIdx.x];
}

static void start_row_pointers(const kvs_cache* out, hipStream_t s) {
  hipLaunchKernelGGL(fill_u32_kernel, dim3(1), dim3(64), 0, s, reinterpret_cast<uint32_t*>(out->k_rowptr), size_t{1}, 0u);
  hipLaunchKernelGGL(fill_u32_kernel, dim3(1), dim3(64), 0, s, reinterpret_cast<uint32_t*>(out->v_rowptr), size_t{1}, 0u);
}

void sparse_given_thresholds(const SparsePlan& p, const uint32_t* given, const kvs_cache* out, hipStream_t s) {
  hipLaunchKernelGGL(fill_u32_kernel, dim3(1), dim3(kCtrlBlock), 0, s, p.tau, static_cast<size_t>(kCtrlBlock), 0u);
  start_row_pointers(out, s);
  hipLaunchKernelGGL(take_thresholds_kernel, dim3(1), dim3(64), 0, s, given, p.tau);
}

void sparse_export_thresholds(const SparsePlan& p, uint32_t* tau_out, hipStream_t s) {
  hipLaunchKernelGGL(copy_thresholds_kernel, dim3(1), dim3(64), 0, s, p.tau, tau_out);
}

// out == nullptr: the search alone (no CSR is going to be built).
void sparse_thresholds(const kvs_desc* d, const SparsePlan& p, const void* K, const void* V,
                       const uint8_t* mask, const kvs_cache* out, hipStream_t s) {
  hipLaunchKernelGGL(fill_u32_kernel, dim3(64), dim3(1024), 0, s, p.hist, static_cast<size_t>(kHistWords + kCtrlBlock), 0u);
  if (out) start_row_pointers(out, s);
  uint32_t* sample = p.hist;                              // [2][kBins]
  uint32_t* full = p.hist + 2 * kBins;                    // [2][kBins]
  uint32_t* fine = p.hist + 4 * kBins;                    // [2][kFineBins]
  uint32_t* ctrl = p.tau + 8;                             // [2][kCtrlWords]
  const TensorPair X{{static_cast<const uint4*>(K), static_cast<const uint4*>(V)}};
  const FastDiv by_n = make_fastdiv(static_cast<uint32_t>(d->n)), by_heads = make_fastdiv(static_cast<uint32_t>(d->Hkv));
  const size_t units = p.rows * 16;
  const size_t blocks = (units + kHistThreads - 1) / kHistThreads;
  const uint32_t stride = static_cast<uint32_t>(blocks / kSampleBlocks < 1 ? 1 : blocks / kSampleBlocks);
  const size_t picks = (blocks + stride - 1) / stride;
  const unsigned sample_grid = static_cast<unsigned>(picks < 4 ? 1 : (picks / 4 > 256 ? 256 : picks / 4));
  hipLaunchKernelGGL(sparse_hist_kernel, dim3(sample_grid, 2), dim3(kHistThreads), 0, s, X, mask, p.rows, by_n, by_heads, 0,
                     stride, sample, ctrl);
  hipLaunchKernelGGL(sparse_bracket_kernel, dim3(2), dim3(1024), 0, s, sample, d->sparse_frac, ctrl);
  // four workgroups per compute unit, each with several steps to pipeline; fewer on small inputs
  const size_t per_wg = static_cast<size_t>(kCountThreads) * kCountLoads * 4;   // units of four steps
  const size_t want = (units + per_wg - 1) / per_wg;
  const unsigned count_grid = static_cast<unsigned>(want < 1 ? 1 : (want > 1024 ? 1024 : want));
  hipLaunchKernelGGL(sparse_count_kernel, dim3(count_grid, 2), dim3(kCountThreads), 0, s, X, p.rows, fine, ctrl);
  hipLaunchKernelGGL(sparse_uncount_kept_kernel, dim3(d->B, 2, (d->Hkv + 3) / 4), dim3(256), 0, s, X, mask, d->n, d->Hkv, fine, ctrl);
  hipLaunchKernelGGL(sparse_threshold_kernel, dim3(2), dim3(1024), 0, s, full, fine, ctrl, d->sparse_frac, 0, p.tau);
  // the full histogram: both launches return at once unless the bracket missed
  const unsigned full_grid = static_cast<unsigned>(blocks < 4 ? 1 : (blocks / 4 > 256 ? 256 : blocks / 4));
  hipLaunchKernelGGL(sparse_hist_kernel, dim3(full_grid, 2), dim3(kHistThreads), 0, s, X, mask, p.rows, by_n, by_heads, 1,
                     1u, full, ctrl);
  hipLaunchKernelGGL(sparse_threshold_kernel, dim3(2), dim3(1024), 0, s, full, fine, ctrl, d->sparse_frac, 1, p.tau);
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

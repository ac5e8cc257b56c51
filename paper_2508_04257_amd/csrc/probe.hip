// Diagnostic: a pure streaming read in the launch shape of the decode kernels (one workgroup of
// eight waves per compute unit, every wave keeping 16 KB of read-once 16-byte loads in flight,
// every workgroup walking a contiguous share of the buffer).  It does no arithmetic worth the
// name, so its duration is what the memory system alone takes for that many bytes: the ceiling
// the benchmark prints next to the decode kernel's own time.
#include "kvs_device.h"

namespace {

typedef uint32_t uint4v __attribute__((ext_vector_type(4)));
constexpr int kProbeThreads = 512;
constexpr int kProbeLoads = 16;                     // 16-byte loads in flight per lane

__global__ __launch_bounds__(kProbeThreads) void probe_stream_read_kernel(const uint4v* __restrict__ src, size_t n16,
                                                                           uint32_t* __restrict__ sink) {
  const size_t per_group = (n16 + gridDim.x - 1) / gridDim.x;
  const size_t begin = blockIdx.x * per_group;
  const size_t end = begin + per_group < n16 ? begin + per_group : n16;
  const int lane = threadIdx.x & (KVS_WAVE - 1), wave = threadIdx.x / KVS_WAVE;
  constexpr size_t kBlock = static_cast<size_t>(KVS_WAVE) * kProbeLoads;      // 16-byte units per wave and step
  uint32_t acc = 0;
  for (size_t base = begin + wave * kBlock; base < end; base += (kProbeThreads / KVS_WAVE) * kBlock) {
    uint4v v[kProbeLoads];
#pragma unroll
    for (int u = 0; u < kProbeLoads; ++u) {
      const size_t i = base + static_cast<size_t>(u) * KVS_WAVE + lane;
      v[u] = i < end ? __builtin_nontemporal_load(src + i) : uint4v{0, 0, 0, 0};
    }
#pragma unroll
    for (int u = 0; u < kProbeLoads; ++u) acc += v[u].x ^ v[u].y ^ v[u].z ^ v[u].w;
  }
  if (acc == 0x9E3779B9u) sink[0] = acc;            // keeps the loads alive; practically never true
}

}  // namespace

extern "C" kvs_status kvs_probe_stream_read(const void* src, size_t bytes, uint32_t* sink, void* stream) {
  if (!src || !sink || bytes < 16 || (reinterpret_cast<uintptr_t>(src) & 15) != 0) return KVS_ERR_INVALID;
  hipLaunchKernelGGL(probe_stream_read_kernel, dim3(256), dim3(kProbeThreads), 0, static_cast<hipStream_t>(stream),
                     static_cast<const uint4v*>(src), bytes / 16, sink);
  return hipGetLastError() == hipSuccess ? KVS_OK : KVS_ERR_DEVICE;
}

// Host-only driver for the sanitizer build of the library (tests/test_host_sanitizers.py): every
// path of the C ABI that runs on the host alone - descriptor validation, buffer sizing, launch
// geometry, and the argument checks that make a call return before anything is launched - under
// AddressSanitizer and UndefinedBehaviorSanitizer.  No call here reaches a kernel launch, so it
// runs without a GPU.  Exit code 0 = every expectation held (the sanitizers abort on their own).
#include <climits>
#include <cstdint>
#include <cstdio>
#include <cstring>
#include <vector>

#include "kvs.h"

static int failures = 0;
#define EXPECT(cond)                                                     \
  do {                                                                   \
    if (!(cond)) { std::printf("FAILED line %d: %s\n", __LINE__, #cond); ++failures; } \
  } while (0)

static kvs_desc desc(int B, int n, int Hq, int Hkv, int bits, int G, int cap, float frac = 0.0f, int64_t scap = 0,
                     int kpt = 0) {
  kvs_desc d;
  std::memset(&d, 0, sizeof d);
  d.B = B; d.n = n; d.Hq = Hq; d.Hkv = Hkv; d.D = 128; d.bits = bits; d.group = G; d.keep_cap = cap;
  d.sparse_frac = frac; d.sparse_cap = scap; d.key_per_token = kpt;
  return d;
}

int main() {
  size_t sizes[KVS_CACHE_FIELDS];
  void* const p = reinterpret_cast<void*>(uintptr_t{4096});   // non-NULL, never dereferenced on the host
  uint8_t* const pm = static_cast<uint8_t*>(p);

  // ---- every supported shape: sizes are consistent, nothing overflows -------------------------
  const int bits_all[] = {2, 3, 4, 8}, groups[] = {32, 64, 128}, reps[] = {1, 2, 4, 8};
  for (int bits : bits_all)
    for (int G : groups)
      for (int rep : reps)
        for (int kpt = 0; kpt < 2; ++kpt)
          for (int n : {128, 4096, 131072}) {
            const kvs_desc d = desc(3, n, 8 * rep, 8, bits, G, 7, 0.0f, 0, kpt);
            EXPECT(kvs_cache_bytes(&d, sizes) == KVS_OK);
            for (size_t s : sizes) EXPECT(s % 16 == 0);
            EXPECT(sizes[0] == sizes[1]);
            EXPECT(kvs_decode_splits(&d) >= 1 && kvs_decode_splits(&d) <= n / 128);
            EXPECT(kvs_workspace_zero_bytes(&d) >= size_t{3} * 8 * 4 && kvs_workspace_zero_bytes(&d) % 256 == 0);
            EXPECT(kvs_workspace_bytes(&d) > kvs_workspace_zero_bytes(&d));
            EXPECT(kvs_calibration_bytes(&d) == size_t{4} * 8 * 128 * 4);
          }
  // dense-and-sparse sizing, small and at the largest capacities the descriptor admits
  for (int64_t cap : {int64_t{1}, int64_t{1} << 20, (int64_t{1} << 31) - 32769}) {
    const kvs_desc d = desc(32, 4096, 32, 32, 3, 128, 8, 0.01f, cap);
    EXPECT(kvs_cache_bytes(&d, sizes) == KVS_OK);
    EXPECT(sizes[10] >= static_cast<size_t>(cap + 4) * 2);      // four entries of padding behind the capacity
    EXPECT(kvs_workspace_bytes(&d) > kvs_workspace_zero_bytes(&d));
  }
  {
    const kvs_desc d = desc(32, 4096, 32, 32, 3, 128, 8, 0.01f, (int64_t{1} << 31) - 32768);
    EXPECT(kvs_cache_bytes(&d, sizes) == KVS_ERR_UNSUPPORTED);
  }
  // the largest row count that passes validation, and the first that does not
  {
    kvs_desc d = desc(1 << 8, 1 << 13, 1 << 8, 1 << 8, 2, 32, 0);          // 2^29 rows
    EXPECT(kvs_cache_bytes(&d, sizes) == KVS_OK);
    EXPECT(kvs_workspace_bytes(&d) > 0);
    d.B = 1 << 9;                                                           // 2^30 rows
    EXPECT(kvs_cache_bytes(&d, sizes) == KVS_ERR_UNSUPPORTED);
    EXPECT(kvs_workspace_bytes(&d) == 0 && kvs_decode_splits(&d) == 0 && kvs_workspace_zero_bytes(&d) == 0);
  }
  // ---- descriptors that must be refused, extreme values included --------------------------------
  {
    kvs_desc d = desc(INT_MAX, INT_MAX - 127, INT_MAX, INT_MAX, 4, 128, INT_MAX);
    EXPECT(kvs_cache_bytes(&d, sizes) != KVS_OK);
    EXPECT(kvs_workspace_bytes(&d) == 0);
    d = desc(2, 1024, 32, 32, 4, 128, 2);
    d.D = 64;  EXPECT(kvs_cache_bytes(&d, sizes) == KVS_ERR_UNSUPPORTED);
    d = desc(2, 1000, 32, 32, 4, 128, 2);  EXPECT(kvs_cache_bytes(&d, sizes) == KVS_ERR_UNSUPPORTED);
    d = desc(2, 1024, 32, 5, 4, 128, 2);   EXPECT(kvs_cache_bytes(&d, sizes) == KVS_ERR_INVALID);
    d = desc(2, 1024, 32, 32, 5, 128, 2);  EXPECT(kvs_cache_bytes(&d, sizes) == KVS_ERR_UNSUPPORTED);
    d = desc(2, 1024, 32, 32, 4, 16, 2);   EXPECT(kvs_cache_bytes(&d, sizes) == KVS_ERR_UNSUPPORTED);
    d = desc(2, 1024, 32, 32, 4, 128, -1); EXPECT(kvs_cache_bytes(&d, sizes) == KVS_ERR_INVALID);
    d = desc(0, 1024, 32, 32, 4, 128, 2);  EXPECT(kvs_cache_bytes(&d, sizes) == KVS_ERR_INVALID);
    d = desc(2, 1024, 32, 32, 4, 128, 2, 1.5f, 10);  EXPECT(kvs_cache_bytes(&d, sizes) == KVS_ERR_INVALID);
    d = desc(2, 1024, 32, 32, 4, 128, 2, 0.01f, 0);  EXPECT(kvs_cache_bytes(&d, sizes) == KVS_ERR_INVALID);
    d = desc(2, 1024, 32, 32, 8, 128, 2, 0.01f, 10); EXPECT(kvs_cache_bytes(&d, sizes) == KVS_ERR_UNSUPPORTED);
    d = desc(2, 1024, 32, 32, 4, 128, 2, 0.0f, 0, 2); EXPECT(kvs_cache_bytes(&d, sizes) == KVS_ERR_INVALID);
    EXPECT(kvs_cache_bytes(nullptr, sizes) == KVS_ERR_INVALID);
    d = desc(2, 1024, 32, 32, 4, 128, 2);
    EXPECT(kvs_cache_bytes(&d, nullptr) == KVS_ERR_INVALID);
  }
  // ---- calls that must return before launching ---------------------------------------------------
  {
    const kvs_desc d = desc(2, 1024, 32, 32, 4, 128, 4);
    kvs_cache none;
    std::memset(&none, 0, sizeof none);
    kvs_cache full;
    void** fields = reinterpret_cast<void**>(&full);
    for (int i = 0; i < KVS_CACHE_FIELDS; ++i) fields[i] = p;
    const int32_t ch_ok[1] = {7}, ch_bad[1] = {5000};
    EXPECT(kvs_quantize_kv(&d, nullptr, p, pm, &full, nullptr, nullptr) == KVS_ERR_INVALID);
    EXPECT(kvs_quantize_kv(&d, p, p, pm, &none, nullptr, nullptr) == KVS_ERR_INVALID);
    EXPECT(kvs_quantize_kv(nullptr, p, p, pm, &full, nullptr, nullptr) == KVS_ERR_INVALID);
    {
      const kvs_desc sp = desc(2, 1024, 32, 32, 3, 128, 2, 0.01f, 4096);
      uint32_t* tau = reinterpret_cast<uint32_t*>(p);
      EXPECT(kvs_outlier_thresholds(&d, p, p, pm, tau, p, nullptr) == KVS_ERR_INVALID);          // a dense descriptor
      EXPECT(kvs_outlier_thresholds(&sp, p, p, pm, nullptr, p, nullptr) == KVS_ERR_INVALID);
      EXPECT(kvs_outlier_thresholds(&sp, p, p, pm, tau, nullptr, nullptr) == KVS_ERR_INVALID);
      EXPECT(kvs_quantize_kv_thresholds(&d, p, p, pm, tau, &full, p, nullptr) == KVS_ERR_INVALID);
      EXPECT(kvs_quantize_kv_thresholds(&sp, p, p, pm, nullptr, &full, p, nullptr) == KVS_ERR_INVALID);
      EXPECT(kvs_quantize_kv_thresholds(&sp, p, p, pm, tau, &none, p, nullptr) == KVS_ERR_INVALID);
      EXPECT(kvs_quantize_kv_thresholds(&sp, p, p, pm, tau, &full, nullptr, nullptr) == KVS_ERR_INVALID);
    }
    EXPECT(kvs_decode_attn(&d, p, &full, p, nullptr, nullptr, nullptr) == KVS_ERR_INVALID);     // no workspace
    EXPECT(kvs_decode_attn(&d, p, &none, p, nullptr, p, nullptr) == KVS_ERR_INVALID);
    EXPECT(kvs_decode_attn_noalloc(&d, nullptr, &full, p, nullptr, nullptr) == KVS_ERR_INVALID);
    {
      const kvs_desc big = desc(128, 1024, 64, 64, 4, 128, 8);           // 8192 output rows, two parts each
      EXPECT(kvs_decode_attn_noalloc(&big, p, &full, p, nullptr, nullptr) == KVS_ERR_SCRATCH);
    }
    EXPECT(kvs_predict_sinks(p, 1, 128, 4096, ch_bad, 1, 2, 0, static_cast<int32_t*>(p), static_cast<uint8_t*>(p), nullptr, nullptr) == KVS_ERR_INVALID);
    EXPECT(kvs_predict_sinks(p, 1, 128, 4096, ch_ok, 1, 200, 0, static_cast<int32_t*>(p), static_cast<uint8_t*>(p), nullptr, nullptr) == KVS_ERR_INVALID);
    EXPECT(kvs_predict_sinks(p, 1, 1 << 20, 4096, ch_ok, 1, 2, 0, static_cast<int32_t*>(p), static_cast<uint8_t*>(p), nullptr, nullptr) == KVS_ERR_UNSUPPORTED);
    {
      const int32_t nine[9] = {1, 2, 3, 4, 5, 6, 7, 8, 9};              // one more channel than a call takes
      EXPECT(kvs_predict_sinks(p, 1, 128, 4096, nine, 9, 2, 0, static_cast<int32_t*>(p), pm, nullptr, nullptr) == KVS_ERR_UNSUPPORTED);
    }
    EXPECT(kvs_predict_workspace_bytes(4, 32768, 8) == size_t{4} * 8 * 8 * 4);
    EXPECT(kvs_quantize_prefix(&d, p, p, static_cast<uint8_t*>(p), 1025, &full, nullptr, nullptr) == KVS_ERR_INVALID);
    EXPECT(kvs_quantize_prefix(&d, p, p, static_cast<uint8_t*>(p), -1, &full, nullptr, nullptr) == KVS_ERR_INVALID);
    EXPECT(kvs_append_kv(&d, p, p, 1024, &full, nullptr, nullptr) == KVS_ERR_INVALID);
    EXPECT(kvs_decode_attn_n(&d, p, &full, 0, p, nullptr, p, nullptr) == KVS_ERR_INVALID);
    EXPECT(kvs_decode_attn_n(&d, p, &full, 1025, p, nullptr, p, nullptr) == KVS_ERR_INVALID);
    EXPECT(kvs_calibrate_reset(&d, nullptr, nullptr) == KVS_ERR_INVALID);
    EXPECT(kvs_calibrate(&d, p, p, static_cast<uint8_t*>(p), nullptr, nullptr) == KVS_ERR_INVALID);
    EXPECT(kvs_static_params(&d, p, nullptr, static_cast<uint32_t*>(p), nullptr) == KVS_ERR_INVALID);
    EXPECT(kvs_quantize_kv_static(&d, p, p, static_cast<uint8_t*>(p), nullptr, static_cast<uint32_t*>(p), &full, nullptr, nullptr) == KVS_ERR_INVALID);
    EXPECT(kvs_quant_error(&d, p, p, &full, nullptr, p, nullptr) == KVS_ERR_INVALID);
    EXPECT(kvs_probe_stream_read(nullptr, 1024, static_cast<uint32_t*>(p), nullptr) == KVS_ERR_INVALID);
    EXPECT(kvs_probe_stream_read(reinterpret_cast<void*>(uintptr_t{4100}), 1024, static_cast<uint32_t*>(p), nullptr) == KVS_ERR_INVALID);
    // kvs_prefill_layers walks host arrays of layer pointers and cache structs
    std::vector<const void*> Ks(5, p), Vs(5, p);
    std::vector<kvs_cache> caches(5, full);
    auto prefill = [&](int L, int le, int k, int first_n) {
      return kvs_prefill_layers(&d, L, le, Ks.data(), Vs.data(), p, 64, ch_ok, 1, k, first_n, static_cast<int32_t*>(p),
                                static_cast<uint8_t*>(p), static_cast<uint8_t*>(p), caches.data(), nullptr, nullptr, nullptr);
    };
    EXPECT(prefill(0, 0, 2, 0) == KVS_ERR_INVALID);
    EXPECT(prefill(5, 6, 2, 0) == KVS_ERR_INVALID);
    EXPECT(prefill(5, 2, 4, 1) == KVS_ERR_INVALID);                  // five kept rows, room for four
    Ks[4] = nullptr;
    EXPECT(prefill(5, 2, 2, 0) == KVS_ERR_INVALID);                  // found at the last layer, before any launch
    Ks[4] = p;
    caches[4] = none;
    EXPECT(prefill(5, 2, 2, 0) == KVS_ERR_INVALID);
  }
  for (int s = 0; s <= 6; ++s) EXPECT(kvs_status_string(static_cast<kvs_status>(s)) != nullptr);
  EXPECT(kvs_version() >= 100);
  std::printf(failures ? "%d expectation(s) failed\n" : "host checks passed (%d failures)\n", failures);
  return failures ? 1 : 0;
}

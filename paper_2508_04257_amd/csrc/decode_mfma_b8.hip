// Matrix-core decode kernels for 8-bit caches (all group sizes); see decode_mfma_impl.h.
#include "decode_mfma_impl.h"

namespace kvs {

void launch_decode_mfma_b8(const kvs_desc* d, const DecodeGeometry& geo, const void* q, const kvs_cache* c,
                            void* out, float* lse, float* ws, int* arrive, int n_used, const float* extra, hipStream_t s) {
  kvs_mfma::launch_bits<8>(d, geo, q, c, out, lse, ws, arrive, n_used, extra, s);
}

}  // namespace kvs

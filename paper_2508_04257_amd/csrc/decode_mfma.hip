// Dispatch to the matrix-core decode kernels (decode_mfma_impl.h, one translation unit per
// bit width) and the shapes they are instantiated for.
#include "kvs_device.h"

namespace kvs {

void launch_decode_mfma_b2(const kvs_desc*, const DecodeGeometry&, const void*, const kvs_cache*, void*, float*, float*, int*, int, const float*, hipStream_t);
void launch_decode_mfma_b3(const kvs_desc*, const DecodeGeometry&, const void*, const kvs_cache*, void*, float*, float*, int*, int, const float*, hipStream_t);
void launch_decode_mfma_b4(const kvs_desc*, const DecodeGeometry&, const void*, const kvs_cache*, void*, float*, float*, int*, int, const float*, hipStream_t);
void launch_decode_mfma_b8(const kvs_desc*, const DecodeGeometry&, const void*, const kvs_cache*, void*, float*, float*, int*, int, const float*, hipStream_t);

void launch_decode_mfma_kpt_b2(const kvs_desc*, const DecodeGeometry&, const void*, const kvs_cache*, void*, float*, float*, int*, int, const float*, hipStream_t);
void launch_decode_mfma_kpt_b3(const kvs_desc*, const DecodeGeometry&, const void*, const kvs_cache*, void*, float*, float*, int*, int, const float*, hipStream_t);
void launch_decode_mfma_kpt_b4(const kvs_desc*, const DecodeGeometry&, const void*, const kvs_cache*, void*, float*, float*, int*, int, const float*, hipStream_t);
void launch_decode_mfma_kpt_b8(const kvs_desc*, const DecodeGeometry&, const void*, const kvs_cache*, void*, float*, float*, int*, int, const float*, hipStream_t);

void launch_decode_mfma(const kvs_desc* d, const DecodeGeometry& geo, const void* q, const kvs_cache* c,
                        void* out, float* lse, float* ws, int* arrive, int n_used, const float* extra, hipStream_t s) {
  if (d->key_per_token) {
    if (d->bits == 2) launch_decode_mfma_kpt_b2(d, geo, q, c, out, lse, ws, arrive, n_used, extra, s);
    else if (d->bits == 3) launch_decode_mfma_kpt_b3(d, geo, q, c, out, lse, ws, arrive, n_used, extra, s);
    else if (d->bits == 4) launch_decode_mfma_kpt_b4(d, geo, q, c, out, lse, ws, arrive, n_used, extra, s);
    else launch_decode_mfma_kpt_b8(d, geo, q, c, out, lse, ws, arrive, n_used, extra, s);
    return;
  }
  if (d->bits == 2) launch_decode_mfma_b2(d, geo, q, c, out, lse, ws, arrive, n_used, extra, s);
  else if (d->bits == 3) launch_decode_mfma_b3(d, geo, q, c, out, lse, ws, arrive, n_used, extra, s);
  else if (d->bits == 4) launch_decode_mfma_b4(d, geo, q, c, out, lse, ws, arrive, n_used, extra, s);
  else launch_decode_mfma_b8(d, geo, q, c, out, lse, ws, arrive, n_used, extra, s);
}

}  // namespace kvs

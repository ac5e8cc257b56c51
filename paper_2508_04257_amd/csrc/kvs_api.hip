// Host-only part of the C ABI: descriptor validation, buffer sizing, launch geometry.
#include "kvs_device.h"

namespace kvs {

kvs_status validate_desc(const kvs_desc* d) {
  if (!d) return KVS_ERR_INVALID;
  if (d->B < 1 || d->n < 1 || d->Hq < 1 || d->Hkv < 1 || d->D < 1) return KVS_ERR_INVALID;
  if (d->keep_cap < 0 || !(d->sparse_frac >= 0.0f) || d->sparse_frac >= 1.0f) return KVS_ERR_INVALID;
  if (d->Hq % d->Hkv != 0) return KVS_ERR_INVALID;
  if (d->sparse_frac > 0.0f && d->sparse_cap < 1) return KVS_ERR_INVALID;
  if (d->key_per_token != 0 && d->key_per_token != 1) return KVS_ERR_INVALID;
  if (d->D != KVS_HEAD_DIM) return KVS_ERR_UNSUPPORTED;
  if (d->bits != 2 && d->bits != 3 && d->bits != 4 && d->bits != 8) return KVS_ERR_UNSUPPORTED;
  if (d->bits == 8 && d->sparse_frac > 0.0f) return KVS_ERR_UNSUPPORTED;       // isolated outliers are a low-bit remedy
  if (d->group != 32 && d->group != 64 && d->group != 128) return KVS_ERR_UNSUPPORTED;
  if (d->n % KVS_V_TILE != 0) return KVS_ERR_UNSUPPORTED;      // also a multiple of 64 and of G
  const int rep = d->Hq / d->Hkv;
  if (rep != 1 && rep != 2 && rep != 4 && rep != 8) return KVS_ERR_UNSUPPORTED;
  if (d->key_per_token && d->sparse_frac > 0.0f) return KVS_ERR_UNSUPPORTED;   // per-token Keys: dense caches only
  // CSR rows and word offsets are 32-bit quantities in places; keep a wide margin.  (Two factors
  // first: the product of three 31-bit numbers does not fit 64 bits.)
  const int64_t pairs = static_cast<int64_t>(d->B) * d->Hkv;
  if (pairs >= (int64_t{1} << 30)) return KVS_ERR_UNSUPPORTED;
  const int64_t rows = pairs * d->n;
  if (rows >= (int64_t{1} << 30)) return KVS_ERR_UNSUPPORTED;
  if (static_cast<int64_t>(d->B) * d->Hq >= (int64_t{1} << 30)) return KVS_ERR_UNSUPPORTED;   // query rows likewise
  if (d->sparse_frac > 0.0f) {
    // CSR positions are int32 (with room for a tile's 16384 entries and a round of loads past any
    // position): the whole tensor must be countable even if every entry ties.
    if (d->sparse_cap > (int64_t{1} << 31) - 1 - 32768 || rows * KVS_HEAD_DIM >= (int64_t{1} << 31)) return KVS_ERR_UNSUPPORTED;
  }
  return KVS_OK;
}

constexpr int kMfmaTargetGroups = 256;   // one workgroup per compute unit

// Splits are whole numbers of 128-token Value tiles: one workgroup per split and (sequence, KV
// head), about one workgroup per compute unit in all, and a single split per (sequence, KV head)
// whenever there are enough of those - then no second kernel is needed.  (Per launch, where the
// query heads of a KV head take several launches.)
// Most splits any token count up to d->n can get (what the workspace is sized for).
int decode_max_splits(const kvs_desc* d) {
  const int pairs = d->B * d->Hkv;
  const int splits = pairs >= kMfmaTargetGroups ? 1 : (kMfmaTargetGroups + pairs / 2) / pairs;
  const int tiles = d->n / KVS_V_TILE;
  return splits > tiles ? tiles : (splits < 1 ? 1 : splits);
}

DecodeGeometry decode_geometry(const kvs_desc* d) { return decode_geometry(d, d->n); }

// The same for the first n_used tokens (a multiple of 128, at least 128) of a cache laid out for d->n.
DecodeGeometry decode_geometry(const kvs_desc* d, int n_used) {
  const int tiles = n_used / KVS_V_TILE;
  DecodeGeometry g;
  int splits = decode_max_splits(d);
  if (splits > tiles) splits = tiles;
  if (splits < 1) splits = 1;
  const int tiles_per_split = (tiles + splits - 1) / splits;
  g.split_tokens = tiles_per_split * KVS_V_TILE;
  g.splits = (tiles + tiles_per_split - 1) / tiles_per_split;
  return g;
}

}  // namespace kvs

namespace {
size_t round16(size_t v) { return v < 16 ? 16 : (v + 15) & ~static_cast<size_t>(15); }
}  // namespace

extern "C" int32_t kvs_version(void) { return 100; }

extern "C" const char* kvs_status_string(kvs_status s) {
  switch (s) {
    case KVS_OK: return "ok";
    case KVS_ERR_INVALID: return "invalid argument";
    case KVS_ERR_UNSUPPORTED: return "unsupported configuration";
    case KVS_ERR_CAPACITY: return "capacity exceeded";
    case KVS_ERR_DEVICE: return "device launch failed";
    case KVS_ERR_SCRATCH: return "descriptor needs more scratch than the library holds";
  }
  return "unknown status";
}

extern "C" kvs_status kvs_cache_bytes(const kvs_desc* d, size_t* sizes) {
  const kvs_status st = kvs::validate_desc(d);
  if (st != KVS_OK) return st;
  if (!sizes) return KVS_ERR_INVALID;
  const size_t bh = static_cast<size_t>(d->B) * d->Hkv;
  const size_t n = d->n;
  const size_t W = kvs::words_per_128(d->bits);
  const size_t code_bytes = bh * n * W * 4;                 // W words per 128 codes, K and V alike
  const size_t keep_rows = bh * d->keep_cap * KVS_HEAD_DIM * 2;
  const bool sparse = d->sparse_frac > 0.0f;
  const size_t cap = sparse ? static_cast<size_t>(d->sparse_cap) + kvs::kCsrPadEntries : 0;   // see kCsrPadEntries
  const size_t v[KVS_CACHE_FIELDS] = {
      code_bytes,                                   // k_codes
      code_bytes,                                   // v_codes
      bh * (n / d->group) * KVS_HEAD_DIM * 4,       // k_params
      bh * n * (KVS_HEAD_DIM / d->group) * 4,       // v_params
      keep_rows,                                    // keep_k
      keep_rows,                                    // keep_v
      static_cast<size_t>(d->B) * d->keep_cap * 4,  // keep_idx
      static_cast<size_t>(d->B) * 4,                // keep_cnt
      static_cast<size_t>(d->B) * n,                // keep_mask
      sparse ? (bh * n + 1) * 4 : 0,                // k_rowptr
      cap * 2,                                      // k_col
      cap * 2,                                      // k_val
      sparse ? (bh * n + 1) * 4 : 0,                // v_rowptr
      cap * 2,                                      // v_col
      cap * 2,                                      // v_val
      4,                                            // status
      bh * KVS_V_TILE * KVS_HEAD_DIM * 2,           // res_k
      bh * KVS_V_TILE * KVS_HEAD_DIM * 2,           // res_v
  };
  for (int i = 0; i < KVS_CACHE_FIELDS; ++i) {
    const bool csr_field = i >= 9 && i <= 14;
    sizes[i] = (csr_field && !sparse) ? 0 : round16(v[i]);
  }
  return KVS_OK;
}

extern "C" int32_t kvs_decode_splits(const kvs_desc* d) {
  if (kvs::validate_desc(d) != KVS_OK) return 0;
  return kvs::decode_geometry(d).splits;
}

// What the decode calls keep in the workspace: the arrival counters, per (b, hq, split) the
// unnormalised fp32 output row plus running max and sum (sized for the most splits any token count
// of a growing cache can get), and one more part per (b, hq) for a growing cache's residual rows.
size_t kvs::decode_workspace_bytes(const kvs_desc* d) {
  const size_t rows = static_cast<size_t>(d->B) * d->Hq * (kvs::decode_max_splits(d) + 1);
  return round16(kvs::workspace_counter_words(d) * 4 + rows * (KVS_HEAD_DIM + 2) * 4);
}

extern "C" size_t kvs_workspace_bytes(const kvs_desc* d) {
  if (kvs::validate_desc(d) != KVS_OK) return 0;
  // quantise (dense-and-sparse only): histograms, thresholds, scan scratch, staging lists - behind
  // the counters, which quantise calls leave alone
  const size_t quant = d->sparse_frac > 0.0f ? kvs::workspace_counter_words(d) * 4 + kvs::sparse_workspace_words(d) * 4 : 0;
  const size_t decode = kvs::decode_workspace_bytes(d);
  return round16(decode > quant ? decode : quant);
}

extern "C" size_t kvs_workspace_zero_bytes(const kvs_desc* d) {
  if (kvs::validate_desc(d) != KVS_OK) return 0;
  return kvs::workspace_counter_words(d) * 4;
}

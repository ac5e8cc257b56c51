// kvs_prefill_layers: the prefill loop of the paper's Algorithm 1 without the model - the order
// in which the layers' K and V are quantised and the sink set is filled, as one submission.
//   S_sink starts empty; layer l = 1 .. L quantises K^l, V^l leaving out the tokens of S_sink as
//   it stands when the layer runs; after layer l_E, S_sink = top-k tokens of |H^{l_E}[:, c]|.
// Layers 1 .. l_E are therefore quantised under the first-N mask alone (empty when N = 0), layers
// l_E + 1 .. L under first-N united with the predicted tokens (Section 4.3, item (2): the
// identification runs once, at the emergence stage).  Host code only: it validates everything,
// then enqueues the kernels of kvs_predict_sinks and kvs_quantize_kv in that order.
#include "kvs_device.h"

extern "C" kvs_status kvs_prefill_layers(const kvs_desc* desc, int32_t n_layers, int32_t emergence_layer,
                                          const void* const* K, const void* const* V, const void* hidden, int32_t d,
                                          const int32_t* channels, int32_t n_channels, int32_t k, int32_t first_n,
                                          int32_t* sink_idx, uint8_t* early_mask, uint8_t* keep_mask,
                                          const kvs_cache* caches, void* workspace, void* predict_workspace,
                                          void* stream) {
  kvs_status st = kvs::validate_desc(desc);
  if (st != KVS_OK) return st;
  if (n_layers < 1 || emergence_layer < 0 || emergence_layer > n_layers) return KVS_ERR_INVALID;
  if (!K || !V || !caches || !early_mask || !keep_mask) return KVS_ERR_INVALID;
  if (static_cast<int64_t>(k) + first_n > desc->keep_cap) return KVS_ERR_INVALID;   // the kept rows must fit
  st = kvs::check_predict_call(hidden, desc->B, desc->n, d, channels, n_channels, k, first_n, sink_idx, keep_mask);
  if (st != KVS_OK) return st;
  for (int l = 0; l < n_layers; ++l) {
    st = kvs::check_quantize_call(desc, K[l], V[l], keep_mask, &caches[l], workspace);
    if (st != KVS_OK) return st;
  }
  // Nothing has been launched so far; from here on only launch failures can stop the sequence.
  if (emergence_layer > 0) {                          // the mask of the layers that run before the set exists
    st = kvs_predict_sinks(hidden, desc->B, desc->n, d, channels, n_channels, /*k=*/0, first_n, nullptr, early_mask,
                           nullptr, stream);
    if (st != KVS_OK) return st;
  }
  for (int l = 1; l <= n_layers; ++l) {
    if (l == emergence_layer + 1) {                   // the "l = l_E" branch has run: S_sink is filled
      st = kvs_predict_sinks(hidden, desc->B, desc->n, d, channels, n_channels, k, first_n, sink_idx, keep_mask,
                             predict_workspace, stream);
      if (st != KVS_OK) return st;
    }
    const uint8_t* mask = l <= emergence_layer ? early_mask : keep_mask;
    st = kvs_quantize_kv(desc, K[l - 1], V[l - 1], mask, &caches[l - 1], workspace, stream);
    if (st != KVS_OK) return st;
  }
  if (emergence_layer == n_layers) {                  // the set is filled after the last layer: no cache sees it
    st = kvs_predict_sinks(hidden, desc->B, desc->n, d, channels, n_channels, k, first_n, sink_idx, keep_mask,
                           predict_workspace, stream);
    if (st != KVS_OK) return st;
  }
  return KVS_OK;
}

/*
 * kvs.h - C ABI of the KVSink hot path on AMD Instinct MI355X (gfx950).
 *
 * KVSink (arXiv 2508.04257) keeps the Key/Value rows of attention-sink tokens in 16 bit while
 * the rest of the KV cache is quantised to 2-4 (or 8) bits, and finds those tokens from the extreme
 * activation outliers of one hidden-state channel.  The three calls below are the data-parallel
 * part of that method:
 *
 *   kvs_predict_sinks  - top-k over tokens of |H[i, c]| (Algorithm 1, the l = l_E branch;
 *                        Section 4.3), united with the first-N tokens of the PFN baseline.
 *   kvs_quantize_kv    - asymmetric uniform b-bit quantisation (Appendix C equations) of K per
 *                        channel and V per token, group size G, skipping the kept tokens, whose
 *                        rows are copied unchanged (Algorithm 1, the two quantise steps);
 *                        optional dense-and-sparse fp16 outliers (Section 5.1).
 *   kvs_decode_attn    - softmax(q K'^T / sqrt(d_k)) V' for one query per sequence and head over
 *                        the packed cache, kept rows merged in 16 bit (Section 2 attention
 *                        equation; the sink / non-sink split of Section 4.2).
 *
 * Conventions common to every call
 *   - Every pointer is a DEVICE pointer owned by the caller unless marked HOST.  The library
 *     allocates and frees nothing and keeps no state between calls.
 *   - Calls enqueue kernels on `stream` (a hipStream_t passed as void*, NULL = default stream)
 *     and return without synchronising.
 *   - Argument errors are found on the host before anything is launched; outputs are then
 *     untouched and the return value says why.  Data-dependent overflow (more kept tokens than
 *     keep_cap, more sparse entries than sparse_cap) cannot be known on the host: it is written
 *     to cache->status on the device (0 = fine, KVS_ERR_CAPACITY otherwise) and the call still
 *     returns KVS_OK.  The caller zeroes *status before the first call and reads it after
 *     synchronising.  With more flagged tokens than keep_cap, keep_cnt[b] still holds the number
 *     flagged, the rows hold the keep_cap lowest token indices, and every flagged token is left
 *     out of the quantisation (code 0): such a cache reports the condition, it is not one to
 *     decode from.
 *   - fp16 is IEEE binary16; inputs must be finite.  All tensors are dense, row-major.
 *   - Every buffer starts at a multiple of 16 bytes (the decode calls return KVS_ERR_INVALID for a
 *     cache whose code, parameter, kept-row or CSR arrays do not).
 *
 * Packed cache layout (D = 128 only)
 *   cpw = codes per 32-bit word: 16 (2 bit), 10 (3 bit), 8 (4 bit), 4 (8 bit);
 *   W = ceil(128 / cpw) = 8, 13, 16, 32.
 *   Slot j of a word sits at bit 2j (2 bit) / 4j (4 bit) / 8j (8 bit); for 3 bit, slots 0-4 sit at bits
 *   3j and slots 5-9 at bits 16 + 3(j - 5), bits 15 and 31 are zero.  Unused slots are zero.
 *   k_codes  uint32 [B, Hkv, n/64, W, 64]   word (T, w, t): channels cpw*w .. of token 64T + t.
 *   v_codes  uint32 [B, Hkv, n/128, W, 128] word (T, u, c): tokens 128T + cpw*u .. of channel c.
 *   k_params uint32 [B, Hkv, n/G, 128]      one per (token group, channel); with per-token Keys
 *            (desc->key_per_token) [B, Hkv, n, 128/G], one per (token, channel group), like v_params.
 *   v_params uint32 [B, Hkv, n, 128/G]      one per (token, channel group).
 *            parameter word = fp16 scale in bits 0-15 | int16 zero in bits 16-31;
 *            dequantised value = scale * (code - zero).
 *   keep_k / keep_v  fp16 [B, Hkv, keep_cap, 128]  rows of the kept tokens, ascending token order,
 *            zero padded;  keep_idx int32 [B, keep_cap] (-1 padded);  keep_cnt int32 [B];
 *            keep_mask uint8 [B, n] (copy of the mask the cache was built with).
 *   CSR of isolated outliers (only when sparse_frac > 0), B*Hkv*n rows per tensor:
 *            rowptr int32 [B*Hkv*n + 1], col uint16 [sparse_cap + 4], val fp16 [sparse_cap + 4]
 *            (the four entries behind the capacity are padding that decode may read and never
 *            uses; kvs_cache_bytes() counts them).
 *            Keys: row = (b, h, token), column = channel.  Values: row = (b, h, 128-token tile,
 *            channel), column = token inside the tile (the transposition of the Value code tiles).
 *            A col word holds the column in bits 0-6 and, in bits 7-13, the row's place inside its
 *            128-row tile (token % 128 for Keys, the channel for Values): decode reads the entries
 *            of a tile as one contiguous run, rowptr[tile start] .. rowptr[tile end], and an entry
 *            then says which quantisation group its row belongs to.  Columns ascend inside a row.
 *   Residual window (growing caches only): res_k / res_v fp16 [B, Hkv, 128, 128], row r = token
 *            128 * (n_tokens / 128) + r of the sequence, still in 16 bit.
 */
#ifndef KVS_H
#define KVS_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define KVS_HEAD_DIM 128
#define KVS_K_TILE 64
#define KVS_V_TILE 128
#define KVS_CACHE_FIELDS 18
#define KVS_MAX_TOPK 1024
#define KVS_MAX_PREDICT_TOKENS 65536
#define KVS_NOALLOC_SCRATCH_BYTES (4u << 20) /* scratch kvs_decode_attn_noalloc holds per GPU */

typedef enum {
  KVS_OK = 0,
  KVS_ERR_INVALID = 1,     /* null pointer, non-positive size, shape rule broken           */
  KVS_ERR_UNSUPPORTED = 2, /* valid request outside what this version implements           */
  KVS_ERR_CAPACITY = 3,    /* only ever written to cache->status, see above                */
  KVS_ERR_DEVICE = 4,      /* a HIP launch failed                                          */
  KVS_ERR_SCRATCH = 5      /* kvs_decode_attn_noalloc: desc needs more than the fixed scratch */
} kvs_status;

/* Shape and quantiser setting of one layer's cache.  Plain data, filled by the caller. */
typedef struct kvs_desc {
  int32_t B, n, Hq, Hkv, D; /* batch, cached tokens, query heads, KV heads, head dim (128)    */
                            /* Hq / Hkv in {1, 2, 4, 8};  n % 128 == 0                        */
  int32_t bits;             /* 2, 3, 4 or 8 (8: not with sparse_frac > 0, KVS_ERR_UNSUPPORTED)    */
  int32_t group;            /* G: 32, 64 or 128.  K groups run along tokens, V along channels */
  int32_t keep_cap;         /* rows of the fp16 side buffer per sequence (>= 0)               */
  float sparse_frac;        /* fraction of entries isolated in fp16; 0 = off                  */
  int32_t key_per_token;    /* 0: per-channel Keys (above); 1: Keys quantised like Values, groups */
                            /* of G channels of one token (the per-token scheme of Section 5.1) - */
                            /* k_params is then [B, Hkv, n, 128/G].  Not with sparse_frac > 0     */
                            /* (KVS_ERR_UNSUPPORTED).                                             */
  int64_t sparse_cap;       /* CSR capacity in entries per tensor when sparse_frac > 0        */
                            /* (1 .. 2^31 - 32769, beyond: KVS_ERR_UNSUPPORTED)               */
} kvs_desc;

/* The quantised cache of one layer: device pointers to caller-owned buffers whose byte sizes
 * kvs_cache_bytes() returns in this field order.  The CSR fields may be NULL when
 * sparse_frac == 0, res_k / res_v when the cache never grows. */
typedef struct kvs_cache {
  uint32_t* k_codes;
  uint32_t* v_codes;
  uint32_t* k_params;
  uint32_t* v_params;
  void* keep_k;
  void* keep_v;
  int32_t* keep_idx;
  int32_t* keep_cnt;
  uint8_t* keep_mask;
  int32_t* k_rowptr;
  uint16_t* k_col;
  void* k_val;
  int32_t* v_rowptr;
  uint16_t* v_col;
  void* v_val;
  int32_t* status;
  void* res_k;
  void* res_v;
} kvs_cache;

/* Library version (major * 100 + minor). */
int32_t kvs_version(void);

/* Static text for a status code. */
const char* kvs_status_string(kvs_status s);

/* Byte size of every kvs_cache buffer for `desc`, in field order (sizes is a HOST array of
 * KVS_CACHE_FIELDS entries; CSR entries are 0 when sparse_frac == 0; every size is rounded up
 * to a multiple of 16 and is at least 16).  Returns KVS_ERR_INVALID / KVS_ERR_UNSUPPORTED for a
 * descriptor the other calls would reject. */
kvs_status kvs_cache_bytes(const kvs_desc* desc, size_t* sizes);

/* Bytes of scratch `workspace` that kvs_quantize_kv and kvs_decode_attn need for `desc`
 * (the larger of the two; 0 for an invalid descriptor).  Calls that share a workspace must be
 * ordered on one stream.
 * The first kvs_workspace_zero_bytes(desc) bytes are arrival counters of the decode kernels (when
 * several workgroups share a (sequence, KV head), the one that finishes last merges their
 * results): the caller ZEROES THEM ONCE after allocating the workspace, every call that runs to
 * completion leaves them zero, and nothing else in the workspace needs to be preserved or
 * initialised.  Like cache->status this is a contract, not checked: with stale counters a decode
 * call still stays inside its buffers and terminates, but output rows may not be written.  After
 * an aborted launch (device reset, failed call) zero them again. */
size_t kvs_workspace_bytes(const kvs_desc* desc);
size_t kvs_workspace_zero_bytes(const kvs_desc* desc);

/* Number of token splits kvs_decode_attn uses for `desc` (each split is one workgroup per
 * (sequence, KV head); informational, 0 for an invalid descriptor). */
int32_t kvs_decode_splits(const kvs_desc* desc);

/*
 * Sink prediction.  For each sequence b: score[i] = max over the listed channels of
 * |hidden[b, i, c]|; the k tokens with the largest score (ties: lower index first) are written
 * ascending to sink_idx[b, 0..k), and keep_mask[b, i] = 1 iff i is one of them or i < first_n
 * (else 0).  With n_channels == 1 this is exactly the paper's single-channel rule.
 *   hidden    fp16 [B, n, d]
 *   channels  HOST int32 [n_channels], each in [0, d), 1 <= n_channels <= 8
 *   k in [0, min(n, KVS_MAX_TOPK)], first_n in [0, n], n <= KVS_MAX_PREDICT_TOKENS
 *   sink_idx  int32 [B, k] (may be NULL when k == 0);  keep_mask uint8 [B, n]
 *   workspace kvs_predict_workspace_bytes(B, n, k) bytes of scratch, or NULL.  With it, sequences
 *             longer than 4096 tokens are scanned by one workgroup per 4096-token slice; without
 *             it (or when that size is 0) one workgroup scans a whole sequence.  Same result.
 */
size_t kvs_predict_workspace_bytes(int32_t B, int32_t n, int32_t k);
kvs_status kvs_predict_sinks(const void* hidden, int32_t B, int32_t n, int32_t d,
                             const int32_t* channels, int32_t n_channels, int32_t k,
                             int32_t first_n, int32_t* sink_idx, uint8_t* keep_mask,
                             void* workspace, void* stream);

/*
 * Quantise one layer's K and V (fp16 [B, Hkv, n, 128]) into `out`.
 * Per group (K: G consecutive tokens of one channel; V: G consecutive channels of one token),
 * over the entries that are neither on a kept token nor an isolated outlier:
 *   scale = fp16_round_up((max - min) / (2^bits - 1)),  zero = -round(min / scale),
 *   code  = clamp(round(x / scale) + zero, 0, 2^bits - 1)
 * in fp32 with round-half-to-even and x / scale evaluated as x * (1 / scale); kept and isolated
 * entries get code 0.  At 8 bit the scale is max((max - min) / 255, |min| / 32766) before the
 * rounding to fp16, which keeps the zero point inside its int16 half (up to 4 bit it always is
 * for fp16 data); the bound only binds for groups whose values lie within 1/128 of their
 * distance from zero, and the step it gives is finer than the fp16 spacing of such data.  A group with no such entry gets (scale 1, zero 0); a constant group gets
 * scale |min| (1 if min == 0).  Rows of kept tokens are copied bit for bit to keep_k / keep_v.
 * With sparse_frac > 0 the entries with |x| >= tau go to the CSR arrays with their fp16 value,
 * tau being the magnitude at which the descending cumulative count over all non-kept entries
 * of the tensor first reaches ceil(sparse_frac * count).
 *   keep_mask uint8 [B, n] (nonzero = keep); copied to out->keep_mask.
 *   workspace: kvs_workspace_bytes(desc) bytes (may be NULL when that is 0).
 */
kvs_status kvs_quantize_kv(const kvs_desc* desc, const void* K, const void* V,
                           const uint8_t* keep_mask, const kvs_cache* out, void* workspace,
                           void* stream);

/*
 * Outlier thresholds apart from the quantise call.  The dense-and-sparse setting of Section 5.1 is
 * KVQuant's, which fixes its outlier thresholds on calibration data before inference (the
 * counterpart, for the isolated entries, of the static quantisation of Appendix C); the search
 * inside kvs_quantize_kv is the dynamic form.  Only with sparse_frac > 0 (KVS_ERR_INVALID else).
 * kvs_outlier_thresholds: the search of kvs_quantize_kv alone.  tau: DEVICE uint32 [2], written:
 *   tau[0] for Keys, tau[1] for Values, each the fp16 magnitude pattern (bits 0-14 of the half;
 *   0x8000 = nothing is isolated) at which the descending cumulative count over the non-kept
 *   entries first reaches ceil(sparse_frac * count).
 * kvs_quantize_kv_thresholds: kvs_quantize_kv with the thresholds given (device words as the
 *   search writes them, of this or of other data; larger values count as 0x8000): every non-kept
 *   entry with magnitude pattern >= tau is isolated, whatever fraction of the tensor that is;
 *   desc->sparse_frac only has to be > 0.  More entries than sparse_cap are reported through
 *   cache->status as in kvs_quantize_kv.  With the thresholds kvs_outlier_thresholds finds on the
 *   same K, V and mask the result is that of kvs_quantize_kv, bit for bit.
 *   workspace: kvs_workspace_bytes(desc) bytes in both.
 */
kvs_status kvs_outlier_thresholds(const kvs_desc* desc, const void* K, const void* V,
                                  const uint8_t* keep_mask, uint32_t* tau, void* workspace,
                                  void* stream);
kvs_status kvs_quantize_kv_thresholds(const kvs_desc* desc, const void* K, const void* V,
                                      const uint8_t* keep_mask, const uint32_t* tau,
                                      const kvs_cache* out, void* workspace, void* stream);

/*
 * The prefill loop of Algorithm 1 without the model: L layers' K and V quantised in the order the
 * algorithm runs them, with the sink set filled once, after the emergence layer l_E (Section 4.3,
 * item (2)).  The set is empty while layers 1 .. l_E run, so those layers are quantised under the
 * first-N mask alone; layers l_E + 1 .. L under first-N united with the top-k tokens of
 * |hidden[b, i, c]| - exactly kvs_quantize_kv(K[l], V[l], mask of the layer's phase, caches[l])
 * for every layer, and kvs_predict_sinks for the masks, enqueued as one sequence on `stream`.
 *   n_layers L >= 1;  emergence_layer l_E in [0, L] (0: the set is known before layer 1; L: no
 *   cache sees it);  k + first_n <= desc->keep_cap.
 *   K, V        HOST arrays of L device pointers, fp16 [B, Hkv, n, 128] each (layer 1 first)
 *   hidden      fp16 [B, n, d], the hidden state after layer l_E;  channels HOST, as in kvs_predict_sinks
 *   sink_idx    int32 [B, k] (may be NULL when k == 0);  early_mask, keep_mask uint8 [B, n]: the
 *               masks of the two phases, both written (early_mask only when l_E > 0)
 *   caches      HOST array of L kvs_cache structs (device buffers sized by kvs_cache_bytes(desc))
 *   workspace   as for kvs_quantize_kv, shared by the layers;  predict_workspace as for
 *               kvs_predict_sinks (may be NULL)
 * Every argument of every layer is checked before anything is launched.
 */
kvs_status kvs_prefill_layers(const kvs_desc* desc, int32_t n_layers, int32_t emergence_layer,
                              const void* const* K, const void* const* V, const void* hidden, int32_t d,
                              const int32_t* channels, int32_t n_channels, int32_t k, int32_t first_n,
                              int32_t* sink_idx, uint8_t* early_mask, uint8_t* keep_mask,
                              const kvs_cache* caches, void* workspace, void* predict_workspace,
                              void* stream);

/*
 * Decode attention of one query per (sequence, query head) over the whole cache:
 *   K'[t], V'[t] = the fp16 keep row if token t is kept, else the dequantised row with isolated
 *   outliers replaced by their fp16 value;  s_t = q . K'[t] / sqrt(128);  p = softmax(s);
 *   out = sum_t p_t V'[t]  (fp32 accumulation, stored fp16);  lse = log sum_t exp(s_t).
 * Query head hq reads KV head hq / (Hq / Hkv).
 *   q fp16 [B, Hq, 128];  out fp16 [B, Hq, 128];  lse float [B, Hq] or NULL.
 *   workspace: kvs_workspace_bytes(desc) bytes, its head zeroed once (kvs_workspace_zero_bytes).
 */
kvs_status kvs_decode_attn(const kvs_desc* desc, const void* q, const kvs_cache* cache,
                           void* out, float* lse, void* workspace, void* stream);

/*
 * kvs_decode_attn for callers that cannot allocate device memory and hold no workspace: code
 * under HIP graph capture, tight serving loops, harnesses that forbid allocation.  Same arguments
 * minus `workspace`, same kernels (after one small kernel that clears the arrival counters at the
 * scratch's head), same result; the scratch is an array of
 * KVS_NOALLOC_SCRATCH_BYTES that the library itself holds on every GPU it runs on (from the first
 * call on that GPU until the process ends).  The call allocates and frees nothing.
 *   - A descriptor whose decode calls need more than KVS_NOALLOC_SCRATCH_BYTES of workspace
 *     (520 bytes per (sequence, query head) and part of the token range, plus the counters; the
 *     benchmark's workloads need less than 1 MiB) is rejected with KVS_ERR_SCRATCH before anything
 *     is launched.
 *   - The GPU is the one current on the calling thread (hipGetDevice); `stream` must belong to it.
 *   - Every call on a GPU shares that GPU's one array: calls that overlap on one GPU (different
 *     streams, or different threads) race on it.  Order them on one stream, or use
 *     kvs_decode_attn with a workspace per stream.
 */
kvs_status kvs_decode_attn_noalloc(const kvs_desc* desc, const void* q, const kvs_cache* cache,
                                   void* out, float* lse, void* stream);

/*
 * Growing caches (Section 2, "KV cache": in the decoding phase every new token's K and V are
 * appended to the cache; Appendix A: quantisation once a number of local tokens has accumulated).
 * desc->n is then the CAPACITY the buffers are laid out for and n_tokens says how many tokens
 * they hold.  Quantisation groups are positional and the largest spans 128 tokens, so tokens are
 * quantised in whole blocks of 128, exactly as kvs_quantize_kv quantises them; the tokens after
 * the last whole block wait unchanged in res_k / res_v until their block is complete.  The state
 * after any sequence of these calls equals what kvs_quantize_prefix makes of the same tokens.
 * Not available with sparse_frac > 0 (KVS_ERR_UNSUPPORTED).
 *
 * kvs_quantize_prefix: a prompt of n_tokens in [0, desc->n] tokens, any length.
 *   K, V fp16 [B, Hkv, n_tokens, 128];  keep_mask uint8 [B, n_tokens] (kept tokens of the last,
 *   incomplete block are remembered in out->keep_mask and honoured when the block is quantised).
 * kvs_append_kv: one more token per sequence; n_tokens in [0, desc->n) = tokens held before the call.
 *   k_new, v_new fp16 [B, Hkv, 128].  The new token is not a kept token.  When it completes a
 *   block, the block is quantised by the same call.
 * kvs_decode_attn_n: kvs_decode_attn over the first n_tokens in [1, desc->n] tokens: quantised
 *   blocks, kept rows and residual rows in one softmax.
 * workspace: kvs_workspace_bytes(desc) bytes in all three.
 * State the calls rely on (not checked; a caller that breaks it gets wrong results, never an
 * access outside the buffers):
 *   - kvs_quantize_prefix initialises a cache: it zeroes keep_mask out to the capacity and writes
 *     keep_idx / keep_cnt.  A cache must have had one kvs_quantize_prefix call (n_tokens = 0 is
 *     allowed, K and V may then be any non-NULL pointers) before its first kvs_append_kv.
 *   - n_tokens in kvs_append_kv is the number of tokens the cache holds, i.e. the n_tokens of the
 *     prefix call plus the appends since; n_tokens in kvs_decode_attn_n is that number after the
 *     last append.  A smaller value still attends to every kept row the cache has recorded.
 */
kvs_status kvs_quantize_prefix(const kvs_desc* desc, const void* K, const void* V,
                               const uint8_t* keep_mask, int32_t n_tokens, const kvs_cache* out,
                               void* workspace, void* stream);
kvs_status kvs_append_kv(const kvs_desc* desc, const void* k_new, const void* v_new, int32_t n_tokens,
                         const kvs_cache* cache, void* workspace, void* stream);
kvs_status kvs_decode_attn_n(const kvs_desc* desc, const void* q, const kvs_cache* cache, int32_t n_tokens,
                             void* out, float* lse, void* workspace, void* stream);

/*
 * Static quantisation (Appendix C, "Dynamic and static quantization": the range is estimated from
 * calibration data before inference and the parameters stay fixed; Table 1's setting: global
 * min-max, kept tokens left out of the calibration as well as of the quantisation).
 * One parameter pair per Key channel of a KV head and one per Value channel group of a KV head.
 *   calib     kvs_calibration_bytes(desc) bytes of device memory: running minimum and maximum per
 *             (KV head, channel) of K and of V over every non-kept token of every kvs_calibrate
 *             call since kvs_calibrate_reset.  Calls on one stream accumulate in order; calls on
 *             several streams may run concurrently (integer atomics).
 *   kvs_calibrate: K, V fp16 [B, Hkv, n, 128], keep_mask uint8 [B, n] as in kvs_quantize_kv.
 *   kvs_static_params: k_static uint32 [Hkv, 128] (with desc->key_per_token: [Hkv, 128 / G], one
 *             per Key channel group), v_static uint32 [Hkv, 128 / G] parameter words
 *             (fp16 scale | int16 zero << 16) by the scale / zero equations of kvs_quantize_kv
 *             applied to the calibrated range (nothing seen: scale 1, zero 0).
 *   kvs_quantize_kv_static: kvs_quantize_kv with those words instead of per-group statistics;
 *             values outside the calibrated range clamp to code 0 or 2^bits - 1.  The cache has
 *             the ordinary layout (every group's parameter word is the static word), so
 *             kvs_decode_attn reads it like any other.  Not with sparse_frac > 0.
 */
size_t kvs_calibration_bytes(const kvs_desc* desc);
kvs_status kvs_calibrate_reset(const kvs_desc* desc, void* calib, void* stream);
kvs_status kvs_calibrate(const kvs_desc* desc, const void* K, const void* V, const uint8_t* keep_mask,
                         void* calib, void* stream);
kvs_status kvs_static_params(const kvs_desc* desc, const void* calib, uint32_t* k_static,
                             uint32_t* v_static, void* stream);
kvs_status kvs_quantize_kv_static(const kvs_desc* desc, const void* K, const void* V,
                                  const uint8_t* keep_mask, const uint32_t* k_static,
                                  const uint32_t* v_static, const kvs_cache* out, void* workspace,
                                  void* stream);

/*
 * Quantisation-error report with the structure of the paper's Table 1 (Section 4.1): for Keys and
 * for Values, the sum of squared errors x - scale * (code - zero) and the number of entries, split
 * into the quantisation groups that contain a flagged token and those that do not.  Entries of
 * kept tokens (cache->keep_mask) are stored exactly and are left out.  A per-channel Key group
 * (G consecutive tokens of one channel) counts as flagged if any of its tokens is; a per-token
 * group (Values; Keys with desc->key_per_token) if its token is.
 *   K, V       fp16 [B, Hkv, n, 128], the tensors `cache` was quantised from (kvs_quantize_kv or
 *              kvs_quantize_kv_static with this desc)
 *   sink_mask  uint8 [B, n]: the tokens that classify the groups (nonzero = flagged); it need not
 *              be the mask the cache was built with
 *   report     DEVICE, 64 bytes, overwritten: double sse[2][2] then uint64 count[2][2], indexed
 *              [0 Keys / 1 Values][0 groups without / 1 groups with a flagged token]
 * The squared differences are formed and summed in fp64; the order of the sums varies from run to
 * run (atomics), so results agree to ~1e-12 relative, not bit for bit.  Not with sparse_frac > 0.
 */
kvs_status kvs_quant_error(const kvs_desc* desc, const void* K, const void* V, const kvs_cache* cache,
                           const uint8_t* sink_mask, void* report, void* stream);

/*
 * Diagnostic, not part of the method: reads `bytes` (a multiple of 16 is read; src 16-byte aligned)
 * of device memory once, in the launch shape of the decode kernels (256 workgroups of 8 waves,
 * 16 KB of read-once loads in flight per wave) and with no arithmetic.  Its duration is what the
 * memory system alone needs for that many bytes - the ceiling the benchmark prints beside the
 * decode kernel's time.  sink: one device word (written practically never).
 */
kvs_status kvs_probe_stream_read(const void* src, size_t bytes, uint32_t* sink, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* KVS_H */

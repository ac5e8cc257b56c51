"""CPU oracle for the KVSink hot path.  TEST INFRASTRUCTURE ONLY.

A plain, slow numpy statement of what the three library calls compute, written from the
paper (arXiv 2508.04257) and from the readings listed below where the paper is silent.
Only tests, the smoke check and the benchmark's CPU-baseline leg may use this module; the
product path never does, and this module imports nothing from the HIP path.

What is defined by the paper
  * sink prediction: top-k over tokens of |H[i, c]| at the emergence layer's outlier
    channel; the sink set is the set of those tokens               (Algorithm 1, Section 4.3)
  * Preserve-First-N: tokens 0..N-1 kept in 16 bit                  (Section 4.3 / 5.1)
  * asymmetric uniform b-bit quantiser Q(X), X', scale, zero        (Appendix C equations)
  * per-channel Keys (groups along tokens), per-token Values
    (groups along channels), group size G, dynamic statistics       (Section 4.1, Appendix C)
  * K, V rows of sink tokens are left unquantised                   (Algorithm 1)
  * attention softmax(q K^T / sqrt(d_k)) V, split into a sink and a
    non-sink sum                                                    (Section 2; Section 4.2 equation)
  * dense-and-sparse: the largest-magnitude entries are isolated in
    16 bit, 16-bit value + 16-bit index each                        (Section 5.1; Table 2 avg-bits)
  * KV-cache memory accounting                                      (Appendix F table)

Readings taken where the paper is silent (every one is restated in the design notes)
  R1  round = round-half-to-even; all quantiser arithmetic in IEEE fp32, in the order
      written in ``group_params`` / ``quantize_entries``; x / scale is evaluated as
      x * (1 / scale) with one reciprocal per group.
  R2  clipped_max / clipped_min use clip ratio 1 (plain max / min; the paper's
      experiments are round-to-nearest min-max).
  R3  scale is stored as fp16 rounded toward +inf, zero as int16 (4 bytes per group).
  R4  quantisation groups are positional: Key group g of a channel is tokens
      [gG, (g+1)G); kept tokens are left out of the statistics and get code 0.
  R5  degenerate groups: no unmasked entry -> scale 1, zero 0; max == min -> scale |min|
      (1 if min == 0), which reproduces the constant exactly.
  R6  prediction returns exactly k tokens; score = max over the listed channels;
      ties go to the lower token index; each sequence of a batch is handled on its own.
  R7  keep set P_b = first-N tokens united with the predicted sinks.
  R8  dense-and-sparse: per call and per tensor, threshold tau = the magnitude at which the
      descending cumulative count over non-kept entries first reaches ceil(f * count);
      outliers are all entries with |x| >= tau; they are left out of the statistics,
      get code 0 and decode uses their fp16 value in place of the dequantised slot.
  R9  decode attends to the whole cache, no mask; Keys are taken as given (post-RoPE).
  R10 packed layout (a storage decision, not the paper's): see ``pack_k`` / ``pack_v``.
  R13 a growing cache quantises whole 128-token blocks; later tokens wait in fp16 (see
      ``GrowingCache``).
  R14 static quantisation: one parameter pair per Key channel and per Value channel group of a
      KV head, from the global min / max of a calibration that leaves kept tokens out (see
      ``static_params``).
  R15 per-token Keys (the other Key scheme of Section 5.1's comparison): a Key row is quantised
      exactly like a Value row - groups of G consecutive channels of one token - and only the
      parameter array changes shape ([B, Hkv, n, D/G]); the packed Key codes keep their layout.
      With static parameters that is one pair per Key channel group of a KV head.
  R16 error report (the structure of Table 1): squared error of every cache entry of a non-kept
      token, summed separately over quantisation groups that contain a flagged (sink) token and
      groups that do not (see ``quant_error``).
  R18 Algorithm 1's loop order (``prefill_layers``): layers up to and including the emergence
      layer are quantised before the sink set is filled, i.e. without predicted sinks.
  R19 outlier thresholds fixed beforehand (``quantize_kv(..., taus=...)``): every non-kept entry
      whose magnitude pattern reaches the given threshold is isolated, whatever fraction of the
      tensor that turns out to be (the calibrated form of R8, as static quantisation is of R1).
  R17 bit widths 2, 3, 4 and 8 (8: four codes per word, 32 words per 128 codes).  So that the
      zero point always fits its int16, the scale is never taken smaller than |min| / 32766.
      For fp16 data and b <= 4 that bound cannot bind (max - min is at least |min| / 2048);
      at 8 bit it binds for groups whose values lie within 1/128 of their distance from zero,
      where the step it gives, |min| / 32766, is still finer than the fp16 spacing of the data.

PPL / MSE figures of the paper need model weights and datasets: parity unpinned for those
(nothing here reproduces them).  Every function below is pinned by tests/test_oracle_*.py.
"""
from __future__ import annotations

import math
from dataclasses import dataclass
from typing import Optional

import numpy as np

K_TILE = 64      # tokens per Key code tile
V_TILE = 128     # tokens per Value code tile
HEAD_DIM = 128

STATUS_OK = 0
STATUS_CAPACITY = 3


# ----------------------------------------------------------------------------------------
# Sink prediction (Algorithm 1, the "if l = l_E" branch; Section 4.3 items (1)-(3))
# ----------------------------------------------------------------------------------------
def predict_sinks(hidden: np.ndarray, channels, k: int, first_n: int):
    """hidden fp16 [B, n, d] -> (sink_idx int32 [B, k] ascending, keep_mask uint8 [B, n])."""
    H = np.asarray(hidden)
    assert H.dtype == np.float16 and H.ndim == 3
    B, n, _ = H.shape
    channels = list(channels)
    score = np.abs(H[:, :, channels].astype(np.float32)).max(axis=2)           # [B, n]
    sink_idx = np.zeros((B, k), np.int32)
    keep_mask = np.zeros((B, n), np.uint8)
    token = np.arange(n)
    for b in range(B):
        # primary key: score descending; secondary: token index ascending
        order = np.lexsort((token, -score[b]))
        top = np.sort(order[:k])
        sink_idx[b] = top
        keep_mask[b, top] = 1
        keep_mask[b, :first_n] = 1
    return sink_idx, keep_mask


# ----------------------------------------------------------------------------------------
# Quantiser (Appendix C equations for Q(X), X', scale, zero)
# ----------------------------------------------------------------------------------------
def fp32_to_fp16_round_up(x32: np.ndarray) -> np.ndarray:
    """Smallest fp16 that is >= x (x finite, within fp16 range)."""
    x32 = np.asarray(x32, np.float32)
    h = x32.astype(np.float16)
    too_small = h.astype(np.float32) < x32
    return np.where(too_small, np.nextafter(h, np.float16(np.inf)), h).astype(np.float16)


def group_params(mn: np.ndarray, mx: np.ndarray, count: np.ndarray, bits: int):
    """scale (fp16) and zero (int16) of each group from its unmasked min / max / count."""
    qmax = np.float32(2 ** bits - 1)
    empty = np.asarray(count) == 0
    mn = np.where(empty, np.float32(0), mn).astype(np.float32)
    mx = np.where(empty, np.float32(0), mx).astype(np.float32)
    s32 = ((mx - mn) / qmax).astype(np.float32)                 # scale equation
    s32 = np.maximum(s32, (np.abs(mn) / np.float32(32766)).astype(np.float32))   # R17: |zero| <= 32766
    scale_h = fp32_to_fp16_round_up(s32)
    const = mx == mn
    const_scale = np.where(mn != 0, np.abs(mn), np.float32(1)).astype(np.float16)
    scale_h = np.where(const, const_scale, scale_h).astype(np.float16)
    s = scale_h.astype(np.float32)
    inv = (np.float32(1) / s).astype(np.float32)
    zero = (-np.rint((mn * inv).astype(np.float32))).astype(np.int32)   # zero equation
    assert np.all(np.abs(zero) <= 32767), "zero point does not fit int16"
    return scale_h, zero.astype(np.int16)


def quantize_entries(x32: np.ndarray, scale_h: np.ndarray, zero: np.ndarray, bits: int,
                     masked: np.ndarray) -> np.ndarray:
    """Q(X) of every entry (broadcasting the group parameters); masked entries get code 0."""
    qmax = 2 ** bits - 1
    inv = (np.float32(1) / scale_h.astype(np.float32)).astype(np.float32)
    r = np.rint((x32.astype(np.float32) * inv).astype(np.float32)).astype(np.int64)
    code = np.clip(r + zero.astype(np.int64), 0, qmax)
    return np.where(masked, 0, code).astype(np.uint8)


def dequantize_entries(code: np.ndarray, scale_h: np.ndarray, zero: np.ndarray) -> np.ndarray:
    """X' = scale * (Q(X) - zero), one fp32 multiply of an exact integer."""
    d = (code.astype(np.int32) - zero.astype(np.int32)).astype(np.float32)
    return (scale_h.astype(np.float32) * d).astype(np.float32)


def encode_params(scale_h: np.ndarray, zero: np.ndarray) -> np.ndarray:
    """uint32 per group: fp16 scale bits in the low half, int16 zero in the high half."""
    lo = scale_h.astype(np.float16).view(np.uint16).astype(np.uint32)
    hi = zero.astype(np.int16).view(np.uint16).astype(np.uint32)
    return lo | (hi << np.uint32(16))


def decode_params(p: np.ndarray):
    p = np.asarray(p, np.uint32)
    scale_h = (p & np.uint32(0xFFFF)).astype(np.uint16).view(np.float16)
    zero = (p >> np.uint32(16)).astype(np.uint16).view(np.int16)
    return scale_h, zero


def quantize_k_head(K: np.ndarray, masked: np.ndarray, bits: int, G: int):
    """Per-channel Key quantisation of one head.  K fp16 [n, D]; masked bool [n, D].

    Group g of channel c = tokens [gG, (g+1)G).  Returns codes uint8 [n, D] and the
    parameters (scale fp16, zero int16), each [n/G, D]."""
    n, D = K.shape
    x = K.astype(np.float32).reshape(n // G, G, D)
    m = masked.reshape(n // G, G, D)
    mn = np.where(m, np.float32(np.inf), x).min(axis=1)
    mx = np.where(m, np.float32(-np.inf), x).max(axis=1)
    cnt = (~m).sum(axis=1)
    scale_h, zero = group_params(mn, mx, cnt, bits)
    codes = quantize_entries(x, scale_h[:, None, :], zero[:, None, :], bits, m)
    return codes.reshape(n, D), scale_h, zero


def quantize_v_head(V: np.ndarray, masked: np.ndarray, bits: int, G: int):
    """Per-token Value quantisation of one head.  Group j of token t = channels [jG, (j+1)G).
    Returns codes uint8 [n, D] and parameters [n, D/G]."""
    n, D = V.shape
    x = V.astype(np.float32).reshape(n, D // G, G)
    m = masked.reshape(n, D // G, G)
    mn = np.where(m, np.float32(np.inf), x).min(axis=2)
    mx = np.where(m, np.float32(-np.inf), x).max(axis=2)
    cnt = (~m).sum(axis=2)
    scale_h, zero = group_params(mn, mx, cnt, bits)
    codes = quantize_entries(x, scale_h[:, :, None], zero[:, :, None], bits, m)
    return codes.reshape(n, D), scale_h, zero


# ----------------------------------------------------------------------------------------
# Packed layout (storage decision R10)
# ----------------------------------------------------------------------------------------
def codes_per_word(bits: int) -> int:
    return {2: 16, 3: 10, 4: 8, 8: 4}[bits]


def words_per_128(bits: int) -> int:
    return -(-128 // codes_per_word(bits))          # 8, 13, 16, 32


def slot_shift(bits: int, j: int) -> int:
    """Bit offset of slot j inside a 32-bit word.  2, 4 and 8 bit: contiguous from bit 0.
    3 bit: five codes in bits 0-14, five in bits 16-30; bits 15 and 31 stay zero."""
    if bits == 3:
        return 3 * (j % 5) + 16 * (j // 5)
    return bits * j


def _pack_last_axis(codes: np.ndarray, bits: int) -> np.ndarray:
    """codes uint8 [..., 128] -> uint32 [..., W]; slot j of word w is element cpw*w + j;
    slots past element 127 are zero."""
    cpw, W = codes_per_word(bits), words_per_128(bits)
    assert codes.shape[-1] == 128
    out = np.zeros(codes.shape[:-1] + (W,), np.uint32)
    for w in range(W):
        for j in range(cpw):
            e = cpw * w + j
            if e < 128:
                out[..., w] |= codes[..., e].astype(np.uint32) << np.uint32(slot_shift(bits, j))
    return out


def _unpack_last_axis(words: np.ndarray, bits: int) -> np.ndarray:
    cpw, W = codes_per_word(bits), words_per_128(bits)
    assert words.shape[-1] == W
    out = np.zeros(words.shape[:-1] + (128,), np.uint8)
    mask = np.uint32(2 ** bits - 1)
    for w in range(W):
        for j in range(cpw):
            e = cpw * w + j
            if e < 128:
                out[..., e] = ((words[..., w] >> np.uint32(slot_shift(bits, j))) & mask).astype(np.uint8)
    return out


def pack_k(codes: np.ndarray, bits: int) -> np.ndarray:
    """Key codes uint8 [n, 128] -> uint32 [n/64, W, 64].
    Word (T, w, t) holds channels cpw*w .. of token 64*T + t (word-major, token-minor tiles)."""
    n = codes.shape[0]
    assert n % K_TILE == 0
    words = _pack_last_axis(codes, bits)                             # [n, W]
    return np.ascontiguousarray(words.reshape(n // K_TILE, K_TILE, -1).transpose(0, 2, 1))


def unpack_k(words: np.ndarray, bits: int) -> np.ndarray:
    T, W, t = words.shape
    return _unpack_last_axis(np.ascontiguousarray(words.transpose(0, 2, 1)).reshape(T * t, W), bits)


def pack_v(codes: np.ndarray, bits: int) -> np.ndarray:
    """Value codes uint8 [n, 128] -> uint32 [n/128, W, 128].
    Word (T, u, c) holds tokens 128*T + cpw*u .. of channel c (packed along tokens)."""
    n, D = codes.shape
    assert n % V_TILE == 0 and D == 128
    per_channel = np.ascontiguousarray(codes.reshape(n // V_TILE, V_TILE, D).transpose(0, 2, 1))  # [T, c, 128 tok]
    words = _pack_last_axis(per_channel, bits)                       # [T, c, W]
    return np.ascontiguousarray(words.transpose(0, 2, 1))            # [T, W, c]


def unpack_v(words: np.ndarray, bits: int) -> np.ndarray:
    T, W, D = words.shape
    per_channel = _unpack_last_axis(np.ascontiguousarray(words.transpose(0, 2, 1)), bits)  # [T, c, 128 tok]
    return np.ascontiguousarray(per_channel.transpose(0, 2, 1)).reshape(T * V_TILE, D)


# ----------------------------------------------------------------------------------------
# Dense-and-sparse threshold (reading R8)
# ----------------------------------------------------------------------------------------
def sparse_threshold(X: np.ndarray, keep_mask: np.ndarray, frac: float) -> int:
    """X fp16 [B, H, n, D], keep_mask [B, n].  Returns tau as a 15-bit fp16 magnitude pattern
    (0x7FFF + 1 = 32768 when nothing is isolated)."""
    X = np.asarray(X)
    hist = np.zeros(32768, np.int64)
    for b in range(X.shape[0]):                                   # one sequence at a time (memory)
        mag = X[b].view(np.uint16) & np.uint16(0x7FFF)            # [H, n, D]
        live = np.asarray(keep_mask[b]) == 0
        hist += np.bincount(mag[:, live, :].ravel(), minlength=32768)
    count = int(hist.sum())
    m = int(math.ceil(float(np.float32(frac)) * count))
    if m <= 0:
        return 32768
    cum = 0
    for bin_ in range(32767, -1, -1):
        cum += int(hist[bin_])
        if cum >= m:
            return bin_
    return 0


# ----------------------------------------------------------------------------------------
# The quantised cache of one layer
# ----------------------------------------------------------------------------------------
@dataclass
class Cache:
    B: int
    n: int
    Hkv: int
    D: int
    bits: int
    group: int
    keep_cap: int
    k_codes: np.ndarray            # uint32 [B, Hkv, n/64, W, 64]
    v_codes: np.ndarray            # uint32 [B, Hkv, n/128, W, 128]
    k_params: np.ndarray           # uint32 [B, Hkv, n/G, D]; per-token Keys: [B, Hkv, n, D/G]
    v_params: np.ndarray           # uint32 [B, Hkv, n, D/G]
    keep_k: np.ndarray             # fp16 [B, Hkv, cap, D]
    keep_v: np.ndarray
    keep_idx: np.ndarray           # int32 [B, cap], ascending, -1 padded
    keep_cnt: np.ndarray           # int32 [B]
    keep_mask: np.ndarray          # uint8 [B, n]
    status: int = STATUS_OK
    # dense-and-sparse part (None when off).  Keys: CSR over rows (b, h, token), column =
    # channel.  Values: CSR over rows (b, h, 128-token tile, channel), column = token inside
    # the tile - the same transposition as the Value code tiles.  Columns ascend in a row.
    k_rowptr: Optional[np.ndarray] = None
    k_col: Optional[np.ndarray] = None
    k_val: Optional[np.ndarray] = None
    v_rowptr: Optional[np.ndarray] = None
    v_col: Optional[np.ndarray] = None
    v_val: Optional[np.ndarray] = None
    k_tau: int = 32768
    v_tau: int = 32768
    # logical (unpacked) codes, kept for tests
    k_codes_logical: Optional[np.ndarray] = None    # uint8 [B, Hkv, n, D]
    v_codes_logical: Optional[np.ndarray] = None
    key_per_token: bool = False    # Keys quantised per token (groups along channels), like Values


def _csr_from_mask(X: np.ndarray, outlier: np.ndarray, by_channel: bool):
    """CSR of the flagged entries, col uint16, val = the original fp16.
    by_channel False: rows (b, h, t), column = channel.
    by_channel True:  rows (b, h, T, c) with T the 128-token tile, column = t - 128 T."""
    B, H, n, D = X.shape
    if by_channel:
        X = X.reshape(B, H, n // V_TILE, V_TILE, D).transpose(0, 1, 2, 4, 3)
        outlier = outlier.reshape(B, H, n // V_TILE, V_TILE, D).transpose(0, 1, 2, 4, 3)
    flat = outlier.reshape(B * H * n, D)
    counts = flat.sum(axis=1)
    rowptr = np.zeros(B * H * n + 1, np.int64)
    np.cumsum(counts, out=rowptr[1:])
    rows, cols = np.nonzero(flat)                    # row-major order: rows ascending, then columns
    vals = X.reshape(B * H * n, D)[rows, cols]
    return rowptr.astype(np.int32), cols.astype(np.uint16), vals.astype(np.float16)


def quantize_kv(K: np.ndarray, V: np.ndarray, keep_mask: np.ndarray, bits: int, group: int,
                keep_cap: int, sparse_frac: float = 0.0, sparse_cap: Optional[int] = None,
                taus: Optional[tuple] = None, key_per_token: bool = False) -> Cache:
    """Algorithm 1's two quantise steps for one layer: K and V rows of tokens outside the
    keep set are quantised, rows inside it are copied unchanged into the fp16 side buffer.
    ``taus`` = (k_tau, v_tau) supplies the thresholds instead of searching them: those that
    ``sparse_threshold`` found on a larger tensor of which K, V are a slice (the threshold is a
    property of the whole layer), or thresholds fixed on other data beforehand (R19).
    ``key_per_token`` selects the per-token Key scheme (Section 5.1; reading R15)."""
    K = np.asarray(K)
    V = np.asarray(V)
    assert K.dtype == np.float16 and V.dtype == np.float16 and K.shape == V.shape
    B, H, n, D = K.shape
    assert D == HEAD_DIM and n % V_TILE == 0 and n % group == 0 and D % group == 0
    keep_mask = (np.asarray(keep_mask) != 0).astype(np.uint8)
    kept = keep_mask.astype(bool)
    W = words_per_128(bits)
    status = STATUS_OK

    tau_k = tau_v = 32768
    if sparse_frac > 0 and taus is not None:
        tau_k, tau_v = taus
    elif sparse_frac > 0:
        tau_k = sparse_threshold(K, keep_mask, sparse_frac)
        tau_v = sparse_threshold(V, keep_mask, sparse_frac)
    not_kept = (~kept)[:, None, :, None]
    out_k = ((K.view(np.uint16) & np.uint16(0x7FFF)) >= tau_k) & not_kept
    out_v = ((V.view(np.uint16) & np.uint16(0x7FFF)) >= tau_v) & not_kept

    k_codes = np.zeros((B, H, n // K_TILE, W, K_TILE), np.uint32)
    v_codes = np.zeros((B, H, n // V_TILE, W, V_TILE), np.uint32)
    k_params = np.zeros((B, H, n, D // group) if key_per_token else (B, H, n // group, D), np.uint32)
    v_params = np.zeros((B, H, n, D // group), np.uint32)
    k_log = np.zeros((B, H, n, D), np.uint8)
    v_log = np.zeros((B, H, n, D), np.uint8)
    for b in range(B):
        row_mask = np.broadcast_to(kept[b][:, None], (n, D))
        for h in range(H):
            quantize_keys = quantize_v_head if key_per_token else quantize_k_head
            ck, sk, zk = quantize_keys(K[b, h], row_mask | out_k[b, h], bits, group)
            cv, sv, zv = quantize_v_head(V[b, h], row_mask | out_v[b, h], bits, group)
            k_log[b, h], v_log[b, h] = ck, cv
            k_codes[b, h], v_codes[b, h] = pack_k(ck, bits), pack_v(cv, bits)
            k_params[b, h], v_params[b, h] = encode_params(sk, zk), encode_params(sv, zv)

    keep_k = np.zeros((B, H, keep_cap, D), np.float16)
    keep_v = np.zeros((B, H, keep_cap, D), np.float16)
    keep_idx = np.full((B, keep_cap), -1, np.int32)
    keep_cnt = np.zeros(B, np.int32)
    for b in range(B):
        idx = np.nonzero(kept[b])[0]
        keep_cnt[b] = len(idx)
        if len(idx) > keep_cap:
            status = STATUS_CAPACITY
            idx = idx[:keep_cap]
        keep_idx[b, :len(idx)] = idx
        keep_k[b, :, :len(idx)] = K[b][:, idx]
        keep_v[b, :, :len(idx)] = V[b][:, idx]

    cache = Cache(B, n, H, D, bits, group, keep_cap, k_codes, v_codes, k_params, v_params,
                  keep_k, keep_v, keep_idx, keep_cnt, keep_mask, status,
                  k_tau=tau_k, v_tau=tau_v, k_codes_logical=k_log, v_codes_logical=v_log,
                  key_per_token=key_per_token)
    if sparse_frac > 0:
        cache.k_rowptr, cache.k_col, cache.k_val = _csr_from_mask(K, out_k, by_channel=False)
        cache.v_rowptr, cache.v_col, cache.v_val = _csr_from_mask(V, out_v, by_channel=True)
        if sparse_cap is not None and max(len(cache.k_col), len(cache.v_col)) > sparse_cap:
            cache.status = STATUS_CAPACITY
    return cache


# ----------------------------------------------------------------------------------------
# Decode attention over the quantised cache (Section 2 attention equation; the split into
# sink and non-sink tokens is the equation of Section 4.2)
# ----------------------------------------------------------------------------------------
def effective_kv(cache: Cache, b: int, h: int):
    """K', V' float64 [n, D] as the decode step sees them: dequantised entries, sparse
    outliers replaced by their fp16 value, kept rows replaced by the fp16 side buffer."""
    n, D, G, bits = cache.n, cache.D, cache.group, cache.bits
    sk, zk = decode_params(cache.k_params[b, h])                     # [n/G, D] ([n, D/G] per token)
    sv, zv = decode_params(cache.v_params[b, h])                     # [n, D/G]
    ck = unpack_k(cache.k_codes[b, h], bits)                         # [n, D]
    cv = unpack_v(cache.v_codes[b, h], bits)
    if cache.key_per_token:
        Kd = dequantize_entries(ck.reshape(n, D // G, G), sk[:, :, None], zk[:, :, None]).reshape(n, D)
    else:
        Kd = dequantize_entries(ck.reshape(n // G, G, D), sk[:, None, :], zk[:, None, :]).reshape(n, D)
    Vd = dequantize_entries(cv.reshape(n, D // G, G), sv[:, :, None], zv[:, :, None]).reshape(n, D)
    Kd = Kd.astype(np.float64)
    Vd = Vd.astype(np.float64)
    if cache.k_rowptr is not None:
        base = (b * cache.Hkv + h) * n                      # both CSRs have n rows per (b, h)
        lo, hi = int(cache.k_rowptr[base]), int(cache.k_rowptr[base + n])
        rows = np.repeat(np.arange(n), np.diff(cache.k_rowptr[base:base + n + 1].astype(np.int64)))
        Kd[rows, cache.k_col[lo:hi].astype(np.int64)] = cache.k_val[lo:hi].astype(np.float64)
        lo, hi = int(cache.v_rowptr[base]), int(cache.v_rowptr[base + n])
        rows = np.repeat(np.arange(n), np.diff(cache.v_rowptr[base:base + n + 1].astype(np.int64)))
        tile, chan = rows // D, rows % D                    # row = tile * 128 + channel
        Vd[tile * V_TILE + cache.v_col[lo:hi].astype(np.int64), chan] = cache.v_val[lo:hi].astype(np.float64)
    for j in range(min(int(cache.keep_cnt[b]), cache.keep_cap)):
        t = int(cache.keep_idx[b, j])
        Kd[t] = cache.keep_k[b, h, j].astype(np.float64)
        Vd[t] = cache.keep_v[b, h, j].astype(np.float64)
    return Kd, Vd


def attention_row(q: np.ndarray, Kp: np.ndarray, Vp: np.ndarray):
    """softmax(q K'^T / sqrt(d_k)) V' for one query row, fp64.  Returns (o [D], lse, p [n])."""
    s = (Kp @ q.astype(np.float64)) / math.sqrt(Kp.shape[1])
    m = s.max()
    e = np.exp(s - m)
    l = e.sum()
    p = e / l
    return p @ Vp, m + math.log(l), p


def decode_attn(q: np.ndarray, cache: Cache, Hq: int, pairs=None):
    """q fp16 [B, Hq, D] -> (out fp16 [B, Hq, D], lse float32 [B, Hq], out64).
    Query head hq reads KV head hq // (Hq / Hkv).  ``pairs`` restricts the work to a list
    of (b, hq); other rows of the result stay zero."""
    q = np.asarray(q)
    assert q.dtype == np.float16
    B, D = cache.B, cache.D
    rep = Hq // cache.Hkv
    out64 = np.zeros((B, Hq, D), np.float64)
    lse = np.zeros((B, Hq), np.float32)
    todo = pairs if pairs is not None else [(b, hq) for b in range(B) for hq in range(Hq)]
    memo = {}
    for b, hq in todo:
        h = hq // rep
        if (b, h) not in memo:
            memo.clear()
            memo[(b, h)] = effective_kv(cache, b, h)
        Kp, Vp = memo[(b, h)]
        o, l, _ = attention_row(q[b, hq], Kp, Vp)
        out64[b, hq] = o
        lse[b, hq] = l
    return out64.astype(np.float16), lse, out64


# ----------------------------------------------------------------------------------------
# A cache that grows during decoding (Section 2, "KV cache": K_cache <- concat(K_cache, t_K),
# V_cache <- concat(V_cache, t_V)).  Reading R13: quantisation groups are positional and the
# largest one spans 128 tokens (the Value code tile), so tokens are quantised in whole
# 128-token blocks; the tokens after the last whole block wait in fp16 (the residual window)
# until their block is complete, and the block is then quantised like any other - the
# accumulate-then-quantise scheme Appendix A describes for dynamic per-channel methods.
# Consequence, pinned by the tests: the state after any number of appends equals the state a
# prefill of the same tokens produces.
# ----------------------------------------------------------------------------------------
BLOCK = V_TILE


@dataclass
class GrowingCache:
    bits: int
    group: int
    keep_cap: int
    n_tokens: int
    quant: Optional[Cache]         # tokens [0, n_quant), n_quant = 128 * (n_tokens // 128); None if 0
    res_k: np.ndarray              # fp16 [B, Hkv, n_tokens - n_quant, D]
    res_v: np.ndarray
    res_mask: np.ndarray           # uint8 [B, n_tokens - n_quant]: keep flags of the residual tokens
    key_per_token: bool = False

    @property
    def n_quant(self) -> int:
        return 0 if self.quant is None else self.quant.n


def _concat_caches(a: Optional[Cache], b: Cache) -> Cache:
    """Cache over the tokens of ``a`` followed by those of ``b`` (both whole blocks)."""
    if a is None:
        return b
    cap = a.keep_cap
    keep_k, keep_v, keep_idx = a.keep_k.copy(), a.keep_v.copy(), a.keep_idx.copy()
    keep_cnt = a.keep_cnt + b.keep_cnt
    status = max(a.status, b.status)
    for bi in range(a.B):
        ca, cb = int(a.keep_cnt[bi]), int(b.keep_cnt[bi])
        for j in range(min(cb, b.keep_cap)):
            if ca + j < cap:
                keep_idx[bi, ca + j] = b.keep_idx[bi, j] + a.n
                keep_k[bi, :, ca + j] = b.keep_k[bi, :, j]
                keep_v[bi, :, ca + j] = b.keep_v[bi, :, j]
            else:
                status = STATUS_CAPACITY
    cat = lambda x, y, ax: np.concatenate([x, y], axis=ax)
    return Cache(a.B, a.n + b.n, a.Hkv, a.D, a.bits, a.group, cap,
                 cat(a.k_codes, b.k_codes, 2), cat(a.v_codes, b.v_codes, 2),
                 cat(a.k_params, b.k_params, 2), cat(a.v_params, b.v_params, 2),
                 keep_k, keep_v, keep_idx, keep_cnt, cat(a.keep_mask, b.keep_mask, 1), status,
                 k_codes_logical=cat(a.k_codes_logical, b.k_codes_logical, 2),
                 v_codes_logical=cat(a.v_codes_logical, b.v_codes_logical, 2),
                 key_per_token=a.key_per_token)


def prefill_cache(K: np.ndarray, V: np.ndarray, keep_mask: np.ndarray, bits: int, group: int,
                  keep_cap: int, key_per_token: bool = False) -> GrowingCache:
    """Cache of a prompt of any length: whole 128-token blocks quantised, the rest in fp16."""
    K, V = np.asarray(K), np.asarray(V)
    B, H, n, D = K.shape
    keep_mask = (np.asarray(keep_mask) != 0).astype(np.uint8)
    nq = (n // BLOCK) * BLOCK
    quant = quantize_kv(K[:, :, :nq], V[:, :, :nq], keep_mask[:, :nq], bits, group, keep_cap,
                        key_per_token=key_per_token) if nq else None
    return GrowingCache(bits, group, keep_cap, n, quant, K[:, :, nq:].copy(), V[:, :, nq:].copy(),
                        keep_mask[:, nq:].copy(), key_per_token)


def append_token(gc: GrowingCache, k_new: np.ndarray, v_new: np.ndarray, keep_new=None) -> GrowingCache:
    """One decoding step's cache update: k_new, v_new fp16 [B, Hkv, D] join the residual window;
    a window that reaches 128 tokens is quantised as one block and joins the quantised part."""
    k_new, v_new = np.asarray(k_new), np.asarray(v_new)
    assert k_new.dtype == np.float16 and v_new.dtype == np.float16
    B = k_new.shape[0]
    flag = np.zeros((B, 1), np.uint8) if keep_new is None else (np.asarray(keep_new).reshape(B, 1) != 0).astype(np.uint8)
    res_k = np.concatenate([gc.res_k, k_new[:, :, None, :]], axis=2)
    res_v = np.concatenate([gc.res_v, v_new[:, :, None, :]], axis=2)
    res_mask = np.concatenate([gc.res_mask, flag], axis=1)
    quant = gc.quant
    if res_k.shape[2] == BLOCK:
        block = quantize_kv(res_k, res_v, res_mask, gc.bits, gc.group, gc.keep_cap,
                            key_per_token=gc.key_per_token)
        quant = _concat_caches(quant, block)
        res_k, res_v, res_mask = res_k[:, :, :0], res_v[:, :, :0], res_mask[:, :0]
    return GrowingCache(gc.bits, gc.group, gc.keep_cap, gc.n_tokens + 1, quant, res_k, res_v, res_mask,
                        gc.key_per_token)


def decode_attn_growing(q: np.ndarray, gc: GrowingCache, Hq: int):
    """Decode attention over all n_tokens cached tokens: the quantised part as ``decode_attn``
    sees it, the residual tokens in fp16.  Returns (out fp16, lse float32, out64)."""
    q = np.asarray(q)
    B, D = q.shape[0], q.shape[2]
    H = gc.res_k.shape[1]
    rep = Hq // H
    out64 = np.zeros((B, Hq, D), np.float64)
    lse = np.zeros((B, Hq), np.float32)
    for b in range(B):
        for h in range(H):
            Kp, Vp = gc.res_k[b, h].astype(np.float64), gc.res_v[b, h].astype(np.float64)
            if gc.quant is not None:
                Kq, Vq = effective_kv(gc.quant, b, h)
                Kp, Vp = np.concatenate([Kq, Kp]), np.concatenate([Vq, Vp])
            for r in range(rep):
                o, l, _ = attention_row(q[b, h * rep + r], Kp, Vp)
                out64[b, h * rep + r] = o
                lse[b, h * rep + r] = l
    return out64.astype(np.float16), lse, out64


# ----------------------------------------------------------------------------------------
# Static quantisation (Appendix C, "Dynamic and static quantization": the range is estimated
# from calibration data before inference and the parameters stay fixed; Section 4.1 / Table 1:
# global min-max, and Algorithm 1's note that sink tokens are excluded from the calibration
# too).  Reading R14: one parameter pair per Key channel of a KV head (per-channel scheme: the
# token groups of the dynamic scheme collapse into one) and one per Value channel group of a
# KV head (per-token scheme with fixed parameters), from the global min / max over every
# non-kept token the calibration has seen; values outside the calibrated range clamp to code
# 0 or qmax (the clamp of the Q(X) equation).
# ----------------------------------------------------------------------------------------
@dataclass
class Calibration:
    k_min: np.ndarray   # float32 [Hkv, D], +inf where nothing was seen
    k_max: np.ndarray
    v_min: np.ndarray   # float32 [Hkv, D] (per channel; reduced to channel groups by static_params)
    v_max: np.ndarray


def new_calibration(Hkv: int, D: int = HEAD_DIM) -> Calibration:
    inf = np.full((Hkv, D), np.inf, np.float32)
    return Calibration(inf.copy(), -inf, inf.copy(), -inf.copy())


def calibrate(cal: Calibration, K: np.ndarray, V: np.ndarray, keep_mask: np.ndarray) -> Calibration:
    """Running global min / max per (KV head, channel) over the tokens outside the keep set."""
    K, V = np.asarray(K), np.asarray(V)
    B, H, n, D = K.shape
    kept = (np.asarray(keep_mask) != 0)[:, None, :, None]
    Kf, Vf = K.astype(np.float32), V.astype(np.float32)
    hi, lo = np.float32(np.inf), np.float32(-np.inf)
    return Calibration(
        np.minimum(cal.k_min, np.where(kept, hi, Kf).min(axis=(0, 2))),
        np.maximum(cal.k_max, np.where(kept, lo, Kf).max(axis=(0, 2))),
        np.minimum(cal.v_min, np.where(kept, hi, Vf).min(axis=(0, 2))),
        np.maximum(cal.v_max, np.where(kept, lo, Vf).max(axis=(0, 2))))


def static_params(cal: Calibration, bits: int, group: int, key_per_token: bool = False):
    """Parameter words: Keys uint32 [Hkv, D] (one per channel; per-token Keys: [Hkv, D/G], one per
    channel group), Values uint32 [Hkv, D/G] (one per channel group), by the same scale / zero
    equations as the dynamic scheme."""
    H, D = cal.k_min.shape
    kmn, kmx = cal.k_min, cal.k_max
    if key_per_token:
        kmn = kmn.reshape(H, D // group, group).min(axis=2)
        kmx = kmx.reshape(H, D // group, group).max(axis=2)
    sk, zk = group_params(kmn, kmx, (kmn <= kmx).astype(np.int64), bits)
    vmn = cal.v_min.reshape(H, D // group, group).min(axis=2)
    vmx = cal.v_max.reshape(H, D // group, group).max(axis=2)
    sv, zv = group_params(vmn, vmx, (vmn <= vmx).astype(np.int64), bits)
    return encode_params(sk, zk), encode_params(sv, zv)


def quantize_kv_static(K: np.ndarray, V: np.ndarray, keep_mask: np.ndarray, bits: int, group: int,
                       keep_cap: int, k_static: np.ndarray, v_static: np.ndarray,
                       key_per_token: bool = False) -> Cache:
    """As quantize_kv, with the given fixed parameters instead of per-group statistics.  The cache
    has the same layout: every group's parameter word is its channel's (channel group's) static
    word, so the decode step reads it like any other cache."""
    dyn = quantize_kv(K, V, keep_mask, bits, group, keep_cap, key_per_token=key_per_token)   # layout, keep rows, mask
    B, H, n, D = K.shape
    kept = (np.asarray(keep_mask) != 0)
    sk, zk = decode_params(k_static)                               # [H, D] ([H, D/G] per token)
    sv, zv = decode_params(v_static)                               # [H, D/G]
    for b in range(B):
        row_mask = np.broadcast_to(kept[b][:, None], (n, D))
        for h in range(H):
            if key_per_token:
                xk = K[b, h].astype(np.float32).reshape(n, D // group, group)
                ck = quantize_entries(xk, sk[h][None, :, None], zk[h][None, :, None], bits,
                                      row_mask.reshape(n, D // group, group)).reshape(n, D)
            else:
                ck = quantize_entries(K[b, h].astype(np.float32), sk[h][None, :], zk[h][None, :], bits, row_mask)
            xv = V[b, h].astype(np.float32).reshape(n, D // group, group)
            cv = quantize_entries(xv, sv[h][None, :, None], zv[h][None, :, None], bits,
                                  row_mask.reshape(n, D // group, group)).reshape(n, D)
            dyn.k_codes_logical[b, h], dyn.v_codes_logical[b, h] = ck, cv
            dyn.k_codes[b, h], dyn.v_codes[b, h] = pack_k(ck, bits), pack_v(cv, bits)
            dyn.k_params[b, h] = np.broadcast_to(np.asarray(k_static, np.uint32)[h][None, :], dyn.k_params[b, h].shape)
            dyn.v_params[b, h] = np.broadcast_to(np.asarray(v_static, np.uint32)[h][None, :], (n, D // group))
    return dyn


# ----------------------------------------------------------------------------------------
# Quantisation-error report (Section 4.1, Table 1: mean squared error of the quantised Keys and
# Values, overall and split into the quantisation groups that contain a sink token and those that
# do not).  Reading R16: the error of an entry is x - x' with x' what the decode step sees; entries
# of kept tokens are stored exactly and are left out of sums and counts; a per-channel Key group
# (G consecutive tokens of one channel) "contains a sink" if any of its tokens is flagged in
# ``sink_mask``, a per-token group (G channels of one token) if its token is.  ``sink_mask`` only
# classifies: whether the flagged tokens were kept or quantised is the cache's business.
# ----------------------------------------------------------------------------------------
def quant_error(K: np.ndarray, V: np.ndarray, cache: Cache, sink_mask: np.ndarray):
    """-> {"k": (sse_without, n_without, sse_with, n_with), "v": (...)}: sums of squared errors
    (float64) and entry counts (int) over the two classes of groups."""
    K, V = np.asarray(K), np.asarray(V)
    B, H, n, D = K.shape
    G = cache.group
    flagged = np.asarray(sink_mask) != 0                                        # [B, n]
    in_group = flagged.reshape(B, n // G, G).any(axis=2).repeat(G, axis=1)      # token's Key group holds a sink
    counted = cache.keep_mask == 0
    out = {}
    for name, X, cls in (("k", K, flagged if cache.key_per_token else in_group), ("v", V, flagged)):
        sse = [0.0, 0.0]
        cnt = [0, 0]
        for b in range(B):
            for h in range(H):
                Kd, Vd = effective_kv(cache, b, h)
                err = X[b, h].astype(np.float64) - (Kd if name == "k" else Vd)
                for c in (0, 1):
                    rows = counted[b] & (cls[b] == bool(c))
                    sse[c] += float((err[rows] ** 2).sum())
                    cnt[c] += int(rows.sum()) * D
        out[name] = (sse[0], cnt[0], sse[1], cnt[1])
    return out


# ----------------------------------------------------------------------------------------
# The prefill loop of Algorithm 1, the part that needs no model: the order in which the layers'
# K, V are quantised and the sink set is filled.
#   S_sink starts empty; layer l = 1 .. L quantises K^l, V^l leaving out the tokens in S_sink as it
#   stands when the layer runs; after layer l_E the set becomes the top-k tokens of |H^{l_E}[:, c]|.
# So layers 1 .. l_E are quantised without any predicted sink (only the first-N tokens of the
# PFN policy, when N > 0, are kept there), layers l_E + 1 .. L with the predicted set.
# ----------------------------------------------------------------------------------------
def prefill_layers(Ks, Vs, hidden_at_emergence: np.ndarray, emergence_layer: int, channels, k: int,
                   first_n: int, bits: int, group: int, keep_cap: int, sparse_frac: float = 0.0,
                   sparse_cap: Optional[int] = None, key_per_token: bool = False):
    """Ks, Vs: lists of L tensors fp16 [B, Hkv, n, D] (layer 1 first); hidden_at_emergence fp16
    [B, n, d] = H^{l_E}; emergence_layer = l_E in [0, L] (0: the set is known before layer 1).
    Returns (caches [L], sink_idx int32 [B, k], early_mask uint8 [B, n], keep_mask uint8 [B, n])."""
    L = len(Ks)
    assert len(Vs) == L and 0 <= emergence_layer <= L
    B, _, n, _ = np.asarray(Ks[0]).shape
    sink = np.zeros((B, n), bool)                      # S_sink = {} (per sequence)
    first = np.zeros((B, n), bool)
    first[:, :first_n] = True
    sink_idx = None
    early_mask = first.astype(np.uint8)
    keep_mask = None

    def fill():                                        # the "if l = l_E" branch
        idx, _ = predict_sinks(hidden_at_emergence, channels, k, 0)
        s = np.zeros((B, n), bool)
        for b in range(B):
            s[b, idx[b]] = True
        return idx, s

    if emergence_layer == 0:
        sink_idx, sink = fill()
    caches = []
    for l in range(1, L + 1):
        mask = (sink | first).astype(np.uint8)         # token not in S_sink (nor among the first N) -> quantised
        caches.append(quantize_kv(Ks[l - 1], Vs[l - 1], mask, bits, group, keep_cap, sparse_frac=sparse_frac,
                                  sparse_cap=sparse_cap, key_per_token=key_per_token))
        if l == emergence_layer:
            sink_idx, sink = fill()
    keep_mask = (sink | first).astype(np.uint8)
    return caches, sink_idx, early_mask, keep_mask


# ----------------------------------------------------------------------------------------
# Memory accounting (Appendix F table; Table 2's average-bits column)
# ----------------------------------------------------------------------------------------
def kv_cache_bytes(n_tokens: int, layers: int, kv_width: int, bits: int) -> float:
    """Bytes of K and V codes for n tokens (kv_width = H_kv * D), parameters excluded, as
    the paper's estimate does."""
    return n_tokens * layers * 2 * kv_width * bits / 8.0


def preserved_token_bytes(k_tokens: int, layers: int, kv_width: int) -> float:
    """Extra bytes of k tokens kept in fp16 (K and V rows, every layer)."""
    return k_tokens * layers * 2 * kv_width * 2.0


def average_bits(bits: int, sparse_frac: float) -> float:
    """Average bits per cache entry with a fraction of entries held as 16-bit value + 16-bit index."""
    return bits + 32.0 * sparse_frac

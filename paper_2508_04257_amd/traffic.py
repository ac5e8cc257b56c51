"""Algorithmic bytes of the calls: what a call must move at the least, the numerator of every
bandwidth figure the benchmark and the shape sweep report."""


def decode_algorithmic_bytes(w, keep_rows_per_seq: int) -> int:
    """Bytes one kvs_decode_attn call must move: packed codes, 4-byte parameter words, the keep
    mask, the fp16 keep rows, q and out.  (Not the fp16 cache it avoids reading.)"""
    W = {2: 8, 3: 13, 4: 16, 8: 32}[w.bits]
    bh = w.B * w.Hkv
    codes = 2 * bh * w.n * W * 4
    params = bh * (w.n // w.group) * w.D * 4 + bh * w.n * (w.D // w.group) * 4
    keep = 2 * bh * keep_rows_per_seq * w.D * 2 + w.B * w.n
    qo = 2 * w.B * w.Hq * w.D * 2
    return codes + params + keep + qo


def quantize_algorithmic_bytes(w) -> int:
    """fp16 K and V read once, codes and parameters written once."""
    W = {2: 8, 3: 13, 4: 16, 8: 32}[w.bits]
    bh = w.B * w.Hkv
    read = 2 * bh * w.n * w.D * 2 + w.B * w.n
    write = 2 * bh * w.n * W * 4 + bh * (w.n // w.group) * w.D * 4 + bh * w.n * (w.D // w.group) * 4
    return read + write

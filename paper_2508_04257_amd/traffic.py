"""Algorithmic bytes of the calls: what a call must move at the least, the numerator of every
bandwidth figure the benchmark reports."""

_WORDS = {2: 8, 3: 13, 4: 16, 8: 32}


def csr_bytes(w, nnz_k: int, nnz_v: int) -> int:
    """Isolated fp16 outliers of one layer: 16-bit value + 16-bit index per entry, one 32-bit
    row pointer per (sequence, KV head, token) row and tensor."""
    rows = w.B * w.Hkv * w.n
    return 4 * (nnz_k + nnz_v) + 2 * 4 * (rows + 1)


def expected_nnz(w) -> int:
    """Entries per tensor that the requested fraction isolates (ties at the threshold add a few)."""
    return int(w.B * w.Hkv * w.n * w.D * w.sparse_frac)


def decode_algorithmic_bytes(w, keep_rows_per_seq: int, nnz=None) -> int:
    """Bytes one kvs_decode_attn call must move: packed codes, 4-byte parameter words, the keep
    mask, the fp16 keep rows, the isolated outliers' CSR arrays, q and out.  (Not the fp16 cache
    it avoids reading.)  nnz = (Key entries, Value entries) of a dense-and-sparse cache; where it
    is not given the requested fraction stands in."""
    W = _WORDS[w.bits]
    bh = w.B * w.Hkv
    codes = 2 * bh * w.n * W * 4
    params = bh * (w.n // w.group) * w.D * 4 + bh * w.n * (w.D // w.group) * 4
    keep = 2 * bh * keep_rows_per_seq * w.D * 2 + w.B * w.n
    qo = 2 * w.B * w.Hq * w.D * 2
    sparse = 0
    if w.sparse_frac > 0:
        nk, nv = nnz if nnz is not None else (expected_nnz(w), expected_nnz(w))
        sparse = csr_bytes(w, nk, nv)
    return codes + params + keep + qo + sparse


def quantize_algorithmic_bytes(w, nnz=None) -> int:
    """fp16 K and V read once, codes, parameters and (dense-and-sparse) CSR arrays written once."""
    W = _WORDS[w.bits]
    bh = w.B * w.Hkv
    read = 2 * bh * w.n * w.D * 2 + w.B * w.n
    write = 2 * bh * w.n * W * 4 + bh * (w.n // w.group) * w.D * 4 + bh * w.n * (w.D // w.group) * 4
    if w.sparse_frac > 0:
        nk, nv = nnz if nnz is not None else (expected_nnz(w), expected_nnz(w))
        write += csr_bytes(w, nk, nv)
    return read + write

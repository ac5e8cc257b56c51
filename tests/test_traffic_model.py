"""The algorithmic byte counts the benchmark divides by: worked out by hand from the cache layout
(kvs.h) for the benchmark workloads, so that a change to the formulas shows up here and not as a
silently different roofline fraction."""
from paper_2508_04257_amd import synth
from paper_2508_04257_amd.traffic import csr_bytes, decode_algorithmic_bytes, expected_nnz, quantize_algorithmic_bytes


def test_decode_bytes_of_the_headline_workload():
    w = synth.WORKLOADS["cfg1"]                       # B 8, n 4096, 32 x 128 heads, INT4, G 128, 5 kept rows
    bh, n = 8 * 32, 4096
    codes = 2 * bh * n * 16 * 4                       # K and V: 16 words per 128 codes
    params = bh * (n // 128) * 128 * 4 + bh * n * 1 * 4
    keep = 2 * bh * 5 * 128 * 2 + 8 * n               # fp16 rows of K and V, the keep mask
    qo = 2 * 8 * 32 * 128 * 2
    assert decode_algorithmic_bytes(w, 5) == codes + params + keep + qo == 143425536


def test_quantise_bytes_of_the_headline_workload():
    w = synth.WORKLOADS["cfg1"]
    bh, n = 8 * 32, 4096
    read = 2 * bh * n * 128 * 2 + 8 * n
    write = 2 * bh * n * 16 * 4 + bh * (n // 128) * 128 * 4 + bh * n * 4
    assert quantize_algorithmic_bytes(w) == read + write == 679510016


def test_bits_and_groups_scale_the_stream():
    cfg2, cfg3 = synth.WORKLOADS["cfg2"], synth.WORKLOADS["cfg3"]
    # INT3: 13 words per 128 codes; G 64: two parameter words per Value token, one per 64 Key tokens and channel
    bh, n = 16 * 8, 8192
    want2 = 2 * bh * n * 13 * 4 + bh * (n // 64) * 128 * 4 + bh * n * 2 * 4 + 2 * bh * 4 * 128 * 2 + 16 * n + 2 * 16 * 32 * 128 * 2
    assert decode_algorithmic_bytes(cfg2, 4) == want2 == 126484480
    # INT2: 8 words; G 32; 24 kept rows (first 16 + top 8)
    bh, n = 4 * 32, 32768
    want3 = 2 * bh * n * 8 * 4 + bh * (n // 32) * 128 * 4 + bh * n * 4 * 4 + 2 * bh * 24 * 128 * 2 + 4 * n + 2 * 4 * 32 * 128 * 2
    assert decode_algorithmic_bytes(cfg3, 24) == want3 == 404422656


def test_isolated_entries_add_their_csr_arrays():
    w = synth.WORKLOADS["cfg4"]                       # B 32, n 4096, 32 heads, INT3, G 128, 1 % isolated
    rows = 32 * 32 * 4096
    nnz = expected_nnz(w)
    assert nnz == rows * 128 // 100
    assert csr_bytes(w, 10, 20) == 4 * 30 + 2 * 4 * (rows + 1)      # 2 + 2 bytes per entry, one row pointer per row and tensor
    dense = decode_algorithmic_bytes(w.scaled(sparse_frac=0.0), 5)
    assert decode_algorithmic_bytes(w, 5, nnz=(1000, 3000)) == dense + csr_bytes(w, 1000, 3000)
    assert decode_algorithmic_bytes(w, 5) == dense + csr_bytes(w, nnz, nnz)
    assert quantize_algorithmic_bytes(w, nnz=(1000, 3000)) == quantize_algorithmic_bytes(w.scaled(sparse_frac=0.0)) + csr_bytes(w, 1000, 3000)

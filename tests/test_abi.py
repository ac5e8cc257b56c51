"""Host-side checks of the C-ABI library: it loads, exports every declared symbol, sizes buffers
as documented and rejects bad arguments before anything is launched (no GPU needed)."""
import ctypes as C
import os
import re

import pytest

from paper_2508_04257_amd import binding as kb

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared_symbols():
    text = open(os.path.join(ROOT, "include", "kvs.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(kvs_[a-z_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    names = _declared_symbols()
    assert {"kvs_predict_sinks", "kvs_quantize_kv", "kvs_decode_attn", "kvs_cache_bytes",
            "kvs_workspace_bytes", "kvs_quantize_prefix", "kvs_append_kv", "kvs_decode_attn_n",
            "kvs_calibrate", "kvs_calibrate_reset", "kvs_static_params", "kvs_quantize_kv_static",
            "kvs_calibration_bytes", "kvs_quant_error"} <= set(names)
    L = kb.lib()
    for name in names:
        assert hasattr(L, name), name
    assert L.kvs_version() >= 100
    assert kb.status_string(kb.KVS_ERR_CAPACITY) == "capacity exceeded"


def test_struct_layouts_match_the_header():
    assert C.sizeof(kb.KvsDesc) == 48                  # 9 x 4 bytes, padding, one int64
    assert kb.KvsDesc.sparse_cap.offset == 40
    assert C.sizeof(kb.KvsCache) == 18 * 8
    text = open(os.path.join(ROOT, "include", "kvs.h")).read()
    body = text[text.index("typedef struct kvs_cache {"):text.index("} kvs_cache;")]
    fields = re.findall(r"\b(\w+);", body)
    assert tuple(fields) == kb.CACHE_FIELD_NAMES


def test_cache_bytes_for_the_headline_workload():
    d = kb.make_desc(B=8, n=4096, Hq=32, Hkv=32, bits=4, group=128, keep_cap=5)
    s = kb.kvs_cache_bytes(d)
    assert s["k_codes"] == s["v_codes"] == 8 * 32 * 4096 * 64          # half a byte per element
    assert s["k_params"] == 8 * 32 * 32 * 128 * 4 and s["v_params"] == 8 * 32 * 4096 * 4
    assert s["keep_k"] == 8 * 32 * 5 * 256 and s["keep_idx"] == 8 * 5 * 4
    assert s["keep_mask"] == 8 * 4096 and s["k_col"] == 0 and s["status"] == 16
    d3 = kb.make_desc(B=16, n=8192, Hq=32, Hkv=8, bits=3, group=64, keep_cap=4)
    assert kb.kvs_cache_bytes(d3)["k_codes"] == 16 * 8 * 8192 * 13 * 4   # 13 words per 128 codes
    d2 = kb.make_desc(B=4, n=32768, Hq=32, Hkv=32, bits=2, group=32, keep_cap=24)
    assert kb.kvs_cache_bytes(d2)["v_params"] == 4 * 32 * 32768 * 4 * 4
    d8 = kb.make_desc(B=8, n=4096, Hq=32, Hkv=32, bits=8, group=128, keep_cap=5)
    assert kb.kvs_cache_bytes(d8)["k_codes"] == kb.kvs_cache_bytes(d8)["v_codes"] == 8 * 32 * 4096 * 128   # a byte per element
    assert kb.kvs_cache_bytes(d8)["k_params"] == s["k_params"]
    assert kb.kvs_workspace_bytes(d) >= 8 * 32 * kb.kvs_decode_splits(d) * 130 * 4
    # the counter block at its head: one word per (sequence, KV head), whole 256-byte lines
    assert kb.kvs_workspace_zero_bytes(d) == 8 * 32 * 4
    small = kb.make_desc(B=1, n=1024, Hq=8, Hkv=2, bits=4, group=128, keep_cap=2)
    assert kb.kvs_workspace_zero_bytes(small) == 256 and kb.kvs_workspace_bytes(small) > 256
    assert 1 <= kb.kvs_decode_splits(d) <= 4096 // 128


@pytest.mark.parametrize("field,value,expected", [
    ("D", 64, kb.KVS_ERR_UNSUPPORTED), ("bits", 5, kb.KVS_ERR_UNSUPPORTED),
    ("group", 16, kb.KVS_ERR_UNSUPPORTED), ("n", 1000, kb.KVS_ERR_UNSUPPORTED),
    ("n", 0, kb.KVS_ERR_INVALID), ("Hkv", 5, kb.KVS_ERR_INVALID), ("keep_cap", -1, kb.KVS_ERR_INVALID),
    ("Hq", 512, kb.KVS_ERR_UNSUPPORTED), ("sparse_frac", 1.5, kb.KVS_ERR_INVALID),
    ("key_per_token", 2, kb.KVS_ERR_INVALID),
])
def test_bad_descriptors_are_rejected_on_the_host(field, value, expected):
    d = kb.make_desc(B=2, n=1024, Hq=32, Hkv=32, bits=4, group=128, keep_cap=2)
    setattr(d, field, value)
    sizes = (C.c_size_t * kb.KVS_CACHE_FIELDS)()
    assert kb.lib().kvs_cache_bytes(C.byref(d), sizes) == expected
    assert kb.kvs_workspace_bytes(d) == 0
    # the compute entry points refuse the same descriptor before touching any pointer
    cache = kb.KvsCache()
    assert kb.lib().kvs_quantize_kv(C.byref(d), 16, 16, 16, C.byref(cache), None, None) == expected
    assert kb.lib().kvs_decode_attn(C.byref(d), 16, C.byref(cache), 16, None, 16, None) == expected


def test_per_token_key_descriptors():
    sizes = (C.c_size_t * kb.KVS_CACHE_FIELDS)()
    ok = kb.make_desc(B=2, n=1024, Hq=32, Hkv=8, bits=4, group=64, keep_cap=2, key_per_token=True)
    assert kb.KvsDesc.key_per_token.offset == 36 and ok.key_per_token == 1
    assert kb.lib().kvs_cache_bytes(C.byref(ok), sizes) == kb.KVS_OK
    plain = kb.make_desc(B=2, n=1024, Hq=32, Hkv=8, bits=4, group=64, keep_cap=2)
    assert kb.kvs_cache_bytes(ok) == kb.kvs_cache_bytes(plain)          # the parameter array only changes shape
    wide = kb.make_desc(B=2, n=1024, Hq=32, Hkv=8, bits=4, group=32, keep_cap=2, key_per_token=True)
    assert kb.lib().kvs_cache_bytes(C.byref(wide), sizes) == kb.KVS_OK
    # isolated outliers: not with per-token Keys
    sp = kb.make_desc(B=2, n=1024, Hq=32, Hkv=32, bits=4, group=128, keep_cap=2, sparse_frac=0.01, sparse_cap=100,
                      key_per_token=True)
    assert kb.lib().kvs_cache_bytes(C.byref(sp), sizes) == kb.KVS_ERR_UNSUPPORTED
    sp8 = kb.make_desc(B=2, n=1024, Hq=32, Hkv=32, bits=8, group=128, keep_cap=2, sparse_frac=0.01, sparse_cap=100)
    assert kb.lib().kvs_cache_bytes(C.byref(sp8), sizes) == kb.KVS_ERR_UNSUPPORTED     # nor with 8-bit codes


def test_null_pointers_are_rejected_on_the_host():
    d = kb.make_desc(B=2, n=1024, Hq=32, Hkv=32, bits=4, group=128, keep_cap=2)
    cache = kb.KvsCache()                              # all NULL
    L = kb.lib()
    assert L.kvs_quantize_kv(C.byref(d), None, None, None, C.byref(cache), None, None) == kb.KVS_ERR_INVALID
    assert L.kvs_quantize_kv(C.byref(d), 16, 16, 16, C.byref(cache), None, None) == kb.KVS_ERR_INVALID
    assert L.kvs_decode_attn(C.byref(d), 16, C.byref(cache), 16, None, 16, None) == kb.KVS_ERR_INVALID
    assert L.kvs_quantize_kv(None, 16, 16, 16, C.byref(cache), None, None) == kb.KVS_ERR_INVALID
    # decode reads the stream 16 bytes a lane and CSR entries 8 bytes at a time: misplaced arrays are refused
    for field, at in (("k_codes", 24), ("v_codes", 20), ("keep_k", 18)):
        odd = kb.KvsCache(**{name: (at if name == field else 16) for name in kb.CACHE_FIELD_NAMES})
        assert L.kvs_decode_attn(C.byref(d), 16, C.byref(odd), 16, None, 16, None) == kb.KVS_ERR_INVALID, field
    ds = kb.make_desc(B=8, n=4096, Hq=32, Hkv=32, bits=3, group=128, keep_cap=5, sparse_frac=0.01, sparse_cap=1 << 20)
    for field in ("k_col", "k_val", "v_col", "v_val"):
        odd = kb.KvsCache(**{name: (18 if name == field else 16) for name in kb.CACHE_FIELD_NAMES})
        assert L.kvs_decode_attn(C.byref(ds), 16, C.byref(odd), 16, None, 16, None) == kb.KVS_ERR_INVALID, field
    ch = (C.c_int32 * 1)(5000)
    assert L.kvs_predict_sinks(16, 1, 128, 4096, ch, 1, 2, 0, 16, 16, None, None) == kb.KVS_ERR_INVALID   # channel >= d
    ch = (C.c_int32 * 1)(7)
    assert L.kvs_predict_sinks(None, 1, 128, 4096, ch, 1, 2, 0, 16, 16, None, None) == kb.KVS_ERR_INVALID
    assert L.kvs_predict_sinks(16, 1, 128, 4096, ch, 1, 200, 0, 16, 16, None, None) == kb.KVS_ERR_INVALID  # k > n
    assert L.kvs_predict_sinks(16, 1, 1 << 20, 4096, ch, 1, 2, 0, 16, 16, None, None) == kb.KVS_ERR_UNSUPPORTED
    assert kb.kvs_predict_workspace_bytes(4, 32768, 8) == 4 * 8 * 8 * 4 and kb.kvs_predict_workspace_bytes(8, 4096, 5) == 0


def test_threshold_calls_check_their_arguments_on_the_host():
    L = kb.lib()
    dense = kb.make_desc(B=2, n=1024, Hq=32, Hkv=32, bits=3, group=128, keep_cap=2)
    sparse = kb.make_desc(B=2, n=1024, Hq=32, Hkv=32, bits=3, group=128, keep_cap=2, sparse_frac=0.01, sparse_cap=4096)
    full = kb.KvsCache(**{name: 16 for name in kb.CACHE_FIELD_NAMES})
    # only for dense-and-sparse descriptors
    assert L.kvs_outlier_thresholds(C.byref(dense), 16, 16, 16, 16, 16, None) == kb.KVS_ERR_INVALID
    assert L.kvs_quantize_kv_thresholds(C.byref(dense), 16, 16, 16, 16, C.byref(full), 16, None) == kb.KVS_ERR_INVALID
    # every pointer is needed
    for hole in range(5):
        args = [16, 16, 16, 16, 16]
        args[hole] = None
        assert L.kvs_outlier_thresholds(C.byref(sparse), *args, None) == kb.KVS_ERR_INVALID, hole
    for hole in (0, 1, 2, 3, 5):
        args = [16, 16, 16, 16, C.byref(full), 16]
        args[hole] = None
        assert L.kvs_quantize_kv_thresholds(C.byref(sparse), *args, None) == kb.KVS_ERR_INVALID, hole
    assert L.kvs_quantize_kv_thresholds(C.byref(sparse), 16, 16, 16, 16, None, 16, None) == kb.KVS_ERR_INVALID


def test_growing_cache_calls_check_their_arguments_on_the_host():
    d = kb.make_desc(B=2, n=1024, Hq=32, Hkv=32, bits=4, group=128, keep_cap=2)
    L = kb.lib()
    cache = kb.KvsCache()                              # all NULL
    assert L.kvs_quantize_prefix(C.byref(d), 16, 16, 16, 300, C.byref(cache), None, None) == kb.KVS_ERR_INVALID
    assert L.kvs_append_kv(C.byref(d), 16, 16, 300, C.byref(cache), None, None) == kb.KVS_ERR_INVALID
    assert L.kvs_decode_attn_n(C.byref(d), 16, C.byref(cache), 300, 16, None, 16, None) == kb.KVS_ERR_INVALID
    full = kb.KvsCache(**{name: 16 for name in kb.CACHE_FIELD_NAMES})   # non-NULL everywhere: only sizes are wrong
    assert L.kvs_quantize_prefix(C.byref(d), 16, 16, 16, 1025, C.byref(full), None, None) == kb.KVS_ERR_INVALID
    assert L.kvs_quantize_prefix(C.byref(d), 16, 16, 16, -1, C.byref(full), None, None) == kb.KVS_ERR_INVALID
    assert L.kvs_append_kv(C.byref(d), 16, 16, 1024, C.byref(full), None, None) == kb.KVS_ERR_INVALID   # full
    assert L.kvs_decode_attn_n(C.byref(d), 16, C.byref(full), 0, 16, None, 16, None) == kb.KVS_ERR_INVALID
    assert L.kvs_decode_attn_n(C.byref(d), 16, C.byref(full), 1025, 16, None, 16, None) == kb.KVS_ERR_INVALID
    ds = kb.make_desc(B=2, n=1024, Hq=32, Hkv=32, bits=3, group=128, keep_cap=2, sparse_frac=0.01, sparse_cap=1000)
    assert L.kvs_quantize_prefix(C.byref(ds), 16, 16, 16, 300, C.byref(full), 16, None) == kb.KVS_ERR_UNSUPPORTED
    assert L.kvs_append_kv(C.byref(ds), 16, 16, 300, C.byref(full), 16, None) == kb.KVS_ERR_UNSUPPORTED
    assert L.kvs_decode_attn_n(C.byref(ds), 16, C.byref(full), 300, 16, None, 16, None) == kb.KVS_ERR_UNSUPPORTED
    s = kb.kvs_cache_bytes(d)
    assert s["res_k"] == s["res_v"] == 2 * 32 * 128 * 128 * 2


def test_static_quantisation_calls_check_their_arguments_on_the_host():
    d = kb.make_desc(B=2, n=1024, Hq=32, Hkv=8, bits=4, group=64, keep_cap=2)
    L = kb.lib()
    assert kb.kvs_calibration_bytes(d) == 4 * 8 * 128 * 4
    assert L.kvs_calibrate_reset(C.byref(d), None, None) == kb.KVS_ERR_INVALID
    assert L.kvs_calibrate(C.byref(d), 16, 16, 16, None, None) == kb.KVS_ERR_INVALID
    assert L.kvs_static_params(C.byref(d), 16, None, 16, None) == kb.KVS_ERR_INVALID
    full = kb.KvsCache(**{name: 16 for name in kb.CACHE_FIELD_NAMES})
    assert L.kvs_quantize_kv_static(C.byref(d), 16, 16, 16, None, 16, C.byref(full), None, None) == kb.KVS_ERR_INVALID
    ds = kb.make_desc(B=2, n=1024, Hq=32, Hkv=32, bits=3, group=128, keep_cap=2, sparse_frac=0.01, sparse_cap=1000)
    assert L.kvs_quantize_kv_static(C.byref(ds), 16, 16, 16, 16, 16, C.byref(full), 16, None) == kb.KVS_ERR_UNSUPPORTED
    bad = kb.make_desc(B=2, n=1000, Hq=32, Hkv=32, bits=4, group=128, keep_cap=2)
    assert kb.kvs_calibration_bytes(bad) == 0


def test_prefill_layers_checks_every_argument_before_launching():
    d = kb.make_desc(B=2, n=1024, Hq=32, Hkv=32, bits=4, group=128, keep_cap=4)
    L = kb.lib()
    full = kb.KvsCache(**{name: 16 for name in kb.CACHE_FIELD_NAMES})
    caches = (kb.KvsCache * 3)(full, full, full)
    ptrs = (C.c_void_p * 3)(16, 16, 16)
    ch = (C.c_int32 * 1)(7)

    def call(n_layers=3, l_e=1, K=ptrs, V=ptrs, hidden=16, dd=64, k=3, first_n=1, idx=16, early=16, keep=16, cs=caches):
        return L.kvs_prefill_layers(C.byref(d), n_layers, l_e, K, V, hidden, dd, ch, 1, k, first_n, idx, early, keep, cs,
                                    None, None, None)

    assert call(n_layers=0) == kb.KVS_ERR_INVALID
    assert call(l_e=4) == kb.KVS_ERR_INVALID and call(l_e=-1) == kb.KVS_ERR_INVALID
    assert call(k=4, first_n=1) == kb.KVS_ERR_INVALID                 # 5 kept rows do not fit keep_cap = 4
    assert call(hidden=None) == kb.KVS_ERR_INVALID and call(keep=None) == kb.KVS_ERR_INVALID
    assert call(early=None) == kb.KVS_ERR_INVALID and call(idx=None) == kb.KVS_ERR_INVALID
    assert call(dd=5) == kb.KVS_ERR_INVALID                             # channel 7 outside the hidden size
    holes = (C.c_void_p * 3)(16, None, 16)
    assert call(K=holes) == kb.KVS_ERR_INVALID and call(V=holes) == kb.KVS_ERR_INVALID
    broken = (kb.KvsCache * 3)(full, full, kb.KvsCache())               # the third layer's cache has no buffers
    assert call(cs=broken) == kb.KVS_ERR_INVALID


def test_header_is_plain_c(tmp_path):
    """The boundary is a C ABI: the header must compile as C99 with a C compiler, and a C program
    must link against the library's host-side calls."""
    import shutil
    import subprocess

    if shutil.which("gcc") is None:
        pytest.skip("no C compiler")
    src = tmp_path / "use_kvs.c"
    src.write_text(
        '#include "kvs.h"\n'
        "int main(void) {\n"
        "  kvs_desc d = {0};\n"
        "  size_t sizes[KVS_CACHE_FIELDS];\n"
        "  d.B = 2; d.n = 1024; d.Hq = 32; d.Hkv = 32; d.D = 128; d.bits = 4; d.group = 128; d.keep_cap = 2;\n"
        "  if (kvs_cache_bytes(&d, sizes) != KVS_OK) return 1;\n"
        "  if (sizes[0] != (size_t)2 * 32 * 1024 * 64) return 2;\n"
        "  d.bits = 5;\n"
        "  return kvs_cache_bytes(&d, sizes) == KVS_ERR_UNSUPPORTED ? 0 : 3;\n"
        "}\n")
    inc = os.path.join(ROOT, "include")
    subprocess.run(["gcc", "-std=c99", "-Wall", "-Werror", "-pedantic", "-fsyntax-only", "-I", inc, str(src)], check=True)
    libdir = os.path.dirname(kb._LIB_PATH)
    exe = tmp_path / "use_kvs"
    subprocess.run(["gcc", "-std=c99", "-I", inc, str(src), "-o", str(exe), "-L", libdir, "-lkvs",
                    "-Wl,-rpath," + libdir, "-Wl,-rpath,/opt/rocm/lib"], check=True)
    assert subprocess.run([str(exe)]).returncode == 0

"""ctypes binding of libkvs.so: same names as the C ABI (include/kvs.h), argument marshalling only.

PyTorch provides device memory and the stream handle; every step of the path runs in the HIP
kernels.  There is no CPU fallback: if the library is not built, loading raises.
"""
from __future__ import annotations

import ctypes as C
import os
from dataclasses import dataclass
from typing import Dict, Optional, Sequence

import torch

_LIB_PATH = os.path.join(os.path.dirname(os.path.abspath(__file__)), "libkvs.so")
_lib = None

KVS_OK, KVS_ERR_INVALID, KVS_ERR_UNSUPPORTED, KVS_ERR_CAPACITY, KVS_ERR_DEVICE, KVS_ERR_SCRATCH = range(6)
KVS_NOALLOC_SCRATCH_BYTES = 4 << 20
KVS_CACHE_FIELDS = 18
CACHE_FIELD_NAMES = (
    "k_codes", "v_codes", "k_params", "v_params", "keep_k", "keep_v", "keep_idx", "keep_cnt",
    "keep_mask", "k_rowptr", "k_col", "k_val", "v_rowptr", "v_col", "v_val", "status",
    "res_k", "res_v",
)
_FIELD_DTYPES = dict(
    k_codes=torch.int32, v_codes=torch.int32, k_params=torch.int32, v_params=torch.int32,
    keep_k=torch.float16, keep_v=torch.float16, keep_idx=torch.int32, keep_cnt=torch.int32,
    keep_mask=torch.uint8, k_rowptr=torch.int32, k_col=torch.int16, k_val=torch.float16,
    v_rowptr=torch.int32, v_col=torch.int16, v_val=torch.float16, status=torch.int32,
    res_k=torch.float16, res_v=torch.float16,
)


class KvsDesc(C.Structure):
    _fields_ = [("B", C.c_int32), ("n", C.c_int32), ("Hq", C.c_int32), ("Hkv", C.c_int32),
                ("D", C.c_int32), ("bits", C.c_int32), ("group", C.c_int32),
                ("keep_cap", C.c_int32), ("sparse_frac", C.c_float), ("key_per_token", C.c_int32),
                ("sparse_cap", C.c_int64)]


class KvsCache(C.Structure):
    _fields_ = [(name, C.c_void_p) for name in CACHE_FIELD_NAMES]


class KvsError(RuntimeError):
    def __init__(self, call: str, status: int):
        self.status = status
        super().__init__(f"{call} failed: {status_string(status)} ({status})")


def lib() -> C.CDLL:
    """Loads libkvs.so once.  Raises if it has not been built (python -m paper_2508_04257_amd.build)."""
    global _lib
    if _lib is None:
        if not os.path.exists(_LIB_PATH):
            raise RuntimeError(f"{_LIB_PATH} is missing: build it with `python -m paper_2508_04257_amd.build`")
        L = C.CDLL(_LIB_PATH)
        L.kvs_version.restype = C.c_int32
        L.kvs_status_string.restype = C.c_char_p
        L.kvs_status_string.argtypes = [C.c_int]
        L.kvs_cache_bytes.restype = C.c_int
        L.kvs_cache_bytes.argtypes = [C.POINTER(KvsDesc), C.POINTER(C.c_size_t)]
        L.kvs_workspace_bytes.restype = C.c_size_t
        L.kvs_workspace_bytes.argtypes = [C.POINTER(KvsDesc)]
        L.kvs_workspace_zero_bytes.restype = C.c_size_t
        L.kvs_workspace_zero_bytes.argtypes = [C.POINTER(KvsDesc)]
        L.kvs_decode_splits.restype = C.c_int32
        L.kvs_decode_splits.argtypes = [C.POINTER(KvsDesc)]
        L.kvs_predict_sinks.restype = C.c_int
        L.kvs_predict_workspace_bytes.restype = C.c_size_t
        L.kvs_predict_workspace_bytes.argtypes = [C.c_int32, C.c_int32, C.c_int32]
        L.kvs_predict_sinks.argtypes = [C.c_void_p, C.c_int32, C.c_int32, C.c_int32, C.POINTER(C.c_int32),
                                        C.c_int32, C.c_int32, C.c_int32, C.c_void_p, C.c_void_p, C.c_void_p,
                                        C.c_void_p]
        L.kvs_quantize_kv.restype = C.c_int
        L.kvs_quantize_kv.argtypes = [C.POINTER(KvsDesc), C.c_void_p, C.c_void_p, C.c_void_p,
                                      C.POINTER(KvsCache), C.c_void_p, C.c_void_p]
        L.kvs_outlier_thresholds.restype = C.c_int
        L.kvs_outlier_thresholds.argtypes = [C.POINTER(KvsDesc), C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p,
                                             C.c_void_p, C.c_void_p]
        L.kvs_quantize_kv_thresholds.restype = C.c_int
        L.kvs_quantize_kv_thresholds.argtypes = [C.POINTER(KvsDesc), C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p,
                                                 C.POINTER(KvsCache), C.c_void_p, C.c_void_p]
        L.kvs_quantize_prefix.restype = C.c_int
        L.kvs_quantize_prefix.argtypes = [C.POINTER(KvsDesc), C.c_void_p, C.c_void_p, C.c_void_p, C.c_int32,
                                          C.POINTER(KvsCache), C.c_void_p, C.c_void_p]
        L.kvs_append_kv.restype = C.c_int
        L.kvs_append_kv.argtypes = [C.POINTER(KvsDesc), C.c_void_p, C.c_void_p, C.c_int32, C.POINTER(KvsCache),
                                    C.c_void_p, C.c_void_p]
        L.kvs_decode_attn_n.restype = C.c_int
        L.kvs_decode_attn_n.argtypes = [C.POINTER(KvsDesc), C.c_void_p, C.POINTER(KvsCache), C.c_int32, C.c_void_p,
                                        C.c_void_p, C.c_void_p, C.c_void_p]
        L.kvs_calibration_bytes.restype = C.c_size_t
        L.kvs_calibration_bytes.argtypes = [C.POINTER(KvsDesc)]
        L.kvs_calibrate_reset.restype = C.c_int
        L.kvs_calibrate_reset.argtypes = [C.POINTER(KvsDesc), C.c_void_p, C.c_void_p]
        L.kvs_calibrate.restype = C.c_int
        L.kvs_calibrate.argtypes = [C.POINTER(KvsDesc), C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p]
        L.kvs_static_params.restype = C.c_int
        L.kvs_static_params.argtypes = [C.POINTER(KvsDesc), C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p]
        L.kvs_quantize_kv_static.restype = C.c_int
        L.kvs_quantize_kv_static.argtypes = [C.POINTER(KvsDesc), C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p,
                                             C.c_void_p, C.POINTER(KvsCache), C.c_void_p, C.c_void_p]
        L.kvs_quant_error.restype = C.c_int
        L.kvs_quant_error.argtypes = [C.POINTER(KvsDesc), C.c_void_p, C.c_void_p, C.POINTER(KvsCache), C.c_void_p,
                                      C.c_void_p, C.c_void_p]
        L.kvs_decode_attn.restype = C.c_int
        L.kvs_decode_attn.argtypes = [C.POINTER(KvsDesc), C.c_void_p, C.POINTER(KvsCache), C.c_void_p,
                                      C.c_void_p, C.c_void_p, C.c_void_p]
        L.kvs_prefill_layers.restype = C.c_int
        L.kvs_prefill_layers.argtypes = [C.POINTER(KvsDesc), C.c_int32, C.c_int32, C.POINTER(C.c_void_p),
                                         C.POINTER(C.c_void_p), C.c_void_p, C.c_int32, C.POINTER(C.c_int32), C.c_int32,
                                         C.c_int32, C.c_int32, C.c_void_p, C.c_void_p, C.c_void_p, C.POINTER(KvsCache),
                                         C.c_void_p, C.c_void_p, C.c_void_p]
        L.kvs_probe_stream_read.restype = C.c_int
        L.kvs_probe_stream_read.argtypes = [C.c_void_p, C.c_size_t, C.c_void_p, C.c_void_p]
        L.kvs_decode_attn_noalloc.restype = C.c_int
        L.kvs_decode_attn_noalloc.argtypes = [C.POINTER(KvsDesc), C.c_void_p, C.POINTER(KvsCache), C.c_void_p,
                                              C.c_void_p, C.c_void_p]
        _lib = L
    return _lib


def status_string(status: int) -> str:
    return lib().kvs_status_string(int(status)).decode()


def make_desc(B, n, Hq, Hkv, bits, group, keep_cap, D=128, sparse_frac=0.0, sparse_cap=0,
              key_per_token=False) -> KvsDesc:
    return KvsDesc(B, n, Hq, Hkv, D, bits, group, keep_cap, sparse_frac, int(bool(key_per_token)), sparse_cap)


def kvs_cache_bytes(desc: KvsDesc) -> Dict[str, int]:
    sizes = (C.c_size_t * KVS_CACHE_FIELDS)()
    st = lib().kvs_cache_bytes(C.byref(desc), sizes)
    if st != KVS_OK:
        raise KvsError("kvs_cache_bytes", st)
    return dict(zip(CACHE_FIELD_NAMES, [int(s) for s in sizes]))


def kvs_workspace_bytes(desc: KvsDesc) -> int:
    return int(lib().kvs_workspace_bytes(C.byref(desc)))


def kvs_decode_splits(desc: KvsDesc) -> int:
    return int(lib().kvs_decode_splits(C.byref(desc)))


def _ptr(t: Optional[torch.Tensor]) -> Optional[int]:
    return None if t is None else t.data_ptr()


def _stream_handle() -> int:
    return torch.cuda.current_stream().cuda_stream


@dataclass
class CacheBuffers:
    """Device buffers of one layer's quantised cache plus the struct of pointers handed to C."""

    desc: KvsDesc
    tensors: Dict[str, Optional[torch.Tensor]]
    struct: KvsCache

    def __getattr__(self, name):
        tensors = object.__getattribute__(self, "tensors")
        if name in tensors:
            return tensors[name]
        raise AttributeError(name)


def alloc_cache(desc: KvsDesc, device="cuda") -> CacheBuffers:
    """Allocates every buffer kvs_cache_bytes asks for (torch is the allocator) and zeroes status."""
    sizes = kvs_cache_bytes(desc)
    tensors: Dict[str, Optional[torch.Tensor]] = {}
    for name in CACHE_FIELD_NAMES:
        nbytes = sizes[name]
        if nbytes == 0:
            tensors[name] = None
            continue
        dt = _FIELD_DTYPES[name]
        tensors[name] = torch.empty(nbytes // dt.itemsize, dtype=dt, device=device)
    tensors["status"].zero_()
    struct = KvsCache(**{name: _ptr(t) for name, t in tensors.items()})
    return CacheBuffers(desc, tensors, struct)


def kvs_workspace_zero_bytes(desc: KvsDesc) -> int:
    return int(lib().kvs_workspace_zero_bytes(C.byref(desc)))


def alloc_workspace(desc: KvsDesc, device="cuda") -> torch.Tensor:
    """Allocates the workspace and zeroes the counter block at its head (once; calls keep it zero)."""
    ws = torch.empty(max(16, kvs_workspace_bytes(desc)), dtype=torch.uint8, device=device)
    ws[:kvs_workspace_zero_bytes(desc)].zero_()
    return ws


def _check_tensor(name: str, t: torch.Tensor, shape, dtype) -> None:
    """The C side only sees pointers: shapes, dtypes and placement are verified here so that a
    kernel never indexes past a buffer."""
    if not (t.is_cuda and t.is_contiguous() and t.dtype == dtype and tuple(t.shape) == tuple(shape)):
        raise ValueError(f"{name}: expected contiguous {dtype} {tuple(shape)} on the GPU, got "
                         f"{t.dtype} {tuple(t.shape)} on {t.device}")


def _check_cache(desc: KvsDesc, cache: CacheBuffers) -> None:
    a, b = desc, cache.desc
    same = all(getattr(a, f) == getattr(b, f) for f, _ in KvsDesc._fields_)
    if not same:
        raise ValueError("cache buffers were allocated for a different descriptor")


def kvs_predict_workspace_bytes(B: int, n: int, k: int) -> int:
    return int(lib().kvs_predict_workspace_bytes(B, n, k))


def kvs_predict_sinks(hidden: torch.Tensor, channels: Sequence[int], k: int, first_n: int,
                      sink_idx: Optional[torch.Tensor], keep_mask: torch.Tensor,
                      workspace: Optional[torch.Tensor] = None) -> None:
    B, n, d = hidden.shape
    _check_tensor("hidden", hidden, (B, n, d), torch.float16)
    _check_tensor("keep_mask", keep_mask, (B, n), torch.uint8)
    if k > 0:
        _check_tensor("sink_idx", sink_idx, (B, k), torch.int32)
    if workspace is not None and (not workspace.is_cuda or
                                  workspace.numel() * workspace.element_size() < kvs_predict_workspace_bytes(B, n, k)):
        raise ValueError("predict workspace too small")
    ch = (C.c_int32 * len(channels))(*channels)
    st = lib().kvs_predict_sinks(hidden.data_ptr(), B, n, d, ch, len(channels), k, first_n,
                                 _ptr(sink_idx), keep_mask.data_ptr(), _ptr(workspace), _stream_handle())
    if st != KVS_OK:
        raise KvsError("kvs_predict_sinks", st)


def kvs_quantize_kv(desc: KvsDesc, K: torch.Tensor, V: torch.Tensor, keep_mask: torch.Tensor,
                    cache: CacheBuffers, workspace: Optional[torch.Tensor]) -> None:
    shape = (desc.B, desc.Hkv, desc.n, desc.D)
    _check_tensor("K", K, shape, torch.float16)
    _check_tensor("V", V, shape, torch.float16)
    _check_tensor("keep_mask", keep_mask, (desc.B, desc.n), torch.uint8)
    _check_cache(desc, cache)
    need = kvs_workspace_bytes(desc)
    if desc.sparse_frac > 0 and (workspace is None or workspace.numel() * workspace.element_size() < need):
        raise ValueError("workspace too small")
    st = lib().kvs_quantize_kv(C.byref(desc), K.data_ptr(), V.data_ptr(), keep_mask.data_ptr(),
                               C.byref(cache.struct), _ptr(workspace), _stream_handle())
    if st != KVS_OK:
        raise KvsError("kvs_quantize_kv", st)


def _check_sparse_call(desc: KvsDesc, K, V, keep_mask, tau, workspace) -> None:
    shape = (desc.B, desc.Hkv, desc.n, desc.D)
    _check_tensor("K", K, shape, torch.float16)
    _check_tensor("V", V, shape, torch.float16)
    _check_tensor("keep_mask", keep_mask, (desc.B, desc.n), torch.uint8)
    _check_tensor("tau", tau, (2,), torch.int32)
    if workspace is None or workspace.numel() * workspace.element_size() < kvs_workspace_bytes(desc):
        raise ValueError("workspace too small")


def kvs_outlier_thresholds(desc: KvsDesc, K: torch.Tensor, V: torch.Tensor, keep_mask: torch.Tensor,
                           tau: torch.Tensor, workspace: torch.Tensor) -> None:
    """The threshold search of kvs_quantize_kv alone; tau int32 [2] on the device, written."""
    _check_sparse_call(desc, K, V, keep_mask, tau, workspace)
    st = lib().kvs_outlier_thresholds(C.byref(desc), K.data_ptr(), V.data_ptr(), keep_mask.data_ptr(), tau.data_ptr(),
                                      _ptr(workspace), _stream_handle())
    if st != KVS_OK:
        raise KvsError("kvs_outlier_thresholds", st)


def kvs_quantize_kv_thresholds(desc: KvsDesc, K: torch.Tensor, V: torch.Tensor, keep_mask: torch.Tensor,
                               tau: torch.Tensor, cache: CacheBuffers, workspace: torch.Tensor) -> None:
    """kvs_quantize_kv with the outlier thresholds given (tau int32 [2] on the device)."""
    _check_sparse_call(desc, K, V, keep_mask, tau, workspace)
    _check_cache(desc, cache)
    st = lib().kvs_quantize_kv_thresholds(C.byref(desc), K.data_ptr(), V.data_ptr(), keep_mask.data_ptr(),
                                          tau.data_ptr(), C.byref(cache.struct), _ptr(workspace), _stream_handle())
    if st != KVS_OK:
        raise KvsError("kvs_quantize_kv_thresholds", st)


def kvs_prefill_layers(desc: KvsDesc, emergence_layer: int, Ks: Sequence[torch.Tensor], Vs: Sequence[torch.Tensor],
                       hidden: torch.Tensor, channels: Sequence[int], k: int, first_n: int,
                       sink_idx: Optional[torch.Tensor], early_mask: torch.Tensor, keep_mask: torch.Tensor,
                       caches: Sequence[CacheBuffers], workspace: Optional[torch.Tensor],
                       predict_workspace: Optional[torch.Tensor] = None) -> None:
    """Algorithm 1's loop order over len(Ks) layers in one submission (see kvs.h)."""
    L = len(Ks)
    if len(Vs) != L or len(caches) != L:
        raise ValueError("one K, one V and one cache per layer")
    shape = (desc.B, desc.Hkv, desc.n, desc.D)
    for l in range(L):
        _check_tensor(f"K[{l}]", Ks[l], shape, torch.float16)
        _check_tensor(f"V[{l}]", Vs[l], shape, torch.float16)
        _check_cache(desc, caches[l])
    B, n, d = hidden.shape
    _check_tensor("hidden", hidden, (desc.B, desc.n, d), torch.float16)
    _check_tensor("early_mask", early_mask, (desc.B, desc.n), torch.uint8)
    _check_tensor("keep_mask", keep_mask, (desc.B, desc.n), torch.uint8)
    if k > 0:
        _check_tensor("sink_idx", sink_idx, (desc.B, k), torch.int32)
    if desc.sparse_frac > 0 and (workspace is None or workspace.numel() * workspace.element_size() < kvs_workspace_bytes(desc)):
        raise ValueError("workspace too small")
    if predict_workspace is not None and (predict_workspace.numel() * predict_workspace.element_size()
                                          < kvs_predict_workspace_bytes(desc.B, desc.n, k)):
        raise ValueError("predict workspace too small")
    kp = (C.c_void_p * L)(*[t.data_ptr() for t in Ks])
    vp = (C.c_void_p * L)(*[t.data_ptr() for t in Vs])
    structs = (KvsCache * L)(*[c.struct for c in caches])
    ch = (C.c_int32 * len(channels))(*channels)
    st = lib().kvs_prefill_layers(C.byref(desc), L, emergence_layer, kp, vp, hidden.data_ptr(), d, ch, len(channels), k,
                                  first_n, _ptr(sink_idx), early_mask.data_ptr(), keep_mask.data_ptr(), structs,
                                  _ptr(workspace), _ptr(predict_workspace), _stream_handle())
    if st != KVS_OK:
        raise KvsError("kvs_prefill_layers", st)


def kvs_decode_attn(desc: KvsDesc, q: torch.Tensor, cache: CacheBuffers, out: torch.Tensor,
                    lse: Optional[torch.Tensor], workspace: torch.Tensor) -> None:
    _check_tensor("q", q, (desc.B, desc.Hq, desc.D), torch.float16)
    _check_tensor("out", out, (desc.B, desc.Hq, desc.D), torch.float16)
    if lse is not None:
        _check_tensor("lse", lse, (desc.B, desc.Hq), torch.float32)
    _check_cache(desc, cache)
    if not workspace.is_cuda or workspace.numel() * workspace.element_size() < kvs_workspace_bytes(desc):
        raise ValueError("workspace too small")
    st = lib().kvs_decode_attn(C.byref(desc), q.data_ptr(), C.byref(cache.struct), out.data_ptr(),
                               _ptr(lse), workspace.data_ptr(), _stream_handle())
    if st != KVS_OK:
        raise KvsError("kvs_decode_attn", st)


def kvs_decode_attn_noalloc(desc: KvsDesc, q: torch.Tensor, cache: CacheBuffers, out: torch.Tensor,
                            lse: Optional[torch.Tensor]) -> None:
    """kvs_decode_attn on the library's own scratch (no workspace, no allocation in the call)."""
    _check_tensor("q", q, (desc.B, desc.Hq, desc.D), torch.float16)
    _check_tensor("out", out, (desc.B, desc.Hq, desc.D), torch.float16)
    if lse is not None:
        _check_tensor("lse", lse, (desc.B, desc.Hq), torch.float32)
    _check_cache(desc, cache)
    st = lib().kvs_decode_attn_noalloc(C.byref(desc), q.data_ptr(), C.byref(cache.struct), out.data_ptr(),
                                       _ptr(lse), _stream_handle())
    if st != KVS_OK:
        raise KvsError("kvs_decode_attn_noalloc", st)


# ---- growing caches: desc.n is the capacity, n_tokens what the cache holds ---------------------
def kvs_quantize_prefix(desc: KvsDesc, K: torch.Tensor, V: torch.Tensor, keep_mask: torch.Tensor, n_tokens: int,
                        cache: CacheBuffers, workspace: Optional[torch.Tensor]) -> None:
    shape = (desc.B, desc.Hkv, n_tokens, desc.D)
    _check_tensor("K", K, shape, torch.float16)
    _check_tensor("V", V, shape, torch.float16)
    _check_tensor("keep_mask", keep_mask, (desc.B, n_tokens), torch.uint8)
    _check_cache(desc, cache)
    st = lib().kvs_quantize_prefix(C.byref(desc), K.data_ptr(), V.data_ptr(), keep_mask.data_ptr(), n_tokens,
                                   C.byref(cache.struct), _ptr(workspace), _stream_handle())
    if st != KVS_OK:
        raise KvsError("kvs_quantize_prefix", st)


def kvs_append_kv(desc: KvsDesc, k_new: torch.Tensor, v_new: torch.Tensor, n_tokens: int, cache: CacheBuffers,
                  workspace: Optional[torch.Tensor]) -> None:
    _check_tensor("k_new", k_new, (desc.B, desc.Hkv, desc.D), torch.float16)
    _check_tensor("v_new", v_new, (desc.B, desc.Hkv, desc.D), torch.float16)
    _check_cache(desc, cache)
    st = lib().kvs_append_kv(C.byref(desc), k_new.data_ptr(), v_new.data_ptr(), n_tokens, C.byref(cache.struct),
                             _ptr(workspace), _stream_handle())
    if st != KVS_OK:
        raise KvsError("kvs_append_kv", st)


def kvs_decode_attn_n(desc: KvsDesc, q: torch.Tensor, cache: CacheBuffers, n_tokens: int, out: torch.Tensor,
                      lse: Optional[torch.Tensor], workspace: torch.Tensor) -> None:
    _check_tensor("q", q, (desc.B, desc.Hq, desc.D), torch.float16)
    _check_tensor("out", out, (desc.B, desc.Hq, desc.D), torch.float16)
    if lse is not None:
        _check_tensor("lse", lse, (desc.B, desc.Hq), torch.float32)
    _check_cache(desc, cache)
    if not workspace.is_cuda or workspace.numel() * workspace.element_size() < kvs_workspace_bytes(desc):
        raise ValueError("workspace too small")
    st = lib().kvs_decode_attn_n(C.byref(desc), q.data_ptr(), C.byref(cache.struct), n_tokens, out.data_ptr(),
                                 _ptr(lse), workspace.data_ptr(), _stream_handle())
    if st != KVS_OK:
        raise KvsError("kvs_decode_attn_n", st)


def kvs_probe_stream_read(src: torch.Tensor, sink: torch.Tensor) -> None:
    """Diagnostic pure streaming read of `src` (see kvs.h)."""
    if not (src.is_cuda and src.is_contiguous() and sink.is_cuda and sink.numel() * sink.element_size() >= 4):
        raise ValueError("kvs_probe_stream_read: device tensors expected")
    st = lib().kvs_probe_stream_read(src.data_ptr(), src.numel() * src.element_size(), sink.data_ptr(), _stream_handle())
    if st != KVS_OK:
        raise KvsError("kvs_probe_stream_read", st)


# ---- static quantisation -------------------------------------------------------------------------
def kvs_calibration_bytes(desc: KvsDesc) -> int:
    return int(lib().kvs_calibration_bytes(C.byref(desc)))


def alloc_calibration(desc: KvsDesc, device="cuda") -> torch.Tensor:
    calib = torch.empty(kvs_calibration_bytes(desc) // 4, dtype=torch.int32, device=device)
    st = lib().kvs_calibrate_reset(C.byref(desc), calib.data_ptr(), _stream_handle())
    if st != KVS_OK:
        raise KvsError("kvs_calibrate_reset", st)
    return calib


def kvs_calibrate(desc: KvsDesc, K: torch.Tensor, V: torch.Tensor, keep_mask: torch.Tensor, calib: torch.Tensor) -> None:
    shape = (desc.B, desc.Hkv, desc.n, desc.D)
    _check_tensor("K", K, shape, torch.float16)
    _check_tensor("V", V, shape, torch.float16)
    _check_tensor("keep_mask", keep_mask, (desc.B, desc.n), torch.uint8)
    _check_tensor("calib", calib, (kvs_calibration_bytes(desc) // 4,), torch.int32)
    st = lib().kvs_calibrate(C.byref(desc), K.data_ptr(), V.data_ptr(), keep_mask.data_ptr(), calib.data_ptr(),
                             _stream_handle())
    if st != KVS_OK:
        raise KvsError("kvs_calibrate", st)


def kvs_static_params(desc: KvsDesc, calib: torch.Tensor):
    """-> (k_static int32 [Hkv, 128] - [Hkv, 128 / G] with per-token Keys -, v_static int32
    [Hkv, 128 / G]) parameter words on the device."""
    _check_tensor("calib", calib, (kvs_calibration_bytes(desc) // 4,), torch.int32)
    ks = torch.empty((desc.Hkv, desc.D // desc.group if desc.key_per_token else desc.D), dtype=torch.int32,
                     device=calib.device)
    vs = torch.empty((desc.Hkv, desc.D // desc.group), dtype=torch.int32, device=calib.device)
    st = lib().kvs_static_params(C.byref(desc), calib.data_ptr(), ks.data_ptr(), vs.data_ptr(), _stream_handle())
    if st != KVS_OK:
        raise KvsError("kvs_static_params", st)
    return ks, vs


def kvs_quantize_kv_static(desc: KvsDesc, K: torch.Tensor, V: torch.Tensor, keep_mask: torch.Tensor,
                           k_static: torch.Tensor, v_static: torch.Tensor, cache: CacheBuffers,
                           workspace: Optional[torch.Tensor]) -> None:
    shape = (desc.B, desc.Hkv, desc.n, desc.D)
    _check_tensor("K", K, shape, torch.float16)
    _check_tensor("V", V, shape, torch.float16)
    _check_tensor("keep_mask", keep_mask, (desc.B, desc.n), torch.uint8)
    _check_tensor("k_static", k_static, (desc.Hkv, desc.D // desc.group if desc.key_per_token else desc.D), torch.int32)
    _check_tensor("v_static", v_static, (desc.Hkv, desc.D // desc.group), torch.int32)
    _check_cache(desc, cache)
    st = lib().kvs_quantize_kv_static(C.byref(desc), K.data_ptr(), V.data_ptr(), keep_mask.data_ptr(),
                                      k_static.data_ptr(), v_static.data_ptr(), C.byref(cache.struct),
                                      _ptr(workspace), _stream_handle())
    if st != KVS_OK:
        raise KvsError("kvs_quantize_kv_static", st)


def kvs_quant_error(desc: KvsDesc, K: torch.Tensor, V: torch.Tensor, cache: CacheBuffers,
                    sink_mask: torch.Tensor) -> Dict[str, tuple]:
    """-> {"k": (sse_without, n_without, sse_with, n_with), "v": (...)} (synchronises)."""
    shape = (desc.B, desc.Hkv, desc.n, desc.D)
    _check_tensor("K", K, shape, torch.float16)
    _check_tensor("V", V, shape, torch.float16)
    _check_tensor("sink_mask", sink_mask, (desc.B, desc.n), torch.uint8)
    _check_cache(desc, cache)
    report = torch.empty(8, dtype=torch.int64, device=K.device)
    st = lib().kvs_quant_error(C.byref(desc), K.data_ptr(), V.data_ptr(), C.byref(cache.struct), sink_mask.data_ptr(),
                               report.data_ptr(), _stream_handle())
    if st != KVS_OK:
        raise KvsError("kvs_quant_error", st)
    host = report.cpu()
    sse = host[:4].view(torch.float64).tolist()
    cnt = host[4:].tolist()
    return {"k": (sse[0], cnt[0], sse[1], cnt[1]), "v": (sse[2], cnt[2], sse[3], cnt[3])}

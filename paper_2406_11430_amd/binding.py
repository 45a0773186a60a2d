"""ctypes binding of libl2kv.so: one Python function per C entry point, same
names, argument marshalling only.  Tensors are torch CUDA(HIP) tensors used as
device memory; every step of the path runs inside the library's kernels.

The library must already be built (``python -m paper_2406_11430_amd.build``);
nothing here falls back to another implementation.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Optional

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libl2kv.so")

L2KV_F32, L2KV_BF16 = 0, 1
L2KV_KEEP_LOWEST, L2KV_KEEP_HIGHEST = 0, 1
L2KV_OK = 0

# name -> (restype, argtypes); mirrors include/l2kv.h declaration by declaration
SIGNATURES = {
    "l2kv_keep_count": (C.c_int64, [C.c_int64, C.c_double]),
    "l2kv_norms": (C.c_int, [C.c_void_p, C.c_int, C.c_int64, C.c_int64, C.c_int32, C.c_int64,
                             C.c_void_p, C.c_void_p]),
    "l2kv_select": (C.c_int, [C.c_void_p, C.c_int64, C.c_int64, C.c_double, C.c_void_p, C.c_void_p,
                              C.c_void_p, C.c_size_t, C.c_void_p]),
    "l2kv_select_k": (C.c_int, [C.c_void_p, C.c_int64, C.c_int64, C.c_int64, C.c_int, C.c_void_p,
                                C.c_void_p, C.c_void_p, C.c_size_t, C.c_void_p]),
    "l2kv_select_workspace_bytes": (C.c_size_t, [C.c_int64, C.c_int64]),
    "l2kv_random_keys": (C.c_int, [C.c_int64, C.c_int64, C.c_uint32, C.c_void_p, C.c_void_p]),
    "l2kv_compact": (C.c_int, [C.c_void_p, C.c_void_p, C.c_int, C.c_void_p, C.c_int64, C.c_int64,
                               C.c_int64, C.c_int32, C.c_int64, C.c_void_p, C.c_void_p, C.c_void_p]),
    "l2kv_compress": (C.c_int, [C.c_void_p, C.c_void_p, C.c_int, C.c_int64, C.c_int64, C.c_int32, C.c_int64,
                                C.c_double, C.c_int64, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p,
                                C.c_void_p, C.c_size_t, C.c_void_p]),
    "l2kv_decode_attn": (C.c_int, [C.c_void_p, C.c_void_p, C.c_void_p, C.c_int, C.c_int32, C.c_int32,
                                   C.c_int32, C.c_int64, C.c_int32, C.c_int64, C.c_float, C.c_void_p,
                                   C.c_void_p, C.c_size_t, C.c_void_p]),
    "l2kv_decode_attn_out": (C.c_int, [C.c_void_p, C.c_void_p, C.c_void_p, C.c_int, C.c_int32, C.c_int32,
                                       C.c_int32, C.c_int64, C.c_int32, C.c_int64, C.c_float, C.c_int,
                                       C.c_void_p, C.c_void_p, C.c_size_t, C.c_void_p]),
    "l2kv_decode_attn_splits": (C.c_int, [C.c_void_p, C.c_void_p, C.c_void_p, C.c_int, C.c_int32,
                                          C.c_int32, C.c_int32, C.c_int64, C.c_int32, C.c_int64,
                                          C.c_float, C.c_int32, C.c_void_p, C.c_void_p, C.c_size_t,
                                          C.c_void_p]),
    "l2kv_decode_attn_static": (C.c_int, [C.c_void_p, C.c_void_p, C.c_void_p, C.c_int, C.c_int32, C.c_int32,
                                          C.c_int32, C.c_int64, C.c_int32, C.c_int64, C.c_float, C.c_void_p,
                                          C.c_void_p]),
    "l2kv_decode_max_splits": (C.c_int32, [C.c_int64]),
    "l2kv_decode_workspace_init": (C.c_int, [C.c_void_p, C.c_size_t, C.c_void_p]),
    "l2kv_decode_workspace_bytes": (C.c_size_t, [C.c_int32, C.c_int32, C.c_int64, C.c_int32]),
    "l2kv_select_ragged": (C.c_int, [C.c_void_p, C.c_int32, C.c_int32, C.c_int64, C.c_void_p, C.c_void_p,
                                     C.c_int64, C.c_int64, C.c_int, C.c_void_p, C.c_void_p]),
    "l2kv_compact_ragged": (C.c_int, [C.c_void_p, C.c_void_p, C.c_void_p, C.c_int, C.c_void_p, C.c_int32,
                                      C.c_int32, C.c_int64, C.c_void_p, C.c_void_p, C.c_int64, C.c_int64,
                                      C.c_void_p, C.c_int64, C.c_int32, C.c_void_p, C.c_void_p, C.c_void_p,
                                      C.c_void_p, C.c_void_p]),
    "l2kv_stream_append": (C.c_int, [C.c_void_p, C.c_void_p, C.c_int, C.c_int32, C.c_int32, C.c_int32,
                                     C.c_int32, C.c_void_p, C.c_void_p, C.c_int64, C.c_void_p, C.c_void_p,
                                     C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p]),
    "l2kv_stream_evict": (C.c_int, [C.c_int, C.c_int32, C.c_int32, C.c_int32, C.c_void_p, C.c_int64,
                                    C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p,
                                    C.c_void_p, C.c_void_p]),
    "l2kv_decode_attn_ragged": (C.c_int, [C.c_void_p, C.c_void_p, C.c_void_p, C.c_int, C.c_int32, C.c_int32,
                                          C.c_int32, C.c_int32, C.c_void_p, C.c_void_p, C.c_void_p, C.c_int64,
                                          C.c_int64, C.c_float, C.c_int32, C.c_void_p, C.c_void_p, C.c_size_t,
                                          C.c_void_p]),
    "l2kv_length_order": (C.c_int, [C.c_void_p, C.c_int32, C.c_void_p, C.c_void_p]),
    "l2kv_decode_ragged_workspace_bytes": (C.c_size_t, [C.c_int32, C.c_int32, C.c_int64, C.c_int32]),
    "l2kv_norm_ranks": (C.c_int, [C.c_void_p, C.c_int64, C.c_int64, C.c_void_p, C.c_void_p, C.c_size_t,
                                  C.c_void_p]),
    "l2kv_norm_ranks_workspace_bytes": (C.c_size_t, [C.c_int64, C.c_int64]),
    "l2kv_alr": (C.c_int, [C.c_void_p, C.c_void_p, C.c_int, C.c_void_p, C.c_int32, C.c_int32, C.c_int32,
                           C.c_int64, C.c_int32, C.c_int64, C.c_float, C.c_int64, C.c_void_p, C.c_void_p,
                           C.c_void_p, C.c_void_p, C.c_size_t, C.c_void_p]),
    "l2kv_alr_workspace_bytes": (C.c_size_t, [C.c_int32, C.c_int32, C.c_int64]),
    "l2kv_device_info": (C.c_int, [C.c_void_p, C.c_void_p, C.c_void_p]),
    "l2kv_read_probe": (C.c_int, [C.c_void_p, C.c_size_t, C.c_void_p, C.c_void_p]),
    "l2kv_status_string": (C.c_char_p, [C.c_int]),
    "l2kv_version": (C.c_int32, []),
}


class L2KVError(RuntimeError):
    def __init__(self, fn: str, status: int, text: str):
        super().__init__("%s failed: status %d (%s)" % (fn, status, text))
        self.status = status


_lib = None


def lib() -> C.CDLL:
    """The loaded libl2kv.so; raises if it has not been built."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(
                "libl2kv.so is missing at %s: build it with "
                "`python -m paper_2406_11430_amd.build` (there is no fallback path)" % LIB_PATH)
        handle = C.CDLL(LIB_PATH)
        for name, (res, args) in SIGNATURES.items():
            fn = getattr(handle, name)
            fn.restype = res
            fn.argtypes = args
        _lib = handle
    return _lib


def _check(fn: str, status: int) -> None:
    if status != L2KV_OK:
        raise L2KVError(fn, status, lib().l2kv_status_string(status).decode())


def _dtype_code(t: torch.Tensor) -> int:
    if t.dtype == torch.float32:
        return L2KV_F32
    if t.dtype == torch.bfloat16:
        return L2KV_BF16
    raise TypeError("l2kv supports float32 and bfloat16 caches, got %s" % t.dtype)


def _dev(*tensors: Optional[torch.Tensor]) -> None:
    for t in tensors:
        if t is not None:
            if not t.is_cuda:
                raise ValueError("l2kv works on device tensors only")
            if not t.is_contiguous():
                raise ValueError("l2kv needs contiguous tensors")


def _ptr(t: Optional[torch.Tensor]):
    return None if t is None else C.c_void_p(t.data_ptr())


def _stream(stream: Optional[torch.cuda.Stream]):
    s = torch.cuda.current_stream() if stream is None else stream
    return C.c_void_p(s.cuda_stream)


# ------------------------------------------------------------ host helpers
def l2kv_keep_count(T: int, keep_ratio: float) -> int:
    return int(lib().l2kv_keep_count(int(T), float(keep_ratio)))


def l2kv_select_workspace_bytes(n_heads: int, T: int) -> int:
    return int(lib().l2kv_select_workspace_bytes(int(n_heads), int(T)))


def l2kv_decode_workspace_bytes(B: int, Hq: int, kv_len: int, D: int) -> int:
    return int(lib().l2kv_decode_workspace_bytes(int(B), int(Hq), int(kv_len), int(D)))


def l2kv_decode_max_splits(kv_len: int) -> int:
    return int(lib().l2kv_decode_max_splits(int(kv_len)))


def l2kv_decode_workspace_init(workspace: torch.Tensor, stream=None) -> None:
    """Zero-fill a decode workspace on the stream (required once before first use)."""
    _dev(workspace)
    _check("l2kv_decode_workspace_init", lib().l2kv_decode_workspace_init(
        _ptr(workspace), workspace.numel() * workspace.element_size(), _stream(stream)))


def l2kv_read_probe(data: torch.Tensor, sink: torch.Tensor, stream=None) -> None:
    """Stream `data` once through the compute units (bare read, nothing stored): a launch whose
    rate is the read-stream ceiling for that buffer.  `sink`: any device tensor of >= 4 bytes."""
    _dev(data, sink)
    _check("l2kv_read_probe", lib().l2kv_read_probe(_ptr(data), data.numel() * data.element_size(),
                                                     _ptr(sink), _stream(stream)))


def l2kv_device_info() -> dict:
    """Compute units, peak memory clock (kHz) and memory bus width (bits) of the current device."""
    cu, clk, bus = C.c_int32(0), C.c_int32(0), C.c_int32(0)
    _check("l2kv_device_info", lib().l2kv_device_info(C.byref(cu), C.byref(clk), C.byref(bus)))
    return {"compute_units": cu.value, "memory_clock_khz": clk.value, "memory_bus_bits": bus.value}


def l2kv_version() -> int:
    return int(lib().l2kv_version())


def _heads(x: torch.Tensor):
    """[..., T, D] -> (n_heads, T, D)."""
    *lead, T, D = x.shape
    n = 1
    for v in lead:
        n *= v
    return n, T, D


# ------------------------------------------------------------ device calls
def l2kv_norms(K: torch.Tensor, norms: torch.Tensor, stream=None) -> None:
    """K ``[..., T, D]`` (f32/bf16) -> norms ``[..., T]`` float32 (pre-allocated)."""
    _dev(K, norms)
    n, T, D = _heads(K)
    assert norms.dtype == torch.float32 and norms.numel() == n * T
    _check("l2kv_norms", lib().l2kv_norms(_ptr(K), _dtype_code(K), n, T, D, T * D, _ptr(norms),
                                          _stream(stream)))


def l2kv_select(norms: torch.Tensor, keep_ratio: float, kept_idx: torch.Tensor,
                kept_count: Optional[torch.Tensor], workspace: torch.Tensor, stream=None) -> None:
    """norms ``[..., T]`` -> kept_idx ``[..., k]`` int32, k = l2kv_keep_count(T, keep_ratio)."""
    _dev(norms, kept_idx, kept_count, workspace)
    T = norms.shape[-1]
    n = norms.numel() // T
    assert norms.dtype == torch.float32 and kept_idx.dtype == torch.int32
    _check("l2kv_select", lib().l2kv_select(_ptr(norms), n, T, float(keep_ratio), _ptr(kept_idx),
                                            _ptr(kept_count), _ptr(workspace),
                                            workspace.numel() * workspace.element_size(),
                                            _stream(stream)))


def l2kv_select_k(norms: torch.Tensor, k: int, mode: int, kept_idx: torch.Tensor,
                  kept_count: Optional[torch.Tensor], workspace: torch.Tensor, stream=None) -> None:
    _dev(norms, kept_idx, kept_count, workspace)
    T = norms.shape[-1]
    n = norms.numel() // T
    assert norms.dtype == torch.float32 and kept_idx.dtype == torch.int32
    _check("l2kv_select_k", lib().l2kv_select_k(_ptr(norms), n, T, int(k), int(mode), _ptr(kept_idx),
                                                _ptr(kept_count), _ptr(workspace),
                                                workspace.numel() * workspace.element_size(),
                                                _stream(stream)))


def l2kv_random_keys(seed: int, keys: torch.Tensor, stream=None) -> None:
    """keys ``[..., T]`` float32 (pre-allocated) <- hash bit patterns of (seed, head, token)."""
    _dev(keys)
    T = keys.shape[-1]
    assert keys.dtype == torch.float32
    _check("l2kv_random_keys", lib().l2kv_random_keys(keys.numel() // T, T, int(seed) & 0xFFFFFFFF,
                                                      _ptr(keys), _stream(stream)))


def l2kv_compact(K: torch.Tensor, V: Optional[torch.Tensor], kept_idx: torch.Tensor,
                 Kc: torch.Tensor, Vc: Optional[torch.Tensor], stream=None) -> None:
    """Gather rows kept_idx ``[..., k]`` of K, V ``[..., T, D]`` into Kc, Vc ``[..., k, D]``."""
    _dev(K, V, kept_idx, Kc, Vc)
    n, T, D = _heads(K)
    k = kept_idx.shape[-1]
    assert kept_idx.dtype == torch.int32 and kept_idx.numel() == n * k
    assert Kc.dtype == K.dtype and Kc.numel() == n * k * D
    if V is not None:
        assert V.shape == K.shape and V.dtype == K.dtype and Vc is not None and Vc.numel() == Kc.numel()
    _check("l2kv_compact", lib().l2kv_compact(_ptr(K), _ptr(V), _dtype_code(K), _ptr(kept_idx), n, T, k,
                                              D, T * D, _ptr(Kc), _ptr(Vc), _stream(stream)))


def l2kv_compress(K: torch.Tensor, V: torch.Tensor, keep_ratio: float, norms: torch.Tensor,
                  kept_idx: torch.Tensor, Kc: torch.Tensor, Vc: torch.Tensor, workspace: torch.Tensor,
                  slab_heads: int = 0, stream=None) -> None:
    """norms -> select -> compact in one call (optionally slab by slab of ``slab_heads`` heads)."""
    _dev(K, V, norms, kept_idx, Kc, Vc, workspace)
    n, T, D = _heads(K)
    k = kept_idx.shape[-1]
    assert V.shape == K.shape and V.dtype == K.dtype == Kc.dtype == Vc.dtype
    assert norms.dtype == torch.float32 and norms.numel() == n * T
    assert kept_idx.dtype == torch.int32 and kept_idx.numel() == n * k
    assert Kc.numel() == n * k * D and Vc.numel() == n * k * D
    _check("l2kv_compress", lib().l2kv_compress(
        _ptr(K), _ptr(V), _dtype_code(K), n, T, D, T * D, float(keep_ratio), int(slab_heads), _ptr(norms),
        _ptr(kept_idx), _ptr(Kc), _ptr(Vc), _ptr(workspace), workspace.numel() * workspace.element_size(),
        _stream(stream)))


def l2kv_decode_attn(Q: torch.Tensor, Kc: torch.Tensor, Vc: torch.Tensor, O: torch.Tensor,
                     workspace: torch.Tensor, scale: float = 0.0, stream=None) -> None:
    """Q ``[B, Hq, D]``, Kc/Vc ``[B, Hkv, n, D]`` -> O ``[B, Hq, D]`` float32."""
    l2kv_decode_attn_splits(Q, Kc, Vc, O, workspace, scale=scale, n_splits=None, stream=stream)


def l2kv_decode_attn_splits(Q: torch.Tensor, Kc: torch.Tensor, Vc: torch.Tensor, O: torch.Tensor,
                            workspace: torch.Tensor, scale: float = 0.0,
                            n_splits: Optional[int] = 0, stream=None) -> None:
    _dev(Q, Kc, Vc, O, workspace)
    B, Hq, D = Q.shape
    Bk, Hkv, n, Dk = Kc.shape
    assert (Bk, Dk) == (B, D) and Vc.shape == Kc.shape and Kc.dtype == Q.dtype == Vc.dtype
    assert O.dtype == torch.float32 and O.numel() == B * Hq * D
    ws_bytes = workspace.numel() * workspace.element_size()
    if n_splits is None:
        st = lib().l2kv_decode_attn(_ptr(Q), _ptr(Kc), _ptr(Vc), _dtype_code(Q), B, Hq, Hkv, n, D,
                                    n * D, float(scale), _ptr(O), _ptr(workspace), ws_bytes,
                                    _stream(stream))
        _check("l2kv_decode_attn", st)
    else:
        st = lib().l2kv_decode_attn_splits(_ptr(Q), _ptr(Kc), _ptr(Vc), _dtype_code(Q), B, Hq, Hkv, n,
                                           D, n * D, float(scale), int(n_splits), _ptr(O),
                                           _ptr(workspace), ws_bytes, _stream(stream))
        _check("l2kv_decode_attn_splits", st)


def l2kv_decode_attn_out(Q: torch.Tensor, Kc: torch.Tensor, Vc: torch.Tensor, O: torch.Tensor,
                         workspace: torch.Tensor, scale: float = 0.0, stream=None) -> None:
    """l2kv_decode_attn with O ``[B, Hq, D]`` in float32 or bfloat16 (the tensor's dtype decides)."""
    _dev(Q, Kc, Vc, O, workspace)
    B, Hq, D = Q.shape
    Bk, Hkv, n, Dk = Kc.shape
    assert (Bk, Dk) == (B, D) and Vc.shape == Kc.shape and Kc.dtype == Q.dtype == Vc.dtype
    assert O.numel() == B * Hq * D
    _check("l2kv_decode_attn_out", lib().l2kv_decode_attn_out(
        _ptr(Q), _ptr(Kc), _ptr(Vc), _dtype_code(Q), B, Hq, Hkv, n, D, n * D, float(scale), _dtype_code(O),
        _ptr(O), _ptr(workspace), workspace.numel() * workspace.element_size(), _stream(stream)))


def l2kv_decode_attn_static(Q: torch.Tensor, Kc: torch.Tensor, Vc: torch.Tensor, O: torch.Tensor,
                            scale: float = 0.0, stream=None) -> None:
    """l2kv_decode_attn over the library's own scratch array (no workspace argument)."""
    _dev(Q, Kc, Vc, O)
    B, Hq, D = Q.shape
    Bk, Hkv, n, Dk = Kc.shape
    assert (Bk, Dk) == (B, D) and Vc.shape == Kc.shape and Kc.dtype == Q.dtype == Vc.dtype
    assert O.dtype == torch.float32 and O.numel() == B * Hq * D
    _check("l2kv_decode_attn_static", lib().l2kv_decode_attn_static(
        _ptr(Q), _ptr(Kc), _ptr(Vc), _dtype_code(Q), B, Hq, Hkv, n, D, n * D, float(scale), _ptr(O),
        _stream(stream)))


# ------------------------------------------------- ragged batches / streaming
def l2kv_decode_ragged_workspace_bytes(n_seq: int, Hq: int, max_len: int, D: int) -> int:
    return int(lib().l2kv_decode_ragged_workspace_bytes(int(n_seq), int(Hq), int(max_len), int(D)))


def _i64(t: torch.Tensor, n: int) -> None:
    assert t.dtype == torch.int64 and t.numel() == n


def _i32(t: torch.Tensor, n: int) -> None:
    assert t.dtype == torch.int32 and t.numel() == n


def l2kv_select_ragged(norms: torch.Tensor, in_offsets: torch.Tensor, out_offsets: torch.Tensor,
                       max_len: int, kept_idx: torch.Tensor, mode: int = L2KV_KEEP_LOWEST,
                       stream=None) -> None:
    """norms ``[n_planes, total_tokens]`` -> kept_idx ``[n_planes, total_kept]`` (positions relative
    to each sequence start); offsets are device int64 ``[n_seq + 1]``."""
    _dev(norms, in_offsets, out_offsets, kept_idx)
    n_planes, total = norms.shape
    n_seq = in_offsets.numel() - 1
    _i64(out_offsets, n_seq + 1)
    assert norms.dtype == torch.float32 and kept_idx.dtype == torch.int32 and kept_idx.shape[0] == n_planes
    _check("l2kv_select_ragged", lib().l2kv_select_ragged(
        _ptr(norms), n_planes, n_seq, total, _ptr(in_offsets), _ptr(out_offsets), kept_idx.shape[1],
        int(max_len), int(mode), _ptr(kept_idx), _stream(stream)))


def l2kv_compact_ragged(K: torch.Tensor, V: torch.Tensor, norms: torch.Tensor, kept_idx: torch.Tensor,
                        in_offsets: torch.Tensor, out_offsets: torch.Tensor, max_kept: int,
                        slot_offsets: torch.Tensor, Kc: torch.Tensor, Vc: torch.Tensor,
                        norms_c: torch.Tensor, pos_c: torch.Tensor, stream=None) -> None:
    """K, V ``[n_planes, total_tokens, D]`` -> slot cache Kc, Vc ``[n_planes, total_slots, D]``,
    norms_c, pos_c ``[n_planes, total_slots]``."""
    _dev(K, V, norms, kept_idx, in_offsets, out_offsets, slot_offsets, Kc, Vc, norms_c, pos_c)
    n_planes, total, D = K.shape
    n_seq = in_offsets.numel() - 1
    total_slots = Kc.shape[1]
    assert V.shape == K.shape and Kc.shape == (n_planes, total_slots, D) and Vc.shape == Kc.shape
    assert norms.shape == (n_planes, total) and norms_c.shape == (n_planes, total_slots)
    assert pos_c.shape == (n_planes, total_slots) and pos_c.dtype == torch.int32
    _i64(out_offsets, n_seq + 1)
    _i64(slot_offsets, n_seq + 1)
    _check("l2kv_compact_ragged", lib().l2kv_compact_ragged(
        _ptr(K), _ptr(V), _ptr(norms), _dtype_code(K), _ptr(kept_idx), n_planes, n_seq, total,
        _ptr(in_offsets), _ptr(out_offsets), kept_idx.shape[1], int(max_kept), _ptr(slot_offsets),
        total_slots, D, _ptr(Kc), _ptr(Vc), _ptr(norms_c), _ptr(pos_c), _stream(stream)))


def l2kv_stream_append(Knew: torch.Tensor, Vnew: torch.Tensor, token_ids: torch.Tensor,
                       slot_offsets: torch.Tensor, lens_in: torch.Tensor, lens_out: torch.Tensor,
                       Kc: torch.Tensor, Vc: torch.Tensor, norms_c: torch.Tensor, pos_c: torch.Tensor,
                       stream=None) -> None:
    """Knew, Vnew ``[n_layers, n_seq, Hkv, D]`` -> next free slot of every sequence."""
    _dev(Knew, Vnew, token_ids, slot_offsets, lens_in, lens_out, Kc, Vc, norms_c, pos_c)
    n_layers, n_seq, Hkv, D = Knew.shape
    n_planes, total_slots, Dc = Kc.shape
    assert Vnew.shape == Knew.shape and n_planes == n_layers * Hkv and Dc == D and Vc.shape == Kc.shape
    _i32(token_ids, n_seq), _i32(lens_in, n_seq), _i32(lens_out, n_seq), _i64(slot_offsets, n_seq + 1)
    _check("l2kv_stream_append", lib().l2kv_stream_append(
        _ptr(Knew), _ptr(Vnew), _dtype_code(Knew), n_layers, n_seq, Hkv, D, _ptr(token_ids),
        _ptr(slot_offsets), total_slots, _ptr(lens_in), _ptr(lens_out), _ptr(Kc), _ptr(Vc),
        _ptr(norms_c), _ptr(pos_c), _stream(stream)))


def l2kv_stream_evict(slot_offsets: torch.Tensor, lens_in: torch.Tensor, budgets: torch.Tensor,
                      lens_out: torch.Tensor, Kc: torch.Tensor, Vc: torch.Tensor,
                      norms_c: torch.Tensor, pos_c: torch.Tensor, stream=None) -> None:
    _dev(slot_offsets, lens_in, budgets, lens_out, Kc, Vc, norms_c, pos_c)
    n_planes, total_slots, D = Kc.shape
    n_seq = lens_in.numel()
    _i32(lens_in, n_seq), _i32(budgets, n_seq), _i32(lens_out, n_seq), _i64(slot_offsets, n_seq + 1)
    _check("l2kv_stream_evict", lib().l2kv_stream_evict(
        _dtype_code(Kc), n_planes, n_seq, D, _ptr(slot_offsets), total_slots, _ptr(lens_in),
        _ptr(budgets), _ptr(lens_out), _ptr(Kc), _ptr(Vc), _ptr(norms_c), _ptr(pos_c), _stream(stream)))


def l2kv_decode_attn_ragged(Q: torch.Tensor, Kc: torch.Tensor, Vc: torch.Tensor, lens: torch.Tensor,
                            slot_offsets: torch.Tensor, max_len: int, O: torch.Tensor,
                            workspace: torch.Tensor, scale: float = 0.0, n_splits: int = 0,
                            seq_order: Optional[torch.Tensor] = None, stream=None) -> None:
    """Q ``[n_seq, Hq, D]``, Kc/Vc ``[Hkv, total_slots, D]`` (one layer) -> O ``[n_seq, Hq, D]``."""
    _dev(Q, Kc, Vc, lens, slot_offsets, O, workspace, seq_order)
    n_seq, Hq, D = Q.shape
    Hkv, total_slots, Dc = Kc.shape
    assert Dc == D and Vc.shape == Kc.shape and Kc.dtype == Q.dtype == Vc.dtype
    assert O.dtype == torch.float32 and O.numel() == n_seq * Hq * D
    _i32(lens, n_seq), _i64(slot_offsets, n_seq + 1)
    if seq_order is not None:
        _i32(seq_order, n_seq)
    _check("l2kv_decode_attn_ragged", lib().l2kv_decode_attn_ragged(
        _ptr(Q), _ptr(Kc), _ptr(Vc), _dtype_code(Q), n_seq, Hq, Hkv, D, _ptr(lens), _ptr(slot_offsets),
        _ptr(seq_order), total_slots, int(max_len), float(scale), int(n_splits), _ptr(O), _ptr(workspace),
        workspace.numel() * workspace.element_size(), _stream(stream)))


def l2kv_length_order(lens: torch.Tensor, order: torch.Tensor, stream=None) -> None:
    """lens ``[n_seq]`` int32 -> order ``[n_seq]`` int32 (pre-allocated): longest sequence first."""
    _dev(lens, order)
    n_seq = lens.numel()
    _i32(lens, n_seq), _i32(order, n_seq)
    _check("l2kv_length_order", lib().l2kv_length_order(_ptr(lens), n_seq, _ptr(order), _stream(stream)))


# ------------------------------------------------------------ attention-loss analysis
def l2kv_norm_ranks_workspace_bytes(n_heads: int, T: int) -> int:
    return int(lib().l2kv_norm_ranks_workspace_bytes(int(n_heads), int(T)))


def l2kv_alr_workspace_bytes(B: int, Hq: int, T: int) -> int:
    return int(lib().l2kv_alr_workspace_bytes(int(B), int(Hq), int(T)))


def l2kv_norm_ranks(norms: torch.Tensor, drop_rank: torch.Tensor, workspace: torch.Tensor,
                    stream=None) -> None:
    """norms ``[..., T]`` float32 -> drop_rank ``[..., T]`` int32 (pre-allocated)."""
    _dev(norms, drop_rank, workspace)
    T = norms.shape[-1]
    n = norms.numel() // T
    assert norms.dtype == torch.float32 and drop_rank.dtype == torch.int32 and drop_rank.numel() == n * T
    _check("l2kv_norm_ranks", lib().l2kv_norm_ranks(
        _ptr(norms), n, T, _ptr(drop_rank), _ptr(workspace), workspace.numel() * workspace.element_size(),
        _stream(stream)))


def l2kv_alr(Q: torch.Tensor, K: torch.Tensor, drop_rank: torch.Tensor, m: int, alr: torch.Tensor,
             loss: Optional[torch.Tensor], loss_ref: Optional[torch.Tensor], workspace: torch.Tensor,
             scale: float = 0.0, stream=None) -> None:
    """Q ``[B, Hq, D]``, K ``[B, Hkv, T, D]``, drop_rank ``[B, Hkv, T]`` int32 -> alr, loss,
    loss_ref ``[B, Hq]`` float64 (pre-allocated; the last two optional)."""
    _dev(Q, K, drop_rank, alr, loss, loss_ref, workspace)
    B, Hq, D = Q.shape
    Bk, Hkv, T, Dk = K.shape
    assert (Bk, Dk) == (B, D) and K.dtype == Q.dtype
    assert drop_rank.dtype == torch.int32 and drop_rank.numel() == B * Hkv * T
    for out in (alr, loss, loss_ref):
        assert out is None or (out.dtype == torch.float64 and out.numel() == B * Hq)
    _check("l2kv_alr", lib().l2kv_alr(
        _ptr(Q), _ptr(K), _dtype_code(Q), _ptr(drop_rank), B, Hq, Hkv, T, D, T * D, float(scale), int(m),
        _ptr(alr), _ptr(loss), _ptr(loss_ref), _ptr(workspace),
        workspace.numel() * workspace.element_size(), _stream(stream)))

"""CPU oracle for the L2-norm KV-cache compression hot path (arXiv 2406.11430).

TEST INFRASTRUCTURE ONLY: tests, the smoke check and the benchmark's
``cpu_baseline`` leg may import this package; the product never does, and this
package never imports the product.  It wraps ``l2kv_oracle.c`` (plain C, built
with gcc) behind NumPy arrays.  bf16 tensors travel as ``uint16`` bit patterns.

Functions, each following the passage named in the C source:

* ``keep_count(T, r)``            -- kept rows k = ceil(r*T) (Sec. 3, |D| = m exact)
* ``norms(K, dtype)``             -- squared key norms, fp32 fixed order + fp64
* ``select(n32, k, mode)``        -- lowest-norm positions (Sec. 1 rule), full sort
* ``compact(X, idx)``             -- gather of kept rows (Sec. 1: values stay with their keys)
* ``decode_attn(Q, Kc, Vc, ...)`` -- single-query softmax attention (Eq. 2 / Eq. 4)
* ``compress(K, V, dtype, r)``    -- the three compression steps in sequence
* ``StreamHead``                  -- one (sequence, head) cache under streaming
                                     eviction (Sec. 4, language-modelling setting)
* ``length_order(lens)``          -- longest-first order of a ragged batch (a scheduling aid
                                     of the library, not part of the paper's method)
* ``attn_probs(Q, K, dtype)``     -- attention scores a_p of one query over the full cache (Eq. 2)
* ``drop_order(n32)``             -- positions in the order the norm rule discards them
* ``attention_loss(a, n32, m)``   -- attention mass of the m dropped pairs (Eq. 5)
* ``attention_loss_ref(a, m)``    -- the same for the ideal rule (lowest attention first)
* ``alr(a, n32)``                 -- gap Y^m (Eq. 6) for m = 1..T and its sum Y (Eq. 7)
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from typing import Optional, Tuple

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "l2kv_oracle.c")
_LIB = os.path.join(_HERE, "libl2kv_oracle.so")

F32, BF16 = 0, 1
_DT = {"f32": F32, "bf16": BF16, F32: F32, BF16: BF16}
MODE_LOWEST, MODE_HIGHEST = 0, 1


def build(force: bool = False) -> str:
    """Compile the C oracle with gcc (no contraction, no fast-math)."""
    stale = (not os.path.exists(_LIB)
             or os.path.getmtime(_LIB) < os.path.getmtime(_SRC))
    if force or stale:
        tmp = _LIB + ".tmp.%d" % os.getpid()
        subprocess.run(
            ["gcc", "-O2", "-std=c11", "-ffp-contract=off", "-fno-fast-math",
             "-Wall", "-Wextra", "-shared", "-fPIC", _SRC, "-o", tmp, "-lm"],
            check=True)
        os.replace(tmp, _LIB)
    return _LIB


_lib = None


def _load():
    global _lib
    if _lib is None:
        lib = ctypes.CDLL(build())
        c = ctypes
        lib.l2kv_oracle_keep_count.restype = c.c_int64
        lib.l2kv_oracle_keep_count.argtypes = [c.c_int64, c.c_double]
        lib.l2kv_oracle_norms.restype = c.c_int
        lib.l2kv_oracle_norms.argtypes = [
            c.c_void_p, c.c_int, c.c_int64, c.c_int64, c.c_int32, c.c_int64,
            c.c_void_p, c.c_void_p]
        lib.l2kv_oracle_select.restype = c.c_int
        lib.l2kv_oracle_select.argtypes = [
            c.c_void_p, c.c_int64, c.c_int64, c.c_int, c.c_void_p]
        lib.l2kv_oracle_compact.restype = None
        lib.l2kv_oracle_compact.argtypes = [
            c.c_void_p, c.c_void_p, c.c_int64, c.c_int64, c.c_void_p]
        lib.l2kv_oracle_decode_attn.restype = c.c_int
        lib.l2kv_oracle_decode_attn.argtypes = [
            c.c_void_p, c.c_void_p, c.c_void_p, c.c_int, c.c_int32, c.c_int32,
            c.c_int32, c.c_int64, c.c_int32, c.c_int64, c.c_double, c.c_void_p]
        lib.l2kv_oracle_random_keys.restype = None
        lib.l2kv_oracle_random_keys.argtypes = [c.c_int64, c.c_int64, c.c_uint32, c.c_void_p]
        lib.l2kv_oracle_stream_append.restype = c.c_int
        lib.l2kv_oracle_stream_append.argtypes = [
            c.c_void_p, c.c_void_p, c.c_void_p, c.c_void_p, c.c_void_p, c.c_int32, c.c_int,
            c.c_int32, c.c_void_p, c.c_void_p, c.c_int32]
        lib.l2kv_oracle_stream_evict.restype = c.c_int
        lib.l2kv_oracle_stream_evict.argtypes = [
            c.c_void_p, c.c_void_p, c.c_void_p, c.c_void_p, c.c_void_p, c.c_int32, c.c_int, c.c_int32]
        _lib = lib
    return _lib


def _np_dtype(dtype) -> np.dtype:
    return np.dtype(np.uint16) if _DT[dtype] == BF16 else np.dtype(np.float32)


def _check(a: np.ndarray, dtype) -> np.ndarray:
    want = _np_dtype(dtype)
    if a.dtype != want:
        raise TypeError("expected %s array for dtype %r, got %s" % (want, dtype, a.dtype))
    return np.ascontiguousarray(a)


def keep_count(T: int, keep_ratio: float) -> int:
    return int(_load().l2kv_oracle_keep_count(int(T), float(keep_ratio)))


def norms(K: np.ndarray, dtype) -> Tuple[np.ndarray, np.ndarray]:
    """K ``[..., T, D]`` -> (n32 ``[..., T]`` float32, n64 ``[..., T]`` float64)."""
    K = _check(K, dtype)
    *lead, T, D = K.shape
    n_heads = int(np.prod(lead)) if lead else 1
    n32 = np.empty((n_heads, T), dtype=np.float32)
    n64 = np.empty((n_heads, T), dtype=np.float64)
    rc = _load().l2kv_oracle_norms(K.ctypes.data, _DT[dtype], n_heads, T, D,
                                   T * D, n32.ctypes.data, n64.ctypes.data)
    if rc != 0:
        raise ValueError("oracle norms: unsupported shape/dtype (D=%d)" % D)
    return n32.reshape(*lead, T), n64.reshape(*lead, T)


def select(n32: np.ndarray, k: int, mode: int = MODE_LOWEST) -> np.ndarray:
    """n32 ``[..., T]`` -> kept indices ``[..., k]`` int32, ascending per head."""
    n32 = np.ascontiguousarray(n32, dtype=np.float32)
    *lead, T = n32.shape
    flat = n32.reshape(-1, T)
    out = np.empty((flat.shape[0], k), dtype=np.int32)
    lib = _load()
    for h in range(flat.shape[0]):
        rc = lib.l2kv_oracle_select(flat[h].ctypes.data, T, k, mode,
                                    out[h].ctypes.data)
        if rc != 0:
            raise ValueError("oracle select failed (rc=%d, T=%d, k=%d)" % (rc, T, k))
    return out.reshape(*lead, k)


def compact(X: np.ndarray, kept_idx: np.ndarray) -> np.ndarray:
    """X ``[..., T, D]``, kept_idx ``[..., k]`` -> ``[..., k, D]`` (byte copy)."""
    X = np.ascontiguousarray(X)
    kept_idx = np.ascontiguousarray(kept_idx, dtype=np.int32)
    *lead, T, D = X.shape
    k = kept_idx.shape[-1]
    Xf = X.reshape(-1, T, D)
    If = kept_idx.reshape(-1, k)
    assert Xf.shape[0] == If.shape[0]
    if k and (If.min() < 0 or If.max() >= T):
        raise IndexError("kept index out of range")
    out = np.empty((Xf.shape[0], k, D), dtype=X.dtype)
    lib = _load()
    for h in range(Xf.shape[0]):
        lib.l2kv_oracle_compact(Xf[h].ctypes.data, If[h].ctypes.data, k,
                                D * X.dtype.itemsize, out[h].ctypes.data)
    return out.reshape(*lead, k, D)


def decode_attn(Q: np.ndarray, Kc: np.ndarray, Vc: np.ndarray, dtype,
                scale: float = 0.0) -> np.ndarray:
    """Q ``[B, Hq, D]``, Kc/Vc ``[B, Hkv, n, D]`` -> O ``[B, Hq, D]`` float32."""
    Q = _check(Q, dtype)
    Kc = _check(Kc, dtype)
    Vc = _check(Vc, dtype)
    B, Hq, D = Q.shape
    Bk, Hkv, n, Dk = Kc.shape
    assert (Bk, Dk) == (B, D) and Vc.shape == Kc.shape
    O = np.empty((B, Hq, D), dtype=np.float32)
    rc = _load().l2kv_oracle_decode_attn(
        Q.ctypes.data, Kc.ctypes.data, Vc.ctypes.data, _DT[dtype], B, Hq, Hkv,
        n, D, n * D, float(scale), O.ctypes.data)
    if rc != 0:
        raise ValueError("oracle decode_attn: bad arguments (rc=%d)" % rc)
    return O


def compress(K: np.ndarray, V: np.ndarray, dtype, keep_ratio: float,
             mode: int = MODE_LOWEST, k: Optional[int] = None):
    """norms -> select -> compact.  Returns (n32, n64, kept_idx, Kc, Vc)."""
    n32, n64 = norms(K, dtype)
    if k is None:
        k = keep_count(K.shape[-2], keep_ratio)
    idx = select(n32, k, mode)
    return n32, n64, idx, compact(K, idx), compact(V, idx)


def random_keys(n_heads: int, T: int, seed: int) -> np.ndarray:
    """Keys of the keep-random control (Sec. 4): ``[n_heads, T]`` float32 whose BIT
    PATTERNS are a counter-based hash of (seed, head, token); feed to ``select``."""
    keys = np.empty((n_heads, T), dtype=np.float32)
    _load().l2kv_oracle_random_keys(int(n_heads), int(T), int(seed) & 0xFFFFFFFF, keys.ctypes.data)
    return keys


def length_order(lens) -> np.ndarray:
    """Indices of the sequences from longest to shortest, equal lengths in index order."""
    lens = np.asarray(lens, dtype=np.int64)
    return np.lexsort((np.arange(lens.shape[0]), -lens)).astype(np.int32)


class StreamHead:
    """One (sequence, head) slot cache under streaming eviction: append a token,
    attend, then drop highest-norm tokens until the budget holds (Sec. 4,
    "Language Modelling Tasks").  Slots carry K/V rows, the fp32 squared norm
    and the original token id; slot order has no meaning."""

    def __init__(self, capacity: int, D: int, dtype):
        self.dtype, self.D, self.capacity = dtype, int(D), int(capacity)
        npdt = _np_dtype(dtype)
        self.K = np.zeros((capacity, D), dtype=npdt)
        self.V = np.zeros((capacity, D), dtype=npdt)
        self.norms = np.zeros(capacity, dtype=np.float32)
        self.pos = np.full(capacity, -1, dtype=np.int32)
        self._len = ctypes.c_int32(0)

    def __len__(self) -> int:
        return int(self._len.value)

    def load(self, K: np.ndarray, V: np.ndarray, n32: np.ndarray, pos: np.ndarray) -> None:
        """Start from an already compressed cache (rows, norms, token ids)."""
        n = K.shape[0]
        assert n <= self.capacity
        self.K[:n], self.V[:n], self.norms[:n], self.pos[:n] = K, V, n32, pos
        self._len.value = n

    def append(self, k_new: np.ndarray, v_new: np.ndarray, token_id: int) -> None:
        k_new = _check(k_new, self.dtype)
        v_new = _check(v_new, self.dtype)
        rc = _load().l2kv_oracle_stream_append(
            self.K.ctypes.data, self.V.ctypes.data, self.norms.ctypes.data, self.pos.ctypes.data,
            ctypes.byref(self._len), self.capacity, _DT[self.dtype], self.D,
            k_new.ctypes.data, v_new.ctypes.data, int(token_id))
        if rc != 0:
            raise ValueError("stream append: cache full or bad shape")

    def evict_to(self, budget: int) -> int:
        return int(_load().l2kv_oracle_stream_evict(
            self.K.ctypes.data, self.V.ctypes.data, self.norms.ctypes.data, self.pos.ctypes.data,
            ctypes.byref(self._len), int(budget), _DT[self.dtype], self.D))

    def attend(self, q: np.ndarray, scale: float = 0.0) -> np.ndarray:
        """q ``[G, D]`` (the query heads sharing this KV head) -> ``[G, D]`` float32."""
        n = len(self)
        return decode_attn(np.ascontiguousarray(q)[None], self.K[None, None, :n], self.V[None, None, :n],
                           self.dtype, scale)[0]

    def kept(self):
        """(token ids ascending, K rows, V rows, norms) of the occupied slots."""
        n = len(self)
        order = np.argsort(self.pos[:n], kind="stable")
        return self.pos[:n][order], self.K[:n][order], self.V[:n][order], self.norms[:n][order]


# ---------------------------------------------------------------------------
# Attention-loss analysis (Sec. 3, Eq. 5-7).  NumPy, float64.
# ---------------------------------------------------------------------------

def _to_f64(x: np.ndarray, dtype) -> np.ndarray:
    x = _check(x, dtype)
    if _DT[dtype] == BF16:                       # bf16 = upper half of an fp32 bit pattern
        return (x.astype(np.uint32) << np.uint32(16)).view(np.float32).astype(np.float64)
    return x.astype(np.float64)


def attn_probs(Q: np.ndarray, K: np.ndarray, dtype, scale: float = 0.0) -> np.ndarray:
    """Attention scores of one query per head over ALL cached keys (Eq. 2):
    Q ``[B, Hq, D]``, K ``[B, Hkv, T, D]`` -> a ``[B, Hq, T]`` float64, each row a
    softmax of q.K_p / sqrt(D) (or q.K_p * scale when scale > 0).  Query head hq
    reads KV head hq // (Hq // Hkv)."""
    q, k = _to_f64(Q, dtype), _to_f64(K, dtype)
    B, Hq, D = q.shape
    Bk, Hkv, T, Dk = k.shape
    assert (Bk, Dk) == (B, D) and Hq % Hkv == 0
    G = Hq // Hkv
    a = np.empty((B, Hq, T), dtype=np.float64)
    for b in range(B):
        for hq in range(Hq):
            s = k[b, hq // G] @ q[b, hq]
            s = s * scale if scale > 0.0 else s / np.sqrt(float(D))
            e = np.exp(s - s.max())
            a[b, hq] = e / e.sum()
    return a


def drop_order(n32: np.ndarray) -> np.ndarray:
    """For one head, n32 ``[T]`` float32 -> the T positions in the order the
    norm rule discards them: highest squared norm first; among equal norms the
    later token goes first (the selection keeps the earlier one, Sec. 1 rule as
    read by ``select``).  The m dropped pairs D of Eq. 5 are the first m entries."""
    n32 = np.ascontiguousarray(n32, dtype=np.float32)
    assert n32.ndim == 1
    bits = n32.view(np.uint32)
    keep_order = np.lexsort((np.arange(n32.shape[0]), bits))      # ascending (bits, index)
    return keep_order[::-1].copy()


def attention_loss(a: np.ndarray, n32: np.ndarray, m: int) -> float:
    """Eq. 5 for the norm rule: sum of the attention scores of the m dropped pairs."""
    D = drop_order(n32)[:m]
    return float(np.sum(np.asarray(a, dtype=np.float64)[D]))


def attention_loss_ref(a: np.ndarray, m: int) -> float:
    """Reference loss of Eq. 6: the ideal rule drops the m lowest attention scores."""
    return float(np.sum(np.sort(np.asarray(a, dtype=np.float64))[:m]))


def alr(a: np.ndarray, n32: np.ndarray) -> Tuple[float, np.ndarray]:
    """For one head, a ``[T]`` attention scores and n32 ``[T]`` squared norms ->
    (Y, Ym) with Ym[m-1] = L^m - L^{m,ref} for m = 1..T (Eq. 6) and Y their sum
    (Eq. 7)."""
    a = np.asarray(a, dtype=np.float64)
    T = a.shape[0]
    L = np.cumsum(a[drop_order(n32)])             # L[m-1]     = loss of dropping m pairs by norm
    Lref = np.cumsum(np.sort(a))                  # Lref[m-1]  = loss of dropping the m lowest scores
    Ym = L - Lref
    assert Ym.shape == (T,)
    return float(Ym.sum()), Ym


def alr_heads(Q: np.ndarray, K: np.ndarray, n32: np.ndarray, dtype, m: int, scale: float = 0.0):
    """Per query head: (Y, L^m, L^{m,ref}), each ``[B, Hq]`` float64, from raw Q
    ``[B, Hq, D]``, K ``[B, Hkv, T, D]`` and the squared norms n32 ``[B, Hkv, T]``."""
    a = attn_probs(Q, K, dtype, scale)
    B, Hq, T = a.shape
    G = Hq // K.shape[1]
    Y = np.empty((B, Hq)); Lm = np.empty((B, Hq)); Lref = np.empty((B, Hq))
    for b in range(B):
        for hq in range(Hq):
            nh = n32[b, hq // G]
            Y[b, hq] = alr(a[b, hq], nh)[0]
            Lm[b, hq] = attention_loss(a[b, hq], nh, m)
            Lref[b, hq] = attention_loss_ref(a[b, hq], m)
    return Y, Lm, Lref

"""ctypes front end of the ShadowKV CPU oracle -- TEST INFRASTRUCTURE ONLY.

Builds ``shadowkv_oracle.c`` with gcc (``-O2 -fopenmp``, no intrinsics) into
``liboracle_shadowkv.so`` beside it and exposes the two operations as numpy
functions.  bf16 tensors travel as ``uint16`` arrays holding the raw bits, FP8 (E5M2) tensors of the
KV cache (``OracleParams.kv_dtype = 1``) as ``uint8`` arrays.

Only tests, the smoke check and the benchmark's ``cpu_baseline`` leg may import
this module; the GPU library never does.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess
from dataclasses import dataclass
from typing import Optional

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "shadowkv_oracle.c")
# SHADOWKV_ORACLE_LIB points the wrapper at another build of the oracle (used by the mutation test only)
_LIB = os.environ.get("SHADOWKV_ORACLE_LIB", os.path.join(_HERE, "liboracle_shadowkv.so"))
_lib = None


def build(force: bool = False) -> str:
    """Compile the oracle if the library is missing or older than its source."""
    if "SHADOWKV_ORACLE_LIB" in os.environ:
        return _LIB
    stale = (not os.path.exists(_LIB)) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC)
    if force or stale:
        tmp = f"{_LIB}.{os.getpid()}.tmp"   # several test workers may build at once: replace atomically
        cmd = ["gcc", "-std=c99", "-O2", "-fopenmp", "-fPIC", "-shared", "-Wall", "-Wextra",
               "-o", tmp, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
        os.replace(tmp, _LIB)
    return _LIB


class _Params(C.Structure):
    _fields_ = [
        ("batch", C.c_int32), ("n_q_heads", C.c_int32), ("n_kv_heads", C.c_int32),
        ("head_dim", C.c_int32), ("ctx_len", C.c_int32), ("chunk_size", C.c_int32),
        ("rank", C.c_int32), ("n_outlier_chunks", C.c_int32), ("topk_chunks", C.c_int32),
        ("local_len", C.c_int32), ("rope_theta", C.c_double), ("inv_freq", C.c_void_p),
        ("softmax_scale", C.c_double), ("ctx_capacity", C.c_int32), ("kv_dtype", C.c_int32),
    ]


@dataclass
class OracleParams:
    batch: int
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    ctx_len: int
    chunk_size: int
    rank: int
    n_outlier_chunks: int
    topk_chunks: int
    local_len: int
    rope_theta: float = 5e5
    inv_freq: Optional[np.ndarray] = None  # float32 [head_dim/2]
    softmax_scale: float = 0.0
    ctx_capacity: int = 0  # tokens the context arrays are laid out for (0 => ctx_len)
    kv_dtype: int = 0      # storage of the KV-cache tensors: 0 = bf16 (uint16 bits), 1 = FP8 E5M2 (uint8 bits)

    @property
    def kv_numpy(self):
        return np.uint8 if self.kv_dtype == 1 else np.uint16

    @property
    def n_chunks(self) -> int:
        return self.ctx_len // self.chunk_size

    @property
    def capacity(self) -> int:
        return self.ctx_capacity or self.ctx_len

    @property
    def landmark_capacity(self) -> int:
        return self.capacity // self.chunk_size - self.n_outlier_chunks

    @property
    def n_landmarks(self) -> int:
        return self.n_chunks - self.n_outlier_chunks

    def _c(self):
        inv = None
        if self.inv_freq is not None:
            inv = np.ascontiguousarray(self.inv_freq, dtype=np.float32)
            assert inv.shape == (self.head_dim // 2,)
        st = _Params(self.batch, self.n_q_heads, self.n_kv_heads, self.head_dim, self.ctx_len,
                     self.chunk_size, self.rank, self.n_outlier_chunks, self.topk_chunks,
                     self.local_len, float(self.rope_theta),
                     inv.ctypes.data if inv is not None else None, float(self.softmax_scale),
                     int(self.ctx_capacity), int(self.kv_dtype))
        return st, inv  # keep `inv` alive while the struct is in use


def _load():
    global _lib
    if _lib is None:
        build()
        _lib = C.CDLL(_LIB)
        _lib.oracle_num_threads.restype = C.c_int
        _lib.oracle_f64_to_bf16.restype = C.c_uint16
        _lib.oracle_f64_to_bf16.argtypes = [C.c_double]
        _lib.oracle_f64_to_e5m2.restype = C.c_uint8
        _lib.oracle_f64_to_e5m2.argtypes = [C.c_double]
        _lib.oracle_e5m2_to_f64.restype = C.c_double
        _lib.oracle_e5m2_to_f64.argtypes = [C.c_uint8]
        _lib.oracle_rope.restype = None
        _lib.oracle_rope.argtypes = [C.c_void_p] * 3 + [C.c_int64, C.c_void_p]
        _lib.oracle_build_landmarks.restype = C.c_int
        _lib.oracle_build_landmarks.argtypes = [C.c_void_p] * 10
        _lib.oracle_decode_step.restype = C.c_int
        _lib.oracle_decode_step.argtypes = [C.c_void_p] * 17
        _lib.oracle_append_chunk.restype = C.c_int
        _lib.oracle_append_chunk.argtypes = [C.c_void_p] * 9
        _lib.oracle_cache_update.restype = C.c_int
        _lib.oracle_cache_update.argtypes = [C.c_int64, C.c_int, C.c_int] + [C.c_void_p] * 6
    return _lib


def num_threads() -> int:
    return int(_load().oracle_num_threads())


def as_bits(x, kv_dtype: int = 0) -> np.ndarray:
    """bf16 torch tensor (CPU) or uint16 ndarray -> contiguous uint16 ndarray of raw bits; with
    ``kv_dtype = 1`` an E5M2 torch tensor, a uint8 torch tensor or a uint8 ndarray -> uint8 ndarray."""
    want = np.uint8 if kv_dtype == 1 else np.uint16
    if isinstance(x, np.ndarray):
        assert x.dtype == want, (x.dtype, want)
        return np.ascontiguousarray(x)
    import torch
    assert x.device.type == "cpu"
    if kv_dtype == 1:
        assert x.dtype in (torch.float8_e5m2, torch.uint8), x.dtype
        return x.contiguous().view(torch.uint8).numpy()
    assert x.dtype == torch.bfloat16
    return x.contiguous().view(torch.int16).numpy().view(np.uint16)


def bits_to_f64(bits: np.ndarray) -> np.ndarray:
    """Exact widening of bf16 bit patterns to float64."""
    return (bits.astype(np.uint32) << 16).view(np.float32).astype(np.float64)


def f64_to_bits(x: np.ndarray) -> np.ndarray:
    """Single-rounding (nearest-even) fp64 -> bf16 bits, elementwise through the C routine."""
    lib = _load()
    flat = np.asarray(x, dtype=np.float64).ravel()
    out = np.fromiter((lib.oracle_f64_to_bf16(float(v)) for v in flat), dtype=np.uint16, count=flat.size)
    return out.reshape(np.shape(x))


def e5m2_bits_to_f64(bits: np.ndarray) -> np.ndarray:
    """Exact widening of E5M2 bytes to float64, elementwise through the C routine's table of 256 values."""
    lib = _load()
    table = np.array([lib.oracle_e5m2_to_f64(i) for i in range(256)], dtype=np.float64)
    return table[np.asarray(bits, dtype=np.uint8)]


def f64_to_e5m2_bits(x: np.ndarray) -> np.ndarray:
    """Single-rounding (nearest-even) fp64 -> E5M2 bytes, elementwise through the C routine."""
    lib = _load()
    flat = np.asarray(x, dtype=np.float64).ravel()
    out = np.fromiter((lib.oracle_f64_to_e5m2(float(v)) for v in flat), dtype=np.uint8, count=flat.size)
    return out.reshape(np.shape(x))


def _ptr(a: Optional[np.ndarray]):
    return None if a is None else a.ctypes.data


def rope(p: OracleParams, x: np.ndarray, pos: np.ndarray) -> np.ndarray:
    """y[n] = RoPE(x[n], pos[n]) in fp64; x [n, d]."""
    lib = _load()
    x = np.ascontiguousarray(x, dtype=np.float64)
    pos = np.ascontiguousarray(pos, dtype=np.float64)
    assert x.ndim == 2 and x.shape[1] == p.head_dim and pos.shape == (x.shape[0],)
    y = np.empty_like(x)
    st, keep = p._c()
    lib.oracle_rope(C.addressof(st), x.ctypes.data, pos.ctypes.data, x.shape[0], y.ctypes.data)
    del keep
    return y


def build_landmarks(p: OracleParams, k_rope, v=None, diagnostics: bool = False) -> dict:
    """Alg. 1 after the SVD.  k_rope [b, h_kv, s, d], v = value store [b, h_kv, cap, d], bf16 bits."""
    lib = _load()
    b, h, s, d, c, o = p.batch, p.n_kv_heads, p.ctx_len, p.head_dim, p.chunk_size, p.n_outlier_chunks
    n_ch, n_c = p.n_chunks, p.landmark_capacity
    k_rope = as_bits(k_rope, p.kv_dtype)
    assert k_rope.shape == (b, h, s, d), k_rope.shape
    if v is not None:
        v = as_bits(v, p.kv_dtype)
        assert v.shape == (b, h, p.capacity, d)
    kvt = p.kv_numpy
    res = {
        "landmarks": np.zeros((b, h, n_c, d), kvt),
        "landmark_chunk_ids": np.zeros((b, h, n_c), np.int32),
        "outlier_chunk_ids": np.zeros((b, h, o), np.int32),
        "k_outlier": np.zeros((b, h, o * c, d), kvt),
        "v_outlier": np.zeros((b, h, o * c, d), kvt) if v is not None else None,
        "chunk_min_cos": np.zeros((b, h, n_ch), np.float64) if diagnostics else None,
        "chunk_mean": np.zeros((b, h, n_ch, d), np.float64) if diagnostics else None,
    }
    st, keep = p._c()
    rc = lib.oracle_build_landmarks(C.addressof(st), _ptr(k_rope), _ptr(v), _ptr(res["landmarks"]),
                                    _ptr(res["landmark_chunk_ids"]), _ptr(res["outlier_chunk_ids"]),
                                    _ptr(res["k_outlier"]), _ptr(res["v_outlier"]),
                                    _ptr(res["chunk_min_cos"]), _ptr(res["chunk_mean"]))
    del keep
    if rc != 0:
        raise ValueError(f"oracle_build_landmarks rejected its arguments (rc={rc})")
    return res


def decode_step(p: OracleParams, q, A, B, landmarks, landmark_chunk_ids, k_outlier, v_outlier,
                k_local, v_local, value_store, pos_offset=None, diagnostics: bool = True) -> dict:
    """Alg. 2 followed by softmax attention over [outliers ; selected chunks ; recent tokens]."""
    lib = _load()
    b, hq, h, s, d = p.batch, p.n_q_heads, p.n_kv_heads, p.ctx_len, p.head_dim
    c, r, o, k, w, n_c = p.chunk_size, p.rank, p.n_outlier_chunks, p.topk_chunks, p.local_len, p.n_landmarks
    cap, nc_cap = p.capacity, p.landmark_capacity
    t = p.kv_dtype
    q, A, B = as_bits(q), as_bits(A, t), as_bits(B, t)
    landmarks, value_store = as_bits(landmarks, t), as_bits(value_store, t)
    k_outlier, v_outlier = as_bits(k_outlier, t), as_bits(v_outlier, t)
    k_local, v_local = as_bits(k_local, t), as_bits(v_local, t)
    ids = np.ascontiguousarray(landmark_chunk_ids, dtype=np.int32)
    assert q.shape == (b, hq, d) and A.shape == (b, cap, r) and B.shape == (b, h, r, d)
    assert landmarks.shape == (b, h, nc_cap, d) and ids.shape == (b, h, nc_cap)
    assert k_outlier.shape == (b, h, o * c, d) and v_outlier.shape == (b, h, o * c, d)
    assert k_local.shape == (b, h, w, d) and v_local.shape == (b, h, w, d)
    assert value_store.shape == (b, h, cap, d)
    pos = None
    if pos_offset is not None:
        pos = np.ascontiguousarray(pos_offset, dtype=np.int32)
        assert pos.shape == (b,)
    res = {
        "out": np.zeros((b, hq, d), np.uint16),
        "out_f64": np.zeros((b, hq, d), np.float64),
        "chunk_ids": np.zeros((b, h, k), np.int32),
        "z2": np.zeros((b, h, n_c), np.float64) if diagnostics else None,
        "k_sparse": np.zeros((b, h, k * c, d), np.float64) if diagnostics else None,
    }
    st, keep = p._c()
    rc = lib.oracle_decode_step(C.addressof(st), _ptr(q), _ptr(A), _ptr(B), _ptr(landmarks), _ptr(ids),
                                _ptr(k_outlier), _ptr(v_outlier), _ptr(k_local), _ptr(v_local),
                                _ptr(value_store), _ptr(pos), _ptr(res["out"]), _ptr(res["out_f64"]),
                                _ptr(res["chunk_ids"]), _ptr(res["z2"]), _ptr(res["k_sparse"]))
    del keep
    if rc != 0:
        raise ValueError(f"oracle_decode_step rejected its arguments (rc={rc})")
    return res


def cache_update(sel_ids: np.ndarray, cache_ids: np.ndarray, stamps: Optional[np.ndarray] = None) -> dict:
    """Chunk cache of the offloaded values (section "High-throughput Decoding"): index scan of this
    step's selection ``sel_ids [units, k]`` (ascending) against the slots ``cache_ids [units, S]``
    (-1 = empty, S >= k), least-recently-used replacement with ``stamps [units, S+1]`` (last entry = the
    unit's clock; None = a fresh all-zero state).  Returns the new slot contents and stamps, the slot of
    every selected chunk, the slots to fill and their number per unit."""
    lib = _load()
    sel = np.ascontiguousarray(sel_ids, dtype=np.int32)
    cache = np.array(cache_ids, dtype=np.int32, order="C", copy=True)
    assert sel.ndim == 2 and cache.ndim == 2 and cache.shape[0] == sel.shape[0]
    units, k = sel.shape
    S = cache.shape[1]
    st = np.zeros((units, S + 1), np.int32) if stamps is None else np.array(stamps, dtype=np.int32, order="C", copy=True)
    assert st.shape == (units, S + 1)
    slots = np.zeros((units, k), np.int32)
    miss = np.zeros((units, k), np.int32)
    n_miss = np.zeros(units, np.int32)
    rc = lib.oracle_cache_update(units, k, S, sel.ctypes.data, cache.ctypes.data, st.ctypes.data, slots.ctypes.data,
                                 miss.ctypes.data, n_miss.ctypes.data)
    if rc != 0:
        raise ValueError(f"oracle_cache_update rejected its arguments (rc={rc})")
    return {"cache_ids": cache, "stamps": st, "sel_slots": slots, "miss_slots": miss, "n_miss": n_miss}


def append_chunk(p: OracleParams, k_pre, k_rope, v, B, A, landmarks, landmark_chunk_ids, value_store) -> None:
    """One more chunk of context from generated tokens (low-rank states K' Psi, landmark, values), written in
    place into ``A``, ``landmarks``, ``landmark_chunk_ids`` (int32) and ``value_store`` (uint16 ndarrays, uint8
    with E5M2 storage, laid out for ``p.capacity`` tokens).  ``p.ctx_len`` is the length BEFORE the call."""
    lib = _load()
    b, h, d, c, r = p.batch, p.n_kv_heads, p.head_dim, p.chunk_size, p.rank
    cap, nc_cap = p.capacity, p.landmark_capacity
    t, kvt = p.kv_dtype, p.kv_numpy
    k_pre, k_rope, v, B = as_bits(k_pre, t), as_bits(k_rope, t), as_bits(v, t), as_bits(B, t)
    assert k_pre.shape == (b, c, h * d) and k_rope.shape == (b, h, c, d) and v.shape == (b, h, c, d)
    assert B.shape == (b, h, r, d)
    for arr, shape, dt in ((A, (b, cap, r), kvt), (landmarks, (b, h, nc_cap, d), kvt),
                           (landmark_chunk_ids, (b, h, nc_cap), np.int32), (value_store, (b, h, cap, d), kvt)):
        assert isinstance(arr, np.ndarray) and arr.dtype == dt and arr.shape == shape and arr.flags.c_contiguous
    st, keep = p._c()
    rc = lib.oracle_append_chunk(C.addressof(st), _ptr(k_pre), _ptr(k_rope), _ptr(v), _ptr(B), _ptr(A),
                                 _ptr(landmarks), _ptr(landmark_chunk_ids), _ptr(value_store))
    del keep
    if rc != 0:
        raise ValueError(f"oracle_append_chunk rejected its arguments (rc={rc})")


def factorize_keys(p: OracleParams, k_pre) -> dict:
    """First line of the pre-filling algorithm, A, B <- SVD(K): per sequence the thin singular value decomposition
    K = Phi Sigma Psi^T of the pre-RoPE keys ``k_pre [b, s, h_kv*d]`` (stored bits, widened exactly to fp64; numpy's
    LAPACK SVD is the library step), truncated to the ``p.rank`` largest singular values.  ``B = Psi^T`` laid out
    ``[b, h_kv, r, d]`` (``B[h, rho, x] = Psi[h*d + x, rho]``), ``A = K Psi`` (``[b, capacity, r]``, rows beyond
    ``ctx_len`` left zero), both rounded once to the storage type.  Sign convention (an SVD leaves the sign of each
    singular pair open): the component of largest magnitude of every right singular vector is positive, ties to the
    lowest index.  Also returns ``psi [b, r, D]`` (rows = right singular vectors), ``sigma [b, r]`` and the unrounded
    ``A_f64 [b, s, r]``."""
    b, h, d, s, r = p.batch, p.n_kv_heads, p.head_dim, p.ctx_len, p.rank
    D = h * d
    bits = as_bits(k_pre, p.kv_dtype)
    assert bits.shape == (b, s, D), bits.shape
    assert 1 <= r <= min(s, D)
    widen = e5m2_bits_to_f64 if p.kv_dtype == 1 else bits_to_f64
    rnd = f64_to_e5m2_bits if p.kv_dtype == 1 else f64_to_bits
    psi = np.zeros((b, r, D))
    sigma = np.zeros((b, r))
    A64 = np.zeros((b, s, r))
    for bi in range(b):
        K = widen(bits[bi])
        _, sv, vt = np.linalg.svd(K, full_matrices=False)      # singular values in descending order
        v = vt[:r].copy()
        lead = np.argmax(np.abs(v), axis=1)                    # first index of the largest magnitude
        sign = np.where(v[np.arange(r), lead] < 0.0, -1.0, 1.0)
        v *= sign[:, None]
        psi[bi], sigma[bi] = v, sv[:r]
        A64[bi] = K @ v.T
    A = np.zeros((b, p.capacity, r), p.kv_numpy)
    A[:, :s] = rnd(A64)
    B = rnd(psi.reshape(b, r, h, d).transpose(0, 2, 1, 3))
    return {"A": A, "B": np.ascontiguousarray(B), "psi": psi, "sigma": sigma, "A_f64": A64}

"""ctypes binding of libshadowkv.so: argument marshalling only.

Every step of the path runs in the HIP library; this module turns torch tensors
into pointers, sizes the workspace and picks the streams.  There is no fallback:
if the library is missing, loading raises.
"""
from __future__ import annotations

import ctypes as C
import os
from dataclasses import dataclass
from typing import Optional

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.environ.get("SHADOWKV_LIB", os.path.join(_HERE, "libshadowkv.so"))

OK, EINVAL, EWORKSPACE, EHIP = 0, -1, -2, -3
VALUES_DEVICE, VALUES_HOST = 0, 1
FLAG_STAGE_VALUES = 1
FLAG_KEEP_REBUILT_KEYS = 2
KV_BF16, KV_FP8_E5M2 = 0, 1     # storage type of the KV-cache tensors (Params.kv_dtype)

EXPORTS = (
    "shadowkv_build_landmarks", "shadowkv_decode_step", "shadowkv_build_workspace_bytes",
    "shadowkv_decode_workspace_bytes", "shadowkv_validate_params", "shadowkv_decode_workspace_view",
    "shadowkv_status_string", "shadowkv_last_error", "shadowkv_version", "shadowkv_shutdown",
    "shadowkv_profile_begin", "shadowkv_profile_end", "shadowkv_decode_step_cached", "shadowkv_value_cache_bytes",
    "shadowkv_value_cache_reset", "shadowkv_append_chunk", "shadowkv_argtopk", "shadowkv_argtopk_workspace_bytes",
    "shadowkv_factorize_keys", "shadowkv_factorize_workspace_bytes", "shadowkv_decode_step_static",
    "shadowkv_static_scratch_bytes", "shadowkv_decode_plan",
)
STAGES = ("score", "select", "gather_values", "attention")


class CParams(C.Structure):
    _fields_ = [
        ("batch", C.c_int32), ("n_q_heads", C.c_int32), ("n_kv_heads", C.c_int32), ("head_dim", C.c_int32),
        ("ctx_len", C.c_int32), ("chunk_size", C.c_int32), ("rank", C.c_int32),
        ("n_outlier_chunks", C.c_int32), ("topk_chunks", C.c_int32), ("local_len", C.c_int32),
        ("value_location", C.c_int32), ("flags", C.c_uint32),
        ("rope_theta", C.c_double), ("softmax_scale", C.c_double), ("inv_freq", C.c_void_p),
        ("ctx_capacity", C.c_int32), ("kv_dtype", C.c_int32),
    ]


class ShadowKVError(RuntimeError):
    def __init__(self, status: int, detail: str):
        super().__init__(f"libshadowkv: {status_string(status)} ({status}): {detail}")
        self.status = status
        self.detail = detail


_lib = None


def lib() -> C.CDLL:
    """Load the HIP library (built beforehand by ``python -m paper_2410_21465_amd.build``)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise FileNotFoundError(
                f"{LIB_PATH} is missing: build it with `python -m paper_2410_21465_amd.build` "
                "(there is no non-HIP fallback)")
        L = C.CDLL(LIB_PATH)
        vp, sz, i32 = C.c_void_p, C.c_size_t, C.c_int
        L.shadowkv_build_landmarks.restype = i32
        L.shadowkv_build_landmarks.argtypes = [vp] * 9 + [sz, vp]
        L.shadowkv_decode_step.restype = i32
        L.shadowkv_decode_step.argtypes = [vp] * 15 + [sz, vp, vp]
        L.shadowkv_decode_step_static.restype = i32
        L.shadowkv_decode_step_static.argtypes = [vp] * 15
        L.shadowkv_static_scratch_bytes.restype = sz
        L.shadowkv_static_scratch_bytes.argtypes = []
        L.shadowkv_decode_step_cached.restype = i32
        L.shadowkv_decode_step_cached.argtypes = [vp] * 12 + [i32] + [vp] * 7 + [sz, vp, vp]
        L.shadowkv_value_cache_bytes.restype = sz
        L.shadowkv_value_cache_bytes.argtypes = [vp, i32]
        L.shadowkv_value_cache_reset.restype = i32
        L.shadowkv_value_cache_reset.argtypes = [vp, i32, vp, vp, vp]
        L.shadowkv_argtopk.restype = i32
        L.shadowkv_argtopk.argtypes = [vp, i32, i32, i32, C.c_double, vp, vp, sz, vp]
        L.shadowkv_argtopk_workspace_bytes.restype = sz
        L.shadowkv_argtopk_workspace_bytes.argtypes = [i32, i32, i32]
        L.shadowkv_append_chunk.restype = i32
        L.shadowkv_append_chunk.argtypes = [vp] * 10
        L.shadowkv_factorize_keys.restype = i32
        L.shadowkv_factorize_keys.argtypes = [vp] * 6 + [i32, vp, sz, vp]
        L.shadowkv_factorize_workspace_bytes.restype = sz
        L.shadowkv_factorize_workspace_bytes.argtypes = [vp]
        L.shadowkv_build_workspace_bytes.restype = sz
        L.shadowkv_build_workspace_bytes.argtypes = [vp]
        L.shadowkv_decode_workspace_bytes.restype = sz
        L.shadowkv_decode_workspace_bytes.argtypes = [vp]
        L.shadowkv_validate_params.restype = i32
        L.shadowkv_validate_params.argtypes = [vp, i32]
        L.shadowkv_decode_workspace_view.restype = vp
        L.shadowkv_decode_workspace_view.argtypes = [vp, vp, i32]
        L.shadowkv_status_string.restype = C.c_char_p
        L.shadowkv_status_string.argtypes = [i32]
        L.shadowkv_last_error.restype = C.c_char_p
        L.shadowkv_version.restype = i32
        L.shadowkv_shutdown.restype = None
        L.shadowkv_profile_begin.restype = i32
        L.shadowkv_profile_begin.argtypes = [i32]
        L.shadowkv_profile_end.restype = i32
        L.shadowkv_profile_end.argtypes = [vp, vp]
        _lib = L
    return _lib


def status_string(status: int) -> str:
    return lib().shadowkv_status_string(status).decode()


def last_error() -> str:
    return lib().shadowkv_last_error().decode()


def version() -> int:
    return int(lib().shadowkv_version())


def profile_begin(max_steps: int) -> None:
    _check(lib().shadowkv_profile_begin(int(max_steps)))


def decode_plan(p: "Params") -> dict:
    """shadowkv_decode_plan: how a plain decode step of this shape is laid out on the GPU."""
    st = p.c_struct()
    plan = (C.c_int32 * 8)()
    _check(lib().shadowkv_decode_plan(C.byref(st), plan))
    return {"splits": plan[0], "rows_per_split": plan[1], "resident_rows_in_selection_launch": bool(plan[2]),
            "key_and_value_waves": bool(plan[3]), "selection_threads": plan[4], "selection_candidates_per_thread": plan[5],
            "selection_launches": plan[6], "logit_row_floats": plan[7]}


def profile_end() -> dict:
    """Stops stage timing; returns {"steps": n, "ms": {stage: mean milliseconds per step}}."""
    ms = (C.c_double * 4)()
    n = C.c_int(0)
    _check(lib().shadowkv_profile_end(ms, C.byref(n)))
    steps = max(n.value, 1)
    return {"steps": n.value, "ms": {name: ms[i] / steps for i, name in enumerate(STAGES)}}


def _check(status: int) -> None:
    if status != OK:
        raise ShadowKVError(status, last_error())


@dataclass
class Params:
    batch: int
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    ctx_len: int
    chunk_size: int = 8
    rank: int = 160
    n_outlier_chunks: int = 48
    topk_chunks: int = 256
    local_len: int = 32
    value_location: int = VALUES_DEVICE
    flags: int = 0
    rope_theta: float = 5e5
    softmax_scale: float = 0.0
    inv_freq: Optional[torch.Tensor] = None   # device float32 [head_dim/2]
    ctx_capacity: int = 0                     # tokens the context arrays are laid out for (0 => ctx_len)
    kv_dtype: int = KV_BF16                   # KV_BF16 | KV_FP8_E5M2: storage of every KV-cache tensor

    @property
    def kv_torch_dtype(self) -> torch.dtype:
        return torch.float8_e5m2 if self.kv_dtype == KV_FP8_E5M2 else torch.bfloat16

    @property
    def kv_bytes(self) -> int:
        return 1 if self.kv_dtype == KV_FP8_E5M2 else 2

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

    def c_struct(self) -> CParams:
        inv = None
        if self.inv_freq is not None:
            assert self.inv_freq.dtype == torch.float32 and self.inv_freq.is_contiguous()
            inv = self.inv_freq.data_ptr()
        return CParams(self.batch, self.n_q_heads, self.n_kv_heads, self.head_dim, self.ctx_len, self.chunk_size,
                       self.rank, self.n_outlier_chunks, self.topk_chunks, self.local_len, self.value_location,
                       self.flags, float(self.rope_theta), float(self.softmax_scale), inv, int(self.ctx_capacity),
                       int(self.kv_dtype))

    @classmethod
    def from_workload(cls, wl, **kw) -> "Params":
        loc = VALUES_HOST if wl.value_location == "host" else VALUES_DEVICE
        base = dict(batch=wl.batch, n_q_heads=wl.n_q_heads, n_kv_heads=wl.n_kv_heads, head_dim=wl.head_dim,
                    ctx_len=wl.ctx_len, chunk_size=wl.chunk_size, rank=wl.rank,
                    n_outlier_chunks=wl.n_outlier_chunks, topk_chunks=wl.topk_chunks, local_len=wl.local_len,
                    value_location=loc, rope_theta=wl.rope_theta)
        base.update(kw)
        return cls(**base)


def validate_params(p: Params, for_decode: bool = True) -> int:
    st = p.c_struct()
    return int(lib().shadowkv_validate_params(C.addressof(st), 1 if for_decode else 0))


def decode_workspace_bytes(p: Params) -> int:
    st = p.c_struct()
    return int(lib().shadowkv_decode_workspace_bytes(C.addressof(st)))


def build_workspace_bytes(p: Params) -> int:
    st = p.c_struct()
    return int(lib().shadowkv_build_workspace_bytes(C.addressof(st)))


def _ptr(t: Optional[torch.Tensor]):
    if t is None:
        return None
    assert t.is_contiguous(), "tensors must be contiguous"
    return t.data_ptr()


def _stream_ptr(stream) -> int:
    if stream is None:
        return torch.cuda.current_stream().cuda_stream
    if isinstance(stream, int):
        return stream
    return stream.cuda_stream


def alloc_workspace(nbytes: int, device="cuda") -> torch.Tensor:
    return torch.empty(max(nbytes, 256), dtype=torch.uint8, device=device)


def build_landmarks(p: Params, k_rope: torch.Tensor, v: Optional[torch.Tensor] = None,
                    workspace: Optional[torch.Tensor] = None, stream=None) -> dict:
    """Pre-filling algorithm after its SVD line.  Returns the new device tensors."""
    b, h, s, d, c, o = p.batch, p.n_kv_heads, p.ctx_len, p.head_dim, p.chunk_size, p.n_outlier_chunks
    n_c = p.landmark_capacity      # rows allocated; the first p.n_landmarks are written
    dev = k_rope.device
    assert k_rope.dtype == p.kv_torch_dtype and tuple(k_rope.shape) == (b, h, s, d)
    if v is not None:
        assert v.dtype == p.kv_torch_dtype and tuple(v.shape) == (b, h, p.capacity, d)
    bf, i32 = p.kv_torch_dtype, torch.int32
    out = {
        "landmarks": torch.empty(b, h, max(n_c, 0), d, dtype=bf, device=dev),
        "landmark_chunk_ids": torch.empty(b, h, max(n_c, 0), dtype=i32, device=dev),
        "outlier_chunk_ids": torch.empty(b, h, o, dtype=i32, device=dev),
        "k_outlier": torch.empty(b, h, o * c, d, dtype=bf, device=dev),
        "v_outlier": torch.empty(b, h, o * c, d, dtype=bf, device=dev) if v is not None else None,
    }
    st = p.c_struct()
    if workspace is None:
        workspace = alloc_workspace(int(lib().shadowkv_build_workspace_bytes(C.addressof(st))), dev)
    rc = lib().shadowkv_build_landmarks(C.addressof(st), _ptr(k_rope), _ptr(v), _ptr(out["landmarks"]),
                                        _ptr(out["landmark_chunk_ids"]), _ptr(out["outlier_chunk_ids"]),
                                        _ptr(out["k_outlier"]), _ptr(out["v_outlier"]), _ptr(workspace),
                                        workspace.numel(), _stream_ptr(stream))
    _check(rc)
    out["workspace"] = workspace
    return out


def decode_step(p: Params, q, A, B, landmarks, landmark_chunk_ids, k_outlier, v_outlier, k_local, v_local,
                value_store, pos_offset=None, out=None, out_chunk_ids=None, workspace=None, stream=None,
                side_stream=None):
    """One decode step.  Returns ``(out [b,h_q,d] bf16, chunk_ids [b,h_kv,k] int32, workspace)``."""
    dev = q.device
    if out is None:
        out = torch.empty(p.batch, p.n_q_heads, p.head_dim, dtype=torch.bfloat16, device=dev)
    if out_chunk_ids is None:
        out_chunk_ids = torch.empty(p.batch, p.n_kv_heads, p.topk_chunks, dtype=torch.int32, device=dev)
    st = p.c_struct()
    if workspace is None:
        workspace = alloc_workspace(int(lib().shadowkv_decode_workspace_bytes(C.addressof(st))), dev)
    rc = lib().shadowkv_decode_step(C.addressof(st), _ptr(q), _ptr(A), _ptr(B), _ptr(landmarks),
                                    _ptr(landmark_chunk_ids), _ptr(k_outlier), _ptr(v_outlier), _ptr(k_local),
                                    _ptr(v_local), _ptr(value_store), _ptr(pos_offset), _ptr(out),
                                    _ptr(out_chunk_ids), _ptr(workspace), workspace.numel(), _stream_ptr(stream),
                                    None if side_stream is None else _stream_ptr(side_stream))
    _check(rc)
    return out, out_chunk_ids, workspace


def static_scratch_bytes() -> int:
    return int(lib().shadowkv_static_scratch_bytes())


def decode_step_static(p: Params, q, A, B, landmarks, landmark_chunk_ids, k_outlier, v_outlier, k_local, v_local,
                       value_store, pos_offset, out, out_chunk_ids, stream=None) -> None:
    """``decode_step`` on the library's static scratch: nothing is allocated, ``out`` and ``out_chunk_ids`` are
    the caller's."""
    st = p.c_struct()
    _check(lib().shadowkv_decode_step_static(C.addressof(st), _ptr(q), _ptr(A), _ptr(B), _ptr(landmarks),
                                             _ptr(landmark_chunk_ids), _ptr(k_outlier), _ptr(v_outlier),
                                             _ptr(k_local), _ptr(v_local), _ptr(value_store), _ptr(pos_offset),
                                             _ptr(out), _ptr(out_chunk_ids), _stream_ptr(stream)))


def append_chunk(p: Params, k_pre, k_rope, v, B, A, landmarks, landmark_chunk_ids, value_store, stream=None) -> None:
    """Append one chunk of generated tokens to the context in place (``p.ctx_len`` is the length before)."""
    st = p.c_struct()
    _check(lib().shadowkv_append_chunk(C.addressof(st), _ptr(k_pre), _ptr(k_rope), _ptr(v), _ptr(B), _ptr(A),
                                       _ptr(landmarks), _ptr(landmark_chunk_ids), _ptr(value_store),
                                       _stream_ptr(stream)))


def factorize_keys(p: Params, k_pre: torch.Tensor, n_iter: int = 0, want_vectors: bool = False, workspace=None,
                   stream=None) -> dict:
    """First line of the pre-filling algorithm: rank-r factors of the pre-RoPE keys ``k_pre [b, s, h_kv*d]``.
    Returns ``A [b, cap, r]`` and ``B [b, h_kv, r, d]`` in the storage type of the KV cache, and with
    ``want_vectors`` also ``psi [b, r, h_kv*d]`` and ``sigma [b, r]`` (fp64)."""
    b, h, d, r = p.batch, p.n_kv_heads, p.head_dim, p.rank
    dev = k_pre.device
    assert k_pre.dtype == p.kv_torch_dtype and tuple(k_pre.shape) == (b, p.ctx_len, h * d)
    out = {"A": torch.empty(b, p.capacity, r, dtype=p.kv_torch_dtype, device=dev),
           "B": torch.empty(b, h, r, d, dtype=p.kv_torch_dtype, device=dev),
           "psi": torch.empty(b, r, h * d, dtype=torch.float64, device=dev) if want_vectors else None,
           "sigma": torch.empty(b, r, dtype=torch.float64, device=dev) if want_vectors else None}
    st = p.c_struct()
    if workspace is None:
        need = int(lib().shadowkv_factorize_workspace_bytes(C.addressof(st)))
        if need == 0:
            _check(lib().shadowkv_validate_params(C.addressof(st), 0))
            raise ValueError("rank must be a multiple of 8 in [8, 256] and at most h_kv * d")
        workspace = alloc_workspace(need, dev)
    _check(lib().shadowkv_factorize_keys(C.addressof(st), _ptr(k_pre), _ptr(out["A"]), _ptr(out["B"]), _ptr(out["psi"]),
                                         _ptr(out["sigma"]), int(n_iter), _ptr(workspace), workspace.numel(),
                                         _stream_ptr(stream)))
    out["workspace"] = workspace
    return out


def argtopk(scores: torch.Tensor, k: int, largest: bool = True, stream=None) -> torch.Tensor:
    """Indices of the k largest (or smallest) of each row of ``scores [units, n]`` (fp64, device), ties to the
    lower index, in ascending index order: ``[units, k]`` int32."""
    assert scores.dtype == torch.float64 and scores.dim() == 2
    units, n = scores.shape
    need = int(lib().shadowkv_argtopk_workspace_bytes(units, n, k))
    ws = alloc_workspace(max(need, 256), scores.device)
    out = torch.empty(units, k, dtype=torch.int32, device=scores.device)
    _check(lib().shadowkv_argtopk(_ptr(scores), units, n, k, 1.0 if largest else -1.0, _ptr(out), _ptr(ws), ws.numel(),
                                  _stream_ptr(stream)))
    return out


class ValueCache:
    """Device buffers of the chunk cache of the value store with ``slots`` >= k slots per (batch, KV head):
    ``values [b,h_kv,slots*c,d]`` in the storage type of the KV cache, ``chunk_ids [b,h_kv,slots]`` int32 (-1 = empty), ``stamps
    [b,h_kv,slots+1]`` int32 (last use per slot, then the unit's clock), ``miss_count [b,h_kv]`` of the last step."""

    def __init__(self, p: Params, slots: Optional[int] = None, device="cuda", stream=None):
        self.slots = int(slots) if slots is not None else p.topk_chunks
        st = p.c_struct()
        n = int(lib().shadowkv_value_cache_bytes(C.addressof(st), self.slots))
        if n == 0:
            _check(lib().shadowkv_validate_params(C.addressof(st), 1))
            raise ValueError(f"cache slots {self.slots} outside [topk_chunks, 8192]")
        self.values = torch.empty(p.batch, p.n_kv_heads, self.slots * p.chunk_size, p.head_dim,
                                  dtype=p.kv_torch_dtype, device=device)
        assert self.values.numel() * p.kv_bytes == n
        self.chunk_ids = torch.empty(p.batch, p.n_kv_heads, self.slots, dtype=torch.int32, device=device)
        self.stamps = torch.empty(p.batch, p.n_kv_heads, self.slots + 1, dtype=torch.int32, device=device)
        self.miss_count = torch.zeros(p.batch, p.n_kv_heads, dtype=torch.int32, device=device)
        self.reset(p, stream)

    def reset(self, p: Params, stream=None):
        st = p.c_struct()
        _check(lib().shadowkv_value_cache_reset(C.addressof(st), self.slots, _ptr(self.chunk_ids), _ptr(self.stamps),
                                                _stream_ptr(stream)))


def decode_step_cached(p: Params, q, A, B, landmarks, landmark_chunk_ids, k_outlier, v_outlier, k_local, v_local,
                       value_store, cache: ValueCache, pos_offset=None, out=None, out_chunk_ids=None, workspace=None,
                       stream=None, side_stream=None):
    """One decode step that fetches only the chunks missing from ``cache``.  Returns like ``decode_step``."""
    dev = q.device
    if out is None:
        out = torch.empty(p.batch, p.n_q_heads, p.head_dim, dtype=torch.bfloat16, device=dev)
    if out_chunk_ids is None:
        out_chunk_ids = torch.empty(p.batch, p.n_kv_heads, p.topk_chunks, dtype=torch.int32, device=dev)
    st = p.c_struct()
    if workspace is None:
        workspace = alloc_workspace(int(lib().shadowkv_decode_workspace_bytes(C.addressof(st))), dev)
    rc = lib().shadowkv_decode_step_cached(C.addressof(st), _ptr(q), _ptr(A), _ptr(B), _ptr(landmarks),
                                           _ptr(landmark_chunk_ids), _ptr(k_outlier), _ptr(v_outlier), _ptr(k_local),
                                           _ptr(v_local), _ptr(value_store), _ptr(pos_offset), cache.slots,
                                           _ptr(cache.values), _ptr(cache.chunk_ids), _ptr(cache.stamps),
                                           _ptr(cache.miss_count), _ptr(out),
                                           _ptr(out_chunk_ids), _ptr(workspace), workspace.numel(),
                                           _stream_ptr(stream),
                                           None if side_stream is None else _stream_ptr(side_stream))
    _check(rc)
    return out, out_chunk_ids, workspace


def workspace_view(p: Params, workspace: torch.Tensor, which: str) -> Optional[torch.Tensor]:
    """Intermediate of the last decode step as a tensor aliasing ``workspace``.

    ``"k_sparse"`` fp32 [b,h_kv,k*c,d]; ``"v_sparse"`` in the KV storage type (staged runs only); ``"logits"`` fp32 [b,h_q,n_c] (the copies the search runs on).
    """
    code = {"k_sparse": 0, "v_sparse": 1, "sel_ids": 2, "logits": 3, "miss_slots": 4, "sel_slots": 5}[which]
    st = p.c_struct()
    ptr = lib().shadowkv_decode_workspace_view(C.addressof(st), workspace.data_ptr(), code)
    if not ptr:
        return None
    off = ptr - workspace.data_ptr()
    rows = (p.batch, p.n_kv_heads, p.topk_chunks * p.chunk_size, p.head_dim)
    if which == "k_sparse":
        n = rows[0] * rows[1] * rows[2] * rows[3]
        return workspace[off:off + 4 * n].view(torch.float32).view(rows)
    if which == "v_sparse":
        n = rows[0] * rows[1] * rows[2] * rows[3]
        return workspace[off:off + p.kv_bytes * n].view(p.kv_torch_dtype).view(rows)
    if which in ("sel_ids", "miss_slots", "sel_slots"):
        n = p.batch * p.n_kv_heads * p.topk_chunks
        return workspace[off:off + 4 * n].view(torch.int32).view(p.batch, p.n_kv_heads, p.topk_chunks)
    ld = (p.n_landmarks + 3) // 4 * 4
    n = p.batch * p.n_q_heads * ld
    return workspace[off:off + 4 * n].view(torch.float32).view(p.batch, p.n_q_heads, ld)[:, :, :p.n_landmarks]

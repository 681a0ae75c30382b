"""Seeded synthetic inputs shaped like the paper's decode workloads.

This module only *draws inputs*; it implements no step of the method.  Both
the CPU oracle and the HIP library are fed the tensors made here, bit for bit,
and neither of them calls anything in this file.

What it makes (all from one ``torch.Generator`` seeded per workload, fixed draw
order):

* pre-RoPE keys ``K_pre [b, s, h_kv*d]`` with a decaying spectrum: a
  token-correlated latent ``U`` (first-order autoregression along tokens,
  correlation ``rho``), singular values ``exp(-i/40)``, a random mixing matrix
  and N(0, 0.02) noise, scaled so that attention logits are peaked rather than
  flat;
* the rank-``r`` factors ``A [b, s, r]``, ``B [b, h_kv, r, d]`` of ``K_pre``
  (top eigenvectors of its Gram matrix through ``torch.linalg.eigh``) -- the
  first line of the paper's pre-filling algorithm, which is an *input* of the
  decode path;
* post-RoPE keys ``k_rope [b, h_kv, s, d]`` (``K_pre`` rotated at positions
  0..s-1; also an input of the pre-filling algorithm), optional planted outlier
  or needle chunks;
* values, recent-token keys/values, and a pool of queries.
"""
from __future__ import annotations

import math
from dataclasses import dataclass, replace
from typing import Dict, Optional

import torch


@dataclass(frozen=True)
class Workload:
    name: str
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
    rope_theta: float = 5e5
    seed: int = 0
    value_location: str = "hbm"      # "hbm" | "host" (pinned, device-readable)
    plant: str = "none"              # "none" | "outliers" | "needles"
    rho: float = 0.9                 # adjacent-token correlation of the latent
    n_queries: int = 16              # size of the query pool
    needle_gain: float = 8.0

    @property
    def group(self) -> int:
        return self.n_q_heads // self.n_kv_heads

    @property
    def key_width(self) -> int:
        return self.n_kv_heads * self.head_dim

    @property
    def n_chunks(self) -> int:
        return self.ctx_len // self.chunk_size

    @property
    def n_landmarks(self) -> int:
        return self.n_chunks - self.n_outlier_chunks

    @property
    def units(self) -> int:
        return self.batch * self.n_kv_heads

    def scaled(self, **kw) -> "Workload":
        return replace(self, **kw)


# The five benchmark configurations (names c1..c5) and the HBM twin of c3.
CONFIGS: Dict[str, Workload] = {
    "c1": Workload("c1", 1, 32, 8, 128, 4096, topk_chunks=64, n_outlier_chunks=8, seed=0),
    "c2": Workload("c2", 8, 32, 8, 128, 32768, seed=1, value_location="host"),
    "c3-host": Workload("c3-host", 16, 32, 8, 128, 131072, seed=2, value_location="host", plant="outliers"),
    "c3-hbm": Workload("c3-hbm", 16, 32, 8, 128, 131072, seed=2, value_location="hbm", plant="outliers"),
    "c4": Workload("c4", 1, 32, 2, 128, 1048576, seed=3, value_location="host", plant="needles"),
    "c5": Workload("c5", 8, 32, 32, 96, 131072, rope_theta=1e4, seed=4, value_location="hbm"),
}

# Further shapes bench.py accepts by name; not part of the benchmark's five.
EXTRA_CONFIGS: Dict[str, Workload] = {
    # c3-hbm with eight query heads per KV head (the grouping of 70B-class models)
    # 28 query / 4 KV heads (seven per group: the last four-head block of a group is partly empty)
    "c3-g7": Workload("c3-g7", 16, 28, 4, 128, 131072, rank=160, seed=2, value_location="hbm", plant="outliers"),
    "c3-g8": Workload("c3-g8", 16, 64, 8, 128, 131072, seed=2, value_location="hbm", plant="outliers"),
}

_LATENT = 320          # latent width; singular values beyond are far below the noise floor
_NOISE = 0.02
_TARGET_STD = 3.0      # per-element std of K_pre: makes q.k/sqrt(d) have std ~3 (peaked softmax)
_AR_TAPS = 128


def _rotate(x: torch.Tensor, pos: torch.Tensor, theta: float, inverse: bool = False) -> torch.Tensor:
    """Rotate pairs (i, i+d/2) of the last axis of ``x [..., n, d]`` by ``pos[n] * theta^(-2i/d)``.

    Input synthesis only: it turns drawn pre-RoPE keys into the post-RoPE keys
    a model would hand to the pre-filling algorithm.
    """
    d = x.shape[-1]
    half = d // 2
    inv = theta ** (-torch.arange(half, dtype=torch.float64, device=x.device) * 2.0 / d)
    ang = pos.to(torch.float64)[:, None] * inv[None, :]
    cs, sn = torch.cos(ang).to(torch.float32), torch.sin(ang).to(torch.float32)
    if inverse:
        sn = -sn
    x0, x1 = x[..., :half].float(), x[..., half:].float()
    return torch.cat([x0 * cs - x1 * sn, x1 * cs + x0 * sn], dim=-1)


def _latent(n: int, width: int, rho: float, gen: torch.Generator, device) -> torch.Tensor:
    """[n, width] stationary AR(1) along tokens (unit variance), as a truncated moving average."""
    eps = torch.randn(width, n + _AR_TAPS - 1, generator=gen, device=device, dtype=torch.float32)
    if rho == 0.0:
        return eps[:, _AR_TAPS - 1:].t().contiguous()
    taps = math.sqrt(1.0 - rho * rho) * rho ** torch.arange(_AR_TAPS - 1, -1, -1, dtype=torch.float32, device=device)
    u = torch.nn.functional.conv1d(eps[:, None, :], taps[None, None, :])[:, 0, :]
    return u.t().contiguous()


def _alloc(shape, dtype, device, pinned: bool) -> torch.Tensor:
    if pinned:
        return torch.empty(shape, dtype=dtype, device="cpu", pin_memory=torch.cuda.is_available())
    return torch.empty(shape, dtype=dtype, device=device)


def generate(wl: Workload, device: Optional[str] = None, want_prefill: bool = True,
             value_device: Optional[str] = None, want_k_pre: bool = False) -> Dict[str, torch.Tensor]:
    """Draw one workload.  Returns bf16 tensors (ids int32):

    ``q_pool [n_queries, b, h_q, d]``, ``A [b, s, r]``, ``B [b, h_kv, r, d]``,
    ``k_rope [b, h_kv, s, d]`` (only if ``want_prefill``), ``v [b, h_kv, s, d]``
    (on ``value_device``; pinned host memory when the workload says "host"),
    ``k_local, v_local [b, h_kv, w, d]``, ``pos_offset [b]`` (zeros),
    ``needle_chunks [b, h_kv, 4]`` for the needle workload, ``planted_chunks
    [b, h_kv, n_ch/100]`` for the planted-outlier workload.
    """
    if device is None:
        device = "cuda" if torch.cuda.is_available() else "cpu"
    dev = torch.device(device)
    gen = torch.Generator(device=dev)
    gen.manual_seed(1000 + wl.seed)
    b, hkv, hq, d, s, c, r, w = (wl.batch, wl.n_kv_heads, wl.n_q_heads, wl.head_dim, wl.ctx_len,
                                 wl.chunk_size, wl.rank, wl.local_len)
    D = wl.key_width
    R = min(_LATENT, D)
    bf = torch.bfloat16
    sigma = torch.exp(-torch.arange(R, dtype=torch.float32, device=dev) / 40.0)
    gain = _TARGET_STD * math.sqrt(D / float((sigma * sigma).sum()))

    host_values = wl.value_location == "host"
    if value_device is None:
        value_device = "cpu" if host_values else device
    out: Dict[str, torch.Tensor] = {
        "A": torch.empty(b, s, r, dtype=bf, device=dev),
        "B": torch.empty(b, hkv, r, d, dtype=bf, device=dev),
        "k_local": torch.empty(b, hkv, w, d, dtype=bf, device=dev),
        "v": _alloc((b, hkv, s, d), bf, value_device, pinned=(value_device == "cpu" and host_values)),
        "pos_offset": torch.zeros(b, dtype=torch.int32, device=dev),
    }
    if want_prefill:
        out["k_rope"] = torch.empty(b, hkv, s, d, dtype=bf, device=dev)
    if want_k_pre:
        out["k_pre"] = torch.empty(b, s, D, dtype=bf, device=dev)
    needle_dirs = None
    n_plant = max(1, (s // c) // 100)
    if wl.plant == "outliers" and want_prefill:
        out["planted_chunks"] = torch.empty(b, hkv, n_plant, dtype=torch.int32, device=dev)
    if wl.plant == "needles":
        out["needle_chunks"] = torch.empty(b, hkv, 4, dtype=torch.int32, device=dev)
        needle_dirs = torch.empty(b, hkv, 4, d, dtype=torch.float32, device=dev)

    pos_all = torch.arange(s + w, device=dev)
    for bi in range(b):
        # 1. low-rank pre-RoPE keys for the s context tokens and the w recent ones
        W = torch.randn(D, R, generator=gen, device=dev, dtype=torch.float32) / math.sqrt(D)
        U = _latent(s + w, R, wl.rho, gen, dev) * gain
        k_pre = (U * sigma[None, :]) @ W.t()
        del U
        k_pre += _NOISE * torch.randn(s + w, D, generator=gen, device=dev, dtype=torch.float32)
        kp_heads = k_pre.view(s + w, hkv, d).permute(1, 0, 2)          # [h_kv, s+w, d] view
        if wl.plant == "needles":
            # four chunks per KV head whose eight rows all equal one direction after rotation
            med = kp_heads[:, :s].norm(dim=-1).median(dim=-1).values    # [h_kv]
            ids = torch.stack([torch.randperm(s // c, generator=gen, device=dev)[:4] for _ in range(hkv)])
            dirs = torch.randn(hkv, 4, d, generator=gen, device=dev, dtype=torch.float32)
            dirs = dirs / dirs.norm(dim=-1, keepdim=True) * (3.0 * med)[:, None, None]
            for h in range(hkv):
                for j in range(4):
                    tok = ids[h, j] * c + torch.arange(c, device=dev)
                    rows = dirs[h, j].expand(c, d)
                    kp_heads[h, tok] = _rotate(rows, tok, wl.rope_theta, inverse=True)
            out["needle_chunks"][bi] = ids.to(torch.int32)
            needle_dirs[bi] = dirs
        # 2. rank-r factors of the context keys (pre-filling algorithm, SVD line)
        ctx = k_pre[:s]
        if want_k_pre:
            out["k_pre"][bi] = ctx.to(bf)
        gram = (ctx.t() @ ctx).to(torch.float64)
        evals, evecs = torch.linalg.eigh(gram)
        psi = evecs[:, -r:].flip(-1).to(torch.float32)                  # [D, r], strongest first
        out["A"][bi] = (ctx @ psi).to(bf)
        out["B"][bi] = psi.t().reshape(r, hkv, d).permute(1, 0, 2).to(bf)
        del gram, evals, evecs, psi
        # 3. post-RoPE keys at positions 0..s+w-1
        rot = _rotate(kp_heads, pos_all, wl.rope_theta)                 # [h_kv, s+w, d] fp32
        out["k_local"][bi] = rot[:, s:].to(bf)
        if want_prefill:
            kr = rot[:, :s]
            if wl.plant == "outliers":
                med = kr.norm(dim=-1).median(dim=-1).values
                for h in range(hkv):
                    ch = torch.randperm(s // c, generator=gen, device=dev)[:n_plant]
                    tok = (ch[:, None] * c + torch.arange(c, device=dev)[None, :]).reshape(-1)
                    # rows alternate between +u and -u (10x the median norm) plus a little noise: the
                    # chunk mean nearly cancels, so the minimum cosine is far below any natural chunk's
                    u = torch.randn(n_plant, 1, d, generator=gen, device=dev, dtype=torch.float32)
                    u = u / u.norm(dim=-1, keepdim=True) * (10.0 * med[h])
                    sign = 1.0 - 2.0 * (torch.arange(c, device=dev) % 2).to(torch.float32)
                    g = (u * sign[None, :, None]).reshape(-1, d)
                    g = g + 0.05 * med[h] / math.sqrt(d) * torch.randn(tok.numel(), d, generator=gen, device=dev)
                    kr[h, tok] = g
                    out["planted_chunks"][bi, h] = ch.to(torch.int32)
            out["k_rope"][bi] = kr.to(bf)
        del rot, k_pre
        # 4. values
        vb = torch.randn(hkv, s, d, generator=gen, device=dev, dtype=torch.float32).to(bf)
        out["v"][bi].copy_(vb)
        del vb
    out["v_local"] = torch.randn(b, hkv, w, d, generator=gen, device=dev, dtype=torch.float32).to(bf)
    # 5. queries
    qp = torch.randn(wl.n_queries, b, hq, d, generator=gen, device=dev, dtype=torch.float32)
    if needle_dirs is not None:
        pull = (needle_dirs / needle_dirs.norm(dim=-1, keepdim=True)).sum(dim=2)   # [b, h_kv, d]
        qp = qp + wl.needle_gain * pull.repeat_interleave(wl.group, dim=1)[None]
    out["q_pool"] = qp.to(bf)
    return out


KV_TENSORS = ("A", "B", "k_rope", "v", "k_local", "v_local")


def to_fp8_storage(t: Dict[str, torch.Tensor]) -> Dict[str, torch.Tensor]:
    """The same workload with its KV-cache tensors (``KV_TENSORS``) stored as FP8 E5M2 (torch's cast, round to
    nearest even): the second storage precision the paper evaluates (section "Precision Sensitivity").  Queries
    stay bf16.  Pinned host memory is kept pinned.  A cast of inputs, not a step of the method: oracle and
    library are handed these bytes."""
    out = dict(t)
    for name in KV_TENSORS:
        if name not in t:
            continue
        x = t[name]
        if x.device.type == "cpu" and x.is_pinned():
            y = _alloc(tuple(x.shape), torch.float8_e5m2, "cpu", pinned=True)
            step = max(1, (1 << 26) // max(1, x[0].numel()))
            for i in range(0, x.shape[0], step):
                y[i:i + step].copy_(x[i:i + step].to(torch.float8_e5m2))
        else:
            y = torch.empty(x.shape, dtype=torch.float8_e5m2, device=x.device)
            for i in range(x.shape[0]):          # per batch item: bounds the temporary of the cast
                y[i].copy_(x[i].to(torch.float8_e5m2))
        out[name] = y
    return out


def query_sequence(wl: Workload, n_steps: int, rho_q: float = 0.9, device: Optional[str] = None) -> torch.Tensor:
    """Queries of ``n_steps`` consecutive decode steps, ``[n_steps, b, h_q, d]`` bf16, correlated from step to
    step so that consecutive selections overlap (the temporal locality the chunk cache of the value store
    lives on).  A stationary AR(1) process ``q_t = rho_q q_{t-1} + sqrt(1 - rho_q^2) eps_t`` on a ring of
    ``n_steps`` steps (built by circular filtering of white noise, so replaying the sequence in a loop has no
    jump at the wrap), unit variance per element.  Own generator (seed ``2000 + wl.seed``): the other tensors
    of the workload are unchanged by drawing it."""
    dev = device or ("cuda" if torch.cuda.is_available() else "cpu")
    gen = torch.Generator(device=dev)
    gen.manual_seed(2000 + wl.seed)
    eps = torch.randn(n_steps, wl.batch, wl.n_q_heads, wl.head_dim, generator=gen, device=dev, dtype=torch.float32)
    f = torch.arange(n_steps, device=dev, dtype=torch.float32)
    z = torch.polar(torch.ones_like(f), -2.0 * math.pi * f / n_steps)
    hf = math.sqrt(1.0 - rho_q * rho_q) / (1.0 - rho_q * z)          # AR(1) transfer function on the ring
    q = torch.fft.ifft(torch.fft.fft(eps, dim=0) * hf[:, None, None, None], dim=0).real
    q = q / q.std()
    return q.to(torch.bfloat16).contiguous()


def with_capacity(t: Dict[str, torch.Tensor], wl: Workload, capacity: int) -> Dict[str, torch.Tensor]:
    """The tensors of ``generate`` whose token axis can grow (``A [b, cap, r]``, ``v [b, h_kv, cap, d]``) moved
    into arrays laid out for ``capacity`` tokens; the unused tail is filled with NaN so that any read of it shows.
    Pinned host memory is kept pinned."""
    s = wl.ctx_len
    assert capacity >= s and capacity % wl.chunk_size == 0
    out = dict(t)
    A = torch.full((wl.batch, capacity, wl.rank), float("nan"), dtype=torch.bfloat16, device=t["A"].device)
    A[:, :s] = t["A"]
    v_old = t["v"]
    v = _alloc((wl.batch, wl.n_kv_heads, capacity, wl.head_dim), torch.bfloat16, v_old.device,
               pinned=v_old.device.type == "cpu" and v_old.is_pinned())
    v.fill_(float("nan"))
    v[:, :, :s] = v_old
    out["A"], out["v"] = A, v
    return out


def generated_chunk(wl: Workload, t: Dict[str, torch.Tensor], index: int, device: Optional[str] = None):
    """Keys and values of the ``index``-th chunk of generated tokens (tokens ``s + index*c ...``), as a model
    would produce them: pre-RoPE keys in the low-rank subspace of the context keys (coefficients with the
    per-column scale of ``A``, times ``B``) plus N(0, 0.02^2) noise, the same keys rotated at their positions,
    and N(0,1) values.  Returns bf16 ``(k_pre [b, c, h_kv*d], k_rope [b, h_kv, c, d], v [b, h_kv, c, d])``.
    Own generator (seed ``3000 + wl.seed + 17*index``)."""
    dev = torch.device(device or ("cuda" if torch.cuda.is_available() else "cpu"))
    gen = torch.Generator(device=dev)
    gen.manual_seed(3000 + wl.seed + 17 * index)
    b, hkv, d, c, r, s = wl.batch, wl.n_kv_heads, wl.head_dim, wl.chunk_size, wl.rank, wl.ctx_len
    A = t["A"][:, :s].to(dev).float()
    Bm = t["B"].to(dev).float()                                        # [b, h, r, d]
    col_std = A.std(dim=1)                                             # [b, r]
    coef = torch.randn(b, c, r, generator=gen, device=dev) * col_std[:, None, :]
    k_pre = torch.einsum("bcr,bhrx->bchx", coef, Bm)
    k_pre = k_pre + 0.02 * torch.randn(b, c, hkv, d, generator=gen, device=dev)
    k_pre = k_pre.to(torch.bfloat16)
    pos = torch.arange(s + index * c, s + (index + 1) * c, device=dev)
    k_rope = _rotate(k_pre.float().permute(0, 2, 1, 3), pos, wl.rope_theta).to(torch.bfloat16).contiguous()
    v = torch.randn(b, hkv, c, d, generator=gen, device=dev).to(torch.bfloat16)
    return k_pre.reshape(b, c, hkv * d).contiguous(), k_rope, v

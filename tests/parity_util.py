"""Shared machinery of the GPU-vs-oracle parity tests.

One seeded workload is drawn once (on the GPU when there is one), the identical
bits go to the CPU oracle and to the HIP library, and the results are compared:

* chunk / outlier index sets: equal, except that an id present on one side only
  is accepted when its oracle score lies within 1e-6 of the oracle's boundary
  score -- the tie rule.  For the selected chunks the score is the log of the
  softmax entry, so an absolute 1e-6 there is 1e-6 relative on the softmax entry;
  for the outliers it is the minimum cosine, which lies in [-1, 1];
* landmarks, gathered outlier rows: bit-exact;
* decode output: max-abs <= 2e-2 and mean-abs <= 2e-3 against the oracle's bf16
  output (the stated acceptance bar), plus a tighter check of the rebuilt keys.
"""
from __future__ import annotations

import numpy as np
import torch

from oracle import shadowkv_oracle as O
from paper_2410_21465_amd import shadowkv as S
from workloads import Workload, generate

OUT_MAX_ABS = 2e-2
OUT_MEAN_ABS = 2e-3
TIE_TOL = 1e-6
# rebuilt keys: fp32 MFMA accumulation over r <= 256 exact bf16 products plus an fp32 rotation;
# error <= ~r * 2^-24 * sum|a||b| -- a few 1e-5 of the key scale.  Bound used: 2e-4 * max|K|.
KSPARSE_REL = 2e-4


def oracle_params(wl: Workload, inv_freq=None, softmax_scale=0.0, kv_dtype=0) -> O.OracleParams:
    return O.OracleParams(wl.batch, wl.n_q_heads, wl.n_kv_heads, wl.head_dim, wl.ctx_len, wl.chunk_size, wl.rank,
                          wl.n_outlier_chunks, wl.topk_chunks, wl.local_len, rope_theta=wl.rope_theta,
                          inv_freq=inv_freq, softmax_scale=softmax_scale, kv_dtype=kv_dtype)


def to_bits(t: torch.Tensor, kv_dtype: int = 0) -> np.ndarray:
    """Raw bits of a bf16 tensor (uint16), or of an E5M2 tensor of the KV cache with kv_dtype = 1 (uint8)."""
    return O.as_bits(t.detach().cpu(), kv_dtype)


def kv_from_bits(bits: np.ndarray, device="cuda") -> torch.Tensor:
    """Oracle-side raw bits (uint16 = bf16, uint8 = E5M2) as a device tensor of that type."""
    if bits.dtype == np.uint8:
        return torch.from_numpy(bits).view(torch.float8_e5m2).to(device)
    return torch.from_numpy(bits.view(np.int16)).view(torch.bfloat16).to(device)


def kv_to_f64(bits: np.ndarray) -> np.ndarray:
    return O.e5m2_bits_to_f64(bits) if bits.dtype == np.uint8 else O.bits_to_f64(bits)


def kv_round(x: np.ndarray, kv_dtype: int) -> np.ndarray:
    return O.f64_to_e5m2_bits(x) if kv_dtype == 1 else O.f64_to_bits(x)


def check_index_sets(got: np.ndarray, want_best_first: np.ndarray, score_of_id, what: str):
    """got/want: [units, k] ids.  score_of_id(u, ids) -> oracle scores (higher = better)."""
    units, k = want_best_first.shape
    n_tied = 0
    for u in range(units):
        g, w = set(int(x) for x in got[u]), set(int(x) for x in want_best_first[u])
        assert len(g) == k, f"{what}: unit {u} returned duplicate ids"
        if g == w:
            continue
        boundary = float(score_of_id(u, want_best_first[u][-1:])[0])
        tol = TIE_TOL
        odd = np.array(sorted(g ^ w))
        sc = score_of_id(u, odd)
        assert np.all(np.abs(sc - boundary) <= tol), (
            f"{what}: unit {u}: ids {odd.tolist()} differ with scores {sc.tolist()} vs boundary {boundary}")
        n_tied += len(odd)
    return n_tied


def run_build_parity(wl: Workload, t: dict, device="cuda", kv_dtype: int = 0):
    """shadowkv_build_landmarks against the oracle.  Returns (oracle result, gpu result)."""
    op = oracle_params(wl, kv_dtype=kv_dtype)
    k_bits, v_bits = to_bits(t["k_rope"], kv_dtype), to_bits(t["v"], kv_dtype)
    ref = O.build_landmarks(op, k_bits, v_bits, diagnostics=True)
    gp = S.Params.from_workload(wl, kv_dtype=kv_dtype)
    v_dev = t["v"]
    got = S.build_landmarks(gp, t["k_rope"], v_dev)
    torch.cuda.synchronize()
    b, h, o, c, d = wl.batch, wl.n_kv_heads, wl.n_outlier_chunks, wl.chunk_size, wl.head_dim
    units = b * h
    g_out = got["outlier_chunk_ids"].cpu().numpy().reshape(units, o)
    w_out = ref["outlier_chunk_ids"].reshape(units, o)
    mc = ref["chunk_min_cos"].reshape(units, -1)
    if o:
        assert np.all(np.diff(g_out, axis=1) > 0), "outlier ids must be ascending"
        ties = check_index_sets(g_out, w_out, lambda u, ids: -mc[u, ids], "outliers")
    else:
        ties = 0
    # gathered rows: bit-exact copies of the chunks the GPU chose
    if o:
        gk = to_bits(got["k_outlier"], kv_dtype).reshape(units, o, c, d)
        gv = to_bits(got["v_outlier"], kv_dtype).reshape(units, o, c, d)
        kk = k_bits.reshape(units, -1, c, d)
        vv = v_bits.reshape(units, -1, c, d)
        for u in range(units):
            np.testing.assert_array_equal(gk[u], kk[u, g_out[u]])
            np.testing.assert_array_equal(gv[u], vv[u, g_out[u]])
    if ties == 0:
        np.testing.assert_array_equal(got["landmark_chunk_ids"].cpu().numpy(), ref["landmark_chunk_ids"])
        np.testing.assert_array_equal(to_bits(got["landmarks"], kv_dtype), ref["landmarks"])
    else:  # compare the landmarks chunk by chunk through the ids
        gid = got["landmark_chunk_ids"].cpu().numpy().reshape(units, -1)
        gl = to_bits(got["landmarks"], kv_dtype).reshape(units, -1, d)
        means = ref["chunk_mean"].reshape(units, -1, d)
        for u in range(units):
            np.testing.assert_array_equal(gl[u], kv_round(means[u, gid[u]], kv_dtype))
    return ref, got


def run_decode_parity(wl: Workload, t: dict, ref_build: dict, qi: int = 0, side_stream: bool = False, flags: int = 0,
                      inv_freq=None, softmax_scale: float = 0.0, pos_offset=None, device="cuda",
                      check_keys: bool = True, kv_dtype: int = 0):
    """shadowkv_decode_step against the oracle, both fed the ORACLE's landmarks and outliers."""
    b, hq, h, d, c, k = wl.batch, wl.n_q_heads, wl.n_kv_heads, wl.head_dim, wl.chunk_size, wl.topk_chunks
    units = b * h
    op = oracle_params(wl, inv_freq=inv_freq, softmax_scale=softmax_scale, kv_dtype=kv_dtype)
    q = t["q_pool"][qi]
    pos = t["pos_offset"] if pos_offset is None else pos_offset
    kd = kv_dtype
    ref = O.decode_step(op, to_bits(q), to_bits(t["A"], kd), to_bits(t["B"], kd), ref_build["landmarks"],
                        ref_build["landmark_chunk_ids"], ref_build["k_outlier"], ref_build["v_outlier"],
                        to_bits(t["k_local"], kd), to_bits(t["v_local"], kd), to_bits(t["v"], kd), pos.cpu().numpy())

    def dev_bf16(bits):
        return kv_from_bits(bits, device)

    gp = S.Params.from_workload(wl, flags=flags | (S.FLAG_KEEP_REBUILT_KEYS if check_keys else 0),
                                softmax_scale=softmax_scale, kv_dtype=kv_dtype,
                                inv_freq=None if inv_freq is None else torch.from_numpy(inv_freq).to(device))
    lm = dev_bf16(ref_build["landmarks"])
    lm_ids = torch.from_numpy(ref_build["landmark_chunk_ids"]).to(device)
    ko, vo = dev_bf16(ref_build["k_outlier"]), dev_bf16(ref_build["v_outlier"])
    side = torch.cuda.Stream() if side_stream else None
    out, ids, ws = S.decode_step(gp, q, t["A"], t["B"], lm, lm_ids, ko, vo, t["k_local"], t["v_local"], t["v"],
                                 pos.to(device), side_stream=side)
    torch.cuda.synchronize()

    # --- selected chunk ids ---
    g_ids = ids.cpu().numpy().reshape(units, k)
    w_ids = ref["chunk_ids"].reshape(units, k)
    assert np.all(np.diff(g_ids, axis=1) > 0), "chunk ids must be ascending"
    lid = ref_build["landmark_chunk_ids"].reshape(units, -1)
    z2 = ref["z2"].reshape(units, -1)

    def score(u, chunk_ids):
        slots = np.searchsorted(lid[u], chunk_ids)
        assert np.all(lid[u][slots] == chunk_ids), "GPU selected a chunk that is not a landmark"
        return z2[u, slots]

    ties = check_index_sets(g_ids, w_ids, score, "top-k chunks")

    # --- rebuilt keys (fp32 workspace) against the oracle's, matched through the chunk ids ---
    ks_ref = ref["k_sparse"].reshape(units, k, c, d)
    kmax = np.abs(ks_ref).max()
    worst_k = 0.0
    ks = None
    if check_keys:
        ks = S.workspace_view(gp, ws, "k_sparse").cpu().numpy().reshape(units, k, c, d).astype(np.float64)
    for u in range(units if check_keys else 0):
        order = np.argsort(w_ids[u])
        common = np.isin(w_ids[u][order], g_ids[u])
        gsel = np.isin(g_ids[u], w_ids[u])
        worst_k = max(worst_k, float(np.abs(ks[u][gsel] - ks_ref[u][order][common]).max()))
    assert worst_k <= KSPARSE_REL * kmax, f"rebuilt keys off by {worst_k} (key scale {kmax})"

    # --- staged values: bit-exact copies ---
    vs = S.workspace_view(gp, ws, "v_sparse")
    if vs is not None:
        vbits = to_bits(t["v"], kd).reshape(units, -1, c, d)
        gv = to_bits(vs, kd).reshape(units, k, c, d)
        for u in range(units):
            np.testing.assert_array_equal(gv[u], vbits[u, g_ids[u]])

    # --- output ---
    got = out.float().cpu().numpy().astype(np.float64)
    want = O.bits_to_f64(ref["out"])
    err = np.abs(got - want)
    stats = {"max_abs": float(err.max()), "mean_abs": float(err.mean()), "ties": ties, "k_err": worst_k,
             "k_scale": float(kmax), "out_scale": float(np.abs(want).mean()),
             "max_abs_vs_f64": float(np.abs(got - ref["out_f64"]).max())}
    assert stats["max_abs"] <= OUT_MAX_ABS and stats["mean_abs"] <= OUT_MEAN_ABS, stats
    return stats, ref, (out, ids, ws)


def draw(wl: Workload, device="cuda"):
    return generate(wl, device=device)

"""Pins of the oracle's capacity layout and of oracle_append_chunk (generated tokens stored as low-rank
states K' Psi: last paragraph of section "High-throughput Decoding" and its footnote).  CPU only."""
import numpy as np
import pytest
import scipy.linalg
import torch

from oracle import shadowkv_oracle as O
from workloads import Workload, generate


def _bits(x: np.ndarray) -> np.ndarray:
    """fp64 values that are exactly representable in bf16 -> their bit patterns."""
    b = O.f64_to_bits(x)
    assert np.array_equal(O.bits_to_f64(b), x)
    return b


def _wl(**kw):
    base = dict(name="append", batch=2, n_q_heads=4, n_kv_heads=2, head_dim=64, ctx_len=512, chunk_size=4, rank=16,
                n_outlier_chunks=3, topk_chunks=20, local_len=3, rope_theta=1e4, seed=21)
    base.update(kw)
    return Workload(**base)


def _params(wl, ctx_len=None, cap=0):
    return O.OracleParams(wl.batch, wl.n_q_heads, wl.n_kv_heads, wl.head_dim, ctx_len or wl.ctx_len, wl.chunk_size,
                          wl.rank, wl.n_outlier_chunks, wl.topk_chunks, wl.local_len, rope_theta=wl.rope_theta,
                          ctx_capacity=cap)


def _pad(a: np.ndarray, axis: int, n: int, fill) -> np.ndarray:
    shape = list(a.shape)
    shape[axis] = n - a.shape[axis]
    return np.ascontiguousarray(np.concatenate([a, np.full(shape, fill, a.dtype)], axis=axis))


def test_layout_with_room_to_grow_changes_nothing():
    """The same context in arrays laid out for more tokens (garbage in the unused part) gives bit-identical
    landmarks, ids, outliers and decode outputs."""
    wl = _wl()
    t = generate(wl, device="cpu")
    s, c, o, cap = wl.ctx_len, wl.chunk_size, wl.n_outlier_chunks, wl.ctx_len + 5 * wl.chunk_size
    bits = {k: O.as_bits(t[k]) for k in ("k_rope", "v", "A", "B", "k_local", "v_local")}
    dense, roomy = _params(wl), _params(wl, cap=cap)
    b0 = O.build_landmarks(dense, bits["k_rope"], bits["v"])
    v_cap, a_cap = _pad(bits["v"], 2, cap, 0x7fc0), _pad(bits["A"], 1, cap, 0x7fc0)   # NaN filler
    b1 = O.build_landmarks(roomy, bits["k_rope"], v_cap)
    n_c = s // c - o
    assert np.array_equal(b1["landmarks"][:, :, :n_c], b0["landmarks"])
    assert np.array_equal(b1["landmark_chunk_ids"][:, :, :n_c], b0["landmark_chunk_ids"])
    for k in ("outlier_chunk_ids", "k_outlier", "v_outlier"):
        assert np.array_equal(b1[k], b0[k])
    lm = b1["landmarks"].copy(); lm[:, :, n_c:] = 0x7fc0
    q = O.as_bits(t["q_pool"][0])
    pos = t["pos_offset"].numpy()
    r0 = O.decode_step(dense, q, bits["A"], bits["B"], b0["landmarks"], b0["landmark_chunk_ids"], b0["k_outlier"],
                       b0["v_outlier"], bits["k_local"], bits["v_local"], bits["v"], pos)
    r1 = O.decode_step(roomy, q, a_cap, bits["B"], lm, b1["landmark_chunk_ids"], b1["k_outlier"], b1["v_outlier"],
                       bits["k_local"], bits["v_local"], v_cap, pos)
    for k in ("out", "out_f64", "chunk_ids", "z2", "k_sparse"):
        assert np.array_equal(r0[k], r1[k]), k


def test_projection_is_exact_for_keys_inside_the_subspace():
    """B = r rows of a Hadamard matrix over the full key width, scaled to unit length (entries +-2^-4, exact in
    bf16), so B B^T = I.  Keys K' = a B with small integer coefficients are exact in bf16, and K' Psi must give
    the coefficients back exactly -- wrong head order, a transposed B or a dropped head would not."""
    b, hkv, d, c, r = 2, 4, 64, 4, 8
    D = hkv * d
    H = scipy.linalg.hadamard(D).astype(np.float64) / 16.0
    rng = np.random.default_rng(0)
    rows = np.stack([rng.choice(D, r, replace=False) for _ in range(b)])
    Psi_T = np.stack([H[rows[i]] for i in range(b)])                     # [b, r, D]
    B = Psi_T.reshape(b, r, hkv, d).transpose(0, 2, 1, 3).copy()         # [b, h_kv, r, d]
    a = rng.integers(-3, 4, size=(b, c, r)).astype(np.float64)
    k_pre = np.einsum("bcr,brx->bcx", a, Psi_T)                          # [b, c, D], multiples of 1/16 up to 24/16
    p = O.OracleParams(b, hkv, hkv, d, 8 * c, c, r, 1, 2, 0, ctx_capacity=9 * c)
    cap, nc_cap = p.capacity, p.landmark_capacity
    A = np.zeros((b, cap, r), np.uint16)
    lm = np.zeros((b, hkv, nc_cap, d), np.uint16)
    ids = -np.ones((b, hkv, nc_cap), np.int32)
    store = np.zeros((b, hkv, cap, d), np.uint16)
    k_rope = rng.integers(-8, 9, size=(b, hkv, c, d)).astype(np.float64)
    v = rng.integers(-8, 9, size=(b, hkv, c, d)).astype(np.float64)
    O.append_chunk(p, _bits(k_pre), _bits(k_rope), _bits(v), _bits(B), A, lm, ids, store)
    s = p.ctx_len
    assert np.array_equal(O.bits_to_f64(A[:, s:s + c]), a)
    assert not A[:, :s].any()                                            # nothing else touched
    n_c = p.n_landmarks
    assert np.array_equal(O.bits_to_f64(lm[:, :, n_c]), k_rope.mean(axis=2))   # multiples of 1/4: exact
    assert np.all(ids[:, :, n_c] == s // c) and np.all(ids[:, :, :n_c] == -1)
    assert np.array_equal(O.bits_to_f64(store[:, :, s:s + c]), v) and not store[:, :, :s].any()


@pytest.mark.parametrize("seed", [21, 23])
def test_append_equals_a_longer_prefill(seed):
    """Pre-filling s + c tokens, or pre-filling s tokens and appending the last chunk, must describe the same
    context (when the last chunk is no outlier): same factors, landmarks, ids and store, hence the same decode
    step bit for bit."""
    wl_long = _wl(seed=seed, ctx_len=516)
    t = generate(wl_long, device="cpu")
    s1, c, o, hkv, d, r = wl_long.ctx_len, wl_long.chunk_size, wl_long.n_outlier_chunks, wl_long.n_kv_heads, wl_long.head_dim, wl_long.rank
    s0 = s1 - c
    bits = {k: O.as_bits(t[k]) for k in ("k_rope", "v", "A", "B", "k_local", "v_local")}
    full = _params(wl_long)
    bf = O.build_landmarks(full, bits["k_rope"], bits["v"])
    assert (s1 // c - 1) not in set(bf["outlier_chunk_ids"].ravel().tolist()), "pick another seed"
    # short context in arrays with room for one more chunk
    short = _params(wl_long, ctx_len=s0, cap=s1)
    v_store = bits["v"].copy(); v_store[:, :, s0:] = 0
    A = bits["A"].copy(); A[:, s0:] = 0
    bs = O.build_landmarks(short, np.ascontiguousarray(bits["k_rope"][:, :, :s0]), v_store)
    assert np.array_equal(np.sort(bs["outlier_chunk_ids"], -1), np.sort(bf["outlier_chunk_ids"], -1))
    # the generator made A = K_pre Psi with Psi^T = B; recover K_pre of the last chunk to bf16 precision is not
    # possible, so take pre-RoPE keys that ARE in the subspace of B: k_pre = bf16(A_last B), then the rows of A
    # the oracle computes are the projections of exactly these keys
    Bf = O.bits_to_f64(bits["B"])                                                    # [b, h, r, d]
    k_pre = np.einsum("bcr,bhrx->bchx", O.bits_to_f64(bits["A"][:, s0:]), Bf).reshape(wl_long.batch, c, hkv * d)
    k_pre_bits = O.f64_to_bits(k_pre)
    want_A = O.f64_to_bits(np.einsum("bchx,bhrx->bcr", O.bits_to_f64(k_pre_bits).reshape(wl_long.batch, c, hkv, d), Bf))
    lm, ids = bs["landmarks"], bs["landmark_chunk_ids"]
    O.append_chunk(short, k_pre_bits, np.ascontiguousarray(bits["k_rope"][:, :, s0:]),
                   np.ascontiguousarray(bits["v"][:, :, s0:]), bits["B"], A, lm, ids, v_store)
    assert np.array_equal(A[:, s0:], want_A)                      # independent einsum of the same projection
    assert np.array_equal(lm, bf["landmarks"]) and np.array_equal(ids, bf["landmark_chunk_ids"])
    assert np.array_equal(v_store, bits["v"])
    # same decode step from both descriptions (A rows of the last chunk taken from the append on both sides)
    A_full = bits["A"].copy(); A_full[:, s0:] = want_A
    q = O.as_bits(t["q_pool"][0]); pos = t["pos_offset"].numpy()
    grown = _params(wl_long, ctx_len=s1, cap=s1)
    r_app = O.decode_step(grown, q, A, bits["B"], lm, ids, bs["k_outlier"], bs["v_outlier"], bits["k_local"],
                          bits["v_local"], v_store, pos)
    r_full = O.decode_step(full, q, A_full, bits["B"], bf["landmarks"], bf["landmark_chunk_ids"], bs["k_outlier"],
                           bs["v_outlier"], bits["k_local"], bits["v_local"], bits["v"], pos)
    for k in ("out", "chunk_ids", "k_sparse"):
        assert np.array_equal(r_app[k], r_full[k]), k


def test_append_needs_room():
    wl = _wl()
    p = _params(wl)            # capacity == ctx_len: no room
    b, h, d, c, r = wl.batch, wl.n_kv_heads, wl.head_dim, wl.chunk_size, wl.rank
    z = lambda *sh: np.zeros(sh, np.uint16)
    with pytest.raises(ValueError):
        O.append_chunk(p, z(b, c, h * d), z(b, h, c, d), z(b, h, c, d), z(b, h, r, d), z(b, p.capacity, r),
                       z(b, h, p.landmark_capacity, d), np.zeros((b, h, p.landmark_capacity), np.int32),
                       z(b, h, p.capacity, d))

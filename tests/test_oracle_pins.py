"""Pins of the CPU oracle to things other than itself (CPU only).

Each test checks the oracle against a definition, identity or special case that
the paper and the mathematics fix:

* a second, loop-by-loop implementation written from the pre-filling and
  decoding algorithms (Alg. 1, Alg. 2) using the *literal* softmax of Alg. 2,
* dense softmax attention (scipy) when the budget covers every chunk,
* exact reconstruction at full rank with an orthogonal factor whose entries
  are exact in bf16,
* RoPE group identities and a high-precision (decimal) angle reduction,
* chunk size 1 (landmarks are the keys: token-level top-k),
* closed forms of the chunk cosine criterion, and the tie rules.
"""
import decimal
import math

import numpy as np
import pytest
import torch
from scipy.special import log_softmax, softmax

from oracle import shadowkv_oracle as O


# ----------------------------------------------------------------------------- helpers
def bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round float array to bf16 (torch's RNE) and return the raw bits."""
    t = torch.from_numpy(np.ascontiguousarray(x, dtype=np.float32)).to(torch.bfloat16)
    return t.view(torch.int16).numpy().view(np.uint16).copy()


def f64(bits):
    return O.bits_to_f64(bits)


def tiny_problem(seed, b=2, hq=4, hkv=2, d=8, s=64, c=4, r=8, k=3, o=2, w=3, theta=1e4, scale_k=2.0):
    rng = np.random.default_rng(seed)
    p = O.OracleParams(b, hq, hkv, d, s, c, r, o, k, w, rope_theta=theta)
    t = {
        "q": bf16_bits(rng.normal(size=(b, hq, d))),
        "A": bf16_bits(rng.normal(size=(b, s, r))),
        "B": bf16_bits(rng.normal(size=(b, hkv, r, d)) * scale_k / math.sqrt(r)),
        "k_rope": bf16_bits(rng.normal(size=(b, hkv, s, d)) * scale_k),
        "v": bf16_bits(rng.normal(size=(b, hkv, s, d))),
        "k_local": bf16_bits(rng.normal(size=(b, hkv, w, d)) * scale_k),
        "v_local": bf16_bits(rng.normal(size=(b, hkv, w, d))),
        "pos_offset": rng.integers(0, 1000, size=(b,)).astype(np.int32),
    }
    return p, t


def textbook_rope(x, pos, theta, d):
    """Complex-number form of the rotation: (x_i + j x_{i+d/2}) * exp(j pos theta^(-2i/d))."""
    half = d // 2
    z = x[..., :half] + 1j * x[..., half:]
    ang = np.asarray(pos, dtype=np.float64)[..., None] * theta ** (-2.0 * np.arange(half) / d)
    z = z * np.exp(1j * ang)
    return np.concatenate([z.real, z.imag], axis=-1)


# ----------------------------------------------------------------------------- T1 brute force
def brute_build(p, k_rope, v):
    """Alg. 1 (after the SVD) with explicit loops, written independently of the C oracle."""
    b, h, s, d, c, o = p.batch, p.n_kv_heads, p.ctx_len, p.head_dim, p.chunk_size, p.n_outlier_chunks
    K, V = f64(k_rope), f64(v)
    res = []
    for bi in range(b):
        for hi in range(h):
            means, spread = [], []
            for j in range(s // c):
                rows = [K[bi, hi, j * c + t] for t in range(c)]
                mu = sum(rows) / c
                cosines = []
                for row in rows:
                    num = float(np.dot(mu, row))
                    den = max(np.linalg.norm(mu), 1e-8) * max(np.linalg.norm(row), 1e-8)
                    cosines.append(num / den)
                means.append(mu)
                spread.append(min(cosines))
            order = sorted(range(s // c), key=lambda j: (spread[j], j))   # lowest cosine first, then lower id
            outl = order[:o]
            keep = [j for j in range(s // c) if j not in outl]
            res.append({
                "outliers": outl,
                "keep": keep,
                "L": np.array([means[j] for j in keep]).reshape(len(keep), d),
                "Ko": np.array([K[bi, hi, j * c + t] for j in outl for t in range(c)]).reshape(o * c, d),
                "Vo": np.array([V[bi, hi, j * c + t] for j in outl for t in range(c)]).reshape(o * c, d),
                "spread": spread,
            })
    return res


def brute_decode(p, t, L_bits, L_ids, Ko_bits, Vo_bits):
    """Alg. 2 with the literal softmax -> group max -> ArgTopK, then softmax attention."""
    b, hq, h, s, d = p.batch, p.n_q_heads, p.n_kv_heads, p.ctx_len, p.head_dim
    c, r, o, k, w = p.chunk_size, p.rank, p.n_outlier_chunks, p.topk_chunks, p.local_len
    G = hq // h
    q, A, B, V = f64(t["q"]), f64(t["A"]), f64(t["B"]), f64(t["v"])
    L, Ko, Vo = f64(L_bits), f64(Ko_bits), f64(Vo_bits)
    Kl, Vl = f64(t["k_local"]), f64(t["v_local"])
    out = np.zeros((b, hq, d))
    sel = np.zeros((b, h, k), dtype=np.int64)
    for bi in range(b):
        for hi in range(h):
            n_c = L.shape[2]
            S = np.zeros((G, n_c))
            for g in range(G):
                P = np.array([np.dot(q[bi, hi * G + g], L[bi, hi, j]) for j in range(n_c)]) / math.sqrt(d)
                e = np.exp(P - P.max())
                S[g] = e / e.sum()
            S2 = S.max(axis=0)
            order = sorted(range(n_c), key=lambda j: (-S2[j], j))[:k]
            keys, vals = [], []
            for i in range(o * c):
                keys.append(Ko[bi, hi, i]); vals.append(Vo[bi, hi, i])
            for slot in order:
                ch = int(L_ids[bi, hi, slot])
                for tt in range(c):
                    n = ch * c + tt
                    kpre = np.zeros(d)
                    for rho in range(r):
                        kpre += A[bi, n, rho] * B[bi, hi, rho]
                    pos = int(t["pos_offset"][bi]) + n
                    half = d // 2
                    rot = np.zeros(d)
                    for i in range(half):
                        phi = pos * p.rope_theta ** (-2.0 * i / d)
                        rot[i] = kpre[i] * math.cos(phi) - kpre[i + half] * math.sin(phi)
                        rot[i + half] = kpre[i + half] * math.cos(phi) + kpre[i] * math.sin(phi)
                    keys.append(rot); vals.append(V[bi, hi, n])
            for i in range(w):
                keys.append(Kl[bi, hi, i]); vals.append(Vl[bi, hi, i])
            Kt, Vt = np.array(keys), np.array(vals)
            sel[bi, hi] = [int(L_ids[bi, hi, sl]) for sl in order]
            for g in range(G):
                a = Kt @ q[bi, hi * G + g] / math.sqrt(d)
                wgt = np.exp(a - a.max()); wgt /= wgt.sum()
                out[bi, hi * G + g] = wgt @ Vt
    return out, sel


@pytest.mark.parametrize("seed,kw", [
    (0, {}),
    (1, dict(b=1, hq=6, hkv=2, d=12, s=60, c=5, r=7, k=4, o=3, w=1)),
    (2, dict(b=2, hq=2, hkv=2, d=4, s=32, c=8, r=3, k=2, o=0, w=0)),
])
def test_t1_brute_force(seed, kw):
    p, t = tiny_problem(seed, **kw)
    got = O.build_landmarks(p, t["k_rope"], t["v"], diagnostics=True)
    ref = brute_build(p, t["k_rope"], t["v"])
    u = 0
    for bi in range(p.batch):
        for hi in range(p.n_kv_heads):
            r_ = ref[u]; u += 1
            assert list(got["outlier_chunk_ids"][bi, hi]) == r_["outliers"]
            assert list(got["landmark_chunk_ids"][bi, hi]) == r_["keep"]
            np.testing.assert_allclose(got["chunk_min_cos"][bi, hi], r_["spread"], rtol=0, atol=1e-13)
            np.testing.assert_array_equal(f64(got["k_outlier"][bi, hi]), r_["Ko"])
            np.testing.assert_array_equal(f64(got["v_outlier"][bi, hi]), r_["Vo"])
            # landmarks are the means rounded once to bf16
            np.testing.assert_array_equal(got["landmarks"][bi, hi], bf16_bits(r_["L"]))
    dec = O.decode_step(p, t["q"], t["A"], t["B"], got["landmarks"], got["landmark_chunk_ids"],
                        got["k_outlier"], got["v_outlier"], t["k_local"], t["v_local"], t["v"], t["pos_offset"])
    out_ref, sel_ref = brute_decode(p, t, got["landmarks"], got["landmark_chunk_ids"],
                                    got["k_outlier"], got["v_outlier"])
    np.testing.assert_array_equal(dec["chunk_ids"], sel_ref)
    np.testing.assert_allclose(dec["out_f64"], out_ref, rtol=0, atol=1e-12)
    np.testing.assert_array_equal(dec["out"], bf16_bits(out_ref))


# ----------------------------------------------------------------------------- T2 full budget == dense
def dense_attention(q_rows, keys, vals, d):
    """softmax(q K^T / sqrt(d)) V with library routines."""
    return softmax(q_rows @ keys.T / math.sqrt(d), axis=-1) @ vals


def full_budget_reference(p, t, bl):
    """Dense attention over [outliers ; RoPE(A B) of every non-outlier chunk ; recent tokens]."""
    G = p.n_q_heads // p.n_kv_heads
    c, d = p.chunk_size, p.head_dim
    out = np.zeros((p.batch, p.n_q_heads, d))
    A, B, V, q = f64(t["A"]), f64(t["B"]), f64(t["v"]), f64(t["q"])
    for bi in range(p.batch):
        for hi in range(p.n_kv_heads):
            toks = (bl["landmark_chunk_ids"][bi, hi][:, None].astype(np.int64) * c + np.arange(c)).reshape(-1)
            kpre = A[bi, toks] @ B[bi, hi]
            krot = textbook_rope(kpre, toks + int(t["pos_offset"][bi]), p.rope_theta, d)
            keys = np.concatenate([f64(bl["k_outlier"][bi, hi]), krot, f64(t["k_local"][bi, hi])])
            vals = np.concatenate([f64(bl["v_outlier"][bi, hi]), V[bi, hi, toks], f64(t["v_local"][bi, hi])])
            out[bi, hi * G:(hi + 1) * G] = dense_attention(q[bi, hi * G:(hi + 1) * G], keys, vals, d)
    return out


def test_t2_full_budget_is_dense_attention_and_ignores_landmarks():
    p, t = tiny_problem(5, b=2, hq=8, hkv=2, d=16, s=96, c=4, r=6, k=21, o=3, w=5)
    assert p.topk_chunks == p.n_landmarks
    bl = O.build_landmarks(p, t["k_rope"], t["v"])
    ref = full_budget_reference(p, t, bl)
    dec = O.decode_step(p, t["q"], t["A"], t["B"], bl["landmarks"], bl["landmark_chunk_ids"], bl["k_outlier"],
                        bl["v_outlier"], t["k_local"], t["v_local"], t["v"], t["pos_offset"])
    np.testing.assert_allclose(dec["out_f64"], ref, rtol=0, atol=1e-12)
    # every non-outlier chunk is selected exactly once
    for bi in range(p.batch):
        for hi in range(p.n_kv_heads):
            assert sorted(dec["chunk_ids"][bi, hi]) == list(bl["landmark_chunk_ids"][bi, hi])
    # any landmark values give the same output when everything is selected
    rng = np.random.default_rng(0)
    junk = bf16_bits(rng.normal(size=bl["landmarks"].shape))
    dec2 = O.decode_step(p, t["q"], t["A"], t["B"], junk, bl["landmark_chunk_ids"], bl["k_outlier"],
                         bl["v_outlier"], t["k_local"], t["v_local"], t["v"], t["pos_offset"])
    np.testing.assert_allclose(dec2["out_f64"], ref, rtol=0, atol=1e-12)


# ----------------------------------------------------------------------------- T3 exact reconstruction
def hadamard(n):
    H = np.array([[1.0]])
    while H.shape[0] < n:
        H = np.block([[H, H], [H, -H]])
    return H


def test_t3_full_rank_orthogonal_factor_reproduces_true_keys():
    b, hq, hkv, d, s, c, w = 2, 4, 2, 8, 48, 4, 2
    D = hkv * d                      # 16: a Hadamard matrix scaled by 1/4 is orthogonal and exact in bf16
    rng = np.random.default_rng(11)
    k_pre = rng.integers(-6, 7, size=(b, s, D)).astype(np.float64)      # small integers: A stays exact
    psi = hadamard(D) / 4.0
    A = k_pre @ psi                                                      # multiples of 1/4, |.| <= 24
    Bm = psi.T                                                           # [r=D, D]
    assert np.array_equal(f64(bf16_bits(A)), A) and np.array_equal(A @ Bm, k_pre)
    p = O.OracleParams(b, hq, hkv, d, s, c, D, 0, s // c, w, rope_theta=5e5)
    t = {
        "q": bf16_bits(rng.normal(size=(b, hq, d))),
        "A": bf16_bits(A),
        "B": bf16_bits(Bm.reshape(D, hkv, d).transpose(1, 0, 2)[None].repeat(b, 0)),
        "v": bf16_bits(rng.normal(size=(b, hkv, s, d))),
        "k_local": bf16_bits(rng.normal(size=(b, hkv, w, d))),
        "v_local": bf16_bits(rng.normal(size=(b, hkv, w, d))),
        "pos_offset": np.array([7, 100000], dtype=np.int32),
    }
    empty = np.zeros((b, hkv, 0, d), np.uint16)
    ids = np.tile(np.arange(s // c, dtype=np.int32), (b, hkv, 1))
    L = bf16_bits(rng.normal(size=(b, hkv, s // c, d)))
    dec = O.decode_step(p, t["q"], t["A"], t["B"], L, ids, empty, empty, t["k_local"], t["v_local"], t["v"],
                        t["pos_offset"])
    # dense attention over the TRUE rotated keys, keys laid out per head
    G = hq // hkv
    q, V = f64(t["q"]), f64(t["v"])
    for bi in range(b):
        for hi in range(hkv):
            true_k = textbook_rope(k_pre[bi, :, hi * d:(hi + 1) * d], np.arange(s) + int(t["pos_offset"][bi]), 5e5, d)
            keys = np.concatenate([true_k, f64(t["k_local"][bi, hi])])
            vals = np.concatenate([V[bi, hi], f64(t["v_local"][bi, hi])])
            ref = dense_attention(q[bi, hi * G:(hi + 1) * G], keys, vals, d)
            np.testing.assert_allclose(dec["out_f64"][bi, hi * G:(hi + 1) * G], ref, rtol=0, atol=1e-11)
            # the rebuilt keys themselves, reordered by selected chunk
            order = dec["chunk_ids"][bi, hi]
            toks = (order[:, None].astype(np.int64) * c + np.arange(c)).reshape(-1)
            np.testing.assert_allclose(dec["k_sparse"][bi, hi], true_k[toks], rtol=0, atol=1e-10)


# ----------------------------------------------------------------------------- T4 RoPE identities
def test_t4_rope_identities():
    d, theta = 16, 5e5
    p = O.OracleParams(1, 1, 1, d, 8, 8, 1, 0, 0, 0, rope_theta=theta)
    rng = np.random.default_rng(3)
    x = rng.normal(size=(6, d)); y = rng.normal(size=(6, d))
    zero = np.zeros(6)
    np.testing.assert_array_equal(O.rope(p, x, zero), x)                       # position 0 is the identity
    a = np.array([1., 17., 300., 4096., 65537., 1048575.]); bpos = np.array([5., 2., 77., 1000., 3., 12345.])
    ra = O.rope(p, x, a)
    half = d // 2
    np.testing.assert_allclose(ra[:, :half] ** 2 + ra[:, half:] ** 2, x[:, :half] ** 2 + x[:, half:] ** 2,
                               rtol=1e-13)                                      # each pair keeps its norm
    np.testing.assert_allclose(O.rope(p, ra, bpos), O.rope(p, x, a + bpos), atol=1e-9)   # rotations compose
    lhs = np.sum(O.rope(p, x, a) * O.rope(p, y, bpos), axis=1)                 # inner product sees m-n only
    rhs = np.sum(O.rope(p, x, a - bpos + 50.0) * O.rope(p, y, np.full(6, 50.0)), axis=1)
    np.testing.assert_allclose(lhs, rhs, atol=1e-8)
    np.testing.assert_allclose(ra, textbook_rope(x, a, theta, d), atol=1e-9)   # complex-exponential form
    # pairing is (i, i+d/2): a unit vector on axis 0 only ever leaks into axis d/2
    e0 = np.zeros((1, d)); e0[0, 0] = 1.0
    r0 = O.rope(p, e0, np.array([1.0]))
    assert abs(r0[0, 0] - math.cos(1.0)) < 1e-15 and abs(r0[0, half] - math.sin(1.0)) < 1e-15
    assert np.count_nonzero(r0) == 2


def test_t4_rope_large_position_against_decimal_reduction():
    d, theta = 128, 5e5
    p = O.OracleParams(1, 1, 1, d, 8, 8, 1, 0, 0, 0, rope_theta=theta)
    decimal.getcontext().prec = 60
    two_pi = 2 * decimal.Decimal("3.14159265358979323846264338327950288419716939937510582097494")
    half = d // 2
    for pos in (1048575, 1048576 + 31, 999983):
        x = np.zeros((1, d)); x[0, :half] = 1.0
        got = O.rope(p, x, np.array([float(pos)]))[0]
        for i in (0, 1, 5, 31, 63):
            f = theta ** (-2.0 * i / d)                     # the double the definition produces
            ang = decimal.Decimal(pos) * decimal.Decimal(f)
            red = float(ang - (ang / two_pi).to_integral_value(rounding=decimal.ROUND_FLOOR) * two_pi)
            # the oracle rounds pos*f to a double before cos/sin: allow that one rounding (<= 2^-33 rad here)
            assert abs(got[i] - math.cos(red)) < 5e-10 and abs(got[i + half] - math.sin(red)) < 5e-10


def test_inv_freq_override_matches_theta_definition():
    d = 8
    rng = np.random.default_rng(1)
    x = rng.normal(size=(4, d)); pos = np.array([3., 50., 700., 9000.])
    inv = (1e4 ** (-2.0 * np.arange(d // 2) / d)).astype(np.float32)
    p1 = O.OracleParams(1, 1, 1, d, 8, 8, 1, 0, 0, 0, rope_theta=123.0, inv_freq=inv)
    z = x[:, :d // 2] + 1j * x[:, d // 2:]
    z = z * np.exp(1j * pos[:, None] * inv.astype(np.float64)[None, :])
    ref = np.concatenate([z.real, z.imag], axis=1)
    np.testing.assert_allclose(O.rope(p1, x, pos), ref, atol=1e-10)


# ----------------------------------------------------------------------------- T5 chunk size 1
def test_t5_chunk_size_one_is_token_topk_attention():
    p, t = tiny_problem(8, b=1, hq=4, hkv=2, d=8, s=40, c=1, r=5, k=6, o=0, w=2)
    bl = O.build_landmarks(p, t["k_rope"], t["v"], diagnostics=True)
    np.testing.assert_array_equal(bl["landmarks"], t["k_rope"])                 # mean of one bf16 row is the row
    np.testing.assert_allclose(bl["chunk_min_cos"], 1.0, atol=1e-14)
    dec = O.decode_step(p, t["q"], t["A"], t["B"], bl["landmarks"], bl["landmark_chunk_ids"], bl["k_outlier"],
                        bl["v_outlier"], t["k_local"], t["v_local"], t["v"], t["pos_offset"])
    q, K, A, B, V = f64(t["q"]), f64(t["k_rope"]), f64(t["A"]), f64(t["B"]), f64(t["v"])
    G = 2
    for hi in range(2):
        ls = log_softmax(q[0, hi * G:(hi + 1) * G] @ K[0, hi].T / math.sqrt(8), axis=-1).max(axis=0)
        top = np.argsort(-ls, kind="stable")[:6]
        assert list(dec["chunk_ids"][0, hi]) == list(top)
        krot = textbook_rope(A[0, top] @ B[0, hi], top + int(t["pos_offset"][0]), p.rope_theta, 8)
        keys = np.concatenate([krot, f64(t["k_local"][0, hi])]); vals = np.concatenate([V[0, hi, top], f64(t["v_local"][0, hi])])
        np.testing.assert_allclose(dec["out_f64"][0, hi * G:(hi + 1) * G],
                                   dense_attention(q[0, hi * G:(hi + 1) * G], keys, vals, 8), atol=1e-12)


# ----------------------------------------------------------------------------- T6 group handling
def test_t6_single_head_group_ranks_by_raw_logits_and_shared_query():
    p, t = tiny_problem(9, b=1, hq=2, hkv=2, d=8, s=128, c=4, r=4, k=5, o=1, w=1)
    bl = O.build_landmarks(p, t["k_rope"], t["v"])
    dec = O.decode_step(p, t["q"], t["A"], t["B"], bl["landmarks"], bl["landmark_chunk_ids"], bl["k_outlier"],
                        bl["v_outlier"], t["k_local"], t["v_local"], t["v"], t["pos_offset"])
    q, L = f64(t["q"]), f64(bl["landmarks"])
    for hi in range(2):
        raw = L[0, hi] @ q[0, hi]
        top = np.argsort(-raw, kind="stable")[:5]
        assert list(dec["chunk_ids"][0, hi]) == list(bl["landmark_chunk_ids"][0, hi][top])
    # G = 3 with the same query repeated in the group selects what a single head selects
    p3 = O.OracleParams(1, 6, 2, 8, 128, 4, 4, 1, 5, 1, rope_theta=p.rope_theta)
    q3 = np.repeat(t["q"], 3, axis=1)
    dec3 = O.decode_step(p3, q3, t["A"], t["B"], bl["landmarks"], bl["landmark_chunk_ids"], bl["k_outlier"],
                         bl["v_outlier"], t["k_local"], t["v_local"], t["v"], t["pos_offset"])
    np.testing.assert_array_equal(dec3["chunk_ids"], dec["chunk_ids"])
    # duplicated query heads give duplicated outputs
    np.testing.assert_array_equal(dec3["out"][:, 0::3], dec3["out"][:, 1::3])
    np.testing.assert_array_equal(dec3["out"][:, 0::3], dec["out"])


def test_g1_group_max_uses_each_heads_own_normaliser():
    """One head with a flat softmax, one with a peaked one: the normaliser changes who wins."""
    d, n_ch, c = 4, 6, 1
    p = O.OracleParams(1, 2, 1, d, n_ch, c, 1, 0, 1, 0, softmax_scale=1.0)
    L = np.zeros((1, 1, n_ch, d)); L[0, 0, :, 0] = [0, 0, 0, 0, 0, 3.0]; L[0, 0, :, 1] = [2.0, 1.9, 1.9, 1.9, 1.9, 0]
    q = np.zeros((1, 2, d)); q[0, 0, 0] = 1.0; q[0, 1, 1] = 1.0
    # head 0: logits (0,0,0,0,0,3) -> softmax of slot 5 = e^3/(5+e^3) = 0.80 ; head 1: nearly flat, max 2.0 -> 0.22
    zeros_kv = np.zeros((1, 1, 0, d), np.uint16)
    dec = O.decode_step(p, bf16_bits(q), bf16_bits(np.zeros((1, n_ch, 1))), bf16_bits(np.zeros((1, 1, 1, d))),
                        bf16_bits(L), np.arange(n_ch, dtype=np.int32).reshape(1, 1, n_ch), zeros_kv, zeros_kv,
                        zeros_kv, zeros_kv, bf16_bits(np.ones((1, 1, n_ch, d))))
    assert dec["chunk_ids"][0, 0, 0] == 5
    # slot 5's group score is head 0's log-softmax; slot 0's is head 1's
    assert abs(dec["z2"][0, 0, 5] - math.log(math.exp(3) / (5 + math.exp(3)))) < 1e-12
    l19 = f64(bf16_bits(np.array([1.9])))[0]
    assert abs(dec["z2"][0, 0, 0] - math.log(math.exp(2.0) / (math.exp(2.0) + 4 * math.exp(l19) + 1.0))) < 1e-12


def test_chunk_logits_are_not_rounded_on_the_way_to_the_ranking():
    """P = Q L^T is the plain product (decoding algorithm, first line): slot 1's logit is 1 + 2^-30, slot 0's is 1.
    The two differ far below fp32 (and bf16) resolution, and the single place in the budget still goes to slot 1;
    with the operands swapped it goes to slot 0.  Any rounding of the logit below fp64 would tie them and hand the
    place to the lower slot both times."""
    d, n_ch = 4, 3
    p = O.OracleParams(1, 1, 1, d, n_ch, 1, 1, 0, 1, 0, softmax_scale=1.0)
    q = np.zeros((1, 1, d)); q[0, 0, 0] = 1.0; q[0, 0, 1] = 2.0 ** -15
    zeros_kv = np.zeros((1, 1, 0, d), np.uint16)

    def best(second):
        L = np.zeros((1, 1, n_ch, d)); L[0, 0, :, 0] = [1.0, 1.0, 0.5]; L[0, 0, :, 1] = second
        dec = O.decode_step(p, bf16_bits(q), bf16_bits(np.zeros((1, n_ch, 1))), bf16_bits(np.zeros((1, 1, 1, d))),
                            bf16_bits(L), np.arange(n_ch, dtype=np.int32).reshape(1, 1, n_ch), zeros_kv, zeros_kv,
                            zeros_kv, zeros_kv, bf16_bits(np.ones((1, 1, n_ch, d))))
        return int(dec["chunk_ids"][0, 0, 0]), dec["z2"][0, 0]

    slot, z2 = best([0.0, 2.0 ** -15, 0.0])     # exact logits 1, 1 + 2^-30, 0.5
    assert slot == 1 and z2[1] > z2[0]
    assert abs((z2[1] - z2[0]) - 2.0 ** -30) < 2.0 ** -50    # the gap survives the normaliser (same for both slots)
    slot, z2 = best([2.0 ** -15, 0.0, 0.0])     # 1 + 2^-30, 1, 0.5
    assert slot == 0 and z2[0] > z2[1]
    slot, z2 = best([0.0, 0.0, 0.0])            # an exact tie: lower slot
    assert slot == 0 and z2[0] == z2[1]


# ----------------------------------------------------------------------------- T7 invariants
def test_t7_output_in_value_hull_and_shift_invariance():
    p, t = tiny_problem(12, b=1, hq=4, hkv=1, d=8, s=64, c=4, r=4, k=4, o=2, w=3)
    bl = O.build_landmarks(p, t["k_rope"], t["v"])
    dec = O.decode_step(p, t["q"], t["A"], t["B"], bl["landmarks"], bl["landmark_chunk_ids"], bl["k_outlier"],
                        bl["v_outlier"], t["k_local"], t["v_local"], t["v"], t["pos_offset"])
    toks = (dec["chunk_ids"][0, 0][:, None].astype(np.int64) * 4 + np.arange(4)).reshape(-1)
    vals = np.concatenate([f64(bl["v_outlier"][0, 0]), f64(t["v"])[0, 0, toks], f64(t["v_local"][0, 0])])
    assert np.all(dec["out_f64"][0] <= vals.max(axis=0) + 1e-12) and np.all(dec["out_f64"][0] >= vals.min(axis=0) - 1e-12)
    # constant values -> output is that constant whatever the weights are
    ones = bf16_bits(np.full((1, 1, 64, 8), 0.75))
    blc = O.build_landmarks(p, t["k_rope"], ones)
    decc = O.decode_step(p, t["q"], t["A"], t["B"], blc["landmarks"], blc["landmark_chunk_ids"], blc["k_outlier"],
                         blc["v_outlier"], t["k_local"], bf16_bits(np.full((1, 1, 3, 8), 0.75)), ones, t["pos_offset"])
    np.testing.assert_allclose(decc["out_f64"], 0.75, atol=1e-14)


# ----------------------------------------------------------------------------- T9 cosine closed forms and tie rules
def test_t9_cosine_closed_forms():
    d, c = 4, 2
    rows = np.zeros((6 * c, d))
    rows[0] = rows[1] = [1.0, 2.0, -1.0, 0.5]            # identical rows: min cos 1
    rows[2] = [1.0, -2.0, 0.25, 4.0]; rows[3] = -rows[2]  # x, -x: zero mean -> cos 0 by the epsilon clamp
    rows[4] = [3.0, 0, 0, 0]; rows[5] = [0, 3.0, 0, 0]    # orthogonal, equal norm: 1/sqrt(2)
    rows[6] = [3.0, 0, 0, 0]; rows[7] = [0, 4.0, 0, 0]    # orthogonal, norms 3 and 4: min(3,4)/5
    rows[8] = 8 * rows[6]; rows[9] = 8 * rows[7]          # positive scaling leaves it unchanged
    rows[10] = [1.0, 0, 0, 0]; rows[11] = [1.0, 1.0, 0, 0]  # mean (1,.5): cos to rows: 1/sqrt(1.25), 1.5/sqrt(2.5)
    p = O.OracleParams(1, 1, 1, d, 6 * c, c, 1, 2, 1, 0)
    bl = O.build_landmarks(p, bf16_bits(rows.reshape(1, 1, -1, d)), None, diagnostics=True)
    m = bl["chunk_min_cos"][0, 0]
    np.testing.assert_allclose(m, [1.0, 0.0, 1 / math.sqrt(2), 0.6, 0.6, 1 / math.sqrt(1.25)], atol=1e-15)
    np.testing.assert_allclose(bl["chunk_mean"][0, 0, 5], [1.0, 0.5, 0, 0], atol=0)
    # the two lowest are chunk 1 (0.0) then chunks 3/4 tied at 0.6 -> lower id 3
    assert list(bl["outlier_chunk_ids"][0, 0]) == [1, 3]
    assert list(bl["landmark_chunk_ids"][0, 0]) == [0, 2, 4, 5]


def test_tie_rules_duplicate_chunks_and_duplicate_landmarks():
    p, t = tiny_problem(21, b=1, hq=2, hkv=1, d=8, s=64, c=4, r=4, k=3, o=2, w=0)
    k = t["k_rope"].copy()
    # find the most outlying chunk, then clone it into two other places: three exact ties
    base = O.build_landmarks(p, k, t["v"])["outlier_chunk_ids"][0, 0, 0]
    src = k[0, 0, base * 4:(base + 1) * 4].copy()
    places = sorted({int(base), 13, 2})
    for j in places:
        k[0, 0, j * 4:(j + 1) * 4] = src
    bl = O.build_landmarks(p, k, t["v"])
    assert list(bl["outlier_chunk_ids"][0, 0]) == places[:2]          # lower chunk ids win the tie
    # duplicate landmark rows tie exactly in the decode score: lower slots win
    L = bl["landmarks"].copy(); L[0, 0, :] = L[0, 0, 0]
    dec = O.decode_step(p, t["q"], t["A"], t["B"], L, bl["landmark_chunk_ids"], bl["k_outlier"], bl["v_outlier"],
                        t["k_local"], t["v_local"], t["v"], t["pos_offset"])
    assert list(dec["chunk_ids"][0, 0]) == list(bl["landmark_chunk_ids"][0, 0, :3])


def test_bf16_rounding_is_single_and_to_even():
    vals = np.array([1.0 + 2 ** -8, 1.0 + 3 * 2 ** -8, 1.0 + 2 ** -8 + 2 ** -30, -(1.0 + 2 ** -8), 2 ** -133 * 1.5,
                     2 ** -134, 3.3895313892515355e38, 3.4e38])
    want = np.array([0x3f80, 0x3f82, 0x3f81, 0xbf80, 0x0002, 0x0000, 0x7f7f, 0x7f80], dtype=np.uint16)
    np.testing.assert_array_equal(O.f64_to_bits(vals), want)
    # a value that double rounding (fp64 -> fp32 -> bf16) would get wrong: just above a bf16 tie, below fp32 resolution
    x = 1.0 + 2 ** -8 + 2 ** -40
    assert O.f64_to_bits(np.array([x]))[0] == 0x3f81
    # agreement with torch on ordinary fp32 values
    rng = np.random.default_rng(0)
    v = rng.normal(size=1000).astype(np.float32)
    np.testing.assert_array_equal(O.f64_to_bits(v.astype(np.float64)), bf16_bits(v))


def test_argument_errors():
    p, t = tiny_problem(0)
    bl = O.build_landmarks(p, t["k_rope"], t["v"])
    bad = O.OracleParams(**{**p.__dict__, "topk_chunks": p.n_landmarks + 1})
    with pytest.raises((ValueError, AssertionError)):
        O.decode_step(bad, t["q"], t["A"], t["B"], bl["landmarks"], bl["landmark_chunk_ids"], bl["k_outlier"],
                      bl["v_outlier"], t["k_local"], t["v_local"], t["v"], t["pos_offset"])

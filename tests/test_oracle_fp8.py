"""Pins of the oracle's FP8 (E5M2) storage mode (section "Precision Sensitivity"), CPU only.

* the decoder against the format's definition written out with exact fractions, against numpy's IEEE
  half (an E5M2 byte is the upper byte of a half) and against torch's own E5M2 type;
* the encoder (one rounding, to nearest, ties to even, overflow to infinity) against a brute-force
  search over the 256 codes, on every midpoint between neighbouring codes and on both sides of it,
  and against torch's cast on values where that cast rounds once;
* the three operations: bytes whose values are exact in bf16 must give, bit for bit, what the bf16
  mode gives on the widened inputs (ids, scores, rebuilt keys, outputs); what the method rounds itself
  (landmarks, low-rank states of generated tokens) must be the brute-force rounding of the fp64 value.
"""
import math
from fractions import Fraction

import numpy as np
import pytest
import torch

from oracle import shadowkv_oracle as O

ALL = np.arange(256, dtype=np.uint8)


def definition(byte: int):
    """Value of an E5M2 byte from the format's definition; None for NaN."""
    sign = -1 if byte >> 7 else 1
    e, m = (byte >> 2) & 31, byte & 3
    if e == 31:
        return None if m else sign * math.inf
    if e == 0:
        return sign * Fraction(m, 4) * Fraction(1, 2 ** 14)
    return sign * (1 + Fraction(m, 4)) * Fraction(2) ** (e - 15)


FINITE = [(b, definition(b)) for b in range(128) if definition(b) is not None and definition(b) != math.inf]


def brute_encode(x: Fraction) -> int:
    """Nearest code of a non-negative exact value; ties to the even code; past the midpoint between the
    largest finite value and 2^16 -> infinity (0x7c)."""
    top = Fraction(57344)
    if x >= (top + 65536) / 2:
        return 0x7C
    best = min(FINITE, key=lambda bv: (abs(bv[1] - x), bv[0] & 1))
    return best[0]


def test_decoder_matches_the_definition_half_floats_and_torch():
    got = O.e5m2_bits_to_f64(ALL)
    half = (ALL.astype(np.uint16) << 8).view(np.float16).astype(np.float64)
    viat = torch.from_numpy(ALL.copy()).view(torch.float8_e5m2).to(torch.float32).numpy().astype(np.float64)
    for b in range(256):
        ref = definition(b)
        if ref is None:
            assert math.isnan(got[b]) and math.isnan(half[b]) and math.isnan(viat[b])
        else:
            assert got[b] == float(ref), (b, got[b], ref)
            assert math.copysign(1.0, got[b]) == (-1.0 if b >> 7 else 1.0)
            assert got[b] == half[b] == viat[b]
    assert got[0x7B] == 57344.0 and got[0x01] == 2.0 ** -16 and got[0x04] == 2.0 ** -14


def test_encoder_against_brute_force_on_midpoints_and_neighbours():
    vals = [v for _, v in FINITE]
    cases = []
    for lo, hi in zip(vals[:-1], vals[1:]):
        mid = (lo + hi) / 2
        cases += [lo, mid, mid - (hi - lo) / 1024, mid + (hi - lo) / 1024, lo + (hi - lo) / 3]
    cases += [Fraction(57344), Fraction(61440), Fraction(61440) - Fraction(1, 64), Fraction(61440) + 1,
              Fraction(65536), Fraction(10 ** 9), Fraction(1, 2 ** 17), Fraction(1, 2 ** 17) + Fraction(1, 2 ** 40),
              Fraction(3, 2 ** 17), Fraction(1, 2 ** 30)]
    for x in cases:
        want = brute_encode(x)
        assert int(O.f64_to_e5m2_bits(np.array([float(x)]))[0]) == want, (float(x), want)
        assert int(O.f64_to_e5m2_bits(np.array([-float(x)]))[0]) == (want | 0x80), (float(x), want)
    assert int(O.f64_to_e5m2_bits(np.array([np.inf]))[0]) == 0x7C
    assert int(O.f64_to_e5m2_bits(np.array([-0.0]))[0]) == 0x80
    assert math.isnan(O.e5m2_bits_to_f64(O.f64_to_e5m2_bits(np.array([np.nan])))[0])


def test_encoder_agrees_with_torch_cast_of_fp32_values():
    rng = np.random.default_rng(5)
    x = (rng.normal(size=20000) * np.exp(rng.uniform(-14, 11, size=20000))).astype(np.float32)
    want = torch.from_numpy(x).to(torch.float8_e5m2).view(torch.uint8).numpy()
    got = O.f64_to_e5m2_bits(x.astype(np.float64))
    np.testing.assert_array_equal(got, want)


# ------------------------------------------------------------------------------------ the operations
def e5m2_bytes(rng, shape, scale=1.0):
    """Random E5M2 bytes: normal draws rounded by torch's cast (finite by construction)."""
    x = torch.from_numpy((rng.normal(size=shape) * scale).astype(np.float32))
    return x.to(torch.float8_e5m2).view(torch.uint8).numpy().copy()


def widen_to_bf16_bits(bits8):
    """E5M2 bytes -> bf16 bit patterns of the same values (every E5M2 value is exact in bf16)."""
    f = O.e5m2_bits_to_f64(bits8).astype(np.float32)
    u = f.view(np.uint32)
    assert not (u & 0xFFFF).any()
    return (u >> 16).astype(np.uint16)


def bf16_bits(x):
    t = torch.from_numpy(np.ascontiguousarray(x, dtype=np.float32)).to(torch.bfloat16)
    return t.view(torch.int16).numpy().view(np.uint16).copy()


def tiny_fp8(seed, b=2, hq=4, hkv=2, d=8, s=64, c=4, r=8, k=3, o=2, w=3, cap=0):
    rng = np.random.default_rng(seed)
    p8 = O.OracleParams(b, hq, hkv, d, s, c, r, o, k, w, rope_theta=1e4, ctx_capacity=cap, kv_dtype=1)
    p16 = O.OracleParams(b, hq, hkv, d, s, c, r, o, k, w, rope_theta=1e4, ctx_capacity=cap, kv_dtype=0)
    n = cap or s
    t = {
        "q": bf16_bits(rng.normal(size=(b, hq, d))),
        "A": e5m2_bytes(rng, (b, n, r)),
        "B": e5m2_bytes(rng, (b, hkv, r, d), 2.0 / math.sqrt(r)),
        "k_rope": e5m2_bytes(rng, (b, hkv, s, d), 2.0),
        "v": e5m2_bytes(rng, (b, hkv, n, d)),
        "k_local": e5m2_bytes(rng, (b, hkv, w, d), 2.0),
        "v_local": e5m2_bytes(rng, (b, hkv, w, d)),
        "pos_offset": rng.integers(0, 1000, size=(b,)).astype(np.int32),
    }
    return p8, p16, t


@pytest.mark.parametrize("seed,kw", [(0, {}), (1, dict(b=1, hq=6, hkv=2, d=12, s=60, c=5, r=7, k=4, o=3, w=1)),
                                     (2, dict(b=2, hq=2, hkv=2, d=4, s=32, c=8, r=3, k=2, o=0, w=0))])
def test_build_and_decode_equal_the_bf16_mode_on_widened_inputs(seed, kw):
    p8, p16, t = tiny_fp8(seed, **kw)
    W = {n: widen_to_bf16_bits(t[n]) for n in ("A", "B", "k_rope", "v", "k_local", "v_local")}
    b8 = O.build_landmarks(p8, t["k_rope"], t["v"], diagnostics=True)
    b16 = O.build_landmarks(p16, W["k_rope"], W["v"], diagnostics=True)
    np.testing.assert_array_equal(b8["outlier_chunk_ids"], b16["outlier_chunk_ids"])
    np.testing.assert_array_equal(b8["landmark_chunk_ids"], b16["landmark_chunk_ids"])
    np.testing.assert_array_equal(b8["chunk_min_cos"], b16["chunk_min_cos"])
    np.testing.assert_array_equal(b8["chunk_mean"], b16["chunk_mean"])
    np.testing.assert_array_equal(widen_to_bf16_bits(b8["k_outlier"]), b16["k_outlier"])
    np.testing.assert_array_equal(widen_to_bf16_bits(b8["v_outlier"]), b16["v_outlier"])
    # the landmarks are the fp64 means rounded once to E5M2: brute-force rounding of the exact mean
    ids = b8["landmark_chunk_ids"]
    for bi in range(p8.batch):
        for h in range(p8.n_kv_heads):
            for slot in range(p8.n_landmarks):
                for x in range(p8.head_dim):
                    rows = [definition(int(v)) for v in
                            t["k_rope"][bi, h, ids[bi, h, slot] * p8.chunk_size:(ids[bi, h, slot] + 1) * p8.chunk_size, x]]
                    mean = sum(rows) / p8.chunk_size
                    want = brute_encode(abs(mean)) | (0x80 if mean < 0 else 0)
                    if mean == 0:
                        want = 0
                    assert int(b8["landmarks"][bi, h, slot, x]) == want
    d8 = O.decode_step(p8, t["q"], t["A"], t["B"], b8["landmarks"], b8["landmark_chunk_ids"], b8["k_outlier"],
                       b8["v_outlier"], t["k_local"], t["v_local"], t["v"], t["pos_offset"])
    d16 = O.decode_step(p16, t["q"], W["A"], W["B"], widen_to_bf16_bits(b8["landmarks"]), b8["landmark_chunk_ids"],
                        b16["k_outlier"], b16["v_outlier"], W["k_local"], W["v_local"], W["v"], t["pos_offset"])
    for name in ("chunk_ids", "z2", "k_sparse", "out_f64", "out"):
        np.testing.assert_array_equal(d8[name], d16[name], err_msg=name)
    assert np.abs(d8["out_f64"]).max() > 1e-3


def test_append_rounds_the_low_rank_states_and_the_landmark_once():
    p8, p16, t = tiny_fp8(7, s=32, cap=48, o=1)
    rng = np.random.default_rng(70)
    b, h, d, c, r = p8.batch, p8.n_kv_heads, p8.head_dim, p8.chunk_size, p8.rank
    k_pre = e5m2_bytes(rng, (b, c, h * d), 2.0)
    k_rope = e5m2_bytes(rng, (b, h, c, d), 2.0)
    v = e5m2_bytes(rng, (b, h, c, d))
    nc_cap = p8.landmark_capacity
    A, store = t["A"].copy(), t["v"].copy()
    L = e5m2_bytes(rng, (b, h, nc_cap, d))
    ids = np.full((b, h, nc_cap), -7, np.int32)
    L0, A0 = L.copy(), A.copy()
    O.append_chunk(p8, k_pre, k_rope, v, t["B"], A, L, ids, store)
    s, n_c = p8.ctx_len, p8.n_landmarks
    Bf = [[[[definition(int(x)) for x in row] for row in hd] for hd in bt] for bt in t["B"]]
    for bi in range(b):
        for tt in range(c):
            for rho in range(r):
                acc = sum(definition(int(k_pre[bi, tt, hh * d + x])) * Bf[bi][hh][rho][x] for hh in range(h) for x in range(d))
                want = 0 if acc == 0 else brute_encode(abs(acc)) | (0x80 if acc < 0 else 0)
                assert int(A[bi, s + tt, rho]) == want
    for bi in range(b):
        for hh in range(h):
            for x in range(d):
                mean = sum(definition(int(k_rope[bi, hh, tt, x])) for tt in range(c)) / c
                want = 0 if mean == 0 else brute_encode(abs(mean)) | (0x80 if mean < 0 else 0)
                assert int(L[bi, hh, n_c, x]) == want
            assert ids[bi, hh, n_c] == s // c
    np.testing.assert_array_equal(store[:, :, s:s + c], v)
    # nothing else moved
    np.testing.assert_array_equal(A[:, :s], A0[:, :s]); np.testing.assert_array_equal(A[:, s + c:], A0[:, s + c:])
    np.testing.assert_array_equal(L[:, :, :n_c], L0[:, :, :n_c]); np.testing.assert_array_equal(L[:, :, n_c + 1:], L0[:, :, n_c + 1:])


def test_subnormal_and_extreme_bytes_pass_through_the_decode_step():
    """Keys and values holding the smallest subnormal and the largest finite value: the output is the exact
    softmax average of those values (one attended row dominates)."""
    p8 = O.OracleParams(1, 1, 1, 4, 8, 4, 2, 0, 1, 0, rope_theta=1e4, kv_dtype=1)
    q = bf16_bits(np.array([[[8.0, 0, 0, 0]]]))
    A = np.zeros((1, 8, 2), np.uint8); B = np.zeros((1, 1, 2, 4), np.uint8)
    A[0, :, 0] = 0x3C                     # 1.0
    B[0, 0, 0, 0] = 0x01                  # 2^-16: every rebuilt key is (2^-16, 0, 0, 0) before the rotation
    L = np.zeros((1, 1, 2, 4), np.uint8); L[0, 0, 1, 0] = 0x7B   # second chunk scores 57344 * 8 / 2
    ids = np.array([[[0, 1]]], np.int32)
    V = np.zeros((1, 1, 8, 4), np.uint8); V[0, 0, 4:, 1] = 0x7B; V[0, 0, 4:, 2] = 0x01; V[0, 0, 4:, 3] = 0x81
    e = np.zeros((1, 1, 0, 4), np.uint8)
    res = O.decode_step(p8, q, A, B, L, ids, e, e, e, e, V)
    assert list(res["chunk_ids"][0, 0]) == [1]
    np.testing.assert_allclose(res["out_f64"][0, 0], [0.0, 57344.0, 2.0 ** -16, -2.0 ** -16], rtol=1e-12, atol=0)
    ks = res["k_sparse"][0, 0]
    np.testing.assert_allclose(np.hypot(ks[:, 0], ks[:, 2]), 2.0 ** -16, rtol=1e-12)

"""Pins of the oracle's SVD line (A, B <- SVD(K), first line of the pre-filling algorithm), CPU only.

The oracle calls LAPACK's SVD; what is pinned is everything around it and the call itself, against things that do
not go through it: matrices built from known orthogonal factors (Hadamard matrices, exact in bf16) and known singular
values; the Eckart-Young optimum computed from the eigenvalues of the Gram matrix (another LAPACK routine on another
matrix); exact recovery of exactly low-rank keys; loop-level checks of the layouts; the sign convention; the FP8 mode
against the bf16 mode on widened inputs.  Planted mistakes in the function's source must fail these pins."""
import inspect
import math

import numpy as np
import pytest
import torch

from oracle import shadowkv_oracle as O


def hadamard(n):
    H = np.array([[1.0]])
    while H.shape[0] < n:
        H = np.block([[H, H], [H, -H]])
    return H


def bf16_bits(x):
    t = torch.from_numpy(np.ascontiguousarray(x, dtype=np.float32)).to(torch.bfloat16)
    return t.view(torch.int16).numpy().view(np.uint16).copy()


def params(b, hkv, d, s, r, cap=0, kd=0):
    return O.OracleParams(b, hkv, hkv, d, s, 4, r, 0, 1, 0, ctx_capacity=cap, kv_dtype=kd)


def known_svd_case(flip_rows=False):
    """K = U diag(sv) V^T with U = 64 x 16 columns of H_64 / 8, V = H_16 / 4 (rows optionally permuted so that the
    first components are not all positive), sv = 16 .. 1: every entry of K is an integer / 32, exact in bf16."""
    s, D = 64, 16
    U = hadamard(s)[:, 1:D + 1] / 8.0
    V = hadamard(D) / 4.0
    if flip_rows:
        V = V[::-1].copy()
    sv = np.arange(D, 0, -1).astype(np.float64)
    K = (U * sv) @ V.T
    bits = bf16_bits(K)
    assert np.array_equal(O.bits_to_f64(bits), K)
    return K, bits, U, V, sv


def pin_known_factors(fn):
    for flip in (False, True):
        K, bits, U, V, sv = known_svd_case(flip)
        r = 6
        res = fn(params(1, 2, 8, 64, r), bits[None])
        np.testing.assert_allclose(res["sigma"][0], sv[:r], rtol=1e-12)
        want = V[:, :r].T.copy()                       # rows = right singular vectors, up to sign: the components
        got = res["psi"][0]                            # all have the same magnitude here, so rounding noise picks
        sgn = np.sign(np.sum(got * want, axis=1))      # the component that the sign convention looks at
        np.testing.assert_allclose(got, want * sgn[:, None], atol=1e-13)
        lead = np.argmax(np.abs(got), axis=1)
        assert np.all(got[np.arange(r), lead] > 0)
        # A = K Psi = Phi Sigma, up to the same signs
        np.testing.assert_allclose(np.abs(res["A_f64"][0]), np.abs(U[:, :r] * sv[:r]), atol=1e-12)
        np.testing.assert_allclose(res["A_f64"][0] @ res["psi"][0], (U[:, :r] * sv[:r]) @ V[:, :r].T, atol=1e-12)


def pin_eckart_young(fn):
    rng = np.random.default_rng(3)
    b, hkv, d, s, r = 2, 3, 8, 200, 7
    bits = bf16_bits(rng.normal(size=(b, s, hkv * d)) * np.exp(-np.arange(hkv * d) / 6.0))
    res = fn(params(b, hkv, d, s, r), bits)
    K = O.bits_to_f64(bits)
    for bi in range(b):
        lam = np.linalg.eigvalsh(K[bi].T @ K[bi])[::-1]
        err = np.linalg.norm(K[bi] - res["A_f64"][bi] @ res["psi"][bi]) ** 2
        assert abs(err - lam[r:].sum()) <= 1e-10 * lam.sum()
        np.testing.assert_allclose(res["sigma"][bi] ** 2, lam[:r], rtol=1e-10)
        np.testing.assert_allclose(res["psi"][bi] @ res["psi"][bi].T, np.eye(r), atol=1e-12)


def pin_exact_low_rank(fn):
    s, D, r = 64, 16, 4
    L = hadamard(s)[:, 3:3 + r] * np.array([4.0, 2.0, 1.0, 0.5])
    R = hadamard(D)[5:5 + r] / 4.0
    K = L @ R
    bits = bf16_bits(K)
    assert np.array_equal(O.bits_to_f64(bits), K)
    res = fn(params(1, 2, 8, s, r), bits[None])
    np.testing.assert_allclose(res["A_f64"][0] @ res["psi"][0], K, atol=1e-12)
    # the row space is that of R
    P, Q = res["psi"][0].T @ res["psi"][0], R.T @ np.linalg.inv(R @ R.T) @ R
    np.testing.assert_allclose(P, Q, atol=1e-12)


def pin_layouts(fn):
    rng = np.random.default_rng(4)
    b, hkv, d, s, r, cap = 2, 2, 4, 24, 3, 32
    bits = bf16_bits(rng.normal(size=(b, s, hkv * d)))
    res = fn(params(b, hkv, d, s, r, cap=cap), bits)
    assert res["A"].shape == (b, cap, r) and res["B"].shape == (b, hkv, r, d)
    K = O.bits_to_f64(bits)
    for bi in range(b):
        for rho in range(r):
            for h in range(hkv):
                for x in range(d):
                    assert res["B"][bi, h, rho, x] == O.f64_to_bits(np.array([res["psi"][bi, rho, h * d + x]]))[0]
            for tok in range(s):
                acc = sum(K[bi, tok, c] * res["psi"][bi, rho, c] for c in range(hkv * d))
                assert abs(acc - res["A_f64"][bi, tok, rho]) < 1e-12
                assert res["A"][bi, tok, rho] == O.f64_to_bits(np.array([res["A_f64"][bi, tok, rho]]))[0]
    assert not res["A"][:, s:].any()
    # sign convention on generic data: the largest-magnitude component of every vector is positive
    lead = np.argmax(np.abs(res["psi"]), axis=2)
    assert np.all(np.take_along_axis(res["psi"], lead[..., None], axis=2) > 0)


def pin_fp8_equals_bf16_on_widened_inputs(fn):
    rng = np.random.default_rng(5)
    b, hkv, d, s, r = 1, 2, 8, 96, 5
    x = torch.from_numpy((rng.normal(size=(b, s, hkv * d)) * np.exp(-np.arange(hkv * d) / 5.0)).astype(np.float32))
    b8 = x.to(torch.float8_e5m2).view(torch.uint8).numpy().copy()
    wide = O.e5m2_bits_to_f64(b8).astype(np.float32)
    b16 = (wide.view(np.uint32) >> 16).astype(np.uint16)
    r8, r16 = fn(params(b, hkv, d, s, r, kd=1), b8), fn(params(b, hkv, d, s, r), b16)
    for name in ("psi", "sigma", "A_f64"):
        np.testing.assert_array_equal(r8[name], r16[name])
    np.testing.assert_array_equal(r8["B"], O.f64_to_e5m2_bits(r8["psi"].reshape(b, r, hkv, d).transpose(0, 2, 1, 3)))
    np.testing.assert_array_equal(r8["A"][:, :s], O.f64_to_e5m2_bits(r8["A_f64"]))


PINS = [pin_known_factors, pin_eckart_young, pin_exact_low_rank, pin_layouts, pin_fp8_equals_bf16_on_widened_inputs]


@pytest.mark.parametrize("pin", PINS, ids=[p.__name__ for p in PINS])
def test_pin(pin):
    pin(O.factorize_keys)


MUTANTS = [
    ("smallest-singular-values-kept", "v = vt[:r].copy()", "v = vt[-r:].copy()"),
    ("sign-convention-inverted", "sign = np.where(v[np.arange(r), lead] < 0.0, -1.0, 1.0)",
     "sign = np.where(v[np.arange(r), lead] < 0.0, 1.0, -1.0)"),
    ("sign-by-smallest-component", "lead = np.argmax(np.abs(v), axis=1)", "lead = np.argmin(np.abs(v), axis=1)"),
    ("sign-not-fixed", "v *= sign[:, None]", "v *= 1.0"),
    ("a-scaled-twice", "A64[bi] = K @ v.T", "A64[bi] = (K @ v.T) * sv[:r]"),
    ("a-is-left-vectors", "A64[bi] = K @ v.T", "A64[bi] = (K @ v.T) / sv[:r]"),
    ("b-head-split", "B = rnd(psi.reshape(b, r, h, d).transpose(0, 2, 1, 3))",
     "B = rnd(psi.reshape(b, r, d, h).transpose(0, 3, 1, 2))"),
    ("sigma-squared", "psi[bi], sigma[bi] = v, sv[:r]", "psi[bi], sigma[bi] = v, sv[:r] ** 2"),
    ("gram-instead-of-keys", "_, sv, vt = np.linalg.svd(K, full_matrices=False)",
     "_, sv, vt = np.linalg.svd(K.T @ K, full_matrices=False)"),
    ("a-not-rounded-to-storage", "A[:, :s] = rnd(A64)", "A[:, :s] = rnd(A64.astype(np.float16).astype(np.float64))"),
]


@pytest.mark.parametrize("name,old,new", MUTANTS, ids=[m[0] for m in MUTANTS])
def test_pins_catch_mutant(name, old, new):
    src = inspect.getsource(O.factorize_keys)
    assert src.count(old) == 1, f"mutant {name}: pattern not found"
    scope = dict(vars(O))
    exec(compile(src.replace(old, new), f"<mutant {name}>", "exec"), scope)
    mutant = scope["factorize_keys"]
    caught = False
    for pin in PINS:
        try:
            pin(mutant)
        except Exception:
            caught = True
            break
    assert caught, f"mutant '{name}' passed every pin"

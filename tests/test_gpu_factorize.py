"""shadowkv_factorize_keys (first line of the pre-filling algorithm, A, B <- SVD(K)) against the oracle's LAPACK
SVD on the same stored keys (-m gpu).  What an SVD fixes uniquely is compared: singular values, the right singular
vectors under the sign convention (their gaps are healthy in these workloads), B and A to one unit in the last place
of the storage type, and the optimal reconstruction error."""
import numpy as np
import pytest
import torch

from oracle import shadowkv_oracle as O
from paper_2410_21465_amd import shadowkv as S
from workloads import Workload, generate

import parity_util as PU

pytestmark = pytest.mark.gpu


def _wl(name, **kw):
    base = dict(batch=2, n_q_heads=4, n_kv_heads=2, head_dim=64, ctx_len=2048, chunk_size=8, rank=32,
                n_outlier_chunks=2, topk_chunks=8, local_len=4, seed=41, n_queries=1)
    base.update(kw)
    return Workload(name, **base)


CASES = [
    (_wl("svd-d64x2"), 0),
    (_wl("svd-d96x2", head_dim=96, rank=40, ctx_len=1536, chunk_size=6), 0),
    (_wl("svd-d128x2-r64", head_dim=128, rank=64, ctx_len=4096, batch=1), 0),
    (_wl("svd-d64x3-ragged", n_q_heads=3, n_kv_heads=3, rank=24, ctx_len=1001 * 3, chunk_size=3), 0),
    (_wl("svd-fp8", head_dim=128, rank=48, ctx_len=2048), 1),
    # key widths above 1024 and above 3072 take the other two orthogonalisation paths
    (_wl("svd-wide-2048", batch=1, n_q_heads=16, n_kv_heads=16, head_dim=128, rank=64, ctx_len=4096), 0),
    (_wl("svd-wide-4096", batch=1, n_q_heads=32, n_kv_heads=32, head_dim=128, rank=32, ctx_len=2048), 0),
]


def ulp_distance(a, b, kd):
    """Distance in units of the last place between stored values (sign-magnitude codes mapped to a line)."""
    top = 0x80 if kd else 0x8000
    def line(x):
        x = x.astype(np.int64)
        return np.where(x & top, -(x & (top - 1)), x & (top - 1))
    return np.abs(line(a) - line(b))


@pytest.mark.parametrize("wl,kd", CASES, ids=[c[0].name for c in CASES])
def test_factors_match_the_svd(wl, kd):
    print(f"\n[case] kv_dtype {kd} {wl}", flush=True)
    t = generate(wl, device="cuda", want_prefill=False, want_k_pre=True)
    k_pre = t["k_pre"].to(torch.float8_e5m2) if kd else t["k_pre"]
    op = PU.oracle_params(wl, kv_dtype=kd)
    ref = O.factorize_keys(op, PU.to_bits(k_pre, kd))
    gp = S.Params.from_workload(wl, kv_dtype=kd)
    got = S.factorize_keys(gp, k_pre, want_vectors=True)
    torch.cuda.synchronize()
    sig, psi = got["sigma"].cpu().numpy(), got["psi"].cpu().numpy()
    r = wl.rank
    # singular values
    np.testing.assert_allclose(sig, ref["sigma"], rtol=1e-9, atol=0)
    # right singular vectors: unit, orthogonal, and equal to the oracle's (relative gaps of a few per cent)
    for bi in range(wl.batch):
        gram = psi[bi] @ psi[bi].T
        assert np.abs(gram - np.eye(r)).max() < 1e-12
    gaps = np.abs(np.diff(ref["sigma"] ** 2, axis=1)).min() / (ref["sigma"][:, :1] ** 2).max()
    print(f"[svd] smallest eigenvalue gap / lambda_1 = {gaps:.2e}; max |psi - psi_ref| = {np.abs(psi - ref['psi']).max():.2e}", flush=True)
    assert np.abs(psi - ref["psi"]).max() < 1e-7
    # B, A: equal to the oracle's roundings except where the fp64 values straddle a rounding boundary
    gB, gA = PU.to_bits(got["B"], kd), PU.to_bits(got["A"], kd)
    dB, dA = ulp_distance(gB, ref["B"], kd), ulp_distance(gA[:, :wl.ctx_len], ref["A"][:, :wl.ctx_len], kd)
    assert dB.max() <= 1 and (dB > 0).mean() < 1e-3, (dB.max(), (dB > 0).mean())
    assert dA.max() <= 1 and (dA > 0).mean() < 1e-3, (dA.max(), (dA > 0).mean())
    # Eckart-Young: the captured energy is the sum of the r largest eigenvalues of K^T K
    K = PU.kv_to_f64(PU.to_bits(k_pre, kd))
    for bi in range(wl.batch):
        lam = np.linalg.eigvalsh(K[bi].T @ K[bi])[::-1]
        captured = np.linalg.norm(K[bi] @ psi[bi].T) ** 2
        assert abs(captured - lam[:r].sum()) <= 1e-10 * lam[:r].sum()


def test_factors_feed_the_decode_step():
    """The factors of the library's own SVD drive a decode step that matches the oracle run on the same factors."""
    wl = _wl("svd-then-decode", head_dim=128, n_q_heads=8, rank=64, ctx_len=4096, topk_chunks=24, n_outlier_chunks=4)
    t = generate(wl, device="cuda", want_k_pre=True)
    gp = S.Params.from_workload(wl)
    f = S.factorize_keys(gp, t["k_pre"])
    torch.cuda.synchronize()
    t["A"], t["B"] = f["A"], f["B"]
    ref_b, _ = PU.run_build_parity(wl, t)
    stats, _, _ = PU.run_decode_parity(wl, t, ref_b, qi=0)
    print(f"[decode] on device-made factors: {stats}", flush=True)
    # and the rebuilt keys approximate the true ones as well as the rank allows
    K = PU.kv_to_f64(PU.to_bits(t["k_pre"]))
    rec = np.einsum("bsr,brx->bsx", PU.kv_to_f64(PU.to_bits(f["A"])),
                    PU.kv_to_f64(PU.to_bits(f["B"])).transpose(0, 2, 1, 3).reshape(wl.batch, wl.rank, -1))
    for bi in range(wl.batch):
        lam = np.linalg.eigvalsh(K[bi].T @ K[bi])[::-1]
        opt = np.sqrt(max(lam[wl.rank:].sum(), 0.0))
        err = np.linalg.norm(K[bi] - rec[bi])
        assert err <= opt * 1.05 + 2e-3 * np.linalg.norm(K[bi]), (err, opt)   # bf16 rounding of A and B on top of the optimum


def test_rejects_bad_arguments():
    wl = _wl("svd-bad")
    p = S.Params.from_workload(wl, rank=136)           # above the key width 128
    with pytest.raises((S.ShadowKVError, ValueError)):
        S.factorize_keys(p, torch.zeros(wl.batch, wl.ctx_len, 128, dtype=torch.bfloat16, device="cuda"))


@pytest.mark.timeout(900)
@pytest.mark.parametrize("name,kd", [("c3-hbm", 0), ("c5", 0), ("c4", 0), ("c2", 1)])
def test_full_size_sequence_by_properties(name, kd):
    """One sequence of a benchmark workload at full length (c3: 128K tokens x 1024, c5: 128K x 3072, c4: 1M x 256; c2
    with FP8 keys), r = 160: the LAPACK SVD of such a matrix is out of reach of the test budget, so what holds at any
    size is checked against fp64 numpy on the same keys: orthonormal right singular vectors, Ritz residuals at rounding level (K^T K psi = sigma^2 psi), the captured
    energy equal to the sum of the 160 largest eigenvalues of the Gram matrix (Eckart-Young), and sampled rows of A and
    all of B equal to the roundings of K psi and psi."""
    from workloads import CONFIGS
    wl = CONFIGS[name].scaled(batch=1, n_queries=1, value_location="hbm")
    print(f"\n[case] kv_dtype {kd} {wl}", flush=True)
    t = generate(wl, device="cuda", want_prefill=False, want_k_pre=True)
    k_pre = t["k_pre"].to(torch.float8_e5m2) if kd else t["k_pre"]
    gp = S.Params.from_workload(wl, kv_dtype=kd)
    got = S.factorize_keys(gp, k_pre, want_vectors=True)
    torch.cuda.synchronize()
    psi, sig = got["psi"][0].cpu().numpy(), got["sigma"][0].cpu().numpy()
    K = PU.kv_to_f64(PU.to_bits(k_pre, kd))[0]
    r = wl.rank
    assert np.abs(psi @ psi.T - np.eye(r)).max() < 1e-12
    G = K.T @ K
    lam = np.linalg.eigvalsh(G)[::-1]
    np.testing.assert_allclose(sig ** 2, lam[:r], rtol=1e-9)
    resid = np.abs(psi @ G - (sig ** 2)[:, None] * psi).max()
    print(f"[svd] {name}: max Ritz residual {resid:.3e} (lambda_1 = {lam[0]:.3e}, lambda_r = {lam[r - 1]:.3e})", flush=True)
    assert resid <= 1e-9 * lam[0]
    captured = (sig ** 2).sum()
    assert abs(captured - lam[:r].sum()) <= 1e-10 * lam[:r].sum()
    lead = np.argmax(np.abs(psi), axis=1)
    assert np.all(psi[np.arange(r), lead] > 0)
    np.testing.assert_array_equal(PU.to_bits(got["B"], kd)[0],
                                  PU.kv_round(psi.reshape(r, wl.n_kv_heads, wl.head_dim).transpose(1, 0, 2), kd))
    rows = np.random.default_rng(0).choice(wl.ctx_len, size=512, replace=False)
    want = PU.kv_round(K[rows] @ psi.T, kd)
    gA = PU.to_bits(got["A"], kd)[0][rows]
    diff = gA != want
    assert diff.mean() < 1e-3 and ulp_distance(gA, want, kd).max() <= 1


def test_degenerate_keys_give_finite_factors():
    """Keys of rank 8 factored at rank 16, and all-zero keys: no NaN or Inf anywhere, the spare singular values are
    zero, and A B still reconstructs the keys (up to the rounding of the factors)."""
    wl = _wl("svd-degenerate", batch=2, rank=16, ctx_len=1024)
    D = wl.n_kv_heads * wl.head_dim
    gen = torch.Generator(device="cuda").manual_seed(5)
    left = torch.randn(wl.ctx_len, 8, generator=gen, device="cuda")
    right = torch.randn(8, D, generator=gen, device="cuda")
    k = torch.zeros(2, wl.ctx_len, D, dtype=torch.bfloat16, device="cuda")
    k[0] = (left @ right).to(torch.bfloat16)                 # rounding adds a little full-rank noise at the 2^-9 level
    gp = S.Params.from_workload(wl)
    got = S.factorize_keys(gp, k, want_vectors=True)
    torch.cuda.synchronize()
    for name in ("psi", "sigma"):
        assert torch.isfinite(got[name]).all(), name
    A, B = got["A"].float(), got["B"].float()
    assert torch.isfinite(A).all() and torch.isfinite(B).all()
    sig = got["sigma"].cpu().numpy()
    assert np.all(sig[1] == 0.0) and not A[1].any()
    assert sig[0, 7] > 50 * sig[0, 8]                        # eight real directions, then the rounding noise
    rec = torch.einsum("sr,rx->sx", A[0], B[0].permute(1, 0, 2).reshape(wl.rank, D))
    err = (rec - k[0].float()).norm() / k[0].float().norm()
    assert err < 1e-2, float(err)

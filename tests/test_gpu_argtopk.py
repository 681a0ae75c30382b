"""The selection primitive on its own (shadowkv_argtopk) against a stable sort in numpy: exact for every fp64
input, ties to the lower index -- including values closer together than the coarse key the search runs on first."""
import numpy as np
import pytest
import torch

from paper_2410_21465_amd import shadowkv as S

pytestmark = pytest.mark.gpu


def reference(x: np.ndarray, k: int, largest: bool) -> np.ndarray:
    key = -x if largest else x
    key = key + 0.0                                  # -0.0 and +0.0 are the same score
    order = np.argsort(key, axis=1, kind="stable")[:, :k]
    return np.sort(order, axis=1).astype(np.int32)


def check(x: np.ndarray, k: int, largest: bool = True):
    got = S.argtopk(torch.from_numpy(np.ascontiguousarray(x)).cuda(), k, largest).cpu().numpy()
    np.testing.assert_array_equal(got, reference(x, k, largest))


@pytest.mark.parametrize("n,k", [(1, 1), (7, 7), (100, 3), (2048, 256), (2049, 256), (5000, 64), (16336, 256),
                                 (16336, 1), (40000, 256), (6000, 4096), (12000, 8192), (131072, 48)])
@pytest.mark.parametrize("largest", [True, False])
def test_random_scores(n, k, largest):
    rng = np.random.default_rng(n * 31 + k)
    check(rng.standard_normal((3, n)) * 5.0 - 8.0, k, largest)


def test_scores_closer_than_the_coarse_key():
    """Log-probability-like scores in (-20, 0] with clusters whose members differ by 1e-14 ... 1e-16: the coarse
    key (score - 1024, 2^-42 apart) cannot tell them apart, the exact keys must."""
    rng = np.random.default_rng(5)
    n, k = 6000, 256
    x = -rng.random((4, n)) * 20.0
    for u in range(4):
        centre = -3.0 - u                              # put a cluster right at the selection boundary
        idx = rng.choice(n, 600, replace=False)
        x[u, idx] = centre + rng.integers(-40, 41, 600) * 2.0 ** -50
        x[u, rng.choice(n, 100, replace=False)] = -0.5 * rng.random(100)       # and ~100 clear winners
    check(x, k, True)
    check(x, k, False)
    check(x, 100 + 300, True)                          # boundary inside the cluster


def test_many_exact_duplicates_and_special_values():
    rng = np.random.default_rng(6)
    n = 9000
    x = rng.integers(-3, 4, (3, n)).astype(np.float64)         # seven distinct values
    check(x, 500, True)
    check(x, 500, False)
    x[0, ::7] = -np.inf
    x[1, ::5] = np.inf
    x[2, ::3] = -0.0
    x[2, 1::3] = 0.0
    check(x, 2000, True)
    check(x, 2000, False)
    y = rng.standard_normal((2, n)) * 1e-300                  # denormal territory
    check(y, 77, True)
    z = rng.standard_normal((2, n)) * 1e300
    check(z, 77, False)


def test_cosine_like_scores_near_one():
    rng = np.random.default_rng(7)
    x = 1.0 - rng.integers(0, 2000, (2, 16384)) * 2.0 ** -53      # values within a few hundred ulps of 1
    check(x, 48, False)
    check(x, 48, True)


def test_rejects_bad_sizes():
    x = torch.zeros(2, 10, dtype=torch.float64, device="cuda")
    with pytest.raises(S.ShadowKVError):
        S.argtopk(x, 11)
    with pytest.raises(S.ShadowKVError):
        S.argtopk(x, 0)

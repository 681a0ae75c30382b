"""Seeded sweep over randomly drawn shapes (head dims, ragged chunk sizes, group sizes, ranks, budgets, windows,
store locations, cache sizes): build, plain decode and two cached decode steps against the oracle."""
import numpy as np
import pytest
import torch

from oracle import shadowkv_oracle as O
from paper_2410_21465_amd import shadowkv as S
from workloads import Workload, generate, query_sequence, to_fp8_storage

import parity_util as PU

pytestmark = pytest.mark.gpu


def draw_shape(seed: int) -> Workload:
    if seed >= 100:
        return draw_shape_large_group(seed)
    rng = np.random.default_rng(1000 + seed)
    d = int(rng.choice([64, 96, 128]))
    hkv = int(rng.choice([1, 2, 3, 4]))
    G = int(rng.choice([1, 2, 3, 4, 6, 8]))
    c = int(rng.choice([1, 2, 3, 4, 5, 8, 8, 8, 12, 16]))
    n_ch = int(rng.integers(40, 700))
    o = int(rng.integers(0, min(12, n_ch // 4)))
    k = int(rng.integers(1, min(n_ch - o, 96)))
    D = hkv * d
    r = int(min(D, 8 * rng.integers(1, 25)))
    return Workload(name=f"rand{seed}", batch=int(rng.choice([1, 2, 3])), n_q_heads=hkv * G, n_kv_heads=hkv, head_dim=d,
                    ctx_len=n_ch * c, chunk_size=c, rank=r, n_outlier_chunks=o, topk_chunks=k,
                    local_len=int(rng.integers(0, 40)), rope_theta=float(rng.choice([1e4, 5e5])), seed=100 + seed,
                    value_location=str(rng.choice(["hbm", "host"])), n_queries=2)


def draw_shape_large_group(seed: int) -> Workload:
    """Shapes with 5 to 20 query heads per KV head (the scoring kernels for large groups, several head blocks per
    unit in the attention)."""
    rng = np.random.default_rng(5000 + seed)
    d = int(rng.choice([64, 96, 128]))
    hkv = int(rng.choice([1, 2, 3]))
    G = int(rng.choice([5, 6, 7, 8, 9, 12, 16, 20]))
    c = int(rng.choice([1, 2, 3, 4, 5, 8, 8, 8, 12, 16]))
    n_ch = int(rng.integers(40, 900))
    o = int(rng.integers(0, min(12, n_ch // 4)))
    k = int(rng.integers(1, min(n_ch - o, 96)))
    r = int(min(hkv * d, 8 * rng.integers(1, 25)))
    return Workload(name=f"rand{seed}", batch=int(rng.choice([1, 2, 3])), n_q_heads=hkv * G, n_kv_heads=hkv, head_dim=d,
                    ctx_len=n_ch * c, chunk_size=c, rank=r, n_outlier_chunks=o, topk_chunks=k,
                    local_len=int(rng.integers(0, 40)), rope_theta=float(rng.choice([1e4, 5e5])), seed=300 + seed,
                    value_location=str(rng.choice(["hbm", "host"])), n_queries=2)


# every shape with bf16 storage of the KV cache; every other one also with FP8 E5M2 storage (seeds 100 + ...)
@pytest.mark.parametrize("seed,kd", [(s, 0) for s in range(14)] + [(s, 1) for s in range(0, 14, 2)] + [(s, 1) for s in range(14, 20)]
                         + [(100 + s, s % 2) for s in range(8)],   # large head groups, alternating storage,
                         ids=lambda v: str(v))
def test_random_shape(seed, kd):
    wl = draw_shape(seed)
    print(f"\n[case] kv_dtype {kd} {wl}", flush=True)
    t = PU.draw(wl)
    if kd:
        t = to_fp8_storage(t)
    ref_b, _ = PU.run_build_parity(wl, t, kv_dtype=kd)
    stats, _, _ = PU.run_decode_parity(wl, t, ref_b, qi=0, check_keys=True, kv_dtype=kd)
    print(f"[decode] {wl.name}: {stats}", flush=True)
    # two cached steps with a cache a little larger than the budget
    rng = np.random.default_rng(2000 + seed)
    slots = wl.topk_chunks + int(rng.integers(0, 2 * wl.topk_chunks + 1))
    op = PU.oracle_params(wl, kv_dtype=kd)
    p = S.Params.from_workload(wl, kv_dtype=kd)
    dev = PU.kv_from_bits

    lm, ids = dev(ref_b["landmarks"]), torch.from_numpy(ref_b["landmark_chunk_ids"]).cuda()
    ko, vo = dev(ref_b["k_outlier"]), dev(ref_b["v_outlier"])
    cache = S.ValueCache(p, slots=slots)
    qs = query_sequence(wl, 2, 0.9)
    units, k = wl.batch * wl.n_kv_heads, wl.topk_chunks
    ocache, ostamps = -np.ones((units, slots), np.int32), None
    fixed = (PU.to_bits(t["A"], kd), PU.to_bits(t["B"], kd), ref_b["landmarks"], ref_b["landmark_chunk_ids"],
             ref_b["k_outlier"], ref_b["v_outlier"], PU.to_bits(t["k_local"], kd), PU.to_bits(t["v_local"], kd),
             PU.to_bits(t["v"], kd), t["pos_offset"].cpu().numpy())
    for step in range(2):
        out, sel, _ = S.decode_step_cached(p, qs[step], t["A"], t["B"], lm, ids, ko, vo, t["k_local"], t["v_local"], t["v"],
                                           cache, t["pos_offset"],
                                           side_stream=torch.cuda.Stream() if step == 1 else None)
        torch.cuda.synchronize()
        ref = O.decode_step(op, PU.to_bits(qs[step]), *fixed, diagnostics=True)
        g_ids = sel.cpu().numpy().reshape(units, k)
        lid, z2 = ref_b["landmark_chunk_ids"].reshape(units, -1), ref["z2"].reshape(units, -1)
        ties = PU.check_index_sets(g_ids, ref["chunk_ids"].reshape(units, k),
                                   lambda u, c_ids: z2[u, np.searchsorted(lid[u], c_ids)], "top-k chunks (cached)")
        model = O.cache_update(g_ids, ocache, ostamps)       # the cache follows the ids the GPU chose
        np.testing.assert_array_equal(cache.chunk_ids.cpu().numpy().reshape(units, slots), model["cache_ids"])
        np.testing.assert_array_equal(cache.miss_count.cpu().numpy().reshape(units), model["n_miss"])
        ocache, ostamps = model["cache_ids"], model["stamps"]
        if ties == 0:
            err = np.abs(out.float().cpu().numpy().astype(np.float64) - O.bits_to_f64(ref["out"]))
            assert err.max() <= PU.OUT_MAX_ABS and err.mean() <= PU.OUT_MEAN_ABS, (step, err.max(), err.mean())

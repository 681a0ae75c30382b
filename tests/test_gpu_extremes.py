"""Parity at the edges of the accepted parameter ranges (largest rank, chunk, group, outlier count, budget;
smallest rank and budget), each on a context small enough for the oracle to finish in seconds."""
import numpy as np
import pytest
import torch

from oracle import shadowkv_oracle as O
from paper_2410_21465_amd import shadowkv as S
from workloads import Workload, generate, query_sequence

import parity_util as PU

pytestmark = pytest.mark.gpu


def wl(name, **kw):
    base = dict(batch=1, n_q_heads=8, n_kv_heads=2, head_dim=128, ctx_len=2048, chunk_size=8, rank=32,
                n_outlier_chunks=4, topk_chunks=24, local_len=5, rope_theta=5e5, seed=41, n_queries=1)
    base.update(kw)
    return Workload(name, **base)


CASES = [
    wl("rank-256", rank=256, topk_chunks=40),                                  # 8 rank steps, B^T above 48 KB of LDS
    wl("rank-8", rank=8),
    wl("rank-200-ragged", rank=200, topk_chunks=33),                           # last rank step partly backed
    wl("chunk-64", chunk_size=64, ctx_len=64 * 48, topk_chunks=6, n_outlier_chunks=2),
    wl("chunk-3", chunk_size=3, ctx_len=3 * 700, topk_chunks=50, n_outlier_chunks=7, head_dim=64, rank=24),
    wl("group-64", n_q_heads=64, n_kv_heads=1, head_dim=64, rank=16, ctx_len=1024, topk_chunks=9),
    wl("group-5", n_q_heads=10, n_kv_heads=2, head_dim=96, rank=24, ctx_len=1536, topk_chunks=11, rope_theta=1e4),
    wl("outliers-1024", chunk_size=2, ctx_len=2 * 1500, n_outlier_chunks=1024, topk_chunks=20, head_dim=64, rank=16),
    wl("window-300", local_len=300, n_outlier_chunks=0, topk_chunks=8),
    wl("budget-1", topk_chunks=1),
    wl("budget-4096", chunk_size=1, ctx_len=6000, n_outlier_chunks=3, topk_chunks=4096, head_dim=64, rank=16,
       n_q_heads=2, n_kv_heads=1),
    wl("three-level-select", chunk_size=1, ctx_len=40000, n_outlier_chunks=3, topk_chunks=256, head_dim=64, rank=16,
       n_q_heads=2, n_kv_heads=1),                                            # 20 slices -> 5120 survivors -> groups
    wl("batch-40-units-320", batch=40, n_q_heads=8, n_kv_heads=8, head_dim=64, rank=64, ctx_len=512, topk_chunks=10,
       n_outlier_chunks=2),
]


@pytest.mark.parametrize("w", CASES, ids=[c.name for c in CASES])
def test_extreme_parameters(w):
    print(f"\n[case] {w}", flush=True)
    t = PU.draw(w)
    ref_b, _ = PU.run_build_parity(w, t)
    stats, _, _ = PU.run_decode_parity(w, t, ref_b, qi=0, check_keys=True)
    print(f"[decode] {w.name}: {stats}", flush=True)
    stats, _, _ = PU.run_decode_parity(w, t, ref_b, qi=0, check_keys=False, flags=S.FLAG_STAGE_VALUES)


def test_chunk_cache_at_its_largest_budget():
    """k = 8192 slots per unit (the cached step's limit; the index-scan kernel needs more than 48 KB of LDS)."""
    w = wl("cache-8192", chunk_size=1, ctx_len=12000, n_outlier_chunks=2, topk_chunks=8192, head_dim=64, rank=16,
           n_q_heads=2, n_kv_heads=1, value_location="host", seed=42)
    t = generate(w, device="cuda")
    op = PU.oracle_params(w)
    ref_b = O.build_landmarks(op, PU.to_bits(t["k_rope"]), PU.to_bits(t["v"]))
    p = S.Params.from_workload(w)

    def dev(bits):
        return torch.from_numpy(bits.view(np.int16)).view(torch.bfloat16).cuda()

    lm, ids = dev(ref_b["landmarks"]), torch.from_numpy(ref_b["landmark_chunk_ids"]).cuda()
    ko, vo = dev(ref_b["k_outlier"]), dev(ref_b["v_outlier"])
    cache = S.ValueCache(p)
    qs = query_sequence(w, 3, 0.9)
    ocache = -np.ones((1, w.topk_chunks), np.int32)
    for step in range(3):
        out, sel, _ = S.decode_step_cached(p, qs[step], t["A"], t["B"], lm, ids, ko, vo, t["k_local"], t["v_local"],
                                           t["v"], cache, t["pos_offset"])
        torch.cuda.synchronize()
        ref = O.decode_step(op, PU.to_bits(qs[step]), PU.to_bits(t["A"]), PU.to_bits(t["B"]), ref_b["landmarks"],
                            ref_b["landmark_chunk_ids"], ref_b["k_outlier"], ref_b["v_outlier"], PU.to_bits(t["k_local"]),
                            PU.to_bits(t["v_local"]), PU.to_bits(t["v"]), t["pos_offset"].cpu().numpy(), diagnostics=False)
        want = np.sort(ref["chunk_ids"].reshape(1, -1), axis=1)
        np.testing.assert_array_equal(sel.cpu().numpy().reshape(1, -1), want)
        model = O.cache_update(want, ocache)
        np.testing.assert_array_equal(cache.chunk_ids.cpu().numpy().reshape(1, -1), model["cache_ids"])
        np.testing.assert_array_equal(cache.miss_count.cpu().numpy().reshape(1), model["n_miss"])
        ocache = model["cache_ids"]
        err = np.abs(out.float().cpu().numpy().astype(np.float64) - O.bits_to_f64(ref["out"]))
        assert err.max() <= PU.OUT_MAX_ABS and err.mean() <= PU.OUT_MEAN_ABS
    p_big = S.Params.from_workload(wl("too-big", chunk_size=1, ctx_len=12000, n_outlier_chunks=2, topk_chunks=8200,
                                      head_dim=64, rank=16, n_q_heads=2, n_kv_heads=1))
    with pytest.raises(S.ShadowKVError):
        S.decode_step_cached(p_big, qs[0], t["A"], t["B"], lm, ids, ko, vo, t["k_local"], t["v_local"], t["v"], cache,
                             t["pos_offset"])

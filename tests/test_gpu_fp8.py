"""FP8 (E5M2) storage of the KV cache (section "Precision Sensitivity"): the HIP library against the CPU
oracle on the same bytes -- pre-filling step (landmarks rounded once to E5M2, outliers), decode step
(in-place, staged, host store, chunk cache), append of generated tokens, and the two conversions
(all 256 codes in, rounding of sums out) -- to the same bar as the bf16 mode (-m gpu)."""
import numpy as np
import pytest
import torch

from oracle import shadowkv_oracle as O
from paper_2410_21465_amd import shadowkv as S
from workloads import Workload, generate, generated_chunk, to_fp8_storage, with_capacity

import parity_util as PU

pytestmark = pytest.mark.gpu
FP8 = S.KV_FP8_E5M2


def small(name, **kw):
    base = dict(batch=2, n_q_heads=8, n_kv_heads=2, head_dim=128, ctx_len=4096, chunk_size=8, rank=32,
                n_outlier_chunks=4, topk_chunks=24, local_len=5, rope_theta=5e5, seed=11, n_queries=2)
    base.update(kw)
    return Workload(name, **base)


CASES = [
    small("fp8-tiny-d64", head_dim=64, ctx_len=512, chunk_size=4, rank=16, topk_chunks=5, n_outlier_chunks=3, local_len=3),
    small("fp8-d128-g4"),
    small("fp8-d96-mha", n_q_heads=4, n_kv_heads=4, head_dim=96, ctx_len=2048, rank=40, topk_chunks=17,
          n_outlier_chunks=2, rope_theta=1e4),
    small("fp8-g16", batch=1, n_q_heads=32, n_kv_heads=2, ctx_len=8192, rank=64, topk_chunks=40),
    small("fp8-g8", batch=1, n_q_heads=16, n_kv_heads=2, ctx_len=8192, rank=64, topk_chunks=40),
    small("fp8-g3-odd", batch=1, n_q_heads=6, n_kv_heads=2, head_dim=64, ctx_len=1536, chunk_size=6, rank=24,
          topk_chunks=9, n_outlier_chunks=1, local_len=1),
    small("fp8-d96-c3", batch=1, n_q_heads=2, n_kv_heads=2, head_dim=96, ctx_len=999, chunk_size=3, rank=8,
          topk_chunks=21, n_outlier_chunks=2, local_len=2, rope_theta=1e4),
    small("fp8-no-outliers-no-local", n_outlier_chunks=0, local_len=0, ctx_len=1024, topk_chunks=7),
    small("fp8-chunk1", batch=1, chunk_size=1, ctx_len=700, topk_chunks=33, n_outlier_chunks=0, rank=16),
    small("fp8-chunk16", batch=1, chunk_size=16, ctx_len=4096, topk_chunks=12, n_outlier_chunks=3, rank=48),
    small("fp8-rank160-k256", batch=1, n_q_heads=8, n_kv_heads=2, ctx_len=32768, rank=160, topk_chunks=256,
          n_outlier_chunks=48, local_len=32),
    small("fp8-rank256", batch=1, n_q_heads=4, n_kv_heads=2, ctx_len=2048, rank=256, topk_chunks=30),
]


def draw(wl):
    return to_fp8_storage(generate(wl, device="cuda"))


@pytest.mark.parametrize("wl", CASES, ids=[c.name for c in CASES])
def test_build_and_decode_small(wl):
    print(f"\n[case] {wl}", flush=True)
    t = draw(wl)
    assert t["A"].dtype == torch.float8_e5m2 and t["q_pool"].dtype == torch.bfloat16
    ref_b, _ = PU.run_build_parity(wl, t, kv_dtype=FP8)
    for qi in range(wl.n_queries):
        stats, _, _ = PU.run_decode_parity(wl, t, ref_b, qi=qi, check_keys=(qi == 0), kv_dtype=FP8)
        print(f"[decode] {wl.name} q{qi}: {stats}", flush=True)


@pytest.mark.parametrize("loc,flags", [("host", 0), ("hbm", S.FLAG_STAGE_VALUES)])
def test_gathered_values_host_store_and_staging(loc, flags):
    wl = small("fp8-gather", value_location=loc, ctx_len=8192, topk_chunks=48)
    t = draw(wl)
    if loc == "host":
        assert t["v"].device.type == "cpu" and t["v"].is_pinned() and t["v"].dtype == torch.float8_e5m2
    ref_b, _ = PU.run_build_parity(wl, t, kv_dtype=FP8)
    s1, _, (o1, i1, _) = PU.run_decode_parity(wl, t, ref_b, side_stream=True, flags=flags, kv_dtype=FP8)
    s2, _, (o2, i2, _) = PU.run_decode_parity(wl, t, ref_b, side_stream=False, flags=flags, kv_dtype=FP8)
    assert torch.equal(o1, o2) and torch.equal(i1, i2)
    print(f"[decode] fp8 {loc}: {s1}", flush=True)


def _state(wl, t, cap=0):
    """Oracle landmarks / outliers for the workload, on both sides."""
    op = PU.oracle_params(wl, kv_dtype=FP8)
    op.ctx_capacity = cap
    ref = O.build_landmarks(op, PU.to_bits(t["k_rope"], FP8), PU.to_bits(t["v"], FP8))
    g = {"landmarks": PU.kv_from_bits(ref["landmarks"]), "ids": torch.from_numpy(ref["landmark_chunk_ids"]).cuda(),
         "k_outlier": PU.kv_from_bits(ref["k_outlier"]), "v_outlier": PU.kv_from_bits(ref["v_outlier"])}
    return op, ref, g


def test_chunk_cache_steps_match_oracle():
    wl = small("fp8-cache", value_location="host", ctx_len=8192, topk_chunks=48, n_queries=6)
    t = draw(wl)
    op, ref, g = _state(wl, t)
    gp = S.Params.from_workload(wl, kv_dtype=FP8)
    cache = S.ValueCache(gp, slots=64)
    assert cache.values.dtype == torch.float8_e5m2
    units, k = wl.batch * wl.n_kv_heads, wl.topk_chunks
    ocache, stamps = -np.ones((units, 64), np.int32), None
    side = torch.cuda.Stream()
    for qi in [0, 1, 1, 2, 0, 3]:
        q = t["q_pool"][qi]
        want = O.decode_step(op, PU.to_bits(q), PU.to_bits(t["A"], FP8), PU.to_bits(t["B"], FP8), ref["landmarks"],
                             ref["landmark_chunk_ids"], ref["k_outlier"], ref["v_outlier"], PU.to_bits(t["k_local"], FP8),
                             PU.to_bits(t["v_local"], FP8), PU.to_bits(t["v"], FP8), t["pos_offset"].cpu().numpy(),
                             diagnostics=False)
        out, ids, _ = S.decode_step_cached(gp, q, t["A"], t["B"], g["landmarks"], g["ids"], g["k_outlier"], g["v_outlier"],
                                           t["k_local"], t["v_local"], t["v"], cache, t["pos_offset"], side_stream=side)
        torch.cuda.synchronize()
        sel = np.sort(want["chunk_ids"].reshape(units, k), axis=1)
        np.testing.assert_array_equal(ids.cpu().numpy().reshape(units, k), sel)
        model = O.cache_update(sel, ocache, stamps)
        ocache, stamps = model["cache_ids"], model["stamps"]
        np.testing.assert_array_equal(cache.chunk_ids.cpu().numpy().reshape(units, 64), ocache)
        np.testing.assert_array_equal(cache.miss_count.cpu().numpy().reshape(units), model["n_miss"])
        # every cached chunk holds exactly the store's bytes
        vb = PU.to_bits(t["v"], FP8).reshape(units, -1, wl.chunk_size, wl.head_dim)
        cb = PU.to_bits(cache.values, FP8).reshape(units, 64, wl.chunk_size, wl.head_dim)
        for u in range(units):
            held = ocache[u] >= 0
            np.testing.assert_array_equal(cb[u][held], vb[u, ocache[u][held]])
        err = np.abs(out.float().cpu().numpy().astype(np.float64) - O.bits_to_f64(want["out"]))
        assert err.max() <= PU.OUT_MAX_ABS and err.mean() <= PU.OUT_MEAN_ABS, (err.max(), err.mean())


@pytest.mark.parametrize("loc,d,c", [("hbm", 128, 8), ("host", 128, 8), ("hbm", 96, 4), ("hbm", 64, 5)])
def test_appended_chunks_match_oracle(loc, d, c):
    wl = small("fp8-grow", value_location=loc, head_dim=d, chunk_size=c, n_q_heads=8 if d == 128 else 4,
               n_kv_heads=2 if d == 128 else 4, rope_theta=5e5 if d == 128 else 1e4, ctx_len=256 * c, rank=64,
               topk_chunks=40, n_outlier_chunks=5, local_len=7, seed=33, n_queries=4)
    s0, n_app = wl.ctx_len, 3
    cap = s0 + (n_app + 1) * c
    t16 = with_capacity(generate(wl, device="cuda"), wl, cap)
    t = to_fp8_storage(t16)
    op, ref, g = _state(wl, t, cap)
    state = {"A": PU.to_bits(t["A"], FP8).copy(), "v": PU.to_bits(t["v"], FP8).copy(), "landmarks": ref["landmarks"],
             "ids": ref["landmark_chunk_ids"]}
    s = s0
    units, k = wl.batch * wl.n_kv_heads, wl.topk_chunks
    for i in range(n_app):
        k_pre, k_rope, v = (x.to(torch.float8_e5m2) for x in generated_chunk(wl, t16, i))
        gp = S.Params.from_workload(wl, ctx_len=s, ctx_capacity=cap, kv_dtype=FP8)
        op.ctx_len = s
        S.append_chunk(gp, k_pre, k_rope, v, t["B"], t["A"], g["landmarks"], g["ids"], t["v"])
        torch.cuda.synchronize()
        O.append_chunk(op, PU.to_bits(k_pre, FP8), PU.to_bits(k_rope, FP8), PU.to_bits(v, FP8), PU.to_bits(t["B"], FP8),
                       state["A"], state["landmarks"], state["ids"], state["v"])
        n_c = s // c - wl.n_outlier_chunks
        np.testing.assert_array_equal(PU.to_bits(g["landmarks"], FP8)[:, :, :n_c + 1], state["landmarks"][:, :, :n_c + 1])
        np.testing.assert_array_equal(g["ids"].cpu().numpy()[:, :, :n_c + 1], state["ids"][:, :, :n_c + 1])
        np.testing.assert_array_equal(PU.to_bits(t["v"], FP8)[:, :, :s + c], state["v"][:, :, :s + c])
        ga, wa = PU.to_bits(t["A"], FP8)[:, s:s + c], state["A"][:, s:s + c]
        diff = ga != wa
        if diff.any():   # different summation order in fp64: a rounding boundary can flip the last bit
            assert diff.mean() < 1e-3 and np.all(np.abs(ga.astype(np.int32) - wa.astype(np.int32))[diff] == 1)
            t["A"][:, s:s + c] = PU.kv_from_bits(wa)
        s += c
        # a decode step on the grown context, pulled towards the new chunk
        op.ctx_len = s
        gp = S.Params.from_workload(wl, ctx_len=s, ctx_capacity=cap, kv_dtype=FP8)
        q = t["q_pool"][1 + i].clone()
        lm_new = g["landmarks"][:, :, n_c].float()                                  # [b, h_kv, d]
        q = (q.float() + 4.0 * lm_new.repeat_interleave(wl.group, dim=1) / lm_new.norm(dim=-1, keepdim=True)
             .repeat_interleave(wl.group, dim=1)).to(torch.bfloat16)
        want = O.decode_step(op, PU.to_bits(q), state["A"], PU.to_bits(t["B"], FP8), state["landmarks"], state["ids"],
                             ref["k_outlier"], ref["v_outlier"], PU.to_bits(t["k_local"], FP8), PU.to_bits(t["v_local"], FP8),
                             state["v"], t["pos_offset"].cpu().numpy(), diagnostics=False)
        out, ids, _ = S.decode_step(gp, q, t["A"], t["B"], g["landmarks"], g["ids"], g["k_outlier"], g["v_outlier"],
                                    t["k_local"], t["v_local"], t["v"], t["pos_offset"], side_stream=torch.cuda.Stream())
        torch.cuda.synchronize()
        np.testing.assert_array_equal(ids.cpu().numpy().reshape(units, k), np.sort(want["chunk_ids"].reshape(units, k), 1))
        assert (ids.cpu().numpy() == s // c - 1).any(), "the appended chunk was never selected"
        err = np.abs(out.float().cpu().numpy().astype(np.float64) - O.bits_to_f64(want["out"]))
        assert err.max() <= PU.OUT_MAX_ABS and err.mean() <= PU.OUT_MEAN_ABS, (err.max(), err.mean())


def test_every_code_is_widened_exactly():
    """Chunks of one token: the landmark of a chunk is its key, so all 248 finite codes (both zeros among them) must come
    back as the oracle says -- through the load, the widening, the fp64 mean and the rounding."""
    finite = np.array([b for b in range(256) if (b >> 2) & 31 != 31], dtype=np.uint8)
    d, s = 64, 256
    rng = np.random.default_rng(0)
    k = rng.choice(finite, size=(1, 1, s, d)).astype(np.uint8)
    k[0, 0, :len(finite), 0] = finite
    k[0, 0, :len(finite), 17] = finite[::-1]
    wl = Workload("codes", batch=1, n_q_heads=1, n_kv_heads=1, head_dim=d, ctx_len=s, chunk_size=1, rank=8,
                  n_outlier_chunks=0, topk_chunks=4, local_len=0)
    op = PU.oracle_params(wl, kv_dtype=FP8)
    ref = O.build_landmarks(op, k, None)
    got = S.build_landmarks(S.Params.from_workload(wl, kv_dtype=FP8), PU.kv_from_bits(k), None)
    torch.cuda.synchronize()
    np.testing.assert_array_equal(PU.to_bits(got["landmarks"], FP8), ref["landmarks"])
    same = (ref["landmarks"] == k) | ((k & 0x7F) == 0)     # a mean of one element is that element (-0 -> +0)
    assert same.all()


def test_rounding_of_sums_to_e5m2_matches_the_oracle():
    """Append with a 0/1 projection: every low-rank state is the sum of two or three stored values, drawn from the
    whole finite code range, so ties, carries into the next binade, overflow to infinity and subnormal results
    all occur; the bytes must equal the oracle's single rounding."""
    b, hkv, d, c, r = 2, 2, 64, 8, 40
    s, cap = 64, 128
    rng = np.random.default_rng(1)
    finite = np.array([x for x in range(256) if (x >> 2) & 31 != 31], dtype=np.uint8)
    near = np.array([x for x in range(256) if 8 <= ((x >> 2) & 31) <= 20], dtype=np.uint8)
    edge = np.array([x for x in range(256) if ((x >> 2) & 31) <= 2 or 28 <= ((x >> 2) & 31) <= 30], dtype=np.uint8)
    pick = rng.random((b, c, hkv * d))
    k_pre = np.where(pick < 0.4, rng.choice(finite, size=pick.shape),
                     np.where(pick < 0.7, rng.choice(edge, size=pick.shape), rng.choice(near, size=pick.shape))).astype(np.uint8)
    B = np.zeros((b, hkv, r, d), np.uint8)
    one = 0x3C
    for rho in range(r):
        B[:, rho % hkv, rho, (3 * rho) % d] = one
        B[:, (rho + 1) % hkv, rho, (3 * rho + 1) % d] = one
        if rho % 3 == 0:
            B[:, rho % hkv, rho, (3 * rho + 2) % d] = 0xBC      # minus one
    k_rope = rng.choice(near, size=(b, hkv, c, d)).astype(np.uint8)
    v = rng.choice(finite, size=(b, hkv, c, d)).astype(np.uint8)
    wl = Workload("sums", batch=b, n_q_heads=hkv, n_kv_heads=hkv, head_dim=d, ctx_len=s, chunk_size=c, rank=r,
                  n_outlier_chunks=1, topk_chunks=2, local_len=0)
    op = PU.oracle_params(wl, kv_dtype=FP8)
    op.ctx_capacity = cap
    nc_cap = cap // c - 1
    A = rng.choice(near, size=(b, cap, r)).astype(np.uint8)
    L = rng.choice(near, size=(b, hkv, nc_cap, d)).astype(np.uint8)
    ids = np.zeros((b, hkv, nc_cap), np.int32)
    store = rng.choice(near, size=(b, hkv, cap, d)).astype(np.uint8)
    gA, gL, gids, gstore = PU.kv_from_bits(A), PU.kv_from_bits(L), torch.from_numpy(ids).cuda(), PU.kv_from_bits(store)
    O.append_chunk(op, k_pre, k_rope, v, B, A, L, ids, store)
    S.append_chunk(S.Params.from_workload(wl, ctx_capacity=cap, kv_dtype=FP8), PU.kv_from_bits(k_pre), PU.kv_from_bits(k_rope),
                   PU.kv_from_bits(v), PU.kv_from_bits(B), gA, gL, gids, gstore)
    torch.cuda.synchronize()
    rows = A[:, s:s + c]
    assert (rows == 0x7C).sum() + (rows == 0xFC).sum() >= 4, "too few overflow cases drawn"
    assert ((rows & 0x7C) == 0).sum() >= 4, "too few subnormal / zero results drawn"
    np.testing.assert_array_equal(PU.to_bits(gA, FP8), A)
    np.testing.assert_array_equal(PU.to_bits(gL, FP8), L)
    np.testing.assert_array_equal(gids.cpu().numpy(), ids)
    np.testing.assert_array_equal(PU.to_bits(gstore, FP8), store)


def test_kv_dtype_is_validated():
    wl = small("bad")
    p = S.Params.from_workload(wl, kv_dtype=7)
    assert S.validate_params(p) == S.EINVAL
    p8, p16 = S.Params.from_workload(wl, kv_dtype=FP8), S.Params.from_workload(wl)
    p8s, p16s = (S.Params.from_workload(wl, kv_dtype=kd, flags=S.FLAG_STAGE_VALUES) for kd in (FP8, 0))
    rows = wl.batch * wl.n_kv_heads * wl.topk_chunks * wl.chunk_size * wl.head_dim
    assert S.decode_workspace_bytes(p16s) - S.decode_workspace_bytes(p8s) == rows   # staged values: 1 byte per element
    assert S.decode_workspace_bytes(p8) == S.decode_workspace_bytes(p16)

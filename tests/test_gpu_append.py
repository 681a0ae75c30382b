"""Context arrays with room to grow (ctx_capacity) and shadowkv_append_chunk against the oracle: the layout
changes nothing, appended chunks equal the oracle's (landmarks, ids, values bit-exact; rows of A to one bf16
ulp at most, almost all identical), and decode steps on the grown context keep parity -- also through the
chunk cache, which must stay valid across an append."""
import numpy as np
import pytest
import torch

from oracle import shadowkv_oracle as O
from paper_2410_21465_amd import shadowkv as S
from workloads import Workload, generate, generated_chunk, with_capacity
from parity_util import OUT_MAX_ABS, OUT_MEAN_ABS, to_bits

pytestmark = pytest.mark.gpu


def _wl(**kw):
    base = dict(name="grow", batch=2, n_q_heads=8, n_kv_heads=2, head_dim=128, ctx_len=2048, chunk_size=8, rank=64,
                n_outlier_chunks=5, topk_chunks=40, local_len=7, rope_theta=5e5, seed=31, n_queries=4)
    base.update(kw)
    return Workload(**base)


def _op(wl, s, cap):
    return O.OracleParams(wl.batch, wl.n_q_heads, wl.n_kv_heads, wl.head_dim, s, wl.chunk_size, wl.rank,
                          wl.n_outlier_chunks, wl.topk_chunks, wl.local_len, rope_theta=wl.rope_theta, ctx_capacity=cap)


def _bf16_dev(bits):
    return torch.from_numpy(bits.view(np.int16)).view(torch.bfloat16).cuda()


def _check_decode(wl, gp, op, q, t, g, ref_state, cache=None, ocache=None):
    """One GPU step (plain or cached) on the device state `g` against the oracle on `ref_state`."""
    units, k = wl.batch * wl.n_kv_heads, wl.topk_chunks
    ref = O.decode_step(op, to_bits(q), ref_state["A"], to_bits(t["B"]), ref_state["landmarks"], ref_state["ids"],
                        ref_state["k_outlier"], ref_state["v_outlier"], to_bits(t["k_local"]), to_bits(t["v_local"]),
                        ref_state["v"], t["pos_offset"].cpu().numpy(), diagnostics=False)
    args = (gp, q, g["A"], t["B"], g["landmarks"], g["ids"], g["k_outlier"], g["v_outlier"], t["k_local"],
            t["v_local"], g["v"])
    if cache is None:
        out, ids, _ = S.decode_step(*args, t["pos_offset"])
    else:
        out, ids, _ = S.decode_step_cached(*args, cache, t["pos_offset"])
    torch.cuda.synchronize()
    want = np.sort(ref["chunk_ids"].reshape(units, k), axis=1)
    np.testing.assert_array_equal(ids.cpu().numpy().reshape(units, k), want)
    err = np.abs(out.float().cpu().numpy().astype(np.float64) - O.bits_to_f64(ref["out"]))
    assert err.max() <= OUT_MAX_ABS and err.mean() <= OUT_MEAN_ABS, (err.max(), err.mean())
    if cache is not None:
        model = O.cache_update(want, ocache)
        np.testing.assert_array_equal(cache.chunk_ids.cpu().numpy().reshape(units, k), model["cache_ids"])
        np.testing.assert_array_equal(cache.miss_count.cpu().numpy().reshape(units), model["n_miss"])
        return want, model["cache_ids"]
    return want, None


@pytest.mark.parametrize("loc", ["hbm", "host"])
def test_layout_with_room_to_grow_matches_oracle(loc):
    wl = _wl(value_location=loc)
    s, c, cap = wl.ctx_len, wl.chunk_size, wl.ctx_len + 6 * wl.chunk_size
    t = with_capacity(generate(wl, device="cuda"), wl, cap)
    op = _op(wl, s, cap)
    ref = O.build_landmarks(op, to_bits(t["k_rope"]), to_bits(t["v"]))
    gp = S.Params.from_workload(wl, ctx_capacity=cap)
    got = S.build_landmarks(gp, t["k_rope"], t["v"])
    torch.cuda.synchronize()
    n_c = s // c - wl.n_outlier_chunks
    np.testing.assert_array_equal(to_bits(got["landmarks"])[:, :, :n_c], ref["landmarks"][:, :, :n_c])
    np.testing.assert_array_equal(got["landmark_chunk_ids"].cpu().numpy()[:, :, :n_c], ref["landmark_chunk_ids"][:, :, :n_c])
    np.testing.assert_array_equal(np.sort(got["outlier_chunk_ids"].cpu().numpy(), -1), np.sort(ref["outlier_chunk_ids"], -1))
    # decode on the oracle's landmarks / outliers
    g = {"A": t["A"], "v": t["v"], "landmarks": _bf16_dev(ref["landmarks"]),
         "ids": torch.from_numpy(ref["landmark_chunk_ids"]).cuda(), "k_outlier": _bf16_dev(ref["k_outlier"]),
         "v_outlier": _bf16_dev(ref["v_outlier"])}
    state = {"A": to_bits(t["A"]), "v": to_bits(t["v"]), "landmarks": ref["landmarks"], "ids": ref["landmark_chunk_ids"],
             "k_outlier": ref["k_outlier"], "v_outlier": ref["v_outlier"]}
    _check_decode(wl, gp, op, t["q_pool"][0], t, g, state)


@pytest.mark.parametrize("loc,d,c", [("hbm", 128, 8), ("host", 128, 8), ("hbm", 96, 4)])
def test_appended_chunks_match_oracle_and_decode_keeps_parity(loc, d, c):
    wl = _wl(value_location=loc, head_dim=d, chunk_size=c, n_q_heads=8 if d == 128 else 4, n_kv_heads=2 if d == 128 else 4,
             rope_theta=5e5 if d == 128 else 1e4, seed=32)
    s0, n_app = wl.ctx_len, 3
    cap = s0 + (n_app + 1) * c
    t = with_capacity(generate(wl, device="cuda"), wl, cap)
    ref = O.build_landmarks(_op(wl, s0, cap), to_bits(t["k_rope"]), to_bits(t["v"]))
    state = {"A": to_bits(t["A"]).copy(), "v": to_bits(t["v"]).copy(), "landmarks": ref["landmarks"],
             "ids": ref["landmark_chunk_ids"], "k_outlier": ref["k_outlier"], "v_outlier": ref["v_outlier"]}
    g = {"A": t["A"], "v": t["v"], "landmarks": _bf16_dev(ref["landmarks"]),
         "ids": torch.from_numpy(ref["landmark_chunk_ids"]).cuda(), "k_outlier": _bf16_dev(ref["k_outlier"]),
         "v_outlier": _bf16_dev(ref["v_outlier"])}
    units, k = wl.batch * wl.n_kv_heads, wl.topk_chunks
    cache = S.ValueCache(S.Params.from_workload(wl, ctx_capacity=cap))
    ocache = -np.ones((units, k), np.int32)
    s = s0
    _, ocache = _check_decode(wl, S.Params.from_workload(wl, ctx_capacity=cap), _op(wl, s, cap), t["q_pool"][0], t, g,
                              state, cache, ocache)
    for i in range(n_app):
        k_pre, k_rope, v = generated_chunk(wl, t, i)
        gp, op = S.Params.from_workload(wl, ctx_len=s, ctx_capacity=cap), _op(wl, s, cap)
        S.append_chunk(gp, k_pre, k_rope, v, t["B"], g["A"], g["landmarks"], g["ids"], g["v"])
        torch.cuda.synchronize()
        O.append_chunk(op, to_bits(k_pre), to_bits(k_rope), to_bits(v), to_bits(t["B"]), state["A"], state["landmarks"],
                       state["ids"], state["v"])
        n_c = s // c - wl.n_outlier_chunks
        np.testing.assert_array_equal(to_bits(g["landmarks"])[:, :, :n_c + 1], state["landmarks"][:, :, :n_c + 1])
        np.testing.assert_array_equal(g["ids"].cpu().numpy()[:, :, :n_c + 1], state["ids"][:, :, :n_c + 1])
        np.testing.assert_array_equal(to_bits(g["v"])[:, :, :s + c], state["v"][:, :, :s + c])
        ga, wa = to_bits(g["A"])[:, s:s + c], state["A"][:, s:s + c]
        diff = ga != wa
        if diff.any():   # different summation order in fp64: a rounding boundary can flip the last bit
            assert diff.mean() < 1e-3
            assert np.all(np.abs(ga.astype(np.int32) - wa.astype(np.int32))[diff] == 1)
            g["A"][:, s:s + c] = _bf16_dev(wa)       # continue from identical states
        np.testing.assert_array_equal(to_bits(g["A"])[:, :s], state["A"][:, :s])
        s += c
        # the next queries are pulled towards the new chunk so that it is selected and its rebuilt keys are used
        q = t["q_pool"][1 + i].clone()
        q += 4.0 * k_rope.float().mean(dim=2).repeat_interleave(wl.group, dim=1).to(torch.bfloat16)
        sel, ocache = _check_decode(wl, S.Params.from_workload(wl, ctx_len=s, ctx_capacity=cap), _op(wl, s, cap), q, t,
                                    g, state, cache, ocache)
        assert np.all((sel == s // c - 1).any(axis=1)), "the appended chunk should be among the selected ones"
        _check_decode(wl, S.Params.from_workload(wl, ctx_len=s, ctx_capacity=cap), _op(wl, s, cap), q, t, g, state)

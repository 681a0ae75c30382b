"""shadowkv_decode_step_static (the decode step on the library's static device scratch, for callers that
cannot allocate) against shadowkv_decode_step with a caller-owned workspace: same kernels, same layout,
so outputs and selected ids must be bit-identical.  Two calls in a row share the one scratch array, the
second on a smaller shape (it finds the first call's intermediates there and must not be disturbed by
them); a host-store shape takes the two-phase path with the gather inside the key-phase launch."""
import pytest
import torch

from paper_2410_21465_amd import shadowkv as S
from workloads import Workload, to_fp8_storage

import parity_util as PU

pytestmark = pytest.mark.gpu


def _wl(name, **kw):
    base = dict(batch=2, n_q_heads=8, n_kv_heads=2, head_dim=128, ctx_len=16384, chunk_size=8, rank=160,
                n_outlier_chunks=8, topk_chunks=64, local_len=32, rope_theta=5e5, seed=21, n_queries=2)
    base.update(kw)
    return Workload(name, **base)


def _both(wl, t, bl, qi, kv_dtype=0):
    p = S.Params.from_workload(wl, kv_dtype=kv_dtype)
    args = (t["q_pool"][qi], t["A"], t["B"], bl["landmarks"], bl["landmark_chunk_ids"], bl["k_outlier"],
            bl["v_outlier"], t["k_local"], t["v_local"], t["v"], t["pos_offset"])
    want_out, want_ids, _ = S.decode_step(p, *args)
    torch.cuda.synchronize()
    out = torch.zeros_like(want_out)
    ids = torch.zeros_like(want_ids)
    before = torch.cuda.memory_allocated()
    S.decode_step_static(p, *args, out, ids)
    torch.cuda.synchronize()
    assert torch.cuda.memory_allocated() == before
    return (want_out, want_ids), (out, ids)


def test_static_scratch_matches_workspace_entry_point_on_two_calls_in_a_row():
    big = _wl("static-big")
    small = _wl("static-small", batch=1, n_q_heads=4, n_kv_heads=1, head_dim=96, ctx_len=2048, rank=40,
                topk_chunks=17, n_outlier_chunks=2, local_len=3, rope_theta=1e4, seed=22)
    host = _wl("static-host", ctx_len=4096, topk_chunks=24, value_location="host", seed=23)
    drawn = []
    for wl in (big, small, host):
        t = PU.draw(wl)
        p = S.Params.from_workload(wl)
        bl = S.build_landmarks(p, t["k_rope"], t["v"])
        torch.cuda.synchronize()
        drawn.append((wl, t, bl))
    assert S.decode_workspace_bytes(S.Params.from_workload(big)) > S.decode_workspace_bytes(S.Params.from_workload(small))
    # big, then small, then big again with another query, then the two-phase (gathered values) path
    for (wl, t, bl), qi in ((drawn[0], 0), (drawn[1], 0), (drawn[0], 1), (drawn[2], 0), (drawn[1], 1)):
        print(f"[static] {wl.name} q{qi}", flush=True)
        (want_out, want_ids), (out, ids) = _both(wl, t, bl, qi)
        assert torch.equal(ids, want_ids), wl.name
        assert torch.equal(out.view(torch.int16), want_out.view(torch.int16)), wl.name
    # and against the oracle, through the usual parity route, so that "equal" is not "equally wrong"
    wl, t, _ = drawn[1]
    ref_b, _ = PU.run_build_parity(wl, t)
    PU.run_decode_parity(wl, t, ref_b, qi=0)


def test_static_scratch_fp8_storage_and_oversized_shape():
    wl = _wl("static-fp8", ctx_len=8192, topk_chunks=32, seed=24)
    t = to_fp8_storage(PU.draw(wl))
    p = S.Params.from_workload(wl, kv_dtype=S.KV_FP8_E5M2)
    bl = S.build_landmarks(p, t["k_rope"], t["v"])
    torch.cuda.synchronize()
    (want_out, want_ids), (out, ids) = _both(wl, t, bl, 0, kv_dtype=S.KV_FP8_E5M2)
    assert torch.equal(ids, want_ids) and torch.equal(out.view(torch.int16), want_out.view(torch.int16))
    # a shape beyond the scratch is refused before anything is enqueued (the pointers are never looked at)
    huge = S.Params(batch=64, n_q_heads=64, n_kv_heads=8, head_dim=128, ctx_len=1 << 20, topk_chunks=256)
    assert S.decode_workspace_bytes(huge) > S.static_scratch_bytes()
    with pytest.raises(S.ShadowKVError) as ei:
        S.decode_step_static(huge, *([t["q_pool"][0]] * 11), out, ids)
    assert ei.value.status == S.EWORKSPACE and "static scratch" in ei.value.detail

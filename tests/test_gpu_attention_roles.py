"""The attention kernel with key waves and value waves (values readable in place, at least three query heads per KV
head, chunk size a multiple of four) against the oracle on shapes picked to reach its corners: a last block of a split
that is partly empty, splits that end inside a step of 192 rows, a head block with fewer than four real heads, every
head dimension, ranks below one matrix step and above five, one-row budgets, no resident rows at all, FP8 storage,
position offsets.  The other GPU tests mostly ask for the diagnostic copy of the rebuilt keys, which takes the
single-role kernel; these do not."""
import numpy as np
import pytest
import torch

from paper_2410_21465_amd import shadowkv as S
from workloads import Workload, to_fp8_storage

import parity_util as PU

pytestmark = pytest.mark.gpu

#        d   hkv G   c   n_ch  r    k    o   w  batch kd
SHAPES = [
    (128, 2, 4, 8, 400, 160, 37, 3, 5, 2, 0),      # 296 selected rows: 18 full blocks and a half one
    (128, 2, 4, 8, 700, 160, 300, 6, 32, 1, 0),    # 2400 rows per unit: several splits, more than one step each
    (64, 3, 3, 4, 500, 40, 50, 2, 7, 2, 0),        # three heads in a block of four, chunks of four tokens
    (96, 2, 7, 12, 300, 96, 33, 4, 9, 1, 0),       # chunks of twelve; second head block has three real heads
    (128, 2, 8, 16, 320, 256, 70, 5, 16, 2, 0),    # rank 256 (eight matrix steps), chunks of sixteen, two head blocks
    (128, 2, 6, 8, 200, 24, 1, 0, 0, 1, 0),        # one chunk selected, no outliers, no recent tokens, rank < 32
    (128, 2, 4, 8, 300, 160, 24, 2, 3, 3, 1),      # FP8 storage
    (64, 2, 5, 4, 450, 72, 61, 3, 11, 1, 1),       # FP8, five heads, d = 64
    (128, 4, 4, 8, 2100, 160, 256, 48, 32, 2, 0),  # the benchmark's budgets on a short context, 8 units
]


@pytest.mark.parametrize("shape", SHAPES, ids=lambda s: "d%d-h%d-G%d-c%d-n%d-r%d-k%d-o%d-w%d-b%d-kd%d" % s)
def test_two_role_kernel_against_the_oracle(shape):
    d, hkv, G, c, n_ch, r, k, o, w, b, kd = shape
    wl = Workload(name="roles", batch=b, n_q_heads=hkv * G, n_kv_heads=hkv, head_dim=d, ctx_len=n_ch * c, chunk_size=c,
                  rank=r, n_outlier_chunks=o, topk_chunks=k, local_len=w, rope_theta=5e5, seed=4242 + n_ch,
                  value_location="hbm", n_queries=2)
    plan = S.decode_plan(S.Params.from_workload(wl, kv_dtype=kd))
    assert plan["key_and_value_waves"], plan
    print(f"\n[case] {wl} plan {plan}", flush=True)
    t = PU.draw(wl)
    if kd:
        t = to_fp8_storage(t)
    ref_b, _ = PU.run_build_parity(wl, t, kv_dtype=kd)
    pos = torch.tensor([0, 77, 1 << 19][:b], dtype=torch.int32)
    for qi in range(2):
        stats, _, _ = PU.run_decode_parity(wl, t, ref_b, qi=qi, check_keys=False, kv_dtype=kd, pos_offset=pos)
        print(f"[decode] q{qi}: {stats}", flush=True)


def test_resident_rows_in_the_selection_launch_eager_graph_and_static():
    """A context long enough for the single-workgroup selection with 16 slots per thread (8192 < n_c <= 16384) and few
    enough units for its launch to carry the attention over the resident rows: the step is checked against the
    oracle, then as a HIP graph replayed several times with eager work in between, then through the entry point that
    works on the library's static scratch -- all three give the same bits."""
    wl = Workload(name="res-in-select", batch=1, n_q_heads=8, n_kv_heads=2, head_dim=128, ctx_len=8 * 10000, chunk_size=8,
                  rank=64, n_outlier_chunks=8, topk_chunks=64, local_len=20, rope_theta=5e5, seed=77, value_location="hbm",
                  n_queries=3)
    p = S.Params.from_workload(wl)
    plan = S.decode_plan(p)
    assert plan["resident_rows_in_selection_launch"] and plan["key_and_value_waves"], plan
    t = PU.draw(wl)
    ref_b, _ = PU.run_build_parity(wl, t)
    stats, _, _ = PU.run_decode_parity(wl, t, ref_b, qi=0, check_keys=False)
    print(f"\n[decode] {wl.name}: {stats} plan {plan}", flush=True)

    lm, lm_ids = PU.kv_from_bits(ref_b["landmarks"]), torch.from_numpy(ref_b["landmark_chunk_ids"]).cuda()
    ko, vo = PU.kv_from_bits(ref_b["k_outlier"]), PU.kv_from_bits(ref_b["v_outlier"])
    ws = S.alloc_workspace(S.decode_workspace_bytes(p))
    q = t["q_pool"][0].clone()
    out = torch.empty(wl.batch, wl.n_q_heads, wl.head_dim, dtype=torch.bfloat16, device="cuda")
    ids = torch.empty(wl.batch, wl.n_kv_heads, wl.topk_chunks, dtype=torch.int32, device="cuda")

    def step():
        S.decode_step(p, q, t["A"], t["B"], lm, lm_ids, ko, vo, t["k_local"], t["v_local"], t["v"], t["pos_offset"],
                      out=out, out_chunk_ids=ids, workspace=ws)

    eager = []
    for qi in range(3):
        q.copy_(t["q_pool"][qi])
        step()
        torch.cuda.synchronize()
        eager.append((out.clone(), ids.clone()))
    cap = torch.cuda.Stream()
    cap.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(cap):
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g, stream=cap):
            step()
    torch.cuda.current_stream().wait_stream(cap)
    for rep in range(6):
        qi = rep % 3
        q.copy_(t["q_pool"][qi])
        out.zero_(); ids.zero_()
        g.replay()
        torch.cuda.synchronize()
        assert torch.equal(out, eager[qi][0]) and torch.equal(ids, eager[qi][1]), f"replay {rep}"
        step()                          # eager work between replays
        torch.cuda.synchronize()
        assert torch.equal(out, eager[qi][0])
    o2, i2 = torch.empty_like(out), torch.empty_like(ids)
    for qi in range(3):
        S.decode_step_static(p, t["q_pool"][qi], t["A"], t["B"], lm, lm_ids, ko, vo, t["k_local"], t["v_local"], t["v"],
                             t["pos_offset"], o2, i2)
        torch.cuda.synchronize()
        assert torch.equal(o2, eager[qi][0]) and torch.equal(i2, eager[qi][1]), f"static entry, query {qi}"

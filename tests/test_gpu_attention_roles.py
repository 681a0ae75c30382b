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

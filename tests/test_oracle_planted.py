"""Planted structure the oracle has to find, at a size the CPU finishes in seconds.

* Outlier chunks (pre-filling algorithm, lines CosineSimilarity -> ArgTopK): chunks whose rows alternate between
  +u and -u have a mean that nearly cancels, so their minimum cosine to the mean is far below any natural
  chunk's.  The o chunks the oracle takes out must all be planted ones.
* Needle chunks (decoding algorithm, lines MatMul -> Softmax -> ArgTopK): four chunks per KV head whose keys all
  equal one direction, and queries pulled towards those directions.  Their landmarks must hold the four best
  group scores, so the oracle's best-first list starts with them.

Neither expectation comes from the oracle's own arithmetic: which chunks are planted is the input generator's
record.  CPU only."""
import numpy as np

from oracle import shadowkv_oracle as O
from workloads import Workload, generate


def _params(wl):
    return O.OracleParams(wl.batch, wl.n_q_heads, wl.n_kv_heads, wl.head_dim, wl.ctx_len, wl.chunk_size, wl.rank,
                          wl.n_outlier_chunks, wl.topk_chunks, wl.local_len, rope_theta=wl.rope_theta)


def _bits(t):
    return {k: O.as_bits(t[k]) for k in ("k_rope", "v", "A", "B", "k_local", "v_local")}


def test_planted_outlier_chunks_are_what_the_cosine_criterion_takes_out():
    # 512 chunks, 5 planted per KV head, 4 taken out
    wl = Workload("planted-outliers", 2, 8, 2, 64, 4096, rank=32, n_outlier_chunks=4, topk_chunks=32, local_len=16,
                  seed=11, plant="outliers")
    t = generate(wl, device="cpu")
    bits = _bits(t)
    ref = O.build_landmarks(_params(wl), bits["k_rope"], bits["v"], diagnostics=True)
    planted = t["planted_chunks"].numpy().reshape(wl.units, -1)
    found = ref["outlier_chunk_ids"].reshape(wl.units, -1)
    mc = ref["chunk_min_cos"].reshape(wl.units, -1)
    assert planted.shape[1] == 5 and found.shape[1] == 4
    for u in range(wl.units):
        assert set(found[u]) <= set(planted[u]), (u, found[u], planted[u])
        # and by a wide margin: every planted chunk scores below every natural one
        natural = np.setdiff1d(np.arange(wl.n_chunks), planted[u])
        assert mc[u, planted[u]].max() < mc[u, natural].min() - 0.3
    # the chunks taken out are not landmarks, and their rows were copied
    ids = ref["landmark_chunk_ids"].reshape(wl.units, -1)
    k = bits["k_rope"].reshape(wl.units, wl.n_chunks, wl.chunk_size, wl.head_dim)
    ko = ref["k_outlier"].reshape(wl.units, 4, wl.chunk_size, wl.head_dim)
    for u in range(wl.units):
        assert not set(found[u]) & set(ids[u])
        assert np.array_equal(ko[u], k[u, found[u]])


def test_needle_chunks_hold_the_four_best_scores():
    wl = Workload("planted-needles", 1, 8, 2, 64, 4096, rank=48, n_outlier_chunks=0, topk_chunks=16, local_len=16,
                  seed=12, plant="needles")
    t = generate(wl, device="cpu")
    bits = _bits(t)
    p = _params(wl)
    b = O.build_landmarks(p, bits["k_rope"], bits["v"])
    needles = t["needle_chunks"].numpy().reshape(wl.units, 4)
    for qi in range(3):
        d = O.decode_step(p, O.as_bits(t["q_pool"][qi]), bits["A"], bits["B"], b["landmarks"], b["landmark_chunk_ids"],
                          b["k_outlier"], b["v_outlier"], bits["k_local"], bits["v_local"], bits["v"],
                          t["pos_offset"].numpy())
        best_first = d["chunk_ids"].reshape(wl.units, -1)
        for u in range(wl.units):
            assert set(best_first[u, :4]) == set(needles[u]), (qi, u, best_first[u, :6], needles[u])

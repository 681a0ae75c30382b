"""Pins of the oracle's chunk-cache model (section "High-throughput Decoding": index scan, fetch only the
missing chunks).  CPU only.  The policy is stated in the oracle; these tests check it against set algebra
done independently in Python, hand-worked cases, and the invariants any correct cache must keep."""
import numpy as np
import pytest

from oracle import shadowkv_oracle as O


def test_hand_worked_case():
    # slots hold chunks [7, 3, 9, 1]; the step selects {1, 4, 7, 8}: 7 and 1 stay where they are,
    # 4 and 8 (ascending) take the freed slots 1 and 2 (ascending)
    r = O.cache_update(np.array([[1, 4, 7, 8]]), np.array([[7, 3, 9, 1]]))
    assert r["cache_ids"].tolist() == [[7, 4, 8, 1]]
    assert r["n_miss"].tolist() == [2]
    assert r["miss_slots"][0, :2].tolist() == [1, 2]


def test_empty_cache_takes_the_selection_in_order():
    sel = np.array([[2, 5, 6], [0, 1, 9]])
    r = O.cache_update(sel, -np.ones((2, 3), np.int32))
    assert np.array_equal(r["cache_ids"], sel)
    assert r["n_miss"].tolist() == [3, 3]
    assert r["miss_slots"].tolist() == [[0, 1, 2], [0, 1, 2]]


def test_same_selection_is_all_hits_and_changes_nothing():
    cache = np.array([[9, 2, 4, 0]])
    r = O.cache_update(np.array([[0, 2, 4, 9]]), cache)
    assert r["n_miss"].tolist() == [0]
    assert np.array_equal(r["cache_ids"], cache)
    assert r["miss_slots"].tolist() == [[-1, -1, -1, -1]]


def test_disjoint_selection_replaces_every_slot():
    r = O.cache_update(np.array([[10, 11, 12]]), np.array([[3, 1, 2]]))
    assert r["cache_ids"].tolist() == [[10, 11, 12]] and r["n_miss"].tolist() == [3]


@pytest.mark.parametrize("seed", range(5))
def test_against_set_algebra_over_a_random_sequence(seed):
    rng = np.random.default_rng(seed)
    units, k, n_chunks = 3, 16, 40
    cache = -np.ones((units, k), np.int32)
    for step in range(12):
        sel = np.stack([np.sort(rng.choice(n_chunks, k, replace=False)) for _ in range(units)]).astype(np.int32)
        r = O.cache_update(sel, cache)
        new = r["cache_ids"]
        for u in range(units):
            before, after, s = cache[u], new[u], set(sel[u].tolist())
            assert sorted(after.tolist()) == sorted(s)                   # holds exactly the selection
            hits = s & set(before.tolist())
            assert r["n_miss"][u] == k - len(hits)                        # misses = selection minus what was there
            for slot in range(k):                                        # a hit never moves
                if before[slot] in hits:
                    assert after[slot] == before[slot]
            ms = r["miss_slots"][u, : r["n_miss"][u]].tolist()
            assert ms == sorted(ms) and len(set(ms)) == len(ms)
            assert ms == [slot for slot in range(k) if before[slot] not in hits]   # exactly the freed slots
            filled = [after[slot] for slot in ms]
            assert filled == sorted(s - hits)                             # new chunks in ascending id
            assert all(x == -1 for x in r["miss_slots"][u, r["n_miss"][u]:])
        cache = new


def test_hit_rate_formula_on_a_shifting_window():
    # selection slides by 2 of 8 chunks per step: 6 hits, 2 misses each step after the first
    k = 8
    cache = -np.ones((1, k), np.int32)
    for step in range(5):
        sel = np.arange(2 * step, 2 * step + k, dtype=np.int32)[None]
        r = O.cache_update(sel, cache)
        assert r["n_miss"][0] == (k if step == 0 else 2)
        cache = r["cache_ids"]


# ---- more slots than selected chunks: least-recently-used replacement ----

def test_lru_hand_worked_case():
    # 5 slots, 2 selected per step
    r = O.cache_update(np.array([[3, 7]]), -np.ones((1, 5), np.int32))              # clock 1: slots 0,1 <- 3,7
    assert r["cache_ids"].tolist() == [[3, 7, -1, -1, -1]] and r["sel_slots"].tolist() == [[0, 1]]
    r = O.cache_update(np.array([[4, 7]]), r["cache_ids"], r["stamps"])             # clock 2: 7 hits, 4 -> first empty
    assert r["cache_ids"].tolist() == [[3, 7, 4, -1, -1]] and r["n_miss"].tolist() == [1]
    assert r["sel_slots"].tolist() == [[2, 1]] and r["miss_slots"][0, 0] == 2
    r = O.cache_update(np.array([[8, 9]]), r["cache_ids"], r["stamps"])             # clock 3: the two empties
    assert r["cache_ids"].tolist() == [[3, 7, 4, 8, 9]]
    r = O.cache_update(np.array([[1, 2]]), r["cache_ids"], r["stamps"])             # clock 4: oldest are 3 (1) and 7/4 (2): 3, then 7 (lower slot)
    assert r["cache_ids"].tolist() == [[1, 2, 4, 8, 9]] and r["miss_slots"][0].tolist() == [0, 1]
    r = O.cache_update(np.array([[4, 5]]), r["cache_ids"], r["stamps"])             # clock 5: 4 hits; 5 evicts the oldest other slot: 8 (stamp 3, slot 3)
    assert r["cache_ids"].tolist() == [[1, 2, 4, 5, 9]] and r["sel_slots"].tolist() == [[2, 3]]
    assert r["stamps"][0].tolist() == [4, 4, 5, 5, 3, 5]


@pytest.mark.parametrize("seed,S", [(0, 16), (1, 24), (2, 40), (3, 64)])
def test_lru_against_an_independent_simulation(seed, S):
    rng = np.random.default_rng(seed)
    k, n_chunks = 16, 60
    cache = -np.ones((1, S), np.int32)
    stamps = None
    model = {}          # chunk -> [slot, last use]; written independently of the C code
    free = list(range(S))
    for step in range(1, 40):
        pool = rng.choice(n_chunks, 24, replace=False) if step % 7 else np.arange(n_chunks)
        sel = np.sort(rng.choice(pool, k, replace=False)).astype(np.int32)
        r = O.cache_update(sel[None], cache, stamps)
        hits = [c for c in sel if c in model]
        for c in hits:
            model[c][1] = step
        new = [c for c in sel if c not in model]
        occupied_not_hit = sorted((v[1], v[0], c) for c, v in model.items() if c not in hits)
        victims = sorted(free)[:len(new)]
        for _, slot, c in occupied_not_hit[:len(new) - len(victims)]:
            victims.append(slot); del model[c]
        free = [f for f in free if f not in victims]
        for c, slot in zip(new, sorted(victims)):
            model[int(c)] = [slot, step]
        want = -np.ones(S, np.int32)
        for c, (slot, _) in model.items():
            want[slot] = c
        assert r["cache_ids"][0].tolist() == want.tolist(), step
        assert r["n_miss"][0] == len(new)
        assert r["miss_slots"][0, :len(new)].tolist() == sorted(victims)
        assert np.array_equal(r["cache_ids"][0][r["sel_slots"][0]], sel)          # every selected chunk is where it says
        cache, stamps = r["cache_ids"], r["stamps"]
        assert stamps[0, S] == step


def test_a_cache_as_large_as_the_context_never_refetches():
    rng = np.random.default_rng(5)
    k, n_chunks = 8, 32
    cache, stamps, seen = -np.ones((1, n_chunks), np.int32), None, set()
    for _ in range(30):
        sel = np.sort(rng.choice(n_chunks, k, replace=False)).astype(np.int32)
        r = O.cache_update(sel[None], cache, stamps)
        assert r["n_miss"][0] == len(set(sel.tolist()) - seen)
        seen |= set(sel.tolist())
        cache, stamps = r["cache_ids"], r["stamps"]


def test_fewer_slots_than_selected_chunks_is_rejected():
    with pytest.raises(ValueError):
        O.cache_update(np.array([[1, 2, 3]]), -np.ones((1, 2), np.int32))

"""Host-only checks of the C ABI: the library loads, exports every declared symbol,
and rejects bad arguments before touching a GPU (none is needed to run these)."""
import ctypes as C
import os
import re

import pytest

from paper_2410_21465_amd import shadowkv as S

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_symbols():
    text = open(os.path.join(ROOT, "include", "shadowkv.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(shadowkv_[a-z0-9_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    lib = S.lib()
    names = declared_symbols()
    assert "shadowkv_build_landmarks" in names and "shadowkv_decode_step" in names
    for n in names:
        assert hasattr(lib, n), f"{n} declared in shadowkv.h but not exported"
    assert set(S.EXPORTS) <= set(names)
    assert S.version() >= 100


def test_status_strings():
    assert S.status_string(S.OK) == "ok"
    for code in (S.EINVAL, S.EWORKSPACE, S.EHIP, -99):
        assert S.status_string(code)


GOOD = dict(batch=2, n_q_heads=8, n_kv_heads=2, head_dim=128, ctx_len=4096, chunk_size=8, rank=160,
            n_outlier_chunks=4, topk_chunks=16, local_len=8)


def test_valid_params_and_workspace_sizes():
    p = S.Params(**GOOD)
    assert S.validate_params(p) == S.OK and S.validate_params(p, for_decode=False) == S.OK
    w = S.decode_workspace_bytes(p)
    assert w > 0 and w % 256 == 0
    bigger = S.decode_workspace_bytes(S.Params(**{**GOOD, "topk_chunks": 32}))
    assert bigger > w
    staged = S.decode_workspace_bytes(S.Params(**{**GOOD, "value_location": S.VALUES_HOST}))
    assert staged >= w + 2 * 8 * 16 * 128 * 2 * 2      # units * c * k * d bf16 values
    assert S.build_workspace_bytes(p) >= 2 * 2 * 512 * (128 * 2 + 8)
    # the five benchmark shapes are all accepted
    from workloads import CONFIGS
    for wl in CONFIGS.values():
        assert S.validate_params(S.Params.from_workload(wl)) == S.OK, wl.name


@pytest.mark.parametrize("bad", [
    dict(batch=0), dict(n_q_heads=9), dict(head_dim=80), dict(head_dim=127), dict(chunk_size=0), dict(chunk_size=65),
    dict(ctx_len=4100), dict(ctx_len=0), dict(rank=12), dict(rank=0), dict(rank=264), dict(topk_chunks=0),
    dict(topk_chunks=509), dict(n_outlier_chunks=-1), dict(n_outlier_chunks=2000), dict(local_len=-1),
    dict(value_location=7), dict(kv_dtype=2), dict(kv_dtype=-1), dict(softmax_scale=-1.0), dict(rope_theta=0.0), dict(n_q_heads=2 * 65, n_kv_heads=2),
])
def test_invalid_params_are_rejected(bad):
    p = S.Params(**{**GOOD, **bad})
    assert S.validate_params(p) == S.EINVAL
    assert S.last_error()
    assert S.decode_workspace_bytes(p) == 0


def test_fp8_storage_halves_the_value_buffers():
    """kv_dtype = FP8 E5M2: one byte per stored element in every size the library reports."""
    host16 = S.Params(**{**GOOD, "value_location": S.VALUES_HOST})
    host8 = S.Params(**{**GOOD, "value_location": S.VALUES_HOST, "kv_dtype": S.KV_FP8_E5M2})
    assert S.validate_params(host8) == S.OK and S.validate_params(host8, for_decode=False) == S.OK
    rows = 2 * 2 * 16 * 8 * 128                    # units * k * c * d staged value elements
    assert S.decode_workspace_bytes(host16) - S.decode_workspace_bytes(host8) == rows
    assert S.decode_workspace_bytes(S.Params(**{**GOOD, "kv_dtype": S.KV_FP8_E5M2})) == S.decode_workspace_bytes(S.Params(**GOOD))
    st16, st8 = host16.c_struct(), host8.c_struct()
    import ctypes as C
    n16 = S.lib().shadowkv_value_cache_bytes(C.addressof(st16), 64)
    n8 = S.lib().shadowkv_value_cache_bytes(C.addressof(st8), 64)
    assert n16 == 2 * n8 == 2 * 2 * 64 * 8 * 128 * 2
    # chunk means of the pre-filling step are kept in the storage type
    assert S.build_workspace_bytes(S.Params(**GOOD)) - S.build_workspace_bytes(S.Params(**{**GOOD, "kv_dtype": 1})) == 2 * 2 * 512 * 128


def test_build_ignores_decode_only_fields():
    p = S.Params(**{**GOOD, "rank": 12, "topk_chunks": 0})
    assert S.validate_params(p, for_decode=False) == S.OK
    assert S.build_workspace_bytes(p) > 0


def test_calls_reject_null_and_bad_workspace_without_a_gpu():
    lib = S.lib()
    st = S.Params(**GOOD).c_struct()
    fake = C.c_void_p(0x1000)        # never dereferenced: validation fails first
    args = [fake] * 11               # q .. pos_offset
    # NULL q
    rc = lib.shadowkv_decode_step(C.addressof(st), None, *args[1:], fake, None, fake, 1 << 40, None, None)
    assert rc == S.EINVAL
    # misaligned tensor pointer
    rc = lib.shadowkv_decode_step(C.addressof(st), C.c_void_p(0x1008), *args[1:], fake, None, fake, 1 << 40, None, None)
    assert rc == S.EINVAL and "aligned" in S.last_error()
    # NULL workspace, misaligned workspace, short workspace
    rc = lib.shadowkv_decode_step(C.addressof(st), *args, fake, None, None, 1 << 40, None, None)
    assert rc == S.EWORKSPACE
    rc = lib.shadowkv_decode_step(C.addressof(st), *args, fake, None, C.c_void_p(0x1010), 1 << 40, None, None)
    assert rc == S.EWORKSPACE
    rc = lib.shadowkv_decode_step(C.addressof(st), *args, fake, None, fake, 1024, None, None)
    assert rc == S.EWORKSPACE and "too small" in S.last_error()
    # NULL params
    rc = lib.shadowkv_decode_step(None, *args, fake, None, fake, 1 << 40, None, None)
    assert rc == S.EINVAL
    # build: NULL k_rope, short workspace
    rc = lib.shadowkv_build_landmarks(C.addressof(st), None, None, fake, fake, fake, fake, None, fake, 1 << 40, None)
    assert rc == S.EINVAL
    rc = lib.shadowkv_build_landmarks(C.addressof(st), fake, None, fake, fake, fake, fake, None, fake, 16, None)
    assert rc == S.EWORKSPACE
    # missing outlier tensors with o > 0
    rc = lib.shadowkv_decode_step(C.addressof(st), *args[:5], None, None, *args[7:], fake, None, fake, 1 << 40, None, None)
    assert rc == S.EINVAL


def test_factorize_keys_rejects_bad_arguments_without_a_gpu():
    lib = S.lib()
    fake = C.c_void_p(0x1000)
    p = S.Params(**GOOD)
    st = p.c_struct()
    need = lib.shadowkv_factorize_workspace_bytes(C.addressof(st))
    # Gram matrix and its split partials (fp64, 256 x 256 per sequence) are the floor of the size
    assert need >= 2 * 2 * 256 * 256 * 8 and need % 256 == 0
    call = lib.shadowkv_factorize_keys
    assert call(C.addressof(st), None, fake, fake, None, None, 0, fake, need, None) == S.EINVAL           # NULL keys
    assert call(C.addressof(st), fake, fake, fake, C.c_void_p(0x1008), None, 0, fake, need, None) == S.EINVAL  # misaligned
    assert call(C.addressof(st), fake, fake, fake, None, None, -1, fake, need, None) == S.EINVAL          # n_iter
    assert call(C.addressof(st), fake, fake, fake, None, None, 0, None, need, None) == S.EWORKSPACE
    assert call(C.addressof(st), fake, fake, fake, None, None, 0, fake, need - 256, None) == S.EWORKSPACE
    wide = S.Params(**{**GOOD, "rank": 256, "n_kv_heads": 1, "n_q_heads": 8}).c_struct()                 # r > h_kv * d
    assert lib.shadowkv_factorize_workspace_bytes(C.addressof(wide)) == 0
    assert call(C.addressof(wide), fake, fake, fake, None, None, 0, fake, 1 << 40, None) == S.EINVAL
    assert "key width" in S.last_error()


def test_append_chunk_rejects_a_full_context_and_bad_capacity():
    lib = S.lib()
    fake = C.c_void_p(0x1000)
    p = S.Params(batch=1, n_q_heads=8, n_kv_heads=2, head_dim=128, ctx_len=1024, chunk_size=8, rank=32,
                 n_outlier_chunks=2, topk_chunks=16, local_len=4)
    st = p.c_struct()
    rc = lib.shadowkv_append_chunk(C.addressof(st), *([fake] * 8), None)
    assert rc == S.EINVAL and "no room" in S.last_error()
    p.ctx_capacity = 1028                      # not a multiple of the chunk size
    st = p.c_struct()
    assert lib.shadowkv_append_chunk(C.addressof(st), *([fake] * 8), None) == S.EINVAL
    assert lib.shadowkv_validate_params(C.addressof(st), 1) == S.EINVAL
    p.ctx_capacity = 1016                      # below ctx_len
    st = p.c_struct()
    assert lib.shadowkv_validate_params(C.addressof(st), 1) == S.EINVAL
    p.ctx_capacity = 1032
    st = p.c_struct()
    assert lib.shadowkv_validate_params(C.addressof(st), 1) == S.OK
    assert lib.shadowkv_append_chunk(C.addressof(st), None, *([fake] * 7), None) == S.EINVAL   # NULL k_pre


def test_decode_plan_of_the_benchmark_shapes():
    """shadowkv_decode_plan is host logic: how the step of a shape is cut into launches, splits and roles."""
    import ctypes as C
    from workloads import CONFIGS
    plan = S.decode_plan(S.Params.from_workload(CONFIGS["c3-hbm"]))
    assert plan == {"splits": 2, "rows_per_split": 1024, "resident_rows_in_selection_launch": True,
                    "key_and_value_waves": True, "selection_threads": 1024, "selection_candidates_per_thread": 16,
                    "selection_launches": 1, "logit_row_floats": 16336}
    # the splits cover the selected rows; one selection launch up to 32768 landmarks, more beyond
    for wl in CONFIGS.values():
        pl = S.decode_plan(S.Params.from_workload(wl))
        assert pl["splits"] * pl["rows_per_split"] >= wl.topk_chunks * wl.chunk_size > (pl["splits"] - 1) * pl["rows_per_split"]
        assert (pl["selection_launches"] == 1) == (wl.n_landmarks <= 32768)
        assert pl["logit_row_floats"] >= wl.n_landmarks and pl["logit_row_floats"] % 4 == 0
        # values that have to be gathered, or one or two heads per KV head, take the single-role kernels
        assert pl["key_and_value_waves"] == (wl.value_location == "hbm" and wl.group >= 3 and wl.chunk_size % 4 == 0)
    st = S.Params.from_workload(CONFIGS["c1"]).c_struct()
    assert S.lib().shadowkv_decode_plan(C.byref(st), None) == S.EINVAL
    bad = S.Params(**{**GOOD, "rank": 12}).c_struct()
    assert S.lib().shadowkv_decode_plan(C.byref(bad), (C.c_int32 * 8)()) == S.EINVAL

"""Host-only checks of the C-ABI library: it loads, exports every symbol the header
declares, and its argument validation answers before anything touches a GPU."""
import ctypes
import os
import re

import numpy as np
import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def R():
    from paper_2508_09072_amd import binding
    if not os.path.exists(binding.LIB_PATH):
        from paper_2508_09072_amd import build
        build.build()
    binding.load()
    return binding


def declared_symbols():
    text = open(os.path.join(ROOT, "include", "reader.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(reader_[a-z_]+)\s*\(", text)))


def test_every_declared_symbol_is_exported(R):
    names = declared_symbols()
    assert set(names) == set(R.EXPORTS)
    lib = ctypes.CDLL(R.LIB_PATH)
    for n in names:
        assert getattr(lib, n) is not None


def test_dims_struct_matches_header(R):
    text = open(os.path.join(ROOT, "include", "reader.h")).read()
    body = re.search(r"typedef struct reader_dims \{(.*?)\} reader_dims;", text, flags=re.S).group(1)
    body = re.sub(r"/\*.*?\*/", "", body, flags=re.S)
    fields = re.findall(r"(int32_t|int64_t|float)\s+(\w+);", body)
    ctype = {"int32_t": ctypes.c_int32, "int64_t": ctypes.c_int64, "float": ctypes.c_float}
    assert [(n, ctype[t]) for t, n in fields] == list(R.ReaderDims._fields_)


def test_version_and_strerror(R):
    assert "gfx950" in R.version()
    assert R.strerror(0) == "ok" and "workspace" in R.strerror(R.READER_EWORKSPACE)


def test_validate_tree(R):
    good = np.asarray([[-1, 0, 0, 2], [-1, 0, 1, 2]], dtype=np.int32)
    assert R.reader_validate_tree(good) == R.READER_OK
    for bad in ([[0, 0, 1]], [[-1, -1, 0]], [[-1, 1, 0]], [[-1, 0, 2]], [[-1, 0, 0], [-1, 0, 7]]):
        assert R.reader_validate_tree(np.asarray(bad, dtype=np.int32)) == R.READER_EINVAL


def test_workspace_bytes_is_pure_and_monotone(R):
    d = R.make_dims(16, 32, 32, 8, 128, 260, 7, 3000)
    a, b = R.reader_workspace_bytes(d, 4096), R.reader_workspace_bytes(d, 4096)
    assert a == b and a % 256 == 0 and a > 0
    assert R.reader_workspace_bytes(R.make_dims(16, 32, 32, 8, 100, 260, 7, 3000), 4096) == 0   # bad D
    assert R.reader_workspace_bytes(d, 64) <= a


def test_attention_plan_follows_the_query_rows_and_the_overrides(R):
    # few query rows per kv head: 128-row workgroups with copying wavefronts; many rows on a long context: 256-row
    # workgroups, four wavefronts at head dimension 128 and eight at 64; the override names either
    small = R.reader_attn_plan(R.make_dims(16, 32, 32, 8, 128, 260, 7, 3000), 4096)
    assert small["kernel_id"] == 1 and small["rows_per_workgroup"] == 128 and small["row_chunks"] == 1
    assert 1 <= small["key_ranges"] <= 256
    big = R.reader_attn_plan(R.make_dims(64, 64, 64, 8, 128, 520, 7, 30000), 8192)
    assert big["kernel_id"] == 3 and big["rows_per_workgroup"] == 256 and big["row_chunks"] == 2
    assert big["kernel"] == "tree_attn_wide_kernel<128>"
    big64 = R.reader_attn_plan(R.make_dims(64, 64, 64, 8, 64, 520, 7, 30000), 8192)
    assert big64["kernel_id"] == 2
    try:
        R.reader_tuning_override(R.TUNE_ATTN_WIDE, 0)
        assert R.reader_attn_plan(R.make_dims(64, 64, 64, 8, 128, 520, 7, 30000), 8192)["kernel_id"] == 2
        R.reader_tuning_override(R.TUNE_ATTN_ROWS, 128)
        forced = R.reader_attn_plan(R.make_dims(64, 64, 64, 8, 128, 520, 7, 30000), 8192)
        assert forced["kernel_id"] == 1 and forced["row_chunks"] == 4
    finally:
        R.reader_tuning_override(R.TUNE_ATTN_WIDE, -1)
        R.reader_tuning_override(R.TUNE_ATTN_ROWS, -1)
    scalar = R.reader_attn_plan(R.make_dims(2, 8, 8, 2, 64, 10, 4, 20, variant=1), 100)
    assert scalar["kernel_id"] == 0
    with pytest.raises(RuntimeError):
        R.reader_attn_plan(R.make_dims(2, 8, 8, 2, 96, 10, 4, 20), 100)


@pytest.mark.parametrize("change,code", [
    (dict(T=0), -1), (dict(T=129), -2), (dict(D=96), -2), (dict(Hkv=3), -1), (dict(page_size=32), -2),
    (dict(max_path=0), -1), (dict(max_path=33), -1), (dict(Hq=64, Hkv=2), -2), (dict(B=-1), -1),
])
def test_bad_dims_are_refused_on_the_host(R, change, code):
    base = dict(B=2, T=32, Hq=32, Hkv=8, D=128, max_pages_per_seq=16, max_path=7, num_pages=40)
    base.update(change)
    page_size = base.pop("page_size", 16)
    d = R.make_dims(**base, page_size=page_size)
    lib = R.load()
    null = [None] * 10
    assert lib.reader_tree_attn(ctypes.byref(d), *null, 0, None, 0, None, None) == code
    assert lib.reader_accept_path(ctypes.byref(d), *[None] * 8) == code
    assert lib.reader_kv_compact(ctypes.byref(d), *[None] * 10) == code
    assert lib.reader_verify_step(ctypes.byref(d), *[None] * 15, 0, None, 0, None, None) == code


def test_null_pointers_and_workspace_are_refused(R):
    d = R.make_dims(2, 32, 32, 8, 128, 16, 7, 40)
    lib = R.load()
    one = ctypes.c_void_p(256)            # never dereferenced: the checks fail first
    assert lib.reader_tree_attn(ctypes.byref(d), *[None] * 10, 128, None, 0, None, None) == R.READER_EINVAL
    assert lib.reader_tree_attn(ctypes.byref(d), *[one] * 9, None, 128, None, 0, None, None) == R.READER_EWORKSPACE
    assert lib.reader_tree_attn(ctypes.byref(d), *[one] * 9, None, 128, one, 16, None, None) == R.READER_EWORKSPACE
    assert lib.reader_tree_attn(ctypes.byref(d), *[one] * 9, None, 10**6, one, 1 << 40, None, None) == R.READER_EINVAL
    assert lib.reader_accept_path(ctypes.byref(d), one, one, None, one, one, one, None, None) == R.READER_EINVAL
    assert lib.reader_kv_compact(ctypes.byref(d), *[one] * 7, None, None, None) == R.READER_EINVAL
    assert lib.reader_tree_attn(None, *[one] * 9, None, 128, one, 1 << 40, None, None) == R.READER_EINVAL
    # B = 0 is a valid empty problem: nothing is enqueued
    d0 = R.make_dims(0, 32, 32, 8, 128, 16, 7, 40)
    assert lib.reader_tree_attn(ctypes.byref(d0), *[None] * 10, 0, None, 0, None, None) == R.READER_OK
    assert lib.reader_accept_path(ctypes.byref(d0), *[None] * 8) == R.READER_OK
    assert lib.reader_kv_compact(ctypes.byref(d0), *[None] * 10) == R.READER_OK
    assert lib.reader_verify_step(ctypes.byref(d0), *[None] * 15, 0, None, 0, None, None) == R.READER_OK
    # the fused step checks what the three calls check
    assert lib.reader_verify_step(ctypes.byref(d), *[None] * 15, 128, None, 0, None, None) == R.READER_EINVAL
    assert lib.reader_verify_step(ctypes.byref(d), *[one] * 8, None, one, one, None, one, one, one, 128, one, 1 << 40,
                                  None, None) == R.READER_EINVAL            # draft tokens missing
    assert lib.reader_verify_step(ctypes.byref(d), *[one] * 11, None, one, one, one, 128, one, 16, None, None) \
        == R.READER_EWORKSPACE


def test_binding_refuses_cpu_tensors(R):
    import torch
    d = R.make_dims(1, 4, 4, 4, 64, 4, 3, 8)
    t = torch.zeros(4, dtype=torch.int32)
    with pytest.raises(ValueError):
        R.reader_accept_path(d, t, t, t, t, t, t)


def test_rearrange_arguments_are_checked_on_the_host(R):
    lib = R.load()
    one = ctypes.c_void_p(256)
    assert R.reader_kv_rearrange_scratch_bytes(16, 4224) >= (16 * 4224 + 64) * 4
    assert R.reader_kv_rearrange_scratch_bytes(16, 4224) % 256 == 0
    assert lib.reader_kv_rearrange(1, 2, 8, 0, 128, one, one, one, one, one, 1 << 20, None) == R.READER_EINVAL
    assert lib.reader_kv_rearrange(1, 2, 8, 2, 96, one, one, one, one, one, 1 << 20, None) == R.READER_EUNSUPPORTED
    assert lib.reader_kv_rearrange(1, 2, 8, 2, 128, None, one, one, one, one, 1 << 20, None) == R.READER_EINVAL
    assert lib.reader_kv_rearrange(1, 2, 8, 2, 128, one, one, one, one, None, 0, None) == R.READER_EWORKSPACE
    assert lib.reader_kv_rearrange(1, 2, 8, 2, 128, one, one, one, one, one, 16, None) == R.READER_EWORKSPACE
    assert lib.reader_kv_rearrange(1, 0, 8, 2, 128, None, None, None, None, None, 0, None) == R.READER_OK   # empty batch
    # more workgroups than one launch holds: layers x samples x (kv heads + 1) must stay below 2^31
    assert lib.reader_kv_rearrange(40000, 8192, 8, 8, 128, one, one, one, one, one, 1 << 20, None) == R.READER_EUNSUPPORTED



def test_target_token_arguments_are_checked_on_the_host(R):
    lib = R.load()
    one = ctypes.c_void_p(256)
    assert lib.reader_target_argmax(-1, 10, one, one, None) == R.READER_EINVAL
    assert lib.reader_target_argmax(4, 0, one, one, None) == R.READER_EINVAL
    assert lib.reader_target_argmax(4, 10, None, one, None) == R.READER_EINVAL
    assert lib.reader_target_argmax(0, 10, None, None, None) == R.READER_OK
    s = lib.reader_target_sample
    assert s(-1, 4, 10, one, one, one, 1.0, one, None) == R.READER_EINVAL
    assert s(2, 0, 10, one, one, one, 1.0, one, None) == R.READER_EINVAL
    assert s(2, 129, 10, one, one, one, 1.0, one, None) == R.READER_EINVAL          # more nodes than a tree may have
    assert s(2, 4, 0, one, one, one, 1.0, one, None) == R.READER_EINVAL
    assert s(2, 4, (1 << 22) + 1, one, one, one, 1.0, one, None) == R.READER_EINVAL  # vocabulary beyond the limit
    for bad in (0.0, -1.0, 1e-9, 1e9, float("inf"), float("nan")):
        assert s(2, 4, 10, one, one, one, bad, one, None) == R.READER_EINVAL
    assert s(2, 4, 10, None, one, one, 1.0, one, None) == R.READER_EINVAL
    assert s(2, 4, 10, one, one, None, 1.0, one, None) == R.READER_EINVAL
    assert s(0, 4, 10, None, None, None, 1.0, None, None) == R.READER_OK             # empty batch


def test_layered_compaction_arguments_are_checked_on_the_host(R):
    lib = R.load()
    one = ctypes.c_void_p(256)
    dims = R.make_dims(2, 16, 8, 2, 128, 8, 8, 40)
    f = lib.reader_kv_compact_layers
    assert f(ctypes.byref(dims), -1, one, one, one, one, one, one, None, None) == R.READER_EINVAL
    assert f(ctypes.byref(dims), 70000, one, one, one, one, one, one, None, None) == R.READER_EINVAL
    assert f(ctypes.byref(dims), 2, None, one, one, one, one, one, None, None) == R.READER_EINVAL
    assert f(ctypes.byref(dims), 2, one, one, None, one, one, one, None, None) == R.READER_EINVAL
    empty = R.make_dims(0, 16, 8, 2, 128, 8, 8, 40)
    assert f(ctypes.byref(empty), 2, None, None, None, None, None, None, None, None) == R.READER_OK

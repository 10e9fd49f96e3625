"""ctypes binding of libreader_hip.so: argument marshalling only.

Every function has the name and argument order of its C entry point in
``include/reader.h``; tensors are torch CUDA (ROCm) tensors whose ``data_ptr()`` is
handed through, and every kernel is enqueued on torch's current stream.  Nothing is
computed here, and there is no fallback: if the library has not been built, or a
tensor is not on the GPU, the call raises.
"""
from __future__ import annotations

import ctypes
import dataclasses
import os

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libreader_hip.so")

READER_OK = 0
READER_EINVAL = -1
READER_EUNSUPPORTED = -2
READER_EWORKSPACE = -3
READER_EHIP = -4
STATUS_BAD_TREE = 1
STATUS_BAD_PAGE = 2
STATUS_BAD_PATH = 4
TUNE_ATTN_ROWS, TUNE_ATTN_RANGES, TUNE_ATTN_PAIR_COST, TUNE_ATTN_AXIS64, TUNE_ATTN_WIDE, TUNE_ATTN_PAIR_FRONT = 0, 1, 2, 3, 4, 5

EXPORTS = (
    "reader_version", "reader_strerror", "reader_last_error_detail", "reader_validate_tree", "reader_workspace_bytes",
    "reader_tree_attn", "reader_tree_attn_noalloc", "reader_accept_path", "reader_kv_compact", "reader_verify_step",
    "reader_kv_rearrange_scratch_bytes", "reader_kv_rearrange", "reader_target_argmax", "reader_target_sample", "reader_kv_compact_layers",
    "reader_trie_create", "reader_trie_destroy", "reader_trie_nodes", "reader_trie_insert", "reader_trie_search_path",
    "reader_trie_extract_tree", "reader_tree_attach_path", "reader_self_repetition", "reader_tree_prune_order",
    "reader_tree_select",
    "reader_profile_enable", "reader_profile_collect", "reader_profile_collect_each", "reader_tuning_override",
    "reader_attn_plan", "reader_measure_peaks",
)


class ReaderAttnPlan(ctypes.Structure):
    """Mirror of ``struct reader_attn_plan_t``."""
    _fields_ = [("kernel", ctypes.c_int32), ("rows_per_workgroup", ctypes.c_int32), ("row_chunks", ctypes.c_int32),
                ("key_ranges", ctypes.c_int32)]


class ReaderDims(ctypes.Structure):
    """Mirror of ``struct reader_dims``."""
    _fields_ = [
        ("B", ctypes.c_int32), ("T", ctypes.c_int32), ("Hq", ctypes.c_int32), ("Hkv", ctypes.c_int32),
        ("D", ctypes.c_int32), ("page_size", ctypes.c_int32), ("max_pages_per_seq", ctypes.c_int32),
        ("max_path", ctypes.c_int32), ("num_pages", ctypes.c_int64), ("sm_scale", ctypes.c_float),
        ("variant", ctypes.c_int32),
    ]


class ReaderError(RuntimeError):
    def __init__(self, code, where):
        self.code = code
        detail = load().reader_last_error_detail().decode() if code == READER_EHIP else ""
        super().__init__("%s: %s (code %d) %s" % (where, strerror(code), code, detail))


_lib = None


def load():
    """Load the library; raises if it has not been built (python -m paper_2508_09072_amd.build)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise RuntimeError("HIP library missing: %s (run `python -m paper_2508_09072_amd.build`)" % LIB_PATH)
    # PyTorch first: it brings its own copy of the HIP runtime, and the tensors and streams handed to
    # the library belong to that one.  Loaded the other way round the process ends up with the
    # library's kernels registered in a runtime that PyTorch's streams do not belong to, and every
    # launch fails with hipErrorNoDevice.
    import torch  # noqa: F401
    lib = ctypes.CDLL(LIB_PATH)
    vp, i32, dp = ctypes.c_void_p, ctypes.c_int32, ctypes.POINTER(ReaderDims)
    lib.reader_version.restype = ctypes.c_char_p
    lib.reader_version.argtypes = []
    lib.reader_strerror.restype = ctypes.c_char_p
    lib.reader_strerror.argtypes = [ctypes.c_int]
    lib.reader_last_error_detail.restype = ctypes.c_char_p
    lib.reader_last_error_detail.argtypes = []
    lib.reader_validate_tree.restype = ctypes.c_int
    lib.reader_validate_tree.argtypes = [vp, i32, i32]
    lib.reader_workspace_bytes.restype = ctypes.c_size_t
    lib.reader_workspace_bytes.argtypes = [dp, i32]
    lib.reader_measure_peaks.restype = ctypes.c_int
    lib.reader_measure_peaks.argtypes = [vp, ctypes.c_size_t, vp, ctypes.c_size_t] + [ctypes.POINTER(ctypes.c_double)] * 3 + [vp]
    lib.reader_attn_plan.restype = ctypes.c_int
    lib.reader_attn_plan.argtypes = [dp, i32, ctypes.POINTER(ReaderAttnPlan)]
    lib.reader_tree_attn.restype = ctypes.c_int
    lib.reader_tree_attn.argtypes = [dp] + [vp] * 10 + [i32, vp, ctypes.c_size_t, vp, vp]
    lib.reader_tree_attn_noalloc.restype = ctypes.c_int
    lib.reader_tree_attn_noalloc.argtypes = [dp] + [vp] * 10 + [i32, vp, vp]
    lib.reader_accept_path.restype = ctypes.c_int
    lib.reader_accept_path.argtypes = [dp] + [vp] * 8
    lib.reader_kv_compact.restype = ctypes.c_int
    lib.reader_kv_compact.argtypes = [dp] + [vp] * 10
    lib.reader_verify_step.restype = ctypes.c_int
    lib.reader_verify_step.argtypes = [dp] + [vp] * 15 + [i32, vp, ctypes.c_size_t, vp, vp]
    lib.reader_kv_rearrange_scratch_bytes.restype = ctypes.c_size_t
    lib.reader_kv_rearrange_scratch_bytes.argtypes = [i32, i32]
    lib.reader_kv_rearrange.restype = ctypes.c_int
    lib.reader_kv_rearrange.argtypes = [i32] * 5 + [vp] * 5 + [ctypes.c_size_t, vp]
    lib.reader_target_argmax.restype = ctypes.c_int
    lib.reader_target_argmax.argtypes = [i32, i32, vp, vp, vp]
    i64 = ctypes.c_int64
    lib.reader_trie_create.restype = vp
    lib.reader_trie_create.argtypes = [i32]
    lib.reader_trie_destroy.restype = None
    lib.reader_trie_destroy.argtypes = [vp]
    lib.reader_trie_nodes.restype = i64
    lib.reader_trie_nodes.argtypes = [vp]
    lib.reader_trie_insert.restype = ctypes.c_int
    lib.reader_trie_insert.argtypes = [vp, vp, i64]
    lib.reader_trie_search_path.restype = i32
    lib.reader_trie_search_path.argtypes = [vp, vp, i32, i32, vp]
    lib.reader_trie_extract_tree.restype = i32
    lib.reader_trie_extract_tree.argtypes = [vp, vp, i32, i32, i32, vp, vp]
    lib.reader_tree_attach_path.restype = i32
    lib.reader_tree_attach_path.argtypes = [vp, vp, i32, i32, i32, vp, i32]
    lib.reader_self_repetition.restype = ctypes.c_double
    lib.reader_self_repetition.argtypes = [vp, i64, vp, i64]
    lib.reader_tree_prune_order.restype = i32
    lib.reader_tree_prune_order.argtypes = [vp, vp, i32, vp]
    lib.reader_tree_select.restype = i32
    lib.reader_tree_select.argtypes = [vp, vp, vp, vp, i32, i32, vp, ctypes.POINTER(ctypes.c_double), ctypes.POINTER(i32)]
    lib.reader_kv_compact_layers.restype = ctypes.c_int
    lib.reader_kv_compact_layers.argtypes = [ctypes.POINTER(ReaderDims), i32, vp, vp, vp, vp, vp, vp, vp, vp]
    lib.reader_target_sample.restype = ctypes.c_int
    lib.reader_target_sample.argtypes = [i32, i32, i32, vp, vp, vp, ctypes.c_float, vp, vp]
    lib.reader_profile_enable.restype = ctypes.c_int
    lib.reader_profile_enable.argtypes = [i32]
    lib.reader_profile_collect.restype = ctypes.c_int
    lib.reader_profile_collect.argtypes = [ctypes.POINTER(ctypes.c_double), ctypes.POINTER(i32)]
    lib.reader_profile_collect_each.restype = ctypes.c_int
    lib.reader_profile_collect_each.argtypes = [vp, i32, ctypes.POINTER(i32)]
    lib.reader_tuning_override.restype = ctypes.c_int
    lib.reader_tuning_override.argtypes = [i32, i32]
    _lib = lib
    return lib


def make_dims(B, T, Hq, Hkv, D, max_pages_per_seq, max_path, num_pages, page_size=16, sm_scale=0.0,
              variant=0) -> ReaderDims:
    return ReaderDims(B, T, Hq, Hkv, D, page_size, max_pages_per_seq, max_path, num_pages, sm_scale, variant)


def version() -> str:
    return load().reader_version().decode()


def strerror(code: int) -> str:
    return load().reader_strerror(int(code)).decode()


def _dev(t, dtype=None, optional=False):
    """Device pointer of a contiguous GPU tensor (None -> NULL when optional)."""
    if t is None:
        if optional:
            return None
        raise ValueError("required tensor is None")
    if not t.is_cuda:
        raise ValueError("tensor must live on the GPU")
    if not t.is_contiguous():
        raise ValueError("tensor must be contiguous")
    if dtype is not None and t.dtype != dtype:
        raise ValueError("expected %s, got %s" % (dtype, t.dtype))
    return ctypes.c_void_p(t.data_ptr())


def _stream():
    import torch
    return ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)


def _check(code, where):
    if code != READER_OK:
        raise ReaderError(code, where)


def reader_validate_tree(parents_host) -> int:
    """parents_host: CPU int32 tensor or numpy array [B, T].  Returns the C return code."""
    import numpy as np
    arr = np.ascontiguousarray(parents_host.numpy() if hasattr(parents_host, "numpy") else parents_host,
                               dtype=np.int32)
    B, T = arr.shape
    return int(load().reader_validate_tree(arr.ctypes.data_as(ctypes.c_void_p), B, T))


ATTN_KERNEL_NAMES = {0: "tree_attn_scalar_kernel", 1: "tree_attn_mfma_kernel<D, 4>", 2: "tree_attn_mfma_kernel<D, 8>",
                     3: "tree_attn_wide_kernel<D>"}


def reader_attn_plan(dims: ReaderDims, max_seq_len: int) -> dict:
    """Kernel, rows per workgroup, row chunks and key ranges reader_tree_attn would use (host only)."""
    plan = ReaderAttnPlan()
    _check(load().reader_attn_plan(ctypes.byref(dims), int(max_seq_len), ctypes.byref(plan)), "reader_attn_plan")
    return {"kernel": ATTN_KERNEL_NAMES[int(plan.kernel)].replace("D", str(int(dims.D))), "kernel_id": int(plan.kernel),
            "rows_per_workgroup": int(plan.rows_per_workgroup), "row_chunks": int(plan.row_chunks),
            "key_ranges": int(plan.key_ranges)}


def reader_measure_peaks(src, scratch) -> dict:
    """HBM read rate of a bare LDS copy ring over `src` and the bf16 matrix rate (with the clock under that load)."""
    out = [ctypes.c_double(0.0) for _ in range(3)]
    code = load().reader_measure_peaks(_dev(src), src.numel() * src.element_size(), _dev(scratch),
                                       scratch.numel() * scratch.element_size(), *[ctypes.byref(x) for x in out], _stream())
    _check(code, "reader_measure_peaks")
    return {"hbm_read_gbs": out[0].value, "mfma_bf16_tflops": out[1].value, "mfma_clock_mhz": out[2].value}


def reader_workspace_bytes(dims: ReaderDims, max_seq_len: int) -> int:
    return int(load().reader_workspace_bytes(ctypes.byref(dims), int(max_seq_len)))


def reader_tree_attn(dims, q, k_tree, v_tree, k_cache, v_cache, page_table, seq_lens, parents, out,
                     lse, max_seq_len, workspace, status=None):
    import torch
    ws_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    code = load().reader_tree_attn(
        ctypes.byref(dims), _dev(q, torch.bfloat16), _dev(k_tree, torch.bfloat16, optional=True),
        _dev(v_tree, torch.bfloat16, optional=True),
        _dev(k_cache, torch.bfloat16), _dev(v_cache, torch.bfloat16), _dev(page_table, torch.int32),
        _dev(seq_lens, torch.int32), _dev(parents, torch.int32), _dev(out, torch.bfloat16),
        _dev(lse, torch.float32, optional=True), int(max_seq_len), _dev(workspace, optional=True),
        ws_bytes, _dev(status, torch.int32, optional=True), _stream())
    _check(code, "reader_tree_attn")


NOALLOC_WORKSPACE_BYTES = 40 << 20


def reader_tree_attn_noalloc(dims, q, k_tree, v_tree, k_cache, v_cache, page_table, seq_lens, parents, out, lse,
                             max_seq_len, status=None):
    import torch
    code = load().reader_tree_attn_noalloc(
        ctypes.byref(dims), _dev(q, torch.bfloat16, optional=dims.B == 0), _dev(k_tree, torch.bfloat16, optional=True),
        _dev(v_tree, torch.bfloat16, optional=True),
        _dev(k_cache, torch.bfloat16, optional=dims.B == 0), _dev(v_cache, torch.bfloat16, optional=dims.B == 0),
        _dev(page_table, torch.int32, optional=dims.B == 0), _dev(seq_lens, torch.int32, optional=dims.B == 0),
        _dev(parents, torch.int32, optional=dims.B == 0), _dev(out, torch.bfloat16, optional=dims.B == 0),
        _dev(lse, torch.float32, optional=True), int(max_seq_len), _dev(status, torch.int32, optional=True), _stream())
    _check(code, "reader_tree_attn_noalloc")


def reader_accept_path(dims, draft_tokens, target_tokens, parents, accept_len, path, bonus_token, status=None):
    import torch
    code = load().reader_accept_path(
        ctypes.byref(dims), _dev(draft_tokens, torch.int32), _dev(target_tokens, torch.int32),
        _dev(parents, torch.int32), _dev(accept_len, torch.int32), _dev(path, torch.int32),
        _dev(bonus_token, torch.int32), _dev(status, torch.int32, optional=True), _stream())
    _check(code, "reader_accept_path")


def reader_kv_compact(dims, k_tree, v_tree, path, accept_len, k_cache, v_cache, page_table, seq_lens, status=None):
    import torch
    code = load().reader_kv_compact(
        ctypes.byref(dims), _dev(k_tree, torch.bfloat16), _dev(v_tree, torch.bfloat16), _dev(path, torch.int32),
        _dev(accept_len, torch.int32), _dev(k_cache, torch.bfloat16), _dev(v_cache, torch.bfloat16),
        _dev(page_table, torch.int32), _dev(seq_lens, torch.int32), _dev(status, torch.int32, optional=True),
        _stream())
    _check(code, "reader_kv_compact")


def reader_verify_step(dims, q, k_tree, v_tree, k_cache, v_cache, page_table, seq_lens, parents, draft_tokens,
                       target_tokens, out, lse, accept_len, path, bonus_token, max_seq_len, workspace, status=None):
    import torch
    ws_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    code = load().reader_verify_step(
        ctypes.byref(dims), _dev(q, torch.bfloat16), _dev(k_tree, torch.bfloat16, optional=True),
        _dev(v_tree, torch.bfloat16, optional=True),
        _dev(k_cache, torch.bfloat16), _dev(v_cache, torch.bfloat16), _dev(page_table, torch.int32),
        _dev(seq_lens, torch.int32), _dev(parents, torch.int32), _dev(draft_tokens, torch.int32),
        _dev(target_tokens, torch.int32), _dev(out, torch.bfloat16), _dev(lse, torch.float32, optional=True),
        _dev(accept_len, torch.int32), _dev(path, torch.int32), _dev(bonus_token, torch.int32), int(max_seq_len),
        _dev(workspace, optional=True), ws_bytes, _dev(status, torch.int32, optional=True), _stream())
    _check(code, "reader_verify_step")


def reader_kv_rearrange_scratch_bytes(B: int, S: int) -> int:
    return int(load().reader_kv_rearrange_scratch_bytes(int(B), int(S)))


def reader_kv_rearrange(k_pad, v_pad, valid, new_len, scratch):
    """k_pad, v_pad: bf16 [NL, B, S, Hkv, D] device tensors (in place); valid: uint8 [B, S] (in place);
    new_len: int32 [B] (out); scratch: uint8 device tensor of reader_kv_rearrange_scratch_bytes(B, S)."""
    import torch
    NL, B, S, Hkv, D = k_pad.shape
    assert tuple(v_pad.shape) == (NL, B, S, Hkv, D) and tuple(valid.shape) == (B, S) and tuple(new_len.shape) == (B,)
    code = load().reader_kv_rearrange(
        NL, B, S, Hkv, D, _dev(k_pad, torch.bfloat16), _dev(v_pad, torch.bfloat16), _dev(valid, torch.uint8),
        _dev(new_len, torch.int32), _dev(scratch), scratch.numel() * scratch.element_size(), _stream())
    _check(code, "reader_kv_rearrange")


def reader_target_argmax(logits, target_tokens):
    """logits: bf16 [..., V] device tensor; target_tokens: int32 tensor with one entry per row."""
    import torch
    V = logits.shape[-1]
    rows = logits.numel() // V
    assert target_tokens.numel() == rows
    code = load().reader_target_argmax(rows, V, _dev(logits, torch.bfloat16), _dev(target_tokens, torch.int32), _stream())
    _check(code, "reader_target_argmax")


def reader_kv_compact_layers(dims, path, accept_len, k_cache, v_cache, page_table, seq_lens, status=None):
    """k_cache, v_cache: bf16 [num_layers, num_pages, Hkv, page_size, D] device tensors (moved in place)."""
    import torch
    NL = k_cache.shape[0]
    assert tuple(v_cache.shape) == tuple(k_cache.shape) and k_cache.dim() == 5
    code = load().reader_kv_compact_layers(
        ctypes.byref(dims), NL, _dev(path, torch.int32), _dev(accept_len, torch.int32), _dev(k_cache, torch.bfloat16),
        _dev(v_cache, torch.bfloat16), _dev(page_table, torch.int32), _dev(seq_lens, torch.int32),
        _dev(status, torch.int32, optional=True), _stream())
    _check(code, "reader_kv_compact_layers")


def reader_target_sample(logits, parents, uniforms, temperature, target_tokens):
    """logits: bf16 [B, T, V]; parents: int32 [B, T]; uniforms: float32 [B, T]; target_tokens: int32 [B, T]."""
    import torch
    B, T, V = logits.shape
    assert tuple(parents.shape) == (B, T) and tuple(uniforms.shape) == (B, T) and tuple(target_tokens.shape) == (B, T)
    code = load().reader_target_sample(B, T, V, _dev(logits, torch.bfloat16), _dev(parents, torch.int32),
                                       _dev(uniforms, torch.float32), float(temperature),
                                       _dev(target_tokens, torch.int32), _stream())
    _check(code, "reader_target_sample")


def _host_i32(a):
    import numpy as np
    a = np.ascontiguousarray(a, dtype=np.int32)
    return a, ctypes.c_void_p(a.ctypes.data)


class Trie:
    """The host-side n-gram trie of the retrieval drafter (numpy int32 arrays in, numpy arrays out)."""

    def __init__(self, max_depth: int):
        self._h = load().reader_trie_create(int(max_depth))
        if not self._h:
            raise ValueError("reader_trie_create refused max_depth=%r" % (max_depth,))

    def close(self):
        if self._h:
            load().reader_trie_destroy(self._h)
            self._h = None

    __del__ = close

    def __len__(self):
        return int(load().reader_trie_nodes(self._h))

    def insert(self, tokens):
        a, p = _host_i32(tokens)
        _check(load().reader_trie_insert(self._h, p, a.size), "reader_trie_insert")

    def search_path(self, suffix, depth: int):
        import numpy as np
        a, p = _host_i32(suffix)
        out = np.zeros(max(int(depth), 1), dtype=np.int32)
        k = load().reader_trie_search_path(self._h, p, a.size, int(depth), ctypes.c_void_p(out.ctypes.data))
        if k < 0:
            raise ValueError("reader_trie_search_path: bad argument")
        return out[:k].copy()

    def extract_tree(self, suffix, max_depth: int, budget: int):
        import numpy as np
        a, p = _host_i32(suffix)
        tokens = np.zeros(max(int(budget), 1), dtype=np.int32)
        parents = np.zeros(max(int(budget), 1), dtype=np.int32)
        n = load().reader_trie_extract_tree(self._h, p, a.size, int(max_depth), int(budget),
                                            ctypes.c_void_p(tokens.ctypes.data), ctypes.c_void_p(parents.ctypes.data))
        if n < 0:
            raise ValueError("reader_trie_extract_tree: bad argument")
        return tokens[:n].copy(), parents[:n].copy()


def reader_tree_attach_path(tokens, parents, n_nodes: int, at_node: int, path_tokens) -> int:
    """tokens, parents: writable numpy int32 arrays of equal capacity; returns the new node count."""
    import numpy as np
    assert tokens.dtype == np.int32 and parents.dtype == np.int32 and tokens.size == parents.size
    a, p = _host_i32(path_tokens)
    n = load().reader_tree_attach_path(ctypes.c_void_p(tokens.ctypes.data), ctypes.c_void_p(parents.ctypes.data),
                                       int(n_nodes), tokens.size, int(at_node), p, a.size)
    if n < 0:
        raise ValueError("reader_tree_attach_path: bad argument")
    return int(n)


def _host_f32(a):
    import numpy as np
    a = np.ascontiguousarray(a, dtype=np.float32)
    return a, ctypes.c_void_p(a.ctypes.data)


def reader_tree_prune_order(parents, alpha):
    """Removal order of Appendix E (numpy int32 array of T - 1 node ids)."""
    import numpy as np
    par, pp = _host_i32(parents)
    al, pa = _host_f32(alpha)
    order = np.zeros(max(par.size - 1, 1), dtype=np.int32)
    n = load().reader_tree_prune_order(pp, pa, par.size, ctypes.c_void_p(order.ctypes.data))
    if n < 0:
        raise ValueError("reader_tree_prune_order: bad argument")
    return order[:n].copy()


def reader_tree_select(parents, alpha, t_draft, tv, exhaustive=False):
    """Returns (n_star, keep mask as numpy bool [T], modelled throughput, trees scored)."""
    import numpy as np
    par, pp = _host_i32(parents)
    al, pa = _host_f32(alpha)
    td, pt = _host_f32(t_draft)
    tvv, pv = _host_f32(tv)
    assert al.size == par.size and td.size == par.size and tvv.size == par.size
    keep = np.zeros(par.size, dtype=np.int32)
    thr, ev = ctypes.c_double(0.0), ctypes.c_int32(0)
    n = load().reader_tree_select(pp, pa, pt, pv, par.size, 1 if exhaustive else 0, ctypes.c_void_p(keep.ctypes.data),
                                  ctypes.byref(thr), ctypes.byref(ev))
    if n < 0:
        raise ValueError("reader_tree_select: bad argument")
    return int(n), keep.astype(bool), float(thr.value), int(ev.value)


def reader_self_repetition(prompt, response) -> float:
    a, pa = _host_i32(prompt)
    b, pb = _host_i32(response)
    r = load().reader_self_repetition(pa, a.size, pb, b.size)
    if r < 0:
        raise ValueError("reader_self_repetition: bad argument")
    return float(r)


def reader_tuning_override(which: int, value: int) -> None:
    """Planner override for tests and experiments (a negative value clears it)."""
    _check(load().reader_tuning_override(int(which), int(value)), "reader_tuning_override")


def reader_profile_enable(on: bool) -> None:
    _check(load().reader_profile_enable(1 if on else 0), "reader_profile_enable")


def reader_profile_collect_each(capacity: int = 65536):
    """Times (ms) of the main attention kernel's launches since the last collect, in launch order (numpy float32)."""
    import numpy as np
    out = np.zeros(int(capacity), dtype=np.float32)
    n = ctypes.c_int32(0)
    _check(load().reader_profile_collect_each(ctypes.c_void_p(out.ctypes.data), int(capacity), ctypes.byref(n)),
           "reader_profile_collect_each")
    return out[:min(int(n.value), int(capacity))].copy()


def reader_profile_collect():
    """Returns (sum of main-kernel milliseconds, number of timed launches) since the last collect."""
    ms, n = ctypes.c_double(0.0), ctypes.c_int32(0)
    _check(load().reader_profile_collect(ctypes.byref(ms), ctypes.byref(n)), "reader_profile_collect")
    return ms.value, n.value


# ------------------------------------------------------------------ convenience (allocation only)

@dataclasses.dataclass
class DeviceWorkload:
    """A workload's arrays as GPU tensors plus the buffers the three calls write."""
    dims: ReaderDims
    max_seq_len: int
    q: object
    k_tree: object
    v_tree: object
    k_cache: object
    v_cache: object
    page_table: object
    seq_lens: object
    parents: object
    draft_tokens: object
    target_tokens: object
    out: object
    lse: object
    accept_len: object
    path: object
    bonus: object
    status: object
    workspace: object


def to_device(w, device="cuda:0", variant=0, sm_scale=0.0) -> DeviceWorkload:
    """Upload a workloads.Workload (numpy) and allocate outputs and workspace.  No arithmetic."""
    import numpy as np
    import torch

    def bf16(a):
        return torch.from_numpy(a.view(np.int16)).to(device).view(torch.bfloat16)

    def i32(a):
        return torch.from_numpy(np.ascontiguousarray(a, dtype=np.int32)).to(device)

    # a bound with room for one accepted path, so that the same buffers serve a second step
    max_seq_len = (int(w.seq_lens.max()) + w.max_path) if w.B else 0
    dims = make_dims(w.B, w.T, w.Hq, w.Hkv, w.D, w.max_pages, w.max_path, w.num_pages,
                     page_size=w.page_size, sm_scale=sm_scale, variant=variant)
    ws = reader_workspace_bytes(dims, max_seq_len)
    return DeviceWorkload(
        dims=dims, max_seq_len=max_seq_len,
        q=bf16(w.q), k_tree=bf16(w.k_tree), v_tree=bf16(w.v_tree), k_cache=bf16(w.k_cache), v_cache=bf16(w.v_cache),
        page_table=i32(w.page_table), seq_lens=i32(w.seq_lens), parents=i32(w.parents),
        draft_tokens=i32(w.draft_tokens), target_tokens=i32(w.target_tokens),
        out=torch.empty((w.B, w.T, w.Hq, w.D), dtype=torch.bfloat16, device=device),
        lse=torch.empty((w.B, w.Hq, w.T), dtype=torch.float32, device=device),
        accept_len=torch.empty((w.B,), dtype=torch.int32, device=device),
        path=torch.empty((w.B, w.max_path), dtype=torch.int32, device=device),
        bonus=torch.empty((w.B,), dtype=torch.int32, device=device),
        status=torch.zeros((1,), dtype=torch.int32, device=device),
        workspace=torch.empty((max(ws, 256),), dtype=torch.uint8, device=device),
    )

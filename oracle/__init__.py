"""CPU oracle for READER's draft-tree verification step -- TEST INFRASTRUCTURE ONLY.

Thin ctypes loader around ``reader_oracle.c`` (plain C, IEEE double arithmetic, no
tiling, explicit masks), plus the functions written directly in numpy at the end of this
file (``target_sample``, ``kv_compact_layers``) and the brute-force drafter oracle in
``oracle/drafter.py``.  Only the tests, ``__graft_entry__.smoke()`` and the
``cpu_baseline`` leg of ``bench.py`` may import this package; the product package
never does, and this package never imports the product package.

All arrays are numpy, C-contiguous.  bf16 tensors are passed as ``uint16`` bit
patterns.  Layouts are the ones listed at the top of ``reader_oracle.c``.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "reader_oracle.c")
_LIB = os.path.join(_HERE, "libreader_oracle.so")
_lib = None


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (-O2, OpenMP over independent (sequence, kv head) pairs)."""
    stale = (not os.path.exists(_LIB)) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC)
    if force or stale:
        tmp = _LIB + ".tmp.%d" % os.getpid()
        subprocess.run(
            ["gcc", "-O2", "-fopenmp", "-fPIC", "-shared", "-std=c11", "-Wall", "-Wextra",
             _SRC, "-o", tmp, "-lm"],
            check=True,
        )
        os.replace(tmp, _LIB)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        build()
        _lib = ctypes.CDLL(_LIB)
    return _lib


def _p(a, dtype):
    assert isinstance(a, np.ndarray) and a.dtype == dtype and a.flags["C_CONTIGUOUS"], (
        "expected C-contiguous %s array, got %r %r" % (dtype, getattr(a, "dtype", None), type(a)))
    return a.ctypes.data_as(ctypes.c_void_p)


def num_threads() -> int:
    return int(_load().oracle_num_threads())


def ancestor_mask(parents: np.ndarray):
    """parents: int32 [T].  Returns (mask uint8 [T, T] with mask[query, key], depth int32 [T])."""
    parents = np.ascontiguousarray(parents, dtype=np.int32)
    T = parents.shape[0]
    mask = np.zeros((T, T), dtype=np.uint8)
    depth = np.zeros(T, dtype=np.int32)
    rc = _load().oracle_ancestor_mask(_p(parents, np.int32), T, _p(mask, np.uint8), _p(depth, np.int32))
    if rc:
        raise ValueError("oracle_ancestor_mask: malformed tree (rc=%d)" % rc)
    return mask, depth


def _attn_common(q, k_tree, v_tree, k_cache, v_cache, page_table, seq_lens, parents):
    B, T, Hq, D = q.shape
    Hkv = k_tree.shape[2]
    assert k_tree.shape == (B, T, Hkv, D) and v_tree.shape == (B, T, Hkv, D)
    num_pages, Hkv2, page_size, D2 = k_cache.shape
    assert Hkv2 == Hkv and D2 == D and v_cache.shape == k_cache.shape
    assert page_table.shape[0] == B and seq_lens.shape == (B,) and parents.shape == (B, T)
    if B:
        used = (seq_lens.astype(np.int64) + page_size - 1) // page_size
        for b in range(B):
            pt = page_table[b, : used[b]]
            assert pt.size == 0 or (pt.min() >= 0 and pt.max() < num_pages), "page table out of range"
    return B, T, Hq, Hkv, D, page_size, page_table.shape[1]


def tree_attn(q, k_tree, v_tree, k_cache, v_cache, page_table, seq_lens, parents, sm_scale=0.0):
    """Tree-masked attention (Section 3.2).  Returns (out float64 [B,T,Hq,D], lse float64 [B,Hq,T])."""
    B, T, Hq, Hkv, D, page_size, max_pages = _attn_common(
        q, k_tree, v_tree, k_cache, v_cache, page_table, seq_lens, parents)
    out = np.zeros((B, T, Hq, D), dtype=np.float64)
    lse = np.zeros((B, Hq, T), dtype=np.float64)
    rc = _load().oracle_tree_attn(
        B, T, Hq, Hkv, D, page_size, max_pages, ctypes.c_double(sm_scale),
        _p(q, np.uint16), _p(k_tree, np.uint16), _p(v_tree, np.uint16),
        _p(k_cache, np.uint16), _p(v_cache, np.uint16), _p(page_table, np.int32),
        _p(seq_lens, np.int32), _p(parents, np.int32), _p(out, np.float64), _p(lse, np.float64))
    if rc:
        raise ValueError("oracle_tree_attn failed (rc=%d)" % rc)
    return out, lse


def tree_attn_rows(q, k_tree, v_tree, k_cache, v_cache, page_table, seq_lens, parents, rows,
                   sm_scale=0.0):
    """Same, for selected (b, hq, node) triples.  rows int32 [n,3] -> (out [n,D], lse [n])."""
    B, T, Hq, Hkv, D, page_size, max_pages = _attn_common(
        q, k_tree, v_tree, k_cache, v_cache, page_table, seq_lens, parents)
    rows = np.ascontiguousarray(rows, dtype=np.int32).reshape(-1, 3)
    n = rows.shape[0]
    out = np.zeros((n, D), dtype=np.float64)
    lse = np.zeros((n,), dtype=np.float64)
    rc = _load().oracle_tree_attn_rows(
        B, T, Hq, Hkv, D, page_size, max_pages, ctypes.c_double(sm_scale),
        _p(q, np.uint16), _p(k_tree, np.uint16), _p(v_tree, np.uint16),
        _p(k_cache, np.uint16), _p(v_cache, np.uint16), _p(page_table, np.int32),
        _p(seq_lens, np.int32), _p(parents, np.int32), n, _p(rows, np.int32),
        _p(out, np.float64), _p(lse, np.float64))
    if rc:
        raise ValueError("oracle_tree_attn_rows failed (rc=%d)" % rc)
    return out, lse


def accept_path(draft_tokens, target_tokens, parents, max_path):
    """Greedy lossless acceptance (Algorithm 5).  Returns (accept_len [B], path [B,max_path], bonus [B])."""
    B, T = parents.shape
    assert draft_tokens.shape == (B, T) and target_tokens.shape == (B, T)
    accept_len = np.zeros(B, dtype=np.int32)
    path = np.full((B, max_path), -1, dtype=np.int32)
    bonus = np.zeros(B, dtype=np.int32)
    rc = _load().oracle_accept_path(
        B, T, int(max_path), _p(draft_tokens, np.int32), _p(target_tokens, np.int32),
        _p(parents, np.int32), _p(accept_len, np.int32), _p(path, np.int32), _p(bonus, np.int32))
    if rc:
        raise ValueError("oracle_accept_path failed (rc=%d)" % rc)
    return accept_len, path, bonus


def kv_compact(k_tree, v_tree, path, accept_len, k_cache, v_cache, page_table, seq_lens):
    """Append the accepted path's K/V rows to each sequence's paged cache IN PLACE
    (Section 4.3 / Algorithm 4); seq_lens is updated in place."""
    B, T, Hkv, D = k_tree.shape
    num_pages, Hkv2, page_size, D2 = k_cache.shape
    assert (Hkv2, D2) == (Hkv, D) and v_cache.shape == k_cache.shape and v_tree.shape == k_tree.shape
    max_path = path.shape[1]
    if B:
        used = (seq_lens.astype(np.int64) + accept_len + 1 + page_size - 1) // page_size
        for b in range(B):
            pt = page_table[b, : used[b]]
            assert pt.min() >= 0 and pt.max() < num_pages, "page table out of range"
    rc = _load().oracle_kv_compact(
        B, T, Hkv, D, page_size, page_table.shape[1], max_path,
        _p(k_tree, np.uint16), _p(v_tree, np.uint16), _p(path, np.int32), _p(accept_len, np.int32),
        _p(k_cache, np.uint16), _p(v_cache, np.uint16), _p(page_table, np.int32), _p(seq_lens, np.int32))
    if rc:
        raise ValueError("oracle_kv_compact failed (rc=%d)" % rc)


def kv_rearrange(k_pad, v_pad, valid):
    """Periodic rearrangement of a padded cache IN PLACE (Section 4.3 / Algorithm 4).

    k_pad, v_pad: uint16 (bf16 bits) [NL, B, S, Hkv, D]; valid: uint8 [B, S], updated in place.
    Returns new_len int32 [B]."""
    NL, B, S, Hkv, D = k_pad.shape
    assert v_pad.shape == k_pad.shape and valid.shape == (B, S)
    new_len = np.zeros(B, dtype=np.int32)
    rc = _load().oracle_kv_rearrange(NL, B, S, Hkv, D, _p(k_pad, np.uint16), _p(v_pad, np.uint16),
                                     _p(valid, np.uint8), _p(new_len, np.int32))
    if rc:
        raise ValueError("oracle_kv_rearrange failed (rc=%d)" % rc)
    return new_len


def target_argmax(logits):
    """logits: uint16 (bf16 bits) [..., V].  Returns int32 [...] greedy tokens (Algorithm 5)."""
    V = logits.shape[-1]
    rows = logits.size // V
    out = np.zeros(rows, dtype=np.int32)
    rc = _load().oracle_target_argmax(rows, V, _p(logits, np.uint16), _p(out, np.int32))
    if rc:
        raise ValueError("oracle_target_argmax failed (rc=%d)" % rc)
    return out.reshape(logits.shape[:-1])



def _bf16_bits_to_f64(bits):
    return (bits.astype(np.uint32) << 16).view(np.float32).astype(np.float64)


def _softmax_weights(x, temperature):
    """exp((x - max) / temperature) for a row without NaNs.  A row of nothing but -inf has no
    weight anywhere; +inf logits take all the weight, one unit each (the limit of the softmax)."""
    m = x.max()
    if m == np.inf:
        return (x == np.inf).astype(np.float64)
    if m == -np.inf:
        return np.zeros(x.shape[0])
    return np.exp((x - m) / temperature)


def target_sample(logits, parents, uniforms, temperature=1.0, with_cdf=False):
    """The base model's tokens under a sampling policy (Appendix C, randomized decoding):
    the policy is a map F(distribution, u) with one uniform u per decoding position, and the
    speculative run uses the same uniforms as the plain run.  Here F is inverse-CDF sampling
    of softmax(logits / temperature): the token is the lowest index k whose cumulative
    probability exceeds u.  Node n of sequence b stands for the position depth(n) behind the
    root, so every node of one depth draws with the same uniform: u = uniforms[b, depth(n)].

    logits: uint16 (bf16 bits) [B, T, V]; parents: int32 [B, T]; uniforms: float [B, T] in
    [0, 1).  A NaN logit carries no probability.  Returns int32 [B, T]; with_cdf=True also
    returns, per node, (threshold, total) = (u * sum of weights, sum of weights) and the row's
    cumulative weights are recomputable from them (used by tolerance checks in tests).
    Plain numpy in double precision, one row at a time, nothing blocked or fused."""
    B, T, V = logits.shape
    assert parents.shape == (B, T) and uniforms.shape == (B, T) and temperature > 0
    out = np.zeros((B, T), dtype=np.int32)
    thr = np.zeros((B, T), dtype=np.float64)
    tot = np.zeros((B, T), dtype=np.float64)
    for b in range(B):
        _, depth = ancestor_mask(np.ascontiguousarray(parents[b], dtype=np.int32))
        for n in range(T):
            x = _bf16_bits_to_f64(logits[b, n])
            x = np.where(np.isnan(x), -np.inf, x)
            w = _softmax_weights(x, temperature)
            cdf = np.cumsum(w)
            t = float(uniforms[b, depth[n]]) * cdf[-1]
            k = int(np.searchsorted(cdf, t, side="right"))      # first index with cdf > t
            if k >= V:                                            # u * total rounded up to the total
                k = int(np.flatnonzero(w > 0)[-1]) if cdf[-1] > 0 else 0
            out[b, n], thr[b, n], tot[b, n] = k, t, cdf[-1]
    return (out, thr, tot) if with_cdf else out


def target_sample_weights(logits_row, temperature=1.0):
    """Cumulative weights of one row as target_sample forms them (double precision)."""
    x = _bf16_bits_to_f64(logits_row)
    x = np.where(np.isnan(x), -np.inf, x)
    return np.cumsum(_softmax_weights(x, temperature))


def kv_compact_layers(k_cache, v_cache, path, accept_len, page_table, seq_lens):
    """Compaction for the in-cache layout, all layers at once, IN PLACE (Section 4.3 /
    Algorithm 4 applied every step).  During the step every layer wrote the K/V rows of the
    draft tree behind the sequence: node n of sequence b sits at position seq_lens[b] + n.
    Afterwards the accepted path becomes the sequence's next rows: for j = 0..accept_len[b]
    position seq_lens[b] + j receives what position seq_lens[b] + path[b][j] held BEFORE the
    pass, in every layer, K and V, all heads; then seq_lens[b] += accept_len[b] + 1.  Rows
    behind the new length keep whatever they held (the next step overwrites them).

    k_cache, v_cache: uint16 (bf16 bits) [NL, num_pages, Hkv, page_size, D]; path int32
    [B, max_path]; accept_len int32 [B]; page_table int32 [B, max_pages]; seq_lens int32 [B].
    The definition written out with numpy indexing: gather the old rows, then scatter."""
    NL, num_pages, Hkv, page_size, D = k_cache.shape
    assert v_cache.shape == k_cache.shape
    B = path.shape[0]
    for b in range(B):
        L, n = int(seq_lens[b]), int(accept_len[b])
        nodes = path[b, : n + 1].astype(np.int64)
        assert nodes[0] == 0 and np.all(np.diff(nodes) > 0), "a path runs from the root through increasing node ids"
        src = L + nodes
        dst = L + np.arange(n + 1)
        sp, ss = page_table[b, src // page_size], src % page_size
        dp, ds = page_table[b, dst // page_size], dst % page_size
        assert sp.min() >= 0 and dp.min() >= 0 and max(sp.max(), dp.max()) < num_pages, "page table out of range"
        for cache in (k_cache, v_cache):
            old = cache[:, sp, :, ss, :].copy()          # [rows, NL, Hkv, D] (advanced indices first)
            cache[:, dp, :, ds, :] = old
        seq_lens[b] = L + n + 1

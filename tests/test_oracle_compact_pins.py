"""Pins for the oracle's KV compaction (Section 4.3, Algorithm 4): after the pass each
sample's cache is its old content followed tightly by the accepted span, and nothing
else has moved.  CPU only."""
import numpy as np

from paper_2508_09072_amd import workloads as W
from helpers import f64, flat_prefix, flat_sequence_row


def snapshot(w):
    return w.k_cache.copy(), w.v_cache.copy(), w.seq_lens.copy()


def test_equals_an_index_gather_and_touches_nothing_else(oracle_mod):
    w = W.make_custom("compact", B=5, Hq=4, Hkv=2, D=16, T=12, seq_lens=[0, 15, 16, 17, 60],
                      tree="trie", depth=5, branch=2, vocab=6, p_match=0.8, seed=31)
    al, path, bonus = oracle_mod.accept_path(w.draft_tokens, w.target_tokens, w.parents, w.max_path)
    assert al.max() >= 2                     # at least one span crosses into a fresh page region
    k0, v0, L0 = snapshot(w)
    oracle_mod.kv_compact(w.k_tree, w.v_tree, path, al, w.k_cache, w.v_cache, w.page_table, w.seq_lens)
    assert (w.seq_lens == L0 + al + 1).all()
    # expected caches by numpy fancy indexing, written independently of the oracle's loops
    ek, ev = k0.copy(), v0.copy()
    for b in range(w.B):
        pos = L0[b] + np.arange(al[b] + 1)
        pages = w.page_table[b, pos // w.page_size]
        ek[pages, :, pos % w.page_size, :] = w.k_tree[b, path[b, : al[b] + 1]]
        ev[pages, :, pos % w.page_size, :] = w.v_tree[b, path[b, : al[b] + 1]]
    assert np.array_equal(w.k_cache, ek) and np.array_equal(w.v_cache, ev)
    # the number of changed slots is exactly the number of appended rows
    changed = (w.k_cache != k0).any(axis=(1, 3)).sum()
    assert changed == int((al + 1).sum())


def test_result_is_tight_concatenation(oracle_mod):
    # "zeros may only remain at the end": the logical cache is old prefix || accepted rows,
    # and every slot behind it still holds the canary.
    w = W.make_custom("tight", B=3, Hq=2, Hkv=2, D=8, T=8, seq_lens=[30, 31, 32], tree="chain",
                      vocab=2, p_match=0.9, seed=32)
    al, path, _ = oracle_mod.accept_path(w.draft_tokens, w.target_tokens, w.parents, w.max_path)
    old = [[flat_prefix(w, c, b, h) for h in range(w.Hkv)] for c in (w.k_cache, w.v_cache) for b in range(w.B)]
    L0 = w.seq_lens.copy()
    oracle_mod.kv_compact(w.k_tree, w.v_tree, path, al, w.k_cache, w.v_cache, w.page_table, w.seq_lens)
    idx = 0
    for cache, tree in ((w.k_cache, w.k_tree), (w.v_cache, w.v_tree)):
        for b in range(w.B):
            for h in range(w.Hkv):
                now = flat_prefix(w, cache, b, h)
                assert now.shape[0] == L0[b] + al[b] + 1
                assert np.array_equal(now[: L0[b]], old[idx][h])
                assert np.array_equal(now[L0[b]:], f64(tree[b, path[b, : al[b] + 1], h]))
            idx += 1
    for b in range(w.B):
        mapped = w.page_table[b][w.page_table[b] >= 0]
        flat = w.k_cache[mapped].transpose(0, 2, 1, 3).reshape(-1, w.Hkv, w.D)
        assert (flat[w.seq_lens[b]:] == W.CANARY).all()


def test_next_step_sees_the_compacted_rows(oracle_mod):
    # End to end: after compaction a one-node tree attends over old prefix || accepted path,
    # which must equal decoding along that path on the *uncompacted* inputs.
    w = W.make_custom("e2e", B=2, Hq=4, Hkv=2, D=16, T=10, seq_lens=[21, 47], tree="trie", depth=4,
                      branch=2, vocab=4, p_match=0.9, seed=33)
    al, path, _ = oracle_mod.accept_path(w.draft_tokens, w.target_tokens, w.parents, w.max_path)
    assert al.max() >= 1
    # reference before mutation: the terminal node's own attention row
    refs = [[flat_sequence_row(w, b, hq, int(path[b, al[b]]))[0] for hq in range(w.Hq)] for b in range(w.B)]
    last_q = np.stack([w.q[b, path[b, al[b]]] for b in range(w.B)])[:, None]
    last_k = np.stack([w.k_tree[b, path[b, al[b]]] for b in range(w.B)])[:, None]
    last_v = np.stack([w.v_tree[b, path[b, al[b]]] for b in range(w.B)])[:, None]
    oracle_mod.kv_compact(w.k_tree, w.v_tree, path, al, w.k_cache, w.v_cache, w.page_table, w.seq_lens)
    # the terminal row is now the last cached row; query it again as a one-node tree whose
    # own key is that same row, over a prefix that excludes it
    short = (w.seq_lens - 1).astype(np.int32)
    out, _ = oracle_mod.tree_attn(np.ascontiguousarray(last_q), np.ascontiguousarray(last_k),
                                  np.ascontiguousarray(last_v), w.k_cache, w.v_cache, w.page_table,
                                  short, np.full((w.B, 1), -1, dtype=np.int32))
    for b in range(w.B):
        for hq in range(w.Hq):
            np.testing.assert_allclose(out[b, 0, hq], refs[b][hq], rtol=1e-9, atol=1e-11)


def test_empty_accept_still_appends_the_root(oracle_mod):
    w = W.make_custom("empty", B=1, Hq=1, Hkv=1, D=8, T=3, seq_lens=[15], tree="chain", p_match=0.0, seed=34)
    al, path, _ = oracle_mod.accept_path(w.draft_tokens, w.target_tokens, w.parents, w.max_path)
    assert al[0] == 0
    oracle_mod.kv_compact(w.k_tree, w.v_tree, path, al, w.k_cache, w.v_cache, w.page_table, w.seq_lens)
    assert w.seq_lens[0] == 16
    assert np.array_equal(flat_prefix(w, w.k_cache, 0, 0)[15], f64(w.k_tree[0, 0, 0]))

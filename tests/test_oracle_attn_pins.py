"""Pins for the oracle's tree-masked attention against things the paper and the
mathematics fix (Section 3.2; Appendix C invariant 2).  CPU only.

Each test is chosen so that one plausible mistake in the oracle fails it: a
transposed mask, a missing diagonal, a dropped scale, a wrong GQA group, a wrong
page slot, a softmax that is not normalised.
"""
import numpy as np
import pytest
import torch

from paper_2508_09072_amd import workloads as W
from helpers import f64, flat_prefix, flat_sequence_row, visible_sets, root_path

TOL = dict(rtol=1e-9, atol=1e-11)


def run(oracle_mod, w, **kw):
    return oracle_mod.tree_attn(w.q, w.k_tree, w.v_tree, w.k_cache, w.v_cache, w.page_table,
                                w.seq_lens, w.parents, **kw)


def test_mask_is_ancestor_or_self(oracle_mod):
    # Section 3.2: M_ij = 1 iff i is an ancestor of j; the query index is the column there,
    # the row here, and a node always sees itself.
    rng = np.random.Generator(np.random.PCG64(7))
    for T in (1, 2, 5, 16, 33, 128):
        par = W.tree_uniform(rng, T, max_depth=9)
        mask, depth = oracle_mod.ancestor_mask(par)
        vis = visible_sets(par)
        for i in range(T):
            assert set(np.nonzero(mask[i])[0].tolist()) == vis[i]
            assert depth[i] == len(vis[i]) - 1
    # hand case: 0 -> 1 -> 3, 0 -> 2
    mask, depth = oracle_mod.ancestor_mask(np.asarray([-1, 0, 0, 1], dtype=np.int32))
    assert mask.tolist() == [[1, 0, 0, 0], [1, 1, 0, 0], [1, 0, 1, 0], [1, 1, 0, 1]]
    assert depth.tolist() == [0, 1, 1, 2]


def test_malformed_trees_rejected(oracle_mod):
    for bad in ([0, 0, 1], [-1, -1, 0], [-1, 1, 0], [-1, 0, 2], [-1, 0, 5]):
        with pytest.raises(ValueError):
            oracle_mod.ancestor_mask(np.asarray(bad, dtype=np.int32))


@pytest.mark.parametrize("L", [0, 1, 37, 130])
def test_chain_tree_is_causal_attention(oracle_mod, L):
    # A chain is ordinary causal decoding of T more tokens: compare with the library's
    # scaled_dot_product_attention under a lower-triangular mask on the flat sequence.
    w = W.make_custom("chain", B=2, Hq=4, Hkv=2, D=32, T=9, seq_lens=[L, L + 3], tree="chain", seed=11)
    out, lse = run(oracle_mod, w)
    G = w.Hq // w.Hkv
    for b in range(w.B):
        Lb = int(w.seq_lens[b])
        for hq in range(w.Hq):
            hkv = hq // G
            K = np.concatenate([flat_prefix(w, w.k_cache, b, hkv), f64(w.k_tree[b, :, hkv])])
            V = np.concatenate([flat_prefix(w, w.v_cache, b, hkv), f64(w.v_tree[b, :, hkv])])
            Q = f64(w.q[b, :, hq])
            n = Lb + w.T
            causal = torch.ones(n, n, dtype=torch.bool).tril()[Lb:]
            ref = torch.nn.functional.scaled_dot_product_attention(
                torch.from_numpy(Q)[None, None], torch.from_numpy(K)[None, None],
                torch.from_numpy(V)[None, None], attn_mask=causal[None, None])[0, 0].numpy()
            np.testing.assert_allclose(out[b, :, hq], ref, **TOL)


def test_single_node_tree_is_plain_decode(oracle_mod):
    # T = 1: one query over L prefix keys plus its own key, no mask at all.
    w = W.make_custom("decode", B=3, Hq=6, Hkv=2, D=64, T=1, seq_lens=[50, 0, 17], tree="chain", seed=5)
    out, lse = run(oracle_mod, w)
    for b in range(w.B):
        for hq in range(w.Hq):
            hkv = hq // 3
            K = np.concatenate([flat_prefix(w, w.k_cache, b, hkv), f64(w.k_tree[b, :, hkv])])
            V = np.concatenate([flat_prefix(w, w.v_cache, b, hkv), f64(w.v_tree[b, :, hkv])])
            Q = f64(w.q[b, :, hq])
            ref = torch.nn.functional.scaled_dot_product_attention(
                torch.from_numpy(Q)[None, None], torch.from_numpy(K)[None, None],
                torch.from_numpy(V)[None, None])[0, 0].numpy()
            np.testing.assert_allclose(out[b, :, hq], ref, **TOL)
            s = (K @ Q[0]) / np.sqrt(w.D)
            np.testing.assert_allclose(lse[b, hq, 0], np.log(np.exp(s).sum()), rtol=1e-10)


@pytest.mark.parametrize("tree,T", [("uniform", 12), ("trie", 20), ("star", 7)])
def test_each_node_equals_decoding_along_its_path(oracle_mod, tree, T):
    # Appendix C invariant 2: brute force over root-to-node paths on small inputs.
    w = W.make_custom("bf", B=2, Hq=4, Hkv=2, D=16, T=T, seq_lens=[23, 40], tree=tree, depth=5,
                      branch=3, seed=3)
    out, lse = run(oracle_mod, w)
    for b in range(w.B):
        for hq in range(w.Hq):
            for i in range(w.T):
                ref, ref_lse = flat_sequence_row(w, b, hq, i)
                np.testing.assert_allclose(out[b, i, hq], ref, **TOL)
                np.testing.assert_allclose(lse[b, hq, i], ref_lse, rtol=1e-10)


def test_zero_query_gives_mean_of_visible_values(oracle_mod):
    # Closed form: q = 0 makes every visible key equally likely, so the output is the
    # plain mean of the value rows of prefix + ancestors-or-self, and lse = log(count).
    w = W.make_custom("mean", B=1, Hq=2, Hkv=1, D=8, T=10, seq_lens=[5], tree="uniform", depth=4, seed=9)
    w.q[:] = 0
    out, lse = run(oracle_mod, w)
    vis = visible_sets(w.parents[0])
    P = flat_prefix(w, w.v_cache, 0, 0)
    for i in range(w.T):
        rows = np.concatenate([P, f64(w.v_tree[0, sorted(vis[i]), 0])])
        for hq in range(w.Hq):
            np.testing.assert_allclose(out[0, i, hq], rows.mean(0), **TOL)
            np.testing.assert_allclose(lse[0, hq, i], np.log(len(rows)), rtol=1e-12)


def test_constant_values_give_constant_output(oracle_mod):
    w = W.make_custom("const", B=1, Hq=4, Hkv=4, D=16, T=6, seq_lens=[33], tree="trie", depth=3, seed=2)
    c = W.to_bf16_bits(np.asarray([1.5], dtype=np.float32))[0]
    w.v_cache[:] = c
    w.v_tree[:] = c
    out, _ = run(oracle_mod, w)
    np.testing.assert_allclose(out, 1.5, rtol=1e-12)


def test_scale_is_one_over_sqrt_d_and_is_settable(oracle_mod):
    # One prefix key and the root: out = sigmoid-weighted mix; the weight pins the scale.
    w = W.make_custom("scale", B=1, Hq=1, Hkv=1, D=4, T=1, seq_lens=[1], tree="chain", seed=1)
    q = f64(w.q[0, 0, 0]); k0 = flat_prefix(w, w.k_cache, 0, 0)[0]; k1 = f64(w.k_tree[0, 0, 0])
    v0 = flat_prefix(w, w.v_cache, 0, 0)[0]; v1 = f64(w.v_tree[0, 0, 0])
    for scale_arg, scale in ((0.0, 0.5), (0.3, 0.3)):
        out, _ = run(oracle_mod, w, sm_scale=scale_arg)
        a = 1.0 / (1.0 + np.exp(scale * (q @ k1 - q @ k0)))     # weight of the prefix key
        np.testing.assert_allclose(out[0, 0, 0], a * v0 + (1 - a) * v1, **TOL)


def test_page_order_does_not_matter(oracle_mod):
    a = W.make_custom("pages", B=2, Hq=4, Hkv=2, D=16, T=8, seq_lens=[45, 70], seed=4, shuffle_pages=False)
    out_a, lse_a = run(oracle_mod, a)
    # same logical content under another physical page permutation
    rng = np.random.Generator(np.random.PCG64(99))
    perm = rng.permutation(a.num_pages)
    k2 = np.empty_like(a.k_cache); v2 = np.empty_like(a.v_cache)
    k2[perm] = a.k_cache; v2[perm] = a.v_cache
    pt2 = np.where(a.page_table >= 0, perm[np.maximum(a.page_table, 0)], -1).astype(np.int32)
    out_b, lse_b = oracle_mod.tree_attn(a.q, a.k_tree, a.v_tree, k2, v2, pt2, a.seq_lens, a.parents)
    assert np.array_equal(out_a, out_b) and np.array_equal(lse_a, lse_b)


def test_relabelling_the_tree_permutes_the_rows(oracle_mod):
    # Another topological numbering of the same tree only permutes the output rows.
    w = W.make_custom("relabel", B=1, Hq=2, Hkv=2, D=16, T=9, seq_lens=[20], tree="given", seed=6,
                      parents=np.asarray([[-1, 0, 0, 1, 1, 2, 3, 5, 5]], dtype=np.int32))
    out, _ = run(oracle_mod, w)
    new_of_old = np.asarray([0, 2, 1, 5, 4, 3, 8, 6, 7])      # children still come after parents
    old_of_new = np.argsort(new_of_old)
    par2 = np.full(9, -1, dtype=np.int32)
    for old in range(1, 9):
        par2[new_of_old[old]] = new_of_old[w.parents[0, old]]
    assert all(par2[i] < i for i in range(1, 9))
    out2, _ = oracle_mod.tree_attn(
        np.ascontiguousarray(w.q[:, old_of_new]), np.ascontiguousarray(w.k_tree[:, old_of_new]),
        np.ascontiguousarray(w.v_tree[:, old_of_new]), w.k_cache, w.v_cache, w.page_table,
        w.seq_lens, par2[None])
    np.testing.assert_allclose(out2[0, new_of_old], out[0], **TOL)


def test_rows_entry_matches_whole_problem(oracle_mod):
    w = W.make_config(0)
    out, lse = run(oracle_mod, w)
    rows = np.asarray([[0, 0, 0], [0, 7, 15], [0, 3, 8]], dtype=np.int32)
    o2, l2 = oracle_mod.tree_attn_rows(w.q, w.k_tree, w.v_tree, w.k_cache, w.v_cache, w.page_table,
                                       w.seq_lens, w.parents, rows)
    for r, (b, hq, i) in enumerate(rows):
        assert np.array_equal(o2[r], out[b, i, hq]) and l2[r] == lse[b, hq, i]


def test_peaked_scores_stay_accurate(oracle_mod):
    # Keys scaled x4 (the long-context preset) give sharply peaked softmax rows; the double
    # oracle must still agree with an independent float64 evaluation and stay finite.
    w = W.make_custom("peaked", B=1, Hq=4, Hkv=1, D=128, T=4, seq_lens=[300], tree="chain", seed=8,
                      k_outlier_frac=0.05)
    out, lse = run(oracle_mod, w)
    assert np.isfinite(out).all()
    for hq in range(4):
        for i in range(4):
            ref, ref_lse = flat_sequence_row(w, 0, hq, i)
            np.testing.assert_allclose(out[0, i, hq], ref, **TOL)


def test_canary_slots_are_never_read(oracle_mod):
    # Slots past L_b hold NaN canaries; a finite result shows they were not touched.
    w = W.make_custom("canary", B=2, Hq=2, Hkv=2, D=16, T=5, seq_lens=[17, 31], seed=12)
    assert (w.k_cache == W.CANARY).any()
    out, lse = run(oracle_mod, w)
    assert np.isfinite(out).all() and np.isfinite(lse).all()

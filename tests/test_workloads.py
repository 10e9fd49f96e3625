"""The input generator: shapes, determinism, tree validity, page-table consistency.  CPU only."""
import numpy as np
import pytest

from paper_2508_09072_amd import workloads as W


def depths(par):
    d = np.zeros(len(par), dtype=int)
    for i in range(1, len(par)):
        d[i] = d[par[i]] + 1
    return d


def test_bf16_round_to_nearest_even():
    import torch
    x = np.random.Generator(np.random.PCG64(1)).standard_normal(4096, dtype=np.float32) * 3
    x[:4] = [1.00390625, 1.01171875, 0.0, -2.5]          # ties: to even
    ref = torch.from_numpy(x).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    assert np.array_equal(W.to_bf16_bits(x), ref)
    assert np.array_equal(W.bf16_bits_to_f32(ref), torch.from_numpy(x).to(torch.bfloat16).float().numpy())


@pytest.mark.parametrize("index,shape", [
    (0, dict(B=1, Hq=8, Hkv=8, D=64, T=16, depth=6, branch=15)),
    (1, dict(B=1, Hq=32, Hkv=8, D=128, T=64, depth=8, branch=4)),
    (2, dict(B=16, Hq=32, Hkv=8, D=128, T=32, depth=6, branch=3)),
])
def test_presets_have_the_stated_shapes(index, shape):
    w = W.make_config(index, length_scale=0.05 if index else 1.0)
    assert (w.B, w.Hq, w.Hkv, w.D, w.T) == (shape["B"], shape["Hq"], shape["Hkv"], shape["D"], shape["T"])
    assert w.page_size == 16 and w.q.shape == (w.B, w.T, w.Hq, w.D)
    assert w.k_cache.shape == (w.num_pages, w.Hkv, 16, w.D)
    for b in range(w.B):
        par = w.parents[b]
        assert par[0] == -1 and all(0 <= par[i] < i for i in range(1, w.T))
        assert depths(par).max() <= shape["depth"] and w.max_path >= depths(par).max() + 1
        assert np.bincount(par[1:], minlength=w.T).max() <= shape["branch"]
        # every position up to L_b + max_path has a page, no page is mapped twice
        need = (int(w.seq_lens[b]) + w.max_path + 15) // 16
        assert (w.page_table[b, :need] >= 0).all() and (w.page_table[b, need:] == -1).all()
    mapped = w.page_table[w.page_table >= 0]
    assert len(set(mapped.tolist())) == mapped.size and mapped.max() < w.num_pages


def test_same_seed_same_input_other_seed_other_input():
    a, b, c = W.make_config(0), W.make_config(0), W.make_config(0, seed=5)
    for f in ("q", "k_tree", "k_cache", "v_cache", "page_table", "parents", "draft_tokens", "target_tokens"):
        assert np.array_equal(getattr(a, f), getattr(b, f))
    assert not np.array_equal(a.q, c.q)


def test_ragged_lengths_and_canaries():
    w = W.make_config(2, length_scale=0.03)
    assert len(set(w.seq_lens.tolist())) > 4 and (w.seq_lens % 16 != 0).any()
    for b in range(w.B):
        L = int(w.seq_lens[b])
        pages = w.page_table[b][w.page_table[b] >= 0]
        flat = w.k_cache[pages].transpose(0, 2, 1, 3).reshape(-1, w.Hkv, w.D)
        assert (flat[L:] == W.CANARY).all() and not (flat[:L] == W.CANARY).all(axis=(1, 2)).any()


def test_trie_siblings_carry_distinct_tokens():
    rng = np.random.Generator(np.random.PCG64(3))
    par, tok = W.tree_trie(rng, 64, depth=8, branch=4, vocab=20)
    for p in range(64):
        kids = [i for i in range(1, 64) if par[i] == p]
        assert len({int(tok[k]) for k in kids}) == len(kids) <= 4


def test_match_probability_of_targets():
    rng = np.random.Generator(np.random.PCG64(4))
    par = W.tree_chain(2)
    hits = 0
    for _ in range(4000):
        dr = rng.integers(0, 100, size=2).astype(np.int32)
        hits += int(W.draw_targets(rng, par, dr, 100, 0.7)[0] == dr[1])
    assert abs(hits / 4000 - 0.7) < 0.04


def test_long_context_preset_has_scaled_keys():
    w = W.make_config(3, length_scale=0.01)
    k = W.bf16_bits_to_f32(w.k_cache[w.page_table[0, :10]])           # [10, Hkv, 16, D]
    per_pos = np.abs(k).mean(axis=(1, 3)).reshape(-1)                  # one number per position
    frac = (per_pos > 2.0).mean()
    assert 0.0 < frac < 0.15

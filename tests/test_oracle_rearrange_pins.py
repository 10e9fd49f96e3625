"""Pins for oracle.kv_rearrange (Section 4.3 / Algorithm 4 on the padded layout).

The pass is a stable per-sample compaction, so it is pinned against numpy boolean indexing
(written here, independently of the oracle's loop), against its invariants (idempotent, order and
content of the real rows kept, nothing but padding behind them, other samples untouched), and
against its special cases (no hole, nothing valid, one long hole).
"""
import numpy as np
import pytest

from paper_2508_09072_amd import workloads as W


def reference(k, v, valid):
    """Tight concatenation by boolean indexing; rows from the new length to the old extent become
    zero, rows past the old extent keep their value."""
    k2, v2 = k.copy(), v.copy()
    NL, B, S, Hkv, D = k.shape
    new_valid = np.zeros_like(valid)
    lens = np.zeros(B, dtype=np.int32)
    for b in range(B):
        keep = valid[b].astype(bool)
        n = int(keep.sum())
        extent = int(np.flatnonzero(keep).max()) + 1 if n else 0
        for l in range(NL):
            k2[l, b, :n] = k[l, b][keep]
            v2[l, b, :n] = v[l, b][keep]
            k2[l, b, n:extent] = 0
            v2[l, b, n:extent] = 0
        new_valid[b, :n] = 1
        lens[b] = n
    return k2, v2, new_valid, lens


@pytest.mark.parametrize("seed", [0, 1, 2, 3])
def test_equals_boolean_indexing(oracle_mod, seed):
    c = W.make_padded_cache("pin", NL=2, B=5, Hkv=2, D=8, prompt_lens=[9, 4, 12, 1, 7], steps=7, p_long=0.3,
                            seed=seed)
    k_ref, v_ref, valid_ref, lens_ref = reference(c.k_pad, c.v_pad, c.valid)
    k, v, valid = c.k_pad.copy(), c.v_pad.copy(), c.valid.copy()
    lens = oracle_mod.kv_rearrange(k, v, valid)
    assert np.array_equal(lens, lens_ref) and np.array_equal(valid, valid_ref)
    assert np.array_equal(k, k_ref) and np.array_equal(v, v_ref)


def test_idempotent_and_padding_only_at_the_end(oracle_mod):
    c = W.make_padded_cache("pin", NL=1, B=4, Hkv=1, D=4, prompt_lens=[3, 8, 5, 6], steps=10, p_long=0.2, seed=11)
    k, v, valid = c.k_pad.copy(), c.v_pad.copy(), c.valid.copy()
    lens = oracle_mod.kv_rearrange(k, v, valid)
    for b in range(4):
        assert valid[b, :lens[b]].all() and not valid[b, lens[b]:].any()
        assert not k[0, b, lens[b]:].any() and not v[0, b, lens[b]:].any()      # generator pads with zeros
        assert lens[b] == c.valid[b].sum()
    k2, v2, valid2 = k.copy(), v.copy(), valid.copy()
    lens2 = oracle_mod.kv_rearrange(k2, v2, valid2)
    assert np.array_equal(lens2, lens) and np.array_equal(k2, k) and np.array_equal(v2, v) and np.array_equal(valid2, valid)


def test_rows_keep_their_order_and_other_samples_are_untouched(oracle_mod):
    # every row carries its own position as a tag, so the expected result can be read off directly
    NL, B, S, Hkv, D = 1, 3, 20, 1, 2
    k = np.zeros((NL, B, S, Hkv, D), dtype=np.uint16)
    for b in range(B):
        for j in range(S):
            k[0, b, j] = 1000 * (b + 1) + j
    v = (k + 7).astype(np.uint16)
    valid = np.zeros((B, S), dtype=np.uint8)
    valid[0, [0, 1, 2, 5, 6, 9, 15]] = 1
    valid[1, :] = 1                      # no hole at all: must not change
    valid[2, 17] = 1                     # a single entry far to the right
    k0, v0 = k.copy(), v.copy()
    lens = oracle_mod.kv_rearrange(k, v, valid)
    assert lens.tolist() == [7, 20, 1]
    assert k[0, 0, :7, 0, 0].tolist() == [1000, 1001, 1002, 1005, 1006, 1009, 1015]
    assert not k[0, 0, 7:16].any() and np.array_equal(k[0, 0, 16:], k0[0, 0, 16:])   # past the old extent: untouched
    assert np.array_equal(k[0, 1], k0[0, 1]) and np.array_equal(v[0, 1], v0[0, 1])
    assert k[0, 2, 0, 0, 0] == 3017 and not k[0, 2, 1:18].any()
    assert np.array_equal(v[0, 0, :7], v0[0, 0, [0, 1, 2, 5, 6, 9, 15]])


def test_degenerate_inputs(oracle_mod):
    k = np.full((2, 2, 6, 1, 4), 5, dtype=np.uint16)
    v = k.copy()
    valid = np.zeros((2, 6), dtype=np.uint8)            # nothing valid: nothing moves, nothing is zeroed
    lens = oracle_mod.kv_rearrange(k, v, valid)
    assert lens.tolist() == [0, 0] and (k == 5).all() and (v == 5).all() and not valid.any()
    empty = np.zeros((1, 0, 6, 1, 4), dtype=np.uint16)  # empty batch
    assert oracle_mod.kv_rearrange(empty, empty.copy(), np.zeros((0, 6), dtype=np.uint8)).shape == (0,)


def test_padding_probability_grows_with_batch_size():
    # Section 4.3: with probability p of a long span per sample, a step pads somebody with
    # probability 1 - (1 - p)^b; the generator reproduces that growth
    p, steps = 0.1, 400
    frac = []
    for B in (1, 4, 16):
        c = W.make_padded_cache("stat", NL=1, B=B, Hkv=1, D=2, prompt_lens=[1] * B, steps=steps, p_long=p, seed=5)
        frac.append(1.0 - c.valid.sum() / (c.valid.shape[0] * (c.valid.shape[1] - 8)))
    assert frac[0] == 0.0 and frac[0] < frac[1] < frac[2]

"""Seeded synthetic inputs for the draft-tree verification step.

This module only *draws inputs*: sequence lengths, page tables, draft trees,
token ids and bf16 tensors.  It contains none of the method's arithmetic (no
attention, no acceptance, no compaction) and imports neither the HIP binding nor
the CPU oracle, so both sides can be fed from it.

The five presets follow the workload shapes the verification step sees in the
paper's experiments (Section 5 and Section 4.1: ~60-node depth-8 draft trees at
batch 1, batched serving at 8-32 sequences, long retrieval-augmented prompts):
their datasets are replaced by random tensors of the same shapes.

Every array is numpy; bf16 tensors are ``uint16`` bit patterns (round-to-nearest-
even from float32).  Layouts:

    q               [B, T, Hq, D]
    k_tree, v_tree  [B, T, Hkv, D]
    k_cache,v_cache [num_pages, Hkv, page_size, D]
    page_table      [B, max_pages]   int32, -1 where no page is mapped
    seq_lens        [B]              int32 prefix length L_b
    parents         [B, T]           int32, parents[b,0] = -1, parents[b,i] < i
    draft_tokens    [B, T]           int32 token drafted at each node (root: last committed token)
    target_tokens   [B, T]           int32 base model's next token after the prefix ending at a node

Draw order (fixed, so a seed names one input): (1) L_b, (2) page permutation,
(3) trees, (4) tokens, (5) prefix K then V, (6) tree K then V, (7) Q.
"""
from __future__ import annotations

import dataclasses
from typing import List, Optional, Sequence

import numpy as np

PAGE_SIZE = 16
SEED_BASE = 250809072
# bf16 quiet-NaN pattern written to every cache slot that holds no token: a kernel
# that reads past a sequence's end, or a compaction that writes where it should
# not, shows up as NaN in the output or as a changed canary.
CANARY = 0x7FC1


def to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """float32 -> bf16 bit pattern (uint16), round to nearest even."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    bias = ((u >> np.uint32(16)) & np.uint32(1)) + np.uint32(0x7FFF)
    return ((u + bias) >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(bits: np.ndarray) -> np.ndarray:
    """bf16 bit pattern (uint16) -> float32, exact."""
    return (np.ascontiguousarray(bits, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


# --------------------------------------------------------------------------- trees

def _depths(parents: Sequence[int]) -> List[int]:
    d = [0] * len(parents)
    for i in range(1, len(parents)):
        d[i] = d[parents[i]] + 1
    return d


def tree_chain(T: int) -> np.ndarray:
    return np.arange(-1, T - 1, dtype=np.int32)


def tree_star(T: int) -> np.ndarray:
    p = np.zeros(T, dtype=np.int32)
    p[0] = -1
    return p


def tree_uniform(rng: np.random.Generator, T: int, max_depth: int) -> np.ndarray:
    """Node i's parent is uniform over [0, i), redrawn while it would exceed max_depth."""
    parents = [-1]
    depth = [0]
    for i in range(1, T):
        while True:
            p = int(rng.integers(0, i))
            if depth[p] + 1 <= max_depth:
                break
        parents.append(p)
        depth.append(depth[p] + 1)
    return np.asarray(parents, dtype=np.int32)


def tree_trie(rng: np.random.Generator, T: int, depth: int, branch: int, vocab: int):
    """Trie of random token paths, the shape a retrieval drafter produces.

    Paths of `depth` tokens are inserted below the root until the trie has T nodes.
    Each path after the first copies the first s ~ U{0..depth-1} tokens of a random
    earlier path and continues with fresh tokens.  A node never gets more than
    `branch` children: where a new child would be needed beyond that, the path
    follows a random existing child instead.  Nodes are numbered in creation order,
    so a parent always precedes its children.  Returns (parents [T], tokens [T]).
    """
    parents = [-1]
    tokens = [int(rng.integers(0, vocab))]
    children: List[dict] = [dict()]
    paths: List[List[int]] = []
    guard = 0
    while len(parents) < T:
        guard += 1
        if guard > 100000:
            raise RuntimeError("trie cannot reach %d nodes with depth=%d branch=%d" % (T, depth, branch))
        if paths:
            src = paths[int(rng.integers(0, len(paths)))]
            s = int(rng.integers(0, depth))
            path = list(src[:s]) + [int(t) for t in rng.integers(0, vocab, size=depth - s)]
        else:
            path = [int(t) for t in rng.integers(0, vocab, size=depth)]
        cur = 0
        for j, tok in enumerate(path):
            kids = children[cur]
            if tok in kids:
                cur = kids[tok]
            elif len(kids) < branch:
                if len(parents) == T:
                    break
                parents.append(cur)
                tokens.append(tok)
                children.append(dict())
                kids[tok] = len(parents) - 1
                cur = kids[tok]
            else:
                keys = sorted(kids.keys())
                tok = keys[int(rng.integers(0, len(keys)))]
                path[j] = tok
                cur = kids[tok]
        paths.append(path)
    return np.asarray(parents, dtype=np.int32), np.asarray(tokens, dtype=np.int32)


def draw_targets(rng: np.random.Generator, parents: np.ndarray, draft: np.ndarray, vocab: int,
                 p_match: float) -> np.ndarray:
    """Base-model token per node: with probability p_match (and if the node has children)
    it equals the drafted token of a random child, otherwise it differs from every child."""
    T = len(parents)
    kids: List[List[int]] = [[] for _ in range(T)]
    for i in range(1, T):
        kids[int(parents[i])].append(i)
    target = np.zeros(T, dtype=np.int32)
    for i in range(T):
        hit = rng.random() < p_match
        if hit and kids[i]:
            target[i] = draft[kids[i][int(rng.integers(0, len(kids[i])))]]
        else:
            taken = {int(draft[c]) for c in kids[i]}
            if len(taken) >= vocab:
                t = vocab          # the children use up the vocabulary: a token none of them drafted
            else:
                while True:
                    t = int(rng.integers(0, vocab))
                    if t not in taken:
                        break
            target[i] = t
    return target


# ----------------------------------------------------------------------- workload

@dataclasses.dataclass
class Workload:
    name: str
    B: int
    T: int
    Hq: int
    Hkv: int
    D: int
    page_size: int
    num_pages: int
    max_pages: int
    max_path: int
    vocab: int
    q: np.ndarray
    k_tree: np.ndarray
    v_tree: np.ndarray
    k_cache: np.ndarray
    v_cache: np.ndarray
    page_table: np.ndarray
    seq_lens: np.ndarray
    parents: np.ndarray
    draft_tokens: np.ndarray
    target_tokens: np.ndarray

    @property
    def kv_token_bytes(self) -> int:
        """Bytes of K plus V of all kv heads for one position."""
        return 4 * self.Hkv * self.D

    def algorithmic_bytes(self) -> int:
        """Bytes the tree-attention step must move: each prefix K/V row once, the tree
        K/V rows once, Q in and O out (Section 3.2: reads grow with b*h*(gamma+s))."""
        kv = int(self.seq_lens.astype(np.int64).sum() + self.B * self.T) * self.kv_token_bytes
        qo = 2 * self.B * self.T * self.Hq * self.D * 2
        return kv + qo

    def attention_flops(self) -> int:
        """2 flops per multiply-add, QK^T and PV, over the keys each query really sees."""
        seen = 0
        for b in range(self.B):
            d = _depths(list(self.parents[b]))
            seen += sum(int(self.seq_lens[b]) + di + 1 for di in d)
        return 4 * self.Hq * self.D * seen


def make_custom(name: str, B: int, Hq: int, Hkv: int, D: int, T: int, seq_lens: Sequence[int],
                tree: str = "trie", depth: int = 6, branch: int = 3, vocab: int = 32000,
                p_match: float = 0.7, seed: int = 0, shuffle_pages: bool = True,
                spare_pages: int = 3, k_outlier_frac: float = 0.0, k_outlier_scale: float = 4.0,
                max_path: Optional[int] = None, parents: Optional[np.ndarray] = None,
                page_size: int = PAGE_SIZE) -> Workload:
    """Draw one workload.  `tree` is 'trie', 'uniform', 'chain' or 'star' ('given' with `parents`)."""
    rng = np.random.Generator(np.random.PCG64(seed))
    seq = np.asarray(list(seq_lens), dtype=np.int32)
    assert seq.shape == (B,) and (seq >= 0).all()
    assert Hq % Hkv == 0 and T >= 1

    if tree == "chain":
        max_depth = T - 1
    elif tree == "star":
        max_depth = min(1, T - 1)
    elif tree == "given":
        max_depth = max(max(_depths(list(parents[b]))) for b in range(B)) if B else 0
    else:
        max_depth = min(depth, T - 1)
    P = int(max_path) if max_path is not None else max_depth + 1

    # (2) pages: every sequence owns pages for positions [0, L_b + P); the pool also holds
    # a few pages no sequence maps.  Physical order is a random permutation.
    n_pages_b = [(int(seq[b]) + P + page_size - 1) // page_size for b in range(B)]
    max_pages = max(n_pages_b) if B else 1
    num_pages = int(sum(n_pages_b)) + spare_pages
    perm = rng.permutation(num_pages) if shuffle_pages else np.arange(num_pages)
    page_table = np.full((B, max_pages), -1, dtype=np.int32)
    at = 0
    for b in range(B):
        page_table[b, : n_pages_b[b]] = perm[at: at + n_pages_b[b]]
        at += n_pages_b[b]

    # (3) trees and (4) tokens
    par = np.zeros((B, T), dtype=np.int32)
    draft = np.zeros((B, T), dtype=np.int32)
    target = np.zeros((B, T), dtype=np.int32)
    for b in range(B):
        if tree == "trie":
            par[b], draft[b] = tree_trie(rng, T, max_depth, branch, vocab) if T > 1 else (
                np.asarray([-1], dtype=np.int32), rng.integers(0, vocab, size=1).astype(np.int32))
        else:
            if tree == "uniform":
                par[b] = tree_uniform(rng, T, max_depth)
            elif tree == "chain":
                par[b] = tree_chain(T)
            elif tree == "star":
                par[b] = tree_star(T)
            elif tree == "given":
                par[b] = np.asarray(parents[b], dtype=np.int32)
            else:
                raise ValueError(tree)
            draft[b] = rng.integers(0, vocab, size=T).astype(np.int32)
    for b in range(B):
        target[b] = draw_targets(rng, par[b], draft[b], vocab, p_match)

    # (5) prefix K then V, drawn in the cache's own layout, page by page per sequence
    k_cache = np.full((num_pages, Hkv, page_size, D), CANARY, dtype=np.uint16)
    v_cache = np.full((num_pages, Hkv, page_size, D), CANARY, dtype=np.uint16)
    for which in (0, 1):
        cache = k_cache if which == 0 else v_cache
        for b in range(B):
            L = int(seq[b])
            used = (L + page_size - 1) // page_size
            if used == 0:
                continue
            vals = rng.standard_normal((used, Hkv, page_size, D), dtype=np.float32)
            if which == 0 and k_outlier_frac > 0.0:
                hot = rng.random(used * page_size) < k_outlier_frac
                vals = vals * np.where(hot, np.float32(k_outlier_scale), np.float32(1.0)).reshape(
                    used, 1, page_size, 1).astype(np.float32)
            bits = to_bf16_bits(vals)
            tail = L - (used - 1) * page_size
            if tail < page_size:
                bits[used - 1, :, tail:, :] = CANARY
            cache[page_table[b, :used]] = bits
            del vals, bits

    # (6) tree K then V, (7) Q
    k_tree = to_bf16_bits(rng.standard_normal((B, T, Hkv, D), dtype=np.float32))
    v_tree = to_bf16_bits(rng.standard_normal((B, T, Hkv, D), dtype=np.float32))
    q = to_bf16_bits(rng.standard_normal((B, T, Hq, D), dtype=np.float32))

    return Workload(name=name, B=B, T=T, Hq=Hq, Hkv=Hkv, D=D, page_size=page_size,
                    num_pages=num_pages, max_pages=max_pages, max_path=P, vocab=vocab,
                    q=q, k_tree=k_tree, v_tree=v_tree, k_cache=k_cache, v_cache=v_cache,
                    page_table=page_table, seq_lens=seq, parents=par, draft_tokens=draft,
                    target_tokens=target)


CONFIG_NAMES = (
    "cfg0_tiny_B1_L512_T16",
    "cfg1_single_prompt_B1_L4096_T64",
    "cfg2_batched_ragged_B16_L1024-4096_T32",
    "cfg3_long_context_rag_B4_L32768_T128",
    "cfg4_large_batch_70b_B64_L2048-8192_T64",
)


def make_config(index: int, seed: Optional[int] = None, length_scale: float = 1.0) -> Workload:
    """One of the five preset workloads.  `length_scale` < 1 shrinks only the prefix
    lengths (for parity runs the CPU oracle can finish); shapes and trees stay."""
    seed = SEED_BASE + index if seed is None else seed
    rng = np.random.Generator(np.random.PCG64(seed))   # (1) sequence lengths

    def sc(n):
        return max(1, int(round(n * length_scale)))

    if index == 0:
        return make_custom(CONFIG_NAMES[0], B=1, Hq=8, Hkv=8, D=64, T=16, seq_lens=[sc(512)],
                           tree="uniform", depth=6, vocab=32000, p_match=0.6, seed=seed + 1000)
    if index == 1:
        return make_custom(CONFIG_NAMES[1], B=1, Hq=32, Hkv=8, D=128, T=64, seq_lens=[sc(4096)],
                           tree="trie", depth=8, branch=4, vocab=128256, p_match=0.7, seed=seed + 1000)
    if index == 2:
        L = rng.integers(1024, 4096 + 1, size=16)
        return make_custom(CONFIG_NAMES[2], B=16, Hq=32, Hkv=8, D=128, T=32, seq_lens=[sc(x) for x in L],
                           tree="trie", depth=6, branch=3, vocab=128256, p_match=0.7, seed=seed + 1000)
    if index == 3:
        return make_custom(CONFIG_NAMES[3], B=4, Hq=32, Hkv=8, D=128, T=128, seq_lens=[sc(32768)] * 4,
                           tree="trie", depth=12, branch=8, vocab=128256, p_match=0.8,
                           k_outlier_frac=0.05, k_outlier_scale=4.0, seed=seed + 1000)
    if index == 4:
        L = rng.integers(2048, 8192 + 1, size=64)
        return make_custom(CONFIG_NAMES[4], B=64, Hq=64, Hkv=8, D=128, T=64, seq_lens=[sc(x) for x in L],
                           tree="trie", depth=10, branch=4, vocab=128256, p_match=0.7, seed=seed + 1000)
    raise ValueError("config index must be 0..4")


# ---------------------------------------------------------------------------------------------
# Padded cache for the periodic rearrangement pass (Section 4.3, Algorithm 4)

@dataclasses.dataclass
class PaddedCache:
    """A batch's KV cache in the padded layout the paper starts from: every sample owns S slots,
    all samples append at one common cursor, a sample that accepted fewer tokens than the longest
    one in a step is padded.  k_pad, v_pad: uint16 (bf16 bits) [NL, B, S, Hkv, D], zero where
    valid == 0; valid: uint8 [B, S]."""
    name: str
    k_pad: np.ndarray
    v_pad: np.ndarray
    valid: np.ndarray

    @property
    def shape(self):
        return self.k_pad.shape

    def moved_bytes(self) -> int:
        """Bytes the pass must move: every valid row behind its sample's first hole is read and
        written once (K and V, all layers); rows in front of the first hole stay where they are."""
        NL, B, S, Hkv, D = self.k_pad.shape
        rows = 0
        for b in range(B):
            v = self.valid[b]
            holes = np.flatnonzero(v == 0)
            if holes.size:
                rows += int(v[holes[0]:].sum())
        return rows * NL * Hkv * D * 2 * 2 * 2


def padded_valid_flags(prompt_lens: Sequence[int], steps: int, p_long: float, rng, slack: int = 8) -> np.ndarray:
    """Validity flags uint8 [B, S] after `steps` decoding steps behind the prompts: per step each sample
    accepts 1 + Geometric tokens, with probability p_long a long span of 8..24 (a long retrieval hit);
    all samples advance by the longest acceptance of the step, the others are padded (the situation
    Section 4.3 describes)."""
    prompt_lens = [int(x) for x in prompt_lens]
    B = len(prompt_lens)
    cursor = max(prompt_lens) if B else 0
    spans = []
    for _ in range(steps):
        a = 1 + rng.geometric(0.5, size=B)                    # 3 on average
        long_hit = rng.random(B) < p_long
        a = np.where(long_hit, rng.integers(8, 25, size=B), a)
        spans.append((cursor, a.astype(np.int64)))
        cursor += int(a.max()) if B else 0
    S = cursor + slack
    valid = np.zeros((B, S), dtype=np.uint8)
    for b in range(B):
        valid[b, :prompt_lens[b]] = 1
    for start, a in spans:
        for b in range(B):
            valid[b, start:start + int(a[b])] = 1
    return valid


def make_padded_cache(name: str, NL: int, B: int, Hkv: int, D: int, prompt_lens: Sequence[int], steps: int,
                      p_long: float = 0.1, seed: int = 0, slack: int = 8) -> PaddedCache:
    """Flags from padded_valid_flags, bf16 ~N(0,1) values in the valid slots, zeros in the padding."""
    rng = np.random.Generator(np.random.PCG64(seed))
    assert len(prompt_lens) == B
    valid = padded_valid_flags(prompt_lens, steps, p_long, rng, slack)
    S = valid.shape[1]
    k = to_bf16_bits(rng.standard_normal((NL, B, S, Hkv, D), dtype=np.float32))
    v = to_bf16_bits(rng.standard_normal((NL, B, S, Hkv, D), dtype=np.float32))
    hole = (valid == 0)[None, :, :, None, None]
    k = np.where(hole, np.uint16(0), k).astype(np.uint16)
    v = np.where(hole, np.uint16(0), v).astype(np.uint16)
    return PaddedCache(name=name, k_pad=np.ascontiguousarray(k), v_pad=np.ascontiguousarray(v), valid=valid)


# ---------------------------------------------------------------------------------------------
# Base-model logits for the target-token step (Algorithm 5; Appendix C for the sampling policy)

def make_logits(B: int, T: int, V: int, rng: np.random.Generator, peaked: bool = True) -> np.ndarray:
    """bf16 bit patterns [B, T, V] shaped like a language model's output: a broad body of
    unlikely tokens (normal, sigma 2) and, when `peaked`, a handful of candidates per row that
    carry most of the probability (raised by 6..12), as trained models produce."""
    x = rng.standard_normal((B, T, V), dtype=np.float32) * 2.0
    if peaked and V >= 8:
        n_top = min(6, V // 2)
        for b in range(B):
            for t in range(T):
                idx = rng.choice(V, size=n_top, replace=False)
                x[b, t, idx] += rng.uniform(6.0, 12.0, size=n_top).astype(np.float32)
    return to_bf16_bits(x)


def make_uniforms(B: int, T: int, rng: np.random.Generator) -> np.ndarray:
    """One uniform in [0, 1) per (sequence, depth), float32."""
    u = rng.random((B, T), dtype=np.float32)
    return np.minimum(u, np.float32(1.0 - 2.0 ** -24))


# ---------------------------------------------------------------------------------------------
# In-cache layout of a step, all layers (Section 4.3): the tree's K/V rows were written behind
# each sequence by the forward pass; compaction moves the accepted path's rows forward in place.

@dataclasses.dataclass
class InCacheStep:
    """k_cache, v_cache: uint16 (bf16 bits) [NL, num_pages, Hkv, page_size, D]; positions
    [0, seq_lens[b] + T) of every sequence hold data (prefix, then tree node n at
    seq_lens[b] + n), every other slot the canary.  path / accept_len: one root-to-node path
    per sequence (node ids increase along a path because a parent precedes its children)."""
    name: str
    k_cache: np.ndarray
    v_cache: np.ndarray
    page_table: np.ndarray
    seq_lens: np.ndarray
    parents: np.ndarray
    path: np.ndarray
    accept_len: np.ndarray
    T: int
    max_path: int

    def moved_bytes(self) -> int:
        """Bytes the pass must move: every accepted row that is not already in place, read
        and written once, K and V, all layers and heads."""
        NL, _, Hkv, _, D = self.k_cache.shape
        rows = 0
        for b in range(self.path.shape[0]):
            n = int(self.accept_len[b])
            rows += int(np.sum(self.path[b, : n + 1] != np.arange(n + 1)))
        return rows * NL * Hkv * D * 2 * 2 * 2


def make_incache_step(name: str, B: int, T: int, Hkv: int, D: int, num_layers: int, seq_lens: Sequence[int],
                      max_path: int = 0, seed: int = 0, page_size: int = PAGE_SIZE,
                      accept_bias: float = 0.5) -> InCacheStep:
    rng = np.random.Generator(np.random.PCG64(seed))
    max_path = max_path or min(T, 16)
    seq = np.asarray(seq_lens, dtype=np.int32)
    n_pages_b = [(int(seq[b]) + T + page_size - 1) // page_size for b in range(B)]
    max_pages = max(n_pages_b) if B else 1
    num_pages = int(sum(n_pages_b)) + 3
    perm = rng.permutation(num_pages)
    page_table = np.full((B, max_pages), -1, dtype=np.int32)
    k_cache = np.full((num_layers, num_pages, Hkv, page_size, D), CANARY, dtype=np.uint16)
    v_cache = np.full((num_layers, num_pages, Hkv, page_size, D), CANARY, dtype=np.uint16)
    parents = np.full((B, T), -1, dtype=np.int32)
    path = np.full((B, max_path), -1, dtype=np.int32)
    accept_len = np.zeros(B, dtype=np.int32)
    cursor = 0
    for b in range(B):
        pages = perm[cursor: cursor + n_pages_b[b]]
        cursor += n_pages_b[b]
        page_table[b, : n_pages_b[b]] = pages
        n_pos = int(seq[b]) + T
        for cache in (k_cache, v_cache):
            rows = to_bf16_bits(rng.standard_normal((num_layers, n_pos, Hkv, D), dtype=np.float32))
            pos = np.arange(n_pos)
            cache[:, pages[pos // page_size], :, pos % page_size, :] = rows.transpose(1, 0, 2, 3)
        # a tree: mostly deep (a parent close behind), so that paths are long
        for n in range(1, T):
            parents[b, n] = n - 1 if rng.random() < accept_bias else rng.integers(0, n)
        # a path: from a random node up to the root, cut to the deepest max_path - 1 non-root nodes
        node = int(rng.integers(0, T))
        chain = []
        while node >= 0:
            chain.append(node)
            node = int(parents[b, node])
        chain = chain[::-1][:max_path]
        path[b, : len(chain)] = chain
        accept_len[b] = len(chain) - 1
    return InCacheStep(name, k_cache, v_cache, page_table, seq, parents, path, accept_len, T, max_path)


def place_tree_in_cache(w: Workload, seed: int = 0):
    """The same step in the in-cache layout: a fresh page pool whose pages cover
    [0, seq_lens[b] + T) of every sequence, holding the prefix rows of `w` and, behind them,
    the tree rows (node n at position seq_lens[b] + n).  Returns (k_cache, v_cache, page_table)
    as numpy arrays (bf16 bits, int32); unused slots hold the canary."""
    rng = np.random.Generator(np.random.PCG64(seed))
    ps = w.page_size
    n_pages_b = [(int(w.seq_lens[b]) + w.T + ps - 1) // ps for b in range(w.B)]
    max_pages = max(n_pages_b) if w.B else 1
    num_pages = int(sum(n_pages_b)) + 2
    perm = rng.permutation(num_pages)
    table = np.full((w.B, max_pages), -1, dtype=np.int32)
    kc = np.full((num_pages, w.Hkv, ps, w.D), CANARY, dtype=np.uint16)
    vc = np.full((num_pages, w.Hkv, ps, w.D), CANARY, dtype=np.uint16)
    cursor = 0
    for b in range(w.B):
        pages = perm[cursor: cursor + n_pages_b[b]]
        cursor += n_pages_b[b]
        table[b, : n_pages_b[b]] = pages
        L = int(w.seq_lens[b])
        pos = np.arange(L)
        old = w.page_table[b, pos // ps]
        for src, tree, dst in ((w.k_cache, w.k_tree, kc), (w.v_cache, w.v_tree, vc)):
            dst[pages[pos // ps], :, pos % ps, :] = src[old, :, pos % ps, :]
            tpos = L + np.arange(w.T)
            dst[pages[tpos // ps], :, tpos % ps, :] = tree[b]
    return kc, vc, table


def make_token_stream(n: int, vocab: int = 128256, n_phrases: int = 64, p_phrase: float = 0.5, seed: int = 0):
    """Token ids with phrases that come back, as in generated text with self-repetition (Section
    4.1): with probability p_phrase one of n_phrases fixed phrases of 3..11 tokens follows, else
    one token with a Zipf-like distribution over the vocabulary.  int32 [n]."""
    rng = np.random.Generator(np.random.PCG64(seed))
    phrases = [rng.integers(0, vocab, size=int(rng.integers(3, 12))) for _ in range(n_phrases)]
    out, have = [], 0
    while have < n:
        if rng.random() < p_phrase:
            piece = phrases[int(rng.integers(0, n_phrases))]
        else:
            piece = np.minimum(vocab - 1, rng.zipf(1.5, size=1) - 1)
        out.append(np.asarray(piece, dtype=np.int64))
        have += len(piece)
    return np.concatenate(out)[:n].astype(np.int32)

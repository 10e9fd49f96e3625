"""Pins for the oracle's greedy lossless acceptance (Algorithm 5; Appendix C;
Equation 1; Lemma 1; Appendix E monotonicity).  CPU only."""
import os

import numpy as np
import pytest

from paper_2508_09072_amd import workloads as W
from helpers import accepted_nodes_bruteforce, root_path

GOLD = os.path.join(os.path.dirname(__file__), "golden")


def accept(oracle_mod, draft, target, parents, max_path=None):
    draft = np.ascontiguousarray(np.atleast_2d(draft), dtype=np.int32)
    target = np.ascontiguousarray(np.atleast_2d(target), dtype=np.int32)
    parents = np.ascontiguousarray(np.atleast_2d(parents), dtype=np.int32)
    P = parents.shape[1] if max_path is None else max_path
    return oracle_mod.accept_path(draft, target, parents, P)


def read_cases():
    cases = []
    with open(os.path.join(GOLD, "accept_cases.txt")) as f:
        for line in f:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            par, dr, tg, n, path, bonus = [[int(x) for x in part.split()] for part in line.split("|")]
            cases.append((par, dr, tg, n[0], path, bonus[0]))
    return cases


@pytest.mark.parametrize("case", read_cases())
def test_hand_worked_cases(oracle_mod, case):
    par, dr, tg, n, path, bonus = case
    al, p, bo = accept(oracle_mod, dr, tg, par)
    assert al[0] == n and bo[0] == bonus
    assert p[0, : n + 1].tolist() == path and (p[0, n + 1:] == -1).all()


def test_chain_is_prefix_match_length(oracle_mod):
    # On a single branch the accepted length is the number of leading drafted tokens that
    # equal the base model's token one position earlier.
    rng = np.random.Generator(np.random.PCG64(21))
    T = 12
    par = W.tree_chain(T)
    for _ in range(300):
        dr = rng.integers(0, 3, size=T).astype(np.int32)
        tg = rng.integers(0, 3, size=T).astype(np.int32)
        n = 0
        while n + 1 < T and dr[n + 1] == tg[n]:
            n += 1
        al, p, bo = accept(oracle_mod, dr, tg, par)
        assert al[0] == n and bo[0] == tg[n]
        assert p[0, : n + 1].tolist() == list(range(n + 1))


def test_all_match_and_none_match(oracle_mod):
    # every node's token equals the base token at its parent -> the deepest leaf, lowest index
    par = np.asarray([-1, 0, 0, 1, 2, 2, 4, 5], dtype=np.int32)     # depths 0 1 1 2 2 2 3 3
    dr = np.full(8, 4, dtype=np.int32)
    tg = np.full(8, 4, dtype=np.int32)
    al, p, bo = accept(oracle_mod, dr, tg, par)
    assert al[0] == 3 and p[0, :4].tolist() == [0, 2, 4, 6]
    tg = np.full(8, 5, dtype=np.int32)
    al, p, bo = accept(oracle_mod, dr, tg, par)
    assert al[0] == 0 and p[0].tolist() == [0] + [-1] * 7 and bo[0] == 5


def test_invariants_on_random_trees(oracle_mod):
    rng = np.random.Generator(np.random.PCG64(22))
    for trial in range(400):
        T = int(rng.integers(1, 40))
        par = W.tree_uniform(rng, T, max_depth=int(rng.integers(1, 9)))
        dr = rng.integers(0, 3, size=T).astype(np.int32)       # tiny vocabulary: duplicate siblings happen
        tg = rng.integers(0, 3, size=T).astype(np.int32)
        al, p, bo = accept(oracle_mod, dr, tg, par)
        n = int(al[0]); path = p[0, : n + 1].tolist()
        ok = accepted_nodes_bruteforce(par, dr, tg)
        depth = [len(root_path(par, i)) - 1 for i in range(T)]
        # contiguous prefix of some root path, parent-linked, length within tree depth
        assert path[0] == 0 and (p[0, n + 1:] == -1).all() and n <= max(depth)
        for j in range(1, n + 1):
            assert par[path[j]] == path[j - 1] and path[j] in ok
        # longest: no matching node lies deeper; ties go to the lowest index
        assert n == max([depth[i] for i in ok], default=0)
        assert path[-1] == min([i for i in ok if depth[i] == n], default=0)
        assert bo[0] == tg[path[-1]]
        # Appendix E: a node can only be accepted if its parent is
        for i in ok:
            assert par[i] == 0 or par[i] in ok


def test_lemma1_identity_on_tries(oracle_mod):
    # Lemma 1 sums per-node acceptance indicators; on a trie (distinct sibling tokens) the
    # accepted nodes form one chain, so their count equals the accepted length in every trial.
    rng = np.random.Generator(np.random.PCG64(23))
    for trial in range(200):
        par, dr = W.tree_trie(rng, 24, depth=6, branch=3, vocab=50)
        tg = W.draw_targets(rng, par, dr, 50, 0.7)
        al, p, bo = accept(oracle_mod, dr, tg, par)
        assert len(accepted_nodes_bruteforce(par, dr, tg)) == al[0]


def test_equation1_expected_length_on_chains(oracle_mod):
    # Equation 1 through the generator's match rule: mean(accept_len) + 1 -> (1-a^(g+1))/(1-a).
    rows = []
    with open(os.path.join(GOLD, "eq1_expected_length.txt")) as f:
        for line in f:
            if line.strip() and not line.startswith("#"):
                g, a, e = line.split()
                rows.append((int(g), float(a), float(e)))
    rng = np.random.Generator(np.random.PCG64(24))
    N = 6000
    for gamma, alpha, expected in rows:
        assert abs((1 - alpha ** (gamma + 1)) / (1 - alpha) - expected) < 1e-12
        T = gamma + 1
        par = np.tile(W.tree_chain(T), (N, 1))
        dr = rng.integers(0, 1000, size=(N, T)).astype(np.int32)
        tg = np.stack([W.draw_targets(rng, par[0], dr[i], 1000, alpha) for i in range(N)])
        al, _, _ = oracle_mod.accept_path(dr, tg, np.ascontiguousarray(par), T)
        mean = al.mean() + 1.0
        sigma = max(al.std(), 1e-9) / np.sqrt(N)
        assert abs(mean - expected) < 5 * sigma + 1e-12, (gamma, alpha, mean, expected)


def test_speculative_loop_reproduces_greedy_decoding(oracle_mod):
    # Deterministic losslessness theorem (Appendix C): committing accepted path + bonus token
    # step after step gives exactly the sequence plain greedy decoding gives.
    def next_token(prefix):                    # a toy deterministic "base model"
        h = 1469598103934665603
        for t in prefix[-3:]:
            h = ((h ^ (t + 1)) * 1099511628211) % (1 << 64)
        return int(h % 7)

    rng = np.random.Generator(np.random.PCG64(25))
    prompt = [1, 2, 3]
    want = list(prompt)
    for _ in range(60):
        want.append(next_token(want))

    got = list(prompt)
    got.append(next_token(got))                # the first root comes from the base model
    while len(got) < len(want):
        T = int(rng.integers(1, 20))
        par = W.tree_uniform(rng, T, max_depth=6)
        dr = np.zeros(T, dtype=np.int32)
        dr[0] = got[-1]
        prefixes = [list(got)]
        for i in range(1, T):                  # drafts are right about half of the time
            base = prefixes[par[i]]
            dr[i] = next_token(base) if rng.random() < 0.5 else int(rng.integers(0, 7))
            prefixes.append(base + [int(dr[i])])
        tg = np.asarray([next_token(p) for p in prefixes], dtype=np.int32)
        al, p, bo = accept(oracle_mod, dr, tg, par)
        got.extend(int(dr[i]) for i in p[0, 1: al[0] + 1])
        got.append(int(bo[0]))
    assert got[: len(want)] == want


def test_max_path_too_small_is_an_error(oracle_mod):
    par = W.tree_chain(5)
    dr = np.asarray([9, 1, 1, 1, 1], dtype=np.int32)
    tg = np.ones(5, dtype=np.int32)
    with pytest.raises(ValueError):
        accept(oracle_mod, dr, tg, par, max_path=3)

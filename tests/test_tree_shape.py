"""Tree-shape selection (Appendix E; Theorem 1): the oracle against what the paper and arithmetic fix,
then the library's host code against the oracle.  No GPU involved."""
import os

import numpy as np
import pytest

from oracle import tree_shape as TS

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def read_case():
    case = {}
    for ln in open(os.path.join(ROOT, "tests", "golden", "tree_prune_case.txt")):
        tok = ln.split()
        if not tok or tok[0].startswith("#"):
            continue
        case[tok[0]] = tok[1:]
    parents = [int(x.split(":")[1]) for x in case["parents"]]
    return (parents, [float(x) for x in case["alpha"]], [float(x) for x in case["t_draft"]], [float(x) for x in case["tv"]],
            [int(x) for x in case["order"]], [float(x) for x in case["scores"]], int(case["best_n"][0]),
            {int(x) for x in case["kept"]})


def random_seed_tree(rng, T, branch=3):
    """Random tree with per-edge acceptance probabilities: alpha = product along the root path, so that a
    child's alpha is at most its parent's (Appendix E)."""
    parents = [-1]
    n_children = [0]
    for i in range(1, T):
        while True:
            p = int(rng.integers(0, i))
            if n_children[p] < branch:
                break
        parents.append(p)
        n_children[p] += 1
        n_children.append(0)
    alpha = [1.0]
    for i in range(1, T):
        alpha.append(alpha[parents[i]] * float(rng.uniform(0.2, 0.95)))
    return parents, alpha


def knee_curve(T, flat, floor_t, slope):
    """A verification-time curve of the measured kind: flat while the step is bound by the cache reads, then linear."""
    return [floor_t + slope * max(0, k - flat) for k in range(1, T + 1)]


# ------------------------------------------------------------------ the oracle

def test_oracle_reproduces_the_hand_worked_case():
    parents, alpha, t_draft, tv, order, scores, best_n, kept = read_case()
    assert TS.prune_order(parents, alpha) == order
    n, nodes, thr, all_scores = TS.select(parents, alpha, t_draft, tv)
    assert n == best_n and nodes == kept
    assert np.allclose(all_scores, scores, atol=5e-10)
    assert abs(thr - 2.9 / 14) < 1e-12


def test_oracle_numerator_is_the_expected_number_of_accepted_nodes():
    # Lemma 1 through the acceptance oracle: with independent per-edge match probabilities and distinct
    # sibling tokens, the mean number of accepted nodes (root included) over many trials is sum(alpha)
    import oracle
    oracle.build()
    rng = np.random.Generator(np.random.PCG64(31))
    T = 24
    parents, alpha = random_seed_tree(rng, T)
    par = np.asarray(parents, dtype=np.int32)
    edge_p = np.asarray([1.0] + [alpha[i] / alpha[parents[i]] for i in range(1, T)])
    children = [[] for _ in range(T)]
    for i in range(1, T):
        children[parents[i]].append(i)
    trials = 20000
    draft = np.tile(np.arange(T, dtype=np.int32), (trials, 1))            # every node carries its own token
    # the base model's token after node v: one of v's children's tokens, child c with probability edge_p[c] each
    # would overcount; the edge probabilities of siblings have to sum to at most one, so they are scaled to fit
    for v in range(T):
        tot = sum(edge_p[c] for c in children[v])
        if tot > 1.0:
            for c in children[v]:
                edge_p[c] /= tot
    alpha_fit = [1.0] * T
    for i in range(1, T):
        alpha_fit[i] = alpha_fit[parents[i]] * edge_p[i]
    target = np.full((trials, T), -1, dtype=np.int32)
    for v in range(T):
        if not children[v]:
            continue
        u = rng.random(trials)
        lo = 0.0
        for c in children[v]:
            hit = (u >= lo) & (u < lo + edge_p[c])
            target[hit, v] = c
            lo += edge_p[c]
    al, path, bonus = oracle.accept_path(draft, target, np.tile(par, (trials, 1)), T)
    mean_nodes = float(al.mean()) + 1.0                                    # accepted non-root nodes + the root
    expect = sum(alpha_fit)
    # standard error of the mean of a count bounded by the depth
    assert abs(mean_nodes - expect) < 4.0 * al.std() / np.sqrt(trials) + 1e-9
    # and the selection's numerator for the unpruned tree is that sum
    n, nodes, thr, scores = TS.select(parents, alpha_fit, [0.0] * T, [1.0] * T)
    assert abs(scores[0] - expect) < 1e-9


def test_oracle_every_pruned_tree_is_a_prefix_subtree_and_alpha_is_removed_in_order():
    rng = np.random.Generator(np.random.PCG64(32))
    for T in (2, 7, 40):
        parents, alpha = random_seed_tree(rng, T)
        order = TS.prune_order(parents, alpha)
        assert sorted(order) == list(range(1, T))
        alive = set(range(T))
        for v in order:
            assert not any(parents[c] == v for c in alive if c != 0 and c != v), "removed a node that still had a child"
            alive.remove(v)
        # monotone alpha along root paths makes the removal order ascending in alpha
        assert all(alpha[a] <= alpha[b] + 1e-15 for a, b in zip(order, order[1:]))


def test_oracle_limits():
    parents, alpha = random_seed_tree(np.random.Generator(np.random.PCG64(33)), 30)
    T = len(parents)
    # free drafting and a verification time that does not depend on the size: keep everything
    n, nodes, thr, _ = TS.select(parents, alpha, [0.0] * T, [5.0] * T)
    assert n == 0 and len(nodes) == T and abs(thr - sum(alpha) / 5.0) < 1e-12
    # drafting so dear that no node pays for itself: prune to the root, one token per verification
    n, nodes, thr, _ = TS.select(parents, alpha, [1e6] * T, [5.0] * T)
    assert n == T - 1 and nodes == {0} and abs(thr - 1.0 / 5.0) < 1e-12
    # a chain with constant per-step acceptance a, free drafting, T_V = c + k per node: the best length maximises
    # (1 - a^(m)) / (1 - a) / (c + m)  (Eq. 1 over a linear verification cost), found here by direct evaluation
    a, c, m_max = 0.8, 6.0, 25
    chain = [-1] + list(range(m_max - 1))
    al = [a ** i for i in range(m_max)]
    n, nodes, thr, _ = TS.select(chain, al, [0.0] * m_max, [c + k for k in range(1, m_max + 1)])
    closed = [(1 - a ** m) / (1 - a) / (c + m) for m in range(1, m_max + 1)]
    assert len(nodes) == int(np.argmax(closed)) + 1 and abs(thr - max(closed)) < 1e-12


# ------------------------------------------------------------------ the library against the oracle

@pytest.fixture(scope="module")
def R():
    from paper_2508_09072_amd import binding
    if not os.path.exists(binding.LIB_PATH):
        from paper_2508_09072_amd import build
        build.build()
    binding.load()
    return binding


def test_library_hand_worked_case(R):
    parents, alpha, t_draft, tv, order, scores, best_n, kept = read_case()
    assert R.reader_tree_prune_order(parents, alpha).tolist() == order
    for exhaustive in (True, False):
        n, keep, thr, evals = R.reader_tree_select(parents, alpha, t_draft, tv, exhaustive=exhaustive)
        assert n == best_n and set(np.flatnonzero(keep).tolist()) == kept and abs(thr - 2.9 / 14) < 1e-7


@pytest.mark.parametrize("seed", range(12))
def test_library_equals_the_oracle_on_random_seed_trees(R, seed):
    rng = np.random.Generator(np.random.PCG64(500 + seed))
    T = int(rng.choice([1, 2, 5, 16, 64, 128]))
    parents, alpha = random_seed_tree(rng, T, branch=int(rng.integers(1, 5)))
    alpha32 = np.asarray(alpha, dtype=np.float32)
    t_draft = np.asarray([0.0] + [float(rng.uniform(0.0, 0.4)) for _ in range(T - 1)], dtype=np.float32)
    tv = np.asarray(knee_curve(T, flat=int(rng.integers(1, max(T // 2, 2))), floor_t=40.0, slope=float(rng.uniform(0.2, 3.0))),
                    dtype=np.float32)
    want_order = TS.prune_order(parents, alpha32)
    assert R.reader_tree_prune_order(parents, alpha32).tolist() == want_order
    n_ref, nodes_ref, thr_ref, scores = TS.select(parents, alpha32, t_draft, tv)
    n, keep, thr, evals = R.reader_tree_select(parents, alpha32, t_draft, tv, exhaustive=True)
    assert n == n_ref and set(np.flatnonzero(keep).tolist()) == nodes_ref and abs(thr - thr_ref) < 1e-9 * max(1.0, thr_ref)
    assert evals == T
    # golden-section: on a curve that rises and then falls it finds the same tree with far fewer scores;
    # on any curve it returns a tree no worse than both ends of the range
    n_g, keep_g, thr_g, evals_g = R.reader_tree_select(parents, alpha32, t_draft, tv, exhaustive=False)
    peak = int(np.argmax(scores))
    unimodal = all(scores[i] <= scores[i + 1] + 1e-15 for i in range(peak)) and \
        all(scores[i] >= scores[i + 1] - 1e-15 for i in range(peak, T - 1))
    if unimodal:
        assert abs(thr_g - thr_ref) < 1e-9 * max(1.0, thr_ref)
    assert thr_g >= min(scores[0], scores[-1]) - 1e-12
    if T >= 64:
        assert evals_g <= 20
    assert keep_g[0] and all(keep_g[parents[i]] for i in range(1, T) if keep_g[i]), "kept nodes must form a prefix subtree"


def test_library_refuses_bad_arguments(R):
    with pytest.raises(ValueError):
        R.reader_tree_select([0, 0], [1, 0.5], [0, 1], [1, 1])             # the root's parent must be -1
    with pytest.raises(ValueError):
        R.reader_tree_select([-1, 0], [1, float("nan")], [0, 1], [1, 1])
    with pytest.raises(ValueError):
        R.reader_tree_select([-1, 0], [1, 0.5], [0, 1], [1, 0])            # verification time must be positive
    with pytest.raises(ValueError):
        R.reader_tree_prune_order([-1, 1], [1, 0.5])

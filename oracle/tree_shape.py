"""Oracle of the tree-shape selection -- TEST INFRASTRUCTURE ONLY.

Appendix E (choosing the tree structure) with the objective of Theorem 1 (Section 3.3), written out plainly:
the seed tree is pruned one leaf at a time, always the leaf with the lowest acceptance frequency, and every
tree T_n of that sequence is scored as

    throughput(T_n) = (sum of alpha_i over the nodes of T_n, root included: Lemma 1)
                      / (sum of the drafting times t_i of its non-root nodes: Lemma 2,  +  T_V(|T_n|)).

The best n is found by scoring every n (the library's golden-section search is compared with this).
Nothing here is shared with the library; plain Python lists and sets, double precision.
"""
from __future__ import annotations


def prune_order(parents, alpha):
    """Node ids in the order Appendix E removes them: repeatedly the leaf with the lowest alpha
    (equal alphas: the highest node id first).  The root is never removed."""
    T = len(parents)
    alive = set(range(T))
    order = []
    while len(alive) > 1:
        has_child = {int(parents[i]) for i in alive if i != 0}
        leaves = [i for i in alive if i != 0 and i not in has_child]
        victim = min(leaves, key=lambda i: (float(alpha[i]), -i))
        order.append(victim)
        alive.remove(victim)
    return order


def throughput(nodes, alpha, t_draft, tv):
    """Theorem 1's objective for the tree made of `nodes` (a set that contains the root 0);
    tv[k - 1] is the verification time of a tree of k nodes."""
    gain = sum(float(alpha[i]) for i in nodes)
    cost = sum(float(t_draft[i]) for i in nodes if i != 0) + float(tv[len(nodes) - 1])
    return gain / cost


def select(parents, alpha, t_draft, tv):
    """Exhaustive search over the pruning level.  Returns (n_star, kept node set, throughput, all scores)."""
    T = len(parents)
    order = prune_order(parents, alpha)
    nodes = set(range(T))
    scores = [throughput(nodes, alpha, t_draft, tv)]
    for v in order:
        nodes = nodes - {v}
        scores.append(throughput(nodes, alpha, t_draft, tv))
    best = max(range(T), key=lambda n: (scores[n], -n))      # equal scores: the smaller n (the larger tree)
    kept = set(range(T)) - set(order[:best])
    return best, kept, scores[best], scores

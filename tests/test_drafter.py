"""The host-side retrieval drafter (Section 4.2, Algorithm 2, self-repetition metric of Section
4.1): first the brute-force oracle against hand-made cases and closed forms, then the library
against the oracle on synthetic text.  CPU only."""
import numpy as np
import pytest

from oracle import drafter as D


@pytest.fixture(scope="module")
def R():
    import os
    from paper_2508_09072_amd import binding
    if not os.path.exists(binding.LIB_PATH):
        from paper_2508_09072_amd import build
        build.build()
    binding.load()
    return binding


A, B_, C, D_, E = 1, 2, 3, 4, 5


# ---- the oracle against what is known ----

def test_oracle_counts_and_ranks_continuations():
    ix = D.NgramIndex(4)
    ix.insert([A, B_, C, A, B_, D_, A, B_, C, E])
    assert ix.count[(A, B_)] == 3 and ix.count[(A, B_, C)] == 2 and ix.count[(A, B_, D_)] == 1
    assert ix.continuations((A, B_)) == [(C, 2), (D_, 1)]
    assert ix.continuations((B_,)) == [(C, 2), (D_, 1)]
    # a tie: after C both A and E were seen once; A came first
    assert ix.continuations((C,)) == [(A, 1), (E, 1)]
    assert ix.search_path([A, B_], 1) == [C]
    # greedy continuation: a b -> c, then the context "a b c" continues with a (seen first), ...
    assert ix.search_path([A, B_], 3) == [C, A, B_]


def test_oracle_drops_leading_tokens_of_an_unseen_context():
    ix = D.NgramIndex(4)
    ix.insert([A, B_, C, D_])
    assert ix.lookup([E, E, B_]) == (B_,)             # "e e b" unseen, "e b" unseen, "b" seen
    assert ix.search_path([E, E, B_], 5) == [C, D_]   # then nothing follows d
    assert ix.lookup([E]) is None and ix.search_path([E], 3) == []
    assert ix.lookup([D_]) is None                    # seen, but nothing ever followed it


def test_oracle_extracts_depth_first_by_frequency():
    ix = D.NgramIndex(5)
    for s in ([A, B_, C], [A, B_, C], [A, B_, D_, E], [A, C, E], [A, B_, C, E]):
        ix.insert(s)
    tokens, parents = ix.extract_tree([A], max_depth=3, budget=16)
    # below a: b (4 times) before c (1); below "a b": c (3) before d (1); below "a b c": e
    assert tokens == [A, B_, C, E, D_, E, C, E]
    assert parents == [-1, 0, 1, 2, 1, 4, 0, 6]
    tokens, parents = ix.extract_tree([A], max_depth=3, budget=4)       # the budget cuts the walk
    assert tokens == [A, B_, C, E] and parents == [-1, 0, 1, 2]
    tokens, parents = ix.extract_tree([A], max_depth=1, budget=16)      # and so does the depth
    assert tokens == [A, B_, C] and parents == [-1, 0, 0]


def test_oracle_self_repetition_closed_forms():
    assert D.self_repetition([], list(range(50))) == 1.0                       # nothing repeats
    text = list(range(40))
    assert D.self_repetition(text, text) == 40.0                               # one stop: the whole response is in the prompt
    # period 3, no prompt: stops of 1, 1, 1, then 3, 6, 12, ... (the match must lie in what was already walked)
    k = 4
    resp = [A, B_, C] * (2 ** k)
    assert D.self_repetition([], resp) == len(resp) / (3 + k)
    assert D.self_repetition([A, B_], [A, B_, A, B_, A]) == 5 / 2              # "a b" from the prompt, then "a b a" from the history


# ---- the library against the oracle ----

def synthetic_text(rng, n, vocab=50, n_phrases=12, p_phrase=0.5):
    """Zipf-like tokens with phrases that come back, as in generated text."""
    phrases = [rng.integers(0, vocab, size=rng.integers(3, 12)).tolist() for _ in range(n_phrases)]
    out = []
    while len(out) < n:
        if rng.random() < p_phrase:
            out += phrases[int(rng.integers(0, n_phrases))]
        else:
            out.append(int(min(vocab - 1, rng.zipf(1.5) - 1)))
    return out[:n]


@pytest.mark.parametrize("seed,max_depth", [(1, 4), (2, 8), (3, 12)])
def test_library_matches_the_oracle_on_synthetic_text(R, seed, max_depth):
    rng = np.random.Generator(np.random.PCG64(seed))
    text = synthetic_text(rng, 600)
    trie, ix = R.Trie(max_depth), D.NgramIndex(max_depth)
    for lo in range(0, 600, 150):                      # several inserts, as decoding appends text
        trie.insert(text[lo:lo + 150])
        ix.insert(text[lo:lo + 150])
    assert len(trie) == len(ix.count) + 1              # one node per distinct n-gram, and the root
    for _ in range(60):
        at = int(rng.integers(1, 600))
        n_ctx = int(rng.integers(1, max_depth + 3))
        ctx = text[max(0, at - n_ctx):at]
        if rng.random() < 0.2:
            ctx = [999] + ctx                          # an unseen token in front
        depth = int(rng.integers(0, 20))
        assert trie.search_path(ctx, depth).tolist() == ix.search_path(ctx, depth)
        md, budget = int(rng.integers(0, max_depth + 2)), int(rng.integers(1, 64))
        tokens, parents = trie.extract_tree(ctx, md, budget)
        et, ep = ix.extract_tree(ctx, md, budget)
        assert tokens.tolist() == et and parents.tolist() == ep
        assert all(parents[i] < i for i in range(1, len(parents)))     # a parent precedes its children


def test_library_self_repetition_and_attach(R):
    rng = np.random.Generator(np.random.PCG64(5))
    for _ in range(5):
        prompt, resp = synthetic_text(rng, 120), synthetic_text(rng, 200)
        assert R.reader_self_repetition(prompt, resp) == pytest.approx(D.self_repetition(prompt, resp), rel=1e-12)
    assert R.reader_self_repetition([], []) == 0.0
    tokens = np.zeros(8, dtype=np.int32); parents = np.zeros(8, dtype=np.int32)
    tokens[:3] = [7, 8, 9]; parents[:3] = [-1, 0, 0]
    n = R.reader_tree_attach_path(tokens, parents, 3, 1, [20, 21, 22])
    assert n == 6 and tokens[:6].tolist() == [7, 8, 9, 20, 21, 22] and parents[:6].tolist() == [-1, 0, 0, 1, 3, 4]
    n = R.reader_tree_attach_path(tokens, parents, 6, 0, [30, 31, 32, 33])      # only two more fit
    assert n == 8 and tokens[6:].tolist() == [30, 31] and parents[6:].tolist() == [0, 6]


def test_an_unbounded_tree_accepts_what_the_metric_counts(R):
    # Section 4.1: the metric equals the average accepted length of speculative decoding with a
    # tree that indexes all history.  Walk a response: at every stop index the history (prompt and
    # walked response), extract the whole tree below the upcoming token, and take the longest
    # root path that spells the upcoming tokens, which is what verification would accept.
    rng = np.random.Generator(np.random.PCG64(6))
    prompt, resp = synthetic_text(rng, 150, vocab=30), synthetic_text(rng, 300, vocab=30)
    depth = 64                                          # deeper than any repeat in this text
    hist, ptr, stops = list(prompt), 0, 0
    while ptr < len(resp):
        trie = R.Trie(depth + 1)
        trie.insert(hist)
        tokens, parents = trie.extract_tree([resp[ptr]], depth, 100000)
        trie.close()
        children = {}
        for i in range(1, len(tokens)):
            children.setdefault(int(parents[i]), {})[int(tokens[i])] = i
        node, m = 0, 0
        while ptr + 1 + m < len(resp) and int(resp[ptr + 1 + m]) in children.get(node, {}):
            node = children[node][int(resp[ptr + 1 + m])]
            m += 1
        run = m + 1 if resp[ptr] in hist else 0         # the upcoming token itself must have been seen
        assert run < depth
        step = run if run else 1
        hist += resp[ptr:ptr + step]
        ptr += step
        stops += 1
    assert len(resp) / stops == pytest.approx(D.self_repetition(prompt, resp), rel=1e-12)

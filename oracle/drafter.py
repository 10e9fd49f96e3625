"""Brute-force oracle of the host-side retrieval drafter -- TEST INFRASTRUCTURE ONLY.

Section 4.2 (short-term trie, extraction of a draft tree), Algorithm 2 (SearchPath, with the
trie as its only structure) and the self-repetition metric of Section 4.1, written with
dictionaries of n-gram counts and plain loops: no trie, nothing shared with the library.
"""
from __future__ import annotations


class NgramIndex:
    """Counts of every n-gram of up to max_depth tokens of the inserted sequences."""

    def __init__(self, max_depth: int):
        self.max_depth = max_depth
        self.count = {}        # n-gram (tuple) -> times seen
        self.first = {}        # n-gram -> rank of its first occurrence (for ties between siblings)
        self._clock = 0

    def insert(self, tokens):
        tokens = [int(t) for t in tokens]
        for i in range(len(tokens)):
            for n in range(1, self.max_depth + 1):
                if i + n > len(tokens):
                    break
                g = tuple(tokens[i:i + n])
                self.count[g] = self.count.get(g, 0) + 1
                if g not in self.first:
                    self.first[g] = self._clock
                    self._clock += 1

    def continuations(self, gram):
        """[(token, count)] of the n-grams gram + (token,), most frequent first, ties by first occurrence."""
        if len(gram) + 1 > self.max_depth:
            return []
        found = [(g[-1], c, self.first[g]) for g, c in self.count.items()
                 if len(g) == len(gram) + 1 and g[:-1] == tuple(gram)]
        found.sort(key=lambda x: (-x[1], x[2]))
        return [(t, c) for t, c, _ in found]

    def lookup(self, context):
        """The longest tail of the context (at most max_depth - 1 tokens, at least one) that was
        seen and has a continuation; a tail that was not loses its first token and is tried again."""
        context = [int(t) for t in context]
        for n in range(min(len(context), self.max_depth - 1), 0, -1):
            tail = tuple(context[len(context) - n:])
            if tail in self.count and self.continuations(tail):
                return tail
        return None

    def search_path(self, suffix, depth):
        """Algorithm 2: repeatedly take the top continuation and append it to the context."""
        ctx, path = [int(t) for t in suffix], []
        for _ in range(depth):
            tail = self.lookup(ctx)
            if tail is None:
                break
            tok = self.continuations(tail)[0][0]
            path.append(tok)
            ctx.append(tok)
        return path

    def extract_tree(self, suffix, max_depth, budget):
        """Depth-first extraction below the context, most frequent continuation first, limited in
        depth and in nodes.  Returns (tokens, parents); node 0 is the last token of the suffix."""
        tokens, parents = [int(suffix[-1])], [-1]
        tail = self.lookup(suffix)

        def visit(gram, me, depth):
            if depth >= max_depth:
                return
            for tok, _ in self.continuations(gram):
                if len(tokens) >= budget:
                    return
                tokens.append(tok)
                parents.append(me)
                visit(gram + (tok,), len(tokens) - 1, depth + 1)

        if tail is not None:
            visit(tail, 0, 0)
        return tokens, parents


def self_repetition(prompt, response):
    """Section 4.1: tokens of the response / number of pointer stops."""
    prompt, response = [int(t) for t in prompt], [int(t) for t in response]
    if not response:
        return 0.0
    ptr = stops = 0
    while ptr < len(response):
        history = prompt + response[:ptr]
        best = 0
        for n in range(1, len(response) - ptr + 1):
            piece = response[ptr:ptr + n]
            if any(history[s:s + n] == piece for s in range(len(history) - n + 1)):
                best = n
            else:
                break
        ptr += best if best else 1
        stops += 1
    return len(response) / stops

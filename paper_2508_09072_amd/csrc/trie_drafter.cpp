// Host-side retrieval drafter over the short-term context (Section 4.2; Algorithm 2 with the
// trie as the only structure): an n-gram trie with continuation counts, the greedy search path,
// and the depth-first extraction of a draft tree.  Plain C++ on host memory; no GPU involved.
// It produces the token / parent arrays that the verification step takes.
#include <algorithm>
#include <cstdint>
#include <new>
#include <unordered_map>
#include <vector>

#include "reader.h"

struct reader_trie {
    struct Node {
        int32_t token;
        int32_t count;                    // how often the n-gram that ends here was seen
        std::vector<int32_t> children;    // in order of creation
    };
    int32_t max_depth;
    std::vector<Node> nodes;              // nodes[0] is the root (empty n-gram)
    std::unordered_map<uint64_t, int32_t> edge;   // (node, token) -> child

    static uint64_t key(int32_t node, int32_t token) { return ((uint64_t)(uint32_t)node << 32) | (uint32_t)token; }
    int32_t child(int32_t node, int32_t token) const {
        const auto it = edge.find(key(node, token));
        return it == edge.end() ? -1 : it->second;
    }
    // The node reached by the longest tail of ctx[0..n) that is in the trie, has a continuation
    // and leaves room below it; a tail that is not present loses its first token and is tried
    // again (Section 4.2).  At least one token of context is kept.  -1: no continuation known.
    int32_t descend(const int32_t *ctx, int32_t n) const {
        const int32_t longest = std::min(n, max_depth - 1);
        for (int32_t len = longest; len >= 1; --len) {
            int32_t at = 0;
            for (int32_t i = n - len; i < n && at >= 0; ++i) at = child(at, ctx[i]);
            if (at >= 0 && !nodes[at].children.empty()) return at;
        }
        return -1;
    }
    // children by descending count; equal counts keep their order of creation (stable)
    std::vector<int32_t> ranked_children(int32_t node) const {
        std::vector<int32_t> c = nodes[node].children;
        std::stable_sort(c.begin(), c.end(), [&](int32_t a, int32_t b) { return nodes[a].count > nodes[b].count; });
        return c;
    }
};

extern "C" reader_trie *reader_trie_create(int32_t max_depth) {
    if (max_depth < 2 || max_depth > 4096) return nullptr;
    reader_trie *t = new (std::nothrow) reader_trie;
    if (!t) return nullptr;
    t->max_depth = max_depth;
    try {
        t->nodes.push_back({-1, 0, {}});
    } catch (const std::bad_alloc &) {
        delete t;
        return nullptr;
    }
    return t;
}

extern "C" void reader_trie_destroy(reader_trie *t) { delete t; }

extern "C" int64_t reader_trie_nodes(const reader_trie *t) { return t ? (int64_t)t->nodes.size() : -1; }

extern "C" int reader_trie_insert(reader_trie *t, const int32_t *tokens, int64_t n) {
    if (!t || n < 0 || (n > 0 && !tokens)) return READER_EINVAL;
    try {
        for (int64_t i = 0; i < n; ++i) {
            int32_t at = 0;
            const int64_t end = std::min<int64_t>(n, i + t->max_depth);
            for (int64_t j = i; j < end; ++j) {
                int32_t c = t->child(at, tokens[j]);
                if (c < 0) {
                    if (t->nodes.size() >= 0x7fffffffu) return READER_EUNSUPPORTED;
                    c = (int32_t)t->nodes.size();
                    t->nodes.push_back({tokens[j], 0, {}});
                    t->nodes[at].children.push_back(c);
                    t->edge.emplace(reader_trie::key(at, tokens[j]), c);
                }
                ++t->nodes[c].count;
                at = c;
            }
        }
    } catch (const std::bad_alloc &) {
        return READER_EUNSUPPORTED;
    }
    return READER_OK;
}

extern "C" int32_t reader_trie_search_path(const reader_trie *t, const int32_t *suffix, int32_t n_suffix, int32_t depth,
                                           int32_t *path_tokens) {
    if (!t || n_suffix < 0 || depth < 0 || (n_suffix > 0 && !suffix) || (depth > 0 && !path_tokens)) return -1;
    try {   // (no exception may cross the C boundary: running out of memory is reported as a bad call)
        std::vector<int32_t> ctx(suffix, suffix + n_suffix);
        int32_t k = 0;
        while (k < depth) {
            const int32_t at = t->descend(ctx.data(), (int32_t)ctx.size());
            if (at < 0) break;
            const int32_t best = t->ranked_children(at)[0];
            path_tokens[k++] = t->nodes[best].token;
            ctx.push_back(t->nodes[best].token);
        }
        return k;
    } catch (const std::bad_alloc &) {
        return -1;
    }
}

extern "C" int32_t reader_trie_extract_tree(const reader_trie *t, const int32_t *suffix, int32_t n_suffix,
                                            int32_t max_depth, int32_t budget, int32_t *tokens, int32_t *parents) {
    if (!t || n_suffix < 1 || !suffix || max_depth < 0 || budget < 1 || !tokens || !parents) return -1;
    tokens[0] = suffix[n_suffix - 1];      // the root is the last committed token
    parents[0] = -1;
    int32_t used = 1;
    const int32_t start = t->descend(suffix, n_suffix);
    if (start < 0) return used;
    // depth-first, most frequent continuation first, within the depth and the node budget
    struct Frame { int32_t trie_node, tree_node, depth; };
    try {
        std::vector<Frame> stack;
        stack.push_back({start, 0, 0});
        while (!stack.empty() && used < budget) {
            const Frame f = stack.back();
            stack.pop_back();
            int32_t me = f.tree_node;
            if (f.depth > 0) {                  // (the start node itself is the root, already numbered)
                me = used++;
                tokens[me] = t->nodes[f.trie_node].token;
                parents[me] = f.tree_node;
            }
            if (f.depth < max_depth) {
                const std::vector<int32_t> c = t->ranked_children(f.trie_node);
                for (auto it = c.rbegin(); it != c.rend(); ++it) stack.push_back({*it, me, f.depth + 1});   // best on top
            }
        }
    } catch (const std::bad_alloc &) {
        return -1;
    }
    return used;
}

extern "C" int32_t reader_tree_attach_path(int32_t *tokens, int32_t *parents, int32_t n_nodes, int32_t capacity,
                                           int32_t at_node, const int32_t *path_tokens, int32_t k) {
    if (!tokens || !parents || n_nodes < 1 || capacity < n_nodes || at_node < 0 || at_node >= n_nodes || k < 0 ||
        (k > 0 && !path_tokens))
        return -1;
    int32_t prev = at_node;
    for (int32_t i = 0; i < k && n_nodes < capacity; ++i) {
        tokens[n_nodes] = path_tokens[i];
        parents[n_nodes] = prev;
        prev = n_nodes++;
    }
    return n_nodes;
}

extern "C" double reader_self_repetition(const int32_t *prompt, int64_t n_prompt, const int32_t *response,
                                         int64_t n_response) {
    if (n_prompt < 0 || n_response < 0 || (n_prompt > 0 && !prompt) || (n_response > 0 && !response)) return -1.0;
    if (n_response == 0) return 0.0;
    // history = prompt, then the processed part of the response; a match must lie inside it
    try {
        std::vector<int32_t> hist(prompt, prompt + n_prompt);
        hist.reserve((size_t)(n_prompt + n_response));
        int64_t ptr = 0, advances = 0;
        while (ptr < n_response) {
            int64_t best = 0;
            const int64_t h = (int64_t)hist.size();
            for (int64_t s = 0; s < h; ++s) {
                if (hist[s] != response[ptr]) continue;
                int64_t len = 0;
                while (s + len < h && ptr + len < n_response && hist[s + len] == response[ptr + len]) ++len;
                best = std::max(best, len);
            }
            const int64_t step = best > 0 ? best : 1;
            hist.insert(hist.end(), response + ptr, response + ptr + step);
            ptr += step;
            ++advances;
        }
        return (double)n_response / (double)advances;
    } catch (const std::bad_alloc &) {
        return -1.0;
    }
}

// Test driver: the host-side code of the library (retrieval drafter, tree-shape selection) behind a
// line protocol, to be built with -fsanitize=address,undefined and fed by tests/test_sanitizers.py.
// One command per input line, one answer line per command; numbers separated by blanks.
//   trie D | insert n t.. | nodes | path depth n c.. | tree max_depth budget n c.. | selfrep np p.. nr r..
//   attach n_nodes capacity at_node k  tokens(n_nodes).. parents(n_nodes).. path(k)..
//   order T parents.. alpha.. | select exhaustive T parents.. alpha.. t_draft.. tv.. | bad
#include <cstdio>
#include <iostream>
#include <sstream>
#include <string>
#include <vector>

#include "reader.h"

template <class T>
static std::vector<T> take(std::istringstream &in, long n) {
    std::vector<T> v((size_t)(n > 0 ? n : 0));
    for (auto &x : v) in >> x;
    return v;
}

int main() {
    reader_trie *trie = nullptr;
    std::string line;
    while (std::getline(std::cin, line)) {
        std::istringstream in(line);
        std::string cmd;
        in >> cmd;
        if (cmd == "trie") {
            int d; in >> d;
            reader_trie_destroy(trie);
            trie = reader_trie_create(d);
            std::printf("%d\n", trie ? 1 : 0);
        } else if (cmd == "insert") {
            long n; in >> n;
            auto t = take<int32_t>(in, n);
            std::printf("%d\n", reader_trie_insert(trie, t.data(), n));
        } else if (cmd == "nodes") {
            std::printf("%lld\n", (long long)reader_trie_nodes(trie));
        } else if (cmd == "path") {
            int depth; long n; in >> depth >> n;
            auto c = take<int32_t>(in, n);
            std::vector<int32_t> out((size_t)(depth > 0 ? depth : 1));
            const int k = reader_trie_search_path(trie, c.data(), (int32_t)n, depth, out.data());
            std::printf("%d", k);
            for (int i = 0; i < k; ++i) std::printf(" %d", out[i]);
            std::printf("\n");
        } else if (cmd == "tree") {
            int md, budget; long n; in >> md >> budget >> n;
            auto c = take<int32_t>(in, n);
            std::vector<int32_t> tok((size_t)(budget > 0 ? budget : 1)), par((size_t)(budget > 0 ? budget : 1));
            const int k = reader_trie_extract_tree(trie, c.data(), (int32_t)n, md, budget, tok.data(), par.data());
            std::printf("%d", k);
            for (int i = 0; i < k; ++i) std::printf(" %d", tok[i]);
            for (int i = 0; i < k; ++i) std::printf(" %d", par[i]);
            std::printf("\n");
        } else if (cmd == "selfrep") {
            long np, nr; in >> np;
            auto p = take<int32_t>(in, np);
            in >> nr;
            auto r = take<int32_t>(in, nr);
            std::printf("%.17g\n", reader_self_repetition(p.data(), np, r.data(), nr));
        } else if (cmd == "attach") {
            int n_nodes, cap, at, k; in >> n_nodes >> cap >> at >> k;
            auto tok = take<int32_t>(in, n_nodes), par = take<int32_t>(in, n_nodes);
            auto path = take<int32_t>(in, k);
            tok.resize((size_t)cap); par.resize((size_t)cap);
            const int n = reader_tree_attach_path(tok.data(), par.data(), n_nodes, cap, at, path.data(), k);
            std::printf("%d", n);
            for (int i = 0; i < n; ++i) std::printf(" %d", tok[i]);
            for (int i = 0; i < n; ++i) std::printf(" %d", par[i]);
            std::printf("\n");
        } else if (cmd == "order") {
            int T; in >> T;
            auto par = take<int32_t>(in, T);
            auto al = take<float>(in, T);
            std::vector<int32_t> ord((size_t)(T > 1 ? T - 1 : 1));
            const int n = reader_tree_prune_order(par.data(), al.data(), T, ord.data());
            std::printf("%d", n);
            for (int i = 0; i < n; ++i) std::printf(" %d", ord[i]);
            std::printf("\n");
        } else if (cmd == "select") {
            int ex, T; in >> ex >> T;
            auto par = take<int32_t>(in, T);
            auto al = take<float>(in, T), td = take<float>(in, T), tv = take<float>(in, T);
            std::vector<int32_t> keep((size_t)T);
            double thr = 0.0; int32_t ev = 0;
            const int n = reader_tree_select(par.data(), al.data(), td.data(), tv.data(), T, ex, keep.data(), &thr, &ev);
            std::printf("%d %.17g", n, thr);
            for (int i = 0; i < T && n >= 0; ++i) std::printf(" %d", keep[i]);
            std::printf("\n");
        } else if (cmd == "bad") {
            // every call here has to come back with an error code and touch nothing
            int32_t x[4] = {0, 0, 0, 0};
            float f[4] = {1.f, 1.f, 1.f, 1.f};
            int bad = 0;
            bad += reader_trie_create(1) != nullptr;
            bad += reader_trie_insert(nullptr, x, 4) != READER_EINVAL;
            bad += reader_trie_insert(trie, nullptr, 4) != READER_EINVAL;
            bad += reader_trie_search_path(nullptr, x, 1, 1, x) != -1;
            bad += reader_trie_search_path(trie, x, -1, 1, x) != -1;
            bad += reader_trie_extract_tree(trie, x, 0, 1, 4, x, x) != -1;
            bad += reader_trie_extract_tree(trie, x, 1, 1, 0, x, x) != -1;
            bad += reader_tree_attach_path(x, x, 0, 4, 0, x, 1) != -1;
            bad += reader_tree_attach_path(x, x, 2, 4, 2, x, 1) != -1;
            bad += reader_self_repetition(nullptr, 3, x, 1) != -1.0;
            bad += reader_tree_prune_order(x, f, 2, x) != -1;        // the root's parent is not -1
            bad += reader_tree_select(x, f, f, f, 2, 1, x, nullptr, nullptr) != -1;
            bad += reader_validate_tree(x, 1, 4) != READER_EINVAL;
            bad += reader_trie_nodes(nullptr) != -1;
            std::printf("%d\n", bad);
        } else {
            std::printf("?\n");
        }
        std::fflush(stdout);
    }
    reader_trie_destroy(trie);
    return 0;
}

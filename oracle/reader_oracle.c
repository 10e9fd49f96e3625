/*
 * CPU oracle for the draft-tree verification step of READER (arXiv 2508.09072).
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, plain definition of what the
 * verification step computes.  It shares no code with the HIP library, is never
 * linked into it, and must only be used by the tests, the smoke check and the
 * "cpu_baseline" leg of the benchmark.
 *
 * Arithmetic: every floating-point step is done in IEEE double.  Inputs are bf16
 * bit patterns (uint16_t) widened exactly; nothing is rounded on the way.  There
 * is no tiling, no running (online) softmax, no bit mask and no reordering: each
 * output row is produced by (1) listing the keys the query may see, (2) scoring
 * them, (3) a two-pass softmax, (4) a weighted sum of value rows.
 *
 * What each function follows in the paper:
 *   oracle_ancestor_mask  - Section 3.2 (Tree Decoding): the decoding mask M with
 *                           M_ij = 1 iff node i is an ancestor of node j.  A node
 *                           also sees itself (a chain must reduce to causal
 *                           attention and a one-node tree to plain decoding).
 *   oracle_tree_attn*     - Section 3.2: scaled dot-product attention of the
 *                           gamma tree queries over s cached keys plus the tree
 *                           keys allowed by M.  Appendix C invariant 2: verifying
 *                           a node equals decoding step by step along its path.
 *   oracle_accept_path    - Algorithm 5 (Verify): compare the base model's token
 *                           with the drafted token along the tree, keep the
 *                           longest prefix consistent with the base model;
 *                           Appendix C invariants 2-3: stop at the first mismatch
 *                           and fall back to the base model's token there.
 *   oracle_kv_compact     - Section 4.3 / Algorithm 4: the accepted span is
 *                           appended tightly behind each sample's cache so that
 *                           no hole remains inside it.
 *   oracle_target_argmax  - Algorithm 5: the base model's own (greedy) token at every
 *                           tree node, i.e. the arg max of its logits there; these
 *                           are the tokens the drafted ones are compared with.
 *   oracle_kv_rearrange   - Section 4.3 / Algorithm 4 as the paper runs it on a
 *                           padded cache, every N-th step: per sample, internal
 *                           padding is removed and the real entries are
 *                           concatenated tightly; padding may only remain at the
 *                           end.  Which positions are padding comes from the
 *                           bookkeeping (a validity flag per position), never
 *                           from testing values for zero.
 *
 * Layouts (shared with the library's boundary by definition of the problem):
 *   q               bf16 [B, T, Hq, D]
 *   k_tree, v_tree  bf16 [B, T, Hkv, D]
 *   k_cache,v_cache bf16 [num_pages, Hkv, page_size, D]
 *   page_table      i32  [B, max_pages]      logical page -> physical page
 *   seq_lens        i32  [B]                 prefix length L_b (tree rows excluded)
 *   parents         i32  [B, T]              parents[b][0] = -1, 0 <= parents[b][i] < i
 *   GQA: query head hq reads kv head hq / (Hq / Hkv).
 *
 * Return value of every function: 0 on success, a negative number when the input
 * is not a valid problem instance (malformed tree, bad sizes).
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

static double widen_bf16(uint16_t bits) {
    uint32_t u = ((uint32_t)bits) << 16;
    float f;
    memcpy(&f, &u, sizeof f);
    return (double)f;
}

/* A tree is valid iff node 0 is the only root and every parent precedes its child. */
static int tree_is_valid(const int32_t *parent, int T) {
    if (T < 1 || parent[0] != -1) return 0;
    for (int i = 1; i < T; ++i)
        if (parent[i] < 0 || parent[i] >= i) return 0;
    return 1;
}

/*
 * mask[i*T + t] = 1 iff the query at node i may attend to the key at node t,
 * i.e. t == i or t is an ancestor of i.  depth[i] = number of proper ancestors.
 * Built by walking the parent pointers from each node up to the root.
 */
int oracle_ancestor_mask(const int32_t *parent, int T, uint8_t *mask, int32_t *depth) {
    if (!tree_is_valid(parent, T)) return -1;
    memset(mask, 0, (size_t)T * (size_t)T);
    for (int i = 0; i < T; ++i) {
        int steps = 0;
        for (int t = i; t != -1; t = parent[t]) {
            mask[(size_t)i * T + t] = 1;
            ++steps;
        }
        if (depth) depth[i] = steps - 1;
    }
    return 0;
}

typedef struct {
    int B, T, Hq, Hkv, D, page_size, max_pages;
    double scale;
    const uint16_t *q, *k_tree, *v_tree, *k_cache, *v_cache;
    const int32_t *page_table, *seq_lens;
} attn_problem;

/* Address of the cached row (position j of sequence b, kv head hkv). */
static const uint16_t *cache_row(const attn_problem *p, const uint16_t *cache, int b, int hkv, int j) {
    int64_t page = p->page_table[(int64_t)b * p->max_pages + j / p->page_size];
    int slot = j % p->page_size;
    return cache + (((page * p->Hkv + hkv) * p->page_size) + slot) * (int64_t)p->D;
}

/*
 * One output row: query (b, hq, node i); mask_row[t] says which tree keys it sees.
 * out_row has D doubles; *lse_out receives log(sum_j exp(score_j)) (natural log).
 */
static int attn_row(const attn_problem *p, int b, int hq, int i, const uint8_t *mask_row,
                    double *out_row, double *lse_out) {
    const int D = p->D, T = p->T, L = p->seq_lens[b];
    const int hkv = hq / (p->Hq / p->Hkv);
    const int n_keys = L + T;
    double *score = (double *)malloc(sizeof(double) * (size_t)n_keys);
    double *qd = (double *)malloc(sizeof(double) * (size_t)D);
    uint8_t *seen = (uint8_t *)malloc((size_t)n_keys);
    if (!score || !qd || !seen) { free(score); free(qd); free(seen); return -2; }

    const uint16_t *qrow = p->q + (((int64_t)b * T + i) * p->Hq + hq) * D;
    for (int d = 0; d < D; ++d) qd[d] = widen_bf16(qrow[d]);

    /* (1)+(2): the keys this query sees, and their scaled scores */
    for (int j = 0; j < n_keys; ++j) {
        const uint16_t *krow;
        if (j < L) {
            seen[j] = 1;
            krow = cache_row(p, p->k_cache, b, hkv, j);
        } else {
            int t = j - L;
            seen[j] = mask_row[t];
            krow = p->k_tree + (((int64_t)b * T + t) * p->Hkv + hkv) * D;
        }
        if (!seen[j]) { score[j] = 0.0; continue; }
        double dot = 0.0;
        for (int d = 0; d < D; ++d) dot += qd[d] * widen_bf16(krow[d]);
        score[j] = p->scale * dot;
    }

    /* (3): two-pass softmax over the seen keys (the node itself is always seen) */
    double m = -INFINITY;
    for (int j = 0; j < n_keys; ++j)
        if (seen[j] && score[j] > m) m = score[j];
    double denom = 0.0;
    for (int j = 0; j < n_keys; ++j) {
        score[j] = seen[j] ? exp(score[j] - m) : 0.0;
        denom += score[j];
    }

    /* (4): weighted sum of the value rows */
    for (int d = 0; d < D; ++d) out_row[d] = 0.0;
    for (int j = 0; j < n_keys; ++j) {
        if (!seen[j]) continue;
        const uint16_t *vrow = (j < L)
            ? cache_row(p, p->v_cache, b, hkv, j)
            : p->v_tree + (((int64_t)b * T + (j - L)) * p->Hkv + hkv) * D;
        double w = score[j] / denom;
        for (int d = 0; d < D; ++d) out_row[d] += w * widen_bf16(vrow[d]);
    }
    if (lse_out) *lse_out = m + log(denom);
    free(score); free(qd); free(seen);
    return 0;
}

static int fill_problem(attn_problem *p, int B, int T, int Hq, int Hkv, int D, int page_size,
                        int max_pages, double scale, const uint16_t *q, const uint16_t *k_tree,
                        const uint16_t *v_tree, const uint16_t *k_cache, const uint16_t *v_cache,
                        const int32_t *page_table, const int32_t *seq_lens) {
    if (B < 0 || T < 1 || Hq < 1 || Hkv < 1 || Hq % Hkv != 0 || D < 1 || page_size < 1) return -1;
    p->B = B; p->T = T; p->Hq = Hq; p->Hkv = Hkv; p->D = D;
    p->page_size = page_size; p->max_pages = max_pages;
    p->scale = scale > 0.0 ? scale : 1.0 / sqrt((double)D);
    p->q = q; p->k_tree = k_tree; p->v_tree = v_tree; p->k_cache = k_cache; p->v_cache = v_cache;
    p->page_table = page_table; p->seq_lens = seq_lens;
    for (int b = 0; b < B; ++b) {
        if (seq_lens[b] < 0) return -1;
        if ((int64_t)max_pages * page_size < seq_lens[b]) return -1;
    }
    return 0;
}

/*
 * Whole problem.  out: double [B, T, Hq, D]; lse: double [B, Hq, T] or NULL.
 * The loop over (sequence, kv head) pairs is independent work and is the only
 * thing spread over host threads.
 */
int oracle_tree_attn(int B, int T, int Hq, int Hkv, int D, int page_size, int max_pages, double scale,
                     const uint16_t *q, const uint16_t *k_tree, const uint16_t *v_tree,
                     const uint16_t *k_cache, const uint16_t *v_cache, const int32_t *page_table,
                     const int32_t *seq_lens, const int32_t *parents, double *out, double *lse) {
    attn_problem p;
    int rc = fill_problem(&p, B, T, Hq, Hkv, D, page_size, max_pages, scale, q, k_tree, v_tree,
                          k_cache, v_cache, page_table, seq_lens);
    if (rc) return rc;
    uint8_t *mask = (uint8_t *)malloc((size_t)(B > 0 ? B : 1) * T * T);
    if (!mask) return -2;
    for (int b = 0; b < B; ++b)
        if (oracle_ancestor_mask(parents + (int64_t)b * T, T, mask + (size_t)b * T * T, NULL)) {
            free(mask);
            return -1;
        }
    const int G = Hq / Hkv;
    int failed = 0;
#pragma omp parallel for collapse(2) schedule(dynamic, 1)
    for (int b = 0; b < B; ++b)
        for (int hkv = 0; hkv < Hkv; ++hkv)
            for (int g = 0; g < G; ++g)
                for (int i = 0; i < T; ++i) {
                    int hq = hkv * G + g;
                    double *orow = out + (((int64_t)b * T + i) * Hq + hq) * D;
                    double *l = lse ? lse + ((int64_t)b * Hq + hq) * T + i : NULL;
                    if (attn_row(&p, b, hq, i, mask + ((size_t)b * T + i) * T, orow, l)) {
#pragma omp atomic write
                        failed = 1;
                    }
                }
    free(mask);
    return failed ? -2 : 0;
}

/*
 * Selected rows only: rows is int32 [n_rows, 3] = (b, hq, node).  out: double
 * [n_rows, D]; lse: double [n_rows] or NULL.  Used to check full-size problems
 * on a sample of outputs.
 */
int oracle_tree_attn_rows(int B, int T, int Hq, int Hkv, int D, int page_size, int max_pages,
                          double scale, const uint16_t *q, const uint16_t *k_tree,
                          const uint16_t *v_tree, const uint16_t *k_cache, const uint16_t *v_cache,
                          const int32_t *page_table, const int32_t *seq_lens, const int32_t *parents,
                          int n_rows, const int32_t *rows, double *out, double *lse) {
    attn_problem p;
    int rc = fill_problem(&p, B, T, Hq, Hkv, D, page_size, max_pages, scale, q, k_tree, v_tree,
                          k_cache, v_cache, page_table, seq_lens);
    if (rc) return rc;
    for (int r = 0; r < n_rows; ++r) {
        int b = rows[3 * r], hq = rows[3 * r + 1], i = rows[3 * r + 2];
        if (b < 0 || b >= B || hq < 0 || hq >= Hq || i < 0 || i >= T) return -1;
        if (!tree_is_valid(parents + (int64_t)b * T, T)) return -1;
    }
    int failed = 0;
#pragma omp parallel for schedule(dynamic, 1)
    for (int r = 0; r < n_rows; ++r) {
        int b = rows[3 * r], hq = rows[3 * r + 1], i = rows[3 * r + 2];
        uint8_t *mask = (uint8_t *)malloc((size_t)T * T);
        if (!mask || oracle_ancestor_mask(parents + (int64_t)b * T, T, mask, NULL) ||
            attn_row(&p, b, hq, i, mask + (size_t)i * T, out + (int64_t)r * D, lse ? lse + r : NULL)) {
#pragma omp atomic write
            failed = 1;
        }
        free(mask);
    }
    return failed ? -2 : 0;
}

/*
 * Greedy lossless acceptance (Algorithm 5; Appendix C invariants 2 and 3).
 *
 * target[i] is the base model's own next token after the prefix that ends at
 * node i.  Node 0 (the root) is the last committed token and is always accepted.
 * A non-root node is accepted iff its parent is accepted and its drafted token
 * equals the base model's token at the parent.  The result is the accepted node
 * of greatest depth (lowest node index among equals), the root-to-node path
 * (node ids, padded with -1 up to max_path), the number of accepted non-root
 * nodes, and the bonus token = the base model's token at the last accepted node.
 */
int oracle_accept_path(int B, int T, int max_path, const int32_t *draft, const int32_t *target,
                       const int32_t *parents, int32_t *accept_len, int32_t *path, int32_t *bonus) {
    if (B < 0 || T < 1 || max_path < 1) return -1;
    uint8_t *ok = (uint8_t *)malloc((size_t)T);
    int32_t *depth = (int32_t *)malloc(sizeof(int32_t) * (size_t)T);
    if (!ok || !depth) { free(ok); free(depth); return -2; }
    int rc = 0;
    for (int b = 0; b < B && rc == 0; ++b) {
        const int32_t *par = parents + (int64_t)b * T;
        const int32_t *dr = draft + (int64_t)b * T, *tg = target + (int64_t)b * T;
        if (!tree_is_valid(par, T)) { rc = -1; break; }
        ok[0] = 1; depth[0] = 0;
        int best = 0;
        for (int i = 1; i < T; ++i) {            /* parents precede children */
            depth[i] = depth[par[i]] + 1;
            ok[i] = ok[par[i]] && dr[i] == tg[par[i]];
            if (ok[i] && depth[i] > depth[best]) best = i;   /* strict: lowest index wins ties */
        }
        if (depth[best] + 1 > max_path) { rc = -1; break; }
        int32_t *prow = path + (int64_t)b * max_path;
        for (int j = 0; j < max_path; ++j) prow[j] = -1;
        for (int t = best; t != -1; t = par[t]) prow[depth[t]] = t;
        accept_len[b] = depth[best];
        bonus[b] = tg[best];
    }
    free(ok); free(depth);
    return rc;
}

/*
 * Compaction of the accepted path (Section 4.3, Algorithm 4 restated per step):
 * for j = 0..accept_len[b] the K and V rows of tree node path[b][j] (all kv
 * heads) are written to cache position seq_lens[b] + j through the page table,
 * then seq_lens[b] grows by accept_len[b] + 1.  Everything else is untouched.
 */
int oracle_kv_compact(int B, int T, int Hkv, int D, int page_size, int max_pages, int max_path,
                      const uint16_t *k_tree, const uint16_t *v_tree, const int32_t *path,
                      const int32_t *accept_len, uint16_t *k_cache, uint16_t *v_cache,
                      const int32_t *page_table, int32_t *seq_lens) {
    if (B < 0 || T < 1 || Hkv < 1 || D < 1 || page_size < 1 || max_path < 1) return -1;
    for (int b = 0; b < B; ++b) {
        int n = accept_len[b];
        if (n < 0 || n + 1 > max_path) return -1;
        if ((int64_t)seq_lens[b] + n + 1 > (int64_t)max_pages * page_size) return -1;
        for (int j = 0; j <= n; ++j) {
            int node = path[(int64_t)b * max_path + j];
            if (node < 0 || node >= T) return -1;
        }
    }
    for (int b = 0; b < B; ++b) {
        int n = accept_len[b];
        for (int j = 0; j <= n; ++j) {
            int node = path[(int64_t)b * max_path + j];
            int pos = seq_lens[b] + j;
            int64_t page = page_table[(int64_t)b * max_pages + pos / page_size];
            int slot = pos % page_size;
            for (int h = 0; h < Hkv; ++h) {
                int64_t dst = (((page * Hkv + h) * page_size) + slot) * (int64_t)D;
                int64_t src = (((int64_t)b * T + node) * Hkv + h) * (int64_t)D;
                for (int d = 0; d < D; ++d) {
                    k_cache[dst + d] = k_tree[src + d];
                    v_cache[dst + d] = v_tree[src + d];
                }
            }
        }
        seq_lens[b] += n + 1;
    }
    return 0;
}

/* Number of host threads the parallel loops above will use. */
/*
 * Padded layout: k_pad, v_pad bf16 [NL, B, S, Hkv, D] (NL layers share one validity
 * map), valid u8 [B, S].  In place, per sample and layer: the rows of the valid
 * positions move to the front in their order, every later row up to the old extent
 * (last valid position + 1) becomes zero, rows past the old extent are left alone.
 * valid becomes ones-then-zeros, new_len[b] = number of valid positions.
 * Walking left to right is safe in place: a row never moves to the right.
 */
int oracle_kv_rearrange(int NL, int B, int S, int Hkv, int D, uint16_t *k_pad, uint16_t *v_pad,
                        uint8_t *valid, int32_t *new_len) {
    if (NL < 0 || B < 0 || S < 0 || Hkv < 1 || D < 1) return 1;
    const size_t row = (size_t)Hkv * (size_t)D;
    for (int b = 0; b < B; ++b) {
        uint8_t *vb = valid + (size_t)b * S;
        int extent = 0;
        for (int j = 0; j < S; ++j)
            if (vb[j]) extent = j + 1;
        int n = 0;
        for (int l = 0; l < NL; ++l) {
            uint16_t *kb = k_pad + ((size_t)l * B + b) * (size_t)S * row;
            uint16_t *vv = v_pad + ((size_t)l * B + b) * (size_t)S * row;
            int w = 0;
            for (int j = 0; j < S; ++j) {
                if (!vb[j]) continue;
                if (w != j) {
                    memcpy(kb + (size_t)w * row, kb + (size_t)j * row, row * sizeof(uint16_t));
                    memcpy(vv + (size_t)w * row, vv + (size_t)j * row, row * sizeof(uint16_t));
                }
                ++w;
            }
            for (int j = w; j < extent; ++j) {
                memset(kb + (size_t)j * row, 0, row * sizeof(uint16_t));
                memset(vv + (size_t)j * row, 0, row * sizeof(uint16_t));
            }
            n = w;
        }
        if (NL == 0)
            for (int j = 0; j < S; ++j) n += vb[j] != 0;
        for (int j = 0; j < S; ++j) vb[j] = j < n;
        new_len[b] = n;
    }
    return 0;
}

/*
 * target[r] = index of the largest of logits[r][0..V) (bf16 bit patterns, compared as
 * the values they encode), the lowest index among equals; NaNs are skipped, a row
 * without any number gives 0.
 */
int oracle_target_argmax(int rows, int V, const uint16_t *logits, int32_t *target) {
    if (rows < 0 || V < 1) return 1;
    for (int r = 0; r < rows; ++r) {
        const uint16_t *row = logits + (size_t)r * V;
        int best_i = -1;
        double best_v = 0.0;
        for (int v = 0; v < V; ++v) {
            const double x = widen_bf16(row[v]);
            if (x != x) continue;
            if (best_i < 0 || x > best_v) { best_i = v; best_v = x; }
        }
        target[r] = best_i < 0 ? 0 : best_i;
    }
    return 0;
}

int oracle_num_threads(void) {
    int n = 1;
#pragma omp parallel
    {
#pragma omp single
        n =
#ifdef _OPENMP
            omp_get_num_threads();
#else
            1;
#endif
    }
    return n;
}

/* Test driver: the CPU oracle (oracle/reader_oracle.c) on one small problem read from a file, results
 * written to another, to be built with -fsanitize=address,undefined by tests/test_sanitizers.py.
 * Input: 12 int32 (B T Hq Hkv D page_size max_pages num_pages max_path n_rows V argmax_rows), then the
 * arrays in the order they are read below.  Output: the results, raw, in the order they are written. */
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>

int oracle_ancestor_mask(const int32_t *parent, int T, uint8_t *mask, int32_t *depth);
int oracle_tree_attn(int B, int T, int Hq, int Hkv, int D, int page_size, int max_pages, double scale,
                     const uint16_t *q, const uint16_t *k_tree, const uint16_t *v_tree,
                     const uint16_t *k_cache, const uint16_t *v_cache, const int32_t *page_table,
                     const int32_t *seq_lens, const int32_t *parents, double *out, double *lse);
int oracle_tree_attn_rows(int B, int T, int Hq, int Hkv, int D, int page_size, int max_pages,
                          double scale, const uint16_t *q, const uint16_t *k_tree,
                          const uint16_t *v_tree, const uint16_t *k_cache, const uint16_t *v_cache,
                          const int32_t *page_table, const int32_t *seq_lens, const int32_t *parents,
                          int n_rows, const int32_t *rows, double *out, double *lse);
int oracle_accept_path(int B, int T, int max_path, const int32_t *draft, const int32_t *target,
                       const int32_t *parents, int32_t *accept_len, int32_t *path, int32_t *bonus);
int oracle_kv_compact(int B, int T, int Hkv, int D, int page_size, int max_pages, int max_path,
                      const uint16_t *k_tree, const uint16_t *v_tree, const int32_t *path,
                      const int32_t *accept_len, uint16_t *k_cache, uint16_t *v_cache,
                      const int32_t *page_table, int32_t *seq_lens);
int oracle_target_argmax(int rows, int V, const uint16_t *logits, int32_t *target);

static void *get(FILE *f, size_t bytes) {
    void *p = malloc(bytes ? bytes : 1);
    if (!p || fread(p, 1, bytes, f) != bytes) { fprintf(stderr, "short input\n"); exit(3); }
    return p;
}
static void put(FILE *f, const void *p, size_t bytes) {
    if (fwrite(p, 1, bytes, f) != bytes) { fprintf(stderr, "short output\n"); exit(4); }
}

int main(int argc, char **argv) {
    if (argc != 3) return 2;
    FILE *in = fopen(argv[1], "rb"), *out = fopen(argv[2], "wb");
    if (!in || !out) return 2;
    int32_t h[12];
    if (fread(h, 4, 12, in) != 12) return 3;
    const int B = h[0], T = h[1], Hq = h[2], Hkv = h[3], D = h[4], ps = h[5], mp = h[6], np = h[7], P = h[8], nr = h[9], V = h[10], ar = h[11];
    const size_t qn = (size_t)B * T * Hq * D, tn = (size_t)B * T * Hkv * D, cn = (size_t)np * Hkv * ps * D;
    uint16_t *q = get(in, qn * 2), *kt = get(in, tn * 2), *vt = get(in, tn * 2), *kc = get(in, cn * 2), *vc = get(in, cn * 2);
    int32_t *table = get(in, (size_t)B * mp * 4), *lens = get(in, (size_t)B * 4), *parents = get(in, (size_t)B * T * 4);
    int32_t *draft = get(in, (size_t)B * T * 4), *target = get(in, (size_t)B * T * 4), *rows = get(in, (size_t)nr * 3 * 4);
    uint16_t *logits = get(in, (size_t)ar * V * 2);
    int rc = 0;

    uint8_t *mask = malloc((size_t)T * T);
    int32_t *depth = malloc((size_t)T * 4);
    for (int b = 0; b < B; ++b) {
        rc |= oracle_ancestor_mask(parents + (size_t)b * T, T, mask, depth);
        put(out, mask, (size_t)T * T);
        put(out, depth, (size_t)T * 4);
    }
    double *o = malloc(qn * 8 + 8), *lse = malloc((size_t)B * Hq * T * 8 + 8);
    rc |= oracle_tree_attn(B, T, Hq, Hkv, D, ps, mp, 0.0, q, kt, vt, kc, vc, table, lens, parents, o, lse);
    put(out, o, qn * 8);
    put(out, lse, (size_t)B * Hq * T * 8);
    double *ro = malloc((size_t)nr * D * 8 + 8), *rl = malloc((size_t)nr * 8 + 8);
    rc |= oracle_tree_attn_rows(B, T, Hq, Hkv, D, ps, mp, 0.0, q, kt, vt, kc, vc, table, lens, parents, nr, rows, ro, rl);
    put(out, ro, (size_t)nr * D * 8);
    put(out, rl, (size_t)nr * 8);
    int32_t *al = malloc((size_t)B * 4 + 4), *path = malloc((size_t)B * P * 4 + 4), *bonus = malloc((size_t)B * 4 + 4);
    rc |= oracle_accept_path(B, T, P, draft, target, parents, al, path, bonus);
    put(out, al, (size_t)B * 4);
    put(out, path, (size_t)B * P * 4);
    put(out, bonus, (size_t)B * 4);
    rc |= oracle_kv_compact(B, T, Hkv, D, ps, mp, P, kt, vt, path, al, kc, vc, table, lens);
    put(out, kc, cn * 2);
    put(out, vc, cn * 2);
    put(out, lens, (size_t)B * 4);
    int32_t *am = malloc((size_t)ar * 4 + 4);
    rc |= oracle_target_argmax(ar, V, logits, am);
    put(out, am, (size_t)ar * 4);
    fclose(in);
    fclose(out);
    free(q); free(kt); free(vt); free(kc); free(vc); free(table); free(lens); free(parents); free(draft); free(target);
    free(rows); free(logits); free(mask); free(depth); free(o); free(lse); free(ro); free(rl); free(al); free(path);
    free(bonus); free(am);
    return rc ? 5 : 0;
}

/*
 * reader.h - C ABI of the MI355X (gfx950) draft-tree verification library for
 * READER (arXiv 2508.09072), the lossless retrieval-drafted speculative decoder.
 *
 * One verification step of the base model over a draft tree (Algorithm 1, "Verify
 * and accept"; Algorithm 5) is, per transformer layer, a tree-masked attention
 * (Section 3.2) and, once per step, a greedy acceptance of the longest draft path
 * that agrees with the base model (Algorithm 5, Appendix C) followed by the
 * append of that path's K/V rows to each sample's cache so that it stays tight
 * (Section 4.3, Algorithm 4).  This library is those three operations, the steps
 * right next to them (the base model's tokens from its logits, greedy or sampled
 * with coupled uniforms; the paper's periodic rearrangement of a padded cache;
 * compaction when the tree rows already sit in every layer's cache), and the
 * host-side retrieval drafter that makes draft trees from the short-term context.
 *
 * Conventions
 *  - Every pointer is a DEVICE pointer unless its name ends in `_host` or the
 *    comment of the entry point says otherwise (the drafter works on host memory).  All
 *    device buffers are borrowed: the caller allocates, owns and frees them.  On the
 *    device side the library
 *    allocates nothing, frees nothing and never synchronises; each call enqueues
 *    its kernels on `stream` (a hipStream_t passed as void*, NULL = default
 *    stream) and returns.  Results are valid once the stream reaches that point.
 *  - bf16 tensors are passed as `void*`; element (i,j,k,l) of a tensor of shape
 *    [A,B,C,D] sits at ((i*B + j)*C + k)*D + l (C order, no padding).
 *  - Return value: READER_OK (0) or a negative READER_E* code.  Argument checks
 *    happen on the host before anything is enqueued, so a failed call has no
 *    effect.  Nothing is printed, no exception crosses the boundary.
 *  - Data-dependent problems that only the device can see (a malformed tree, a
 *    page id outside the pool, an accepted length that does not fit) never fault:
 *    the kernel skips the offending item and ORs a READER_STATUS_* bit into the
 *    optional device word `status`.  In the attention a bad link of a tree counts as
 *    a root link and the cached keys behind a bad page id are left out of the sums;
 *    tree rows that live in the cache (in-cache layout) behind a bad page id leave
 *    the outputs of their sequence unspecified (finite or NaN, never a fault).
 *  - Tree convention: node 0 is the root = the last committed token (it comes
 *    from the base model, acceptance rate 1, Section 3.3); parents[b][0] = -1 and
 *    0 <= parents[b][i] < i.  Trees may differ between sequences; the paper's
 *    fixed per-batch shape is the case where all rows of `parents` are equal.
 *  - Grouped-query attention: query head hq reads kv head hq / (Hq / Hkv).
 *  - Paged cache: position j of sequence b lives in physical page
 *    page_table[b][j / page_size], slot j % page_size.
 *  - Threads: the compute entry points keep no state between calls and may be called
 *    from several host threads, each on its own stream and with its own workspace,
 *    outputs and status word; calls that share a workspace or write the same cache
 *    pages or lengths must be ordered by the caller (one stream, or events).
 *    reader_last_error_detail and the reader_profile_* hooks share one process-wide
 *    buffer and are meant for one thread.  The library reads no environment variable.
 *  - Size limits (a call beyond them returns READER_EUNSUPPORTED, nothing is enqueued):
 *    T <= READER_MAX_T, D in {64, 128}, page_size == READER_PAGE_SIZE, Hq / Hkv <= 16,
 *    B <= READER_MAX_B, num_pages * Hkv < 2^31, B * max_pages_per_seq < 2^31.
 */
#ifndef READER_H
#define READER_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

enum {
    READER_OK = 0,
    READER_EINVAL = -1,       /* null pointer, non-positive size, inconsistent dims, malformed host tree */
    READER_EUNSUPPORTED = -2, /* a size outside what the kernels are built for */
    READER_EWORKSPACE = -3,   /* workspace pointer missing or too small */
    READER_EHIP = -4          /* the HIP runtime refused a launch */
};

enum {
    READER_STATUS_BAD_TREE = 1, /* parents[b][0] != -1 or parents[b][i] not in [0, i) */
    READER_STATUS_BAD_PAGE = 2, /* a page id outside [0, num_pages) was met */
    READER_STATUS_BAD_PATH = 4  /* accept_len/path entry out of range, or path longer than max_path */
};

enum {
    READER_MAX_T = 128,  /* draft-tree nodes per sequence */
    READER_PAGE_SIZE = 16,
    READER_MAX_B = 4096  /* sequences per call (what the in-kernel prefix scan over the lengths is sized for) */
};

/* Problem sizes; plain data, passed by const pointer (host memory). */
typedef struct reader_dims {
    int32_t B;                 /* sequences in the batch, 0..READER_MAX_B (0 = nothing to do) */
    int32_t T;                 /* draft-tree nodes per sequence, 1..READER_MAX_T */
    int32_t Hq;                /* query heads */
    int32_t Hkv;               /* kv heads, Hq % Hkv == 0, Hq / Hkv <= 16 */
    int32_t D;                 /* head dimension, 64 or 128 */
    int32_t page_size;         /* tokens per cache page, must be READER_PAGE_SIZE */
    int32_t max_pages_per_seq; /* row stride of page_table */
    int32_t max_path;          /* row stride of `path`: >= deepest node's depth + 1, <= T */
    int64_t num_pages;         /* pages in the pool (first dim of k_cache / v_cache) */
    float sm_scale;            /* softmax scale; <= 0 selects 1/sqrt(D) */
    int32_t variant;           /* 0 = default kernel selection.  1 = force the scalar reference
                                  kernel of reader_tree_attn (slow; for cross-checks only) */
} reader_dims;

/* Library version string (static storage). */
const char *reader_version(void);

/* Text for a READER_E* code (static storage). */
const char *reader_strerror(int code);

/* Which HIP call failed last and how, after a READER_EHIP return ("" if none so far; static storage). */
const char *reader_last_error_detail(void);

/*
 * Host-side check of the tree convention above on HOST arrays parents_host[B][T].
 * Pure function, no GPU needed.  READER_OK or READER_EINVAL.
 */
int reader_validate_tree(const int32_t *parents_host, int32_t B, int32_t T);

/*
 * Bytes of device workspace reader_tree_attn needs for these dims when no
 * sequence is longer than max_seq_len.  Pure host function.  Returns 0 when the
 * dims are invalid.  The workspace holds the partial (bf16 output normalised by its
 * own sum, running max, running sum) records of key ranges that were split across workgroups; its
 * contents are meaningless between calls and it may be shared by calls that are
 * ordered on one stream.
 */
size_t reader_workspace_bytes(const reader_dims *dims, int32_t max_seq_len);

/*
 * How reader_tree_attn would run these dims when no sequence is longer than max_seq_len: which of its
 * kernels, how many query rows a workgroup carries, into how many chunks the rows of a (sequence, kv head)
 * pair are cut, and how many ranges of key tiles the launch has (workgroups = key_ranges * row_chunks).
 * For benchmarks and profiles that name the kernel they time; the choice follows Section 3.2's
 * memory-bound / compute-bound distinction (few query rows: stream K/V with dedicated copy wavefronts;
 * many: all wavefronts on the matrix cores).  Pure host function; honours reader_tuning_override.
 * READER_OK, or the error reader_tree_attn would return for the dims.
 */
enum reader_attn_kernel {
    READER_ATTN_KERNEL_SCALAR = 0,          /* dims->variant = 1: the scalar reference kernel */
    READER_ATTN_KERNEL_ROWS128 = 1,         /* tree_attn_mfma_kernel<D, 4>: 128 rows, 4 computing + 4 copying wavefronts */
    READER_ATTN_KERNEL_ROWS256_WAVES8 = 2,  /* tree_attn_mfma_kernel<D, 8>: 256 rows, 8 wavefronts of 32 rows */
    READER_ATTN_KERNEL_ROWS256_WAVES4 = 3   /* tree_attn_wide_kernel<D>: 256 rows, 4 wavefronts of 64 rows */
};
typedef struct reader_attn_plan_t {
    int32_t kernel;                /* enum reader_attn_kernel */
    int32_t rows_per_workgroup;    /* 128 or 256 (0 for the scalar kernel) */
    int32_t row_chunks;
    int32_t key_ranges;
} reader_attn_plan_t;
int reader_attn_plan(const reader_dims *dims, int32_t max_seq_len, reader_attn_plan_t *plan);

/*
 * Tree-masked attention (Section 3.2; Appendix C invariant 2).
 * For every sequence b, query head hq and tree node i:
 *     out[b,i,hq,:] = sum_j softmax_j( sm_scale * <q[b,i,hq,:], k_j> ) * v_j
 * where j runs over the seq_lens[b] cached positions of b (kv head hq/(Hq/Hkv))
 * and over the tree nodes that are i itself or an ancestor of i.
 *
 *   q            bf16 [B, T, Hq, D]                     in
 *   k_tree,v_tree bf16 [B, T, Hkv, D]                   in   K/V rows of the tree nodes; or both NULL:
 *                the in-cache layout (Section 4.3), where the forward pass wrote the row of node n
 *                of sequence b at cache position seq_lens[b] + n; page_table must then map pages
 *                for [0, seq_lens[b] + T) and max_pages_per_seq * page_size >= max_seq_len + T
 *   k_cache,v_cache bf16 [num_pages, Hkv, page_size, D] in   paged prefix cache
 *   page_table   i32 [B, max_pages_per_seq]             in   must map pages for [0, seq_lens[b])
 *   seq_lens     i32 [B]                                in   prefix length L_b, tree rows excluded
 *   parents      i32 [B, T]                             in
 *   out          bf16 [B, T, Hq, D]                     out  fp32 accumulation, rounded to nearest even
 *   lse          f32 [B, Hq, T] or NULL                 out  natural-log sum of exp of the scaled scores
 *   max_seq_len  upper bound of seq_lens[b] (host value) used to size the launch; a sequence
 *                longer than this is truncated to it and nothing faults
 *   workspace    >= reader_workspace_bytes(dims, max_seq_len) bytes, 256-byte aligned
 *   status       i32 [1] or NULL                        in/out  READER_STATUS_* bits are ORed in
 *
 * Arithmetic: bf16 products accumulated in fp32 on the matrix cores; softmax
 * weights are rounded to bf16 before they multiply V.  Rows of a malformed tree
 * are computed as if the bad node were a root.
 */
int reader_tree_attn(const reader_dims *dims,
                     const void *q, const void *k_tree, const void *v_tree,
                     const void *k_cache, const void *v_cache,
                     const int32_t *page_table, const int32_t *seq_lens, const int32_t *parents,
                     void *out, float *lse,
                     int32_t max_seq_len, void *workspace, size_t workspace_bytes,
                     int32_t *status, void *stream);

/*
 * reader_tree_attn for callers that cannot allocate device memory or hand in a workspace: code
 * under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments
 * (without workspace and workspace_bytes), same kernels and the same results as reader_tree_attn
 * with dims->variant = 0; the partial records go to a workspace of READER_NOALLOC_WORKSPACE_BYTES
 * that is part of the library's device code (every GPU the library is used on holds its own copy
 * until the process ends).  The call allocates and frees nothing, on the host or the device.
 *
 *  - Dims whose reader_workspace_bytes(dims, max_seq_len) exceeds READER_NOALLOC_WORKSPACE_BYTES
 *    are refused with READER_EWORKSPACE (reader_last_error_detail says by how much).  The planner
 *    keeps key ranges x row chunks within the number of compute units, so the records never need
 *    more than 34.7 MB and the limit covers every shape with B * Hkv up to about 600,000 (the
 *    header holds 8 bytes per (sequence, kv head)); more ranges forced with
 *    reader_tuning_override can exceed it.
 *  - All calls on one GPU share that GPU's workspace: calls that may overlap in time (different
 *    streams, or host threads without ordering) race on it and must be ordered by the caller.
 *  - The first call on a device looks up the workspace's device address (this may load the
 *    library's device code).  A call with dims->B == 0 does only that and is the way to set a
 *    device up ahead of time, outside any graph capture.
 * dims->variant must be 0.  Returns as reader_tree_attn, READER_EUNSUPPORTED for a device index
 * above 63.
 */
#define READER_NOALLOC_WORKSPACE_BYTES (40u << 20)
int reader_tree_attn_noalloc(const reader_dims *dims,
                             const void *q, const void *k_tree, const void *v_tree,
                             const void *k_cache, const void *v_cache,
                             const int32_t *page_table, const int32_t *seq_lens, const int32_t *parents,
                             void *out, float *lse,
                             int32_t max_seq_len, int32_t *status, void *stream);

/*
 * Greedy lossless acceptance (Algorithm 5; Appendix C invariants 2 and 3).
 * target_tokens[b][i] is the base model's own next token after the prefix that
 * ends at node i.  A non-root node is accepted iff its parent is accepted and
 * draft_tokens[b][i] == target_tokens[b][parents[b][i]]; draft_tokens[b][0] is
 * ignored.  Among accepted nodes the deepest wins, the lowest node id among
 * equally deep ones (siblings may carry equal tokens, Section 4.2 "deepening").
 *
 *   draft_tokens, target_tokens, parents   i32 [B, T]       in
 *   accept_len   i32 [B]            out  number of accepted non-root nodes, 0..max_path-1
 *   path         i32 [B, max_path]  out  node ids root..terminal, then -1
 *   bonus_token  i32 [B]            out  target token at the terminal node (always committed)
 *   status       i32 [1] or NULL    in/out
 *
 * A path deeper than max_path-1 is cut at max_path-1 and READER_STATUS_BAD_PATH is set.
 * Integer work; results are exact.
 */
int reader_accept_path(const reader_dims *dims,
                       const int32_t *draft_tokens, const int32_t *target_tokens,
                       const int32_t *parents,
                       int32_t *accept_len, int32_t *path, int32_t *bonus_token,
                       int32_t *status, void *stream);

/*
 * Compaction of the accepted path into the cache (Section 4.3; Algorithm 4, done
 * every step so that no padding ever enters a sample's cache).  For every b and
 * j = 0..accept_len[b]: the K and V rows (all kv heads) of tree node path[b][j]
 * are copied to cache position seq_lens[b] + j, then seq_lens[b] += accept_len[b] + 1.
 * The root row (j = 0) is included: its K/V were first computed in this step.
 *
 *   k_tree, v_tree   bf16 [B, T, Hkv, D]                    in
 *   path             i32 [B, max_path], accept_len i32 [B]  in
 *   k_cache, v_cache bf16 [num_pages, Hkv, page_size, D]    in/out
 *   page_table       i32 [B, max_pages_per_seq]             in   must map pages for
 *                                                                [0, seq_lens[b] + accept_len[b] + 1)
 *   seq_lens         i32 [B]                                in/out
 *   status           i32 [1] or NULL                        in/out
 *
 * A sequence whose accept_len, path entry, target position or page id is out of
 * range is left untouched (cache and seq_lens) and a status bit is set.  Bit-exact copy.
 */
int reader_kv_compact(const reader_dims *dims,
                      const void *k_tree, const void *v_tree,
                      const int32_t *path, const int32_t *accept_len,
                      void *k_cache, void *v_cache, const int32_t *page_table,
                      int32_t *seq_lens, int32_t *status, void *stream);

/*
 * Compaction in the in-cache layout, all layers of the model in one call (Section 4.3;
 * Algorithm 4 applied every step).  The step's forward pass wrote the draft tree's K/V rows
 * behind each sequence in every layer's cache: node n of sequence b at position
 * seq_lens[b] + n.  For every b, layer, kv head and j = 1..accept_len[b], position
 * seq_lens[b] + j receives the row that position seq_lens[b] + path[b][j] held before the
 * call (the root, j = 0, is in place); then seq_lens[b] += accept_len[b] + 1.  Rows behind the
 * new length keep what they held.  The move is done in place: node ids increase along a path
 * (a parent precedes its children), so path[b][j] >= j and no row is overwritten before it
 * has been read.
 *
 *   num_layers       >= 0 (0: only the lengths are updated)
 *   path             i32 [B, max_path], accept_len i32 [B]               in
 *   k_cache, v_cache bf16 [num_layers, num_pages, Hkv, page_size, D]     in/out
 *   page_table       i32 [B, max_pages_per_seq]   in   must map pages for every position
 *                                                      the call touches
 *   seq_lens         i32 [B]                      in/out
 *   status           i32 [1] or NULL              in/out
 *
 * A sequence whose accept_len is out of range, whose path does not start at node 0 or does
 * not increase strictly, or that would touch a position outside the page table or a page id
 * out of range is left untouched (cache and seq_lens) and READER_STATUS_BAD_PATH /
 * READER_STATUS_BAD_PAGE is set.  Bit-exact copy.  dims->Hq and dims->sm_scale are not used.
 * One kernel launch: the workgroup of a sequence that finishes last writes its new length, found through
 * per-sequence counters that are device memory of the library (zero between calls).  Two calls that run on
 * one GPU at the same time (different streams) would share those counters: order them.
 * Returns READER_OK, READER_EINVAL (bad dims, num_layers outside 0..65535, null pointer).
 */
int reader_kv_compact_layers(const reader_dims *dims, int32_t num_layers,
                             const int32_t *path, const int32_t *accept_len,
                             void *k_cache, void *v_cache, const int32_t *page_table,
                             int32_t *seq_lens, int32_t *status, void *stream);

/*
 * One whole verification step (Algorithm 5: base-model pass over the draft tree, longest
 * accepted path; Section 4.3 / Algorithm 4: the accepted rows join the cache), with the
 * arguments, layouts, results and status bits of
 *     reader_tree_attn -> reader_accept_path -> reader_kv_compact
 * called in that order on one stream, but in two kernel launches instead of four: the
 * second launch merges the attention partials, accepts a path per sequence and compacts
 * it.  target_tokens are an input here too (the base model's tokens come from outside
 * this library), so the attention output is not consulted by the acceptance.
 * k_cache, v_cache and seq_lens are read by the attention and then updated by the
 * compaction.  dims->variant must be 0.  Errors as for the three calls.
 *
 * k_tree and v_tree both NULL: the in-cache layout of reader_tree_attn, one layer.  The step
 * is then reader_tree_attn -> reader_accept_path -> reader_kv_compact_layers(num_layers = 1)
 * on k_cache, v_cache [num_pages, Hkv, page_size, D]: the accepted rows move in place (one
 * more small launch).  A model with several layers runs the attention of each layer, and
 * after the last one reader_accept_path and one reader_kv_compact_layers over all of them.
 */
int reader_verify_step(const reader_dims *dims,
                       const void *q, const void *k_tree, const void *v_tree,
                       void *k_cache, void *v_cache,
                       const int32_t *page_table, int32_t *seq_lens,
                       const int32_t *parents,
                       const int32_t *draft_tokens, const int32_t *target_tokens,
                       void *out, float *lse,
                       int32_t *accept_len, int32_t *path, int32_t *bonus_token,
                       int32_t max_seq_len, void *workspace, size_t workspace_bytes,
                       int32_t *status, void *stream);

/*
 * Periodic rearrangement of a padded cache (Section 4.3; Algorithm 4, KVCacheRearrange).
 * The padded layout is the one the paper starts from: every sample owns S slots, all
 * samples append at one common position, and a sample that accepted fewer tokens than
 * the longest acceptance of a step is padded.  Which slots hold a token is bookkeeping
 * (`valid`), never read off the values.  In place, for every sample b and layer l:
 *     the rows of the valid positions move to the front, in their order;
 *     every later row up to the old extent (last valid position + 1) becomes zero;
 *     rows past the old extent, and rows in front of the first hole, are not touched.
 * valid[b] becomes ones-then-zeros and new_len[b] the number of valid positions.
 *
 *   k_pad, v_pad  bf16 [NL, B, S, Hkv, D]   in/out   NL layers share one validity map
 *   valid         u8   [B, S]               in/out   nonzero = the slot holds a token
 *   new_len       i32  [B]                  out
 *   scratch       >= reader_kv_rearrange_scratch_bytes(B, S) bytes of device memory,
 *                 4-byte aligned; contents meaningless between calls
 * D must be 64 or 128 and NL * B * (Hkv + 1) below 2^31 (READER_EUNSUPPORTED otherwise).
 * Two launches (scan of the flags; the moves and the clearing).  Returns READER_OK or a READER_E* code
 * (nothing is enqueued then).
 */
size_t reader_kv_rearrange_scratch_bytes(int32_t B, int32_t S);
int reader_kv_rearrange(int32_t NL, int32_t B, int32_t S, int32_t Hkv, int32_t D,
                        void *k_pad, void *v_pad, uint8_t *valid, int32_t *new_len,
                        void *scratch, size_t scratch_bytes, void *stream);

/*
 * The base model's greedy tokens from its logits (Algorithm 5, "compare base logits with
 * drafted tokens"): target_tokens[r] = argmax over v of logits[r][v], for the B*T rows of
 * a verification step; the result is the target_tokens input of reader_accept_path.
 *
 *   logits         bf16 [rows, V]   in    compared exactly as bf16 values
 *   target_tokens  i32  [rows]      out   lowest index among equal maxima; a NaN is never
 *                                         the maximum (a row of NaNs gives 0)
 * Returns READER_OK or READER_EINVAL (rows < 0, V < 1, null pointer).
 */
int reader_target_argmax(int32_t rows, int32_t V, const void *logits, int32_t *target_tokens, void *stream);

/*
 * The base model's tokens under a sampling policy (Appendix C, randomized decoding).  The
 * policy is a map F(distribution, u) fed with one uniform per decoding position, and the
 * speculative run draws with the same uniforms as the plain run, which makes the two runs
 * emit the same tokens.  F is inverse-CDF sampling of softmax(logits / temperature):
 *   target_tokens[b][n] = lowest k with  sum_{v <= k} w_v  >  u * sum_v w_v,
 *   w_v = exp((logits[b][n][v] - max_v logits[b][n][v]) / temperature),
 *   u = uniforms[b][depth(n)]   (the root has depth 0; every node of one depth stands for the
 *                                same position and therefore draws with the same uniform).
 * The result is the target_tokens input of reader_accept_path, whose bonus token is then the
 * policy's own draw at the first position the draft does not cover.  Top-k / top-p filtering
 * is not applied.
 *
 *   logits         bf16 [B, T, V]  in    a NaN carries no probability; a +inf logit takes all of
 *                                        it (shared equally among the +inf tokens of the row)
 *   parents        i32  [B, T]     in    as for reader_tree_attn; a pointer that does not lead
 *                                        towards the root ends the depth walk there
 *   uniforms       f32  [B, T]     in    values in [0, 1); entry d serves depth d
 *   temperature    in [READER_MIN_TEMPERATURE, READER_MAX_TEMPERATURE] (below the lower end the
 *                  policy is the arg max in all but name: use reader_target_argmax)
 *   target_tokens  i32  [B, T]     out   a token of zero weight is never returned; a row
 *                                        without any weight gives 0
 * Sums are formed in fp32 (blocks of 512 tokens, then over the blocks): where u * total lies
 * within rounding (about 1e-5 of the total) of a boundary between two tokens' cumulative
 * weights, either of them may be returned.
 * Returns READER_OK or READER_EINVAL (B < 0, T outside 1..READER_MAX_T, V outside
 * 1..READER_MAX_SAMPLE_V, temperature outside its range or not a number, null pointer).
 */
#define READER_MAX_SAMPLE_V 4194304
#define READER_MIN_TEMPERATURE 1e-6f
#define READER_MAX_TEMPERATURE 1e6f
int reader_target_sample(int32_t B, int32_t T, int32_t V, const void *logits, const int32_t *parents,
                         const float *uniforms, float temperature, int32_t *target_tokens, void *stream);

/*
 * Host-side retrieval drafter over the short-term context (Section 4.2; Algorithm 2 with the
 * trie as its only structure).  Everything below runs on the CPU with HOST pointers; it makes
 * the token and parent arrays a verification step takes.  Not thread-safe per trie.
 *
 * The trie holds every n-gram of up to max_depth tokens of the sequences inserted so far, with
 * the number of times each was seen; inserting n tokens costs O(n * max_depth).
 * Looking up a context: the longest tail of the context (at most max_depth - 1 tokens, at least
 * one) that is in the trie and has a continuation; a tail that is not there loses its first
 * token and is tried again.  Continuations are ranked by descending count, equal counts in the
 * order they were first seen.
 */
typedef struct reader_trie reader_trie;
/* max_depth in 2..4096; NULL on a bad argument or when memory runs out */
reader_trie *reader_trie_create(int32_t max_depth);
void reader_trie_destroy(reader_trie *trie);   /* NULL is allowed */
/* number of nodes including the root, -1 for NULL */
int64_t reader_trie_nodes(const reader_trie *trie);
/* READER_OK, READER_EINVAL (NULL trie, n < 0, NULL tokens), READER_EUNSUPPORTED (out of memory) */
int reader_trie_insert(reader_trie *trie, const int32_t *tokens, int64_t n);
/*
 * SearchPath (Algorithm 2): starting from the context `suffix`, up to `depth` times take the
 * best-ranked continuation of the current context and append it to the context.  Writes the k
 * tokens found to path_tokens[0..k) and returns k (0 <= k <= depth), or -1 on a bad argument.
 */
int32_t reader_trie_search_path(const reader_trie *trie, const int32_t *suffix, int32_t n_suffix, int32_t depth,
                                int32_t *path_tokens);
/*
 * Draft tree by depth-first extraction (Section 4.2): the root (node 0) is the last token of
 * `suffix`; below it the continuations of the context, most frequent first, depth-first, at
 * most max_depth levels and `budget` nodes in all.  Nodes are numbered in the order they are
 * visited, so a parent precedes its children.  tokens, parents: i32 [budget] out.
 * Returns the number of nodes (>= 1), or -1 on a bad argument (n_suffix < 1, budget < 1, ...).
 */
int32_t reader_trie_extract_tree(const reader_trie *trie, const int32_t *suffix, int32_t n_suffix,
                                 int32_t max_depth, int32_t budget, int32_t *tokens, int32_t *parents);
/*
 * Attaches a path as one chain below node at_node of a tree of n_nodes nodes stored in arrays
 * of `capacity` entries (the widening and deepening of Section 4.2 attach one retrieved
 * path at the root, or at a drafted node); tokens that do not fit are dropped.  Returns the
 * new number of nodes, or -1 on a bad argument.
 */
int32_t reader_tree_attach_path(int32_t *tokens, int32_t *parents, int32_t n_nodes, int32_t capacity,
                                int32_t at_node, const int32_t *path_tokens, int32_t k);
/*
 * Self-repetition metric (Section 4.1): a pointer walks the response; at each stop the longest
 * run of tokens starting at the pointer that also occurs in the prompt or in the part of the
 * response already walked (entirely inside it) is skipped, or one token if there is none.
 * Returns response tokens / number of stops (0 for an empty response, -1 on a bad argument).
 */
double reader_self_repetition(const int32_t *prompt, int64_t n_prompt, const int32_t *response, int64_t n_response);

/*
 * Tree-shape selection (Appendix E; objective of Theorem 1, Section 3.3).  Host pointers, no GPU.
 * A seed tree (parents as everywhere: parents[0] = -1, 0 <= parents[i] < i) carries per node an
 * acceptance frequency alpha[i] (alpha[0] = 1 for the root; a child's is at most its parent's) and
 * an effective drafting time t_draft[i] (Lemma 2; t_draft[0] is ignored).  T_n is the seed tree after
 * n removals, each of the leaf with the lowest alpha (equal alphas: the highest node id), so
 * every T_n is a prefix subtree of the seed tree.  Its modelled throughput is
 *     ( sum of alpha_i over its nodes ) / ( sum of t_draft_i over its non-root nodes + tv[|T_n| - 1] ),
 * tv[k - 1] = measured verification time of a tree of k nodes (same unit as t_draft), k = 1..T.
 *
 * reader_tree_prune_order writes the removal order (T - 1 node ids) and returns T - 1.
 * reader_tree_select returns the pruning level n* with the best throughput and marks the nodes of
 * T_n* in keep[T] (1 = stays).  exhaustive != 0 scores every n; otherwise a golden-section search
 * is run, which assumes that the curve rises and then falls (Appendix E: close to unimodal) and
 * scores O(log T) trees: the way to go when a score is a benchmark run.  *throughput and
 * *evaluations (both optional) receive the best score and the number of trees scored.
 * Both return -1 on a bad argument (malformed tree, null pointer, negative or undefined value,
 * tv not positive) or when memory runs out.
 */
int32_t reader_tree_prune_order(const int32_t *parents, const float *alpha, int32_t T, int32_t *order);
int32_t reader_tree_select(const int32_t *parents, const float *alpha, const float *t_draft, const float *tv,
                           int32_t T, int32_t exhaustive, int32_t *keep, double *throughput, int32_t *evaluations);

/*
 * Measurement hooks for benchmarks (not operations of the method).  While enabled,
 * every reader_tree_attn / reader_verify_step call launches its main streaming kernel
 * with a HIP event pair that takes the kernel's own start and end time stamps (the
 * second launch of the call is outside the pair).
 * reader_profile_collect waits for the recorded events (it synchronises the host with
 * them), adds up the elapsed times of all pairs recorded since the last collect into
 * *kernel_ms_sum, stores their count in *launches, and forgets them.  The event
 * objects are host-side handles owned by the library; at most 65536 pairs are kept
 * between collects (further launches are simply not timed).  Not thread-safe.
 * reader_profile_collect_each does the same but hands out every pair's time: ms_each
 * (host, float [capacity]) receives the first min(count, capacity) times in launch
 * order, *launches the count; READER_EINVAL for a null pointer or capacity < 0.
 */
int reader_profile_enable(int32_t on);
int reader_profile_collect(double *kernel_ms_sum, int32_t *launches);
int reader_profile_collect_each(float *ms_each, int32_t capacity, int32_t *launches);

/*
 * What this GPU gives the two things the attention kernels are made of, for the roofline discussion
 * (not an operation of the method).  Runs two bare loops on `stream` and waits for them:
 *   - every compute unit copies 32 KB tiles of `src` into a ring of LDS buffers with the instruction
 *     and the ring depth of the attention kernel and does nothing else: *hbm_read_gbs (src should be
 *     larger than the last-level cache, 256 MB, for the figure to be an HBM figure; the first
 *     src_bytes rounded down to a multiple of 8 MB are read);
 *   - one wavefront per SIMD issues the matrix instruction (v_mfma_f32_32x32x16_bf16) back to back on
 *     register operands: *mfma_bf16_tflops, and the shader clock the part runs at under that load in
 *     *mfma_clock_mhz (it lowers its clock under matrix load).
 *   src      device, src_bytes >= 32 MB, read only;  scratch  device, >= 262160 bytes, overwritten
 *   the three results are HOST doubles.
 * Creates and destroys two events; synchronises the host with the stream.  READER_OK, READER_EINVAL
 * (null pointer, sizes too small), READER_EHIP.
 */
int reader_measure_peaks(const void *src, size_t src_bytes, void *scratch, size_t scratch_bytes,
                         double *hbm_read_gbs, double *mfma_bf16_tflops, double *mfma_clock_mhz, void *stream);

/*
 * Launch-planner overrides for tests and experiments (not operations of the method; a caller
 * never needs them).  The planner of reader_tree_attn / reader_verify_step picks the number of
 * query rows per workgroup, the number of key ranges, the cost it books for the start of a
 * (sequence, kv head) pair when it cuts the ranges, and 32- or 64-bit arithmetic for the cut,
 * all from the dims alone.  An override replaces one of these choices for every later call of
 * the process (reader_workspace_bytes included, so sizes stay consistent) until it is cleared
 * with a negative value.  Every choice gives the same results up to rounding; only the speed
 * and the code path differ.  Stored atomically: a call sees the old or the new value.
 *   READER_TUNE_ATTN_ROWS       128 or 256 query rows per workgroup (other values: planner decides)
 *   READER_TUNE_ATTN_RANGES     >= 1 key ranges asked for (capped at the number of compute units)
 *   READER_TUNE_ATTN_PAIR_COST  0..64 tile times booked per pair beyond its tiles
 *   READER_TUNE_ATTN_PAIR_FRONT how many of them are booked to the workgroup that starts the pair (the rest to
 *                               the one that finishes it); capped at the pair cost
 *   READER_TUNE_ATTN_AXIS64     1 = cut the ranges in 64-bit arithmetic even where 32 bits suffice
 *   READER_TUNE_ATTN_WIDE       which kernel 256-row workgroups run: 1 = four wavefronts with 64 rows each (one per
 *                               SIMD, the accumulation registers managed by hand), 0 = eight with 32 rows each;
 *                               the planner takes the first at head dimension 128 and the second at 64
 * Returns READER_OK, or READER_EINVAL for an unknown `which`.
 */
enum {
    READER_TUNE_ATTN_ROWS = 0,
    READER_TUNE_ATTN_RANGES = 1,
    READER_TUNE_ATTN_PAIR_COST = 2,
    READER_TUNE_ATTN_AXIS64 = 3,
    READER_TUNE_ATTN_WIDE = 4,
    READER_TUNE_ATTN_PAIR_FRONT = 5,
    READER_TUNE_COUNT_ = 6
};
int reader_tuning_override(int32_t which, int32_t value);

#ifdef __cplusplus
}
#endif
#endif /* READER_H */

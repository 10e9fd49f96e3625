// C ABI entry points: argument validation on the host, launch planning, dispatch.
// The operations themselves are defined in include/reader.h with their citations.
#include <math.h>
#include <stdio.h>
#include <stdlib.h>

#include <atomic>
#include <mutex>
#include <utility>
#include <vector>

#include "internal.h"

namespace reader {

static char g_error_detail[256] = "";

// Planner overrides set through reader_tuning_override (tests, experiments); -1 = the planner decides.
static std::atomic<int32_t> g_tuning[READER_TUNE_COUNT_] = {{-1}, {-1}, {-1}, {-1}, {-1}, {-1}};
#ifdef READER_WG_STAMPS
static std::atomic<long long *> g_wg_stamps{nullptr};
#endif
static int tuning(int which) { return g_tuning[which].load(std::memory_order_relaxed); }

// The runtime keeps the last error of the calling thread until somebody reads it, whoever caused
// it: an error another library left behind must not be taken for a failed launch of ours.
static void forget_stale_error() { (void)hipGetLastError(); }

hipError_t note_hip_error(const char *where, hipError_t e) {
    if (e != hipSuccess) snprintf(g_error_detail, sizeof g_error_detail, "%s: %s", where, hipGetErrorName(e));
    return e;
}

static bool dims_ok(const reader_dims *d, int *err) {
    if (!d) { *err = READER_EINVAL; return false; }
    if (d->B < 0 || d->T < 1 || d->Hq < 1 || d->Hkv < 1 || d->D < 1 || d->max_pages_per_seq < 0 ||
        d->max_path < 1 || d->num_pages < 0 || d->Hq % d->Hkv != 0 || d->max_path > d->T) {
        *err = READER_EINVAL;
        return false;
    }
    if (d->T > READER_MAX_T || (d->D != 64 && d->D != 128) || d->page_size != READER_PAGE_SIZE ||
        d->Hq / d->Hkv > 16 || d->B > kMaxBatchScan || d->num_pages * d->Hkv > 0x7fffffffLL ||
        (long long)d->B * d->max_pages_per_seq > 0x7fffffffLL) {
        *err = READER_EUNSUPPORTED;
        return false;
    }
    return true;
}

// Query rows a workgroup carries: 128 (four computing wavefronts, four that move data) or 256
// (all eight compute and copy).  Up to 128 rows per (sequence, kv head) there is nothing to
// choose.  Beyond that 256-row workgroups do more matrix work per byte they fetch and win once
// a workgroup has some tens of tiles to stream; a small problem (one or two prompts of a few
// thousand tokens) is over sooner when it is cut into more, lighter workgroups (measured
// crossover with 256 and with 512 rows per kv head: about 10000 workgroup-tiles, i.e. 40 per
// workgroup; at a fifth of that the 128-row workgroups are a quarter faster).
int attn_rows_per_wg(const reader_dims &d, int32_t max_seq_len) {
    const int forced = tuning(READER_TUNE_ATTN_ROWS);
    if (forced == 128 || forced == 256) return forced;
    const int M = d.T * (d.Hq / d.Hkv);
    if (M <= 128) return 128;
    const long long tiles_per_pair = (max_seq_len + kTile - 1) / kTile + (d.T + kTile - 1) / kTile;
    const long long units = (long long)d.B * d.Hkv * tiles_per_pair;
    return units * ((M + 127) / 128) <= 10000 ? 128 : 256;
}

int attn_plan_ranges(const reader_dims &d, int32_t max_seq_len) {
    // One range workgroup streams a contiguous run of 64-key tiles of the flattened
    // (sequence, kv head, tile) axis.  One workgroup (8 waves, ~150 KB of LDS) occupies a
    // compute unit, so at most 256 ranges; short problems get fewer so that a range holds
    // at least two tiles (what a workgroup spends before its first tile arrives is worth
    // several tiles, so tiny problems want many short ranges; measured), and when the rows
    // are cut into chunks, so few that all workgroups run at once: a second round of
    // workgroups pays the start of a workgroup again and cuts twice as many pairs (measured:
    // 128 ranges x 2 chunks against 256 x 2 is 4-5 % faster on long contexts, the same on large batches).
    const int forced = tuning(READER_TUNE_ATTN_RANGES);
    long long tiles_per_pair = (max_seq_len + kTile - 1) / kTile + (d.T + kTile - 1) / kTile;
    long long units = (long long)d.B * d.Hkv * tiles_per_pair;
    long long n = forced > 0 ? forced : units / 2;
    if (n > kNumCU) n = kNumCU;
    const int M = d.T * (d.Hq / d.Hkv);
    if (forced <= 0) {
        const int rows = attn_rows_per_wg(d, max_seq_len), chunks = (M + rows - 1) / rows;
        if (chunks > 1 && n > kNumCU / chunks) n = kNumCU / chunks;
    }
    if (n > units) n = units;
    if (n < 1) n = 1;
    if (n >= kNumXCD) n -= n % kNumXCD;  // row chunks of one key range then share an XCD's L2
    return (int)n;
}

// Measurement hook state: event pairs recorded around the main attention kernel.
struct ProfileState {
    bool on = false;
    size_t used = 0;
    std::vector<std::pair<hipEvent_t, hipEvent_t>> pairs;
};
static ProfileState g_profile;
constexpr size_t kMaxProfilePairs = 65536;

static bool profile_next(hipEvent_t *a, hipEvent_t *b) {
    *a = nullptr; *b = nullptr;
    if (!g_profile.on || g_profile.used >= kMaxProfilePairs) return false;
    if (g_profile.used == g_profile.pairs.size()) {
        hipEvent_t s, t;
        if (hipEventCreate(&s) != hipSuccess) return false;
        if (hipEventCreate(&t) != hipSuccess) { (void)hipEventDestroy(s); return false; }
        g_profile.pairs.emplace_back(s, t);
    }
    *a = g_profile.pairs[g_profile.used].first;
    *b = g_profile.pairs[g_profile.used].second;
    ++g_profile.used;
    return true;
}

// Workspace of reader_tree_attn_noalloc: device memory that belongs to the library's code object,
// so that the call allocates nothing.  Every GPU the library runs on holds its own copy of the
// array, at its own address, until the process ends.  In host code the array's name is only a
// handle for hipGetSymbolAddress; `scratch_on_current_device` turns it into the device address
// once per device, and everything else (kernel arguments) uses that address.
static __device__ __align__(256) unsigned char scratch[READER_NOALLOC_WORKSPACE_BYTES];
constexpr int kMaxDevices = 64;
static void *g_scratch_ptr[kMaxDevices];   // guarded by g_scratch_guard
static std::mutex g_scratch_guard;

static int scratch_on_current_device(void **ptr) {
    int dev = -1;
    if (note_hip_error("hipGetDevice", hipGetDevice(&dev)) != hipSuccess) return READER_EHIP;
    if (dev < 0 || dev >= kMaxDevices) return READER_EUNSUPPORTED;
    std::lock_guard<std::mutex> lock(g_scratch_guard);
    if (!g_scratch_ptr[dev]) {
        void *addr = nullptr;
        const hipError_t e = hipGetSymbolAddress(&addr, HIP_SYMBOL(scratch));
        if (e != hipSuccess || !addr) {
            (void)hipGetLastError();
            (void)note_hip_error("hipGetSymbolAddress(scratch)", e != hipSuccess ? e : hipErrorInvalidSymbol);
            return READER_EHIP;
        }
        g_scratch_ptr[dev] = addr;
    }
    *ptr = g_scratch_ptr[dev];
    return READER_OK;
}

static int row_chunks(const reader_dims &d, int32_t max_seq_len) {
    int M = d.T * (d.Hq / d.Hkv);
    int rows = attn_rows_per_wg(d, max_seq_len);
    return (M + rows - 1) / rows;
}

}  // namespace reader

using namespace reader;

extern "C" const char *reader_version(void) { return "reader-hip 0.1 (gfx950)"; }

extern "C" const char *reader_strerror(int code) {
    switch (code) {
        case READER_OK: return "ok";
        case READER_EINVAL: return "invalid argument";
        case READER_EUNSUPPORTED: return "size not supported by the kernels";
        case READER_EWORKSPACE: return "workspace missing or too small";
        case READER_EHIP: return "HIP launch failed";
        default: return "unknown error";
    }
}

extern "C" const char *reader_last_error_detail(void) { return g_error_detail; }

#ifdef READER_WG_STAMPS
// Profiling build only (not declared in the public header): device buffer of kWgStamps 64-bit stamps per
// workgroup of the attention main kernel, at least 2048 workgroups; null switches the stamps off.
extern "C" int reader_profile_wg_stamps(void *device_buffer) {
    g_wg_stamps.store(static_cast<long long *>(device_buffer), std::memory_order_relaxed);
    return READER_OK;
}
#endif

extern "C" int reader_tuning_override(int32_t which, int32_t value) {
    if (which < 0 || which >= READER_TUNE_COUNT_) return READER_EINVAL;
    g_tuning[which].store(value < 0 ? -1 : value, std::memory_order_relaxed);
    return READER_OK;
}

extern "C" int reader_validate_tree(const int32_t *parents_host, int32_t B, int32_t T) {
    if (!parents_host || B < 0 || T < 1) return READER_EINVAL;
    for (int32_t b = 0; b < B; ++b) {
        const int32_t *p = parents_host + (size_t)b * T;
        if (p[0] != -1) return READER_EINVAL;
        for (int32_t i = 1; i < T; ++i)
            if (p[i] < 0 || p[i] >= i) return READER_EINVAL;
    }
    return READER_OK;
}

extern "C" size_t reader_workspace_bytes(const reader_dims *dims, int32_t max_seq_len) {
    int err = 0;
    if (!dims_ok(dims, &err) || max_seq_len < 0) return 0;
    if (dims->B == 0) return 256;
    size_t slots = 2 * (size_t)attn_plan_ranges(*dims, max_seq_len) * (size_t)row_chunks(*dims, max_seq_len);
    size_t bytes = slots * attn_slot_floats(dims->D, attn_rows_per_wg(*dims, max_seq_len)) * sizeof(float);
    return attn_header_bytes(dims->B, dims->Hkv) + ((bytes + 255) & ~(size_t)255);
}

static int attn_use_wide(const reader_dims &d, int rows_per_wg) {
    // 256-row workgroups: four wavefronts of 64 rows at head dimension 128 (measured 2 to 4 % faster than eight of
    // 32 rows at the two matrix-bound presets), eight of 32 at head dimension 64 (measured: no difference)
    const int wide = tuning(READER_TUNE_ATTN_WIDE);
    return rows_per_wg == 256 && (wide == 1 || (wide < 0 && d.D == 128)) ? 1 : 0;
}

extern "C" int reader_attn_plan(const reader_dims *dims, int32_t max_seq_len, reader_attn_plan_t *plan) {
    int err = 0;
    if (!plan) return READER_EINVAL;
    if (!dims_ok(dims, &err)) return err;
    if (max_seq_len < 0) return READER_EINVAL;
    const bool scalar = dims->variant == 1;
    plan->rows_per_workgroup = scalar ? 0 : attn_rows_per_wg(*dims, max_seq_len);
    plan->row_chunks = scalar ? 0 : row_chunks(*dims, max_seq_len);
    plan->key_ranges = scalar ? 0 : attn_plan_ranges(*dims, max_seq_len);
    plan->kernel = scalar ? READER_ATTN_KERNEL_SCALAR
                          : plan->rows_per_workgroup == 128 ? READER_ATTN_KERNEL_ROWS128
                          : attn_use_wide(*dims, plan->rows_per_workgroup) ? READER_ATTN_KERNEL_ROWS256_WAVES4
                                                                           : READER_ATTN_KERNEL_ROWS256_WAVES8;
    return READER_OK;
}

// Argument checks and kernel parameters of the attention step (shared by reader_tree_attn and
// reader_verify_step).  Returns READER_OK and fills `p`, or an error code; *empty is set when
// there is nothing to do.
static int attn_prepare(const reader_dims *dims, const void *q, const void *k_tree, const void *v_tree,
                        const void *k_cache, const void *v_cache, const int32_t *page_table,
                        const int32_t *seq_lens, const int32_t *parents, void *out, float *lse,
                        int32_t max_seq_len, void *workspace, int32_t *status, AttnParams &p, bool *empty) {
    int err = 0;
    *empty = false;
    if (!dims_ok(dims, &err)) return err;
    if (max_seq_len < 0) return READER_EINVAL;
    if (dims->B == 0) { *empty = true; return READER_OK; }
    if (!q || !k_cache || !v_cache || !page_table || !seq_lens || !parents || !out) return READER_EINVAL;
    if ((k_tree == nullptr) != (v_tree == nullptr)) return READER_EINVAL;
    const bool tree_in_cache = k_tree == nullptr;     // the tree rows sit behind each sequence in the cache
    if ((long long)dims->max_pages_per_seq * dims->page_size < (long long)max_seq_len + (tree_in_cache ? dims->T : 0))
        return READER_EINVAL;
    if ((max_seq_len > 0 || tree_in_cache) && (dims->num_pages < 1 || dims->max_pages_per_seq < 1)) return READER_EINVAL;
    if (dims->variant != 0 && dims->variant != 1) return READER_EINVAL;

    p.q = (const uint16_t *)q; p.k_tree = (const uint16_t *)k_tree; p.v_tree = (const uint16_t *)v_tree;
    p.k_cache = (const uint16_t *)k_cache; p.v_cache = (const uint16_t *)v_cache;
    p.page_table = page_table; p.seq_lens = seq_lens; p.parents = parents;
    p.out = (uint16_t *)out; p.lse = lse; p.status = status;
    p.range_tiles = (int32_t *)workspace;
    p.redo = workspace ? (int32_t *)((char *)workspace + kNumCU * 4) : nullptr;
    p.pair_info = workspace ? (int32_t *)((char *)workspace + kNumCU * 4 + kMaxAttnWorkgroups * 4) : nullptr;
    p.workspace = workspace ? (float *)((char *)workspace + attn_header_bytes(dims->B, dims->Hkv)) : nullptr;
    p.B = dims->B; p.T = dims->T; p.Hq = dims->Hq; p.Hkv = dims->Hkv; p.D = dims->D;
    p.G = dims->Hq / dims->Hkv; p.M = p.T * p.G;
    p.max_pages = dims->max_pages_per_seq; p.max_seq_len = max_seq_len;
    p.n_tree_tiles = (dims->T + kTile - 1) / kTile;
    p.rows_per_wg = attn_rows_per_wg(*dims, max_seq_len);
    p.n_row_chunks = row_chunks(*dims, max_seq_len);
    p.n_ranges = attn_plan_ranges(*dims, max_seq_len);
    {
        // A pair costs the workgroups that start and finish it extra, mostly the one that finishes it (the ragged
        // last prefix tile, the masks of the tree tiles, normalising and writing the rows; the start has the
        // query rows to fetch): with dedicated copy wavefronts about one tile time in front of the pair's
        // tiles and two behind them; with four wavefronts of 64 rows, whose tiles at the ends of a pair leave the
        // software pipeline and whose accumulators are read out of the other half of the register file, four and
        // four (measured at the large-batch preset: kernel 703 -> 685 us against one in front; 16 and more lose
        // again); otherwise one in front.
        const bool wide = attn_use_wide(*dims, p.rows_per_wg);
        const int forced_cost = tuning(READER_TUNE_ATTN_PAIR_COST);
        p.pair_cost = forced_cost >= 0 && forced_cost <= 64 ? forced_cost : (p.rows_per_wg == 128 ? 3 : (wide ? 8 : 1));
        const int forced_front = tuning(READER_TUNE_ATTN_PAIR_FRONT);
        p.pair_front = forced_front >= 0 ? forced_front : (wide ? 4 : 1);
        if (p.pair_front > p.pair_cost) p.pair_front = p.pair_cost;
        // the kernel cuts the ranges with 32-bit arithmetic when nothing on the cost axis can overflow it
        const long long axis_max = (long long)p.Hkv * p.B * ((max_seq_len + kTile - 1) / kTile + p.n_tree_tiles + p.pair_cost);
        p.axis32 = (axis_max + 2) * (p.n_ranges + 1) < 0x7fffffffLL ? 1 : 0;
        if (tuning(READER_TUNE_ATTN_AXIS64) == 1) p.axis32 = 0;   // tests: force the 64-bit path
        p.ranges_shift = -1;
        for (int sh = 0; sh < 16; ++sh)
            if (p.n_ranges == (1 << sh)) p.ranges_shift = sh;
    }
    p.num_pages = dims->num_pages;
    // few pairs, many ranges: a pair is cut into eight parts or more on average, the merge fetches them four abreast
    p.merge_groups = (long long)dims->B * dims->Hkv * 8 <= p.n_ranges ? 4 : 1;
    p.tree_in_cache = tree_in_cache ? 1 : 0;
    p.wide = attn_use_wide(*dims, p.rows_per_wg);
    p.redo_only = 0;
#ifdef READER_WG_STAMPS
    p.stamps = g_wg_stamps.load(std::memory_order_relaxed);
#endif
    float scale = dims->sm_scale > 0.f ? dims->sm_scale : 1.0f / sqrtf((float)dims->D);
    p.scale_log2 = scale * 1.44269504088896340736f;
    return READER_OK;
}

static void accept_fill(const reader_dims *dims, const int32_t *draft_tokens, const int32_t *target_tokens,
                        const int32_t *parents, int32_t *accept_len, int32_t *path, int32_t *bonus_token,
                        int32_t *status, AcceptParams &p) {
    p.draft = draft_tokens; p.target = target_tokens; p.parents = parents;
    p.accept_len = accept_len; p.path = path; p.bonus = bonus_token; p.status = status;
    p.B = dims->B; p.T = dims->T; p.max_path = dims->max_path;
}

static void compact_fill(const reader_dims *dims, const void *k_tree, const void *v_tree, const int32_t *path,
                         const int32_t *accept_len, void *k_cache, void *v_cache, const int32_t *page_table,
                         int32_t *seq_lens, int32_t *status, CompactParams &p) {
    p.k_tree = (const uint16_t *)k_tree; p.v_tree = (const uint16_t *)v_tree;
    p.path = path; p.accept_len = accept_len; p.page_table = page_table;
    p.k_cache = (uint16_t *)k_cache; p.v_cache = (uint16_t *)v_cache;
    p.seq_lens = seq_lens; p.status = status;
    p.B = dims->B; p.T = dims->T; p.Hkv = dims->Hkv; p.D = dims->D;
    p.max_pages = dims->max_pages_per_seq; p.max_path = dims->max_path; p.num_pages = dims->num_pages;
}

static void compact_layers_fill(const reader_dims *dims, int32_t num_layers, const int32_t *path,
                                const int32_t *accept_len, void *k_cache, void *v_cache, const int32_t *page_table,
                                int32_t *seq_lens, int32_t *status, CompactLayersParams &p) {
    p.k_cache = (uint16_t *)k_cache; p.v_cache = (uint16_t *)v_cache;
    p.path = path; p.accept_len = accept_len; p.page_table = page_table;
    p.seq_lens = seq_lens; p.status = status;
    p.B = dims->B; p.T = dims->T; p.Hkv = dims->Hkv; p.D = dims->D;
    p.max_pages = dims->max_pages_per_seq; p.max_path = dims->max_path; p.NL = num_layers;
    p.num_pages = dims->num_pages;
}

extern "C" int reader_tree_attn(const reader_dims *dims, const void *q, const void *k_tree,
                                const void *v_tree, const void *k_cache, const void *v_cache,
                                const int32_t *page_table, const int32_t *seq_lens,
                                const int32_t *parents, void *out, float *lse, int32_t max_seq_len,
                                void *workspace, size_t workspace_bytes, int32_t *status,
                                void *stream) {
    AttnParams p;
    bool empty = false;
    const int rc = attn_prepare(dims, q, k_tree, v_tree, k_cache, v_cache, page_table, seq_lens, parents, out, lse,
                                max_seq_len, workspace, status, p, &empty);
    if (rc != READER_OK || empty) return rc;
    hipError_t e;
    if (dims->variant == 1) {
        forget_stale_error();
        e = launch_tree_attn_scalar(p, (hipStream_t)stream);
    } else {
        if (!workspace || ((uintptr_t)workspace & 255) != 0) return READER_EWORKSPACE;
        if (workspace_bytes < reader_workspace_bytes(dims, max_seq_len)) return READER_EWORKSPACE;
        hipEvent_t ev_a, ev_b;
        profile_next(&ev_a, &ev_b);
        forget_stale_error();
        e = launch_tree_attn_mfma(p, (hipStream_t)stream, ev_a, ev_b);
    }
    return e == hipSuccess ? READER_OK : READER_EHIP;
}

extern "C" int reader_tree_attn_noalloc(const reader_dims *dims, const void *q, const void *k_tree,
                                        const void *v_tree, const void *k_cache, const void *v_cache,
                                        const int32_t *page_table, const int32_t *seq_lens,
                                        const int32_t *parents, void *out, float *lse, int32_t max_seq_len,
                                        int32_t *status, void *stream) {
    int err = 0;
    if (!dims_ok(dims, &err)) return err;
    if (max_seq_len < 0 || dims->variant != 0) return READER_EINVAL;
    // the size check comes first: a problem that does not fit is refused whatever the device's state
    const size_t need = reader_workspace_bytes(dims, max_seq_len);
    if (need > (size_t)READER_NOALLOC_WORKSPACE_BYTES) {
        snprintf(g_error_detail, sizeof g_error_detail,
                 "reader_tree_attn_noalloc: these dims need %zu bytes of workspace, the built-in one holds %zu", need,
                 (size_t)READER_NOALLOC_WORKSPACE_BYTES);
        return READER_EWORKSPACE;
    }
    void *ws = nullptr;
    const int rc_ws = scratch_on_current_device(&ws);   // first call on a device: looks the address up (B = 0 does only this)
    if (rc_ws != READER_OK) return rc_ws;
    AttnParams p;
    bool empty = false;
    const int rc = attn_prepare(dims, q, k_tree, v_tree, k_cache, v_cache, page_table, seq_lens, parents, out, lse,
                                max_seq_len, ws, status, p, &empty);
    if (rc != READER_OK || empty) return rc;
    // Nothing in the workspace has to start at zero: every range workgroup writes its tile count and the
    // pair table afresh before the merge reads them, and a record slot is only read when this call's
    // tile count of its range says that this call wrote it.
    forget_stale_error();
    return launch_tree_attn_mfma(p, (hipStream_t)stream, nullptr, nullptr) == hipSuccess ? READER_OK : READER_EHIP;
}

extern "C" int reader_verify_step(const reader_dims *dims, const void *q, const void *k_tree, const void *v_tree,
                                  void *k_cache, void *v_cache, const int32_t *page_table, int32_t *seq_lens,
                                  const int32_t *parents, const int32_t *draft_tokens,
                                  const int32_t *target_tokens, void *out, float *lse, int32_t *accept_len,
                                  int32_t *path, int32_t *bonus_token, int32_t max_seq_len, void *workspace,
                                  size_t workspace_bytes, int32_t *status, void *stream) {
    AttnParams p;
    bool empty = false;
    const int rc = attn_prepare(dims, q, k_tree, v_tree, k_cache, v_cache, page_table, seq_lens, parents, out, lse,
                                max_seq_len, workspace, status, p, &empty);
    if (rc != READER_OK || empty) return rc;
    if (!draft_tokens || !target_tokens || !accept_len || !path || !bonus_token) return READER_EINVAL;
    if (dims->variant != 0) return READER_EINVAL;   // the fused step exists for the matrix-core kernel only
    if (!workspace || ((uintptr_t)workspace & 255) != 0) return READER_EWORKSPACE;
    if (workspace_bytes < reader_workspace_bytes(dims, max_seq_len)) return READER_EWORKSPACE;
    AcceptParams ap;
    CompactParams cp;
    accept_fill(dims, draft_tokens, target_tokens, parents, accept_len, path, bonus_token, status, ap);
    compact_fill(dims, k_tree, v_tree, path, accept_len, k_cache, v_cache, page_table, seq_lens, status, cp);
    hipEvent_t ev_a, ev_b;
    profile_next(&ev_a, &ev_b);
    forget_stale_error();
    if (launch_tree_attn_mfma(p, (hipStream_t)stream, ev_a, ev_b, &ap, &cp) != hipSuccess) return READER_EHIP;
    if (p.tree_in_cache) {
        // the tree rows are in the cache already: the accepted ones move in place (this layer's cache)
        CompactLayersParams lp;
        compact_layers_fill(dims, 1, path, accept_len, k_cache, v_cache, page_table, seq_lens, status, lp);
        if (launch_kv_compact_layers(lp, (hipStream_t)stream) != hipSuccess) return READER_EHIP;
    }
    return READER_OK;
}

extern "C" int reader_profile_enable(int32_t on) {
    g_profile.on = on != 0;
    return READER_OK;
}

extern "C" int reader_profile_collect(double *kernel_ms_sum, int32_t *launches) {
    if (!kernel_ms_sum || !launches) return READER_EINVAL;
    double sum = 0.0;
    int32_t n = 0;
    int rc = READER_OK;
    for (size_t i = 0; i < g_profile.used; ++i) {
        float ms = 0.f;
        if (hipEventSynchronize(g_profile.pairs[i].second) != hipSuccess ||
            hipEventElapsedTime(&ms, g_profile.pairs[i].first, g_profile.pairs[i].second) != hipSuccess) {
            rc = READER_EHIP;
            continue;
        }
        sum += ms;
        ++n;
    }
    g_profile.used = 0;
    *kernel_ms_sum = sum;
    *launches = n;
    return rc;
}

extern "C" int reader_profile_collect_each(float *ms_each, int32_t capacity, int32_t *launches) {
    if (!ms_each || !launches || capacity < 0) return READER_EINVAL;
    int32_t n = 0;
    int rc = READER_OK;
    for (size_t i = 0; i < g_profile.used; ++i) {
        float ms = 0.f;
        if (hipEventSynchronize(g_profile.pairs[i].second) != hipSuccess ||
            hipEventElapsedTime(&ms, g_profile.pairs[i].first, g_profile.pairs[i].second) != hipSuccess) {
            rc = READER_EHIP;
            continue;
        }
        if (n < capacity) ms_each[n] = ms;
        ++n;
    }
    g_profile.used = 0;
    *launches = n;
    return rc;
}

extern "C" int reader_measure_peaks(const void *src, size_t src_bytes, void *scratch, size_t scratch_bytes,
                                    double *hbm_read_gbs, double *mfma_bf16_tflops, double *mfma_clock_mhz, void *stream) {
    if (!src || !scratch || !hbm_read_gbs || !mfma_bf16_tflops || !mfma_clock_mhz) return READER_EINVAL;
    if (src_bytes < (size_t)kNumCU * 32768 * 4 || scratch_bytes < kProbeScratchBytes) return READER_EINVAL;
    forget_stale_error();
    hipStream_t st = static_cast<hipStream_t>(stream);
    hipEvent_t a = nullptr, b = nullptr;
    if (hipEventCreate(&a) != hipSuccess || hipEventCreate(&b) != hipSuccess) {
        if (a) (void)hipEventDestroy(a);
        (void)hipGetLastError();
        return READER_EHIP;
    }
    int rc = READER_OK;
    auto timed = [&](auto &&launch, float *ms) {
        // one untimed run, then one between two events
        for (int rep = 0; rep < 2 && rc == READER_OK; ++rep) {
            if (rep == 1 && hipEventRecord(a, st) != hipSuccess) rc = READER_EHIP;
            if (rc == READER_OK && launch() != hipSuccess) rc = READER_EHIP;
            if (rep == 1 && rc == READER_OK && hipEventRecord(b, st) != hipSuccess) rc = READER_EHIP;
        }
        if (rc == READER_OK && (hipEventSynchronize(b) != hipSuccess || hipEventElapsedTime(ms, a, b) != hipSuccess)) rc = READER_EHIP;
    };
    float copy_ms = 0.f, mfma_ms = 0.f;
    size_t moved = 0;
    timed([&]() { return launch_probe_copy(src, src_bytes, scratch, st, &moved); }, &copy_ms);
    constexpr int kIters = 2000;   // x 64 matrix instructions per wavefront: about 2 ms
    timed([&]() { return launch_probe_mfma(kIters, scratch, st); }, &mfma_ms);
    long long clocks[2] = {0, 0};
    if (rc == READER_OK &&
        hipMemcpyAsync(clocks, static_cast<const char *>(scratch) + (size_t)kNumCU * 256 * sizeof(float), sizeof clocks,
                       hipMemcpyDeviceToHost, st) != hipSuccess)
        rc = READER_EHIP;
    if (rc == READER_OK && hipStreamSynchronize(st) != hipSuccess) rc = READER_EHIP;
    (void)hipEventDestroy(a);
    (void)hipEventDestroy(b);
    if (rc != READER_OK) { (void)hipGetLastError(); return rc; }
    *hbm_read_gbs = copy_ms > 0.f ? (double)moved / (copy_ms * 1e-3) / 1e9 : 0.0;
    const double flops = (double)kNumCU * 4.0 * kIters * 64.0 * 32768.0;
    *mfma_bf16_tflops = mfma_ms > 0.f ? flops / (mfma_ms * 1e-3) / 1e12 : 0.0;
    *mfma_clock_mhz = clocks[1] > 0 ? (double)clocks[0] / ((double)clocks[1] / 100.0) : 0.0;
    return READER_OK;
}

extern "C" int reader_accept_path(const reader_dims *dims, const int32_t *draft_tokens,
                                  const int32_t *target_tokens, const int32_t *parents,
                                  int32_t *accept_len, int32_t *path, int32_t *bonus_token,
                                  int32_t *status, void *stream) {
    int err = 0;
    if (!dims_ok(dims, &err)) return err;
    if (dims->B == 0) return READER_OK;
    if (!draft_tokens || !target_tokens || !parents || !accept_len || !path || !bonus_token)
        return READER_EINVAL;
    AcceptParams p;
    accept_fill(dims, draft_tokens, target_tokens, parents, accept_len, path, bonus_token, status, p);
    forget_stale_error();
    return launch_accept_path(p, (hipStream_t)stream) == hipSuccess ? READER_OK : READER_EHIP;
}

extern "C" int reader_kv_compact(const reader_dims *dims, const void *k_tree, const void *v_tree,
                                 const int32_t *path, const int32_t *accept_len, void *k_cache,
                                 void *v_cache, const int32_t *page_table, int32_t *seq_lens,
                                 int32_t *status, void *stream) {
    int err = 0;
    if (!dims_ok(dims, &err)) return err;
    if (dims->B == 0) return READER_OK;
    if (!k_tree || !v_tree || !path || !accept_len || !k_cache || !v_cache || !page_table || !seq_lens)
        return READER_EINVAL;
    CompactParams p;
    compact_fill(dims, k_tree, v_tree, path, accept_len, k_cache, v_cache, page_table, seq_lens, status, p);
    forget_stale_error();
    return launch_kv_compact(p, (hipStream_t)stream) == hipSuccess ? READER_OK : READER_EHIP;
}

extern "C" int reader_kv_compact_layers(const reader_dims *dims, int32_t num_layers, const int32_t *path,
                                        const int32_t *accept_len, void *k_cache, void *v_cache,
                                        const int32_t *page_table, int32_t *seq_lens, int32_t *status,
                                        void *stream) {
    int err = 0;
    if (!dims_ok(dims, &err)) return err;
    if (num_layers < 0 || num_layers > 65535) return READER_EINVAL;
    if (dims->B == 0) return READER_OK;
    if (!path || !accept_len || !page_table || !seq_lens || (num_layers > 0 && (!k_cache || !v_cache)))
        return READER_EINVAL;
    CompactLayersParams p;
    compact_layers_fill(dims, num_layers, path, accept_len, k_cache, v_cache, page_table, seq_lens, status, p);
    forget_stale_error();
    return launch_kv_compact_layers(p, (hipStream_t)stream) == hipSuccess ? READER_OK : READER_EHIP;
}

extern "C" size_t reader_kv_rearrange_scratch_bytes(int32_t B, int32_t S) {
    if (B < 0 || S < 0) return 0;
    return (((size_t)B * (size_t)S + (size_t)B * 4) * sizeof(int32_t) + 255) & ~(size_t)255;
}

extern "C" int reader_kv_rearrange(int32_t NL, int32_t B, int32_t S, int32_t Hkv, int32_t D, void *k_pad,
                                   void *v_pad, uint8_t *valid, int32_t *new_len, void *scratch,
                                   size_t scratch_bytes, void *stream) {
    if (NL < 0 || B < 0 || S < 0 || Hkv < 1 || D < 1) return READER_EINVAL;
    if (D != 64 && D != 128) return READER_EUNSUPPORTED;
    if ((long long)B * ((long long)Hkv + 1) > 0x7fffffffLL || (long long)B * ((long long)Hkv + 1) * (NL > 0 ? NL : 1) > 0x7fffffffLL)
        return READER_EUNSUPPORTED;
    if (B == 0 || S == 0) return READER_OK;
    if (!valid || !new_len || (NL > 0 && (!k_pad || !v_pad))) return READER_EINVAL;
    if (!scratch || ((uintptr_t)scratch & 3) != 0 || scratch_bytes < reader_kv_rearrange_scratch_bytes(B, S))
        return READER_EWORKSPACE;
    RearrangeParams p;
    p.k_pad = (uint16_t *)k_pad; p.v_pad = (uint16_t *)v_pad; p.valid = valid; p.new_len = new_len;
    p.dest = (int32_t *)scratch;
    p.NL = NL; p.B = B; p.S = S; p.Hkv = Hkv; p.D = D;
    forget_stale_error();
    return launch_kv_rearrange(p, (hipStream_t)stream) == hipSuccess ? READER_OK : READER_EHIP;
}

extern "C" int reader_target_argmax(int32_t rows, int32_t V, const void *logits, int32_t *target_tokens,
                                    void *stream) {
    if (rows < 0 || V < 1) return READER_EINVAL;
    if (rows == 0) return READER_OK;
    if (!logits || !target_tokens) return READER_EINVAL;
    forget_stale_error();
    return launch_target_argmax((const uint16_t *)logits, target_tokens, rows, V, (hipStream_t)stream) == hipSuccess
               ? READER_OK : READER_EHIP;
}

extern "C" int reader_target_sample(int32_t B, int32_t T, int32_t V, const void *logits, const int32_t *parents,
                                    const float *uniforms, float temperature, int32_t *target_tokens, void *stream) {
    if (B < 0 || T < 1 || T > READER_MAX_T || V < 1 || V > READER_MAX_SAMPLE_V) return READER_EINVAL;
    if (!(temperature >= READER_MIN_TEMPERATURE) || !(temperature <= READER_MAX_TEMPERATURE)) return READER_EINVAL;
    if ((long long)B * T > 0x7fffffffLL) return READER_EINVAL;
    if (B == 0) return READER_OK;
    if (!logits || !parents || !uniforms || !target_tokens) return READER_EINVAL;
    forget_stale_error();
    return launch_target_sample((const uint16_t *)logits, parents, uniforms, target_tokens, B, T, V, temperature,
                                (hipStream_t)stream) == hipSuccess
               ? READER_OK : READER_EHIP;
}


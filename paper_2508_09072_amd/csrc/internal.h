// Internal declarations shared by the translation units of libreader_hip.so.
// Nothing here is part of the C ABI (see include/reader.h).
#pragma once

#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include "reader.h"

namespace reader {

// Remember which HIP call failed (text returned by reader_last_error_detail()); returns e.
hipError_t note_hip_error(const char *where, hipError_t e);

// MI355X: 256 compute units in 8 XCDs; the launch planner is written for this part only.
constexpr int kNumCU = 256;
constexpr int kNumXCD = 8;

constexpr int kTile = 64;          // keys per tile of the attention main loop
constexpr int kThreads = 512;      // 8 wavefronts per attention workgroup, one workgroup per compute unit
constexpr int kMaxBatchScan = READER_MAX_B;  // sequences the in-kernel prefix scan is sized for

// Query rows (tree node, grouped head) one attention workgroup carries: 4 row blocks of 32
// with the tile's keys split between two wave groups, or 8 row blocks when T*G > 128.

int attn_rows_per_wg(const reader_dims &d, int32_t max_seq_len);   // host: 128 or 256 query rows per workgroup (reader_api.hip)

// Everything the attention kernels need, passed by value as the kernel argument.
struct AttnParams {
    const uint16_t *q, *k_tree, *v_tree, *k_cache, *v_cache;
    const int32_t *page_table, *seq_lens, *parents;
    uint16_t *out;
    float *lse;
    float *workspace;  // partial records, see attn_slot_floats() (behind the header, see attn_header_bytes())
    int32_t *pair_info;      // header: per (sequence, kv head) the first and the last workgroup that hold its tiles
    int32_t *range_tiles;    // header: per range workgroup the number of tiles it holds (0: it wrote no record)
    int32_t *redo;           // header: per workgroup of the wide kernel 1 if its range has to be computed again (kMaxAttnWorkgroups entries)
#ifdef READER_WG_STAMPS
    long long *stamps;       // profiling build only: kWgStamps time stamps per workgroup (100 MHz counter), or null
#endif
    int32_t pair_cost;       // what a pair costs beyond its tiles, in tile times, when the ranges are cut
    int32_t pair_front;      // the part of it booked in front of the pair's tiles (the rest behind them)
    int32_t axis32;          // 1: every position of the cost axis times n_ranges fits in an int
    int32_t ranges_shift;    // log2(n_ranges) when it is a power of two (the even cut is then a shift), else -1
    int32_t merge_groups;    // thread groups that share a query row's partial records in the merge: 1, or 4 when pairs are cut into many parts
    int32_t tree_in_cache;   // 1: k_tree / v_tree are null, tree node n of sequence b sits at cache position L_b + n
    int32_t wide;            // (256 rows per workgroup) 1: four wavefronts of 64 rows, 0: eight of 32
    int32_t redo_only;       // 1: second pass behind the wide kernel, only the workgroups flagged in `redo` do anything
    int32_t *status;
    int32_t B, T, Hq, Hkv, D, G, M;       // G = Hq/Hkv, M = T*G query rows per (sequence, kv head)
    int32_t max_pages, max_seq_len;
    int32_t n_tree_tiles;                  // ceil(T / kTile)
    int32_t rows_per_wg;                   // attn_rows_per_wg(dims, max_seq_len)
    int32_t n_row_chunks;                  // ceil(M / rows_per_wg)
    int32_t n_ranges;                      // workgroups along the flattened (pair, tile) axis
    int64_t num_pages;
    float scale_log2;                      // sm_scale * log2(e)
};

// Size of one partial record in 4-byte units: `rows` rows of D bf16 outputs (normalised by the
// record's own sum), then the rows' running maxima and running sums as fp32.
__host__ __device__ inline size_t attn_slot_floats(int D, int rows) { return (size_t)rows * (size_t)(D / 2 + 2); }

// The workspace starts with a header the main kernel leaves for the kernels after it: one int per
// range workgroup (kNumCU of them at most), one int per workgroup of the 256-row kernels (the
// "compute again" flags), then two ints per (sequence, kv head).
#ifdef READER_WG_STAMPS
// What a workgroup of the 128-row attention kernel records in the profiling build (thread 0 of a
// computing wavefront, or of a copying one where noted): the constant-rate counter at each point.
enum WgStamp {
    kStampEntry = 0,        // kernel entry
    kStampRange = 1,        // share of the tile axis known
    kStampList = 2,         // tile list written
    kStampFirstIssue = 3,   // (copying wavefront) the first two key tiles are asked for
    kStampFirstItem = 4,    // first item complete in LDS
    kStampFirstTile = 5,    // first key tile computed
    kStampLastTile = 6,     // last item done
    kStampExit = 7,         // after the last record / output row is written
    kStampCopyReady = 8,    // (copying wavefront) per-lane copy constants made, nothing asked for yet
    kStampItem0Issued = 9,  // (copying wavefront) the first key tile is asked for
    kStampLoopWait = 10,    // (copying wavefront, iteration 8) at the top of the iteration, before the wait for its copies
    kStampLoopIssue = 11,   // ... past the barrier, about to ask for the item three ahead
    kStampLoopIssued = 12,  // ... that item asked for
    kStampTileLanded = 13,  // first key tile complete in LDS (past the barrier that says so)
    kStampTileDone = 14,    // first key tile computed by this wavefront (before the next barrier)
    kWgStamps = 15
};
#endif
constexpr int kMaxRowChunks = 8;                           // ceil(READER_MAX_T * 16 grouped heads / 256 rows)
constexpr int kMaxAttnWorkgroups = kNumCU * kMaxRowChunks;  // range workgroups x row chunks of the 256-row kernels
__host__ __device__ inline size_t attn_header_bytes(int B, int Hkv) {
    return ((size_t)kNumCU * 4 + (size_t)kMaxAttnWorkgroups * 4 + (size_t)B * (size_t)Hkv * 8 + 255) & ~(size_t)255;
}

// Number of range workgroups the planner picks; a pure function of the dims so that
// reader_workspace_bytes and the launch agree.
int attn_plan_ranges(const reader_dims &d, int32_t max_seq_len);

struct AcceptParams;
struct CompactParams;
// ev_start / ev_stop: optional events recorded around the main kernel only.  With `ap` and
// `cp` the second launch also accepts a path per sequence and compacts it (the fused step).
hipError_t launch_tree_attn_mfma(const AttnParams &p, hipStream_t stream, hipEvent_t ev_start, hipEvent_t ev_stop,
                                 const AcceptParams *ap = nullptr, const CompactParams *cp = nullptr);
hipError_t launch_tree_attn_scalar(const AttnParams &p, hipStream_t stream);
// main kernel of the 256-row flavour with four wavefronts of 64 rows (tree_attn_wide.hip); no second launch
hipError_t launch_tree_attn_wide_main(const AttnParams &p, hipStream_t stream, hipEvent_t ev_start, hipEvent_t ev_stop);

struct AcceptParams {
    const int32_t *draft, *target, *parents;
    int32_t *accept_len, *path, *bonus, *status;
    int32_t B, T, max_path;
};
hipError_t launch_accept_path(const AcceptParams &p, hipStream_t stream);

struct CompactParams {
    const uint16_t *k_tree, *v_tree;
    const int32_t *path, *accept_len, *page_table;
    uint16_t *k_cache, *v_cache;
    int32_t *seq_lens, *status;
    int32_t B, T, Hkv, D, max_pages, max_path;
    int64_t num_pages;
};
hipError_t launch_kv_compact(const CompactParams &p, hipStream_t stream);

struct CompactLayersParams {
    uint16_t *k_cache, *v_cache;   // [NL, num_pages, Hkv, page_size, D]
    const int32_t *path, *accept_len, *page_table;
    int32_t *seq_lens, *status;
    int32_t B, T, Hkv, D, max_pages, max_path, NL;
    int64_t num_pages;
};
hipError_t launch_kv_compact_layers(const CompactLayersParams &p, hipStream_t stream);

// peak_probes.hip: the bare copy ring and the bare matrix loop behind reader_measure_peaks
hipError_t launch_probe_copy(const void *src, size_t bytes, void *scratch, hipStream_t stream, size_t *bytes_moved);
hipError_t launch_probe_mfma(int iters, void *scratch, hipStream_t stream);
constexpr size_t kProbeScratchBytes = (size_t)kNumCU * 256 * sizeof(float) + 16;

struct RearrangeParams {
    uint16_t *k_pad, *v_pad;   // [NL, B, S, Hkv, D]
    uint8_t *valid;            // [B, S]
    int32_t *new_len;          // [B]
    int32_t *dest;             // scratch: [B, S] destinations, then [B][4] = new length, old extent, first hole
    int32_t NL, B, S, Hkv, D;
};
hipError_t launch_kv_rearrange(const RearrangeParams &p, hipStream_t stream);

// 16-byte load of data that is read once: the non-temporal hint streams it past the caches
// (about a sixth more bandwidth out of HBM than a plain load on this part).
__device__ inline uint4 load_stream16(const uint4 *ptr) {
    typedef unsigned int u32x4_native __attribute__((ext_vector_type(4)));
    const u32x4_native v = __builtin_nontemporal_load(reinterpret_cast<const u32x4_native *>(ptr));
    return make_uint4(v.x, v.y, v.z, v.w);
}

hipError_t launch_target_argmax(const uint16_t *logits, int32_t *out, int rows, int V, hipStream_t stream);
hipError_t launch_target_sample(const uint16_t *logits, const int32_t *parents, const float *uniforms, int32_t *out,
                                int B, int T, int V, float temperature, hipStream_t stream);

}  // namespace reader

// Tree-masked attention on the gfx950 matrix cores (Section 3.2 of the READER paper).
//
// Work decomposition
//   A "pair" is (sequence b, kv head).  Its keys are cut into 64-key tiles: first the
//   prefix tiles (paged cache, mask-free except for the ragged last one), then the
//   tree tiles (the T tree rows, masked by ancestor-or-self bit masks held in LDS).
//   All tiles of all pairs form one flat axis.  The grid has n_ranges workgroups per
//   chunk of query rows, one per compute unit; a workgroup streams a contiguous range of
//   the axis, cut so that every range costs the same (a tile counts one, the start of a
//   pair a few more), whatever the ragged sequence lengths are.  A range may cover several
//   whole pairs and at most one pair at each end in part.  Whole pairs are finished
//   in place; a pair cut between workgroups leaves one partial record (bf16 output
//   normalised by its own sum, running max, running sum) per workgroup and a second
//   kernel merges them.  When T*G exceeds what a workgroup carries, the query rows are cut
//   into chunks, one workgroup per (range, chunk); the chunks of a range run at the same
//   time on one XCD, so that only the first of them fetches the range's tiles from HBM.
//   Each workgroup first writes the list of its items (page ids, row counts, segment
//   flags) into LDS, from a copy of the page table it fetched while the sequence lengths
//   were on their way, so the main loop does no bookkeeping.
//
// One workgroup = 8 wavefronts.  A query row is a (tree node, grouped query head) pair, so
// one K/V tile serves all heads of the group and all tree nodes.
//   128 rows per workgroup (T*G <= 128, or a small problem with more rows, cut into
//               128-row chunks): wavefronts 0..3 compute one block of 32 query rows each, wavefronts 4..7
//               only move data, always ahead of the computation: the tiles, the query
//               rows of every segment (a list item of their own that travels through the
//               ring like a tile), parent pointers and the ancestor masks made from them,
//               the list itself.  A computing wavefront never issues a memory instruction
//               inside the loop except to store finished rows.
//   256 rows per workgroup (T*G > 128): 8 row blocks of 32 rows, every wavefront computes and copies; the two
//               wavefronts of a SIMD copy at opposite ends of the tile so that they run
//               out of step.
// Per tile a computing wavefront runs
//     S^T[64 keys][32 rows] = K . Q^T             2 x 8 v_mfma_f32_32x32x16_bf16 (D = 128)
//     online softmax down the key axis: the scores a lane holds all belong to one query
//     row; weights are taken against the running reference at once and the row maximum is
//     looked for only in tiles that need it (first of a segment, masked, overflowing)
//     O^T[D][32 rows] += V^T . P^T                2 x 8 v_mfma_f32_32x32x16_bf16
//   The S^T accumulator registers of a lane are, eight at a time, exactly the B
//   operand of the second product, so the softmax weights never leave the registers.
//   V^T fragments come out of the row-major V tile through the transposing LDS load
//   (ds_read_b64_tr_b16), K fragments through plain 128-bit LDS loads.  (Matrix and vector
//   instructions overlap little on this part, within a wavefront or between the two
//   wavefronts of a SIMD, whatever their order; the tile code is a plain sequence.)
//
// K/V tiles go HBM -> LDS directly (global_load_lds_dwordx4 with the non-temporal hint: each
// wavefront instruction moves 1 KB, no staging registers) into a ring of four (three with
// 256-row workgroups) tile
// buffers; one barrier per item.  16-byte chunks are XOR-swizzled inside a tile row
// (applied on the global-address side of the copy) so that operand reads hit every LDS
// bank once.
#include <hip/hip_ext.h>

#include "accept_compact.h"
#include <mutex>

#include "internal.h"

#include "tree_attn_common.h"

namespace reader {


// RB: row blocks of 32 query rows a workgroup carries = wavefronts that compute.
//   RB = 4 (T*G <= 128): wavefronts 0..3 compute; wavefronts 4..7 only move data: they copy
//        the tiles, stage the next pair's query rows in LDS, fetch parent pointers and turn
//        them into ancestor masks, and extend the tile list, all ahead of the computation,
//        so that a computing wavefront never waits on a memory counter inside the loop.
//   RB = 8: every wavefront computes and copies its share of each tile.
// Profiling build (-DREADER_WG_STAMPS): thread `who` of the workgroup notes the time at point k
#ifdef READER_WG_STAMPS
#define READER_STAMP(k, who)                                                                              \
    do {                                                                                                  \
        if (p.stamps && threadIdx.x == (who))                                                             \
            p.stamps[(size_t)blockIdx.x * kWgStamps + (k)] = (long long)__builtin_amdgcn_s_memrealtime(); \
    } while (0)
#else
#define READER_STAMP(k, who) do { } while (0)
#endif

template <int D, int RB>
__global__ __launch_bounds__(kThreads) void tree_attn_mfma_kernel(AttnParams p,
                                                                    const int32_t *__restrict__ page_table,
                                                                    const int32_t *__restrict__ seq_lens) {
    constexpr bool kDma = RB == 4;
    constexpr int CW = kDma ? 4 : 8;
    using G = Geometry<D, CW>;
    constexpr int kRowsPerWG = 32 * RB;
    constexpr int kCopiesPerTile = 2 * G::kCopies;   // per copying wavefront
    constexpr int kS = ring_stages(RB);              // tile buffers in the ring
    constexpr int kHelpers = kDma ? 256 : kThreads;  // threads that build the tile list and the masks
    static_assert(!kDma || kRowsPerWG * G::kRowBytes == G::kStageBytes, "a query unit fills exactly one ring stage");

    extern __shared__ __attribute__((aligned(1024))) char smem[];
    char *ring = smem;                                                               // [kS][kStageBytes]
    uint32_t *s_anc = reinterpret_cast<uint32_t *>(smem + kS * G::kStageBytes);      // [2][READER_MAX_T][4]
    int *s_par = reinterpret_cast<int *>(s_anc + 2 * READER_MAX_T * 4);              // [2][READER_MAX_T]
    float *s_sink = reinterpret_cast<float *>(s_par + 2 * READER_MAX_T);             // [64] landing zone of cache-warming copies
    int *s_wsum = reinterpret_cast<int *>(s_sink + 64);                              // [8]
    TileDesc *s_desc = reinterpret_cast<TileDesc *>(s_wsum + 8);                     // [kDescSlots]
    int *s_pref = reinterpret_cast<int *>(s_desc + kDescSlots);                      // [B + 1]
    const unsigned ring_lds = (unsigned)(size_t)(lds_char *)ring;
    const unsigned par_lds = (unsigned)(size_t)(lds_char *)reinterpret_cast<char *>(s_par);
    const unsigned prefetch_lds = (unsigned)(size_t)(lds_char *)reinterpret_cast<char *>(s_sink);

    // 1-D grid.  Workgroups are handed to the XCDs round robin (id mod 8); the row chunks of
    // one range get ids 8 apart, so they run at the same time on the same XCD and the second
    // one finds the range's K/V tiles in that XCD's L2.
    int range_id, chunk_id;
    if (p.n_ranges % kNumXCD == 0) {
        const int per_group = kNumXCD * p.n_row_chunks, g = blockIdx.x / per_group, r = blockIdx.x - g * per_group;
        chunk_id = r / kNumXCD;
        range_id = g * kNumXCD + r % kNumXCD;
    } else {
        chunk_id = blockIdx.x / p.n_ranges;
        range_id = blockIdx.x - chunk_id * p.n_ranges;
    }
    // second pass behind the wide kernel: only the workgroups it asks for (same grid, same ranges)
    if (!kDma && p.redo_only && !p.redo[blockIdx.x]) return;
    READER_STAMP(kStampEntry, 0);
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave_s = __builtin_amdgcn_readfirstlane(tid >> 6);
    const bool is_computer = !kDma || wave_s < 4;
    const bool is_copier = !kDma || wave_s >= 4;
    const int cw = kDma ? (wave_s & 3) : wave_s;         // index among the copying wavefronts
    const int rb = kDma ? (wave_s & 3) : wave_s;         // row block of a computing wavefront
    const int htid = kDma ? tid - 256 : tid;             // index among the helper threads, negative: none
    const int n = lane & 31, h = lane >> 5;
    const int chunk_base = chunk_id * kRowsPerWG;
    const int row_local = rb * 32 + n;             // row inside this workgroup's chunk
    const int m_row = chunk_base + row_local;      // query row inside the pair
    const bool row_real = m_row < p.M;
    const int node = row_real ? m_row / p.G : 0;   // tree node of this lane's query row
    const int group = row_real ? m_row - node * p.G : 0;
    const bool wave_active = is_computer && chunk_base + rb * 32 < p.M;

    // Lengths -> tile counts -> this workgroup's share [lo, hi) of the tile axis; a small page table is
    // fetched whole into the last ring stage (idle until the main loop starts) on the way.
    RangeSetup rs;
    setup_range<kThreads>(p, page_table, seq_lens, ring + (kS - 1) * G::kStageBytes, ring_lds + (kS - 1) * G::kStageBytes,
                          G::kStageBytes, s_pref, s_wsum, range_id, rs);
    const TilePos lo = rs.lo, hi = rs.hi;
    const int32_t *table = rs.table;
    const bool table_in_lds = rs.table_in_lds;
    int *s_len = rs.s_len;
    const int n_tiles = hi.flat - lo.flat;
    if (chunk_id == 0 && tid == 0) p.range_tiles[range_id] = n_tiles;
    if (n_tiles <= 0) return;
    READER_STAMP(kStampRange, 0);
    // items of the list: the tiles, and with dedicated copy wavefronts one query unit per segment
    // (one segment per pair the range touches)
    int n_iter = n_tiles;
    if (kDma) n_iter += (hi.b * p.Hkv + hi.hkv) - (lo.b * p.Hkv + lo.hkv) + (hi.t > 0 ? 1 : 0);

    int bad = 0;
    auto write_item = [&](int i) {
        const bool from_lds = table_in_lds && i < kDescSlots;   // (the stage that held the copy is in use later)
        build_item<kDma>(p, from_lds ? table : page_table, from_lds, seq_lens, s_len, s_pref, lo, n_tiles, i,
                         s_desc + (i & (kDescSlots - 1)), bad);
    };
    if (htid >= 0)
        for (int i = htid; i < min(n_iter, kDescSlots); i += kHelpers) write_item(i);
    __syncthreads();   // the list is written
    READER_STAMP(kStampList, 0);

    // (off the path to the first copy: with dedicated copy wavefronts the computing ones do it, which wait anyway)
    write_pair_info(p, s_pref, lo, hi, range_id, tid);

    auto desc_of = [&](int i) -> const TileDesc * { return s_desc + (i & (kDescSlots - 1)); };
    auto desc_b = [&](int i) { return __builtin_amdgcn_readfirstlane(desc_of(i)->b); };
    auto desc_hkv = [&](int i) { return __builtin_amdgcn_readfirstlane(desc_of(i)->hkv); };
    auto desc_flags = [&](int i) { return __builtin_amdgcn_readfirstlane(desc_of(i)->flags); };
    constexpr int kQuarterShift = kDma ? 0 : 1;   // copying wavefront -> 16-key quarter of the tile

    // This lane's query row as the B operand of the QK product.
    bf16x8 qf[G::kKSteps];
    auto load_q = [&](int b, int hkv) {
        const uint16_t *qrow = p.q + (((size_t)b * p.T + node) * p.Hq + hkv * p.G + group) * D;
#pragma unroll
        for (int kk = 0; kk < G::kKSteps; ++kk)
            qf[kk] = __builtin_bit_cast(bf16x8, keep_if(row_real, ld16(qrow + kk * 16 + h * 8)));
    };
    // RB = 8: touch the next pair's query rows one tile before they are needed, so that they
    // wait in the cache: an LDS copy of 4 bytes per lane into a scratch area nobody reads.
    auto prefetch_q = [&](int b, int hkv) {
        const uint16_t *qrow = p.q + (((size_t)b * p.T + node) * p.Hq + hkv * p.G + group) * D;
        asm volatile("s_mov_b32 m0, %1\n\tglobal_load_lds_dword %0, off"
                     :: "v"(qrow + (h * 64) % D), "s"(prefetch_lds) : "memory", "m0");
    };
    // RB = 4: a query unit.  The copying wavefronts move the pair's query rows into a ring
    // stage (rows swizzled like a K tile, rows past the last one as zeros); the computing
    // wavefronts read their fragments from there.
    const float g_rcp = 1.0f / (float)p.G;
    auto issue_q = [&](int b, int hkv, unsigned stage_lds) {
        // (the lane's part of the addresses is made here, once per pair, out of the compiler's sight: made ahead
        // of the loop it stands between the start of the kernel and the first copy of a key tile)
        int ql = lane;
        asm volatile("" : "+v"(ql));
        const char *qbase = reinterpret_cast<const char *>(p.q) + ((size_t)b * p.T * p.Hq + hkv * p.G) * (D * 2);
        const char *zeros = reinterpret_cast<const char *>(kZeroRow) + (ql & 15) * 16;
#pragma unroll
        for (int i = 0; i < kCopiesPerTile; ++i) {
            const int r = (cw * kCopiesPerTile + i) * G::kRowsPerCopy + ql / G::kChunks;
            const int c = (ql % G::kChunks) ^ swizzle_k<D>(r);
            const int m = chunk_base + r;                  // query row inside the pair
            // m / G without the integer division (sixteen of them per query unit held the first copies back
            // by a microsecond): m + 0.5 is at least 0.5 / G away from the next multiple of G, far more
            // than the rounding of the product moves it (m / G <= 128)
            const int nd = (int)(((float)m + 0.5f) * g_rcp), gr = m - nd * p.G;
            const char *src = m < p.M ? qbase + ((size_t)nd * p.Hq + gr) * (D * 2) + c * 16 : zeros;
            copy16_lane(src, stage_lds + (cw * kCopiesPerTile + i) * 1024);
        }
    };
    auto read_q_stage = [&](const char *stage) {
#pragma unroll
        for (int kk = 0; kk < G::kKSteps; ++kk)
            qf[kk] = *reinterpret_cast<const bf16x8 *>(stage + row_local * G::kRowBytes +
                                                       (((2 * kk + h) ^ swizzle_k<D>(row_local)) << 4));
    };

    // Parent pointers of a sequence into s_par[buf] (asynchronous, copying wavefronts 0 and 1),
    // and from there the ancestor-or-self masks into s_anc[buf] (helper threads).
    auto copy_parents = [&](int b, int buf) {
        if (cw * 64 < p.T) {
            const int t = min(cw * 64 + lane, p.T - 1);
            const int32_t *src = p.parents + (size_t)b * p.T + t;
            const unsigned dst = par_lds + (buf * READER_MAX_T + cw * 64) * 4;
            asm volatile("s_mov_b32 m0, %1\n\tglobal_load_lds_dword %0, off" :: "v"(src), "s"(dst) : "memory", "m0");
        }
    };
    auto build_masks = [&](int buf) {
        if (htid >= 0 && htid < p.T) {
            const int *par = s_par + buf * READER_MAX_T;
            uint32_t a0 = 0u, a1 = 0u, a2 = 0u, a3 = 0u;
            int t = htid;
            for (int step = 0; step < p.T && t >= 0; ++step) {
                const uint32_t bit = 1u << (t & 31);
                const int w = t >> 5;
                a0 |= w == 0 ? bit : 0u; a1 |= w == 1 ? bit : 0u;
                a2 |= w == 2 ? bit : 0u; a3 |= w == 3 ? bit : 0u;
                int pi = par[t];
                const bool valid = t == 0 ? pi == -1 : (pi >= 0 && pi < t);
                if (!valid) { bad |= READER_STATUS_BAD_TREE; pi = -1; }
                t = pi;
            }
            uint32_t *dst = s_anc + (buf * READER_MAX_T + htid) * 4;
            dst[0] = a0; dst[1] = a1; dst[2] = a2; dst[3] = a3;
        }
    };

    // (the per-lane copy constants are made where they are used, so that they occupy registers
    // only in the wavefronts and loops that copy)
    auto issue_tile = [&](const CopyLane<D, CW> &cl, int blk, int nv, int fl, unsigned stage_lds) {
        if (p.tree_in_cache && (fl & kDescTree)) {
            // Tree rows that live in the cache: row r of tree tile tt is position L + 64 tt + r of
            // the sequence.  The positions are not aligned to pages, so every lane looks up the
            // page of its row (the table is small and sits in the caches) and gathers from there;
            // rows past the last node and rows behind a bad page id come from the block of zeros.
            const int sb = blk / p.Hkv, shkv = blk - sb * p.Hkv;
            const int pos0 = (s_len ? s_len[sb] : clamp_len(p, seq_lens, sb)) + (fl >> 8) * kTile;
            const char *zeros = reinterpret_cast<const char *>(kZeroRow) + (lane & 15) * 16;
#pragma unroll
            for (int i = 0; i < G::kCopies; ++i) {
                const int row = cl.row[i], pos = pos0 + row;
                bool ok = row < nv;
                long long page = 0;
                if (ok) {
                    page = page_table[(size_t)sb * p.max_pages + (pos >> 4)];   // pos < 16 max_pages: checked on the host
                    if (page < 0 || page >= p.num_pages) { bad |= READER_STATUS_BAD_PAGE; ok = false; }
                }
                const size_t row_off = ((size_t)(page * p.Hkv + shkv) * READER_PAGE_SIZE + (pos & 15)) * G::kRowBytes;
                const unsigned in_row = (unsigned)(row & 15) * G::kRowBytes;      // the lane's offsets are relative to a 16-row block
                const unsigned dst = stage_lds + cw * G::kRowsPerWave * G::kRowBytes + i * 1024;
                copy16_lane(ok ? reinterpret_cast<const char *>(p.k_cache) + row_off + (cl.k_cache_off[i] - in_row) : zeros, dst);
                copy16_lane(ok ? reinterpret_cast<const char *>(p.v_cache) + row_off + (cl.v_cache_off[i] - in_row) : zeros,
                            dst + G::kTileBytes);
            }
            return;
        }
        const CopyPlan cp = plan_copy<D, CW>(p, blk, nv, fl, cw);
#pragma unroll
        for (int j = 0; j < kCopiesPerTile; ++j) emit_copy<D, CW>(cp, cl, stage_lds, cw, j);
    };
    auto issue_tile_at = [&](const CopyLane<D, CW> &cl, int i, unsigned stage_lds) {
        const TileDesc *d = desc_of(i);
        issue_tile(cl, __builtin_amdgcn_readfirstlane(d->blk[cw >> kQuarterShift]),
                   __builtin_amdgcn_readfirstlane(d->n_valid), __builtin_amdgcn_readfirstlane(d->flags), stage_lds);
    };

    // Which mask buffer a segment uses: segments that need masks alternate between the two
    // buffers; the parent copies, the mask builds and the computation each count them.
    int gen_cpy = 0, gen_bld = 0, gen_use = 0;
    const uint32_t *anc = s_anc;

    // One item of the list into a ring stage (RB = 4): a query unit, or a tile, preceded by the
    // parent pointers if the tile starts a segment that reaches its tree.
    auto issue_item = [&](const CopyLane<D, CW> &cl, int i, unsigned stage_lds) {
        const TileDesc *d = desc_of(i);
        const int fl = __builtin_amdgcn_readfirstlane(d->flags);
        if (fl & kDescQ) {
            issue_q(__builtin_amdgcn_readfirstlane(d->b), __builtin_amdgcn_readfirstlane(d->hkv), stage_lds);
        } else {
            if (fl & kDescMasks) { copy_parents(__builtin_amdgcn_readfirstlane(d->b), gen_cpy & 1); ++gen_cpy; }
            issue_tile(cl, __builtin_amdgcn_readfirstlane(d->blk[cw >> kQuarterShift]),
                       __builtin_amdgcn_readfirstlane(d->n_valid), fl, stage_lds);
        }
    };

    // The same for a caller that holds the item's descriptor words already: a whole prefix tile (the common
    // item) is asked for with its copy instructions and nothing else.
    auto issue_known = [&](const CopyLane<D, CW> &cl, int i, unsigned stage_lds, int blk, int nv, int fl) {
        const bool plain = !(fl & (kDescQ | kDescMasks | kDescTree)) && blk >= 0 && (cw + 1) * G::kRowsPerWave <= nv;
        if (plain) {
            const size_t boff = (size_t)blk * (16 * G::kRowBytes);
            const char *kb = reinterpret_cast<const char *>(p.k_cache) + boff;
            const char *vb = reinterpret_cast<const char *>(p.v_cache) + boff;
            const unsigned dst = stage_lds + cw * G::kRowsPerWave * G::kRowBytes;
#pragma unroll
            for (int c = 0; c < G::kCopies; ++c) copy16_uniform(kb, cl.k_cache_off[c], dst + c * 1024);
#pragma unroll
            for (int c = 0; c < G::kCopies; ++c) copy16_uniform(vb, cl.v_cache_off[c], dst + G::kTileBytes + c * 1024);
        } else {
            issue_item(cl, i, stage_lds);
        }
    };

    // prologue: the first kS - 1 items are put in flight
    if (is_copier) {
        const CopyLane<D, CW> cl = make_copy_lane<D, CW>(p, cw, lane);
        READER_STAMP(kStampCopyReady, kDma ? 256 : 0);
        if (kDma) {
            // (item 0, the first pair's query unit, is not copied: the computing wavefronts, idle until the
            // first tile arrives, read their rows straight into registers meanwhile, and the first
            // K/V tiles are asked for that much sooner)
            int4 words[kS - 1];          // (asked for together: one LDS round trip for both items)
#pragma unroll
            for (int i = 1; i < kS - 1; ++i) {
                const TileDesc *d = desc_of(i);
                words[i] = make_int4(d->blk[cw], d->n_valid, d->flags, 0);
            }
#pragma unroll
            for (int i = 1; i < kS - 1; ++i) {
                if (i < n_iter)
                    issue_known(cl, i, ring_lds + i * G::kStageBytes, __builtin_amdgcn_readfirstlane(words[i].x),
                                __builtin_amdgcn_readfirstlane(words[i].y), __builtin_amdgcn_readfirstlane(words[i].z));
                if (i == 1) READER_STAMP(kStampItem0Issued, 256);
            }
        } else {
            issue_tile_at(cl, 0, ring_lds);
            if (n_iter > 1) issue_tile_at(cl, 1, ring_lds + G::kStageBytes);
        }
    }
    READER_STAMP(kStampFirstIssue, kDma ? 256 : 0);
    if (!kDma || wave_active) load_q(desc_b(0), desc_hkv(0));

    // per-lane LDS offsets of the matrix-core operand reads (relative to the stage)
    int k_rd[G::kKSteps];   // K fragment of k-step kk, key block 0
#pragma unroll
    for (int kk = 0; kk < G::kKSteps; ++kk)
        k_rd[kk] = n * G::kRowBytes + (((2 * kk + h) ^ swizzle_k<D>(n)) << 4);
    int v_rd[G::kOBlocks];  // V fragment of output block db, keys 0..3 (+4h) of the first 16-key group
    {
        const int i16 = lane & 15, g16 = (lane >> 4) & 1;
        const int key_lo = 4 * h + (i16 >> 2);                       // key row inside an 8-key group
        const int c_lo = 2 * g16 + ((i16 & 3) >> 1);                 // 16-byte chunk inside the 32-wide d block
#pragma unroll
        for (int db = 0; db < G::kOBlocks; ++db)
            v_rd[db] = G::kTileBytes + key_lo * G::kRowBytes +
                       ((((db * 4) | c_lo) ^ swizzle_v<D>(key_lo)) << 4) + (i16 & 1) * 8;
    }

    f32x16 o[G::kOBlocks];
    float m_run = -INFINITY, l_run = 0.f;
    bool seg_from_pair_start = false;
    const float c2 = p.scale_log2;

    uint32_t pk[2][8];     // softmax weights of the current tile, bf16 pairs, in B-operand order
    // The running reference m_run is only raised when a row's maximum outgrows it by more
    // than 2^8 (in the exp2 domain), so the accumulator rescale is rare; weights stay <= 256.
    const float grow_margin = 8.f / c2;

    f32x16 s[2];           // S^T of the current tile, one per 32-key block

    // A wavefront's vector instructions do not run under its own matrix instructions (only
    // another wavefront's do), so the tile is a plain sequence with as little exposed latency
    // as possible:
    //   K fragments of both 32-key blocks; S0, S1 = K.Q^T as two independent accumulation
    //   chains, alternating; V fragments of the first 32 keys asked for; masks, row maximum
    //   (one cross-lane swap), weights; V fragments of the other 32 keys asked for while the
    //   first half of O += V^T.P^T runs.
    // `between(j)`, j = 0..3, is called at four points of the tile (the wavefronts that also
    // copy put their copy instructions there).
    auto compute_tile = [&](const char *stage, int flags, int n_valid, auto &&between) {
        const bool is_tree = (flags & kDescTree) != 0;
        const int tt = flags >> 8;
        {
            bf16x8 ka0[G::kKSteps], ka1[G::kKSteps];
#pragma unroll
            for (int kk = 0; kk < G::kKSteps; ++kk) {
                ka0[kk] = *reinterpret_cast<const bf16x8 *>(stage + k_rd[kk]);
                ka1[kk] = *reinterpret_cast<const bf16x8 *>(stage + k_rd[kk] + 32 * G::kRowBytes);
            }
#pragma unroll
            for (int i = 0; i < 16; ++i) { s[0][i] = 0.f; s[1][i] = 0.f; }
#pragma unroll
            for (int kk = 0; kk < G::kKSteps; ++kk) {
                s[0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ka0[kk], qf[kk], s[0], 0, 0, 0);
                s[1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ka1[kk], qf[kk], s[1], 0, 0, 0);
            }
            // order handed to the scheduler: the first two reads, then one read per product
            __builtin_amdgcn_sched_group_barrier(0x100, 2, 0);
#pragma unroll
            for (int j = 0; j < 2 * G::kKSteps - 2; ++j) {
                __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
                __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
            }
            __builtin_amdgcn_sched_group_barrier(0x008, 2, 0);
        }
        between(0);

        // V^T fragments, as the two transposed reads of each (16-key step, output block); the
        // reads of a step are issued one step ahead of its products (asking for all of them
        // before the softmax costs more in registers than it saves in waiting).
        s16x4 vh[2][G::kOBlocks][2];
        auto read_v_step = [&](int ks) {
            const int key_base = ((ks >> 1) * 32 + (ks & 1) * 16) * G::kRowBytes;
#pragma unroll
            for (int db = 0; db < G::kOBlocks; ++db) {
                const char *src = stage + v_rd[db] + key_base;
                vh[ks & 1][db][0] = lds_read_tr16(src);                         // keys +0..3 (+4h)
                vh[ks & 1][db][1] = lds_read_tr16(src + 8 * G::kRowBytes);      // keys +8..11 (+4h)
            }
        };

        // softmax weights of the tile relative to the running reference -> pk; returns the lane's sum
        auto weights = [&]() {
            const float mc = (m_run == -INFINITY) ? 0.f : m_run * c2;
            float lsum0 = 0.f, lsum1 = 0.f;
#pragma unroll
            for (int kb = 0; kb < 2; ++kb)
#pragma unroll
                for (int i = 0; i < 16; i += 2) {
                    const float p0 = __builtin_amdgcn_exp2f(s[kb][i] * c2 - mc);
                    const float p1 = __builtin_amdgcn_exp2f(s[kb][i + 1] * c2 - mc);
                    lsum0 += p0;
                    lsum1 += p1;
                    pk[kb][i >> 1] = pack_bf16x2(p0, p1);
                }
            return lsum0 + lsum1;
        };
        // A whole prefix tile that does not start a segment: every row already has a finite
        // reference, so the weights are taken against it right away, without looking for the
        // row maximum first; only if some weight comes out huge (a score far above the
        // reference) is the tile redone the careful way.  bf16 and fp32 share the exponent
        // range, so large weights lose nothing.
        const int holes = (flags & kDescHoles) ? (flags >> 8) & 15 : 0;   // quarters of a prefix tile to skip
        bool careful = is_tree || n_valid < kTile || (flags & (kDescFresh | kDescHoles));
        if (!careful) {
            const float lsum = weights();
            if (__any(!(lsum < 0x1p40f))) careful = true;
            else l_run += lsum;
        }
        between(1);
        if (careful) {
            // ---- masks (ragged last prefix tile, tree tiles) ----
            if (is_tree) {
#pragma unroll
                for (int kb = 0; kb < 2; ++kb) {
                    uint32_t bits = row_real ? anc[node * 4 + tt * 2 + kb] : 0u;
                    bits >>= 4 * h;
#pragma unroll
                    for (int i = 0; i < 16; ++i) {
                        const int r = (i >> 2) * 8 + (i & 3);    // + 4h, already shifted out
                        if (!((bits >> r) & 1u)) s[kb][i] = -INFINITY;
                    }
                }
            } else if (n_valid < kTile || holes) {
#pragma unroll
                for (int kb = 0; kb < 2; ++kb)
#pragma unroll
                    for (int i = 0; i < 16; ++i) {
                        const int key = kb * 32 + (i >> 2) * 8 + 4 * h + (i & 3);
                        const int quarter = kb * 2 + (i >> 3);     // = key / 16
                        if (key >= n_valid || ((holes >> quarter) & 1)) s[kb][i] = -INFINITY;
                    }
            }
            // ---- online softmax along the keys (all values of a lane share one query row) ----
            float mx0 = fmaxf(s[0][0], s[0][1]), mx1 = fmaxf(s[1][0], s[1][1]);
#pragma unroll
            for (int i = 2; i < 16; i += 2) {
                mx0 = fmaxf(fmaxf(mx0, s[0][i]), s[0][i + 1]);
                mx1 = fmaxf(fmaxf(mx1, s[1][i]), s[1][i + 1]);
            }
            float mx = fmaxf(mx0, mx1);
            {   // the other half of the row's keys sits in lane ^ 32
                const auto sw = __builtin_amdgcn_permlane32_swap(__float_as_uint(mx), __float_as_uint(mx), false, false);
                mx = fmaxf(__uint_as_float(sw[0]), __uint_as_float(sw[1]));
            }
            const bool grow = mx > m_run + grow_margin;     // also the first finite maximum (m_run = -inf)
            if (__any(grow)) {
                const float alpha = grow ? __builtin_amdgcn_exp2f((m_run - mx) * c2) : 1.f;   // m_run = -inf gives 0
                m_run = grow ? mx : m_run;
                l_run *= alpha;
#pragma unroll
                for (int db = 0; db < G::kOBlocks; ++db)
#pragma unroll
                    for (int i = 0; i < 16; ++i) o[db][i] *= alpha;
            }
            l_run += weights();
            // A row whose every key so far was skipped (quarters behind bad page ids) has no reference yet; the
            // whole tiles that follow take their weights against the reference without looking, so it gets a
            // finite one, so low that the first real score overflows the check there and is handled with care.
            if (holes) m_run = fmaxf(m_run, -1e30f);
        }
        between(2);

        // ---- O^T += V^T . P^T : the S^T registers of a lane are, 8 at a time, the B operand ----
        auto pv_step = [&](int ks) {
            const int kb = ks >> 1, m2 = ks & 1;
            u32x4 pv;
            pv.x = pk[kb][4 * m2]; pv.y = pk[kb][4 * m2 + 1]; pv.z = pk[kb][4 * m2 + 2]; pv.w = pk[kb][4 * m2 + 3];
            const bf16x8 pb = __builtin_bit_cast(bf16x8, pv);
#pragma unroll
            for (int db = 0; db < G::kOBlocks; ++db) {
                const s16x8 a8 = __builtin_shufflevector(vh[ks & 1][db][0], vh[ks & 1][db][1], 0, 1, 2, 3, 4, 5, 6, 7);
                o[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a8), pb, o[db], 0, 0, 0);
            }
        };
        read_v_step(0);
#pragma unroll
        for (int ks = 0; ks < 4; ++ks) {
            if (ks + 1 < 4) read_v_step(ks + 1);
            pv_step(ks);
        }
        between(3);
    };

    auto reset_state = [&](int flags) {
        seg_from_pair_start = (flags & kDescPairStart) != 0;
        m_run = -INFINITY;
        l_run = 0.f;
#pragma unroll
        for (int db = 0; db < G::kOBlocks; ++db)
#pragma unroll
            for (int i = 0; i < 16; ++i) o[db][i] = 0.f;
    };

    // End of a segment (its pair ends, or the range does): a pair that this workgroup saw
    // from its first to its last tile is normalised and written out, anything else leaves
    // a partial record for the merge kernel.
    auto finish_segment = [&](int it, bool pair_ends) {
        const int e_b = desc_b(it), e_hkv = desc_hkv(it);
        const float l_tot = l_run + __shfl_xor(l_run, 32);
        if (seg_from_pair_start && pair_ends) {
            // A lane holds, per 8-wide chunk of the output row, 4 values and its partner lane
            // (lane ^ 32) the other 4.  One half-wave swap per pair of chunks gives every lane
            // whole 16-byte chunks: lane h of the pair ends up with chunk 2k + h.
            const float inv = 1.f / l_tot;
            uint16_t *orow = p.out + (((size_t)e_b * p.T + node) * p.Hq + e_hkv * p.G + group) * D;
#pragma unroll
            for (int db = 0; db < G::kOBlocks; ++db)
#pragma unroll
                for (int i4 = 0; i4 < 4; i4 += 2) {
                    const uint32_t a0 = pack_bf16x2(o[db][4 * i4] * inv, o[db][4 * i4 + 1] * inv);
                    const uint32_t a1 = pack_bf16x2(o[db][4 * i4 + 2] * inv, o[db][4 * i4 + 3] * inv);
                    const uint32_t b0 = pack_bf16x2(o[db][4 * i4 + 4] * inv, o[db][4 * i4 + 5] * inv);
                    const uint32_t b1 = pack_bf16x2(o[db][4 * i4 + 6] * inv, o[db][4 * i4 + 7] * inv);
                    const auto s0 = __builtin_amdgcn_permlane32_swap(a0, b0, false, false);
                    const auto s1 = __builtin_amdgcn_permlane32_swap(a1, b1, false, false);
                    u32x4 w;
                    w.x = s0[0]; w.y = s1[0]; w.z = s0[1]; w.w = s1[1];
                    if (row_real) *reinterpret_cast<u32x4 *>(orow + db * 32 + (i4 + h) * 8) = w;
                }
            if (row_real && p.lse && h == 0)
                p.lse[((size_t)e_b * p.Hq + e_hkv * p.G + group) * p.T + node] =
                    (m_run * c2 + __builtin_amdgcn_logf(l_tot)) * kLn2;
        } else {
            // Partial record: the output so far, normalised by its own sum and rounded to bf16,
            // as [D / 8 chunks][rows][8 values] (the order the swapped registers hold it, so every
            // store instruction writes whole 512-byte runs), then the maxima and the sums.
            const size_t slot = ((size_t)(2 * range_id + (seg_from_pair_start ? 1 : 0)) * p.n_row_chunks + chunk_id);
            float *rec = p.workspace + slot * attn_slot_floats(D, kRowsPerWG);
            u32x4 *rec16 = reinterpret_cast<u32x4 *>(rec);
            const float inv = l_tot > 0.f ? 1.f / l_tot : 0.f;   // a row may see no key of this segment
#pragma unroll
            for (int db = 0; db < G::kOBlocks; ++db)
#pragma unroll
                for (int i4 = 0; i4 < 4; i4 += 2) {
                    const uint32_t a0 = pack_bf16x2(o[db][4 * i4] * inv, o[db][4 * i4 + 1] * inv);
                    const uint32_t a1 = pack_bf16x2(o[db][4 * i4 + 2] * inv, o[db][4 * i4 + 3] * inv);
                    const uint32_t b0 = pack_bf16x2(o[db][4 * i4 + 4] * inv, o[db][4 * i4 + 5] * inv);
                    const uint32_t b1 = pack_bf16x2(o[db][4 * i4 + 6] * inv, o[db][4 * i4 + 7] * inv);
                    const auto s0 = __builtin_amdgcn_permlane32_swap(a0, b0, false, false);
                    const auto s1 = __builtin_amdgcn_permlane32_swap(a1, b1, false, false);
                    u32x4 w;
                    w.x = s0[0]; w.y = s1[0]; w.z = s0[1]; w.w = s1[1];
                    // (streamed past the caches: read next by the merge kernel, on other compute units; on short
                    // launches the end of the kernel has less to write back, 0.7 us of the single-prompt step)
                    __builtin_nontemporal_store(w, &rec16[(size_t)(db * 4 + i4 + h) * kRowsPerWG + row_local]);
                }
            if (h == 0) {
                float *ml = rec + (size_t)kRowsPerWG * (D / 2);
                ml[row_local] = m_run * c2;
                ml[kRowsPerWG + row_local] = l_tot;
            }
        }
    };

    // The tile list is extended half a list at a time while the half it replaces is no
    // longer read and long before the new half is.
    auto extend_list = [&](int it) {
        if ((it & (kDescSlots / 2 - 1)) == 0 && it > 0 && htid >= 0 && htid < kDescSlots / 2) {
            const int i = it + kDescSlots / 2 + htid;
            if (i < n_iter) write_item(i);
        }
    };

    // LDS byte offsets of the ring stages (RB = 8, three stages): tile being computed, next
    // tile, tile being copied
    int st_cur = 0, st_nxt = G::kStageBytes, st_cpy = 2 * G::kStageBytes;
    auto rotate_stages = [&]() {
        const int t = st_cur;
        st_cur = st_nxt; st_nxt = st_cpy; st_cpy = t;
    };

    if (kDma && is_copier) {
        // ---------------- wavefronts that only move data (RB = 4) ----------------
        const CopyLane<D, CW> cl = make_copy_lane<D, CW>(p, cw, lane);
        // Between two barriers this wavefront has one item to ask for, and how long that takes sets the
        // pace of a workgroup whenever memory is not the limit (short contexts, the first tiles of any
        // launch): the words of the item's descriptor are therefore read one iteration ahead, so
        // that nothing here waits for LDS, and a whole prefix tile (the common item) is asked for
        // with eight copy instructions and nothing else.
        int n_flags = desc_flags(1);        // flags of item it + 1
        int flags_2 = desc_flags(2);        // flags of item it + 2
        int d_blk = desc_of(kS - 1)->blk[cw];                                       // of item it + kS - 1,
        int2 d_nf = *reinterpret_cast<const int2 *>(&desc_of(kS - 1)->n_valid);    // the next one to ask for
        for (int it = 0; it < n_iter; ++it) {
            // This wavefront's part of item `it` has landed once at most its copies of the items
            // after it are outstanding (copies complete in the order they were issued).
            const int ahead = n_iter - 1 - it;
            const int c_blk = __builtin_amdgcn_readfirstlane(d_blk);
            const int c_valid = __builtin_amdgcn_readfirstlane(d_nf.x);
            const int c_flags = __builtin_amdgcn_readfirstlane(d_nf.y);
            if (it == 8) READER_STAMP(kStampLoopWait, 256);
            if (ahead >= kS - 2) wait_vmcnt<(kS - 2) * kCopiesPerTile>();
            else if (ahead == 1) wait_vmcnt<kCopiesPerTile>();
            else wait_vmcnt<0>();
            __syncthreads();   // item `it` is complete in LDS; every wavefront is done with item it - 1

            d_blk = desc_of(it + kS)->blk[cw];
            d_nf = *reinterpret_cast<const int2 *>(&desc_of(it + kS)->n_valid);
            extend_list(it);
            // masks of a segment that starts with the next item (its parent pointers were asked
            // for before copies this wavefront has just waited for)
            if (ahead >= 1 && (n_flags & kDescMasks)) { build_masks(gen_bld & 1); ++gen_bld; }
            n_flags = flags_2;
            flags_2 = c_flags;

            // item it + kS - 1 goes into the stage that item it - 1 has left
            if (it == 8) READER_STAMP(kStampLoopIssue, 256);
            if (it + kS - 1 < n_iter) {
                issue_known(cl, it + kS - 1, ring_lds + ((it + kS - 1) % kS) * G::kStageBytes, c_blk, c_valid, c_flags);
            }
            if (it == 8) READER_STAMP(kStampLoopIssued, 256);
        }
    } else if (kDma) {
        // ---------------- wavefronts that only compute (RB = 4) ----------------
        int2 d_cur = *reinterpret_cast<const int2 *>(&desc_of(0)->n_valid);
        for (int it = 0; it < n_iter; ++it) {
            const char *stage = ring + (it % kS) * G::kStageBytes;
            const int t_valid = __builtin_amdgcn_readfirstlane(d_cur.x);
            const int t_flags = __builtin_amdgcn_readfirstlane(d_cur.y);
            const bool last_iter = it + 1 == n_iter;
            const bool pair_ends = (t_flags & kDescPairEnd) != 0;
            __syncthreads();   // item `it` is complete in LDS
            if (it == 0) READER_STAMP(kStampFirstItem, 0);
            if (it == 1) READER_STAMP(kStampTileLanded, 0);
            if (it == 2) READER_STAMP(kStampFirstTile, 0);   // (item 0 is the query unit: item 1, the first key tile, is done)
            d_cur = *reinterpret_cast<const int2 *>(&desc_of(it + 1)->n_valid);

            if (t_flags & kDescQ) {
                if (wave_active && it > 0) read_q_stage(stage);   // (the first one was read from memory before the loop)
                continue;
            }
            if (t_flags & kDescFresh) {
                reset_state(t_flags);
                if (t_flags & kDescMasks) { anc = s_anc + (gen_use & 1) * READER_MAX_T * 4; ++gen_use; }
            }
            if (wave_active) {
                compute_tile(stage, t_flags, t_valid, [](int) {});
                if (it == 1) READER_STAMP(kStampTileDone, 0);
                if (last_iter) READER_STAMP(kStampLastTile, 0);
                if (pair_ends || last_iter) finish_segment(it, pair_ends);
            }
        }
    } else {
        // ---------------- every wavefront computes and copies (RB = 8) ----------------
        const CopyLane<D, CW> cl = make_copy_lane<D, CW>(p, cw, lane);
        // descriptor words of the tile to compute (rows, flags) and of the tile to copy, read one
        // iteration ahead so that the LDS latency hides behind the barrier
        int2 d_cur = *reinterpret_cast<const int2 *>(&desc_of(0)->n_valid);
        int2 d_cpy = *reinterpret_cast<const int2 *>(&desc_of(2)->n_valid);
        int d_blk = desc_of(2)->blk[cw >> kQuarterShift];
        for (int it = 0; it < n_iter; ++it) {
            const char *stage = ring + st_cur;
            const int t_valid = __builtin_amdgcn_readfirstlane(d_cur.x);
            const int t_flags = __builtin_amdgcn_readfirstlane(d_cur.y);
            const int c_valid = __builtin_amdgcn_readfirstlane(d_cpy.x);
            const int c_flags = __builtin_amdgcn_readfirstlane(d_cpy.y);
            const int c_blk = __builtin_amdgcn_readfirstlane(d_blk);
            const bool last_iter = it + 1 == n_iter;
            const bool copy_next = it + 2 < n_iter;
            const bool pair_ends = (t_flags & kDescPairEnd) != 0;
            const unsigned next_stage = ring_lds + st_cpy;

            if (!last_iter) wait_vmcnt<kCopiesPerTile>(); else wait_vmcnt<0>();
            __syncthreads();   // tile `it` is complete in LDS; every wavefront is done with tile it - 1
            if (it == 0) READER_STAMP(kStampFirstItem, 0);
            if (it == 1) READER_STAMP(kStampFirstTile, 0);

            d_cur = *reinterpret_cast<const int2 *>(&desc_of(it + 1)->n_valid);
            d_cpy = *reinterpret_cast<const int2 *>(&desc_of(it + 3)->n_valid);
            d_blk = desc_of(it + 3)->blk[cw >> kQuarterShift];
            extend_list(it);

            if (t_flags & kDescFresh) {
                reset_state(t_flags);
                const int sb = desc_b(it);
                if (it != 0) load_q(sb, desc_hkv(it));
                // ancestor-or-self masks of this sequence's tree, if this segment reaches its tree tiles
                if (t_flags & kDescMasks) {
                    if (tid < p.T) s_par[tid] = p.parents[(size_t)sb * p.T + tid];
                    __syncthreads();
                    build_masks(0);
                    __syncthreads();
                }
            }
            if (pair_ends && !last_iter) prefetch_q(desc_b(it + 1), desc_hkv(it + 1));

            // Tile it + 2 is copied into the stage that tile it - 1 has left.  A wavefront stalls on
            // a copy instruction while the memory pipeline is full.  The two wavefronts that share a
            // SIMD (w and w + 4) are kept out of step by it: one copies before it computes, the other
            // after, so that one's matrix work tends to run under the other's vector work.
            // (a tree tile whose rows live in the cache has no tree tensor to copy from: it is
            // gathered row by row through the page table, by the same code as in the prologue)
            const bool gather_next = p.tree_in_cache && (c_flags & kDescTree);
            CopyPlan cp;
            if (copy_next && !gather_next) cp = plan_copy<D, CW>(p, c_blk, c_valid, c_flags, cw);
            auto copy_all = [&]() {
                if (copy_next) {
                    if (gather_next) {
                        issue_tile(cl, c_blk, c_valid, c_flags, next_stage);
                    } else {
#pragma unroll
                        for (int j = 0; j < kCopiesPerTile; ++j) emit_copy<D, CW>(cp, cl, next_stage, cw, j);
                    }
                }
            };
            if (wave_active) {
                if (wave_s >= 4) copy_all();
                compute_tile(stage, t_flags, t_valid, [](int) {});
                if (wave_s < 4) copy_all();
                if (last_iter) READER_STAMP(kStampLastTile, 0);
                if (pair_ends || last_iter) finish_segment(it, pair_ends);
            } else {
                copy_all();
            }
            rotate_stages();
        }
    }

    READER_STAMP(kStampExit, 0);
    if (p.status && bad) atomicOr(p.status, bad);
}

// Merge the partial records of every pair that was cut between workgroups.
// A record holds [D / 8 chunks][rows][8 bf16] of output normalised by the record's own sum, then
// the rows' running maxima, then their running sums.  One thread takes one 8-wide chunk of one
// query row: D / 8 threads per row, 256 / (D / 8) rows per workgroup; grid = (B * Hkv, rows / that).
// Which workgroups hold a pair's records, and which ranges are empty, come from the header the
// main kernel wrote.
template <int D>
__device__ inline void merge_body(const AttnParams &p, int pair, int block_y) {
    const int b = pair / p.Hkv, hkv = pair - b * p.Hkv;
    const int2 info = reinterpret_cast<const int2 *>(p.pair_info)[pair];
    const int w_first = info.x, w_last = info.y;
    if (w_first == w_last) return;   // finished in place by one workgroup (the whole workgroup leaves)

    // p.merge_groups (1 or 4) thread groups share a query row's records: with few pairs and many
    // ranges a pair is cut into dozens of parts, and the groups fetch theirs side by side.
    constexpr int kC = D / 8;                   // chunks (threads) per row
    const int groups = p.merge_groups, group_threads = 256 / groups;
    const int rows_per_block = group_threads / kC;
    const int tid = threadIdx.x, grp = tid / group_threads, t2 = tid - grp * group_threads;
    const int blocks_per_chunk = p.rows_per_wg / rows_per_block;
    const int row_chunk = block_y / blocks_per_chunk;
    const int block_in_chunk = block_y - row_chunk * blocks_per_chunk;
    // Thread -> (row, 8-wide chunk).  One group: a workgroup takes rows_per_block whole rows, a row's chunks on
    // neighbouring threads.  Four groups (one wavefront each): a record is laid out [chunk][row], so a wavefront
    // takes 16 consecutive rows of four chunks (256 contiguous bytes per chunk and load) instead of four whole
    // rows (64), and the workgroups of a row block take a quarter of the chunks each; same number of workgroups.
    int row_local, c;
    if (groups == 1) {
        row_local = block_in_chunk * rows_per_block + t2 / kC;
        c = t2 % kC;
    } else {
        constexpr int kQuarters = kC / 4;
        row_local = (block_in_chunk / kQuarters) * 16 + (t2 & 15);
        c = (block_in_chunk % kQuarters) * 4 + (t2 >> 4);
    }
    const int m_row = row_chunk * p.rows_per_wg + row_local;
    const bool live = m_row < p.M;
    const int node = live ? m_row / p.G : 0, group = live ? m_row - node * p.G : 0;
    const size_t rows = p.rows_per_wg;
    const size_t rec_floats = attn_slot_floats(D, p.rows_per_wg);
    // this group's share of the parts, in range order
    const int n_parts = w_last - w_first + 1, share = (n_parts + groups - 1) / groups;
    const int my_first = w_first + grp * share, my_last = min(w_last, my_first + share - 1);

    // online merge: every part's loads are independent of the other parts' values
    float m_all = -INFINITY, l_all = 0.f;
    float acc[8];
#pragma unroll
    for (int d = 0; d < 8; ++d) acc[d] = 0.f;
    // Records are fetched eight at a time (all their loads in flight together) and folded in in range order.
    constexpr int kBatch = 8;
    for (int w0 = my_first; w0 <= my_last && live; w0 += kBatch) {
        float mw[kBatch], lw[kBatch];
        uint4 v[kBatch];
#pragma unroll
        for (int j = 0; j < kBatch; ++j) {
            const int w = w0 + j;
            mw[j] = -INFINITY;
            if (w <= my_last) {
                // A range that holds no tile (more workgroups than tiles) wrote no record: its slot
                // holds stale bytes.  The slot is read all the same, next to the range's tile count and
                // not behind it (one round trip less), and dropped afterwards.
                const int n_here = p.range_tiles[w];
                const size_t slot = ((size_t)(2 * w + (w == w_first ? 1 : 0)) * p.n_row_chunks + row_chunk);
                const float *rec = p.workspace + slot * rec_floats;
                const float m_rec = rec[rows * (D / 2) + row_local];
                lw[j] = rec[rows * (D / 2 + 1) + row_local];
                v[j] = reinterpret_cast<const uint4 *>(rec)[(size_t)c * rows + row_local];
                mw[j] = n_here != 0 ? m_rec : -INFINITY;
            }
        }
#pragma unroll
        for (int j = 0; j < kBatch; ++j) {
            if (mw[j] == -INFINITY) continue;   // no record, or this row saw no key of that part
            const float m_new = fmaxf(m_all, mw[j]);
            const float fa = __builtin_amdgcn_exp2f(m_all - m_new);      // 0 for the first part
            const float fb = __builtin_amdgcn_exp2f(mw[j] - m_new) * lw[j];
            const uint32_t u[4] = {v[j].x, v[j].y, v[j].z, v[j].w};
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                acc[2 * e] = acc[2 * e] * fa + fb * __uint_as_float(u[e] << 16);
                acc[2 * e + 1] = acc[2 * e + 1] * fa + fb * __uint_as_float(u[e] & 0xffff0000u);
            }
            l_all = l_all * fa + fb;
            m_all = m_new;
        }
    }
    if (groups > 1) {
        // groups 1.. leave their state in LDS; group 0 folds them in, in range order
        __shared__ float s_state[3][64][10];
        if (grp > 0) {
            float *st = s_state[grp - 1][t2];
            st[0] = m_all; st[1] = l_all;
#pragma unroll
            for (int d = 0; d < 8; ++d) st[2 + d] = acc[d];
        }
        __syncthreads();
        if (grp > 0) return;
        for (int g = 0; g < groups - 1; ++g) {
            const float *st = s_state[g][t2];
            const float m_g = st[0];
            if (m_g == -INFINITY) continue;
            const float m_new = fmaxf(m_all, m_g);
            const float fa = __builtin_amdgcn_exp2f(m_all - m_new), fb = __builtin_amdgcn_exp2f(m_g - m_new);
#pragma unroll
            for (int d = 0; d < 8; ++d) acc[d] = acc[d] * fa + st[2 + d] * fb;
            l_all = l_all * fa + st[1] * fb;
            m_all = m_new;
        }
    }
    if (!live) return;
    // l_all > 0: every query row sees at least its own tree node
    const float inv = 1.f / l_all;
    uint16_t *orow = p.out + (((size_t)b * p.T + node) * p.Hq + hkv * p.G + group) * D + c * 8;
    uint4 w;
    w.x = pack_bf16x2(acc[0] * inv, acc[1] * inv);
    w.y = pack_bf16x2(acc[2] * inv, acc[3] * inv);
    w.z = pack_bf16x2(acc[4] * inv, acc[5] * inv);
    w.w = pack_bf16x2(acc[6] * inv, acc[7] * inv);
    *reinterpret_cast<uint4 *>(orow) = w;
    if (p.lse && c == 0)
        p.lse[((size_t)b * p.Hq + hkv * p.G + group) * p.T + node] = (m_all + __builtin_amdgcn_logf(l_all)) * kLn2;
}

template <int D>
__global__ __launch_bounds__(256) void tree_attn_merge_kernel(AttnParams p) {
    merge_body<D>(p, blockIdx.x, blockIdx.y);
}

// Tail of the fused step: one workgroup per sequence that accepts a path and appends its rows
// to the cache, then the merge blocks.  The three jobs touch disjoint data (the merge reads
// the workspace and writes `out`; acceptance reads tokens; compaction writes cache slots past
// the old lengths and the lengths themselves, which the merge does not read).
template <int D>
__global__ __launch_bounds__(256) void verify_tail_kernel(AttnParams p, AcceptParams ap, CompactParams cp,
                                                           int merge_blocks_y) {
    // the per-sequence workgroups come first in the grid: theirs is the longest chain of
    // dependent memory accesses, so they should start first
    if ((int)blockIdx.x >= p.B) {
        const int m = blockIdx.x - p.B;
        merge_body<D>(p, m / merge_blocks_y, m % merge_blocks_y);
        return;
    }
    __shared__ AcceptShared sh;
    __shared__ CompactShared cs;
    const int b = blockIdx.x, tid = threadIdx.x;
    // (in-cache layout, no tree tensors: the in-place move of the accepted rows follows as a launch of its own)
    const bool append = cp.k_tree != nullptr;
    if (append) kv_compact_prefetch(cp, b, tid, cs);   // on its way while the path is being chosen
    accept_path_body(ap, b, tid, tid < 64, sh);
    if (!append) return;
    __syncthreads();
    kv_compact_body(cp, b, tid, sh.accept_len, sh.path, cs);
}

template <int D, int RB>
static hipError_t launch_mfma(const AttnParams &p, hipStream_t stream, hipEvent_t ev_start, hipEvent_t ev_stop) {
    using G = Geometry<D, RB == 4 ? 4 : 8>;
    const size_t pref_bytes = ((size_t)(p.B + 1) * sizeof(int) + 15) & ~(size_t)15;
    const size_t main_lds = (size_t)ring_stages(RB) * G::kStageBytes +
                            2 * READER_MAX_T * 4 * sizeof(uint32_t) + 2 * READER_MAX_T * sizeof(int) +
                            64 * sizeof(float) + 8 * sizeof(int) + kDescSlots * sizeof(TileDesc) + pref_bytes +
                            (p.B <= kMaxLensInLds ? (size_t)p.B * sizeof(int) + 16 : 0);
    // More than 64 KB of LDS per workgroup has to be asked for; the limit counts the
    // kernel's static LDS too, so ask for exactly what this launch needs.
    {
        static std::mutex guard;             // host threads may call in at the same time
        static size_t lds_allowed = 0;
        std::lock_guard<std::mutex> lock(guard);
        if (main_lds > lds_allowed) {
            hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(&tree_attn_mfma_kernel<D, RB>),
                                               hipFuncAttributeMaxDynamicSharedMemorySize, (int)main_lds);
            if (e != hipSuccess) { (void)hipGetLastError(); return note_hip_error("hipFuncSetAttribute(attention LDS size)", e); }
            lds_allowed = main_lds;
        }
    }
    // with events: they take the kernel's own start and end time stamps
    if (ev_start && ev_stop)
        hipExtLaunchKernelGGL((tree_attn_mfma_kernel<D, RB>), dim3(p.n_ranges * p.n_row_chunks), dim3(kThreads),
                              main_lds, stream, ev_start, ev_stop, 0, p, p.page_table, p.seq_lens);
    else
        hipLaunchKernelGGL((tree_attn_mfma_kernel<D, RB>), dim3(p.n_ranges * p.n_row_chunks), dim3(kThreads),
                           main_lds, stream, p, p.page_table, p.seq_lens);
    return note_hip_error("launch tree_attn_mfma_kernel", hipGetLastError());
}

// Second launch: merge of the partial records, and in the fused step acceptance and compaction.
template <int D>
static hipError_t launch_tail(const AttnParams &p, hipStream_t stream, const AcceptParams *ap, const CompactParams *cp) {
    const int merge_y = p.n_row_chunks * (p.rows_per_wg / (256 / p.merge_groups / (D / 8)));
    if (ap && cp) {
        const int n_merge = p.B * p.Hkv * merge_y;
        hipLaunchKernelGGL(verify_tail_kernel<D>, dim3(p.B + n_merge), dim3(256), 0, stream, p, *ap, *cp, merge_y);
        return note_hip_error("launch verify_tail_kernel", hipGetLastError());
    }
    hipLaunchKernelGGL(tree_attn_merge_kernel<D>, dim3(p.B * p.Hkv, merge_y), dim3(256), 0, stream, p);
    return note_hip_error("launch tree_attn_merge_kernel", hipGetLastError());
}

hipError_t launch_tree_attn_mfma(const AttnParams &p, hipStream_t stream, hipEvent_t ev_start, hipEvent_t ev_stop,
                                 const AcceptParams *ap, const CompactParams *cp) {
    hipError_t e;
    if (p.rows_per_wg == 128) {
        e = p.D == 64 ? launch_mfma<64, 4>(p, stream, ev_start, ev_stop) : launch_mfma<128, 4>(p, stream, ev_start, ev_stop);
    } else if (p.wide) {
        // Four wavefronts of 64 rows with a softmax reference that is fixed per segment; a workgroup whose
        // scores outgrew that reference says so, and the kernel that moves its reference (eight wavefronts of
        // 32 rows, same ranges, same records) then computes those workgroups' ranges again.  It is launched
        // every time and leaves at once where nothing is asked of it.
        e = launch_tree_attn_wide_main(p, stream, ev_start, ev_stop);
        if (e != hipSuccess) return e;
        AttnParams again = p;
        again.redo_only = 1;
        e = p.D == 64 ? launch_mfma<64, 8>(again, stream, nullptr, nullptr) : launch_mfma<128, 8>(again, stream, nullptr, nullptr);
    } else {
        e = p.D == 64 ? launch_mfma<64, 8>(p, stream, ev_start, ev_stop) : launch_mfma<128, 8>(p, stream, ev_start, ev_stop);
    }
    if (e != hipSuccess) return e;
    return p.D == 64 ? launch_tail<64>(p, stream, ap, cp) : launch_tail<128>(p, stream, ap, cp);
}

}  // namespace reader

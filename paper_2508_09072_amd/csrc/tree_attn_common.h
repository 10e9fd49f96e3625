// Device code shared by the tree-attention kernels (Section 3.2 of the READER paper): the cut of the
// flattened (sequence, kv head, tile) axis into ranges of equal cost, the per-workgroup tile list in
// LDS, the asynchronous HBM -> LDS tile copies and their LDS swizzle, and small register helpers.
// Included by the translation units that hold the kernels; nothing here is part of the C ABI.
#pragma once

#include <hip/hip_runtime.h>

#include <type_traits>
#include <utility>

#include "internal.h"

namespace reader {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
// 16 bytes as a native vector (selects and copies of it stay in registers)
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef short s16x8 __attribute__((ext_vector_type(8)));
typedef __attribute__((address_space(3))) s16x4 lds_s16x4;
typedef __attribute__((address_space(3))) char lds_char;

// 256 bytes of zeros: the copy source of tile rows that do not exist.
static __device__ __attribute__((aligned(256))) const unsigned int kZeroRow[64] = {0u};

namespace {

constexpr float kLn2 = 0.69314718055994530942f;
// ring depth: 4 tile buffers when dedicated wavefronts copy (up to 128 query rows), else 3
constexpr int ring_stages(int rb) { return rb == 4 ? 4 : 3; }
constexpr int kMaxLensInLds = 1024;   // batches up to this size keep the clamped lengths in LDS

__device__ inline int clamp_len(const AttnParams &p, const int32_t *__restrict__ seq_lens, int b) {
    int L = seq_lens[b];
    L = L < 0 ? 0 : L;
    return L > p.max_seq_len ? p.max_seq_len : L;
}

// Exclusive prefix sums of tiles-per-pair over the sequences, into s_pref[0..B].
// Works for any workgroup size that is a multiple of 64 up to 512; s_wsum has 8 entries.
// s_len (optional) receives the clamped lengths.
__device__ inline void scan_units(const AttnParams &p, const int32_t *__restrict__ seq_lens, int *s_pref,
                                  int *s_wsum, int *s_len = nullptr) {
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int n_threads = blockDim.x, n_waves = n_threads >> 6;
    int carry = 0;
    if (tid == 0) s_pref[0] = 0;
    for (int base = 0; base < p.B; base += n_threads) {
        const int b = base + tid;
        int v = 0;
        if (b < p.B) {
            const int L = clamp_len(p, seq_lens, b);
            if (s_len) s_len[b] = L;
            v = (L + kTile - 1) / kTile + p.n_tree_tiles;
        }
#pragma unroll
        for (int off = 1; off < 64; off <<= 1) {
            const int t = __shfl_up(v, off);
            if (lane >= off) v += t;
        }
        if (lane == 63) s_wsum[wave] = v;
        __syncthreads();
        int woff = 0, total = 0;
        for (int w = 0; w < n_waves; ++w) {
            if (w < wave) woff += s_wsum[w];
            total += s_wsum[w];
        }
        if (b < p.B) s_pref[b + 1] = carry + woff + v;
        carry += total;
        __syncthreads();
    }
}

// Cutting the tile axis into ranges of equal cost.  Every pair (sequence b, kv head) is given
// E extra positions (E = pair_cost: what a pair costs the workgroups that start and finish it
// beyond its tiles, in tile times), F of them in front of its tiles (F = pair_front: the query
// rows to fetch, the first tile's row maxima) and E - F behind them (the ragged last prefix tile,
// the masks of the tree tiles, normalising and writing the rows), and the axis of these "cost
// positions" is cut evenly; a workgroup owns the tiles whose positions fall into its share.  The
// pair's n_b tiles and its padding start at
//     Hkv * (pref[b] + b * E) + hkv * (n_b + E),
// tile t sits F + t positions further.
// I is the integer type of the axis: int when the host has checked that every position times
// the number of ranges fits (64-bit division costs a workgroup a good part of a microsecond).
template <typename I>
__device__ inline I range_begin(I w, I U, int n_ranges) { return w * U / n_ranges; }

// Workgroup whose range contains cost position x.
template <typename I>
__device__ inline int range_of_position(I x, I U, int n_ranges) {
    // largest w with floor(w * U / n) <= x  <=>  w * U < (x + 1) * n  <=>  w <= ((x + 1) * n - 1) / U
    const I w = ((x + 1) * n_ranges - 1) / U;
    return (int)(w < n_ranges ? w : n_ranges - 1);
}

template <typename I>
__device__ inline I cost_total(const AttnParams &p, const int *s_pref) {
    return (I)p.Hkv * (s_pref[p.B] + (I)p.B * p.pair_cost);
}
template <typename I>
__device__ inline I cost_pos_of_tile(const AttnParams &p, const int *s_pref, int b, int hkv, int t) {
    const int n_b = s_pref[b + 1] - s_pref[b];
    return (I)p.Hkv * (s_pref[b] + (I)b * p.pair_cost) + (I)hkv * (n_b + p.pair_cost) + p.pair_front + t;
}

// Inclusive prefix sum over the 64 lanes of a wavefront with data-parallel-primitive moves:
// four shifted adds inside each row of 16 lanes (lanes shifted in from outside the row read 0),
// then lane 15 of rows 0 and 2 is added to rows 1 and 3, then lane 31 to rows 2 and 3.
__device__ inline int wave_inclusive_scan(int v) {
    v += __builtin_amdgcn_update_dpp(0, v, 0x111, 0xf, 0xf, true);   // row_shr:1
    v += __builtin_amdgcn_update_dpp(0, v, 0x112, 0xf, 0xf, true);   // row_shr:2
    v += __builtin_amdgcn_update_dpp(0, v, 0x114, 0xf, 0xf, true);   // row_shr:4
    v += __builtin_amdgcn_update_dpp(0, v, 0x118, 0xf, 0xf, true);   // row_shr:8
    v += __builtin_amdgcn_update_dpp(0, v, 0x142, 0xa, 0xf, false);  // row_bcast:15 into rows 1 and 3
    v += __builtin_amdgcn_update_dpp(0, v, 0x143, 0xc, 0xf, false);  // row_bcast:31 into rows 2 and 3
    return v;
}

// A place on the tile axis: tile t of pair (b, hkv); `flat` counts the tiles in front of it.
// The end of the axis is (B, 0, 0).
struct TilePos {
    int b, hkv, t, flat;
};
// First tile whose cost position is at or after v.
template <typename I>
__device__ inline TilePos locate(const AttnParams &p, const int *s_pref, I v) {
    TilePos r;
    if (v >= cost_total<I>(p, s_pref)) {
        r.b = p.B; r.hkv = 0; r.t = 0; r.flat = p.Hkv * s_pref[p.B];
        return r;
    }
    int lo = 0, hi = p.B - 1;
    while (lo < hi) {
        const int mid = (lo + hi + 1) >> 1;
        if ((I)p.Hkv * (s_pref[mid] + (I)mid * p.pair_cost) <= v) lo = mid; else hi = mid - 1;
    }
    const int b = lo, n_b = s_pref[b + 1] - s_pref[b];
    const int rel = (int)(v - (I)p.Hkv * (s_pref[b] + (I)b * p.pair_cost));   // < Hkv * (n_b + E)
    int hkv = rel / (n_b + p.pair_cost);
    hkv = hkv > p.Hkv - 1 ? p.Hkv - 1 : hkv;
    const int rr = rel - hkv * (n_b + p.pair_cost) - p.pair_front;
    r.b = b; r.hkv = hkv; r.t = rr > 0 ? (rr < n_b ? rr : n_b) : 0;
    r.flat = p.Hkv * s_pref[b] + hkv * n_b + r.t;
    if (r.t == n_b) {   // a position in the padding behind the pair's tiles: the next pair's first tile
        r.t = 0;
        if (++r.hkv == p.Hkv) { r.hkv = 0; ++r.b; }
    }
    return r;
}

__device__ inline u32x4 ld16(const void *ptr) { return *reinterpret_cast<const u32x4 *>(ptr); }
__device__ inline u32x4 keep_if(bool ok, u32x4 v) {
    v.x = ok ? v.x : 0u; v.y = ok ? v.y : 0u; v.z = ok ? v.z : 0u; v.w = ok ? v.w : 0u;
    return v;
}

// CW: wavefronts that copy tiles (each takes 64 / CW rows of every tile).
template <int D, int CW>
struct Geometry {
    static constexpr int kChunks = D / 8;                       // 16-byte chunks per K/V row
    static constexpr int kRowBytes = D * 2;
    static constexpr int kTileBytes = kTile * kRowBytes;        // one K (or V) tile in LDS
    static constexpr int kStageBytes = 2 * kTileBytes;          // K tile then V tile
    static constexpr int kRowsPerCopy = 1024 / kRowBytes;       // tile rows one wavefront copy instruction moves
    static constexpr int kRowsPerWave = kTile / CW;             // tile rows a copying wavefront moves per tile (8 or 16)
    static constexpr int kCopies = kRowsPerWave / kRowsPerCopy; // copy instructions per copying wavefront, per tile, for K and for V each
    static constexpr int kKSteps = D / 16;                      // MFMA k-steps of the QK product
    static constexpr int kOBlocks = D / 32;                     // 32-wide blocks of the output dim
};

// LDS has 64 four-byte banks.  The 16-byte chunks of a tile row are XOR-swizzled by the
// row index so that each pass of an operand read touches every bank once:
//  - a K fragment read (ds_read_b128) serves 16 lanes = 16 consecutive rows, same chunk;
//  - a V fragment read (ds_read_b64_tr_b16) serves 32 lanes = 4 consecutive rows x 4
//    adjacent chunks x both halves of a chunk.
// Rows are 256 bytes (D = 128, all banks) or 128 bytes (D = 64, half of the banks, so
// the row's parity already separates two rows).
template <int D> __device__ inline int swizzle_k(int row) { return D == 128 ? (row & 15) : ((row >> 1) & 7); }
template <int D> __device__ inline int swizzle_v(int row) {
    // only bits 0..2 of the row: fragment reads step through the tile in multiples of 8 rows
    return D == 128 ? (((row & 3) << 2) | ((row >> 2) & 1)) : (((row >> 1) & 1) << 2);
}

// One entry of a workgroup's tile list, kept in LDS.  The workgroup writes the list itself,
// up to kDescSlots tiles ahead of the tile being computed, so the main loop reads neither the
// sequence lengths nor the page table and spends no scalar work on finding its place.
struct TileDesc {
    int blk[4];    // prefix tile: page * Hkv + kv head of each 16-key quarter, -1 where the quarter
                   // reads as zeros; tree tile: all four = ((b * T + first node) * Hkv + kv head)
    int n_valid;   // rows of the tile that exist (1..64)
    int flags;     // kDesc* bits; from bit 8 up the number of the tree tile, or (kDescHoles) which quarters are missing
    int b;         // sequence
    int hkv;       // kv head
};
enum {
    kDescTree = 1,        // keys are tree nodes (masked by ancestor sets), else prefix positions
    kDescFresh = 2,       // first tile of a segment: new pair, or start of the workgroup's range
    kDescPairEnd = 4,     // last tile of its pair
    kDescMasks = 8,       // (on a fresh tile) the segment reaches the pair's tree tiles and needs its sequence's masks built
    kDescPairStart = 16,  // first tile of its pair
    kDescQ = 32,          // not a tile: the query rows of the segment that starts with the next item
    kDescHoles = 64,      // prefix tile with quarters behind a page id outside the pool: their keys are skipped
};
constexpr int kDescSlots = 256;

// Descriptor of tile idx of pair (b, hkv); it is tile i_tile of a range of n_tiles tiles.
// `table` is the page table or a copy of it in LDS (table_in_lds); `s_len` the clamped lengths in LDS, or null.
__device__ inline void write_tile_desc(const AttnParams &p, const int32_t *table, bool table_in_lds,
                                       const int32_t *__restrict__ seq_lens, const int *s_len, int b, int hkv, int idx,
                                       int i_tile, int n_tiles, TileDesc *slot, int &bad) {
    const int L = s_len ? s_len[b] : clamp_len(p, seq_lens, b);
    const int n_pre = (L + kTile - 1) / kTile, n_units = n_pre + p.n_tree_tiles;
    int blk[4], n_valid, flags = 0;
    if (idx < n_pre) {
        n_valid = min(kTile, L - idx * kTile);
        // The page ids of the quarters that hold rows, asked for together (one wait, not four) and
        // from the address space the table is in; position idx*64 + j*16 < L <= 16 * max_pages for
        // every quarter j <= j_last, so the reads stay inside the sequence's row of the table.
        const int j_last = (n_valid - 1) >> 4;
        const size_t at = (size_t)b * p.max_pages + idx * 4;
        int page[4];
        if (table_in_lds) {
            typedef __attribute__((address_space(3))) const int32_t lds_i32;
            lds_i32 *row = (lds_i32 *)table + at;
#pragma unroll
            for (int j = 0; j < 4; ++j) page[j] = j <= j_last ? row[j] : -1;
        } else {
            const int32_t *row = table + at;
#pragma unroll
            for (int j = 0; j < 4; ++j) page[j] = j <= j_last ? row[j] : -1;
        }
        int holes = 0;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            blk[j] = -1;
            if (j <= j_last) {
                if (page[j] >= 0 && page[j] < p.num_pages) blk[j] = page[j] * p.Hkv + hkv;
                else { bad |= READER_STATUS_BAD_PAGE; holes |= 1 << j; }
            }
        }
        if (holes) flags |= kDescHoles | (holes << 8);
    } else {
        const int tt = idx - n_pre;
        n_valid = min(kTile, p.T - tt * kTile);
        flags = kDescTree | (tt << 8);
        // rows of the tree tensors from (b, first node) on; with the tree in the cache: the pair
        blk[0] = blk[1] = blk[2] = blk[3] = p.tree_in_cache ? b * p.Hkv + hkv : (b * p.T + tt * kTile) * p.Hkv + hkv;
    }
    if (idx == 0) flags |= kDescPairStart;
    if (idx + 1 == n_units) flags |= kDescPairEnd;
    if (idx == 0 || i_tile == 0) {
        flags |= kDescFresh;
        // The ancestor masks belong to the sequence, not to the kv head: a segment that follows
        // another one of the same sequence in this range finds them in place (the one before it
        // ran to the end of its pair, through the tree tiles).
        if (idx + (n_tiles - i_tile) > n_pre && (i_tile == 0 || hkv == 0)) flags |= kDescMasks;
    }
    int4 *dst = reinterpret_cast<int4 *>(slot);
    dst[0] = make_int4(blk[0], blk[1], blk[2], blk[3]);
    dst[1] = make_int4(n_valid, flags, b, hkv);
}

// Item i of the list of a range of n_tiles tiles that starts at tile `start`.  The items are
// the tiles in order; with kWithQ every segment (the part of a pair inside the range) is
// preceded by one query unit: the pair's query rows, which travel through the ring like a
// tile.  The item is found by walking the pairs from the start of the range (a range holds
// few pairs unless the sequences are very short); i must be below the number of items.
template <bool kWithQ>
__device__ inline void build_item(const AttnParams &p, const int32_t *table, bool table_in_lds,
                                  const int32_t *__restrict__ seq_lens, const int *s_len, const int *s_pref,
                                  const TilePos &start, int n_tiles, int i, TileDesc *slot, int &bad) {
    int b = start.b, hkv = start.hkv, t = start.t, pos = i, tiles_before = 0;
    while (b < p.B) {
        if (kWithQ) {
            if (pos == 0) {
                int4 *dst = reinterpret_cast<int4 *>(slot);
                dst[0] = make_int4(-1, -1, -1, -1);
                dst[1] = make_int4(0, kDescQ, b, hkv);
                return;
            }
            --pos;
        }
        const int avail = s_pref[b + 1] - s_pref[b] - t;   // tiles of this pair from t on
        if (pos < avail) {
            write_tile_desc(p, table, table_in_lds, seq_lens, s_len, b, hkv, t + pos, tiles_before + pos, n_tiles, slot, bad);
            return;
        }
        pos -= avail;
        tiles_before += avail;
        t = 0;
        if (++hkv == p.Hkv) { hkv = 0; ++b; }
    }
}

// Asynchronous copy HBM -> LDS: lane l moves 16 bytes from its global address to LDS byte
// lds_base + 16 * l.  The compiler does not track these copies; the caller counts them
// (every wavefront issues the same number per tile) and waits with s_waitcnt vmcnt.
// The copies carry the non-temporal hint: K/V rows are read once per launch, and streamed
// that way the same loop moves about a sixth more bytes per second out of HBM (measured:
// 6.9 against 5.9 TB/s for a bare copy ring) while rows that are in the caches still hit.
__device__ inline void copy16_uniform(const void *sbase, unsigned lane_off, unsigned lds_base) {
    asm volatile("s_mov_b32 m0, %2\n\tglobal_load_lds_dwordx4 %0, %1 nt"
                 :: "v"(lane_off), "s"(sbase), "s"(lds_base) : "memory", "m0");
}
__device__ inline void copy16_lane(const void *addr, unsigned lds_base) {
    asm volatile("s_mov_b32 m0, %1\n\tglobal_load_lds_dwordx4 %0, off nt"
                 :: "v"(addr), "s"(lds_base) : "memory", "m0");
}

// Per-lane constants of the tile copy: byte offsets of this lane's 16 bytes inside a
// (page, head) block of the cache / inside a 64-row slab of the tree tensors, for each copy
// instruction, with the LDS swizzle already applied to the chunk index.
template <int D, int CW>
struct CopyLane {
    unsigned k_cache_off[Geometry<D, CW>::kCopies], v_cache_off[Geometry<D, CW>::kCopies];
    unsigned k_tree_off[Geometry<D, CW>::kCopies], v_tree_off[Geometry<D, CW>::kCopies];
    int row[Geometry<D, CW>::kCopies];   // tile row this lane copies
};

// cw: index of the copying wavefront (0 .. CW-1)
template <int D, int CW>
__device__ inline CopyLane<D, CW> make_copy_lane(const AttnParams &p, int cw, int lane) {
    using G = Geometry<D, CW>;
    CopyLane<D, CW> cl;
    const int rin = lane / G::kChunks, pchunk = lane % G::kChunks;   // row inside the copy, physical chunk
    const unsigned tree_row_bytes = (unsigned)p.Hkv * D * 2;
#pragma unroll
    for (int i = 0; i < G::kCopies; ++i) {
        const int r = cw * G::kRowsPerWave + i * G::kRowsPerCopy + rin;
        const unsigned kc = (unsigned)(pchunk ^ swizzle_k<D>(r)) << 4;
        const unsigned vc = (unsigned)(pchunk ^ swizzle_v<D>(r)) << 4;
        cl.row[i] = r;
        cl.k_cache_off[i] = (r & 15) * G::kRowBytes + kc;
        cl.v_cache_off[i] = (r & 15) * G::kRowBytes + vc;
        cl.k_tree_off[i] = r * tree_row_bytes + kc;
        cl.v_tree_off[i] = r * tree_row_bytes + vc;
    }
    return cl;
}

// What one copying wavefront needs for its rows of a tile: wave-uniform base addresses and
// which kind of source it is.  It issues exactly 2 * kCopies copy instructions per tile,
// whatever the tile looks like: rows that do not exist (past the sequence end, past the last
// tree node, behind an invalid page id) are copied from a block of zeros; their scores are masked
// before the softmax (rows past the end by the row count, quarters behind a bad page by the
// tile's kDescHoles bits) and the zero V rows keep the masked products finite.
struct CopyPlan {
    const char *kb, *vb;   // base of this wavefront's (page, head) block, or of the tree slab
    int n_valid;           // rows of the tile that exist
    bool whole;            // all rows of this wavefront exist in the paged cache: uniform fast path
    bool tree;
    bool page_ok;
};

template <int D, int CW>
__device__ inline CopyPlan plan_copy(const AttnParams &p, int blk, int n_valid, int flags, int cw) {
    using G = Geometry<D, CW>;
    CopyPlan cp;
    cp.n_valid = n_valid;
    cp.tree = (flags & kDescTree) != 0;
    cp.page_ok = blk >= 0;
    if (!cp.tree) {
        const size_t boff = (size_t)(cp.page_ok ? blk : 0) * (16 * G::kRowBytes);
        cp.kb = reinterpret_cast<const char *>(p.k_cache) + boff;
        cp.vb = reinterpret_cast<const char *>(p.v_cache) + boff;
        cp.whole = cp.page_ok && (cw + 1) * G::kRowsPerWave <= n_valid;
    } else {
        const size_t origin = (size_t)blk * G::kRowBytes;
        cp.kb = reinterpret_cast<const char *>(p.k_tree) + origin;
        cp.vb = reinterpret_cast<const char *>(p.v_tree) + origin;
        cp.whole = false;
        // without tree tensors (rows in the cache) the caller gathers through the page table instead;
        // should this plan be used all the same, every row reads as zeros and nothing is dereferenced
        if (p.tree_in_cache) cp.page_ok = false;
    }
    return cp;
}

// Copy instruction j of the tile (j < kCopies: K rows, else V rows) into the stage at LDS
// byte address `stage`.
template <int D, int CW>
__device__ inline void emit_copy(const CopyPlan &cp, const CopyLane<D, CW> &cl, unsigned stage, int cw, int j) {
    using G = Geometry<D, CW>;
    const bool is_v = j >= G::kCopies;
    const int i = is_v ? j - G::kCopies : j;
    const unsigned dst = stage + (is_v ? G::kTileBytes : 0) + cw * G::kRowsPerWave * G::kRowBytes + i * 1024;
    const char *base = is_v ? cp.vb : cp.kb;
    if (cp.whole) {
        copy16_uniform(base, is_v ? cl.v_cache_off[i] : cl.k_cache_off[i], dst);
    } else {
        const char *zeros = reinterpret_cast<const char *>(kZeroRow) + (threadIdx.x & 15) * 16;
        const bool ok = cp.page_ok && cl.row[i] < cp.n_valid;
        const unsigned off = cp.tree ? (is_v ? cl.v_tree_off[i] : cl.k_tree_off[i])
                                     : (is_v ? cl.v_cache_off[i] : cl.k_cache_off[i]);
        copy16_lane(ok ? base + off : zeros, dst);
    }
}

// s_waitcnt vmcnt(n) only (expcnt and lgkmcnt left alone), n < 64
template <int N>
__device__ inline void wait_vmcnt() {
    __builtin_amdgcn_s_waitcnt((N & 15) | ((N >> 4) << 14) | (7 << 4) | (15 << 8));
}

__device__ inline uint32_t pack_bf16x2(float lo, float hi) {
    typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
    bf16x2 v;
    v[0] = (__bf16)lo;
    v[1] = (__bf16)hi;
    return __builtin_bit_cast(uint32_t, v);
}

// Transposing LDS load of gfx950: within each group of 16 lanes the 16 x 4 block of
// 16-bit elements the lanes point at (lane k supplies 4 consecutive elements) is read
// as 4 rows of 16, and lane i receives element i of each row.
__device__ inline s16x4 lds_read_tr16(const char *ptr) {
    return __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4 *)(ptr));
}

// f(integral_constant<int, 0>), f(integral_constant<int, 1>), ...: a loop the compiler sees as straight-line
// code with compile-time indices (the fixed instruction order of a tile is written with it)
template <class F, int... I>
__device__ __forceinline__ void static_for_impl(F &&f, std::integer_sequence<int, I...>) {
    (f(std::integral_constant<int, I>{}), ...);
}
template <int N, class F>
__device__ __forceinline__ void static_for(F &&f) {
    static_for_impl(static_cast<F &&>(f), std::make_integer_sequence<int, N>{});
}

// What a range workgroup knows once it has found its place: its share [lo, hi) of the tile axis, where
// to read page ids from while the list is written, and the clamped lengths in LDS (or null).
struct RangeSetup {
    TilePos lo, hi;
    const int32_t *table;
    bool table_in_lds;
    int *s_len;
};

// Start of every range workgroup (NT threads, all of them call this): fetch a small page table into an
// idle ring stage (table_stage / table_stage_lds, stage_bytes large), scan the lengths into tile counts
// (s_pref, s_wsum in LDS) and find the workgroup's share of the cost axis.  On return the copy of the
// page table, if any, is complete and visible to the whole workgroup.
template <int NT>
__device__ __forceinline__ void setup_range(const AttnParams &p, const int32_t *__restrict__ page_table,
                                            const int32_t *__restrict__ seq_lens, char *table_stage,
                                            unsigned table_stage_lds, int stage_bytes, int *s_pref, int *s_wsum,
                                            int range_id, RangeSetup &rs) {
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave_s = __builtin_amdgcn_readfirstlane(tid >> 6);
    TilePos lo, hi;
    const int32_t *table;
    bool table_in_lds;
    int *s_len;
    // A small page table is fetched whole into the last ring stage (idle until the main loop
    // starts) while the sequence lengths are on their way, so that the tile list can be written
    // without a second trip to memory.
    const long long table_ints_all = (long long)p.B * p.max_pages;
    table_in_lds = table_ints_all * 4 + 256 <= (long long)stage_bytes;   // copies come in 256-byte pieces
    const int table_ints = table_in_lds ? (int)table_ints_all : 0;
    table = page_table;
    if (table_in_lds) {
        const unsigned table_lds = table_stage_lds;
        for (int base = wave_s * 64; base < table_ints; base += NT) {
            const int32_t *src = page_table + min(base + lane, table_ints - 1);
            asm volatile("s_mov_b32 m0, %1\n\tglobal_load_lds_dword %0, off" :: "v"(src), "s"(table_lds + base * 4) : "memory", "m0");
        }
        table = reinterpret_cast<const int32_t *>(table_stage);
    }

    // Tiles per sequence as prefix sums in LDS (and the clamped lengths, for up to 1024 sequences).
    // With at most 64 sequences every wavefront scans on its own and all of them write the
    // same values, so a wavefront may read them back without a barrier (its own LDS accesses
    // execute in order).
    s_len = p.B <= kMaxLensInLds ? s_pref + p.B + 1 : nullptr;
    if (p.B <= 64 && p.Hkv <= 64 && p.axis32) {
        int units = 0;
        if (lane < p.B) {
            const int L = clamp_len(p, seq_lens, lane);
            s_len[lane] = L;
            units = (L + kTile - 1) / kTile + p.n_tree_tiles;
        }
        const int v = wave_inclusive_scan(units);
        if (lane < p.B) s_pref[lane + 1] = v;
        if (lane == 0) s_pref[0] = 0;
        // This workgroup's tiles: [lo, hi) of the tile axis, an even share of the cost axis.  Lane b
        // holds sequence b's tile count and the tiles in front of it, so a place on the cost axis
        // is found with two votes (which sequence, which kv head) instead of searches and divisions;
        // what the chosen lane holds is read with a scalar lane index.
        const int excl = v - units;
        const int base = p.Hkv * (excl + lane * p.pair_cost);   // where sequence `lane` starts on the cost axis
        const int total = __builtin_amdgcn_readlane(v, 63);      // (lanes past the last sequence add nothing)
        const int cost_all = p.Hkv * (total + p.B * p.pair_cost);
        auto locate_by_vote = [&](int pos) {
            TilePos r;
            if (pos >= cost_all) {
                r.b = p.B; r.hkv = 0; r.t = 0; r.flat = p.Hkv * total;
                return r;
            }
            const int b = __builtin_amdgcn_readfirstlane(__popcll(__ballot(lane < p.B && base <= pos)) - 1);   // pos >= 0 = base of sequence 0
            const int span = __builtin_amdgcn_readlane(units, b) + p.pair_cost;   // cost positions per pair
            const int rel = pos - __builtin_amdgcn_readlane(base, b);
            const int hkv = __popcll(__ballot(lane < p.Hkv && lane * span <= rel)) - 1;
            const int rr = rel - hkv * span - p.pair_front, n_b = span - p.pair_cost;
            r.b = b; r.hkv = hkv; r.t = rr > 0 ? (rr < n_b ? rr : n_b) : 0;
            r.flat = p.Hkv * __builtin_amdgcn_readlane(excl, b) + hkv * n_b + r.t;
            if (r.t == n_b) {   // a position in the padding behind the pair's tiles: the next pair's first tile
                r.t = 0;
                if (++r.hkv == p.Hkv) { r.hkv = 0; ++r.b; }
            }
            return r;
        };
        auto cut = [&](int w) {   // where range w starts on the cost axis
            return p.ranges_shift >= 0 ? (int)(((unsigned)w * (unsigned)cost_all) >> p.ranges_shift)
                                       : range_begin<int>(w, cost_all, p.n_ranges);
        };
        lo = locate_by_vote(cut(range_id));
        hi = locate_by_vote(cut(range_id + 1));
    } else {
        if (p.B <= 64) {
            int v = 0;
            if (lane < p.B) {
                const int L = clamp_len(p, seq_lens, lane);
                s_len[lane] = L;
                v = (L + kTile - 1) / kTile + p.n_tree_tiles;
            }
#pragma unroll
            for (int off = 1; off < 64; off <<= 1) {
                const int t = __shfl_up(v, off);
                if (lane >= off) v += t;
            }
            if (lane < p.B) s_pref[lane + 1] = v;
            if (lane == 0) s_pref[0] = 0;
        } else {
            scan_units(p, seq_lens, s_pref, s_wsum, s_len);
        }
        // this workgroup's tiles: [lo, hi) of the tile axis, an even share of the cost axis
        if (p.axis32) {
            const int cost_all = cost_total<int>(p, s_pref);
            lo = locate<int>(p, s_pref, range_begin<int>(range_id, cost_all, p.n_ranges));
            hi = locate<int>(p, s_pref, range_begin<int>(range_id + 1, cost_all, p.n_ranges));
        } else {
            const long long cost_all = cost_total<long long>(p, s_pref);
            lo = locate<long long>(p, s_pref, range_begin<long long>(range_id, cost_all, p.n_ranges));
            hi = locate<long long>(p, s_pref, range_begin<long long>(range_id + 1, cost_all, p.n_ranges));
        }
    }
    lo.b = __builtin_amdgcn_readfirstlane(lo.b); lo.hkv = __builtin_amdgcn_readfirstlane(lo.hkv);
    lo.t = __builtin_amdgcn_readfirstlane(lo.t); lo.flat = __builtin_amdgcn_readfirstlane(lo.flat);
    hi.b = __builtin_amdgcn_readfirstlane(hi.b); hi.hkv = __builtin_amdgcn_readfirstlane(hi.hkv);
    hi.t = __builtin_amdgcn_readfirstlane(hi.t); hi.flat = __builtin_amdgcn_readfirstlane(hi.flat);
    if (table_in_lds) {
        wait_vmcnt<0>();
        __syncthreads();   // the copy of the page table is complete (every wavefront reaches this)
    }
    rs.lo = lo; rs.hi = hi; rs.table = table; rs.table_in_lds = table_in_lds; rs.s_len = s_len;
}

// For the merge kernel: which workgroups hold tiles of each pair that starts in this range (first =
// this one, last from the position of the pair's last tile).  Called by the first 256 threads.
__device__ __forceinline__ void write_pair_info(const AttnParams &p, const int *s_pref, const TilePos &lo,
                                                const TilePos &hi, int range_id, int tid) {
    const int first = lo.b * p.Hkv + lo.hkv + (lo.t > 0 ? 1 : 0);
    const int last = hi.b * p.Hkv + hi.hkv - (hi.t > 0 ? 0 : 1);
    for (int q = first + tid; q <= last && tid < 256; q += 256) {
        const int b = q / p.Hkv, hkv = q - b * p.Hkv, n_units = s_pref[b + 1] - s_pref[b];
        const int w_last =
            p.axis32 ? range_of_position<int>(cost_pos_of_tile<int>(p, s_pref, b, hkv, n_units - 1),
                                              cost_total<int>(p, s_pref), p.n_ranges)
                     : range_of_position<long long>(cost_pos_of_tile<long long>(p, s_pref, b, hkv, n_units - 1),
                                                    cost_total<long long>(p, s_pref), p.n_ranges);
        reinterpret_cast<int2 *>(p.pair_info)[q] = make_int2(range_id, w_last);
    }
}

}  // namespace

}  // namespace reader

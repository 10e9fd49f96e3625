// Tree-masked attention (Section 3.2 of the READER paper) for many query rows per kv head:
// the matrix-bound flavour of the main kernel.
//
// Same decomposition as tree_attn_mfma.hip (flat tile axis cut into ranges of equal cost, tile
// list in LDS, HBM -> LDS copies into a ring of tile buffers, partial records for pairs that are
// cut between workgroups), but a workgroup is 4 wavefronts, one per SIMD, and each wavefront
// carries 64 query rows (two blocks of 32): with the SIMD to itself a wavefront may use all 512
// vector registers, which is what 64 rows take (128 output accumulators, 64 score accumulators,
// 64 for the query rows' fragments, then operands and weights).  A K or V fragment read from
// LDS serves both row blocks, so a tile costs half the LDS operand traffic per matrix
// instruction of the 8 x 32-row layout, and one barrier covers twice the work.
//
// A wavefront has nobody to hide its waiting behind, so nothing in the tile may wait:
//   - the ring has 4 stages and tiles are asked for three tiles ahead;
//   - operand fragments are read from LDS ahead of the matrix instructions that use them;
//   - whole prefix tiles run as a software pipeline over two tiles: the scores of the next
//     tile, the products of the current one and, one per matrix instruction, the softmax
//     weights in between (a wavefront's vector instructions do issue under its own matrix
//     instructions when the two kinds alternate finely; in long runs of one kind they do not).
#include <hip/hip_ext.h>

#include <mutex>
#include <type_traits>
#include <utility>

#include "internal.h"
#include "tree_attn_common.h"

namespace reader {

namespace {
constexpr int kWideThreads = 256;   // 4 wavefronts
constexpr int kWideStages = 4;      // tile buffers in the ring
constexpr int kWideRows = 256;      // query rows per workgroup

// The accumulation registers (a0..a255 of every lane) are managed by hand in this kernel: the compiler is
// told never to use them (-amdgpu-spill-vgpr-to-agpr=0 and no operand of that class anywhere), the
// instructions below name them by number, and what they hold is invisible to the register allocator, which
// is left with the ~200 vector registers of scores, weights and operand fragments.  Layout per lane:
//   output accumulators O^T of row block r, output block db:  16 registers from o(r, db)
//   query fragment of row block r, k-step kk (B operand of the first product):  4 registers from q(r, kk)
template <int D>
struct AccMap {
    static constexpr int kOB = D / 32, kK = D / 16;
    static constexpr int o(int r, int db) { return (r * kOB + db) * 16; }
    static constexpr int q(int r, int kk) { return 2 * kOB * 16 + (r * kK + kk) * 4; }
    static constexpr int kCount = 2 * kOB * 16 + 2 * kK * 4;   // 192 (D = 128), 96 (D = 64)
    // ... and per-lane values that are needed once per tile or per segment, kept out of the vector
    // registers the pipelined tile code needs for itself (one instruction brings one back):
    static constexpr int kParked = kCount;
    static constexpr int node(int r) { return kParked + r; }            // tree node of the lane's row in row block r
    static constexpr int group(int r) { return kParked + 2 + r; }       // ... and its query head within the kv head
    static constexpr int m_ref(int r) { return kParked + 4 + r; }       // the row's softmax reference (a score, not yet scaled)
    static constexpr int k_off(int i) { return kParked + 6 + i; }       // byte offsets of the lane's part of copy i of a whole prefix tile (K, V)
    static constexpr int v_off(int i) { return kParked + 6 + D / 32 + i; }
    static constexpr int kEnd = kParked + 6 + 2 * (D / 32);
};
// Nothing here is known to the compiler as a matrix instruction, so the waits the hardware leaves to software
// are the caller's business: a result is read by the vector ALU (v_accvgpr_read, or any instruction on a
// score register) no sooner than 11 instructions after the matrix instruction that wrote it; a dependent
// matrix instruction on exactly the same accumulator needs none.
template <int LO> __device__ __forceinline__ void mfma_o(const bf16x8 &a, const bf16x8 &b) {   // a[LO..LO+15] += a . b
    asm volatile("v_mfma_f32_32x32x16_bf16 a[%c0:%c1], %2, %3, a[%c0:%c1]" :: "n"(LO), "n"(LO + 15), "v"(a), "v"(b));
}
template <int Q> __device__ __forceinline__ void mfma_s0(f32x16 &acc, const bf16x8 &k) {       // acc = k . a[Q..Q+3]
    asm volatile("v_mfma_f32_32x32x16_bf16 %0, %1, a[%c2:%c3], 0" : "=&v"(acc) : "v"(k), "n"(Q), "n"(Q + 3));
}
template <int Q> __device__ __forceinline__ void mfma_s(f32x16 &acc, const bf16x8 &k) {        // acc += k . a[Q..Q+3]
    asm volatile("v_mfma_f32_32x32x16_bf16 %0, %1, a[%c2:%c3], %0" : "+v"(acc) : "v"(k), "n"(Q), "n"(Q + 3));
}
template <int I> __device__ __forceinline__ void acc_write(uint32_t v) { asm volatile("v_accvgpr_write_b32 a%c0, %1" :: "n"(I), "v"(v)); }
template <int I> __device__ __forceinline__ void acc_zero() { asm volatile("v_accvgpr_write_b32 a%c0, 0" :: "n"(I)); }
template <int I> __device__ __forceinline__ float acc_read() {
    float x;
    asm volatile("v_accvgpr_read_b32 %0, a%c1" : "=v"(x) : "n"(I));
    return x;
}
template <int I> __device__ __forceinline__ uint32_t acc_read_u32() {
    uint32_t x;
    asm volatile("v_accvgpr_read_b32 %0, a%c1" : "=v"(x) : "n"(I));
    return x;
}
#define READER_RESULT_WAIT() asm volatile("s_nop 15")   /* 16 wait states: matrix result -> vector ALU */
}  // namespace

template <int D>
__global__ __launch_bounds__(kWideThreads) void tree_attn_wide_kernel(AttnParams p,
                                                                       const int32_t *__restrict__ page_table,
                                                                       const int32_t *__restrict__ seq_lens) {
    constexpr int CW = 4;                            // every wavefront copies a quarter (16 rows) of each tile
    using G = Geometry<D, CW>;
    constexpr int kCopiesPerTile = 2 * G::kCopies;   // per wavefront
    constexpr int kS = kWideStages;

    using Acc = AccMap<D>;
    // (for the kernel's register count: the accumulation registers up to the last one used by hand)
    static_assert(AccMap<128>::kEnd == 206 && AccMap<64>::kEnd == 106, "the register count below is the map's last register");
    if constexpr (D == 128) asm volatile("" ::: "a0", "a205");
    else asm volatile("" ::: "a0", "a105");

    extern __shared__ __attribute__((aligned(1024))) char smem[];
    char *ring = smem;                                                               // [kS][kStageBytes]
    uint32_t *s_anc = reinterpret_cast<uint32_t *>(smem + kS * G::kStageBytes);      // [READER_MAX_T][4]
    int *s_par = reinterpret_cast<int *>(s_anc + READER_MAX_T * 4);                  // [READER_MAX_T]
    float *s_sink = reinterpret_cast<float *>(s_par + READER_MAX_T);                 // [64] landing zone of cache-warming copies
    int *s_wsum = reinterpret_cast<int *>(s_sink + 64);                              // [8]
    TileDesc *s_desc = reinterpret_cast<TileDesc *>(s_wsum + 8);                     // [kDescSlots]
    int *s_pref = reinterpret_cast<int *>(s_desc + kDescSlots);                      // [B + 1], then the lengths
    const unsigned ring_lds = (unsigned)(size_t)(lds_char *)ring;
    const unsigned prefetch_lds = (unsigned)(size_t)(lds_char *)reinterpret_cast<char *>(s_sink);
    __shared__ int s_over;
    if (threadIdx.x == 0) s_over = 0;   // (the barriers of the set-up below come before anybody sets it)

    // 1-D grid; the row chunks of one range get ids 8 apart (same XCD, same time: the second one
    // finds the range's K/V tiles in that XCD's L2)
    int range_id, chunk_id;
    if (p.n_ranges % kNumXCD == 0) {
        const int per_group = kNumXCD * p.n_row_chunks, g = blockIdx.x / per_group, r = blockIdx.x - g * per_group;
        chunk_id = r / kNumXCD;
        range_id = g * kNumXCD + r % kNumXCD;
    } else {
        chunk_id = blockIdx.x / p.n_ranges;
        range_id = blockIdx.x - chunk_id * p.n_ranges;
    }
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave_s = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int cw = wave_s;
    const int n = lane & 31, h = lane >> 5;
    const int chunk_base = chunk_id * kWideRows;
    // the two row blocks of this wavefront
    int row_local[2];
    bool row_real[2];
    static_for<2>([&](auto rc) {
        constexpr int r = decltype(rc)::value;
        row_local[r] = wave_s * 64 + r * 32 + n;
        const int m_row = chunk_base + row_local[r];
        row_real[r] = m_row < p.M;
        const int node = row_real[r] ? m_row / p.G : 0;
        acc_write<Acc::node(r)>((uint32_t)node);
        acc_write<Acc::group(r)>((uint32_t)(row_real[r] ? m_row - node * p.G : 0));
    });
    auto node_of = [](auto rc) { return (int)acc_read_u32<Acc::node(decltype(rc)::value)>(); };
    auto group_of = [](auto rc) { return (int)acc_read_u32<Acc::group(decltype(rc)::value)>(); };
    const bool wave_active = chunk_base + wave_s * 64 < p.M;

    RangeSetup rs;
    setup_range<kWideThreads>(p, page_table, seq_lens, ring + (kS - 1) * G::kStageBytes,
                              ring_lds + (kS - 1) * G::kStageBytes, G::kStageBytes, s_pref, s_wsum, range_id, rs);
    const TilePos lo = rs.lo, hi = rs.hi;
    const int32_t *table = rs.table;
    const bool table_in_lds = rs.table_in_lds;
    int *s_len = rs.s_len;
    const int n_tiles = hi.flat - lo.flat;
    if (chunk_id == 0 && tid == 0) p.range_tiles[range_id] = n_tiles;
    if (n_tiles <= 0) {
        if (tid == 0) p.redo[blockIdx.x] = 0;
        return;
    }
    const int n_iter = n_tiles;

    int bad = 0;
    auto write_item = [&](int i) {
        const bool from_lds = table_in_lds && i < kDescSlots;   // (the stage that held the copy is in use later)
        build_item<false>(p, from_lds ? table : page_table, from_lds, seq_lens, s_len, s_pref, lo, n_tiles, i,
                          s_desc + (i & (kDescSlots - 1)), bad);
    };
    for (int i = tid; i < min(n_iter, kDescSlots); i += kWideThreads) write_item(i);
    __syncthreads();   // the list is written
    write_pair_info(p, s_pref, lo, hi, range_id, tid);

    auto desc_of = [&](int i) -> const TileDesc * { return s_desc + (i & (kDescSlots - 1)); };
    auto desc_b = [&](int i) { return __builtin_amdgcn_readfirstlane(desc_of(i)->b); };
    auto desc_hkv = [&](int i) { return __builtin_amdgcn_readfirstlane(desc_of(i)->hkv); };

    // The query rows of this lane (one per row block) as B operands of the first product: loaded once per
    // segment into the accumulation registers, where they stay.
    auto load_q = [&](int b, int hkv) {
        // (the rows of both row blocks are asked for before any is put away: one trip to memory, not two; the score
        // and weight registers are free at this point)
        u32x4 w[2][G::kKSteps];
        static_for<2>([&](auto rc) {
            constexpr int r = decltype(rc)::value;
            const uint16_t *qrow = p.q + (((size_t)b * p.T + node_of(rc)) * p.Hq + hkv * p.G + group_of(rc)) * D;
#pragma unroll
            for (int kk = 0; kk < G::kKSteps; ++kk) w[r][kk] = keep_if(row_real[r], ld16(qrow + kk * 16 + h * 8));
        });
        static_for<2>([&](auto rc) {
            constexpr int r = decltype(rc)::value;
            static_for<G::kKSteps>([&](auto kc) {
                constexpr int kk = decltype(kc)::value;
                acc_write<Acc::q(r, kk)>(w[r][kk].x);
                acc_write<Acc::q(r, kk) + 1>(w[r][kk].y);
                acc_write<Acc::q(r, kk) + 2>(w[r][kk].z);
                acc_write<Acc::q(r, kk) + 3>(w[r][kk].w);
            });
        });
        asm volatile("s_nop 3");
    };
    // touch the next pair's query rows one tile before they are needed, so that they wait in the
    // cache: an LDS copy of 4 bytes per lane into a scratch area nobody reads
    auto prefetch_q = [&](int b, int hkv) {
        static_for<2>([&](auto rc) {
            const uint16_t *qrow = p.q + (((size_t)b * p.T + node_of(rc)) * p.Hq + hkv * p.G + group_of(rc)) * D;
            const uint16_t *src = qrow + (h * 64) % D;
            const unsigned dst = prefetch_lds;
            asm volatile("s_mov_b32 m0, %1\n\tglobal_load_lds_dword %0, off" :: "v"(src), "s"(dst) : "memory", "m0");
        });
    };

    auto build_masks = [&]() {
        if (tid < p.T) {
            uint32_t a0 = 0u, a1 = 0u, a2 = 0u, a3 = 0u;
            int t = tid;
            for (int step = 0; step < p.T && t >= 0; ++step) {
                const uint32_t bit = 1u << (t & 31);
                const int w = t >> 5;
                a0 |= w == 0 ? bit : 0u; a1 |= w == 1 ? bit : 0u;
                a2 |= w == 2 ? bit : 0u; a3 |= w == 3 ? bit : 0u;
                int pi = s_par[t];
                const bool valid = t == 0 ? pi == -1 : (pi >= 0 && pi < t);
                if (!valid) { bad |= READER_STATUS_BAD_TREE; pi = -1; }
                t = pi;
            }
            uint32_t *dst = s_anc + tid * 4;
            dst[0] = a0; dst[1] = a1; dst[2] = a2; dst[3] = a3;
        }
    };

    // Per-lane byte offsets of the copies of a whole prefix tile (the common case, issued from inside the
    // tile code); everything else about a lane's copies is made again whenever a tile needs it, so that
    // it does not sit in registers through the main loop.
    {
        const CopyLane<D, CW> cl0 = make_copy_lane<D, CW>(p, cw, lane);
        static_for<G::kCopies>([&](auto ic) {
            constexpr int i = decltype(ic)::value;
            acc_write<Acc::k_off(i)>(cl0.k_cache_off[i]);
            acc_write<Acc::v_off(i)>(cl0.v_cache_off[i]);
        });
    }
    // Copies of this wavefront's 16 rows of a tile into the stage at LDS byte address stage_lds:
    // exactly kCopiesPerTile copy instructions, whatever the tile looks like.
    auto issue_tile = [&](int blk, int nv, int fl, unsigned stage_lds) {
        int lane_again = lane;
        asm volatile("" : "+v"(lane_again));   // (opaque: the constants below are not hoisted out of the loop)
        const CopyLane<D, CW> cl = make_copy_lane<D, CW>(p, cw, lane_again);
        if (p.tree_in_cache && (fl & kDescTree)) {
            // tree rows that live in the cache: row r of tree tile tt is position L + 64 tt + r, any
            // alignment to the pages, so every lane looks up the page of its row
            const int sb = blk / p.Hkv, shkv = blk - sb * p.Hkv;
            const int pos0 = (s_len ? s_len[sb] : clamp_len(p, seq_lens, sb)) + (fl >> 8) * kTile;
            const char *zeros = reinterpret_cast<const char *>(kZeroRow) + (lane_again & 15) * 16;
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
                const unsigned in_row = (unsigned)(row & 15) * G::kRowBytes;
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
    auto issue_tile_at = [&](int i) {
        const TileDesc *d = desc_of(i);
        issue_tile(__builtin_amdgcn_readfirstlane(d->blk[cw]), __builtin_amdgcn_readfirstlane(d->n_valid),
                   __builtin_amdgcn_readfirstlane(d->flags), ring_lds + ((unsigned)i % kS) * G::kStageBytes);
    };

    // prologue: the first kS - 1 tiles are put in flight
#pragma unroll
    for (int i = 0; i < kS - 1; ++i)
        if (i < n_iter) issue_tile_at(i);
    load_q(desc_b(0), desc_hkv(0));

    // per-lane LDS offsets of the operand reads (relative to the stage)
    int k_rd[G::kKSteps];   // K fragment of k-step kk, key block 0
#pragma unroll
    for (int kk = 0; kk < G::kKSteps; ++kk)
        k_rd[kk] = n * G::kRowBytes + (((2 * kk + h) ^ swizzle_k<D>(n)) << 4);
    int v_rd[G::kOBlocks];  // V fragment of output block db, keys 0..3 (+4h) of the first 16-key group
    {
        const int i16 = lane & 15, g16 = (lane >> 4) & 1;
        const int key_lo = 4 * h + (i16 >> 2);
        const int c_lo = 2 * g16 + ((i16 & 3) >> 1);
#pragma unroll
        for (int db = 0; db < G::kOBlocks; ++db)
            v_rd[db] = G::kTileBytes + key_lo * G::kRowBytes +
                       ((((db * 4) | c_lo) ^ swizzle_v<D>(key_lo)) << 4) + (i16 & 1) * 8;
    }

    float mc[2] = {0.f, 0.f};   // the rows' softmax references in the exp2 domain (the references themselves are parked)
    float lsum[2][2] = {{0.f, 0.f}, {0.f, 0.f}};   // per row block two partial sums of the segment's weights
    bool seg_from_pair_start = false;
    bool overflowed = false;              // a weight came out too large for the fixed reference: this workgroup's work is redone
    const float c2 = p.scale_log2;
    u32x4 pk[2][2][2];                    // [key block][row block][16-key step]: softmax weights as bf16 pairs, the B operands of the second product
    f32x16 s[2][2];                       // [key block][row block]: S^T of the current tile

    // The softmax reference of a row is fixed by the first tile of a segment (the row's maximum there)
    // and never moved afterwards: a lower reference only makes all weights of the row larger by one
    // factor, which fp32 sums and bf16 weights carry without loss (both have 8 exponent bits), so
    // the output accumulators are never rescaled, which would take them through the vector ALU's
    // registers.  A later score more than ~2^100 above the reference is the one thing this cannot
    // hold; it shows in the row's sum at the end of the segment, and the workgroup's whole range is
    // then computed again by the kernel that does move its reference (see the launch code).
    constexpr float kTooLarge = 0x1p100f;

    auto k_frag = [&](const char *stage, int kb, int kk) {
        return *reinterpret_cast<const bf16x8 *>(stage + k_rd[kk] + kb * 32 * G::kRowBytes);
    };
    // half `hf` of the V^T fragment of (16-key step ks, output block db): keys +0..3 (+4h) or +8..11 (+4h)
    auto v_half = [&](const char *stage, int ks, int db, int hf) {
        const int key_base = ((ks >> 1) * 32 + (ks & 1) * 16 + hf * 8) * G::kRowBytes;
        return lds_read_tr16(stage + v_rd[db] + key_base);
    };
    auto p_frag = [&](int kb, int r, int m2) { return __builtin_bit_cast(bf16x8, pk[kb][r][m2]); };
    // weights of scores i, i + 1 of block (kb, r) against the row's reference
    auto weight_pair = [&](int kb, int r, int i) {
        const float p0 = __builtin_amdgcn_exp2f(s[kb][r][i] * c2 - mc[r]);
        const float p1 = __builtin_amdgcn_exp2f(s[kb][r][i + 1] * c2 - mc[r]);
        lsum[r][0] += p0;
        lsum[r][1] += p1;
        pk[kb][r][i >> 3][(i >> 1) & 3] = pack_bf16x2(p0, p1);
    };
    // The weights of pipelined tiles are made one per matrix instruction slot, and as a pipeline of their own,
    // so that no instruction of a slot waits for another of the same slot: slot e takes the exponential
    // of the argument made in slot e - 1, makes the argument of weight e + 1, adds weight e - 1 to its
    // row's sum and, when e is even, packs weights e - 2 and e - 1.  Between slots:
    float w_x = 0.f;             // argument of the exponential of the slot's own weight
    float w_p1 = 0.f, w_p2 = 0.f;   // the weights of one and two slots ago
    auto weight_arg = [&](float score, float ref) {
        // (written out, so that it stays in the slot it is written in: the instruction selector moves
        // plain arithmetic freely within the unrolled tile, and bunches it up ahead of the matrix work)
        float x;
        asm volatile("v_fma_f32 %0, %1, %2, -%3" : "=v"(x) : "v"(score), "v"(c2), "v"(ref));
        return x;
    };
    // Slot e (0..31) of the half step that computes the weights of key block wkb; the block before it in
    // this order is the other key block (of the same tile for wkb = 1, of the tile before for wkb = 0).
    auto weight_slot = [&](auto wkbc, auto ec) {
        constexpr int wkb = decltype(wkbc)::value, e = decltype(ec)::value;
        // (written out for the same reason as the argument: left to the compiler the exponential moves up to just
        // behind the instruction that makes its argument, one slot earlier, and waits for it there)
        float p_cur;
        asm volatile("v_exp_f32 %0, %1" : "=v"(p_cur) : "v"(w_x));
        // the next argument: score e + 1 of this block, or score 0 of the other one (complete by now: its last
        // matrix instruction was issued at least two matrix instructions ago)
        constexpr int nb = e == 31 ? 1 - wkb : wkb, ne = (e + 1) & 31;
        w_x = weight_arg(s[nb][ne / 16][ne % 16], mc[ne / 16]);
        constexpr int pe = (e + 31) & 31;                     // the weight of one slot ago
        lsum[pe / 16][pe & 1] += w_p1;
        if constexpr ((e & 1) == 0) {
            constexpr int pb = e == 0 ? 1 - wkb : wkb, p2 = (e + 30) & 31, r = p2 / 16, i = p2 % 16;
            pk[pb][r][i >> 3][(i >> 1) & 3] = pack_bf16x2(w_p2, w_p1);
        }
        w_p2 = w_p1;
        w_p1 = p_cur;
    };

    // ---------------------------------------------------------------------------------------------
    // Whole prefix tiles that do not start a segment (no masks, no maxima) are run as a software
    // pipeline over two tiles.  A tile is handled in two half steps, one per block of 32 keys; half
    // step kb of tile t holds, interleaved:
    //   S(t+1, kb) = K.Q^T        2 kK matrix instructions, into the score registers of key block kb,
    //                             whose weights were taken in the half step before;
    //   O += V(t, kb)^T.P(t, kb)^T  4 kOB matrix instructions, with the weights made in the half step before;
    //   weights of the other key block: of (t, 1) in half step 0, of (t+1, 0) in half step 1, one
    //                             score per matrix instruction (a wavefront's vector instructions
    //                             run under its own matrix instructions only in the second half
    //                             of each, so a slot has room for about four of them).
    // Every operand fragment is read from LDS once, two groups of four matrix instructions ahead of
    // its use, and serves both row blocks back to back.
    auto v_frag = [&](const char *stage, int ks, int db) {
        return __builtin_shufflevector(v_half(stage, ks, db, 0), v_half(stage, ks, db, 1), 0, 1, 2, 3, 4, 5, 6, 7);
    };

    // S = K.Q^T of a tile
    auto scores = [&](const char *stage) {
        constexpr int kK = G::kKSteps;
        bf16x8 kf[3][2];
        kf[0][0] = k_frag(stage, 0, 0); kf[0][1] = k_frag(stage, 1, 0);
        kf[1][0] = k_frag(stage, 0, 1); kf[1][1] = k_frag(stage, 1, 1);
        static_for<kK>([&](auto kc) {
            constexpr int kk = decltype(kc)::value;
            if constexpr (kk + 2 < kK) { kf[(kk + 2) % 3][0] = k_frag(stage, 0, kk + 2); kf[(kk + 2) % 3][1] = k_frag(stage, 1, kk + 2); }
            static_for<4>([&](auto gc) {
                constexpr int kb = decltype(gc)::value >> 1, r = decltype(gc)::value & 1;
                if constexpr (kk == 0) mfma_s0<Acc::q(r, kk)>(s[kb][r], kf[kk % 3][kb]);
                else mfma_s<Acc::q(r, kk)>(s[kb][r], kf[kk % 3][kb]);
            });
        });
        READER_RESULT_WAIT();
    };
    // O^T += V^T.P^T of a tile whose weights are in pk: a V fragment serves both row blocks
    auto products = [&](const char *stage) {
        constexpr int kOB = G::kOBlocks;
        s16x4 vf[2][kOB][2];
#pragma unroll
        for (int db = 0; db < kOB; ++db) { vf[0][db][0] = v_half(stage, 0, db, 0); vf[0][db][1] = v_half(stage, 0, db, 1); }
        static_for<4>([&](auto kc) {
            constexpr int ks = decltype(kc)::value;
            if constexpr (ks + 1 < 4) {
#pragma unroll
                for (int db = 0; db < kOB; ++db) {
                    vf[(ks + 1) & 1][db][0] = v_half(stage, ks + 1, db, 0);
                    vf[(ks + 1) & 1][db][1] = v_half(stage, ks + 1, db, 1);
                }
            }
            static_for<2 * kOB>([&](auto jc) {
                constexpr int r = decltype(jc)::value / kOB, db = decltype(jc)::value % kOB;
                const s16x8 a8 = __builtin_shufflevector(vf[ks & 1][db][0], vf[ks & 1][db][1], 0, 1, 2, 3, 4, 5, 6, 7);
                mfma_o<Acc::o(r, db)>(__builtin_bit_cast(bf16x8, a8), p_frag(ks >> 1, r, ks & 1));
            });
        });
    };
    auto weights_of_key_block = [&](int kb) {
#pragma unroll
        for (int r = 0; r < 2; ++r)
#pragma unroll
            for (int i = 0; i < 16; i += 2) weight_pair(kb, r, i);
        asm volatile("s_nop 3");   // (weights written by the vector ALU are matrix operands next)
    };
    // Start of a run of whole tiles: the weights of key block 0, left the way slot 31 of a pipelined tile leaves them
    // (the last weight not yet added to its sum, the last pair not yet packed, the next argument made).
    auto begin_run = [&]() {
#pragma unroll
        for (int r = 0; r < 2; ++r)
#pragma unroll
            for (int i = 0; i < (r == 0 ? 16 : 14); i += 2) weight_pair(0, r, i);
        w_p2 = __builtin_amdgcn_exp2f(s[0][1][14] * c2 - mc[1]);
        w_p1 = __builtin_amdgcn_exp2f(s[0][1][15] * c2 - mc[1]);
        lsum[1][0] += w_p2;
        w_x = weight_arg(s[1][0][0], mc[0]);
    };
    // End of a run: what slot 0 of a further pipelined tile would have done with key block 0
    auto end_run = [&]() {
        lsum[1][1] += w_p1;
        pk[0][1][1][3] = pack_bf16x2(w_p2, w_p1);
    };

    // One pipelined tile: products and key-block-1 weights of the tile in `stage`, scores and
    // key-block-0 weights of the next tile in `next_stage`.  with_copy: the copies of a whole prefix
    // tile (base addresses kbase / vbase, LDS address copy_stage_lds) are issued on the way.
    auto tile_pipelined = [&](auto with_copy, const char *stage, const char *next_stage, const char *kbase, const char *vbase,
                              unsigned copy_stage_lds) {
        constexpr int kK = G::kKSteps, kOB = G::kOBlocks;
        static_assert(kK == 2 * kOB, "a half step has as many score as product instructions");
        bf16x8 kf[3];
        s16x8 vf[3];
        // fragments of group g of half step kb: K rows of key block kb, k-step g; V^T of 16-key step 2 kb + g / kOB, output block g % kOB
        auto load_group = [&](auto kbc, auto gc) {
            constexpr int kb = decltype(kbc)::value, g = decltype(gc)::value;
            kf[(kb * kK + g) % 3] = k_frag(next_stage, kb, g);
            vf[(kb * kK + g) % 3] = v_frag(stage, 2 * kb + g / kOB, g % kOB);
        };
        load_group(std::integral_constant<int, 0>{}, std::integral_constant<int, 0>{});
        load_group(std::integral_constant<int, 0>{}, std::integral_constant<int, 1>{});
        __builtin_amdgcn_sched_barrier(0);
        static_for<2 * kK>([&](auto gg) {
            constexpr int kb = decltype(gg)::value / kK, g = decltype(gg)::value % kK;
            // two groups ahead, into the registers the group before this one has left
            if constexpr (g + 2 < kK) load_group(std::integral_constant<int, kb>{}, std::integral_constant<int, g + 2>{});
            else if constexpr (kb == 0) load_group(std::integral_constant<int, 1>{}, std::integral_constant<int, g + 2 - kK>{});
            static_for<4>([&](auto mc4) {
                constexpr int m = decltype(mc4)::value, j = g * 4 + m;      // slot j of 4 kK in this half step
                // Half step 0: P S P S (the first K fragment is the last to arrive); half step 1: S S P P.  Either
                // way the last score instruction of row block 0 is followed by at least two more matrix
                // instructions before the vector ALU, in the last slot of the half step, reads the first of those
                // scores: a result needs 11 issue slots after its instruction before it may be read.
                constexpr bool is_p = kb == 0 ? (m & 1) == 0 : m >= 2;
                constexpr int r = kb == 0 ? m >> 1 : m & 1;
                constexpr int w3 = (kb * kK + g) % 3;                        // this group's place in the window of three
                if constexpr (is_p) {
                    mfma_o<Acc::o(r, g % kOB)>(__builtin_bit_cast(bf16x8, vf[w3]), p_frag(kb, r, g / kOB));
                } else {
                    if constexpr (g == 0) mfma_s0<Acc::q(r, g)>(s[kb][r], kf[w3]);
                    else mfma_s<Acc::q(r, g)>(s[kb][r], kf[w3]);
                }
                // Copies of the tile three ahead: spread evenly over the tile, so that the copy instructions reach
                // the memory pipeline as a trickle: issued together they fill its queue, and a wavefront that
                // waits there issues no matrix instructions either.
                if constexpr (decltype(with_copy)::value) {
                    constexpr int J = kb * 4 * kK + j, kSpacing = 8 * kK / kCopiesPerTile;
                    if constexpr (J % kSpacing == 1) {
                        constexpr int c = J / kSpacing;
                        constexpr bool is_v = c >= G::kCopies;
                        constexpr int i = is_v ? c - G::kCopies : c;
                        copy16_uniform(is_v ? vbase : kbase, acc_read_u32<is_v ? Acc::v_off(i) : Acc::k_off(i)>(),
                                       copy_stage_lds + (is_v ? G::kTileBytes : 0) + cw * G::kRowsPerWave * G::kRowBytes + i * 1024);
                    }
                }
                // weights of the other key block (of the next tile in half step 1), 32 scores over 4 kK slots
                constexpr int lo = j * 32 / (4 * kK), hi = (j + 1) * 32 / (4 * kK);
                static_for<hi - lo>([&](auto ic) { weight_slot(std::integral_constant<int, 1 - kb>{}, std::integral_constant<int, lo + decltype(ic)::value>{}); });
                __builtin_amdgcn_sched_barrier(0);
            });
        });
    };

    // Any tile, one step after the other: scores, masks, (first tile of a segment) row maxima,
    // weights, products.
    auto tile_plain = [&](const char *stage, int flags, int n_valid) {
        constexpr int kK = G::kKSteps, kOB = G::kOBlocks;
        const bool is_tree = (flags & kDescTree) != 0;
        const bool first = (flags & kDescFresh) != 0;
        const int tt = flags >> 8;
        const int holes = (flags & kDescHoles) ? (flags >> 8) & 15 : 0;   // quarters of a prefix tile to skip
        scores(stage);

        // keep(kb, r, i): does score i of block (kb, r) belong to a key this row attends to
        auto softmax = [&](auto &&keep) {
#pragma unroll
            for (int r = 0; r < 2; ++r) {
                // the keys the row does not attend to get -inf (weight 0)
#pragma unroll
                for (int kb = 0; kb < 2; ++kb)
#pragma unroll
                    for (int i = 0; i < 16; ++i) s[kb][r][i] = keep(kb, r, i) ? s[kb][r][i] : -INFINITY;
                if (first) {
                    // the row's maximum over the tile is its reference for the whole segment
                    float mx = fmaxf(s[0][r][0], s[1][r][0]);
#pragma unroll
                    for (int i = 1; i < 16; ++i) mx = fmaxf(fmaxf(mx, s[0][r][i]), s[1][r][i]);
                    // the other half of the row's keys sits in lane ^ 32
                    const auto sw = __builtin_amdgcn_permlane32_swap(__float_as_uint(mx), __float_as_uint(mx), false, false);
                    mx = fmaxf(__uint_as_float(sw[0]), __uint_as_float(sw[1]));
                    // (a row whose every key was skipped because of bad page ids gets a finite, very low reference)
                    const float ref = holes ? fmaxf(mx, -1e30f) : mx;
                    if (r == 0) acc_write<Acc::m_ref(0)>(__float_as_uint(ref));
                    else acc_write<Acc::m_ref(1)>(__float_as_uint(ref));
                    mc[r] = (ref == -INFINITY) ? 0.f : ref * c2;
                }
#pragma unroll
                for (int kb = 0; kb < 2; ++kb)
#pragma unroll
                    for (int i = 0; i < 16; i += 2) weight_pair(kb, r, i);
            }
        };
        if (is_tree) {
            uint32_t bits[2][2];
            static_for<2>([&](auto rc) {
                constexpr int r = decltype(rc)::value;
                const int nd = node_of(rc);
#pragma unroll
                for (int kb = 0; kb < 2; ++kb) bits[kb][r] = (row_real[r] ? s_anc[nd * 4 + tt * 2 + kb] : 0u) >> (4 * h);
            });
            // score i of a block is key (i / 4) * 8 + 4 h + i % 4 of its 32 keys (the 4 h is shifted out above)
            softmax([&](int kb, int r, int i) { return ((bits[kb][r] >> ((i >> 2) * 8 + (i & 3))) & 1u) != 0; });
        } else if (n_valid < kTile || holes) {
            // score i of block kb is key kb * 32 + (i / 4) * 8 + 4 h + i % 4; the lane's part of that is made here,
            // out of the compiler's sight, or 64 key numbers would wait in registers through the whole main loop
            int lim = n_valid - 4 * h;
            asm volatile("" : "+v"(lim));
            softmax([&](int kb, int, int i) {
                return kb * 32 + (i >> 2) * 8 + (i & 3) < lim && !((holes >> (kb * 2 + (i >> 3))) & 1);
            });
        } else {
            softmax([](int, int, int) { return true; });
        }
        asm volatile("s_nop 3");   // (weights written by the vector ALU are matrix operands next)

        products(stage);
    };

    auto reset_state = [&](int flags) {
        seg_from_pair_start = (flags & kDescPairStart) != 0;
#pragma unroll
        for (int r = 0; r < 2; ++r) {
            if (r == 0) acc_write<Acc::m_ref(0)>(__float_as_uint(-INFINITY));
            else acc_write<Acc::m_ref(1)>(__float_as_uint(-INFINITY));
            mc[r] = 0.f;
            lsum[r][0] = lsum[r][1] = 0.f;
        }
        static_for<2 * G::kOBlocks * 16>([&](auto ic) { acc_zero<decltype(ic)::value>(); });   // the output accumulators
    };

    // End of a segment (its pair ends, or the range does): a pair this workgroup saw from its first
    // to its last tile is normalised and written out, anything else leaves a partial record.
    auto finish_segment = [&](int it, bool pair_ends) {
        const int e_b = desc_b(it), e_hkv = desc_hkv(it);
        READER_RESULT_WAIT();   // the last products of the segment are about to be read by the vector ALU
        static_for<2>([&](auto rc) {
            constexpr int R = decltype(rc)::value;
            const int r = R;
            const float l_mine = lsum[r][0] + lsum[r][1];
            const float l_tot = l_mine + __shfl_xor(l_mine, 32);
            if (__any(!(l_tot < kTooLarge))) overflowed = true;   // (also an infinite or undefined sum)
            const bool whole = seg_from_pair_start && pair_ends;
            const float inv = whole ? 1.f / l_tot : (l_tot > 0.f ? 1.f / l_tot : 0.f);   // (a row may see no key of a part)
            const int nd = node_of(rc), gr = group_of(rc);
            const float ref = __uint_as_float(acc_read_u32<Acc::m_ref(R)>());
            uint16_t *orow = p.out + (((size_t)e_b * p.T + nd) * p.Hq + e_hkv * p.G + gr) * D;
            const size_t slot = ((size_t)(2 * range_id + (seg_from_pair_start ? 1 : 0)) * p.n_row_chunks + chunk_id);
            float *rec = p.workspace + slot * attn_slot_floats(D, kWideRows);
            u32x4 *rec16 = reinterpret_cast<u32x4 *>(rec);
            // A lane holds, per 8-wide chunk of the output row, 4 values and its partner lane (lane ^ 32)
            // the other 4: one half-wave swap per pair of chunks gives every lane whole 16-byte chunks.
            static_for<G::kOBlocks * 2>([&](auto cc) {
                constexpr int db = decltype(cc)::value / 2, i4 = (decltype(cc)::value % 2) * 2;
                float v[8];
                static_for<8>([&](auto ec) { v[decltype(ec)::value] = acc_read<Acc::o(R, db) + 4 * i4 + decltype(ec)::value>() * inv; });
                const uint32_t a0 = pack_bf16x2(v[0], v[1]), a1 = pack_bf16x2(v[2], v[3]);
                const uint32_t b0 = pack_bf16x2(v[4], v[5]), b1 = pack_bf16x2(v[6], v[7]);
                const auto s0 = __builtin_amdgcn_permlane32_swap(a0, b0, false, false);
                const auto s1 = __builtin_amdgcn_permlane32_swap(a1, b1, false, false);
                u32x4 w;
                w.x = s0[0]; w.y = s1[0]; w.z = s0[1]; w.w = s1[1];
                if (whole) {
                    if (row_real[r]) *reinterpret_cast<u32x4 *>(orow + db * 32 + (i4 + h) * 8) = w;
                } else {
                    // [D / 8 chunks][rows][8 values], then the rows' references, then their sums
                    rec16[(size_t)(db * 4 + i4 + h) * kWideRows + row_local[r]] = w;
                }
            });
            if (whole) {
                if (row_real[r] && p.lse && h == 0)
                    p.lse[((size_t)e_b * p.Hq + e_hkv * p.G + gr) * p.T + nd] = (ref * c2 + __builtin_amdgcn_logf(l_tot)) * kLn2;
            } else if (h == 0) {
                float *ml = rec + (size_t)kWideRows * (D / 2);
                ml[row_local[r]] = ref * c2;
                ml[kWideRows + row_local[r]] = l_tot;
            }
        });
    };

    auto extend_list = [&](int it) {
        if ((it & (kDescSlots / 2 - 1)) == 0 && it > 0 && tid < kDescSlots / 2) {
            const int i = it + kDescSlots / 2 + tid;
            if (i < n_iter) write_item(i);
        }
    };

    // descriptor words (rows, flags) of the tile to compute and of the one after it, and of the tile to copy,
    // read ahead so that the LDS latency hides behind the barrier
    int2 d_cur = *reinterpret_cast<const int2 *>(&desc_of(0)->n_valid);
    int2 d_nxt = *reinterpret_cast<const int2 *>(&desc_of(1)->n_valid);
    int2 d_cpy = *reinterpret_cast<const int2 *>(&desc_of(kS - 1)->n_valid);
    int d_blk = desc_of(kS - 1)->blk[cw];
    // (integer arithmetic on purpose: conditions kept as booleans become 64-bit lane masks and pairs of
    // compare/select instructions, and this runs once per tile on the only wavefront of its SIMD)
    auto is_whole = [](int valid, int flags) { return ((valid ^ kTile) | (flags & (kDescTree | kDescFresh | kDescHoles))) == 0; };

    // What every iteration starts with, whichever tile code follows: wait for the tiles, barrier, the tile
    // list, the copies of the tile three ahead (unless they go inside a pipelined tile).
    struct Iter {
        int t_valid, t_flags;          // the tile to compute
        int c_blk;                     // first page block of the tile to copy (this wavefront's rows), or -1
        unsigned copy_stage_lds;
        bool last_iter, pair_ends, whole, pipelined, copy_inside;
    };
    auto begin_iteration = [&](int it) {
        Iter I;
        I.t_valid = __builtin_amdgcn_readfirstlane(d_cur.x);
        I.t_flags = __builtin_amdgcn_readfirstlane(d_cur.y);
        const int n_valid = __builtin_amdgcn_readfirstlane(d_nxt.x);
        const int n_flags = __builtin_amdgcn_readfirstlane(d_nxt.y);
        const int c_valid = __builtin_amdgcn_readfirstlane(d_cpy.x);
        const int c_flags = __builtin_amdgcn_readfirstlane(d_cpy.y);
        I.c_blk = __builtin_amdgcn_readfirstlane(d_blk);
        I.last_iter = it + 1 == n_iter;
        I.pair_ends = (I.t_flags & kDescPairEnd) != 0;

        // Tiles up to it + 1 have to be complete in LDS (the pipelined tile code reads the next tile's K):
        // this wavefront's copies of them have landed once at most those of tile it + 2 are outstanding.
        if (it + 2 < n_iter) wait_vmcnt<kCopiesPerTile>();
        else wait_vmcnt<0>();
        __syncthreads();   // tiles it and it + 1 are complete in LDS; every wavefront is done with tile it - 1

        d_cur = d_nxt;
        d_nxt = *reinterpret_cast<const int2 *>(&desc_of(it + 2)->n_valid);
        d_cpy = *reinterpret_cast<const int2 *>(&desc_of(it + kS)->n_valid);
        d_blk = desc_of(it + kS)->blk[cw];
        extend_list(it);

        // Tile it + kS - 1 goes into the stage that tile it - 1 has left.  A whole prefix tile copied
        // behind a pipelined tile has its copy instructions spread over that tile's matrix instructions;
        // every other tile is asked for here.
        const bool copy_next = it + kS - 1 < n_iter;
        I.copy_stage_lds = ring_lds + ((unsigned)(it + kS - 1) % kS) * G::kStageBytes;
        I.whole = is_whole(I.t_valid, I.t_flags);
        I.pipelined = wave_active && I.whole && !I.last_iter && is_whole(n_valid, n_flags);
        const bool whole_next = I.c_blk >= 0 && !(c_flags & kDescTree) && (cw + 1) * G::kRowsPerWave <= c_valid;
        I.copy_inside = copy_next && I.pipelined && whole_next;
        if (copy_next && !I.copy_inside) issue_tile(I.c_blk, c_valid, c_flags, I.copy_stage_lds);
        if (I.pair_ends && !I.last_iter) prefetch_q(desc_b(it + 1), desc_hkv(it + 1));
        return I;
    };
    auto stage_of = [&](int it) { return ring + ((unsigned)it % kS) * G::kStageBytes; };   // (unsigned: a mask, not a signed remainder)

    for (int it = 0; it < n_iter; ++it) {
        Iter I = begin_iteration(it);
        if (I.t_flags & kDescFresh) {
            reset_state(I.t_flags);
            const int sb = desc_b(it);
            if (it != 0) load_q(sb, desc_hkv(it));
            // ancestor-or-self masks of this sequence's tree, if this segment reaches its tree tiles
            if (I.t_flags & kDescMasks) {
                if (tid < p.T) s_par[tid] = p.parents[(size_t)sb * p.T + tid];
                __syncthreads();
                build_masks();
                __syncthreads();
            }
        }
        if (!wave_active) continue;
        if (!I.whole) {
            tile_plain(stage_of(it), I.t_flags, I.t_valid);
        } else {
            // A run of whole tiles.  All but its last tile are pipelined, in a loop of their own: the
            // registers of scores and weights then pass from tile to tile without meeting another path
            // (where paths meet, the compiler moves every one of them into place with a copy).
            scores(stage_of(it));
            begin_run();
            while (I.pipelined) {
                const size_t boff = (size_t)(I.c_blk >= 0 ? I.c_blk : 0) * (16 * G::kRowBytes);
                const char *kbase = reinterpret_cast<const char *>(p.k_cache) + boff;
                const char *vbase = reinterpret_cast<const char *>(p.v_cache) + boff;
                if (I.copy_inside) tile_pipelined(std::true_type{}, stage_of(it), stage_of(it + 1), kbase, vbase, I.copy_stage_lds);
                else tile_pipelined(std::false_type{}, stage_of(it), stage_of(it + 1), kbase, vbase, I.copy_stage_lds);
                ++it;
                I = begin_iteration(it);    // (a whole tile that starts no segment: nothing else to prepare)
            }
            end_run();
            weights_of_key_block(1);
            products(stage_of(it));
        }
        if (I.pair_ends || I.last_iter) finish_segment(it, I.pair_ends);
    }

    // one word per workgroup, written every time: 1 asks for this workgroup's range to be computed again
    if (overflowed) s_over = 1;
    __syncthreads();
    if (tid == 0) p.redo[blockIdx.x] = s_over;
    if (p.status && bad) atomicOr(p.status, bad);
}

template <int D>
static hipError_t launch_wide(const AttnParams &p, hipStream_t stream, hipEvent_t ev_start, hipEvent_t ev_stop) {
    using G = Geometry<D, 4>;
    const size_t pref_bytes = ((size_t)(p.B + 1) * sizeof(int) + 15) & ~(size_t)15;
    const size_t main_lds = (size_t)kWideStages * G::kStageBytes + READER_MAX_T * 4 * sizeof(uint32_t) +
                            READER_MAX_T * sizeof(int) + 64 * sizeof(float) + 8 * sizeof(int) +
                            kDescSlots * sizeof(TileDesc) + pref_bytes +
                            (p.B <= kMaxLensInLds ? (size_t)p.B * sizeof(int) + 16 : 0);
    {
        static std::mutex guard;             // host threads may call in at the same time
        static size_t lds_allowed = 0;
        std::lock_guard<std::mutex> lock(guard);
        if (main_lds > lds_allowed) {
            hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(&tree_attn_wide_kernel<D>),
                                               hipFuncAttributeMaxDynamicSharedMemorySize, (int)main_lds);
            if (e != hipSuccess) { (void)hipGetLastError(); return note_hip_error("hipFuncSetAttribute(wide attention LDS size)", e); }
            lds_allowed = main_lds;
        }
    }
    if (ev_start && ev_stop)
        hipExtLaunchKernelGGL((tree_attn_wide_kernel<D>), dim3(p.n_ranges * p.n_row_chunks), dim3(kWideThreads), main_lds,
                              stream, ev_start, ev_stop, 0, p, p.page_table, p.seq_lens);
    else
        hipLaunchKernelGGL((tree_attn_wide_kernel<D>), dim3(p.n_ranges * p.n_row_chunks), dim3(kWideThreads), main_lds,
                           stream, p, p.page_table, p.seq_lens);
    return note_hip_error("launch tree_attn_wide_kernel", hipGetLastError());
}

hipError_t launch_tree_attn_wide_main(const AttnParams &p, hipStream_t stream, hipEvent_t ev_start, hipEvent_t ev_stop) {
    return p.D == 64 ? launch_wide<64>(p, stream, ev_start, ev_stop) : launch_wide<128>(p, stream, ev_start, ev_stop);
}

}  // namespace reader

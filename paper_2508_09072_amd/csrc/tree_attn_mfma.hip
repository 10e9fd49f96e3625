// Tree-masked attention on the gfx950 matrix cores (Section 3.2 of the READER paper).
//
// Work decomposition
//   A "pair" is (sequence b, kv head).  Its keys are cut into 64-key tiles: first the
//   prefix tiles (paged cache, mask-free except for the ragged last one), then the
//   tree tiles (the T tree rows, masked by ancestor-or-self bit masks held in LDS).
//   All tiles of all pairs form one flat axis of U units.  The grid has n_ranges
//   workgroups along x; workgroup w streams the contiguous unit range
//   [w*U/n_ranges, (w+1)*U/n_ranges), so every workgroup moves the same number of
//   K/V bytes whatever the ragged sequence lengths are.  A range may cover several
//   whole pairs and at most one pair at each end in part.  Whole pairs are finished
//   in place; a pair cut between workgroups leaves one partial record (unnormalised
//   output, running max, running sum) per workgroup and a second kernel merges them.
//   blockIdx.y selects a chunk of 128 query rows when T*G > 128.
//
// One workgroup = 4 wavefronts; wavefront w owns 32 query rows (a row is a
// (tree node, grouped query head) pair, so one K/V tile serves all heads of the
// group and all tree nodes).  Per tile, per wavefront:
//     S^T[64 keys][32 rows] = K_tile . Q^T        16 x v_mfma_f32_32x32x16_bf16 (D = 128)
//     online softmax down the key axis: the 32 scores a lane holds all belong to
//     one query row, so the row max is 31 in-lane max ops and one cross-lane swap
//     O^T[D][32 rows] += V_tile^T . P^T           16 x v_mfma_f32_32x32x16_bf16
//   The S^T accumulator layout of the first product is exactly the B-operand
//   layout the second one needs, up to a fixed permutation of the 64 keys of the
//   tile; V is stored transposed in LDS under that same permutation, so the
//   softmax weights never leave the registers.
//
// K/V tiles go HBM -> registers (128-bit loads, issued one tile ahead) -> LDS
// (double buffered, XOR-swizzled 16-byte chunks, one barrier per tile).
#include "internal.h"

namespace reader {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

namespace {

constexpr float kLn2 = 0.69314718055994530942f;

// Position along the flat unit axis: which pair, which tile of it.
struct Cursor {
    int b, hkv, idx;      // idx: unit index inside the pair
    int n_pre, n_units;   // prefix tiles / all tiles of this pair
    int L;                // clamped prefix length of sequence b
};

__device__ inline int clamp_len(const AttnParams &p, int b) {
    int L = p.seq_lens[b];
    L = L < 0 ? 0 : L;
    return L > p.max_seq_len ? p.max_seq_len : L;
}

__device__ inline void cursor_enter_seq(Cursor &c, const AttnParams &p) {
    c.L = clamp_len(p, c.b);
    c.n_pre = (c.L + kTile - 1) / kTile;
    c.n_units = c.n_pre + p.n_tree_tiles;
}

__device__ inline void cursor_advance(Cursor &c, const AttnParams &p) {
    if (++c.idx == c.n_units) {
        c.idx = 0;
        if (++c.hkv == p.Hkv) {
            c.hkv = 0;
            ++c.b;
            if (c.b < p.B) cursor_enter_seq(c, p);
        }
    }
}

// Exclusive prefix sums of tiles-per-pair over the sequences, into s_pref[0..B].
__device__ inline void scan_units(const AttnParams &p, int *s_pref, int *s_wsum) {
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    int carry = 0;
    if (tid == 0) s_pref[0] = 0;
    for (int base = 0; base < p.B; base += kThreads) {
        const int b = base + tid;
        int v = 0;
        if (b < p.B) v = (clamp_len(p, b) + kTile - 1) / kTile + p.n_tree_tiles;
#pragma unroll
        for (int off = 1; off < 64; off <<= 1) {
            const int t = __shfl_up(v, off);
            if (lane >= off) v += t;
        }
        if (lane == 63) s_wsum[wave] = v;
        __syncthreads();
        int woff = 0;
        for (int w = 0; w < wave; ++w) woff += s_wsum[w];
        const int total = s_wsum[0] + s_wsum[1] + s_wsum[2] + s_wsum[3];
        if (b < p.B) s_pref[b + 1] = carry + woff + v;
        carry += total;
        __syncthreads();
    }
}

// Largest b in [0, B) with Hkv * s_pref[b] <= x   (x < Hkv * s_pref[B]).
__device__ inline int find_seq(const int *s_pref, int B, int Hkv, long long x) {
    int lo = 0, hi = B - 1;
    while (lo < hi) {
        const int mid = (lo + hi + 1) >> 1;
        if ((long long)Hkv * s_pref[mid] <= x) lo = mid; else hi = mid - 1;
    }
    return lo;
}

__device__ inline long long range_begin(long long w, long long U, int n_ranges) { return w * U / n_ranges; }

// Workgroup whose range contains unit x.
__device__ inline int range_of_unit(long long x, long long U, int n_ranges) {
    long long w = ((x + 1) * n_ranges - 1) / U;
    if (w >= n_ranges) w = n_ranges - 1;
    while (w + 1 < n_ranges && range_begin(w + 1, U, n_ranges) <= x) ++w;
    while (w > 0 && range_begin(w, U, n_ranges) > x) --w;
    return (int)w;
}

// 16 bytes as a native vector (selects and copies of it stay in registers)
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
__device__ inline u32x4 ld16(const void *ptr) { return *reinterpret_cast<const u32x4 *>(ptr); }
__device__ inline u32x4 keep_if(bool ok, u32x4 v) {
    v.x = ok ? v.x : 0u; v.y = ok ? v.y : 0u; v.z = ok ? v.z : 0u; v.w = ok ? v.w : 0u;
    return v;
}

template <int D>
struct Geometry {
    static constexpr int kChunks = D / 8;                       // 16-byte chunks per K/V row
    static constexpr int kRowBytes = D * 2;
    static constexpr int kTileBytes = kTile * kRowBytes;        // one K (or V) tile in LDS
    static constexpr int kBufBytes = 2 * kTileBytes;            // K tile then V tile
    static constexpr int kKeysPerPass = kThreads / kChunks;     // keys one load instruction of the workgroup covers
    static constexpr int kLoads = kTile / kKeysPerPass;         // loads per thread per tile, for K and for V each
    static constexpr int kKSteps = D / 16;                      // MFMA k-steps of the QK product
    static constexpr int kOBlocks = D / 32;                     // 32-wide blocks of the output dim
};

// 16-byte chunks of a row are XOR-swizzled by the row index so that the matrix-core
// operand reads below touch every LDS bank once.  K is read 16 bytes per lane from 8
// consecutive rows; V is read through the transposing 8-byte load from 4 consecutive
// rows, two adjacent chunks each, hence the different bit order.
__device__ inline int swizzle_k(int row) { return row & 7; }
__device__ inline int swizzle_v(int row) { return ((row & 3) << 1) | ((row >> 2) & 1); }

// Registers a thread holds for the tile that is in flight from HBM.
template <int D>
struct Staged {
    u32x4 k[Geometry<D>::kLoads];
    u32x4 v[Geometry<D>::kLoads];
    unsigned real;   // bit i: load i fetched an existing row (others are written to LDS as zeros)
};

// Issue the global loads of one unit: a wave-uniform base address per load instruction
// plus one 32-bit lane offset.  Rows that do not exist (past the sequence end, past the
// last tree node, behind an invalid page id) read a harmless valid address and are
// replaced by zeros when they are written to LDS: a zero K row is masked later, a zero V
// row contributes nothing.
template <int D>
__device__ inline void issue_loads(const AttnParams &p, const Cursor &c, Staged<D> &st, int &bad) {
    using G = Geometry<D>;
    const int tid = threadIdx.x;
    const int wave_s = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int key0 = tid / G::kChunks, chunk = tid % G::kChunks;   // this thread's key in pass 0
    st.real = 0u;
    if (c.idx < c.n_pre) {
        const int base = c.idx * kTile;
        const int n_valid = min(kTile, c.L - base);
        const int32_t *pt = p.page_table + (size_t)c.b * p.max_pages + (base >> 4);
        int pg[4];
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            pg[j] = -1;
            if (16 * j < n_valid) {
                const int v = pt[j];
                if (v >= 0 && v < p.num_pages) pg[j] = v; else bad |= READER_STATUS_BAD_PAGE;
            }
        }
        const size_t page_stride = (size_t)p.Hkv * 16 * D;           // elements
        const size_t head_off = (size_t)c.hkv * 16 * D;
        const unsigned voff = ((key0 & 15) * D + chunk * 8) * 2;      // bytes inside the (page, head) block
#pragma unroll
        for (int i = 0; i < G::kLoads; ++i) {
            const int pj = i * (G::kKeysPerPass / 16) + (wave_s * 64 / G::kChunks) / 16;   // wave-uniform
            const int page = pj == 0 ? pg[0] : pj == 1 ? pg[1] : pj == 2 ? pg[2] : pg[3];
            const bool ok = page >= 0 && key0 + i * G::kKeysPerPass < n_valid;
            const size_t eoff = (size_t)(page >= 0 ? page : 0) * page_stride + head_off;
            const unsigned vo = ok ? voff : 0u;
            st.k[i] = ld16(reinterpret_cast<const char *>(p.k_cache + eoff) + vo);
            st.v[i] = ld16(reinterpret_cast<const char *>(p.v_cache + eoff) + vo);
            st.real |= ok ? (1u << i) : 0u;
        }
    } else {
        const int base = (c.idx - c.n_pre) * kTile;
        const int n_valid = min(kTile, p.T - base);
        const unsigned row_bytes = (unsigned)p.Hkv * D * 2;
        const size_t origin = (((size_t)c.b * p.T + base) * p.Hkv + c.hkv) * D;
#pragma unroll
        for (int i = 0; i < G::kLoads; ++i) {
            const int key = key0 + i * G::kKeysPerPass;
            const bool ok = key < n_valid;
            const unsigned vo = ok ? (unsigned)key * row_bytes + chunk * 16 : 0u;
            st.k[i] = ld16(reinterpret_cast<const char *>(p.k_tree + origin) + vo);
            st.v[i] = ld16(reinterpret_cast<const char *>(p.v_tree + origin) + vo);
            st.real |= ok ? (1u << i) : 0u;
        }
    }
}

// Staged registers -> LDS, both tiles row-major with swizzled 16-byte chunks.
template <int D>
__device__ inline void write_stage(const Staged<D> &st, char *k_lds, char *v_lds) {
    using G = Geometry<D>;
    const int tid = threadIdx.x;
    const int key0 = tid / G::kChunks, chunk = tid % G::kChunks;
    // kKeysPerPass is a multiple of 8, so the swizzle of a thread's row is the same in every pass
    const int koff = key0 * G::kRowBytes + ((chunk ^ swizzle_k(key0)) << 4);
    const int voff = key0 * G::kRowBytes + ((chunk ^ swizzle_v(key0)) << 4);
#pragma unroll
    for (int i = 0; i < G::kLoads; ++i) {
        const bool real = (st.real >> i) & 1u;
        *reinterpret_cast<u32x4 *>(k_lds + koff + i * G::kKeysPerPass * G::kRowBytes) = keep_if(real, st.k[i]);
        *reinterpret_cast<u32x4 *>(v_lds + voff + i * G::kKeysPerPass * G::kRowBytes) = keep_if(real, st.v[i]);
    }
}

__device__ inline uint32_t pack_bf16x2(float lo, float hi) {
    typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
    bf16x2 v;
    v[0] = (__bf16)lo;
    v[1] = (__bf16)hi;
    return __builtin_bit_cast(uint32_t, v);
}

typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef __attribute__((address_space(3))) s16x4 lds_s16x4;

// Transposing LDS load of gfx950: within each group of 16 lanes the 16 x 4 block of
// 16-bit elements the lanes point at (lane k supplies 4 consecutive elements) is read
// as 4 rows of 16, and lane i receives element i of each row.
__device__ inline s16x4 lds_read_tr16(const char *ptr) {
    return __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4 *)(ptr));
}

}  // namespace

template <int D>
__global__ __launch_bounds__(kThreads, 2) void tree_attn_mfma_kernel(AttnParams p) {
    using G = Geometry<D>;
    extern __shared__ __attribute__((aligned(16))) char smem[];
    char *buf0 = smem;
    char *buf1 = smem + G::kBufBytes;
    uint32_t *s_anc = reinterpret_cast<uint32_t *>(smem + 2 * G::kBufBytes);   // [READER_MAX_T][4]
    int *s_par = reinterpret_cast<int *>(s_anc + READER_MAX_T * 4);            // [READER_MAX_T]
    int *s_wsum = s_par + READER_MAX_T;                                        // [4]
    int *s_pref = s_wsum + 4;                                                  // [B + 1]

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int n = lane & 31, h = lane >> 5;
    const int chunk_base = blockIdx.y * kRowsPerWG;
    const int row_local = wave * 32 + n;           // row inside this workgroup's chunk
    const int m_row = chunk_base + row_local;      // query row inside the pair
    const bool row_real = m_row < p.M;
    const int node = row_real ? m_row / p.G : 0;   // tree node of this lane's query row
    const int group = row_real ? m_row - node * p.G : 0;
    const bool wave_active = chunk_base + wave * 32 < p.M;

    scan_units(p, s_pref, s_wsum);
    const long long U = (long long)p.Hkv * s_pref[p.B];
    const long long lo = range_begin(blockIdx.x, U, p.n_ranges);
    const long long hi = range_begin(blockIdx.x + 1, U, p.n_ranges);
    if (lo >= hi) return;
    const int n_iter = (int)(hi - lo);

    Cursor cc;   // unit being computed; every field is wave-uniform and kept in scalar registers
    cc.b = __builtin_amdgcn_readfirstlane(find_seq(s_pref, p.B, p.Hkv, lo));
    cursor_enter_seq(cc, p);
    {
        const long long rel = lo - (long long)p.Hkv * s_pref[cc.b];
        const int hkv = (int)(rel / cc.n_units);
        cc.hkv = __builtin_amdgcn_readfirstlane(hkv);
        cc.idx = __builtin_amdgcn_readfirstlane((int)(rel - (long long)hkv * cc.n_units));
    }
    Cursor lc = cc;   // unit being loaded (one ahead)

    int bad = 0;
    Staged<D> st;
    issue_loads<D>(p, lc, st, bad);
    write_stage<D>(st, buf0, buf0 + G::kTileBytes);
    cursor_advance(lc, p);
    __syncthreads();

    // per-lane LDS offsets of the matrix-core operand reads
    int k_rd[4];   // K fragment of k-step kk: k_rd[kk & 3] + (kk >> 2) * 128 (+ 32 rows for the second key block)
#pragma unroll
    for (int kk = 0; kk < 4; ++kk) k_rd[kk] = n * G::kRowBytes + (((2 * kk + h) ^ swizzle_k(n)) << 4);
    int v_rd[2];   // V fragment of output block db: v_rd[db & 1] + (db >> 1) * 128 (+ key rows)
    {
        const int i16 = lane & 15, g16 = (lane >> 4) & 1;
        const int key_lo = 4 * h + (i16 >> 2);                       // key row inside an 8-key group
        const int c_lo = 2 * g16 + ((i16 & 3) >> 1);                 // 16-byte chunk inside the 32-wide d block
#pragma unroll
        for (int db = 0; db < 2; ++db)
            v_rd[db] = key_lo * G::kRowBytes + ((((db * 4) | c_lo) ^ swizzle_v(key_lo)) << 4) + (i16 & 1) * 8;
    }

    bf16x8 qf[G::kKSteps];
    f32x16 o[G::kOBlocks];
    float m_run = -INFINITY, l_run = 0.f;
    bool fresh = true;                 // the next unit starts a segment (new pair or range start)
    bool seg_from_pair_start = false;
    const float c2 = p.scale_log2;

    for (int it = 0; it < n_iter; ++it) {
        char *k_lds = (it & 1) ? buf1 : buf0;
        char *v_lds = k_lds + G::kTileBytes;
        const bool more = it + 1 < n_iter;

        if (fresh) {
            fresh = false;
            seg_from_pair_start = (cc.idx == 0);
            m_run = -INFINITY;
            l_run = 0.f;
#pragma unroll
            for (int db = 0; db < G::kOBlocks; ++db)
#pragma unroll
                for (int i = 0; i < 16; ++i) o[db][i] = 0.f;
            // this lane's query row as the B operand of the QK product
            const uint16_t *qrow = p.q + (((size_t)cc.b * p.T + node) * p.Hq + cc.hkv * p.G + group) * D;
#pragma unroll
            for (int kk = 0; kk < G::kKSteps; ++kk) {
                qf[kk] = __builtin_bit_cast(bf16x8, keep_if(row_real, ld16(qrow + kk * 16 + h * 8)));
            }
            // ancestor-or-self masks of this sequence's tree, if this segment reaches its tree tiles
            if (cc.idx + (n_iter - it) > cc.n_pre) {
                __syncthreads();   // previous users of s_anc / s_par are done
                if (tid < p.T) {
                    int pi = p.parents[(size_t)cc.b * p.T + tid];
                    const bool valid = tid == 0 ? pi == -1 : (pi >= 0 && pi < tid);
                    if (!valid) { bad |= READER_STATUS_BAD_TREE; pi = -1; }
                    s_par[tid] = pi;
                }
                __syncthreads();
                if (tid < p.T) {
                    uint32_t a[4] = {0u, 0u, 0u, 0u};
                    int t = tid;
                    for (int step = 0; step < p.T && t >= 0; ++step) {
                        a[t >> 5] |= 1u << (t & 31);
                        t = s_par[t];
                    }
#pragma unroll
                    for (int w = 0; w < 4; ++w) s_anc[tid * 4 + w] = a[w];
                }
                __syncthreads();
            }
        }

        if (more) issue_loads<D>(p, lc, st, bad);

        if (wave_active) {
            // ---- S^T = K . Q^T : two 32-key blocks ----
            // All fragment reads of a block are issued before its first matrix instruction,
            // and the second block's reads are interleaved with the first block's products.
            f32x16 s[2];
            bf16x8 ka[2][G::kKSteps];
#pragma unroll
            for (int kb = 0; kb < 2; ++kb)
#pragma unroll
                for (int kk = 0; kk < G::kKSteps; ++kk)
                    ka[kb][kk] = *reinterpret_cast<const bf16x8 *>(
                        k_lds + k_rd[kk & 3] + (kk >> 2) * 128 + kb * 32 * G::kRowBytes);
#pragma unroll
            for (int kb = 0; kb < 2; ++kb) {
#pragma unroll
                for (int i = 0; i < 16; ++i) s[kb][i] = 0.f;
#pragma unroll
                for (int kk = 0; kk < G::kKSteps; ++kk)
                    s[kb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ka[kb][kk], qf[kk], s[kb], 0, 0, 0);
            }
            __builtin_amdgcn_sched_group_barrier(0x100, G::kKSteps, 0);          // LDS reads of block 0
#pragma unroll
            for (int kk = 0; kk < G::kKSteps; ++kk) {
                __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);               // one product of block 0
                __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);               // one read of block 1
            }
            __builtin_amdgcn_sched_group_barrier(0x008, G::kKSteps, 0);          // products of block 1
            // ---- masks: ragged last prefix tile, tree tiles ----
            const bool is_tree = cc.idx >= cc.n_pre;
            if (is_tree) {
                const int tt = cc.idx - cc.n_pre;
#pragma unroll
                for (int kb = 0; kb < 2; ++kb) {
                    uint32_t bits = row_real ? s_anc[node * 4 + tt * 2 + kb] : 0u;
                    bits >>= 4 * h;
#pragma unroll
                    for (int i = 0; i < 16; ++i) {
                        const int r = (i >> 2) * 8 + (i & 3);    // + 4h, already shifted out
                        if (!((bits >> r) & 1u)) s[kb][i] = -INFINITY;
                    }
                }
            } else if ((cc.idx + 1) * kTile > cc.L) {
                const int n_valid = cc.L - cc.idx * kTile;
#pragma unroll
                for (int kb = 0; kb < 2; ++kb)
#pragma unroll
                    for (int i = 0; i < 16; ++i) {
                        const int key = kb * 32 + (i >> 2) * 8 + 4 * h + (i & 3);
                        if (key >= n_valid) s[kb][i] = -INFINITY;
                    }
            }
            // ---- online softmax along the keys (all 32 values of a lane share one query row) ----
            float mx = s[0][0];
#pragma unroll
            for (int kb = 0; kb < 2; ++kb)
#pragma unroll
                for (int i = 0; i < 16; ++i) mx = fmaxf(mx, s[kb][i]);
            mx = fmaxf(mx, __shfl_xor(mx, 32));
            const float m_new = fmaxf(m_run, mx);
            const float m_eff = (m_new == -INFINITY) ? 0.f : m_new;
            const float alpha = __builtin_amdgcn_exp2f((m_run - m_eff) * c2);
            m_run = m_new;
            const float mc = m_eff * c2;
            float lsum = 0.f;
            uint32_t pk[2][8];
#pragma unroll
            for (int kb = 0; kb < 2; ++kb)
#pragma unroll
                for (int i = 0; i < 16; i += 2) {
                    const float p0 = __builtin_amdgcn_exp2f(s[kb][i] * c2 - mc);
                    const float p1 = __builtin_amdgcn_exp2f(s[kb][i + 1] * c2 - mc);
                    lsum += p0 + p1;
                    pk[kb][i >> 1] = pack_bf16x2(p0, p1);
                }
            l_run = l_run * alpha + lsum;
            if (__any(alpha != 1.f)) {
#pragma unroll
                for (int db = 0; db < G::kOBlocks; ++db)
#pragma unroll
                    for (int i = 0; i < 16; ++i) o[db][i] *= alpha;
            }
            // ---- O^T += V^T . P^T : the S^T registers of a lane are, 8 at a time, the B operand ----
#pragma unroll
            for (int ks = 0; ks < 4; ++ks) {
                const int kb = ks >> 1, m2 = ks & 1;
                u32x4 pv;
                pv.x = pk[kb][4 * m2]; pv.y = pk[kb][4 * m2 + 1]; pv.z = pk[kb][4 * m2 + 2]; pv.w = pk[kb][4 * m2 + 3];
                const bf16x8 pb = __builtin_bit_cast(bf16x8, pv);
                const int key_base = (kb * 32 + m2 * 16) * G::kRowBytes;
#pragma unroll
                for (int db = 0; db < G::kOBlocks; ++db) {
                    const char *src = v_lds + v_rd[db & 1] + (db >> 1) * 128 + key_base;
                    const s16x4 lo4 = lds_read_tr16(src);                         // keys +0..3 (+4h)
                    const s16x4 hi4 = lds_read_tr16(src + 8 * G::kRowBytes);      // keys +8..11 (+4h)
                    typedef short s16x8 __attribute__((ext_vector_type(8)));
                    const s16x8 a8 = __builtin_shufflevector(lo4, hi4, 0, 1, 2, 3, 4, 5, 6, 7);
                    o[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a8), pb, o[db], 0, 0, 0);
                }
            }
        }

        // ---- end of a segment: this pair ends here, or the range does ----
        const bool pair_ends = cc.idx + 1 == cc.n_units;
        if (pair_ends || !more) {
            if (wave_active) {
                const float l_tot = l_run + __shfl_xor(l_run, 32);
                if (seg_from_pair_start && pair_ends) {
                    if (row_real) {
                        const float inv = 1.f / l_tot;
                        uint16_t *orow = p.out + (((size_t)cc.b * p.T + node) * p.Hq + cc.hkv * p.G + group) * D;
#pragma unroll
                        for (int db = 0; db < G::kOBlocks; ++db)
#pragma unroll
                            for (int i4 = 0; i4 < 4; ++i4) {
                                uint2 w;
                                w.x = pack_bf16x2(o[db][4 * i4] * inv, o[db][4 * i4 + 1] * inv);
                                w.y = pack_bf16x2(o[db][4 * i4 + 2] * inv, o[db][4 * i4 + 3] * inv);
                                *reinterpret_cast<uint2 *>(orow + db * 32 + i4 * 8 + 4 * h) = w;
                            }
                        if (p.lse && h == 0)
                            p.lse[((size_t)cc.b * p.Hq + cc.hkv * p.G + group) * p.T + node] =
                                (m_run * c2 + __builtin_amdgcn_logf(l_tot)) * kLn2;
                    }
                } else {
                    const size_t slot = ((size_t)(2 * blockIdx.x + (seg_from_pair_start ? 1 : 0)) * p.n_row_chunks + blockIdx.y);
                    float *rec = p.workspace + slot * attn_slot_floats(D);
                    float *orow = rec + (size_t)row_local * D;
#pragma unroll
                    for (int db = 0; db < G::kOBlocks; ++db)
#pragma unroll
                        for (int i4 = 0; i4 < 4; ++i4)
                            *reinterpret_cast<float4 *>(orow + db * 32 + i4 * 8 + 4 * h) =
                                make_float4(o[db][4 * i4], o[db][4 * i4 + 1], o[db][4 * i4 + 2], o[db][4 * i4 + 3]);
                    if (h == 0) {
                        rec[(size_t)kRowsPerWG * D + row_local] = m_run * c2;
                        rec[(size_t)kRowsPerWG * (D + 1) + row_local] = l_tot;
                    }
                }
            }
            fresh = true;
        }

        if (more) {
            char *nk = (it & 1) ? buf0 : buf1;
            write_stage<D>(st, nk, nk + G::kTileBytes);
            cursor_advance(lc, p);
        }
        cursor_advance(cc, p);
        __syncthreads();
    }

    if (p.status && bad) atomicOr(p.status, bad);
}

// Merge the partial records of every pair that was cut between workgroups.
// grid = (B * Hkv, row chunks); 2 threads per query row, each half of D.
template <int D>
__global__ __launch_bounds__(kThreads) void tree_attn_merge_kernel(AttnParams p) {
    extern __shared__ __attribute__((aligned(16))) char smem[];
    int *s_pref = reinterpret_cast<int *>(smem);
    __shared__ int s_wsum[4];
    scan_units(p, s_pref, s_wsum);

    const int pair = blockIdx.x, b = pair / p.Hkv, hkv = pair - b * p.Hkv;
    const int n_units = s_pref[b + 1] - s_pref[b];
    const long long U = (long long)p.Hkv * s_pref[p.B];
    const long long start = (long long)p.Hkv * s_pref[b] + (long long)hkv * n_units;
    const int w_first = range_of_unit(start, U, p.n_ranges);
    const int w_last = range_of_unit(start + n_units - 1, U, p.n_ranges);
    if (w_first == w_last) return;   // finished in place by one workgroup

    const int tid = threadIdx.x;
    const int row_local = tid >> 1, half = tid & 1;
    const int m_row = blockIdx.y * kRowsPerWG + row_local;
    if (m_row >= p.M) return;
    const int node = m_row / p.G, group = m_row - node * p.G;
    const size_t rec_floats = attn_slot_floats(D);

    // Ranges that hold no unit (more workgroups than units) wrote no record.
    auto empty = [&](int w) { return range_begin(w, U, p.n_ranges) >= range_begin(w + 1, U, p.n_ranges); };
    auto record = [&](int w) -> const float * {
        const size_t slot = ((size_t)(2 * w + (w == w_first ? 1 : 0)) * p.n_row_chunks + blockIdx.y);
        return p.workspace + slot * rec_floats;
    };

    float m_all = -INFINITY;
    for (int w = w_first; w <= w_last; ++w)
        if (!empty(w)) m_all = fmaxf(m_all, record(w)[(size_t)kRowsPerWG * D + row_local]);
    // m_all is finite: every query row sees at least its own tree node

    constexpr int kHalf = D / 2;
    float acc[kHalf];
#pragma unroll
    for (int d = 0; d < kHalf; ++d) acc[d] = 0.f;
    float l_all = 0.f;
    for (int w = w_first; w <= w_last; ++w) {
        if (empty(w)) continue;
        const float *rec = record(w);
        const float mw = rec[(size_t)kRowsPerWG * D + row_local];
        if (mw == -INFINITY) continue;
        const float f = __builtin_amdgcn_exp2f(mw - m_all);
        l_all += f * rec[(size_t)kRowsPerWG * (D + 1) + row_local];
        const float4 *src = reinterpret_cast<const float4 *>(rec + (size_t)row_local * D + half * kHalf);
#pragma unroll
        for (int d4 = 0; d4 < kHalf / 4; ++d4) {
            const float4 v = src[d4];
            acc[4 * d4] += f * v.x; acc[4 * d4 + 1] += f * v.y;
            acc[4 * d4 + 2] += f * v.z; acc[4 * d4 + 3] += f * v.w;
        }
    }
    const float inv = 1.f / l_all;
    uint16_t *orow = p.out + (((size_t)b * p.T + node) * p.Hq + hkv * p.G + group) * D + half * kHalf;
#pragma unroll
    for (int d8 = 0; d8 < kHalf / 8; ++d8) {
        uint4 w;
        w.x = pack_bf16x2(acc[8 * d8] * inv, acc[8 * d8 + 1] * inv);
        w.y = pack_bf16x2(acc[8 * d8 + 2] * inv, acc[8 * d8 + 3] * inv);
        w.z = pack_bf16x2(acc[8 * d8 + 4] * inv, acc[8 * d8 + 5] * inv);
        w.w = pack_bf16x2(acc[8 * d8 + 6] * inv, acc[8 * d8 + 7] * inv);
        *reinterpret_cast<uint4 *>(orow + 8 * d8) = w;
    }
    if (p.lse && half == 0)
        p.lse[((size_t)b * p.Hq + hkv * p.G + group) * p.T + node] = (m_all + __builtin_amdgcn_logf(l_all)) * kLn2;
}

template <int D>
static hipError_t launch_mfma(const AttnParams &p, hipStream_t stream, hipEvent_t ev_start, hipEvent_t ev_stop) {
    using G = Geometry<D>;
    const size_t pref_bytes = ((size_t)(p.B + 1) * sizeof(int) + 15) & ~(size_t)15;
    const size_t main_lds = 2 * (size_t)G::kBufBytes + READER_MAX_T * 4 * sizeof(uint32_t) +
                            READER_MAX_T * sizeof(int) + 4 * sizeof(int) + pref_bytes;
    // More than 64 KB of LDS per workgroup has to be asked for; the limit counts the
    // kernel's static LDS too, so ask for exactly what this launch needs.
    static size_t lds_allowed = 0;
    if (main_lds > lds_allowed) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(&tree_attn_mfma_kernel<D>),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, (int)main_lds);
        if (e != hipSuccess) { (void)hipGetLastError(); return note_hip_error("hipFuncSetAttribute(attention LDS size)", e); }
        lds_allowed = main_lds;
    }
    if (ev_start) (void)hipEventRecord(ev_start, stream);
    hipLaunchKernelGGL(tree_attn_mfma_kernel<D>, dim3(p.n_ranges, p.n_row_chunks), dim3(kThreads),
                       main_lds, stream, p);
    hipError_t e = hipGetLastError();
    if (ev_stop) (void)hipEventRecord(ev_stop, stream);
    if (e != hipSuccess) return note_hip_error("launch tree_attn_mfma_kernel", e);
    hipLaunchKernelGGL(tree_attn_merge_kernel<D>, dim3(p.B * p.Hkv, p.n_row_chunks), dim3(kThreads),
                       pref_bytes, stream, p);
    return note_hip_error("launch tree_attn_merge_kernel", hipGetLastError());
}

hipError_t launch_tree_attn_mfma(const AttnParams &p, hipStream_t stream, hipEvent_t ev_start, hipEvent_t ev_stop) {
    return p.D == 64 ? launch_mfma<64>(p, stream, ev_start, ev_stop) : launch_mfma<128>(p, stream, ev_start, ev_stop);
}

}  // namespace reader

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

__device__ inline int pick4(int a0, int a1, int a2, int a3, int idx) {
    int lo = (idx & 1) ? a1 : a0;
    int hi = (idx & 1) ? a3 : a2;
    return (idx & 2) ? hi : lo;
}

__device__ inline uint4 ld16(const uint16_t *ptr) { return *reinterpret_cast<const uint4 *>(ptr); }

template <int D>
struct Geometry {
    static constexpr int kChunks = D / 8;                          // 16-byte chunks per K/V row
    static constexpr int kKLoads = kTile * kChunks / kThreads;     // K chunks per thread per tile
    static constexpr int kVLoads = (kTile / 2) * kChunks / kThreads;  // key pairs x chunks per thread
    static constexpr int kKBytes = kTile * D * 2;
    static constexpr int kVBytes = D * kTile * 2;
    static constexpr int kBufBytes = kKBytes + kVBytes;
    static constexpr int kKSteps = D / 16;                         // MFMA k-steps of the QK product
    static constexpr int kOBlocks = D / 32;                        // 32-wide blocks of the output dim
};

// Registers a thread holds for the tile that is in flight from HBM.
template <int D>
struct Staged {
    uint4 k[Geometry<D>::kKLoads];
    uint4 va[Geometry<D>::kVLoads], vb[Geometry<D>::kVLoads];
};

// Issue the global loads of one unit.  Rows that do not exist (past the sequence end, past
// the last tree node, behind an invalid page id) are staged as zeros: a zero K row is
// masked later, a zero V row contributes nothing.
template <int D>
__device__ inline void issue_loads(const AttnParams &p, const Cursor &c, Staged<D> &st, int &bad) {
    using G = Geometry<D>;
    const int tid = threadIdx.x;
    const uint4 zero = make_uint4(0u, 0u, 0u, 0u);
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
#pragma unroll
        for (int i = 0; i < G::kKLoads; ++i) {
            const int id = tid + kThreads * i;
            const int key = id / G::kChunks, chunk = id % G::kChunks;
            const int page = pick4(pg[0], pg[1], pg[2], pg[3], key >> 4);
            const bool ok = key < n_valid && page >= 0;
            const size_t off = (((size_t)(ok ? page : 0) * p.Hkv + c.hkv) * 16 + (key & 15)) * D + chunk * 8;
            st.k[i] = ok ? ld16(p.k_cache + off) : zero;
        }
#pragma unroll
        for (int i = 0; i < G::kVLoads; ++i) {
            const int id = tid + kThreads * i;
            const int key = 2 * (id / G::kChunks), chunk = id % G::kChunks;
            const int page = pick4(pg[0], pg[1], pg[2], pg[3], key >> 4);
            const bool ok0 = key < n_valid && page >= 0, ok1 = key + 1 < n_valid && page >= 0;
            const size_t off = (((size_t)(ok0 ? page : 0) * p.Hkv + c.hkv) * 16 + (key & 15)) * D + chunk * 8;
            st.va[i] = ok0 ? ld16(p.v_cache + off) : zero;
            st.vb[i] = ok1 ? ld16(p.v_cache + off + D) : zero;
        }
    } else {
        const int base = (c.idx - c.n_pre) * kTile;
        const int n_valid = min(kTile, p.T - base);
        const size_t row_stride = (size_t)p.Hkv * D;
        const size_t origin = (((size_t)c.b * p.T + base) * p.Hkv + c.hkv) * D;
#pragma unroll
        for (int i = 0; i < G::kKLoads; ++i) {
            const int id = tid + kThreads * i;
            const int key = id / G::kChunks, chunk = id % G::kChunks;
            const bool ok = key < n_valid;
            st.k[i] = ok ? ld16(p.k_tree + origin + (size_t)key * row_stride + chunk * 8) : zero;
        }
#pragma unroll
        for (int i = 0; i < G::kVLoads; ++i) {
            const int id = tid + kThreads * i;
            const int key = 2 * (id / G::kChunks), chunk = id % G::kChunks;
            const size_t off = origin + (size_t)key * row_stride + chunk * 8;
            st.va[i] = key < n_valid ? ld16(p.v_tree + off) : zero;
            st.vb[i] = key + 1 < n_valid ? ld16(p.v_tree + off + row_stride) : zero;
        }
    }
}

// Where key `key` of a tile sits along the key axis of the transposed V tile: the order
// in which the S^T accumulator registers of a lane enumerate the keys.
__device__ inline int vt_column(int key) {
    const int r = key & 31;
    return (key & 32) + ((r >> 4) << 4) + (((r >> 2) & 1) << 3) + (((r >> 3) & 1) << 2) + (r & 3);
}

// Staged registers -> LDS.  K keeps its row-major form; V is written transposed,
// two keys (one 32-bit word) at a time.  Both use 16-byte chunks XOR-swizzled by row.
template <int D>
__device__ inline void write_stage(const Staged<D> &st, char *k_lds, char *vt_lds) {
    using G = Geometry<D>;
    const int tid = threadIdx.x;
#pragma unroll
    for (int i = 0; i < G::kKLoads; ++i) {
        const int id = tid + kThreads * i;
        const int key = id / G::kChunks, chunk = id % G::kChunks;
        *reinterpret_cast<uint4 *>(k_lds + key * (D * 2) + ((chunk ^ (key & 7)) << 4)) = st.k[i];
    }
#pragma unroll
    for (int i = 0; i < G::kVLoads; ++i) {
        const int id = tid + kThreads * i;
        const int key = 2 * (id / G::kChunks), chunk = id % G::kChunks;
        const int col = vt_column(key);           // even; key + 1 sits at col + 1
        const uint32_t a[4] = {st.va[i].x, st.va[i].y, st.va[i].z, st.va[i].w};
        const uint32_t b[4] = {st.vb[i].x, st.vb[i].y, st.vb[i].z, st.vb[i].w};
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            const uint32_t lo = (e & 1) ? (a[e >> 1] >> 16) : (a[e >> 1] & 0xffffu);
            const uint32_t hi = (e & 1) ? (b[e >> 1] & 0xffff0000u) : (b[e >> 1] << 16);
            const int d = chunk * 8 + e;
            const int swz = (e ^ chunk) & 7;      // (d ^ (d >> 3)) & 7
            *reinterpret_cast<uint32_t *>(vt_lds + d * (kTile * 2) + (((col >> 3) ^ swz) << 4) + (col & 7) * 2) = lo | hi;
        }
    }
}

__device__ inline uint32_t pack_bf16x2(float lo, float hi) {
    typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
    bf16x2 v;
    v[0] = (__bf16)lo;
    v[1] = (__bf16)hi;
    return __builtin_bit_cast(uint32_t, v);
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
    int *s_pref = s_par + READER_MAX_T;                                        // [B + 1]
    __shared__ int s_wsum[4];

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

    Cursor cc;   // unit being computed
    cc.b = find_seq(s_pref, p.B, p.Hkv, lo);
    cursor_enter_seq(cc, p);
    {
        const long long rel = lo - (long long)p.Hkv * s_pref[cc.b];
        cc.hkv = (int)(rel / cc.n_units);
        cc.idx = (int)(rel - (long long)cc.hkv * cc.n_units);
    }
    Cursor lc = cc;   // unit being loaded (one ahead)

    int bad = 0;
    Staged<D> st;
    issue_loads<D>(p, lc, st, bad);
    write_stage<D>(st, buf0, buf0 + G::kKBytes);
    cursor_advance(lc, p);
    __syncthreads();

    bf16x8 qf[G::kKSteps];
    f32x16 o[G::kOBlocks];
    float m_run = -INFINITY, l_run = 0.f;
    bool fresh = true;                 // the next unit starts a segment (new pair or range start)
    bool seg_from_pair_start = false;
    const float c2 = p.scale_log2;

    for (long long x = lo; x < hi; ++x) {
        const int cur = (int)((x - lo) & 1);
        char *k_lds = (cur ? buf1 : buf0);
        char *vt_lds = k_lds + G::kKBytes;
        const bool more = x + 1 < hi;
        if (more) issue_loads<D>(p, lc, st, bad);

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
                uint4 v = row_real ? ld16(qrow + kk * 16 + h * 8) : make_uint4(0u, 0u, 0u, 0u);
                qf[kk] = __builtin_bit_cast(bf16x8, v);
            }
            // ancestor-or-self masks of this sequence's tree, if this segment reaches its tree tiles
            const long long seg_end_idx = (long long)cc.idx + (hi - x);   // exclusive, in pair units
            if (seg_end_idx > cc.n_pre) {
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

        if (wave_active) {
            // ---- S^T = K . Q^T : two 32-key blocks ----
            f32x16 s[2];
#pragma unroll
            for (int kb = 0; kb < 2; ++kb) {
#pragma unroll
                for (int i = 0; i < 16; ++i) s[kb][i] = 0.f;
                const int row = kb * 32 + n;
#pragma unroll
                for (int kk = 0; kk < G::kKSteps; ++kk) {
                    const int chunk = kk * 2 + h;
                    const bf16x8 a = *reinterpret_cast<const bf16x8 *>(k_lds + row * (D * 2) + ((chunk ^ (row & 7)) << 4));
                    s[kb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, qf[kk], s[kb], 0, 0, 0);
                }
            }
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
            // ---- O^T += V^T . P^T ----
#pragma unroll
            for (int ks = 0; ks < 4; ++ks) {
                const int kb = ks >> 1, m2 = ks & 1;
                const uint4 pv = make_uint4(pk[kb][4 * m2], pk[kb][4 * m2 + 1], pk[kb][4 * m2 + 2], pk[kb][4 * m2 + 3]);
                const bf16x8 pb = __builtin_bit_cast(bf16x8, pv);
                const int chunk = ks * 2 + h;
#pragma unroll
                for (int db = 0; db < G::kOBlocks; ++db) {
                    const int d = db * 32 + n;
                    const int swz = (d ^ (d >> 3)) & 7;
                    const bf16x8 a = *reinterpret_cast<const bf16x8 *>(vt_lds + d * (kTile * 2) + ((chunk ^ swz) << 4));
                    o[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, pb, o[db], 0, 0, 0);
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
            char *nk = (cur ? buf0 : buf1);
            write_stage<D>(st, nk, nk + G::kKBytes);
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
                            READER_MAX_T * sizeof(int) + pref_bytes;
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

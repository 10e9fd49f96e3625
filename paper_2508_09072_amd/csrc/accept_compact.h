// Device code of the acceptance and compaction steps, shared by their own kernels and by the
// fused tail kernel of reader_verify_step.
//
// Acceptance (Algorithm 5; Appendix C invariants 2-3): one 64-lane wavefront per
// sequence.  Each lane owns up to two tree nodes.  A node "matches" when its drafted
// token equals the base model's token at its parent; the matches of all nodes are
// gathered with two wavefront ballots.  Every lane then walks its nodes' parent
// chains to get their ancestor-or-self sets as 128-bit masks; a node is accepted
// iff its whole set lies inside the match ballot, and its depth is the set's
// population count minus one.  A wavefront max-reduction over (depth, lowest id)
// picks the terminal node; the nodes of its ancestor set scatter themselves into
// `path` at their own depth.
//
// Compaction (Section 4.3 / Algorithm 4, applied every step): one workgroup per
// sequence copies the accepted rows with 128-bit accesses and then bumps seq_lens.
#pragma once

#include "internal.h"

namespace reader {

// LDS the acceptance of one sequence needs.
struct AcceptShared {
    int par[READER_MAX_T];
    int target[READER_MAX_T];        // the base model's tokens, so that target[parent] is an LDS read
    int path[READER_MAX_T];          // the accepted path, for a compaction that follows in the same workgroup
    unsigned long long term[2];
    int accept_len;
};

// Called by every thread of the workgroup (it contains barriers); the work is done by the
// first wavefront (`active`: threadIdx.x < 64, lane = threadIdx.x).
__device__ inline void accept_path_body(const AcceptParams &p, int b, int lane, bool active, AcceptShared &sh) {
    const int T = p.T;
    const int32_t *par = p.parents + (size_t)b * T;
    const int32_t *draft = p.draft + (size_t)b * T;
    const int32_t *target = p.target + (size_t)b * T;

    bool bad_tree = false;
    bool match[2] = {false, false};
    int my_target[2] = {0, 0}, my_draft[2] = {0, 0}, my_par[2] = {-1, -1};
    bool my_valid[2] = {false, false};
    unsigned long long m_lo = 0ull, m_hi = 0ull;
    if (active) {
        // one trip to memory for the three token/parent rows; target[parent] then comes from LDS
#pragma unroll
        for (int s = 0; s < 2; ++s) {
            const int i = lane + 64 * s;
            if (i < T) {
                int pi = par[i];
                my_draft[s] = draft[i];
                my_target[s] = target[i];
                my_valid[s] = (i == 0) ? (pi == -1) : (pi >= 0 && pi < i);
                if (!my_valid[s]) { bad_tree = true; pi = -1; }
                my_par[s] = pi;
                sh.par[i] = pi;
                sh.target[i] = my_target[s];
            }
        }
    }
    __syncthreads();
    if (active) {
#pragma unroll
        for (int s = 0; s < 2; ++s) {
            const int i = lane + 64 * s;
            if (i < T) match[s] = (i == 0) || (my_valid[s] && my_draft[s] == sh.target[my_par[s]]);
        }
        m_lo = __ballot(match[0]);
        m_hi = __ballot(match[1]);
    }

    // ancestor-or-self sets by walking the parent chain (at most T steps, always ends)
    unsigned long long a_lo[2] = {0ull, 0ull}, a_hi[2] = {0ull, 0ull};
    int n_out = 0, depth_term = 0;
    if (active) {
        int key[2] = {-1, -1};
#pragma unroll
        for (int s = 0; s < 2; ++s) {
            const int i = lane + 64 * s;
            if (i < T) {
                int t = i;
                for (int step = 0; step < T && t >= 0; ++step) {
                    if (t < 64) a_lo[s] |= 1ull << t; else a_hi[s] |= 1ull << (t - 64);
                    t = sh.par[t];
                }
                const bool ok = ((a_lo[s] & ~m_lo) == 0) && ((a_hi[s] & ~m_hi) == 0);
                const int depth = __popcll(a_lo[s]) + __popcll(a_hi[s]) - 1;
                if (ok) key[s] = depth * 256 + (255 - i);   // deeper first, then lower node id
            }
        }
        int best = max(key[0], key[1]);
#pragma unroll
        for (int off = 32; off >= 1; off >>= 1) best = max(best, __shfl_xor(best, off));
        // the root always qualifies, so best >= 255
        const int term = 255 - (best & 255);
        depth_term = best >> 8;
        n_out = min(depth_term, p.max_path - 1);
        if (lane == (term & 63)) {
            const int s = term >> 6;
            sh.term[0] = a_lo[s];
            sh.term[1] = a_hi[s];
        }
        if (lane == 0) sh.accept_len = n_out;
    }
    __syncthreads();

    if (active) {
        const unsigned long long t_lo = sh.term[0], t_hi = sh.term[1];
        int32_t *path = p.path + (size_t)b * p.max_path;
#pragma unroll
        for (int s = 0; s < 2; ++s) {
            const int i = lane + 64 * s;
            if (i < T) {
                const bool on_path = (s == 0) ? ((t_lo >> lane) & 1ull) : ((t_hi >> lane) & 1ull);
                if (on_path) {
                    const int depth = __popcll(a_lo[s]) + __popcll(a_hi[s]) - 1;
                    if (depth < p.max_path) { path[depth] = i; sh.path[depth] = i; }
                    if (depth == n_out) {
                        p.accept_len[b] = n_out;
                        p.bonus[b] = my_target[s];
                    }
                }
            }
        }
        for (int j = n_out + 1 + lane; j < p.max_path; j += 64) path[j] = -1;

        const bool any_bad_tree = __ballot(bad_tree) != 0ull;
        if (p.status && lane == 0) {
            int bits = (any_bad_tree ? READER_STATUS_BAD_TREE : 0) |
                       (depth_term > n_out ? READER_STATUS_BAD_PATH : 0);
            if (bits) atomicOr(p.status, bits);
        }
    }
}

// What compaction needs that does not depend on the accepted path: the old length and the page
// ids of the positions a path could be appended to.  Loaded up front so that, in the fused tail
// kernel, they travel while the acceptance runs.
struct CompactShared {
    int L;
    int page[READER_MAX_T];   // page id of position L + j (or -1 past the page table)
};

// Called by all 256 threads of the workgroup, before a barrier.
__device__ inline void kv_compact_prefetch(const CompactParams &p, int b, int tid, CompactShared &cs) {
    const int L = p.seq_lens[b];
    if (tid == 0) cs.L = L;
    if (tid < p.max_path) {
        const long long pos = (long long)L + tid;
        const bool in_table = L >= 0 && pos < (long long)p.max_pages * READER_PAGE_SIZE;
        cs.page[tid] = in_table ? p.page_table[(size_t)b * p.max_pages + pos / READER_PAGE_SIZE] : -1;
    }
}

// Called by all 256 threads of the workgroup, after kv_compact_prefetch and a barrier.
// n = accept_len of the sequence, path = its accepted path (global or LDS).
__device__ inline void kv_compact_body(const CompactParams &p, int b, int tid, int n, const int *path,
                                       const CompactShared &cs) {
    const int L = cs.L;

    // Every item this sequence would touch is checked before anything is written.
    int bad = 0;
    if (n < 0 || n > p.max_path - 1 || L < 0 || (long long)L + n + 1 > (long long)p.max_pages * READER_PAGE_SIZE) {
        bad = READER_STATUS_BAD_PATH;
    } else {
        for (int j = tid; j <= n; j += 256) {
            const int node = path[j];
            if (node < 0 || node >= p.T) bad |= READER_STATUS_BAD_PATH;
            const int page = cs.page[j];
            if (page < 0 || page >= p.num_pages) bad |= READER_STATUS_BAD_PAGE;
        }
    }
    // the barriers also order every thread's read of seq_lens before its update below
    const int bad_path = __syncthreads_or(bad & READER_STATUS_BAD_PATH);
    const int bad_page = __syncthreads_or(bad & READER_STATUS_BAD_PAGE);
    if (bad_path || bad_page) {
        if (tid == 0 && p.status)
            atomicOr(p.status, (bad_path ? READER_STATUS_BAD_PATH : 0) | (bad_page ? READER_STATUS_BAD_PAGE : 0));
        return;
    }

    const int chunks_per_head = p.D / 8;                 // 16-byte chunks
    const int chunks_per_row = p.Hkv * chunks_per_head;  // one position, all kv heads, K or V
    // A thread keeps its place inside a position (K or V, head, chunk) and walks the path entries, eight at a
    // time: their rows are asked for together and stored afterwards (taken one by one, every accepted token
    // costs a trip to memory).  The loads carry no condition (an entry past the path reads the last one
    // again), so that they stay together in front of the stores.
    constexpr int kBatch = 8;
    for (int rem = tid; rem < 2 * chunks_per_row; rem += 256) {
        const int which = rem / chunks_per_row;
        const int c = rem - which * chunks_per_row;
        const int h = c / chunks_per_head;
        const int dc = c - h * chunks_per_head;
        const uint16_t *tree = (which ? p.v_tree : p.k_tree) + ((size_t)b * p.T * p.Hkv + h) * p.D + dc * 8;
        uint16_t *cache = (which ? p.v_cache : p.k_cache) + (size_t)h * READER_PAGE_SIZE * p.D + dc * 8;
        for (int j0 = 0; j0 <= n; j0 += kBatch) {
            uint4 held[kBatch];
#pragma unroll
            for (int u = 0; u < kBatch; ++u)
                held[u] = *reinterpret_cast<const uint4 *>(tree + (size_t)path[min(j0 + u, n)] * p.Hkv * p.D);
#pragma unroll
            for (int u = 0; u < kBatch; ++u) {
                const int j = j0 + u;
                if (j <= n) {
                    const long long page = cs.page[j];
                    const int slot = (L + j) % READER_PAGE_SIZE;
                    *reinterpret_cast<uint4 *>(cache + ((size_t)page * p.Hkv * READER_PAGE_SIZE + slot) * p.D) = held[u];
                }
            }
        }
    }
    if (tid == 0) p.seq_lens[b] = L + n + 1;
}

}  // namespace reader

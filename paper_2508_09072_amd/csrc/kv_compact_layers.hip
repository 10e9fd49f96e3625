// Compaction in the in-cache layout, all layers at once (Section 4.3; Algorithm 4 applied
// every step).  The forward pass of the step wrote the draft tree's K/V rows behind each
// sequence, node n at position L + n, in every layer's cache; once the accepted path is known,
// position L + j takes the row of position L + path[j], j = 1..accept_len (the root, j = 0, is
// in place), and the sequence grows by accept_len + 1.
//
// The move is in place.  A parent precedes its children, so node ids increase along a path and
// path[j] >= j: a destination is never the source of a later row.  It can be the source of an
// earlier one, so the rows of a pass are all read before any is written (a barrier between the
// two halves); passes take the rows in increasing j, which keeps that guarantee across passes.
//
// One launch, one workgroup per (sequence, layer).  Every workgroup of a sequence needs its old
// length, so the new one is written by whichever of them finishes last: each takes a ticket per
// sequence when its rows are moved, and the holder of the last ticket writes the length and
// puts the ticket counter back to zero.  The counters are device memory of the library itself
// (one word per possible sequence, zero when the library is loaded and after every call), which
// is why calls on the same GPU must not overlap in time.
#include "internal.h"

namespace reader {

namespace {

constexpr int kMoveThreads = 256;
constexpr int kMovePerThread = 8;      // 16-byte chunks a thread carries through one pass

// tickets taken by the workgroups of sequence b in the call that is running (0 between calls)
__device__ unsigned g_tickets[READER_MAX_B];

struct MoveShared {
    int L, n, bad;
    int node[READER_MAX_T];            // path
    int src_page[READER_MAX_T], dst_page[READER_MAX_T];
};

// Checks everything the sequence would touch before anything is written; called by at least
// READER_MAX_T threads, with a barrier behind it.  Result in sh (bad: status bits, 0 = go).
__device__ inline void check_sequence(const CompactLayersParams &p, int b, int tid, MoveShared &sh) {
    // (the path entries are asked for together with the two scalars, not after them: one memory round trip less)
    const int32_t *path = p.path + (size_t)b * p.max_path;
    const int my_node = tid < p.max_path ? path[tid] : -1;
    const int before = tid >= 1 && tid < p.max_path ? path[tid - 1] : -1;
    if (tid == 0) {
        sh.L = p.seq_lens[b];
        sh.n = p.accept_len[b];
        sh.bad = 0;
    }
    __syncthreads();
    const int L = sh.L, n = sh.n;
    int bad = 0;
    const long long mapped = (long long)p.max_pages * READER_PAGE_SIZE;
    if (n < 0 || n > p.max_path - 1 || L < 0 || (long long)L + n + 1 > mapped) {
        bad = READER_STATUS_BAD_PATH;
    } else if (tid <= n) {
        const int j = tid;
        const int node = my_node;
        const bool ok = node >= 0 && node < p.T && (j == 0 ? node == 0 : node > before) && (long long)L + node < mapped;
        if (!ok) {
            bad = READER_STATUS_BAD_PATH;
        } else {
            const int sp = p.page_table[(size_t)b * p.max_pages + (L + node) / READER_PAGE_SIZE];
            const int dp = p.page_table[(size_t)b * p.max_pages + (L + j) / READER_PAGE_SIZE];
            if (sp < 0 || sp >= p.num_pages || dp < 0 || dp >= p.num_pages) bad = READER_STATUS_BAD_PAGE;
            sh.node[j] = node;
            sh.src_page[j] = sp;
            sh.dst_page[j] = dp;
        }
    }
    if (bad) atomicOr(&sh.bad, bad);
    __syncthreads();
}

__global__ __launch_bounds__(kMoveThreads) void compact_layers_move_kernel(CompactLayersParams p) {
    __shared__ MoveShared sh;
    const int b = blockIdx.x, layer = blockIdx.y, tid = threadIdx.x;
    check_sequence(p, b, tid, sh);
    if (sh.bad) {
        if (layer == 0 && tid == 0 && p.status) atomicOr(p.status, sh.bad);
        return;
    }
    const int L = sh.L, n = sh.n;
    const int cpr = p.D / 8;                               // 16-byte chunks per row and head
    const size_t layer_off = (size_t)layer * (size_t)p.num_pages * p.Hkv * READER_PAGE_SIZE * p.D;
    // items: (K or V, head, j = 1..n, chunk), in that order; a pass takes kMoveThreads * kMovePerThread of them
    const int per_stream = n * cpr, total = 2 * p.Hkv * per_stream;
    for (int base = 0; base < total; base += kMoveThreads * kMovePerThread) {
        uint4 held[kMovePerThread];
        size_t dst[kMovePerThread];
        uint16_t *cache_of[kMovePerThread];
#pragma unroll
        for (int r = 0; r < kMovePerThread; ++r) {
            const int idx = base + r * kMoveThreads + tid;
            cache_of[r] = nullptr;
            if (idx < total) {
                const int stream = idx / per_stream, rem = idx - stream * per_stream;
                const int which = stream / p.Hkv, h = stream - which * p.Hkv;
                const int j = 1 + rem / cpr, c = rem - (j - 1) * cpr;
                const int node = sh.node[j];
                if (node != j) {                            // a row that is already in place stays
                    uint16_t *cache = (which ? p.v_cache : p.k_cache) + layer_off;
                    const size_t src = (((size_t)sh.src_page[j] * p.Hkv + h) * READER_PAGE_SIZE + (L + node) % READER_PAGE_SIZE) * p.D + c * 8;
                    dst[r] = (((size_t)sh.dst_page[j] * p.Hkv + h) * READER_PAGE_SIZE + (L + j) % READER_PAGE_SIZE) * p.D + c * 8;
                    held[r] = *reinterpret_cast<const uint4 *>(cache + src);
                    cache_of[r] = cache;
                }
            }
        }
        __syncthreads();   // every row of this pass has been read
#pragma unroll
        for (int r = 0; r < kMovePerThread; ++r)
            if (cache_of[r]) *reinterpret_cast<uint4 *>(cache_of[r] + dst[r]) = held[r];
    }
    // the last workgroup of the sequence to get here writes the new length (nobody needs the old one any more)
    if (tid == 0) {
        const unsigned ticket = atomicAdd(&g_tickets[b], 1u);
        if (ticket == (unsigned)p.NL - 1u) {
            g_tickets[b] = 0u;
            p.seq_lens[b] = L + n + 1;
        }
    }
}

__global__ __launch_bounds__(128) void compact_layers_lengths_kernel(CompactLayersParams p) {
    __shared__ MoveShared sh;
    const int b = blockIdx.x, tid = threadIdx.x;
    check_sequence(p, b, tid, sh);
    if (sh.bad) {
        if (tid == 0 && p.status) atomicOr(p.status, sh.bad);
        return;
    }
    if (tid == 0) p.seq_lens[b] = sh.L + sh.n + 1;
}

}  // namespace

hipError_t launch_kv_compact_layers(const CompactLayersParams &p, hipStream_t stream) {
    if (p.NL > 0) {
        hipLaunchKernelGGL(compact_layers_move_kernel, dim3(p.B, p.NL), dim3(kMoveThreads), 0, stream, p);
        return note_hip_error("launch compact_layers_move_kernel", hipGetLastError());
    }
    hipLaunchKernelGGL(compact_layers_lengths_kernel, dim3(p.B), dim3(128), 0, stream, p);   // no layers: only the lengths
    return note_hip_error("launch compact_layers_lengths_kernel", hipGetLastError());
}

}  // namespace reader

// Periodic rearrangement of a padded KV cache (Section 4.3 / Algorithm 4 of the READER paper):
// per sample, internal padding is removed and the real entries are concatenated tightly, in
// place, so that padding may only remain at the end.
//
// Two kernels.
//   plan:   one workgroup per sample scans its validity flags: every valid position gets its
//           destination (the number of valid positions before it), noted the other way round:
//           source[d] = the position whose row goes to d; the sample's new length n, its old
//           extent (last valid position + 1) and its first hole are noted; for the positions
//           from n on (their slots of `source` are free) it is noted whether they held a row;
//           the flags become ones-then-zeros.
//   apply:  two kinds of workgroup in one launch, which never touch the same bytes.
//           Movers, one per (sample, kv head, layer), walk the destinations from the first hole
//           to n in passes: all rows of a pass are loaded (128-bit accesses) before any is
//           stored, and sources never lie to the left of their destinations, so the move is
//           safe in place (a pass writes [a, a + P); the sources of later passes lie at or
//           behind a + P); a source at or behind n is cleared once it has been read.  Rows in
//           front of the first hole are not touched, so a pass moves only what acceptance spans
//           of unequal length have left out of place: few rows, scattered (memory serves such
//           pieces at a fraction of its streaming rate).
//           Clearers take the positions between n and the old extent that held no row: per
//           (sample, layer) one stretch of K and one of V, contiguous but for the few sources
//           in it, cut into pieces for as many workgroups as fill the GPU.  This is most of the
//           traffic of a pass (a short prompt leaves a long hole in front of the first decoding
//           step); as plain stores it runs at the rate of a fill, with the movers underneath.
#include "internal.h"

namespace reader {

namespace {

constexpr int kPlanThreads = 1024;
constexpr int kPlanPerThread = 8;                    // consecutive positions a thread scans per round

__global__ __launch_bounds__(kPlanThreads) void rearrange_plan_kernel(RearrangeParams p) {
    const int b = blockIdx.x, tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    uint8_t *valid = p.valid + (size_t)b * p.S;
    int32_t *source = p.dest + (size_t)b * p.S;
    __shared__ int s_wsum[kPlanThreads / 64];
    __shared__ int s_first_hole, s_extent;
    if (tid == 0) { s_first_hole = p.S; s_extent = 0; }
    __syncthreads();

    // rounds of kPlanThreads * kPlanPerThread positions (one round up to 8192 slots per sample: the flags of a
    // round are asked for together, so a round costs one trip to memory)
    int carry = 0, first_hole = p.S, extent = 0;
    for (int base = 0; base < p.S; base += kPlanThreads * kPlanPerThread) {
        const int j0 = base + tid * kPlanPerThread;
        bool f[kPlanPerThread];
        int mine = 0;
#pragma unroll
        for (int i = 0; i < kPlanPerThread; ++i) f[i] = j0 + i < p.S && valid[j0 + i] != 0;
#pragma unroll
        for (int i = 0; i < kPlanPerThread; ++i) mine += f[i] ? 1 : 0;
        int incl = mine;
#pragma unroll
        for (int off = 1; off < 64; off <<= 1) {
            const int t = __shfl_up(incl, off);
            if (lane >= off) incl += t;
        }
        if (lane == 63) s_wsum[wave] = incl;
        __syncthreads();
        int woff = 0, total = 0;
#pragma unroll
        for (int w = 0; w < kPlanThreads / 64; ++w) {
            const int x = s_wsum[w];
            if (w < wave) woff += x;
            total += x;
        }
        int d = carry + woff + incl - mine;            // valid positions in front of j0
#pragma unroll
        for (int i = 0; i < kPlanPerThread; ++i) {
            const int j = j0 + i;
            if (j < p.S) {
                if (f[i]) {
                    source[d++] = j;
                    extent = j + 1;
                } else if (j < first_hole) {
                    first_hole = j;
                }
            }
        }
        carry += total;
        __syncthreads();
    }
    atomicMin(&s_first_hole, first_hole);
    atomicMax(&s_extent, extent);
    __syncthreads();   // every flag has been read; all threads know the new length (carry)
    for (int j = tid; j < p.S; j += kPlanThreads) {
        if (j >= carry) source[j] = valid[j] ? 1 : 0;   // (destinations end at carry - 1: these slots are free)
        valid[j] = j < carry;
    }
    if (tid == 0) {
        p.new_len[b] = carry;
        int32_t *meta = p.dest + (size_t)p.B * p.S + (size_t)b * 4;
        meta[0] = carry;
        meta[1] = s_extent;
        meta[2] = s_first_hole;
    }
}

constexpr int kApplyThreads = 256;
constexpr int kMoveSub = 4;                          // groups of rows a mover's thread carries through one pass
constexpr int kZeroPerThread = 8;                    // 16-byte stores per clearer thread and tensor
constexpr int kZeroPiece = kApplyThreads * kZeroPerThread * 16;   // bytes of K (and of V) a clearer takes at a time

template <int D>
__device__ inline void rearrange_move(const RearrangeParams &p, int b, int hkv, int layer) {
    constexpr int kThreadsPerRow = D / 8;            // 16-byte chunks of one (position, kv head) row
    constexpr int kRowsPerGroup = kApplyThreads / kThreadsPerRow;
    const int tid = threadIdx.x, r = tid / kThreadsPerRow, c = tid % kThreadsPerRow;
    const int32_t *source = p.dest + (size_t)b * p.S;
    const int32_t *meta = p.dest + (size_t)p.B * p.S + (size_t)b * 4;
    const int n = meta[0], extent = meta[1], first_hole = meta[2];
    if (first_hole >= extent) return;               // no hole inside the sample: nothing to do

    const size_t pos_stride = (size_t)p.Hkv * D;    // elements between consecutive positions
    uint16_t *k = p.k_pad + (((size_t)layer * p.B + b) * p.S) * pos_stride + (size_t)hkv * D + c * 8;
    uint16_t *v = p.v_pad + (((size_t)layer * p.B + b) * p.S) * pos_stride + (size_t)hkv * D + c * 8;
    const uint4 zero = make_uint4(0u, 0u, 0u, 0u);

    // destinations first_hole .. n - 1, in passes of kMoveSub groups: the sources of a pass are asked for
    // together, then their rows, so that a pass costs two memory round trips
    for (int base = first_hole; base < n; base += kRowsPerGroup * kMoveSub) {
        int src[kMoveSub];
        uint4 kv[kMoveSub], vv[kMoveSub];
#pragma unroll
        for (int u = 0; u < kMoveSub; ++u) {
            const int d = base + u * kRowsPerGroup + r;
            src[u] = d < n ? source[d] : -1;
        }
#pragma unroll
        for (int u = 0; u < kMoveSub; ++u) {
            kv[u] = zero; vv[u] = zero;
            if (src[u] >= 0) {
                kv[u] = *reinterpret_cast<const uint4 *>(k + (size_t)src[u] * pos_stride);
                vv[u] = *reinterpret_cast<const uint4 *>(v + (size_t)src[u] * pos_stride);
            }
        }
        __syncthreads();   // every row of the pass is in registers (the barrier waits for the loads)
#pragma unroll
        for (int u = 0; u < kMoveSub; ++u) {
            const int d = base + u * kRowsPerGroup + r;
            if (src[u] >= 0) {
                *reinterpret_cast<uint4 *>(k + (size_t)d * pos_stride) = kv[u];
                *reinterpret_cast<uint4 *>(v + (size_t)d * pos_stride) = vv[u];
                if (src[u] >= n) {                   // (no destination lies there: they end at n - 1)
                    *reinterpret_cast<uint4 *>(k + (size_t)src[u] * pos_stride) = zero;
                    *reinterpret_cast<uint4 *>(v + (size_t)src[u] * pos_stride) = zero;
                }
            }
        }
    }
}

// The `lanes` clearers of a (sample, layer) take the pieces of its stretch in turn.
__device__ inline void rearrange_clear(const RearrangeParams &p, int b, int first_piece, int lanes, int layer) {
    const int32_t *held_row = p.dest + (size_t)b * p.S;             // meaningful from position n on
    const int32_t *meta = p.dest + (size_t)p.B * p.S + (size_t)b * 4;
    const int n = meta[0], extent = meta[1], first_hole = meta[2];
    if (first_hole >= extent) return;
    const unsigned pos_bytes = (unsigned)p.Hkv * p.D * 2;
    const size_t bytes = (size_t)(extent - n) * pos_bytes;           // a multiple of 16
    const size_t at = ((((size_t)layer * p.B + b) * p.S) + n) * pos_bytes;
    char *k = reinterpret_cast<char *>(p.k_pad) + at, *v = reinterpret_cast<char *>(p.v_pad) + at;
    const uint4 zero = make_uint4(0u, 0u, 0u, 0u);
    for (size_t begin = (size_t)first_piece * kZeroPiece; begin < bytes; begin += (size_t)lanes * kZeroPiece) {
        bool mine[kZeroPerThread];
#pragma unroll
        for (int i = 0; i < kZeroPerThread; ++i) {
            const size_t off = begin + ((size_t)i * kApplyThreads + threadIdx.x) * 16;
            mine[i] = off < bytes && held_row[n + (int)(off / pos_bytes)] == 0;   // (a position that held a row is its mover's)
        }
#pragma unroll
        for (int i = 0; i < kZeroPerThread; ++i) {
            const size_t off = begin + ((size_t)i * kApplyThreads + threadIdx.x) * 16;
            if (mine[i]) {
                *reinterpret_cast<uint4 *>(k + off) = zero;
                *reinterpret_cast<uint4 *>(v + off) = zero;
            }
        }
    }
}

// 1-D grid: the movers of all layers first (their scattered accesses take longest), then the clearers
template <int D>
__global__ __launch_bounds__(kApplyThreads) void rearrange_apply_kernel(RearrangeParams p, int lanes) {
    const int per_layer = p.B * p.Hkv, movers = per_layer * p.NL;
    if ((int)blockIdx.x < movers) {
        const int layer = blockIdx.x / per_layer, i = blockIdx.x - layer * per_layer, b = i / p.Hkv;
        rearrange_move<D>(p, b, i - b * p.Hkv, layer);
    } else {
        const int c = blockIdx.x - movers, per = p.B * lanes;
        const int layer = c / per, i = c - layer * per, b = i / lanes;
        rearrange_clear(p, b, i - b * lanes, lanes, layer);
    }
}

}  // namespace

hipError_t launch_kv_rearrange(const RearrangeParams &p, hipStream_t stream) {
    hipLaunchKernelGGL(rearrange_plan_kernel, dim3(p.B), dim3(kPlanThreads), 0, stream, p);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return note_hip_error("launch rearrange_plan_kernel", e);
    if (p.NL == 0) return hipSuccess;
    // clearers per (sample, layer): enough for sixteen workgroups per compute unit over the whole grid, no more
    // than the longest stretch has pieces
    const size_t longest = (size_t)p.S * p.Hkv * p.D * 2;            // bytes of one tensor a sample can have to clear
    const long long most = (long long)((longest + kZeroPiece - 1) / kZeroPiece);
    long long lanes = (16LL * kNumCU + (long long)p.B * p.NL - 1) / ((long long)p.B * p.NL);
    lanes = lanes < 1 ? 1 : (lanes > most ? most : lanes);
    if ((long long)p.NL * p.B * (p.Hkv + lanes) > 0x7fffffffLL) lanes = 1;   // (NL * B * (Hkv + 1) fits: checked by the caller)
    const dim3 grid((unsigned)((long long)p.NL * p.B * (p.Hkv + lanes)));
    if (p.D == 64)
        hipLaunchKernelGGL(rearrange_apply_kernel<64>, grid, dim3(kApplyThreads), 0, stream, p, (int)lanes);
    else
        hipLaunchKernelGGL(rearrange_apply_kernel<128>, grid, dim3(kApplyThreads), 0, stream, p, (int)lanes);
    return note_hip_error("launch rearrange_apply_kernel", hipGetLastError());
}

}  // namespace reader

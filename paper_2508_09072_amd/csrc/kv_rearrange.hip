// Periodic rearrangement of a padded KV cache (Section 4.3 / Algorithm 4 of the READER paper):
// per sample, internal padding is removed and the real entries are concatenated tightly, in
// place, so that padding may only remain at the end.
//
// Two kernels.
//   plan:  one workgroup per sample scans its validity flags: every valid position gets its
//          destination (the number of valid positions before it); the sample's new length, its
//          old extent (last valid position + 1) and its first hole are noted; the flags become
//          ones-then-zeros.
//   move:  one workgroup per (sample, kv head, layer) walks the positions from the first hole
//          to the old extent in passes of 16 (D = 128) or 32 (D = 64) positions: all rows of a
//          pass are loaded (128-bit accesses) before any is stored, and destinations never lie
//          to the right of their sources, so the move is safe in place; positions between the
//          new length and the old extent are zeroed in the pass that has just read them.
// Rows in front of the first hole are not touched, so the pass moves only what acceptance
// spans of unequal length have left out of place.
#include "internal.h"

namespace reader {

namespace {

constexpr int kPlanThreads = 256;

__global__ __launch_bounds__(kPlanThreads) void rearrange_plan_kernel(RearrangeParams p) {
    const int b = blockIdx.x, tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    uint8_t *valid = p.valid + (size_t)b * p.S;
    int32_t *dest = p.dest + (size_t)b * p.S;
    __shared__ int s_wsum[kPlanThreads / 64];
    __shared__ int s_first_hole, s_extent;
    if (tid == 0) { s_first_hole = p.S; s_extent = 0; }
    __syncthreads();

    int carry = 0, first_hole = p.S, extent = 0;
    for (int base = 0; base < p.S; base += kPlanThreads) {
        const int j = base + tid;
        const int v = (j < p.S && valid[j]) ? 1 : 0;
        int incl = v;
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
            if (w < wave) woff += s_wsum[w];
            total += s_wsum[w];
        }
        if (j < p.S) {
            dest[j] = v ? carry + woff + incl - 1 : -1;
            if (v) extent = j + 1;
            else if (j < first_hole) first_hole = j;
        }
        carry += total;
        __syncthreads();
    }
    atomicMin(&s_first_hole, first_hole);
    atomicMax(&s_extent, extent);
    __syncthreads();   // every flag has been read; all threads know the new length (carry)
    for (int j = tid; j < p.S; j += kPlanThreads) valid[j] = j < carry;
    if (tid == 0) {
        p.new_len[b] = carry;
        int32_t *meta = p.dest + (size_t)p.B * p.S + (size_t)b * 4;
        meta[0] = carry;
        meta[1] = s_extent;
        meta[2] = s_first_hole;
    }
}

template <int D>
__global__ __launch_bounds__(256) void rearrange_move_kernel(RearrangeParams p) {
    constexpr int kThreadsPerRow = D / 8;            // 16-byte chunks of one (position, kv head) row
    constexpr int kPosPerPass = 256 / kThreadsPerRow;
    const int b = blockIdx.x / p.Hkv, hkv = blockIdx.x - b * p.Hkv, layer = blockIdx.y;
    const int tid = threadIdx.x, r = tid / kThreadsPerRow, c = tid % kThreadsPerRow;
    const int32_t *dest = p.dest + (size_t)b * p.S;
    const int32_t *meta = p.dest + (size_t)p.B * p.S + (size_t)b * 4;
    const int n = meta[0], extent = meta[1], first_hole = meta[2];
    if (first_hole >= extent) return;               // no hole inside the sample: nothing to do

    const size_t pos_stride = (size_t)p.Hkv * D;    // elements between consecutive positions
    uint16_t *k = p.k_pad + (((size_t)layer * p.B + b) * p.S) * pos_stride + (size_t)hkv * D + c * 8;
    uint16_t *v = p.v_pad + (((size_t)layer * p.B + b) * p.S) * pos_stride + (size_t)hkv * D + c * 8;
    const uint4 zero = make_uint4(0u, 0u, 0u, 0u);

    for (int base = (first_hole / kPosPerPass) * kPosPerPass; base < extent; base += kPosPerPass) {
        const int j = base + r;
        int d = -1;
        uint4 kv = zero, vv = zero;
        if (j >= first_hole && j < extent) {
            d = dest[j];
            if (d >= 0 && d != j) {
                kv = *reinterpret_cast<const uint4 *>(k + (size_t)j * pos_stride);
                vv = *reinterpret_cast<const uint4 *>(v + (size_t)j * pos_stride);
            }
        }
        __syncthreads();   // every row of the pass is in registers (the barrier waits for the loads)
        if (d >= 0 && d != j) {
            *reinterpret_cast<uint4 *>(k + (size_t)d * pos_stride) = kv;
            *reinterpret_cast<uint4 *>(v + (size_t)d * pos_stride) = vv;
        }
        if (j >= n && j >= first_hole && j < extent) {
            *reinterpret_cast<uint4 *>(k + (size_t)j * pos_stride) = zero;
            *reinterpret_cast<uint4 *>(v + (size_t)j * pos_stride) = zero;
        }
    }
}

}  // namespace

hipError_t launch_kv_rearrange(const RearrangeParams &p, hipStream_t stream) {
    hipLaunchKernelGGL(rearrange_plan_kernel, dim3(p.B), dim3(kPlanThreads), 0, stream, p);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return note_hip_error("launch rearrange_plan_kernel", e);
    if (p.NL == 0) return hipSuccess;
    if (p.D == 64)
        hipLaunchKernelGGL(rearrange_move_kernel<64>, dim3(p.B * p.Hkv, p.NL), dim3(256), 0, stream, p);
    else
        hipLaunchKernelGGL(rearrange_move_kernel<128>, dim3(p.B * p.Hkv, p.NL), dim3(256), 0, stream, p);
    return note_hip_error("launch rearrange_move_kernel", hipGetLastError());
}

}  // namespace reader

// The base model's greedy tokens from its logits (Algorithm 5: "compare base logits with
// drafted tokens"): target_tokens[r] = argmax_v logits[r][v] for the B*T rows of one
// verification step.  The logits of a step are as large as its KV stream (vocabulary 128256:
// 256 KB per row), so this is a plain streaming reduction: one workgroup per row, 128-bit
// loads (eight in flight per thread), a running (value, index) per thread, then a wavefront
// and a workgroup reduction.
// Ties go to the lowest index; a NaN is never larger than anything (a row of NaNs gives 0).
#include "internal.h"

namespace reader {

namespace {

struct Best {
    float v;
    int i;
};

__device__ inline void take(Best &b, float v, int i) {
    // strictly larger, or equal with a lower index (indices arrive out of order across threads)
    if (v > b.v || (v == b.v && i < b.i)) { b.v = v; b.i = i; }
}

__global__ __launch_bounds__(256) void target_argmax_kernel(const uint16_t *__restrict__ logits, int32_t *__restrict__ out,
                                                            int V) {
    const int row = blockIdx.x, tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const uint16_t *src = logits + (size_t)row * V;
    Best best = {-INFINITY, 0x7fffffff};
    // rows start at any multiple of 2 bytes: scalar head up to the first 16-byte boundary
    const int head = min(V, (int)(((16 - ((uintptr_t)src & 15)) & 15) >> 1));
    if (tid < head) take(best, __uint_as_float((uint32_t)src[tid] << 16), tid);
    const int n_vec = (V - head) / 8;
    const uint4 *vec = reinterpret_cast<const uint4 *>(src + head);
    auto scan = [&](const uint4 &w, int c) {
        const uint32_t u[4] = {w.x, w.y, w.z, w.w};
        const int base = head + c * 8;
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            take(best, __uint_as_float(u[e] << 16), base + 2 * e);
            take(best, __uint_as_float(u[e] & 0xffff0000u), base + 2 * e + 1);
        }
    };
    int c = tid;
    for (; c + 7 * 256 < n_vec; c += 8 * 256) {      // eight loads in flight per thread
        // read once: streamed past the caches (about a sixth more bandwidth out of HBM than plain loads)
        uint4 w[8];
#pragma unroll
        for (int j = 0; j < 8; ++j) w[j] = load_stream16(vec + c + j * 256);
#pragma unroll
        for (int j = 0; j < 8; ++j) scan(w[j], c + j * 256);
    }
    for (; c < n_vec; c += 256) scan(load_stream16(vec + c), c);
    for (int j = head + n_vec * 8 + tid; j < V; j += 256) take(best, __uint_as_float((uint32_t)src[j] << 16), j);

#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) {
        const float ov = __shfl_xor(best.v, off);
        const int oi = __shfl_xor(best.i, off);
        take(best, ov, oi);
    }
    __shared__ float s_v[4];
    __shared__ int s_i[4];
    if (lane == 0) { s_v[wave] = best.v; s_i[wave] = best.i; }
    __syncthreads();
    if (tid == 0) {
        Best b = {s_v[0], s_i[0]};
        for (int w = 1; w < 4; ++w) take(b, s_v[w], s_i[w]);
        out[row] = b.i == 0x7fffffff ? 0 : b.i;
    }
}

}  // namespace

hipError_t launch_target_argmax(const uint16_t *logits, int32_t *out, int rows, int V, hipStream_t stream) {
    hipLaunchKernelGGL(target_argmax_kernel, dim3(rows), dim3(256), 0, stream, logits, out, V);
    return note_hip_error("launch target_argmax_kernel", hipGetLastError());
}

}  // namespace reader

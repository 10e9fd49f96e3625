// The base model's greedy tokens from its logits (Algorithm 5: "compare base logits with
// drafted tokens"): target_tokens[r] = argmax_v logits[r][v] for the B*T rows of one
// verification step.  The logits of a step are as large as its KV stream (vocabulary 128256:
// 256 KB per row), so this is a plain streaming reduction: one workgroup per row, 128-bit
// loads (eight in flight per thread), a running (value, index) per thread, then a wavefront
// and a workgroup reduction.  The workgroup is 512 threads wide, 1024 when there are few rows
// (measured: 512 rows take 24 us with 1024 threads; from 1024 rows on 512 threads are the fastest).
// Ties go to the lowest index; a NaN is never larger than anything (a row of NaNs gives 0).
#include <stdlib.h>

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

// The same for values that arrive in increasing index order (a thread's own scan): an equal value never wins.
// (Half the vector instructions per logit of `take`; with `take` the kernel was bound by them, not by memory.)
__device__ inline void first_larger(Best &b, float v, int i) {
    if (v > b.v) { b.v = v; b.i = i; }
}

template <int NT, int NL>
__global__ __launch_bounds__(NT) void target_argmax_kernel(const uint16_t *__restrict__ logits, int32_t *__restrict__ out,
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
            first_larger(best, __uint_as_float(u[e] << 16), base + 2 * e);
            first_larger(best, __uint_as_float(u[e] & 0xffff0000u), base + 2 * e + 1);
        }
    };
    for (int c = tid; c < n_vec; c += NL * NT) {      // NL loads in flight per thread, also in the last round
        // read once: streamed past the caches (about a sixth more bandwidth out of HBM than plain loads)
        uint4 w[NL];
#pragma unroll
        for (int j = 0; j < NL; ++j)
            if (c + j * NT < n_vec) w[j] = load_stream16(vec + c + j * NT);
#pragma unroll
        for (int j = 0; j < NL; ++j)
            if (c + j * NT < n_vec) scan(w[j], c + j * NT);
    }
    for (int j = head + n_vec * 8 + tid; j < V; j += NT) take(best, __uint_as_float((uint32_t)src[j] << 16), j);

#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) {
        const float ov = __shfl_xor(best.v, off);
        const int oi = __shfl_xor(best.i, off);
        take(best, ov, oi);
    }
    __shared__ float s_v[NT / 64];
    __shared__ int s_i[NT / 64];
    if (lane == 0) { s_v[wave] = best.v; s_i[wave] = best.i; }
    __syncthreads();
    if (tid == 0) {
        Best b = {s_v[0], s_i[0]};
        for (int w = 1; w < NT / 64; ++w) take(b, s_v[w], s_i[w]);
        out[row] = b.i == 0x7fffffff ? 0 : b.i;
    }
}

}  // namespace

hipError_t launch_target_argmax(const uint16_t *logits, int32_t *out, int rows, int V, hipStream_t stream) {
    // threads per row so that the rows of the launch fill the chip's 256 x 2048 thread slots
    // (measured: 1024 threads per row are ahead up to 768 rows, 512 beyond)
    if (rows <= 768) hipLaunchKernelGGL((target_argmax_kernel<1024, 8>), dim3(rows), dim3(1024), 0, stream, logits, out, V);
    else hipLaunchKernelGGL((target_argmax_kernel<512, 8>), dim3(rows), dim3(512), 0, stream, logits, out, V);
    return note_hip_error("launch target_argmax_kernel", hipGetLastError());
}

}  // namespace reader

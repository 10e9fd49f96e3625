// Two bare loops that measure what this GPU gives the access pattern and the instruction the attention
// kernels are built from, for the denominators quoted next to the published peaks:
//   - the K/V stream: every compute unit copies 32 KB tiles from HBM into a ring of LDS buffers with
//     the same instruction (global_load_lds_dwordx4, non-temporal) and ring depth as the 128-row
//     attention kernel, and does nothing else;
//   - the matrix pipes: one wavefront per SIMD issues v_mfma_f32_32x32x16_bf16 back to back on
//     register operands (four independent accumulators), and nothing else; the shader clock it runs at
//     under that load is measured alongside (the part lowers its clock under matrix load).
// Not operations of the method; used by bench.py and documented in reader.h.
#include <hip/hip_runtime.h>

#include "internal.h"

namespace reader {

namespace {

constexpr int kCopyThreads = 512;             // 8 wavefronts, as the attention kernels
constexpr int kCopyTile = 32768;              // bytes per tile (64 keys x 256 bytes, K and V)
constexpr int kCopyStages = 4;

__global__ __launch_bounds__(kCopyThreads) void probe_copy_kernel(const char *src, long long tiles_per_wg,
                                                                    unsigned *sink) {
    extern __shared__ __attribute__((aligned(1024))) char ring[];
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const unsigned ring_lds = (unsigned)(size_t)(__attribute__((address_space(3))) char *)ring;
    const char *base = src + (size_t)blockIdx.x * (size_t)tiles_per_wg * kCopyTile;
    // a wavefront moves 4 KB of every tile with four 1 KB instructions
    auto issue = [&](long long t) {
        const char *from = base + (size_t)t * kCopyTile + wave * 4096;
        const unsigned to = ring_lds + (unsigned)(t % kCopyStages) * kCopyTile + wave * 4096;
#pragma unroll
        for (int i = 0; i < 4; ++i)
            asm volatile("s_mov_b32 m0, %2\n\tglobal_load_lds_dwordx4 %0, %1 nt"
                         :: "v"(lane * 16 + i * 1024), "s"(from), "s"(to + i * 1024) : "memory", "m0");
    };
    for (long long t = 0; t < kCopyStages - 1 && t < tiles_per_wg; ++t) issue(t);
    for (long long t = 0; t < tiles_per_wg; ++t) {
        // tile t has landed once at most the copies of the tiles asked for after it are outstanding
        const long long ahead = tiles_per_wg - 1 - t;
        if (ahead >= kCopyStages - 2) asm volatile("s_waitcnt vmcnt(8)");
        else if (ahead == 1) asm volatile("s_waitcnt vmcnt(4)");
        else asm volatile("s_waitcnt vmcnt(0)");
        __syncthreads();
        if (t + kCopyStages - 1 < tiles_per_wg) issue(t + kCopyStages - 1);
    }
    __syncthreads();
    if (threadIdx.x == 0) sink[blockIdx.x] = reinterpret_cast<const unsigned *>(ring)[blockIdx.x & 1023];
}

typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef float f32x16_t __attribute__((ext_vector_type(16)));

__global__ __launch_bounds__(256) void probe_mfma_kernel(int iters, float *sink, long long *clocks) {
    const int lane = threadIdx.x & 63;
    bf16x8_t a, b;
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        a[i] = (__bf16)(0.001f * lane + 0.37f * i - 1.0f);
        b[i] = (__bf16)(0.5f - 0.002f * lane + 0.11f * i);
    }
    f32x16_t c0, c1, c2, c3;
#pragma unroll
    for (int i = 0; i < 16; ++i) { c0[i] = 0.f; c1[i] = 0.f; c2[i] = 0.f; c3[i] = 0.f; }
    const long long t0 = __builtin_readcyclecounter(), r0 = (long long)__builtin_amdgcn_s_memrealtime();
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int k = 0; k < 16; ++k) {
            c0 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c0, 0, 0, 0);
            c1 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c1, 0, 0, 0);
            c2 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c2, 0, 0, 0);
            c3 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c3, 0, 0, 0);
        }
    }   // (the sums stay far inside fp32: 16 products of magnitude one per instruction and accumulator)
    const long long t1 = __builtin_readcyclecounter(), r1 = (long long)__builtin_amdgcn_s_memrealtime();
    float acc = 0.f;
#pragma unroll
    for (int i = 0; i < 16; ++i) acc += c0[i] + c1[i] + c2[i] + c3[i];
    sink[blockIdx.x * 256 + threadIdx.x] = acc;
    if (blockIdx.x == 0 && threadIdx.x == 0) { clocks[0] = t1 - t0; clocks[1] = r1 - r0; }
}

}  // namespace

hipError_t launch_probe_copy(const void *src, size_t bytes, void *scratch, hipStream_t stream, size_t *bytes_moved) {
    const long long tiles_per_wg = (long long)(bytes / ((size_t)kNumCU * kCopyTile));
    *bytes_moved = (size_t)tiles_per_wg * kNumCU * kCopyTile;
    if (tiles_per_wg < 1) return hipSuccess;
    // (asked for on every call: the attribute belongs to the device that is current, and the call is rare)
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(&probe_copy_kernel),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, kCopyStages * kCopyTile);
    if (e != hipSuccess) { (void)hipGetLastError(); return note_hip_error("hipFuncSetAttribute(copy probe)", e); }
    hipLaunchKernelGGL(probe_copy_kernel, dim3(kNumCU), dim3(kCopyThreads), kCopyStages * kCopyTile, stream,
                       static_cast<const char *>(src), tiles_per_wg, static_cast<unsigned *>(scratch));
    return note_hip_error("launch probe_copy_kernel", hipGetLastError());
}

hipError_t launch_probe_mfma(int iters, void *scratch, hipStream_t stream) {
    // scratch: 256 x 256 floats of sink, then two 64-bit clock readings
    float *sink = static_cast<float *>(scratch);
    long long *clocks = reinterpret_cast<long long *>(static_cast<char *>(scratch) + (size_t)kNumCU * 256 * sizeof(float));
    hipLaunchKernelGGL(probe_mfma_kernel, dim3(kNumCU), dim3(256), 0, stream, iters, sink, clocks);
    return note_hip_error("launch probe_mfma_kernel", hipGetLastError());
}

}  // namespace reader

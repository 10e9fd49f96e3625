// Kernels of reader_accept_path and reader_kv_compact (the device code is in accept_compact.h).
#include "accept_compact.h"

namespace reader {

__global__ __launch_bounds__(64) void accept_path_kernel(AcceptParams p) {
    __shared__ AcceptShared sh;
    accept_path_body(p, blockIdx.x, threadIdx.x, true, sh);
}

hipError_t launch_accept_path(const AcceptParams &p, hipStream_t stream) {
    hipLaunchKernelGGL(accept_path_kernel, dim3(p.B), dim3(64), 0, stream, p);
    return note_hip_error("launch accept_path_kernel", hipGetLastError());
}

__global__ __launch_bounds__(256) void kv_compact_kernel(CompactParams p) {
    __shared__ CompactShared cs;
    const int b = blockIdx.x;
    kv_compact_prefetch(p, b, threadIdx.x, cs);
    const int n = p.accept_len[b];
    __syncthreads();
    kv_compact_body(p, b, threadIdx.x, n, p.path + (size_t)b * p.max_path, cs);
}

hipError_t launch_kv_compact(const CompactParams &p, hipStream_t stream) {
    hipLaunchKernelGGL(kv_compact_kernel, dim3(p.B), dim3(256), 0, stream, p);
    return note_hip_error("launch kv_compact_kernel", hipGetLastError());
}

}  // namespace reader

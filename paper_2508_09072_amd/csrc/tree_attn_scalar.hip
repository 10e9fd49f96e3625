// Scalar cross-check kernel for reader_tree_attn (dims.variant = 1).
//
// One workgroup per output row (sequence, query head, tree node).  Every thread
// takes keys tid, tid+256, ... of  prefix || tree, scores them with plain fp32
// multiply-adds, keeps its own running (max, sum, weighted V) and the workgroup
// merges the 256 partial states at the end.  It re-reads the K/V stream once per
// row, so it is T*G times slower on memory traffic than the matrix-core kernel; it
// exists so that the two device implementations can be compared with each other.
#include "internal.h"

namespace reader {

__device__ inline float bf16_to_f32(uint16_t b) { return __uint_as_float(((uint32_t)b) << 16); }

__device__ inline uint16_t f32_to_bf16_rne(float f) {
    uint32_t u = __float_as_uint(f);
    if ((u & 0x7fffffffu) > 0x7f800000u) return (uint16_t)((u >> 16) | 0x40);  // NaN stays NaN
    u += 0x7fffu + ((u >> 16) & 1u);
    return (uint16_t)(u >> 16);
}

template <int D>
__global__ __launch_bounds__(256) void tree_attn_scalar_kernel(AttnParams p) {
    const int i = blockIdx.x, hq = blockIdx.y, b = blockIdx.z;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int hkv = hq / p.G;
    const int T = p.T;
    int L = p.seq_lens[b];
    L = L < 0 ? 0 : (L > p.max_seq_len ? p.max_seq_len : L);

    __shared__ float s_q[D];
    __shared__ uint32_t s_anc[4];
    __shared__ float s_m[4], s_l[4];
    __shared__ float s_acc[4][D];
    __shared__ int s_bad;

    if (tid == 0) {
        uint32_t anc[4] = {0u, 0u, 0u, 0u};
        int bad = 0;
        int t = i;
        for (int step = 0; step < T && t >= 0; ++step) {
            anc[t >> 5] |= 1u << (t & 31);
            int pt = p.parents[(size_t)b * T + t];
            if (t == 0 ? pt != -1 : (pt < 0 || pt >= t)) { bad |= READER_STATUS_BAD_TREE; pt = -1; }
            t = pt;
        }
        for (int w = 0; w < 4; ++w) s_anc[w] = anc[w];
        s_bad = bad;
    }
    if (tid < D) s_q[tid] = bf16_to_f32(p.q[(((size_t)b * T + i) * p.Hq + hq) * D + tid]) * p.scale_log2;
    __syncthreads();

    float m = -INFINITY, l = 0.f;
    float acc[D];
#pragma unroll
    for (int d = 0; d < D; ++d) acc[d] = 0.f;
    int bad = 0;

    for (int j = tid; j < L + T; j += 256) {
        const uint16_t *krow, *vrow;
        if (j < L) {
            const long long page = p.page_table[(size_t)b * p.max_pages + (j >> 4)];
            if (page < 0 || page >= p.num_pages) { bad |= READER_STATUS_BAD_PAGE; continue; }
            const size_t off = ((page * p.Hkv + hkv) * READER_PAGE_SIZE + (j & 15)) * (size_t)D;
            krow = p.k_cache + off;
            vrow = p.v_cache + off;
        } else {
            const int t = j - L;
            if (!((s_anc[t >> 5] >> (t & 31)) & 1u)) continue;
            if (p.tree_in_cache) {
                const int pos = L + t;      // below max_pages * 16: checked on the host
                const long long page = p.page_table[(size_t)b * p.max_pages + (pos >> 4)];
                if (page < 0 || page >= p.num_pages) { bad |= READER_STATUS_BAD_PAGE; continue; }
                const size_t off = ((page * p.Hkv + hkv) * READER_PAGE_SIZE + (pos & 15)) * (size_t)D;
                krow = p.k_cache + off;
                vrow = p.v_cache + off;
            } else {
                const size_t off = (((size_t)b * T + t) * p.Hkv + hkv) * (size_t)D;
                krow = p.k_tree + off;
                vrow = p.v_tree + off;
            }
        }
        float s = 0.f;
#pragma unroll
        for (int c = 0; c < D / 8; ++c) {
            const uint4 kk = *reinterpret_cast<const uint4 *>(krow + c * 8);
            const uint32_t w[4] = {kk.x, kk.y, kk.z, kk.w};
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                s += s_q[c * 8 + 2 * e] * __uint_as_float(w[e] << 16);
                s += s_q[c * 8 + 2 * e + 1] * __uint_as_float(w[e] & 0xffff0000u);
            }
        }
        const float m_new = fmaxf(m, s);
        const float alpha = exp2f(m - m_new);   // m = -inf on the first key gives 0
        const float pj = exp2f(s - m_new);
        l = l * alpha + pj;
#pragma unroll
        for (int c = 0; c < D / 8; ++c) {
            const uint4 vv = *reinterpret_cast<const uint4 *>(vrow + c * 8);
            const uint32_t w[4] = {vv.x, vv.y, vv.z, vv.w};
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                acc[c * 8 + 2 * e] = acc[c * 8 + 2 * e] * alpha + pj * __uint_as_float(w[e] << 16);
                acc[c * 8 + 2 * e + 1] = acc[c * 8 + 2 * e + 1] * alpha + pj * __uint_as_float(w[e] & 0xffff0000u);
            }
        }
        m = m_new;
    }

    // merge the 256 thread states: common max, rescale, sum
    float wm = m;
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) wm = fmaxf(wm, __shfl_xor(wm, off));
    if (lane == 0) s_m[wave] = wm;
    __syncthreads();
    const float gm = fmaxf(fmaxf(s_m[0], s_m[1]), fmaxf(s_m[2], s_m[3]));   // finite: the node sees itself
    const float f = (m == -INFINITY) ? 0.f : exp2f(m - gm);
    float wl = l * f;
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) wl += __shfl_xor(wl, off);
    if (lane == 0) s_l[wave] = wl;
#pragma unroll
    for (int d = 0; d < D; ++d) {
        float v = acc[d] * f;
#pragma unroll
        for (int off = 32; off >= 1; off >>= 1) v += __shfl_xor(v, off);
        if (lane == 0) s_acc[wave][d] = v;
    }
    __syncthreads();
    const float gl = s_l[0] + s_l[1] + s_l[2] + s_l[3];
    if (tid < D) {
        const float o = (s_acc[0][tid] + s_acc[1][tid] + s_acc[2][tid] + s_acc[3][tid]) / gl;
        p.out[(((size_t)b * T + i) * p.Hq + hq) * D + tid] = f32_to_bf16_rne(o);
    }
    if (tid == 0 && p.lse) p.lse[((size_t)b * p.Hq + hq) * T + i] = (gm + log2f(gl)) * 0.69314718055994530942f;

    bad = __syncthreads_or(bad);
    if (tid == 0 && p.status && (bad || s_bad))
        atomicOr(p.status, (bad ? READER_STATUS_BAD_PAGE : 0) | s_bad);
}

hipError_t launch_tree_attn_scalar(const AttnParams &p, hipStream_t stream) {
    dim3 grid(p.T, p.Hq, p.B);
    if (p.D == 64)
        hipLaunchKernelGGL(tree_attn_scalar_kernel<64>, grid, dim3(256), 0, stream, p);
    else
        hipLaunchKernelGGL(tree_attn_scalar_kernel<128>, grid, dim3(256), 0, stream, p);
    return note_hip_error("launch tree_attn_scalar_kernel", hipGetLastError());
}

}  // namespace reader

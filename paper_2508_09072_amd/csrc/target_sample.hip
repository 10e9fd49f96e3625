// The base model's tokens under a sampling policy with coupled uniforms (Appendix C,
// randomized decoding): the policy is a map F(distribution, u) with one uniform per decoding
// position, shared by the plain run and the speculative run.  Here F is inverse-CDF sampling of
// softmax(logits / temperature): the lowest index whose cumulative probability exceeds u.
// Node n of sequence b stands for the position depth(n) behind the root, so all nodes of one
// depth draw with the same uniform, uniforms[b][depth(n)].
//
// One workgroup per (sequence, node) row, one pass over the row (256 KB at vocabulary 128256,
// as large as the step's KV stream): the row is cut into slots of 2048 consecutive tokens (four
// 16-byte loads per lane), a wavefront reduces a slot to (maximum, sum of exp relative to that
// maximum) and leaves the pair in LDS; the slots' sums, brought to the row maximum, are scanned
// in index order to find the slot that crosses u * total, and only that slot (4 KB, still in
// cache) is read again to find the token.  All sums are fp32: where u * total falls within rounding of a
// token boundary the neighbouring token may come out.
#include <stdlib.h>

#include "internal.h"

namespace reader {

namespace {

constexpr int kGroup = 4;            // 512-token blocks (64 lanes x 8 tokens) per slot

// Wavefront reductions on the vector ALU's lane-crossing paths (no LDS traffic): four shifts
// inside each row of 16 lanes leave the row's result in its last lane, two row broadcasts
// carry it on to lane 63, which is read back as a wavefront-uniform value.
template <int kCtrl, int kRowMask>
__device__ inline float dpp_from(float identity, float v) {
    return __int_as_float(__builtin_amdgcn_update_dpp(__float_as_int(identity), __float_as_int(v), kCtrl, kRowMask, 0xf, false));
}
__device__ inline float wave_max(float v) {
    v = fmaxf(v, dpp_from<0x111, 0xf>(-INFINITY, v));   // row_shr:1
    v = fmaxf(v, dpp_from<0x112, 0xf>(-INFINITY, v));   // row_shr:2
    v = fmaxf(v, dpp_from<0x114, 0xf>(-INFINITY, v));   // row_shr:4
    v = fmaxf(v, dpp_from<0x118, 0xf>(-INFINITY, v));   // row_shr:8
    v = fmaxf(v, dpp_from<0x142, 0xa>(-INFINITY, v));   // row_bcast:15 into rows 1 and 3
    v = fmaxf(v, dpp_from<0x143, 0xc>(-INFINITY, v));   // row_bcast:31 into rows 2 and 3
    return __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), 63));
}
__device__ inline float wave_sum(float v) {
    v += dpp_from<0x111, 0xf>(0.f, v);
    v += dpp_from<0x112, 0xf>(0.f, v);
    v += dpp_from<0x114, 0xf>(0.f, v);
    v += dpp_from<0x118, 0xf>(0.f, v);
    v += dpp_from<0x142, 0xa>(0.f, v);
    v += dpp_from<0x143, 0xc>(0.f, v);
    return __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), 63));
}
// Scaled logits never exceed this: a +inf logit (or a product that overflows) sits exactly
// there, so that it takes all the probability, shared among equals, instead of producing NaNs.
constexpr float kCeil = 0x1p127f;
// bf16 bits -> logit * c as fp32; a NaN carries no probability
__device__ inline float scaled(uint32_t bits16_hi, float c) {
    const float x = __uint_as_float(bits16_hi);
    return x != x ? -INFINITY : fminf(x * c, kCeil);
}
// A weight relative to its slot's maximum lies in [0, 1] (rounding may leave the largest a hair above); the
// weight of a NaN logit is a NaN and becomes 0 here.  Written so that the compiler folds it into the
// instruction that makes the weight (its result clamp), at no cost.
__device__ inline float unit_clamp(float w) { return fminf(fmaxf(w, 0.f), 1.f); }
__device__ inline void unpack8(const uint4 &w, float c, float y[8]) {
    const uint32_t u[4] = {w.x, w.y, w.z, w.w};
#pragma unroll
    for (int e = 0; e < 4; ++e) {
        y[2 * e] = scaled(u[e] << 16, c);
        y[2 * e + 1] = scaled(u[e] & 0xffff0000u, c);
    }
}

// Row layout: `head` tokens in front of the first 16-byte boundary, n_vec groups of 8 tokens,
// a tail of fewer than 8.  Statistics slot 0 is the head, slot 1 + k block k of the aligned
// part, the last slot the tail.
// kSampleThreads: 512, or 1024 when the launch has few rows (more loads in flight per row).
template <int kSampleThreads>
__global__ __launch_bounds__(kSampleThreads) void target_sample_kernel(const uint16_t *__restrict__ logits,
                                                                       const int32_t *__restrict__ parents,
                                                                       const float *__restrict__ uniforms,
                                                                       int32_t *__restrict__ out, int T, int V, float c) {
    constexpr int kSampleWaves = kSampleThreads / 64;
    extern __shared__ float2 s_stat[];        // (maximum, sum) per slot
    __shared__ int s_par[READER_MAX_T];
    __shared__ float s_wsum[kSampleWaves];
    __shared__ int s_pick[2];                 // slot that crosses the threshold, stand-in
    __shared__ float s_thr, s_front;          // threshold; weight in front of the chosen slot
    const int row = blockIdx.x, tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int b = row / T, node = row - b * T;
    const uint16_t *src = logits + (size_t)row * V;
    if (tid < T) s_par[tid] = parents[(size_t)b * T + tid];

    const int head = min(V, (int)(((16 - ((uintptr_t)src & 15)) & 15) >> 1));
    const int n_vec = (V - head) / 8;
    const int n_blocks = (n_vec + 63) / 64, n_groups = (n_blocks + kGroup - 1) / kGroup;
    const int tail_at = head + n_vec * 8, n_slots = n_groups + 2;
    const uint4 *vec = reinterpret_cast<const uint4 *>(src + head);

    // head and tail: at most 7 tokens each, wavefront 0 and 1
    if (wave < 2) {
        const int at = wave == 0 ? 0 : tail_at, cnt = wave == 0 ? head : V - tail_at;
        const float y = lane < cnt ? scaled((uint32_t)src[at + lane] << 16, c) : -INFINITY;
        const float m = wave_max(y);
        const float s = wave_sum(m == -INFINITY ? 0.f : __builtin_amdgcn_exp2f(y - m));
        if (lane == 0) s_stat[wave == 0 ? 0 : n_slots - 1] = make_float2(m, s);
    }
    // slots: a wavefront takes the four blocks of a slot at once.  Per token: widen, half a three-way
    // maximum, one fused multiply-add, exp2 (a NaN becomes weight 0 in its result clamp), add;
    // per slot: one maximum and one sum across the wavefront.  Lanes past the end of the row hold
    // -inf bit patterns, so nothing is selected per token.
    const uint4 nothing = make_uint4(0xff80ff80u, 0xff80ff80u, 0xff80ff80u, 0xff80ff80u);
    for (int grp = wave; grp < n_groups; grp += kSampleWaves) {
        uint4 w[kGroup];
#pragma unroll
        for (int j = 0; j < kGroup; ++j) {
            const int g = (grp * kGroup + j) * 64 + lane;
            w[j] = g < n_vec ? load_stream16(vec + g) : nothing;
        }
        float x[8 * kGroup];
#pragma unroll
        for (int j = 0; j < kGroup; ++j) {
            const uint32_t u[4] = {w[j].x, w[j].y, w[j].z, w[j].w};
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                x[8 * j + 2 * e] = __uint_as_float(u[e] << 16);
                x[8 * j + 2 * e + 1] = __uint_as_float(u[e] & 0xffff0000u);
            }
        }
        // (the maximum of a NaN and a number is the number: a NaN never becomes the maximum unless all are)
        float m = fmaxf(x[0], -INFINITY);
#pragma unroll
        for (int e = 1; e < 8 * kGroup; e += 2) m = fmaxf(fmaxf(m, x[e]), e + 1 < 8 * kGroup ? x[e + 1] : -INFINITY);
        m = wave_max(m);
        float s0 = 0.f, s1 = 0.f, m_store;
        if (m * c < kCeil) {                              // (wavefront-uniform)
            const float mc = fmaxf(m, -0x1p126f) * c;     // a slot of nothing but -inf: every weight becomes exp2(-inf) = 0
#pragma unroll
            for (int e = 0; e < 8 * kGroup; e += 2) {
                s0 += unit_clamp(__builtin_amdgcn_exp2f(__builtin_fmaf(x[e], c, -mc)));
                s1 += unit_clamp(__builtin_amdgcn_exp2f(__builtin_fmaf(x[e + 1], c, -mc)));
            }
            m_store = m * c;
        } else {
            // a +inf logit, or one so large that scaling overflows: go through the clamped values
#pragma unroll
            for (int e = 0; e < 8 * kGroup; e += 2) {
                s0 += __builtin_amdgcn_exp2f(fminf(fmaxf(x[e], -INFINITY) * c, kCeil) - kCeil);
                s1 += __builtin_amdgcn_exp2f(fminf(fmaxf(x[e + 1], -INFINITY) * c, kCeil) - kCeil);
            }
            m_store = kCeil;                              // some token of the slot sits at the ceiling
        }
        const float s = wave_sum(s0 + s1);
        if (lane == 0) s_stat[1 + grp] = make_float2(m_store, s);
    }
    __syncthreads();

    // depth of the node -> its uniform (a parent pointer that does not lead towards the root
    // ends the walk: the tree checks belong to reader_validate_tree / the attention kernel)
    float u = 0.f;
    if (tid == 0) {
        int n = node, d = 0;
        while (n > 0 && d < T) {
            const int pn = s_par[n];
            if (pn < 0 || pn >= n) break;
            n = pn;
            ++d;
        }
        u = uniforms[(size_t)b * T + d];
        u = u < 0.f ? 0.f : u;
    }

    // row maximum, then the slots' weights relative to it, scanned in index order
    float m_row = -INFINITY;
    for (int i = tid; i < n_slots; i += kSampleThreads) m_row = fmaxf(m_row, s_stat[i].x);
    m_row = wave_max(m_row);
    if (lane == 0) s_wsum[wave] = m_row;
    __syncthreads();
    m_row = s_wsum[0];
#pragma unroll
    for (int w = 1; w < kSampleWaves; ++w) m_row = fmaxf(m_row, s_wsum[w]);
    __syncthreads();
    if (m_row == -INFINITY) {           // no token has any probability
        if (tid == 0) out[row] = 0;
        return;
    }
    // thread t owns the slots [t * per, (t + 1) * per): its weight, then an exclusive scan over threads
    const int per = (n_slots + kSampleThreads - 1) / kSampleThreads;
    float mine = 0.f;
    for (int i = tid * per; i < min(n_slots, (tid + 1) * per); ++i) {
        const float2 st = s_stat[i];
        const float wgt = st.x == -INFINITY ? 0.f : st.y * __builtin_amdgcn_exp2f(st.x - m_row);
        s_stat[i].y = wgt;              // the slot's weight relative to the row maximum
        mine += wgt;
    }
    float incl = mine;
#pragma unroll
    for (int off = 1; off < 64; off <<= 1) {
        const float t = __shfl_up(incl, off);
        if (lane >= off) incl += t;
    }
    if (lane == 63) s_wsum[wave] = incl;
    __syncthreads();
    float before = incl - mine;
    for (int w = 0; w < wave; ++w) before += s_wsum[w];
    float total = 0.f;
#pragma unroll
    for (int w = 0; w < kSampleWaves; ++w) total += s_wsum[w];
    if (tid == 0) {
        // u * total, kept below the total so that some slot crosses it
        const float t = u * total, cap = total * (1.f - 0x1p-23f);
        s_thr = t < cap ? t : cap;
        s_pick[0] = 0x7fffffff;
        s_pick[1] = -1;
    }
    __syncthreads();
    const float thr = s_thr;
    // The slot that crosses the threshold: the first whose cumulative weight exceeds it.  Each
    // thread looks at its own slots; rounding of the per-thread sums may let no thread (or two)
    // see the crossing, so the lowest claimed slot wins, and the last slot with weight that
    // starts at or below the threshold stands in when nobody claims.
    {
        float cum = before;
        for (int i = tid * per; i < min(n_slots, (tid + 1) * per); ++i) {
            const float wgt = s_stat[i].y;
            if (wgt > 0.f && cum <= thr) {
                atomicMax(&s_pick[1], i);
                if (thr < cum + wgt) atomicMin(&s_pick[0], i);
            }
            cum += wgt;
        }
    }
    __syncthreads();
    const int slot = s_pick[0] != 0x7fffffff ? s_pick[0] : s_pick[1];   // >= 0: the first slot with weight starts at 0
    if (slot < 0 || slot >= n_slots) {   // only if the weights were not numbers at all: never index with it
        if (tid == 0) out[row] = 0;
        return;
    }
    {
        float cum = before;
        for (int i = tid * per; i < min(n_slots, (tid + 1) * per); ++i) {
            if (i == slot) s_front = cum;      // weight in front of the slot
            cum += s_stat[i].y;
        }
    }
    __syncthreads();
    const float front = s_front;

    // inside the slot: wavefront 0 reads its tokens again and scans their weights in index order,
    // block by block (a lane's 8 tokens are consecutive, the lanes of a block follow each other)
    if (wave == 0) {
        const bool edge = slot == 0 || slot == n_slots - 1;      // head or tail: up to 7 tokens, one per lane
        float carry = front;
        int pick = 0x7fffffff, last_pos = -1;
        // (the four blocks of the slot are asked for together: one trip to memory, not four)
        uint4 again[kGroup];
#pragma unroll
        for (int j = 0; j < kGroup; ++j) {
            const int g = ((slot - 1) * kGroup + j) * 64 + lane;
            again[j] = (!edge && g < n_vec) ? vec[g] : nothing;
        }
#pragma unroll
        for (int j = 0; j < kGroup; ++j) {
            if (edge && j > 0) break;
            float y[8];
            int first, cnt;              // this lane's tokens: indices first .. first + cnt - 1
            if (edge) {
                const int at = slot == 0 ? 0 : tail_at, n_here = slot == 0 ? head : V - tail_at;
                first = at + lane;
                cnt = lane < n_here ? 1 : 0;
                y[0] = cnt ? scaled((uint32_t)src[first] << 16, c) : -INFINITY;
#pragma unroll
                for (int e = 1; e < 8; ++e) y[e] = -INFINITY;
            } else {
                const int g = ((slot - 1) * kGroup + j) * 64 + lane;
                cnt = g < n_vec ? 8 : 0;
                first = head + g * 8;
                unpack8(again[j], c, y);
                if (!cnt) {
#pragma unroll
                    for (int e = 0; e < 8; ++e) y[e] = -INFINITY;
                }
            }
            float wgt[8], lane_sum = 0.f;
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                wgt[e] = y[e] == -INFINITY ? 0.f : __builtin_amdgcn_exp2f(y[e] - m_row);
                lane_sum += wgt[e];
            }
            float incl_l = lane_sum;
#pragma unroll
            for (int off = 1; off < 64; off <<= 1) {
                const float t = __shfl_up(incl_l, off);
                if (lane >= off) incl_l += t;
            }
            float cum = carry + (incl_l - lane_sum);
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                if (e < cnt && wgt[e] > 0.f) {
                    if (pick == 0x7fffffff && thr < cum + wgt[e]) pick = first + e;
                    last_pos = first + e;
                }
                cum += wgt[e];
            }
            carry += __shfl(incl_l, 63);
        }
#pragma unroll
        for (int off = 32; off >= 1; off >>= 1) {
            pick = min(pick, __shfl_xor(pick, off));
            last_pos = max(last_pos, __shfl_xor(last_pos, off));
        }
        // the slot's own sum, added up in another order, may stop just short of the threshold
        if (lane == 0) out[row] = pick != 0x7fffffff ? pick : (last_pos >= 0 ? last_pos : 0);
    }
}

}  // namespace

hipError_t launch_target_sample(const uint16_t *logits, const int32_t *parents, const float *uniforms, int32_t *out,
                                int B, int T, int V, float temperature, hipStream_t stream) {
    // one (maximum, sum) slot per kGroup blocks of 512 tokens, plus the unaligned head and tail of the row
    // (the kernel computes the same number from the row's alignment; this is its upper bound)
    const int n_slots = ((V / 8 + 63) / 64 + kGroup - 1) / kGroup + 2;
    const float c = 1.44269504088896340736f / temperature;
    const int nt = (long long)B * T <= 384 ? 1024 : 512;   // (measured: equal at 512 rows, 512 threads ahead beyond)
    if (nt == 1024)
        hipLaunchKernelGGL(target_sample_kernel<1024>, dim3(B * T), dim3(1024), (size_t)n_slots * sizeof(float2), stream,
                           logits, parents, uniforms, out, T, V, c);
    else
        hipLaunchKernelGGL(target_sample_kernel<512>, dim3(B * T), dim3(512), (size_t)n_slots * sizeof(float2), stream,
                           logits, parents, uniforms, out, T, V, c);
    return note_hip_error("launch target_sample_kernel", hipGetLastError());
}

}  // namespace reader

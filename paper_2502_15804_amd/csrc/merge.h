// Log-sum-exp merge of the token chunks of each (sequence, KV head) pair.
#pragma once
#include "common.h"

namespace fairkv {

// Combine the chunks of a pair:  m* = max_c m_c,  l* = sum_c l_c 2^(m_c - m*),
// out = sum_c o_c 2^(m_c - m*) / l*.  Exact in real arithmetic, so chunked equals unchunked.
// One workgroup per pair; a thread owns four consecutive output coordinates of one query
// head and fetches the partials of up to kBatch chunks at once so that their latencies
// overlap.  Pairs that were a single item were already written by the decode kernel; pairs
// without tokens get out = 0, lse = -inf here.
constexpr int kMergeBatch = 8;

__global__ __launch_bounds__(kThreads) void fairkv_merge_kernel(const float *__restrict__ part_o,
                                                               const float *__restrict__ part_ml,
                                                               const int32_t *__restrict__ part_base, void *out,
                                                               float *lse, int Hq, int Hkv, int G, int D,
                                                               int out_dtype)
{
    const int pair = blockIdx.x;
    const int b = pair / Hkv, h = pair % Hkv;
    const int p0 = part_base[pair];
    const int nc = part_base[pair + 1] - p0;
    if (nc == 1) return;
    const int d4n = D / 4;
    for (int idx = threadIdx.x; idx < G * d4n; idx += kThreads) {
        const int g = idx / d4n, d = (idx % d4n) * 4;
        float m_star = -INFINITY, l_star = 0.f;
        float acc[4] = {0.f, 0.f, 0.f, 0.f};
        for (int c0 = 0; c0 < nc; c0 += kMergeBatch) {
            float4 o[kMergeBatch];
            float2 ml[kMergeBatch];
#pragma unroll
            for (int j = 0; j < kMergeBatch; ++j) {
                const int c = min(c0 + j, nc - 1);     // past the end: re-read the last chunk, weight 0 below
                const size_t pg = static_cast<size_t>(p0 + c) * G + g;
                ml[j] = *reinterpret_cast<const float2 *>(part_ml + pg * 2);
                o[j] = *reinterpret_cast<const float4 *>(part_o + pg * D + d);
            }
            float m_new = m_star;
#pragma unroll
            for (int j = 0; j < kMergeBatch; ++j)
                if (c0 + j < nc) m_new = fmaxf(m_new, ml[j].x);
            const float keep = m_star == -INFINITY ? 0.f : __builtin_amdgcn_exp2f(m_star - m_new);
            l_star *= keep;
#pragma unroll
            for (int e = 0; e < 4; ++e) acc[e] *= keep;
#pragma unroll
            for (int j = 0; j < kMergeBatch; ++j) {
                const bool live = c0 + j < nc && ml[j].x != -INFINITY;
                const float f = live ? __builtin_amdgcn_exp2f(ml[j].x - m_new) : 0.f;
                l_star = fmaf(ml[j].y, f, l_star);
                acc[0] = fmaf(o[j].x, f, acc[0]);
                acc[1] = fmaf(o[j].y, f, acc[1]);
                acc[2] = fmaf(o[j].z, f, acc[2]);
                acc[3] = fmaf(o[j].w, f, acc[3]);
            }
            m_star = m_new;
        }
        const size_t oi = (static_cast<size_t>(b) * Hq + h * G + g) * D + d;
        const float inv = l_star > 0.f ? 1.f / l_star : 0.f;
#pragma unroll
        for (int e = 0; e < 4; ++e) store_out(out, out_dtype, oi + e, acc[e] * inv);
        if (d == 0 && lse)
            lse[b * Hq + h * G + g] = l_star > 0.f ? (m_star + __builtin_amdgcn_logf(l_star)) * kLn2 : -INFINITY;
    }
}

}  // namespace fairkv

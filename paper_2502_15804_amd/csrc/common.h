// Shared pieces of the decode kernels: argument block, layout facts, small device helpers,
// and the workgroup epilogue that folds the waves of a workgroup and writes either the
// final output (an item that is a whole pair) or the item's partial result.
#pragma once
#include <hip/hip_runtime.h>

#include <cmath>
#include <cstdint>

#include "fairkv.h"

namespace fairkv {

constexpr int kWaves = 4;                 // waves per workgroup
constexpr int kThreads = kWaves * 64;
constexpr int kTile = 64;                 // tokens a wave handles per step: one per lane
constexpr float kLog2e = 1.4426950408889634f;
constexpr float kLn2 = 0.6931471805599453f;

typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2_t;

__device__ __forceinline__ float wave_max(float x)
{
#pragma unroll
    for (int o = 32; o >= 1; o >>= 1) x = fmaxf(x, __shfl_xor(x, o, 64));
    return x;
}

__device__ __forceinline__ float wave_sum(float x)
{
#pragma unroll
    for (int o = 32; o >= 1; o >>= 1) x += __shfl_xor(x, o, 64);
    return x;
}

__device__ __forceinline__ float bf16_lo(uint32_t w) { return __uint_as_float(w << 16); }
__device__ __forceinline__ float bf16_hi(uint32_t w) { return __uint_as_float(w & 0xffff0000u); }

__device__ __forceinline__ uint16_t f32_to_bf16_rne(float f)
{
    uint32_t u = __float_as_uint(f);
    if ((u & 0x7fffffffu) > 0x7f800000u) return static_cast<uint16_t>((u >> 16) | 0x40u);  // NaN
    u += 0x7fffu + ((u >> 16) & 1u);
    return static_cast<uint16_t>(u >> 16);
}

__device__ __forceinline__ void store_out(void *out, int out_dtype, size_t idx, float x)
{
    if (out_dtype == FAIRKV_F32)
        static_cast<float *>(out)[idx] = x;
    else
        static_cast<uint16_t *>(out)[idx] = f32_to_bf16_rne(x);
}

struct DecodeArgs {
    const void *q, *k, *v;
    const int64_t *off;
    const int32_t *len;
    const fairkv_item *items;
    float *part_o;    // [n_parts][G][D]   unnormalised outputs relative to the item's maximum
    float *part_ml;   // [n_parts][G][2]   (maximum in log2 units, sum of weights)
    void *out;
    float *lse;
    int32_t B, Hq, Hkv, out_dtype;
    float scale_log2;  // scale * log2(e): scores are kept in log2 units so exp is one v_exp_f32
};

// Layout facts shared by the stages.  A row of K or V is LPR 16-byte pieces; one wave-wide
// 16-byte-per-lane access covers RPI whole rows, so every global access is a run of
// contiguous, fully used cache lines.
template <int IN_DT, int D>
struct Geo {
    static constexpr int ES = IN_DT == FAIRKV_BF16 ? 2 : 4;
    static constexpr int ROW_BYTES = D * ES;
    static constexpr int LPR = ROW_BYTES / 16;   // lanes (16-byte pieces) per row
    static constexpr int RPI = 64 / LPR;         // rows per wave-wide access
    static constexpr int NI = kTile / RPI;       // wave-wide accesses per 64-token tile
    static constexpr int EPC = 16 / ES;          // elements per 16-byte piece
    static constexpr int DW = ROW_BYTES / 4;     // dwords per row
};


// Workgroup epilogue.  st_o [kWaves][G][D] and st_ml [kWaves][G][2] in LDS hold each wave's
// unnormalised output, running maximum (log2 units) and weight sum.  Combines them with
//   m* = max_w m_w,  l* = sum_w l_w 2^(m_w - m*),  o* = sum_w o_w 2^(m_w - m*)
// and writes out = o*/l* and lse when the item is the whole pair, else the partial (m*, l*, o*).
template <int D, int G>
__device__ __forceinline__ void workgroup_epilogue(const DecodeArgs &a, const fairkv_item &it, const float *st_o,
                                                   const float *st_ml)
{
    const int b = it.b, h = it.h;
    const bool whole_pair = it.n_chunks == 1;
    for (int idx = threadIdx.x; idx < G * D; idx += kThreads) {
        const int g = idx / D, d = idx % D;
        float m_star = -INFINITY;
#pragma unroll
        for (int w = 0; w < kWaves; ++w) m_star = fmaxf(m_star, st_ml[(w * G + g) * 2]);
        float acc = 0.f, l_star = 0.f;
#pragma unroll
        for (int w = 0; w < kWaves; ++w) {
            const float mw = st_ml[(w * G + g) * 2];
            const float f = mw == -INFINITY ? 0.f : __builtin_amdgcn_exp2f(mw - m_star);
            acc += st_o[(w * G + g) * D + d] * f;
            l_star += st_ml[(w * G + g) * 2 + 1] * f;
        }
        if (whole_pair) {
            const size_t oi = (static_cast<size_t>(b) * a.Hq + h * G + g) * D + d;
            store_out(a.out, a.out_dtype, oi, l_star > 0.f ? acc / l_star : 0.f);
            if (d == 0 && a.lse)
                a.lse[b * a.Hq + h * G + g] =
                    l_star > 0.f ? (m_star + __builtin_amdgcn_logf(l_star)) * kLn2 : -INFINITY;
        } else {
            a.part_o[(static_cast<size_t>(it.part) * G + g) * D + d] = acc;
            if (d == 0) {
                a.part_ml[(static_cast<size_t>(it.part) * G + g) * 2 + 0] = m_star;
                a.part_ml[(static_cast<size_t>(it.part) * G + g) * 2 + 1] = l_star;
            }
        }
    }
}

}  // namespace fairkv

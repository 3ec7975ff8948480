// Split-KV decode attention over a packed ragged KV cache, and the log-sum-exp merge of
// token chunks, for gfx950 (wave64, 256 compute units).
//
// The paper (Section 3.2) observes that decoding one token is bound by memory bandwidth
// and costs time linear in batch x retained tokens, so the job of these kernels is to
// stream every retained K and V row from HBM exactly once, at full rate, whatever the
// per-head lengths are.  One workgroup takes one work item of the plan (a token chunk of
// one (sequence, KV head) pair) and serves all G query heads of the group from the same
// K/V rows.  Heavy pairs arrive cut into several items (the single-GPU form of
// Fair-Copying, Section 4.2); their partial results are combined by the merge kernel.
#include <hip/hip_runtime.h>

#include <cmath>
#include <cstdint>

#include "fairkv.h"

namespace {

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

template <int IN_DT, int D, int G>
__global__ __launch_bounds__(kThreads, 2) void fairkv_decode_kernel(DecodeArgs a)
{
    using geo = Geo<IN_DT, D>;
    constexpr int LPR = geo::LPR, RPI = geo::RPI, NI = geo::NI, EPC = geo::EPC, DW = geo::DW;
    constexpr int ROW_BYTES = geo::ROW_BYTES;

    // K tile per wave, 16-byte pieces; piece p of row r sits at column p ^ (r % LPR) so that
    // both the row-contiguous fill and the one-row-per-lane read are free of bank conflicts.
    __shared__ uint4 lds_k[kWaves][kTile * LPR];
    __shared__ float lds_p[kWaves][kTile][G];

    const int lane = threadIdx.x & 63;
    const int wave = threadIdx.x >> 6;

    const fairkv_item it = a.items[blockIdx.x];
    const int b = it.b, h = it.h;
    // an item that does not belong to this problem is skipped by the whole workgroup
    if (b < 0 || b >= a.B || h < 0 || h >= a.Hkv || it.tok_begin < 0 || it.part < 0) return;
    const int pair = b * a.Hkv + h;
    const int64_t row0 = a.off[pair] + it.tok_begin;
    int n = min(it.tok_count, a.len[pair] - it.tok_begin);   // never read past the pair's rows
    n = max(n, 0);
    const int n_tiles = (n + kTile - 1) / kTile;

    const char *kbase = static_cast<const char *>(a.k) + row0 * ROW_BYTES;
    const char *vbase = static_cast<const char *>(a.v) + row0 * ROW_BYTES;
    const uint32_t *qrow = static_cast<const uint32_t *>(a.q) + static_cast<size_t>(b * a.Hq + h * G) * DW;

    const int my_piece = lane % LPR;   // which 16 bytes of a row this lane moves / accumulates
    const int my_sub = lane / LPR;     // which of the RPI rows of a wave-wide access

    float o[G][EPC];
    float m_run[G], l_lane[G];
#pragma unroll
    for (int g = 0; g < G; ++g) {
        m_run[g] = -INFINITY;
        l_lane[g] = 0.f;
#pragma unroll
        for (int e = 0; e < EPC; ++e) o[g][e] = 0.f;
    }

    for (int tile = wave; tile < n_tiles; tile += kWaves) {
        const int t0 = tile * kTile;
        const int nv = min(kTile, n - t0);          // valid rows of this tile (>= 1)

        // ---- fetch: K rows into LDS (swizzled), V rows into registers --------------------
        uint4 kreg[NI], vreg[NI];
#pragma unroll
        for (int i = 0; i < NI; ++i) {
            const int r = i * RPI + my_sub;
            const int rc = min(r, nv - 1);          // rows past the end re-read the last valid row
            const int piece = my_piece ^ (r % LPR);
            kreg[i] = *reinterpret_cast<const uint4 *>(kbase + static_cast<size_t>(t0 + rc) * ROW_BYTES + piece * 16);
        }
#pragma unroll
        for (int i = 0; i < NI; ++i) {
            const int r = i * RPI + my_sub;
            const int rc = min(r, nv - 1);
            vreg[i] = *reinterpret_cast<const uint4 *>(vbase + static_cast<size_t>(t0 + rc) * ROW_BYTES + my_piece * 16);
        }
#pragma unroll
        for (int i = 0; i < NI; ++i) lds_k[wave][(i * RPI + my_sub) * LPR + my_piece] = kreg[i];
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup");

        // ---- scores: lane t owns token t0 + t and all G query heads ----------------------
        float s[G];
#pragma unroll
        for (int g = 0; g < G; ++g) s[g] = 0.f;
#pragma unroll
        for (int c = 0; c < LPR; ++c) {
            const uint4 kk = lds_k[wave][lane * LPR + (c ^ (lane % LPR))];
            const uint32_t kw[4] = {kk.x, kk.y, kk.z, kk.w};
#pragma unroll
            for (int j = 0; j < 4; ++j) {
#pragma unroll
                for (int g = 0; g < G; ++g) {
                    const uint32_t qw = qrow[g * DW + c * 4 + j];   // wave-uniform: a scalar load
                    if constexpr (IN_DT == FAIRKV_BF16) {
                        s[g] = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2_t, qw),
                                                               __builtin_bit_cast(bf16x2_t, kw[j]), s[g], false);
                    } else {
                        s[g] = fmaf(__uint_as_float(qw), __uint_as_float(kw[j]), s[g]);
                    }
                }
            }
        }

        // ---- online softmax in log2 units ------------------------------------------------
#pragma unroll
        for (int g = 0; g < G; ++g) {
            const float sv = lane < nv ? s[g] * a.scale_log2 : -INFINITY;
            const float m_new = fmaxf(m_run[g], wave_max(sv));
            const float alpha = __builtin_amdgcn_exp2f(m_run[g] - m_new);   // 0 on the first tile
            const float p = __builtin_amdgcn_exp2f(sv - m_new);
            l_lane[g] = l_lane[g] * alpha + p;
            m_run[g] = m_new;
#pragma unroll
            for (int e = 0; e < EPC; ++e) o[g][e] *= alpha;
            lds_p[wave][lane][g] = p;
        }
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup");

        // ---- weighted sum: lane owns EPC output coordinates, rows r = i*RPI + my_sub ------
#pragma unroll
        for (int i = 0; i < NI; ++i) {
            const int r = i * RPI + my_sub;
            float vf[EPC];
            const uint32_t vw[4] = {vreg[i].x, vreg[i].y, vreg[i].z, vreg[i].w};
            if constexpr (IN_DT == FAIRKV_BF16) {
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    vf[2 * j] = bf16_lo(vw[j]);
                    vf[2 * j + 1] = bf16_hi(vw[j]);
                }
            } else {
#pragma unroll
                for (int j = 0; j < 4; ++j) vf[j] = __uint_as_float(vw[j]);
            }
            if (r >= nv) {   // the re-read row must not contribute, even if it holds inf or NaN
#pragma unroll
                for (int e = 0; e < EPC; ++e) vf[e] = 0.f;
            }
#pragma unroll
            for (int g = 0; g < G; ++g) {
                const float p = lds_p[wave][r][g];
#pragma unroll
                for (int e = 0; e < EPC; ++e) o[g][e] = fmaf(p, vf[e], o[g][e]);
            }
        }
        __builtin_amdgcn_wave_barrier();
    }

    // ---- fold the RPI row groups of a wave, then the waves of the workgroup ---------------
#pragma unroll
    for (int g = 0; g < G; ++g) {
#pragma unroll
        for (int e = 0; e < EPC; ++e) {
#pragma unroll
            for (int s = LPR; s < 64; s <<= 1) o[g][e] += __shfl_xor(o[g][e], s, 64);
        }
        l_lane[g] = wave_sum(l_lane[g]);
    }

    __syncthreads();   // every wave is done with its K tile: reuse that memory
    float *st_o = reinterpret_cast<float *>(&lds_k[0][0]);   // [kWaves][G][D]
    float *st_ml = st_o + kWaves * G * D;                    // [kWaves][G][2]
    static_assert(sizeof(float) * (kWaves * G * (D + 2)) <= sizeof(uint4) * kWaves * kTile * LPR,
                  "merge staging must fit in the K tiles");
    if (my_sub == 0) {
#pragma unroll
        for (int g = 0; g < G; ++g)
#pragma unroll
            for (int e = 0; e < EPC; ++e) st_o[(wave * G + g) * D + my_piece * EPC + e] = o[g][e];
    }
    if (lane == 0) {
#pragma unroll
        for (int g = 0; g < G; ++g) {
            st_ml[(wave * G + g) * 2 + 0] = m_run[g];
            st_ml[(wave * G + g) * 2 + 1] = l_lane[g];
        }
    }
    __syncthreads();

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
                a.lse[b * a.Hq + h * G + g] = l_star > 0.f ? (m_star + __builtin_amdgcn_logf(l_star)) * kLn2 : -INFINITY;
        } else {
            a.part_o[(static_cast<size_t>(it.part) * G + g) * D + d] = acc;
            if (d == 0) {
                a.part_ml[(static_cast<size_t>(it.part) * G + g) * 2 + 0] = m_star;
                a.part_ml[(static_cast<size_t>(it.part) * G + g) * 2 + 1] = l_star;
            }
        }
    }
}

// Combine the chunks of each pair:  m* = max_c m_c,  l* = sum_c l_c 2^(m_c - m*),
// out = sum_c o_c 2^(m_c - m*) / l*.  Exact in real arithmetic, so chunked equals unchunked.
// One workgroup per (sequence, KV head) pair.  Pairs that were a single item were already
// written by the decode kernel; pairs without tokens get out = 0, lse = -inf here.
__global__ __launch_bounds__(kThreads) void fairkv_merge_kernel(const float *part_o, const float *part_ml,
                                                               const int32_t *part_base, void *out, float *lse,
                                                               int Hq, int Hkv, int G, int D, int out_dtype)
{
    const int pair = blockIdx.x;
    const int b = pair / Hkv, h = pair % Hkv;
    const int p0 = part_base[pair];
    const int nc = part_base[pair + 1] - p0;
    if (nc == 1) return;
    for (int idx = threadIdx.x; idx < G * D; idx += kThreads) {
        const int g = idx / D, d = idx % D;
        float m_star = -INFINITY;
        for (int c = 0; c < nc; ++c) m_star = fmaxf(m_star, part_ml[(static_cast<size_t>(p0 + c) * G + g) * 2]);
        float acc = 0.f, l_star = 0.f;
        for (int c = 0; c < nc; ++c) {
            const float mc = part_ml[(static_cast<size_t>(p0 + c) * G + g) * 2];
            const float f = mc == -INFINITY ? 0.f : __builtin_amdgcn_exp2f(mc - m_star);
            acc += part_o[(static_cast<size_t>(p0 + c) * G + g) * D + d] * f;
            l_star += part_ml[(static_cast<size_t>(p0 + c) * G + g) * 2 + 1] * f;
        }
        const size_t oi = (static_cast<size_t>(b) * Hq + h * G + g) * D + d;
        store_out(out, out_dtype, oi, l_star > 0.f ? acc / l_star : 0.f);
        if (d == 0 && lse)
            lse[b * Hq + h * G + g] = l_star > 0.f ? (m_star + __builtin_amdgcn_logf(l_star)) * kLn2 : -INFINITY;
    }
}

template <int IN_DT, int D>
hipError_t launch_decode_g(int G, const DecodeArgs &a, int n_items, hipStream_t st)
{
    const dim3 grid(static_cast<unsigned>(n_items)), block(kThreads);
    switch (G) {
    case 1: hipLaunchKernelGGL((fairkv_decode_kernel<IN_DT, D, 1>), grid, block, 0, st, a); break;
    case 2: hipLaunchKernelGGL((fairkv_decode_kernel<IN_DT, D, 2>), grid, block, 0, st, a); break;
    case 4: hipLaunchKernelGGL((fairkv_decode_kernel<IN_DT, D, 4>), grid, block, 0, st, a); break;
    case 8: hipLaunchKernelGGL((fairkv_decode_kernel<IN_DT, D, 8>), grid, block, 0, st, a); break;
    default: return hipErrorInvalidValue;
    }
    return hipGetLastError();
}

bool aligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

}  // namespace

extern "C" size_t fairkv_workspace_bytes(int32_t n_parts, int32_t G, int32_t D)
{
    if (n_parts < 0 || G < 1 || D < 1) return 0;
    const size_t bytes = static_cast<size_t>(n_parts) * G * (static_cast<size_t>(D) + 2) * sizeof(float);
    return (bytes + 255) / 256 * 256 + 256;
}

extern "C" int fairkv_decode_attn(const void *q, const void *k, const void *v, const int64_t *off,
                                  const int32_t *len, const fairkv_item *items, int32_t n_items,
                                  const int32_t *part_base, int32_t n_parts, void *workspace,
                                  size_t workspace_bytes, void *out, float *lse, int32_t B, int32_t Hq,
                                  int32_t Hkv, int32_t D, int32_t in_dtype, int32_t out_dtype, float scale,
                                  void *hip_stream)
{
    if (!q || !k || !v || !off || !len || !part_base || !out) return FAIRKV_EINVAL;
    if (B < 1 || Hq < 1 || Hkv < 1 || D < 1 || n_items < 0 || n_parts < 0) return FAIRKV_EINVAL;
    if (Hq % Hkv != 0) return FAIRKV_EINVAL;
    if (n_items > 0 && !items) return FAIRKV_EINVAL;
    if (n_parts < n_items) return FAIRKV_EINVAL;
    if (!(scale == scale) || std::isinf(scale)) return FAIRKV_EINVAL;
    if (in_dtype != FAIRKV_BF16 && in_dtype != FAIRKV_F32) return FAIRKV_EUNSUPPORTED;
    if (out_dtype != FAIRKV_BF16 && out_dtype != FAIRKV_F32) return FAIRKV_EUNSUPPORTED;
    const int G = Hq / Hkv;
    if (D != 64 && D != 128) return FAIRKV_EUNSUPPORTED;
    if (G != 1 && G != 2 && G != 4 && G != 8) return FAIRKV_EUNSUPPORTED;
    if (!aligned16(k) || !aligned16(v) || !aligned16(q)) return FAIRKV_EINVAL;
    if (static_cast<int64_t>(B) * Hq * D > INT32_MAX) return FAIRKV_EINVAL;
    const size_t need = fairkv_workspace_bytes(n_parts, G, D);
    if (n_parts > 0 && (!workspace || workspace_bytes < need)) return FAIRKV_EWORKSPACE;
    if (workspace && !aligned16(workspace)) return FAIRKV_EINVAL;

    hipStream_t st = static_cast<hipStream_t>(hip_stream);
    DecodeArgs a;
    a.q = q;
    a.k = k;
    a.v = v;
    a.off = off;
    a.len = len;
    a.items = items;
    a.part_o = static_cast<float *>(workspace);
    a.part_ml = a.part_o ? a.part_o + static_cast<size_t>(n_parts) * G * D : nullptr;
    a.out = out;
    a.lse = lse;
    a.B = B;
    a.Hq = Hq;
    a.Hkv = Hkv;
    a.out_dtype = out_dtype;
    a.scale_log2 = scale * kLog2e;

    if (n_items > 0) {
        hipError_t e;
        if (in_dtype == FAIRKV_BF16)
            e = D == 128 ? launch_decode_g<FAIRKV_BF16, 128>(G, a, n_items, st)
                         : launch_decode_g<FAIRKV_BF16, 64>(G, a, n_items, st);
        else
            e = D == 128 ? launch_decode_g<FAIRKV_F32, 128>(G, a, n_items, st)
                         : launch_decode_g<FAIRKV_F32, 64>(G, a, n_items, st);
        if (e != hipSuccess) return FAIRKV_EHIP;
    }
    hipLaunchKernelGGL(fairkv_merge_kernel, dim3(static_cast<unsigned>(B * Hkv)), dim3(kThreads), 0, st,
                       a.part_o, a.part_ml, part_base, out, lse, Hq, Hkv, G, D, out_dtype);
    if (hipGetLastError() != hipSuccess) return FAIRKV_EHIP;
    return FAIRKV_OK;
}

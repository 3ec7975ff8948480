// Decode kernel on the vector ALU: any supported element type.  It is the path for fp32
// inputs; bf16 inputs normally take the matrix-core kernel instead.
#pragma once
#include "common.h"

namespace fairkv {

template <int IN_DT, int D, int G>
__global__ __launch_bounds__(kThreads, 2) void fairkv_decode_valu_kernel(DecodeArgs a)
{
    using geo = Geo<IN_DT, D>;
    constexpr int LPR = geo::LPR, RPI = geo::RPI, NI = geo::NI, EPC = geo::EPC, DW = geo::DW;
    constexpr int ROW_BYTES = geo::ROW_BYTES;

    // K tile per wave, 16-byte pieces; piece p of row r sits at column p ^ (r % LPR) so that
    // both the row-contiguous fill and the one-row-per-lane read are free of bank conflicts.
    __shared__ uint4 lds_k[kWaves][kTile * LPR];
    __shared__ float lds_p[kWaves][kTile][G];
    __shared__ PendingParts<D, G> pend;
    int n_pend = 0;

    const int lane = threadIdx.x & 63;
    const int wave = threadIdx.x >> 6;
    const int my_piece = lane % LPR;   // which 16 bytes of a row this lane moves / accumulates
    const int my_sub = lane / LPR;     // which of the RPI rows of a wave-wide access
    float *st_o = reinterpret_cast<float *>(&lds_k[0][0]);   // [kWaves][G][D], reuses the K tiles
    float *st_ml = st_o + kWaves * G * D;                    // [kWaves][G][2]
    static_assert(sizeof(float) * (kWaves * G * (D + 2)) <= sizeof(uint4) * kWaves * kTile * LPR,
                  "merge staging must fit in the K tiles");

    // persistent workgroup: walk the items the planner gave this slot
    const int i_begin = a.slot_ptr[blockIdx.x], i_end = a.slot_ptr[blockIdx.x + 1];
    for (int ii = i_begin; ii < i_end; ++ii) {
    const fairkv_item it = a.items[ii];
    const int b = it.b, h = it.h;
    // an item that does not belong to this problem is skipped by the whole workgroup
    if (b < 0 || b >= a.B || h < 0 || h >= a.Hkv || it.row < 0 || it.part < 0 || it.part >= a.n_parts ||
        it.row + max(it.tok_count, 0) > a.n_rows)
        continue;
    const int n = max(it.tok_count, 0);
    const int n_tiles = (n + kTile - 1) / kTile;

    const char *kbase = static_cast<const char *>(a.k) + it.row * ROW_BYTES;
    const char *vbase = static_cast<const char *>(a.v) + it.row * ROW_BYTES;
    const uint32_t *qrow = static_cast<const uint32_t *>(a.q) + static_cast<size_t>(b * a.Hq + h * G) * DW;

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
    item_epilogue<D, G, true>(a, it, st_o, st_ml, pend, n_pend, a.v_scale);
    }   // items of the slot
    if (n_pend > 0) flush_pending<D, G, true>(a, pend, n_pend);
}

}  // namespace fairkv

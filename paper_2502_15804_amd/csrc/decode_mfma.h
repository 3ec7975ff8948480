// Decode kernel for bf16 K/V/q on the matrix cores.
//
// Why matrix cores on a bandwidth-bound path: with G = 8 query heads per KV head the
// scores and the weighted sum cost 4*G*D = 4096 flop per retained token, i.e. 8 flop per
// byte streamed.  At the 5.6 TB/s this kernel aims for that is 45 TFLOP/s of plain fp32
// FMAs plus the bf16 unpacking, more than half of what the vector ALUs can issue, and it
// left the vector kernel compute bound at about 1.7 TB/s.  As 16x16 MFMA tiles the same
// contraction keeps the matrix pipes under 5 % busy and leaves the vector ALU only the
// softmax of 4 scores per lane per tile.
//
// Shapes.  A wave works on tiles of 16 tokens.  The G query heads sit in the N dimension,
// padded with zero queries to 16:
//     S^T[token][head] = K[token][:] . q[head][:]       4 x mfma_16x16x32 (contract over d)
//     O^T[d][head]    += V^T[d][token] P[token][head]   8 x mfma_16x16x16 (contract over tokens)
// A lane owns head (lane % 16) in the scores, in P and in O^T alike, so the running
// maximum, the rescaling and the bf16 weights never leave the lane.
//
// Data path.  K and V rows go from HBM straight into LDS (global_load_lds_dwordx4, no
// registers), each wave filling its own ring of kStages tiles, so up to kStages-1 tiles
// per wave are in flight while one is being consumed.  The workgroup is persistent: it
// walks the items the planner gave its slot, and a wave's ring runs on into the next item
// while the current one is being finished, so only the first tile of a slot waits for HBM.  16-byte pieces are stored
// XOR-swizzled (the swizzle is applied to the global address a lane fetches, since the
// LDS slot of a lane is fixed) so that the row-per-lane reads of K and the transposing
// reads of V (ds_read_b64_tr_b16) spread over all banks.
#pragma once
#include "common.h"

namespace fairkv {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8_t;
typedef __attribute__((ext_vector_type(4))) __bf16 bf16x4_t;
typedef __attribute__((ext_vector_type(4))) short i16x4_t;
typedef __attribute__((ext_vector_type(4))) float f32x4_t;

constexpr int kTok = 16;      // tokens per tile (the M of the score MFMA, the K of the PV MFMA)
constexpr int kStages = 2;    // tiles per wave resident in LDS: one being consumed, one in flight

#define FAIRKV_LDS_PTR(p) ((__attribute__((address_space(3))) void *)(p))

// One wave-wide direct load HBM -> LDS: lane j's 16 bytes at `src` land at LDS byte address
// lds_base + 16 j (lds_base is wave-uniform and travels in M0).  Written as inline assembly
// so that the compiler does not track it: it would otherwise drain ALL outstanding loads
// (s_waitcnt vmcnt(0)) before any LDS read, which defeats the multi-stage ring.  The waits
// are placed by hand with wait_vmcnt below.
__device__ __forceinline__ void load16_to_lds(const void *src, uint32_t lds_base)
{
    asm volatile("s_mov_b32 m0, %1\n\tglobal_load_lds_dwordx4 %0, off" ::"v"(src), "s"(lds_base) : "memory", "m0");
}

// s_waitcnt that waits for the vector-memory counter only (gfx9 encoding: vmcnt is split
// over bits [3:0] and [15:14]; expcnt [6:4] and lgkmcnt [11:8] are left at "no wait").
template <int N>
__device__ __forceinline__ void wait_vmcnt()
{
    static_assert(N >= 0 && N < 64, "vmcnt is a 6-bit counter");
    asm volatile("s_waitcnt vmcnt(%0)" ::"n"(N) : "memory");
}

// LDS table of the slot's items: what the waves need of a fairkv_item, 16 bytes each.
struct ItemRef {
    int64_t row;
    int32_t n;
    int32_t valid;   // 0: the item does not belong to this problem and is skipped
};
constexpr int kTable = 64;   // items per table fill; longer slot lists are walked in batches

template <int D, int G>
__global__ __launch_bounds__(kThreads, 1) void fairkv_decode_mfma_kernel(DecodeArgs a)
{
    static_assert(D == 64 || D == 128, "head_dim");
    static_assert(G >= 1 && G <= 16, "query heads of a group fit the N dimension");
    constexpr int ROWB = D * 2;              // bytes per K or V row
    constexpr int PPR = ROWB / 16;           // 16-byte pieces per row: 16 or 8
    constexpr int RPI = 64 / PPR;            // rows one wave-wide 16-byte load covers
    constexpr int LPT = kTok / RPI;          // wave-wide loads per K (or V) tile
    constexpr int TILEB = kTok * ROWB;       // bytes of one K (or V) tile
    constexpr int STAGEB = 2 * TILEB;        // K tile then V tile
    constexpr int LOADS = 2 * LPT;           // vector-memory instructions per stage
    constexpr int NSL = D / 32;              // d slices of the score contraction
    constexpr int NDB = D / 16;              // 16-wide d blocks of the output

    __shared__ __attribute__((aligned(1024))) char lds[kWaves * kStages * STAGEB];
    __shared__ __attribute__((aligned(16))) float st_o[kWaves * G * D];
    __shared__ float st_ml[kWaves * G * 2];
    __shared__ __attribute__((aligned(16))) ItemRef table[kTable];
    __shared__ PendingParts<D, G> pend;
    int n_pend = 0;

    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);   // wave-uniform: loop control is scalar
    const int l16 = lane & 15;      // head in B/C operands, token row in the K operand, d in the V operand
    const int lq = lane >> 4;       // which quarter of the contraction index this lane feeds

    const int i_begin = a.slot_ptr[blockIdx.x], i_end = a.slot_ptr[blockIdx.x + 1];
    const uint32_t ring_lds =
        static_cast<uint32_t>(reinterpret_cast<uintptr_t>(FAIRKV_LDS_PTR(lds))) + wave * (kStages * STAGEB);
    const char *ring = lds + wave * (kStages * STAGEB);
    const int ld_row = lane / PPR, ld_col = lane % PPR;

    // tiles of an n-token item that fall to this wave: tiles wave, wave + kWaves, ...
    auto tiles_of = [&](int n) {
        const int n_tiles = (n + kTok - 1) / kTok;
        return n_tiles > wave ? (n_tiles - wave + kWaves - 1) / kWaves : 0;
    };

    // Fetch of this wave's t-th tile of an item into one stage.  Lane j of load i fills LDS slot
    // (row i*RPI + j/PPR, column j%PPR); the piece it fetches is column ^ swizzle(row).  Rows past
    // the end of the item re-read its last row, so that every stage costs exactly LOADS loads.
    auto fetch = [&](int64_t row, int n, int t, int stage) {
        const int tok0 = (wave + t * kWaves) * kTok;
        const int last = n - 1 - tok0;
        const char *kbase = static_cast<const char *>(a.k) + (row + tok0) * ROWB;
        const char *vbase = static_cast<const char *>(a.v) + (row + tok0) * ROWB;
        const uint32_t kst = ring_lds + stage * STAGEB;
        const uint32_t vst = kst + TILEB;
#pragma unroll
        for (int i = 0; i < LPT; ++i) {
            const int r = i * RPI + ld_row;
            const int rc = min(r, last);
            const int kcol = ld_col ^ (r % PPR);
            const int vcol = ld_col ^ ((2 * r) % PPR);
            load16_to_lds(kbase + rc * ROWB + kcol * 16, kst + i * 1024);
            load16_to_lds(vbase + rc * ROWB + vcol * 16, vst + i * 1024);
        }
    };

    // q of an item as the B operand of the score MFMA: lane holds q[head l16][32 s + 8 lq .. +8]; heads >= G are zero.
    auto load_q = [&](const fairkv_item &it, bf16x8_t (&qb)[NSL]) {
        const uint4 *qrow = reinterpret_cast<const uint4 *>(
            static_cast<const char *>(a.q) + (static_cast<size_t>(it.b) * a.Hq + it.h * G + min(l16, G - 1)) * ROWB);
#pragma unroll
        for (int s = 0; s < NSL; ++s) {
            uint4 w = qrow[4 * s + lq];
            if (l16 >= G) w = make_uint4(0u, 0u, 0u, 0u);
            qb[s] = __builtin_bit_cast(bf16x8_t, w);
        }
    };

    // Ring bookkeeping: the fetch cursor (f_*) runs ahead of the compute cursor, possibly into
    // later items; `ahead` tiles are fetched and not yet consumed.
    int f_item = 0, f_t = 0, f_stage = 0, c_stage = 0, ahead = 0, f_n = 0, f_tiles = 0;

    // Early start: row and length of the slot's first item came with the kernel arguments, so
    // its first tiles are requested before the item list has been read from memory.
    const int n0 = static_cast<int>(a.first_n[blockIdx.x]);
    const bool seeded = i_end > i_begin && n0 > 0;
    if (seeded) {
        const int64_t row_first = a.first_row[blockIdx.x];
        f_n = n0;
        f_tiles = tiles_of(n0);
        while (ahead < kStages && f_t < f_tiles) {
            fetch(row_first, f_n, f_t, f_stage);
            f_stage = (f_stage + 1) % kStages;
            ++f_t;
            ++ahead;
        }
    }

    for (int batch = i_begin; batch < i_end; batch += kTable) {
        const int nb = min(kTable, i_end - batch);
        const bool early = seeded && batch == i_begin;
        __syncthreads();                      // nobody still reads the previous table
        if (threadIdx.x < nb) {
            const fairkv_item it = a.items[batch + threadIdx.x];
            const bool ok = it.b >= 0 && it.b < a.B && it.h >= 0 && it.h < a.Hkv && it.row >= 0 && it.part >= 0 &&
                            it.part < a.n_parts && it.n_chunks >= 1;
            int n = ok ? max(it.tok_count, 0) : 0;      // a foreign item reads nothing
            if (early && threadIdx.x == 0) n = n0;      // its tiles are already on their way
            table[threadIdx.x] = ItemRef{it.row, n, ok ? 1 : 0};
        }
        __syncthreads();

        if (!early) {
            f_item = 0;
            f_t = 0;
            f_n = __builtin_amdgcn_readfirstlane(table[0].n);
            f_tiles = tiles_of(f_n);
        }
        auto top_up = [&]() {
            while (ahead < kStages && f_item < nb) {
                if (f_t < f_tiles) {
                    const int64_t row = table[f_item].row;
                    fetch(row, f_n, f_t, f_stage);
                    f_stage = (f_stage + 1) % kStages;
                    ++f_t;
                    ++ahead;
                } else {
                    ++f_item;
                    f_t = 0;
                    f_n = f_item < nb ? __builtin_amdgcn_readfirstlane(table[f_item].n) : 0;
                    f_tiles = tiles_of(f_n);
                }
            }
        };
        top_up();

        bf16x8_t q_next[NSL];
        if (__builtin_amdgcn_readfirstlane(table[0].valid)) load_q(a.items[batch], q_next);

        for (int ci = 0; ci < nb; ++ci) {
            const fairkv_item it = a.items[batch + ci];
            const int n = __builtin_amdgcn_readfirstlane(table[ci].n);
            const int my_tiles = tiles_of(n);
            bf16x8_t qb[NSL];
#pragma unroll
            for (int s = 0; s < NSL; ++s) qb[s] = q_next[s];
            if (ci + 1 < nb && __builtin_amdgcn_readfirstlane(table[ci + 1].valid))
                load_q(a.items[batch + ci + 1], q_next);   // lands while this item streams

            f32x4_t o[NDB];
#pragma unroll
            for (int nb_ = 0; nb_ < NDB; ++nb_) o[nb_] = f32x4_t{0.f, 0.f, 0.f, 0.f};
            float m_run = -INFINITY, l_run = 0.f;

            for (int t = 0; t < my_tiles; ++t) {
                top_up();
                // tile t is complete once at most the loads of the tiles fetched after it are outstanding
                const int later = ahead - 1;
                if (later >= 3) wait_vmcnt<3 * LOADS>();
                else if (later == 2) wait_vmcnt<2 * LOADS>();
                else if (later == 1) wait_vmcnt<LOADS>();
                else wait_vmcnt<0>();
                static_assert(kStages <= 4, "the wait ladder above handles at most three later tiles");

                const char *kst = ring + c_stage * STAGEB;
                const char *vst = kst + TILEB;
                const int tok0 = (wave + t * kWaves) * kTok;
                const int nv = min(kTok, n - tok0);

                // ---- scores: S^T[token 4 lq + i][head l16] -----------------------------------------
                f32x4_t sacc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
                for (int s = 0; s < NSL; ++s) {
                    const int piece = 4 * s + lq;
                    const uint4 kw = *reinterpret_cast<const uint4 *>(kst + l16 * ROWB + ((piece ^ (l16 % PPR)) * 16));
                    sacc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8_t, kw), qb[s], sacc, 0, 0, 0);
                }

                // ---- online softmax, all in this lane's head ----------------------------------------
                float sv[4];
                float mx = -INFINITY;
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    sv[i] = (4 * lq + i) < nv ? sacc[i] * a.scale_log2 : -INFINITY;
                    mx = fmaxf(mx, sv[i]);
                }
                mx = fmaxf(mx, __shfl_xor(mx, 16, 64));
                mx = fmaxf(mx, __shfl_xor(mx, 32, 64));
                const float m_new = fmaxf(m_run, mx);
                const float alpha = __builtin_amdgcn_exp2f(m_run - m_new);     // 0 on the first tile
                float p[4];
#pragma unroll
                for (int i = 0; i < 4; ++i) p[i] = __builtin_amdgcn_exp2f(sv[i] - m_new);
                const bf16x4_t pb = __builtin_convertvector(f32x4_t{p[0], p[1], p[2], p[3]}, bf16x4_t);
                // the sum uses the rounded weights, so out is an exact convex combination of V rows
                float psum = 0.f;
#pragma unroll
                for (int i = 0; i < 4; ++i) psum += static_cast<float>(pb[i]);
                l_run = l_run * alpha + psum;
                m_run = m_new;
                if (__builtin_amdgcn_ballot_w64(alpha != 1.f) != 0) {
#pragma unroll
                    for (int nb_ = 0; nb_ < NDB; ++nb_)
#pragma unroll
                        for (int i = 0; i < 4; ++i) o[nb_][i] *= alpha;
                }

                // ---- O^T[d][head] += V^T P: transposing LDS read gives V[token 4 lq + i][16 nb + l16] ----
                const int vrow = 4 * lq + (l16 >> 2);     // row this lane addresses for the transposing read
                const int vsub = l16 & 3;                 // which 4 d's (8 bytes) of the 16-wide block
#pragma unroll
                for (int nb_ = 0; nb_ < NDB; ++nb_) {
                    const int piece = 2 * nb_ + (vsub >> 1);
                    const char *src = vst + vrow * ROWB + ((piece ^ ((2 * vrow) % PPR)) * 16) + (vsub & 1) * 8;
                    i16x4_t vt = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
                        (__attribute__((address_space(3))) i16x4_t *)FAIRKV_LDS_PTR(src));
                    if (nv < kTok) {     // rows past the end hold a re-read row: keep inf/NaN in it from leaking in
#pragma unroll
                        for (int i = 0; i < 4; ++i)
                            if (4 * lq + i >= nv) vt[i] = 0;
                    }
                    o[nb_] = __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(vt, __builtin_bit_cast(i16x4_t, pb), o[nb_], 0, 0, 0);
                }
                c_stage = (c_stage + 1) % kStages;
                --ahead;
            }

            // ---- fold the four token quarters of l, stage this wave's result, finish the item ------
            l_run += __shfl_xor(l_run, 16, 64);
            l_run += __shfl_xor(l_run, 32, 64);
            if (l16 < G) {
#pragma unroll
                for (int nb_ = 0; nb_ < NDB; ++nb_)
                    *reinterpret_cast<float4 *>(st_o + (wave * G + l16) * D + 16 * nb_ + 4 * lq) =
                        make_float4(o[nb_][0], o[nb_][1], o[nb_][2], o[nb_][3]);
                if (lq == 0) {
                    st_ml[(wave * G + l16) * 2 + 0] = m_run;
                    st_ml[(wave * G + l16) * 2 + 1] = l_run;
                }
            }
            if (__builtin_amdgcn_readfirstlane(table[ci].valid)) item_epilogue<D, G>(a, it, st_o, st_ml, pend, n_pend);
        }
        wait_vmcnt<0>();   // nothing of this batch may still be landing in the rings
    }
    if (n_pend > 0) flush_pending<D, G>(a, pend, n_pend);
}

}  // namespace fairkv

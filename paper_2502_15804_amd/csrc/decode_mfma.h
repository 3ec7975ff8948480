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
// padded to 16 with copies of the last head (their columns are computed and never stored):
//     S^T[token][head] = K[token][:] . q[head][:]       4 x mfma_16x16x32 (contract over d)
//     O^T[d][head]    += V^T[d][token] P[token][head]   8 x mfma_16x16x16 (contract over tokens)
// A lane owns head (lane % 16) in the scores, in P and in O^T alike, so the reference
// maximum, the rescaling and the bf16 weights never leave the lane.
//
// One wave per SIMD means nothing hides a wave's own latencies, so the work on a tile is
// laid out as one LDS round trip (all K and V reads issued together), the score MFMAs, a
// handful of vector instructions and the PV MFMAs.  To that end the softmax keeps a stale
// reference maximum m per head: weights are 2^(s - m) with m raised (and O, l rescaled,
// which needs the only cross-lane exchange) only when some score exceeds m by more than
// kBump, so the weights stay below 2^kBump and the result is the same softmax.
//
// Data path.  K and V rows, the query rows of each item and the slot's item list go from
// HBM straight into LDS (global_load_lds_dwordx4, no registers), each wave filling its own
// ring of kStages tiles.  Inside the item loop there is no load the compiler knows about: it
// would answer each with an s_waitcnt vmcnt(0) that also waits for every tile in flight,
// i.e. one exposed memory latency per item.  The workgroup is persistent: it walks the
// items the planner gave its slot, and a wave's ring runs on into the next item while the
// current one is being finished, so only the first tile of a slot waits for HBM.  16-byte
// pieces are stored XOR-swizzled (the swizzle is applied to the global address a lane
// fetches, since the LDS slot of a lane is fixed) so that the row-per-lane reads of K and
// the transposing reads of V (ds_read_b64_tr_b16) spread over all banks.
#pragma once
#include "common.h"

namespace fairkv {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8_t;
typedef __attribute__((ext_vector_type(4))) __bf16 bf16x4_t;
typedef __attribute__((ext_vector_type(4))) short i16x4_t;
typedef __attribute__((ext_vector_type(4))) float f32x4_t;
typedef __attribute__((ext_vector_type(8))) float f32x8_t;
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2_v;
typedef __attribute__((ext_vector_type(2))) int i32x2_t;

constexpr int kTok = 16;      // tokens per tile (the M of the score MFMA, the K of the PV MFMA)
// Tiles per wave resident in LDS: one being consumed, the other in flight; 64 KB per compute unit are on their way
// at any time.  Three stages (96 KB) fit the LDS for up to 8 columns and were measured side by side on one GPU:
// 0.3-0.4 us slower per launch on the workloads that keep HBM saturated (deeper queues, no more bandwidth) and
// no faster on the one that does not.
constexpr int ring_stages(int) { return 2; }
constexpr float kBump = 8.f;  // log2 units a score may exceed the reference maximum before it is raised

#define FAIRKV_LDS_PTR(p) ((__attribute__((address_space(3))) void *)(p))

// One wave-wide direct load HBM -> LDS: lane j's 16 bytes at base + off land at LDS byte
// address lds_base + 16 j (base and lds_base are wave-uniform; lds_base travels in M0).
// Written as inline assembly so that the compiler does not track it: it would otherwise
// drain ALL outstanding loads (s_waitcnt vmcnt(0)) before any LDS read, which defeats the
// multi-stage ring.  The waits are placed by hand with wait_vmcnt below.
// The load is non-temporal (nt): K and V rows are read once per launch, and a stream marked that way does not
// displace or wait on the L2's other contents.  Measured against the same kernel without the hint: 8 % less time per launch on the 188 MB and 174 MB layers, 4 % on the 68 MB layer,
// 14 % on a layer of whole pairs of equal length; the sc0 / sc1 bits on top of it change nothing.
__device__ __forceinline__ void load16_to_lds(const void *base, uint32_t off, uint32_t lds_base)
{
    asm volatile("s_mov_b32 m0, %2\n\tglobal_load_lds_dwordx4 %0, %1 nt" ::"v"(off), "s"(base), "s"(lds_base) : "memory", "m0");
}
// The same without the hint, for what several workgroups read (the query rows of a pair whose pieces sit in
// different slots) or what comes back on every decode step (a layer's item list): 0.3 us per launch less on the
// workloads with many cut pairs or many items, 0.2 us more on a layer of whole pairs.
__device__ __forceinline__ void load16_to_lds_keep(const void *base, uint32_t off, uint32_t lds_base)
{
    asm volatile("s_mov_b32 m0, %2\n\tglobal_load_lds_dwordx4 %0, %1" ::"v"(off), "s"(base), "s"(lds_base) : "memory", "m0");
}

// s_waitcnt that waits for the vector-memory counter only (gfx9 encoding: vmcnt is split
// over bits [3:0] and [15:14]; expcnt [6:4] and lgkmcnt [11:8] are left at "no wait").
template <int N>
__device__ __forceinline__ void wait_vmcnt()
{
    static_assert(N >= 0 && N < 64, "vmcnt is a 6-bit counter");
    asm volatile("s_waitcnt vmcnt(%0)" ::"n"(N) : "memory");
}

// Wait until at most `tiles` tile fetches (LOADS loads each) and `qs` query-block fetches
// (QL loads each) are outstanding, i.e. everything requested before them has landed.
template <int LOADS, int QL>
__device__ __forceinline__ void wait_all_but(int tiles, int qs)
{
    static_assert(3 * (LOADS + QL) < 64, "vmcnt is a 6-bit counter");
    switch (tiles * 4 + qs) {
    case 4: wait_vmcnt<LOADS>(); break;
    case 5: wait_vmcnt<LOADS + QL>(); break;
    case 8: wait_vmcnt<2 * LOADS>(); break;
    case 9: wait_vmcnt<2 * LOADS + QL>(); break;
    case 10: wait_vmcnt<2 * LOADS + 2 * QL>(); break;
    case 12: wait_vmcnt<3 * LOADS>(); break;
    case 13: wait_vmcnt<3 * LOADS + QL>(); break;
    case 14: wait_vmcnt<3 * LOADS + 2 * QL>(); break;
    case 15: wait_vmcnt<3 * LOADS + 3 * QL>(); break;
    default: wait_vmcnt<0>(); break;
    }
}

__device__ __forceinline__ int64_t uniform64(int64_t x)   // a wave-uniform value, moved to scalar registers
{
    const uint32_t lo = __builtin_amdgcn_readfirstlane(static_cast<int>(x));
    const uint32_t hi = __builtin_amdgcn_readfirstlane(static_cast<int>(x >> 32));
    return static_cast<int64_t>((static_cast<uint64_t>(hi) << 32) | lo);
}

// Eight E4M3 bytes widened to eight bf16 (exact; v_cvt_scalef32_pk_bf16_fp8 with scale 1 takes two bytes
// at a time: the low or the high half of a dword).
__device__ __forceinline__ bf16x8_t widen8(uint2 w)
{
    const bf16x2_v a0 = __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(w.x, 1.0f, false);
    const bf16x2_v a1 = __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(w.x, 1.0f, true);
    const bf16x2_v a2 = __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(w.y, 1.0f, false);
    const bf16x2_v a3 = __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(w.y, 1.0f, true);
    return bf16x8_t{a0[0], a0[1], a1[0], a1[1], a2[0], a2[1], a3[0], a3[1]};
}

// LDS copy of the slot's items: what the waves need of a fairkv_item, plus the checked length.
struct ItemSlot {
    int64_t row;
    int32_t n;        // tokens to read; 0 for an item that does not belong to this problem
    int32_t valid;    // 0: such an item; it is skipped
    int32_t b, h, chunk, n_chunks, part;
    int32_t owner;    // -1: the four waves share the item's tiles; else the wave that runs the whole item alone
    int32_t pad[2];
};
// A whole pair of at most this many tokens is run by one wave alone: it streams all the pair's tiles through its
// own ring and writes the output straight from its registers, with no fold across waves and no barrier.  Short
// pairs shared by four waves leave most of the rings empty (a 32-token pair is two tiles: two waves have nothing
// to fetch and the other two one tile each), so a slot of many short pairs had about one pair in flight at a time
// and each cost a memory round trip; alone, four pairs stream side by side.
constexpr int kSoloTokens = FAIRKV_SHORT_PAIR_TOKENS;
static_assert(sizeof(ItemSlot) == 48, "item table entry");
constexpr int kTable = 32 * kWaves;   // items per table fill (each wave fetches 32); longer slot lists go in batches

// KV8: K and V are stored as 8-bit floats (E4M3), one byte per element, and widened to bf16 in registers
// (exactly: every E4M3 value is a bf16 value), so the arithmetic is that of the bf16 path.  A row is half as
// long, so a stage holds 32 tokens instead of 16 in the same 8 KB, and a step works on two 16-token score
// tiles and one 32-token P.V product:
//     S^T = K . q^T    2 x 4 x mfma_16x16x32 on K widened 8 bytes at a time
//     O^T += V^T . P   8 x mfma_16x16x32; the contraction index k = 8 lq + r of a lane stands for token
//                      4 lq + r of the first score tile (r < 4) or of the second (r >= 4), which is how the
//                      lane's own eight weights are laid out already; V^T comes out of the LDS through the
//                      8-bit transposing read: lane i of a 16-lane group addresses the 8 bytes (token
//                      t_(i/2), columns 8 (i%2) .. +7) and lane j receives byte j%8 of the fragments
//                      j/8, j/8 + 2, ..., i.e. column j of tokens t_0 .. t_7 (layout checked on the GPU).
// TRACE: the measurement instantiation behind fairkv_decode_attn_trace; it writes wall-clock stamps of its phases
// (see trace_stamp) and is otherwise the same code.
// SOLO: the plan has short whole pairs (at most kSoloTokens tokens) and they are run by single waves.  Plans
// without any run an instantiation without that code: its presence alone cost 0.3-0.4 us per launch on every
// workload (measured side by side on one GPU), on a kernel of under 20 us.
template <int D, int G, bool DEEP, bool KV8, bool SOLO, bool TRACE = false>
__global__ __launch_bounds__(kThreads, 1) void fairkv_decode_mfma_kernel(DecodeArgs a)
{
    static_assert(D == 64 || D == 128, "head_dim");
    static_assert(G >= 1 && G <= 16, "query heads of a group fit the N dimension");
    constexpr int TOK = KV8 ? 2 * kTok : kTok;          // tokens per stage and per step
    constexpr int kStages = ring_stages(G);
    // Tiles per wave the early start requests: one.  With the whole ring requested at once (two tiles per wave,
    // 16 MB over the chip before anything has come back) the memory system serves the 1024 waves in no fair
    // order, some workgroups see their first tile a microsecond after the others and, each having a fixed share of
    // the work, finish that much later; the second stage is requested when the item list has landed instead.
    // Side by side on one GPU: 0.4-0.5 us per launch less on all four workloads.
    constexpr int kEarly = 1;
    static_assert(kStages >= 2 && kStages <= 4 && kEarlyTok >= kEarly * kWaves * TOK && kEarlyTok < 512, "ring, early start");
    static_assert(sizeof(fairkv_item) == 32, "two 16-byte pieces per item");
    constexpr int QROWB = D * 2;             // bytes per q row (bf16)
    constexpr int ROWB = KV8 ? D : D * 2;    // bytes per K or V row
    constexpr int PPR = ROWB / 16;           // 16-byte pieces per row: 16 or 8
    constexpr int RPI = 64 / PPR;            // rows one wave-wide 16-byte load covers
    constexpr int LPT = TOK / RPI;           // wave-wide loads per K (or V) tile
    constexpr int TILEB = TOK * ROWB;        // bytes of one K (or V) tile
    constexpr int STAGEB = 2 * TILEB;        // K tile then V tile
    constexpr int LOADS = 2 * LPT;           // vector-memory instructions per stage
    constexpr int NSL = D / 32;              // d slices of the score contraction
    constexpr int NDB = D / 16;              // 16-wide d blocks of the output
    constexpr int QBYTES = G * QROWB;        // the G query rows of a group are contiguous in q
    constexpr int QL = (QBYTES + 1023) / 1024;   // wave-wide loads per query block
    constexpr int QBUF = QL * 1024;

    __shared__ __attribute__((aligned(1024))) char lds[kWaves * kStages * STAGEB];
    __shared__ __attribute__((aligned(1024))) char qlds[kWaves * kStages * QBUF];   // a query block per ring stage: the tiles in
                                                                                    // the ring may belong to kStages different items
    __shared__ __attribute__((aligned(1024))) fairkv_item raw[kTable];        // items as fetched
    __shared__ __attribute__((aligned(16))) ItemSlot table[kTable];           // items as checked
    __shared__ __attribute__((aligned(16))) float st_o[kWaves * G * D];
    __shared__ __attribute__((aligned(16))) float st_ml[kWaves * G * 2];
    __shared__ PendingParts<D, G> pend;
    __shared__ float head_mul[2 * kScaleHeads];      // 8-bit caches: the per-head factors, out of the kernel arguments
    int n_pend = 0;

    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);   // wave-uniform: loop control is scalar
    const int l16 = lane & 15;      // head in B/C operands, token row in the K operand, d in the V operand
    const int lq = lane >> 4;       // which quarter of the contraction index this lane feeds

    if constexpr (TRACE) trace_stamp(a, kTraceStart, threadIdx.x == 0);
    const int i_begin = a.slot_ptr[blockIdx.x], i_end = a.slot_ptr[blockIdx.x + 1];
    if (i_end <= i_begin) return;   // an idle slot
    if constexpr (KV8) {
        // Fixed indices: scalar loads that come back with the other kernel arguments.  Indexed by the item's head
        // they would be a scalar load per item, waited for in front of its first tile.
        if (threadIdx.x == 0) {
#pragma unroll
            for (int i = 0; i < kScaleHeads; ++i) {
                head_mul[i] = a.scale_log2 * a.k_head[i];
                head_mul[kScaleHeads + i] = a.v_scale * a.v_head[i];
            }
        }                           // read after the barriers that precede the first item
    }
    const uint32_t ring_lds =
        static_cast<uint32_t>(reinterpret_cast<uintptr_t>(FAIRKV_LDS_PTR(lds))) + wave * (kStages * STAGEB);
    const char *ring = lds + wave * (kStages * STAGEB);
    const uint32_t q_lds = static_cast<uint32_t>(reinterpret_cast<uintptr_t>(FAIRKV_LDS_PTR(qlds))) + wave * (kStages * QBUF);
    const char *q_ring = qlds + wave * (kStages * QBUF);
    const uint32_t raw_lds = static_cast<uint32_t>(reinterpret_cast<uintptr_t>(FAIRKV_LDS_PTR(raw))) + wave * 1024;

    // Lane j of load i of a tile fills LDS slot (row i*RPI + j/PPR, column j%PPR); the piece it
    // fetches is column ^ swizzle(row).  Byte offsets of that piece inside a full K and V tile:
    const int ld_row = lane / PPR, ld_col = lane % PPR;
    uint32_t k_off[LPT], v_off[LPT];
#pragma unroll
    for (int i = 0; i < LPT; ++i) {
        const int r = i * RPI + ld_row;
        k_off[i] = r * ROWB + (ld_col ^ (r % PPR)) * 16;
        v_off[i] = r * ROWB + (ld_col ^ ((2 * r) % PPR)) * 16;
    }
    // ... and where a lane reads its operands: the K row l16 (pieces 4 s + lq) and, through the
    // transposing read, 4 d's of V row 4 lq + l16/4 (lane j of a 16-lane group receives element
    // j%4 of the rows its lanes 4i + j/4 address).
    // (8-bit caches: 8 bytes of K row l16 or 16 + l16 at byte 32 s + 8 lq; for V the fragment this
    // lane addresses in the transposing read, see above.)
    constexpr int NKR = KV8 ? 2 * NSL : NSL;
    uint32_t k_rd[NKR], v_rd[NDB];
    if constexpr (!KV8) {
#pragma unroll
        for (int s = 0; s < NSL; ++s) k_rd[s] = l16 * ROWB + ((4 * s + lq) ^ (l16 % PPR)) * 16;
        const int vrow = 4 * lq + (l16 >> 2), vsub = l16 & 3;
#pragma unroll
        for (int nb_ = 0; nb_ < NDB; ++nb_)
            v_rd[nb_] = TILEB + vrow * ROWB + (((2 * nb_ + (vsub >> 1)) ^ ((2 * vrow) % PPR)) * 16) + (vsub & 1) * 8;
    } else {
#pragma unroll
        for (int u = 0; u < 2; ++u)
#pragma unroll
            for (int s = 0; s < NSL; ++s) {
                const int row = 16 * u + l16;
                k_rd[u * NSL + s] = row * ROWB + (((2 * s + (lq >> 1)) ^ (row % PPR)) * 16) + (lq & 1) * 8;
            }
        const int r = l16 >> 1;                                            // which of the lane group's 8 tokens
        const int vrow = r < 4 ? 4 * lq + r : 16 + 4 * lq + (r - 4);
#pragma unroll
        for (int nb_ = 0; nb_ < NDB; ++nb_) v_rd[nb_] = TILEB + vrow * ROWB + ((nb_ ^ ((2 * vrow) % PPR)) * 16) + (l16 & 1) * 8;
    }

    // tiles of an n-token item that fall to this wave: tiles wave, wave + kWaves, ... of an item the waves share;
    // all of them, or none, of an item that one wave runs alone
    auto tiles_of = [&](int n, int owner) __attribute__((always_inline)) {
        const int n_tiles = (n + TOK - 1) / TOK;
        if (SOLO && owner >= 0) return owner == wave ? n_tiles : 0;
        return n_tiles > wave ? (n_tiles - wave + kWaves - 1) / kWaves : 0;
    };
    // first token of this wave's t-th tile of an item
    auto tile_tok0 = [&](int t, int owner) __attribute__((always_inline)) { return (SOLO && owner >= 0 ? t : wave + t * kWaves) * TOK; };

    // Fetch of this wave's t-th tile of an item into one stage: always exactly LOADS loads.
    // Rows past the end of the item re-read its last row (finite data with weight 0).
    auto fetch = [&](int64_t row, int n, int t, int owner, int stage) __attribute__((always_inline)) {
        const int tok0 = tile_tok0(t, owner);
        const int last = n - 1 - tok0;
        const char *kbase = static_cast<const char *>(a.k) + (row + tok0) * ROWB;
        const char *vbase = static_cast<const char *>(a.v) + (row + tok0) * ROWB;
        const uint32_t kst = ring_lds + stage * STAGEB;
        const uint32_t vst = kst + TILEB;
        if (last >= TOK - 1) {
#pragma unroll
            for (int i = 0; i < LPT; ++i) {
                load16_to_lds(kbase, k_off[i], kst + i * 1024);
                load16_to_lds(vbase, v_off[i], vst + i * 1024);
            }
        } else {
#pragma unroll
            for (int i = 0; i < LPT; ++i) {
                const int r = i * RPI + ld_row;
                const int rc = min(r, last);
                load16_to_lds(kbase, rc * ROWB + (ld_col ^ (r % PPR)) * 16, kst + i * 1024);
                load16_to_lds(vbase, rc * ROWB + (ld_col ^ ((2 * r) % PPR)) * 16, vst + i * 1024);
            }
        }
    };

    // Fetch of the G query rows of pair (b, h) into one of the wave's q buffers: exactly QL loads.
    // Column c = (new token c >> g_shift, head c & mask) of q [B][q_len][Hq][D]: the heads of one new
    // token are contiguous, the new tokens are Hq rows apart.
    auto fetch_q = [&](int b, int h, int buf) __attribute__((always_inline)) {
        const char *src = static_cast<const char *>(a.q) +
                          (static_cast<size_t>(b) * a.q_len * a.Hq + (h << a.g_shift)) * QROWB;
#pragma unroll
        for (int i = 0; i < QL; ++i) {
            const int o = min(i * 1024 + lane * 16, QBYTES - 16);      // byte o of the [G][QROWB] image in LDS
            const int c = o / QROWB;
            const int row = (c >> a.g_shift) * a.Hq + (c & ((1 << a.g_shift) - 1));
            load16_to_lds_keep(src, row * QROWB + o % QROWB, q_lds + buf * QBUF + i * 1024);
        }
    };

    // Fetch of this wave's 32 of the kTable items that start at `first`: one load.  Past the end of
    // the slot's list the last item is read again.
    auto fetch_items = [&](int first) __attribute__((always_inline)) {
        const int rel = min(32 * wave + (lane >> 1), i_end - 1 - first);
        load16_to_lds_keep(a.items + first, rel * 32 + (lane & 1) * 16, raw_lds);
    };

    // Ring bookkeeping: the fetch cursor (f_*) runs ahead of the compute cursor, possibly into
    // later items; `ahead` tiles are fetched and not yet consumed.  The query block of an item is
    // requested right before the item's first tile, into the q buffer of that tile's stage, so it
    // has landed when the tile has; bit s of q_mask says that the tile now in stage s came with one.
    int f_item = 0, f_t = 0, f_stage = 0, c_stage = 0, ahead = 0, f_n = 0, f_tiles = 0, f_b = 0, f_h = 0, f_owner = -1;
    int64_t f_row = 0;
    uint32_t q_mask = 0;
    auto fetch_next = [&]() __attribute__((always_inline)) {      // the cursor's tile, f_t < f_tiles
        if (f_t == 0) {
            // (scalar registers for the load's base address, wherever the compiler kept these wave-uniform values)
            fetch_q(__builtin_amdgcn_readfirstlane(f_b), __builtin_amdgcn_readfirstlane(f_h), f_stage);
            q_mask |= 1u << f_stage;
        }
        fetch(f_row, f_n, f_t, f_owner, f_stage);
        f_stage = f_stage + 1 == kStages ? 0 : f_stage + 1;
        ++f_t;
        ++ahead;
    };

    // Early start: the kernel arguments carry pair, first row and the first kEarlyTok tokens' worth
    // of the length of the slot's first item, so the item list, the first query block and the first
    // tiles are all requested at once, before anything has come back from memory.
    fetch_items(i_begin);
    const uint32_t np0 = a.first_np[blockIdx.x];
    const int n0 = static_cast<int>(np0 & 0x1ffu);
    const bool seeded = n0 > 0;
    if (seeded) {
        const int pair0 = static_cast<int>(np0 >> 9);
        f_b = __builtin_amdgcn_readfirstlane(pair0 / a.Hkv);      // the division runs on the vector ALU
        f_h = pair0 - f_b * a.Hkv;
        f_row = a.first_row[blockIdx.x];
        f_n = n0;
        f_tiles = tiles_of(n0, -1);          // the early start always shares the first item among the waves
        while (ahead < kEarly && f_t < f_tiles) fetch_next();
    }

    for (int batch = i_begin; batch < i_end; batch += kTable) {
        const int nb = min(kTable, i_end - batch);
        const bool early = seeded && batch == i_begin;
        if (batch != i_begin) {
            __syncthreads();                  // nobody still reads the previous table
            fetch_items(batch);
        }
        // the items have landed once only what was requested after them is outstanding
        wait_all_but<LOADS, QL>(ahead, __builtin_popcount(q_mask));
        __syncthreads();
        if (threadIdx.x < nb) {
            const fairkv_item it = raw[threadIdx.x];
            const bool ok = it.b >= 0 && it.b < a.B && it.h >= 0 && it.h < a.Hkv && it.row >= 0 && it.part >= 0 &&
                            it.part < a.n_parts && it.n_chunks >= 1 && it.chunk >= 0 && it.chunk <= it.part &&
                            it.row + max(it.tok_count, 0) <= a.n_rows;
            int n = ok ? max(it.tok_count, 0) : 0;      // a foreign item reads nothing
            if (early && threadIdx.x == 0)              // its first tiles are on their way, as many as n0 said
                n = n0 < kEarlyTok ? n0 : max(n, kEarlyTok);
            // short whole pairs go to single waves in turn (not the item the early start has already shared out)
            const bool solo = SOLO && ok && it.n_chunks == 1 && n <= kSoloTokens && !(early && threadIdx.x == 0);
            table[threadIdx.x] = ItemSlot{it.row, n, ok ? 1 : 0, ok ? it.b : 0, ok ? it.h : 0,
                                          it.chunk, it.n_chunks, it.part, solo ? static_cast<int32_t>(threadIdx.x % kWaves) : -1, {0, 0}};
        }
        __syncthreads();
        if constexpr (TRACE)
            if (batch == i_begin) trace_stamp(a, kTraceTable, threadIdx.x == 0);

        auto seek = [&](int item) __attribute__((always_inline)) {           // point the fetch cursor at an item of the table
            f_item = item;
            f_t = 0;
            if (item < nb) {
                f_row = uniform64(table[item].row);
                f_n = __builtin_amdgcn_readfirstlane(table[item].n);
                f_b = __builtin_amdgcn_readfirstlane(table[item].b);
                f_h = __builtin_amdgcn_readfirstlane(table[item].h);
                f_owner = SOLO ? __builtin_amdgcn_readfirstlane(table[item].owner) : -1;
            } else {
                f_n = 0;
                f_owner = -1;
            }
            f_tiles = tiles_of(f_n, f_owner);
        };
        if (early) {                          // the cursor is already inside item 0: learn its full length
            f_n = __builtin_amdgcn_readfirstlane(table[0].n);
            f_tiles = tiles_of(f_n, -1);
        } else {
            seek(0);
        }
        auto top_up = [&]() __attribute__((always_inline)) {
            while (ahead < kStages && f_item < nb) {
                if (f_t < f_tiles)
                    fetch_next();
                else
                    seek(f_item + 1);
            }
        };
        top_up();

        for (int ci = 0; ci < nb; ++ci) {
            fairkv_item it;
            it.row = 0;
            it.tok_count = 0;
            it.b = __builtin_amdgcn_readfirstlane(table[ci].b);
            it.h = __builtin_amdgcn_readfirstlane(table[ci].h);
            it.chunk = __builtin_amdgcn_readfirstlane(table[ci].chunk);
            it.n_chunks = __builtin_amdgcn_readfirstlane(table[ci].n_chunks);
            it.part = __builtin_amdgcn_readfirstlane(table[ci].part);
            const int n = __builtin_amdgcn_readfirstlane(table[ci].n);
            const int owner = SOLO ? __builtin_amdgcn_readfirstlane(table[ci].owner) : -1;
            if (SOLO && owner >= 0 && owner != wave) continue;      // another wave runs this pair alone
            const int my_tiles = tiles_of(n, owner);
            // scores to log2 units, and what multiplies the output: the same for every pair unless an 8-bit cache has
            // a scale per KV head
            const float s_mul = KV8 ? head_mul[it.h % kScaleHeads] : a.scale_log2;
            const float v_mul = KV8 ? head_mul[kScaleHeads + it.h % kScaleHeads] : a.v_scale;
            // Several new tokens per sequence: their K/V rows are the last q_len rows of the pair, and
            // new token j does not see the rows of the new tokens after it.  Only the pair's last
            // chunk holds such rows; n_col = tokens of this item the lane's column may see.
            const int hidden_max = it.chunk == it.n_chunks - 1 ? a.q_len - 1 : 0;
            const int n_col = n - (it.chunk == it.n_chunks - 1 ? a.q_len - 1 - (min(l16, G - 1) >> a.g_shift) : 0);
            bf16x8_t qb[NSL];
#pragma unroll
            for (int s = 0; s < NSL; ++s) qb[s] = bf16x8_t{0, 0, 0, 0, 0, 0, 0, 0};

            f32x4_t o[NDB];
#pragma unroll
            for (int nb_ = 0; nb_ < NDB; ++nb_) o[nb_] = f32x4_t{0.f, 0.f, 0.f, 0.f};
            float m_run = -INFINITY, l_run = 0.f;   // reference maximum of the lane's head, this lane's share of the weights

            for (int t = 0; t < my_tiles; ++t) {
                top_up();
                // Tile t has landed once no more is outstanding than was requested after it: the later
                // tiles in the ring and their query blocks.
                wait_all_but<LOADS, QL>(ahead - 1, __builtin_popcount(q_mask & ~(1u << c_stage)));
                q_mask &= ~(1u << c_stage);
                if constexpr (TRACE)
                    if (batch == i_begin && ci == 0 && t == 0) trace_stamp(a, kTraceFirstTile, threadIdx.x == 0);
                if (t == 0) {
                    // q as the B operand of the score MFMA: lane holds q[head l16][32 s + 8 lq .. +8].  Heads
                    // >= G repeat head G-1: their columns of the products are computed and never stored.
                    const char *qsrc = q_ring + c_stage * QBUF + min(l16, G - 1) * QROWB + lq * 16;
#pragma unroll
                    for (int s = 0; s < NSL; ++s)
                        qb[s] = __builtin_bit_cast(bf16x8_t, *reinterpret_cast<const uint4 *>(qsrc + s * 64));
                }

                if constexpr (KV8) {
                    // ---- every LDS read of the step, issued together ---------------------------------
                    const char *st = ring + c_stage * STAGEB;
                    uint2 kw[NKR];
                    i32x2_t vt[NDB];
#pragma unroll
                    for (int s = 0; s < NKR; ++s) kw[s] = *reinterpret_cast<const uint2 *>(st + k_rd[s]);
#pragma unroll
                    for (int nb_ = 0; nb_ < NDB; ++nb_)
                        vt[nb_] = __builtin_amdgcn_ds_read_tr8_b64_v2i32(
                            (__attribute__((address_space(3))) i32x2_t *)FAIRKV_LDS_PTR(st + v_rd[nb_]));

                    // ---- scores of two 16-token tiles: S^T[token 16 u + 4 lq + i][head l16] ----------
                    f32x4_t sacc[2] = {{0.f, 0.f, 0.f, 0.f}, {0.f, 0.f, 0.f, 0.f}};
#pragma unroll
                    for (int u = 0; u < 2; ++u)
#pragma unroll
                        for (int s = 0; s < NSL; ++s)
                            sacc[u] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(widen8(kw[u * NSL + s]), qb[s], sacc[u], 0, 0, 0);
                    const int tok0 = tile_tok0(t, owner);
                    const bool masked = n - hidden_max - tok0 < TOK;     // some column does not see the whole step
                    float sv[8];
#pragma unroll
                    for (int r = 0; r < 8; ++r) sv[r] = sacc[r >> 2][r & 3] * s_mul;
                    if (masked) {
#pragma unroll
                        for (int r = 0; r < 8; ++r)
                            if (16 * (r >> 2) + 4 * lq + (r & 3) >= n_col - tok0) sv[r] = -INFINITY;
                    }

                    // ---- raise the reference maximum if some score is far above it ------------------
                    float mx = fmaxf(fmaxf(fmaxf(sv[0], sv[1]), fmaxf(sv[2], sv[3])), fmaxf(fmaxf(sv[4], sv[5]), fmaxf(sv[6], sv[7])));
                    if (__builtin_amdgcn_ballot_w64(mx > m_run + kBump) != 0) {
                        mx = fmaxf(mx, __shfl_xor(mx, 16, 64));
                        mx = fmaxf(mx, __shfl_xor(mx, 32, 64));
                        const float m_new = fmaxf(m_run, mx);
                        const float alpha = m_new == m_run ? 1.f : __builtin_amdgcn_exp2f(m_run - m_new);
                        l_run *= alpha;
#pragma unroll
                        for (int nb_ = 0; nb_ < NDB; ++nb_)
#pragma unroll
                            for (int i = 0; i < 4; ++i) o[nb_][i] *= alpha;
                        m_run = m_new;
                    }

                    // ---- weights, rounded to bf16, in the order the contraction index wants them ------
                    float p[8];
#pragma unroll
                    for (int r = 0; r < 8; ++r) p[r] = __builtin_amdgcn_exp2f(sv[r] - m_run);
                    if (masked) {
#pragma unroll
                        for (int r = 0; r < 8; ++r)
                            if (sv[r] == -INFINITY) p[r] = 0.f;
                    }
                    const bf16x8_t pb = __builtin_convertvector(f32x8_t{p[0], p[1], p[2], p[3], p[4], p[5], p[6], p[7]}, bf16x8_t);
#pragma unroll
                    for (int r = 0; r < 8; ++r) l_run += static_cast<float>(pb[r]);

                    // ---- O^T[d][head] += V^T P over the 32 tokens ------------------------------------
#pragma unroll
                    for (int nb_ = 0; nb_ < NDB; ++nb_)
                        o[nb_] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(
                            widen8(uint2{static_cast<uint32_t>(vt[nb_][0]), static_cast<uint32_t>(vt[nb_][1])}), pb, o[nb_], 0, 0, 0);
                } else {
                    // ---- every LDS read of the tile, issued together -----------------------------------
                    const char *st = ring + c_stage * STAGEB;
                    uint4 kw[NSL];
                    i16x4_t vt[NDB];
    #pragma unroll
                    for (int s = 0; s < NSL; ++s) kw[s] = *reinterpret_cast<const uint4 *>(st + k_rd[s]);
    #pragma unroll
                    for (int nb_ = 0; nb_ < NDB; ++nb_)
                        vt[nb_] = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
                            (__attribute__((address_space(3))) i16x4_t *)FAIRKV_LDS_PTR(st + v_rd[nb_]));

                    // ---- scores: S^T[token 4 lq + i][head l16], in log2 units --------------------------
                    f32x4_t sacc = {0.f, 0.f, 0.f, 0.f};
    #pragma unroll
                    for (int s = 0; s < NSL; ++s)
                        sacc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8_t, kw[s]), qb[s], sacc, 0, 0, 0);
                    const int tok0 = tile_tok0(t, owner);
                    const bool masked = n - hidden_max - tok0 < TOK;    // some column does not see the whole tile
                    float sv[4];
    #pragma unroll
                    for (int i = 0; i < 4; ++i) sv[i] = sacc[i] * s_mul;
                    if (masked) {
    #pragma unroll
                        for (int i = 0; i < 4; ++i)
                            if (4 * lq + i >= n_col - tok0) sv[i] = -INFINITY;
                    }

                    // ---- raise the reference maximum if some score is far above it (always on the first tile)
                    float mx = fmaxf(fmaxf(sv[0], sv[1]), fmaxf(sv[2], sv[3]));
                    if (__builtin_amdgcn_ballot_w64(mx > m_run + kBump) != 0) {
                        mx = fmaxf(mx, __shfl_xor(mx, 16, 64));
                        mx = fmaxf(mx, __shfl_xor(mx, 32, 64));
                        const float m_new = fmaxf(m_run, mx);
                        const float alpha = m_new == m_run ? 1.f : __builtin_amdgcn_exp2f(m_run - m_new);   // 0 on the first tile
                        l_run *= alpha;
    #pragma unroll
                        for (int nb_ = 0; nb_ < NDB; ++nb_)
    #pragma unroll
                            for (int i = 0; i < 4; ++i) o[nb_][i] *= alpha;
                        m_run = m_new;
                    }

                    // ---- weights, rounded to bf16; their sum uses the rounded values, so out is an exact
                    //      convex combination of V rows -------------------------------------------------
                    float p[4];
    #pragma unroll
                    for (int i = 0; i < 4; ++i) p[i] = __builtin_amdgcn_exp2f(sv[i] - m_run);
                    if (masked) {     // a column that has seen nothing yet has m = -inf: its weights are 0, not exp2(nan)
    #pragma unroll
                        for (int i = 0; i < 4; ++i)
                            if (sv[i] == -INFINITY) p[i] = 0.f;
                    }
                    const bf16x4_t pb = __builtin_convertvector(f32x4_t{p[0], p[1], p[2], p[3]}, bf16x4_t);
    #pragma unroll
                    for (int i = 0; i < 4; ++i) l_run += static_cast<float>(pb[i]);

                    // ---- O^T[d][head] += V^T P ---------------------------------------------------------
    #pragma unroll
                    for (int nb_ = 0; nb_ < NDB; ++nb_)
                        o[nb_] = __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(vt[nb_], __builtin_bit_cast(i16x4_t, pb), o[nb_], 0, 0, 0);
                }
                c_stage = c_stage + 1 == kStages ? 0 : c_stage + 1;
                --ahead;
            }

            if constexpr (TRACE) {
                if (batch == i_begin && ci == 0) trace_stamp(a, kTraceItem0Streamed, threadIdx.x == 0);
                if (batch + ci == i_end - 1) trace_stamp(a, kTraceLastStreamed, threadIdx.x == 0);
            }
            // ---- fold the four token quarters of l, stage this wave's result, finish the item ------
            l_run += __shfl_xor(l_run, 16, 64);
            l_run += __shfl_xor(l_run, 32, 64);
            if (SOLO && owner >= 0) {
                // This wave has seen the whole pair: out = O / l and lse straight from its registers.  A lane holds
                // coordinates 16 nb + 4 lq .. + 3 of head l16.
                if (l16 < G && __builtin_amdgcn_readfirstlane(table[ci].valid)) {
                    const size_t orow = out_row(a, it.b, it.h, l16);
                    const float inv = l_run > 0.f ? v_mul / l_run : 0.f;
#pragma unroll
                    for (int nb_ = 0; nb_ < NDB; ++nb_)
                        store_out4(a.out, a.out_dtype, orow * D + 16 * nb_ + 4 * lq,
                                   make_float4(o[nb_][0] * inv, o[nb_][1] * inv, o[nb_][2] * inv, o[nb_][3] * inv));
                    if (lq == 0 && a.lse)
                        a.lse[orow] = l_run > 0.f ? (m_run + __builtin_amdgcn_logf(l_run)) * kLn2 : -INFINITY;
                }
                continue;
            }
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
            if (__builtin_amdgcn_readfirstlane(table[ci].valid)) item_epilogue<D, G, DEEP, TRACE>(a, it, st_o, st_ml, pend, n_pend, v_mul);
            if constexpr (TRACE)
                if (batch == i_begin && ci == 0) trace_stamp(a, kTraceItem0Done, threadIdx.x == 0);
        }
        wait_vmcnt<0>();   // nothing of this batch may still be landing in the rings
    }
    if (n_pend > 0) flush_pending<D, G, DEEP, TRACE>(a, pend, n_pend);
    if constexpr (TRACE) trace_stamp(a, kTraceEnd, threadIdx.x == 0);
}

}  // namespace fairkv

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

// four consecutive outputs, idx a multiple of 4 (out is 16-byte aligned).  Results are written once and not read
// again by this launch: non-temporal stores keep them from waiting in the L2 for the write-back at the end of the
// kernel (0.45 us per launch on a layer of whole pairs, 0.25 us on the many-small-pairs workload).
__device__ __forceinline__ void store_out4(void *out, int out_dtype, size_t idx, float4 x)
{
    if (out_dtype == FAIRKV_F32) {
        typedef __attribute__((ext_vector_type(4))) float f4;
        __builtin_nontemporal_store(f4{x.x, x.y, x.z, x.w}, reinterpret_cast<f4 *>(static_cast<float *>(out) + idx));
    } else {
        typedef __attribute__((ext_vector_type(2))) uint32_t u2;
        const u2 w = {f32_to_bf16_rne(x.x) | (static_cast<uint32_t>(f32_to_bf16_rne(x.y)) << 16),
                      f32_to_bf16_rne(x.z) | (static_cast<uint32_t>(f32_to_bf16_rne(x.w)) << 16)};
        __builtin_nontemporal_store(w, reinterpret_cast<u2 *>(static_cast<uint16_t *>(out) + idx));
    }
}

struct DecodeArgs;
// Where column c of pair (b, h) lives in out (times D) and in lse: [B][q_len][Hq].
__device__ __forceinline__ size_t out_row(const DecodeArgs &a, int b, int h, int c);

// Partial results travel between workgroups that may sit on different XCDs, whose L2 caches
// are not coherent with each other.  Agent-scope relaxed atomics are plain 4-byte stores and
// loads that go through to the level all XCDs share, without the cache-wide write-back and
// invalidate that a device fence costs (measured: tens of microseconds per launch).
__device__ __forceinline__ void publish_f32(float *p, float x)
{
    __hip_atomic_store(p, x, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
// Four floats as one 16-byte store that goes through to the same level (the sc1 bit is what the
// agent-scope store above carries); p is 16-byte aligned.  A quarter of the write transactions.
// The compiler does not see this store: drain_vmem() waits for it.
__device__ __forceinline__ void publish_f32x4(float *p, float4 x)
{
    typedef __attribute__((ext_vector_type(4))) float f4;
    const f4 v = {x.x, x.y, x.z, x.w};
    asm volatile("global_store_dwordx4 %0, %1, off sc1" ::"v"(p), "v"(v) : "memory");
}
__device__ __forceinline__ float fetch_f32(const float *p)
{
    return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

constexpr int kScaleHeads = 8;            // KV heads that may carry scales of their own (8-bit caches)

struct DecodeArgs {
    const void *q, *k, *v;
    const fairkv_item *items;   // grouped by slot
    float *part_o;              // [n_parts][G][D]   unnormalised outputs relative to the item's maximum
    float *part_ml;             // [n_parts][G][2]   (maximum in log2 units, sum of weights)
    int32_t *arrivals;          // [B*Hkv] items (or groups of items) of a cut pair that have delivered; 0 between calls
    int32_t *group_arrivals;    // [n_group_counters] the same per group of kGroup items, index first part + group
    void *out;
    float *lse;
    int32_t B, Hq, Hkv, out_dtype, n_parts, n_group_counters;
    int64_t n_rows;             // rows of k and of v
    int32_t q_len, g_shift;     // new tokens per sequence; log2 of the query heads per KV head.  A kernel's
                                // template parameter G counts columns: q_len * (1 << g_shift), column
                                // c = new token (c >> g_shift), head (c & mask) of the group
    float scale_log2;           // scale * log2(e) (times the K scale of an 8-bit cache): scores are kept in log2
                                // units so exp is one v_exp_f32
    float v_scale;              // 1, or the V scale of an 8-bit cache: multiplies out
    float k_head[kScaleHeads];  // 8-bit caches with a scale per KV head: further factors on scale_log2 and v_scale,
    float v_head[kScaleHeads];  // indexed h % kScaleHeads (all 1 otherwise; read by the 8-bit kernels only)
    // What a workgroup needs before it has read anything from memory, riding in the kernel arguments:
    int32_t slot_ptr[FAIRKV_MAX_SLOTS + 1];   // slot j runs items[slot_ptr[j] .. slot_ptr[j+1])
    uint32_t first_row[FAIRKV_MAX_SLOTS];     // first K/V row of slot j's first item ...
    uint32_t first_np[FAIRKV_MAX_SLOTS];      // ... its pair b*Hkv+h in bits 9..31 and min(tok_count, kEarlyTok) in
                                              // bits 0..8; 0 = no early start for this slot
    unsigned long long *trace;                // fairkv_decode_attn_trace only: [workgroups][kTraceStamps], else null
};

// Phases a traced launch stamps with the 100 MHz wall clock, per workgroup (thread 0 of wave 0).  A stamp
// keeps its latest value: the hand-over stamps are those of the workgroup's last hand-over.
enum {
    kTraceStart = 0,         // first instruction
    kTraceTable,             // item list landed and checked
    kTraceFirstTile,         // first K/V tile landed
    kTraceItem0Streamed,     // wave 0 has consumed its tiles of the first item
    kTraceItem0Done,         // first item folded and written (or kept pending)
    kTraceLastStreamed,      // wave 0 has consumed its tiles of the last item
    kTraceFlushBegin,        // hand-over: all waves are there
    kTraceFlushPublished,    // partials' stores issued
    kTraceFlushCounted,      // count-in returned, roles known
    kTraceFlushMerged,       // merges (if any) computed and written
    kTraceFlushEnd,
    kTraceEnd,               // last instruction
    kTraceMergeLoaded,       // the first batch of partials of the merges has landed (this stamp makes the merge wait for it)
    kTraceStamps = 16
};
__device__ __forceinline__ void trace_stamp(const DecodeArgs &a, int what, bool who)
{
    if (a.trace && who) a.trace[static_cast<size_t>(blockIdx.x) * kTraceStamps + what] = wall_clock64();
}
constexpr int kEarlyTok = 384;            // tokens of a slot's first item that the early start may request
static_assert(sizeof(DecodeArgs) <= 4096, "kernel arguments are limited to 4 KiB");

__device__ __forceinline__ size_t out_row(const DecodeArgs &a, int b, int h, int c)
{
    const int tok = c >> a.g_shift, g = c & ((1 << a.g_shift) - 1);
    return (static_cast<size_t>(b) * a.q_len + tok) * a.Hq + (h << a.g_shift) + g;
}

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


constexpr int kMergeBatch = 8;   // partials of a cut pair fetched at once by the merging workgroup

// Two floats fetched as one 8-byte agent-scope load (see publish_f32 / fetch_f32 above).
__device__ __forceinline__ float2 fetch_f32x2(const float *p)
{
    const uint64_t w = __hip_atomic_load(reinterpret_cast<const uint64_t *>(p), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    return make_float2(__uint_as_float(static_cast<uint32_t>(w)), __uint_as_float(static_cast<uint32_t>(w >> 32)));
}

// Partial results of cut pairs that a workgroup has finished but not yet handed over.  They
// wait in LDS until the slot's list is done (or the buffer is full) and are then published
// together, so that the hand-over, which costs several memory round trips, happens once per
// workgroup and not in the middle of the stream.
// Two: a line cut leaves a slot at most two pieces of cut pairs (its first and its last item).  A third
// slot made the hand-over code half as long again, and that code runs cold on the critical tail:
// 0.15 us per launch on the headline workload.
constexpr int pend_slots(int, int) { return 2; }

template <int D, int G>
struct PendingParts {
    static constexpr int kPend = pend_slots(D, G);
    __attribute__((aligned(16))) float o[kPend][G * D];
    float ml[kPend][G * 2];
    int32_t pair[kPend], part[kPend], first_part[kPend], n_chunks[kPend];
    int32_t role[kPend], src_first[kPend], src_stride[kPend], src_count[kPend];   // what this workgroup merges, if anything
    float v_mul[kPend];      // what multiplies the pair's output (1, or the V scale of an 8-bit cache)
};

// s_waitcnt vmcnt(0), once as an instruction the compiler accounts for (simm16 of gfx9: vmcnt 0,
// expcnt 7 and lgkmcnt 15 = no wait) and once as a fence for its own reordering of memory operations.
__device__ __forceinline__ void drain_vmem()
{
    __builtin_amdgcn_s_waitcnt(0x0F70);
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
}

// Hand over the pending partials.  Called by all threads of the workgroup.
//
// A pair cut into fewer than kDeepFrom pieces: publish the partial, wait until the stores are
// acknowledged, count in on the pair's counter; the workgroup that finds itself last merges the
// pair's partials (all of them were published before their workgroups counted in):
//   m* = max_c m_c,  l* = sum_c l_c 2^(m_c - m*),  out = sum_c o_c 2^(m_c - m*) / l*
// (exact in real arithmetic, so a cut pair gives what the whole pair would) and sets the counter
// back to zero.
//
// A pair cut into more pieces would make one workgroup fetch all of them at the rate of a single
// compute unit (79 pieces of a 16k-token head: 14 us).  Its pieces form groups of kGroup
// consecutive ones, each group with a counter of its own: the last piece of a group to arrive
// merges the group into one partial (m*, l*, sum_c o_c 2^(m_c - m*), not divided), stores it in the
// slot of the group's first piece, waits for the acknowledgement and only then counts in on the
// pair's counter, on which the last GROUP to arrive merges the group partials.  Two short merges
// by different workgroups instead of one long one.
constexpr int kGroup = 8;
// One merge by one workgroup costs about 0.7 us per kMergeBatch partials; the two-level way costs about
// 4 us of fixed round trips plus the short final merge.  It pays from about 30 pieces on.
constexpr int kDeepFrom = 32;
enum { kRoleNone = 0, kRoleFinal = 1, kRoleGroup = 2 };

template <int D, int G, bool DEEP, bool TRACE = false>
__device__ __forceinline__ void merge_round_one(const DecodeArgs &a, PendingParts<D, G> &pend, int n_pend)
{
    // A thread owns four consecutive coordinates of one column.  The first batch of loads of ALL
    // pending merges is issued before any is used: one memory round trip, not one per pair.
    constexpr int D4 = D / 4;
    constexpr int kPend = pend_slots(D, G);
    for (int idx = threadIdx.x; idx < G * D4; idx += kThreads) {
        const int g = idx / D4, d = (idx % D4) * 4;
        float2 ml[kPend][kMergeBatch], o01[kPend][kMergeBatch], o23[kPend][kMergeBatch];
#pragma unroll
        for (int p = 0; p < kPend; ++p) {
            if (p >= n_pend || pend.role[p] == kRoleNone || pend.src_count[p] < 2) continue;
            const int nc = pend.src_count[p], p0 = pend.src_first[p], st = pend.src_stride[p];
#pragma unroll
            for (int j = 0; j < kMergeBatch; ++j) {
                ml[p][j] = make_float2(-INFINITY, 0.f);        // past the end: weight 0 below, and no load
                o01[p][j] = o23[p][j] = make_float2(0.f, 0.f);
                if (j < nc) {
                    const size_t pg = static_cast<size_t>(p0 + st * j) * G + g;
                    ml[p][j] = fetch_f32x2(a.part_ml + pg * 2);
                    o01[p][j] = fetch_f32x2(a.part_o + pg * D + d);
                    o23[p][j] = fetch_f32x2(a.part_o + pg * D + d + 2);
                }
            }
        }
        if constexpr (TRACE) {      // measurement only: when the first batch of partials has landed
            drain_vmem();
            trace_stamp(a, kTraceMergeLoaded, threadIdx.x == 0);
        }
#pragma unroll
        for (int p = 0; p < kPend; ++p) {
            if (p >= n_pend || pend.role[p] == kRoleNone || pend.src_count[p] < 2) continue;
            const int nc = pend.src_count[p], p0 = pend.src_first[p], st = pend.src_stride[p], pair = pend.pair[p];
            float m_star = -INFINITY, l_star = 0.f, acc[4] = {0.f, 0.f, 0.f, 0.f};
            for (int c0 = 0; c0 < nc; c0 += kMergeBatch) {
                if (c0 > 0) {   // more than kMergeBatch partials: fetch the next batch
#pragma unroll
                    for (int j = 0; j < kMergeBatch; ++j) {
                        ml[p][j] = make_float2(-INFINITY, 0.f);
                        o01[p][j] = o23[p][j] = make_float2(0.f, 0.f);
                        if (c0 + j < nc) {
                            const size_t pg = static_cast<size_t>(p0 + st * (c0 + j)) * G + g;
                            ml[p][j] = fetch_f32x2(a.part_ml + pg * 2);
                            o01[p][j] = fetch_f32x2(a.part_o + pg * D + d);
                            o23[p][j] = fetch_f32x2(a.part_o + pg * D + d + 2);
                        }
                    }
                }
                float m_new = m_star;
#pragma unroll
                for (int j = 0; j < kMergeBatch; ++j)
                    if (c0 + j < nc) m_new = fmaxf(m_new, ml[p][j].x);
                const float keep = m_star == -INFINITY ? 0.f : __builtin_amdgcn_exp2f(m_star - m_new);
                l_star *= keep;
#pragma unroll
                for (int e = 0; e < 4; ++e) acc[e] *= keep;
#pragma unroll
                for (int j = 0; j < kMergeBatch; ++j) {
                    const bool live = c0 + j < nc && ml[p][j].x != -INFINITY;
                    const float f = live ? __builtin_amdgcn_exp2f(ml[p][j].x - m_new) : 0.f;
                    l_star = fmaf(ml[p][j].y, f, l_star);
                    acc[0] = fmaf(o01[p][j].x, f, acc[0]);
                    acc[1] = fmaf(o01[p][j].y, f, acc[1]);
                    acc[2] = fmaf(o23[p][j].x, f, acc[2]);
                    acc[3] = fmaf(o23[p][j].y, f, acc[3]);
                }
                m_star = m_new;
            }
            if (DEEP && pend.role[p] == kRoleGroup) {  // the group's partial, in the slot of its first piece
                const size_t pg = static_cast<size_t>(p0) * G + g;
                publish_f32x4(a.part_o + pg * D + d, make_float4(acc[0], acc[1], acc[2], acc[3]));
                if (d == 0) {
                    publish_f32(a.part_ml + pg * 2 + 0, m_star);
                    publish_f32(a.part_ml + pg * 2 + 1, l_star);
                }
                continue;
            }
            const int b = pair / a.Hkv, h = pair % a.Hkv;
            const size_t orow = out_row(a, b, h, g);
            const float inv = l_star > 0.f ? pend.v_mul[p] / l_star : 0.f;
            store_out4(a.out, a.out_dtype, orow * D + d, make_float4(acc[0] * inv, acc[1] * inv, acc[2] * inv, acc[3] * inv));
            if (d == 0 && a.lse)
                a.lse[orow] = l_star > 0.f ? (m_star + __builtin_amdgcn_logf(l_star)) * kLn2 : -INFINITY;
        }
    }
}

template <int D, int G, bool DEEP>
__device__ __forceinline__ void merge_round_many(const DecodeArgs &a, PendingParts<D, G> &pend, int n_pend)
{
    // A thread owns four consecutive coordinates of one column (of two columns, when there are 16 of them).
    // The first batch of loads of ALL pending merges and of all the thread's coordinates is issued before
    // any is used: one memory round trip, not one per pair or per coordinate.
    constexpr int D4 = D / 4, NC4 = G * D4;
    constexpr int kPend = pend_slots(D, G);
    constexpr int IT = (NC4 + kThreads - 1) / kThreads;            // coordinates per thread
    constexpr int MB = IT > 1 ? kMergeBatch / 2 : kMergeBatch;     // 6 IT kPend MB registers hold the batches
    float2 ml[IT][kPend][MB], o01[IT][kPend][MB], o23[IT][kPend][MB];
    auto fetch_batch = [&](int it, int p, int c0) __attribute__((always_inline)) {
        const int idx = threadIdx.x + it * kThreads, g = idx / D4, d = (idx % D4) * 4;
        const int nc = pend.src_count[p], p0 = pend.src_first[p], st = pend.src_stride[p];
#pragma unroll
        for (int j = 0; j < MB; ++j) {
            ml[it][p][j] = make_float2(-INFINITY, 0.f);        // past the end: weight 0 below, and no load
            o01[it][p][j] = o23[it][p][j] = make_float2(0.f, 0.f);
            if (c0 + j < nc) {
                const size_t pg = static_cast<size_t>(p0 + st * (c0 + j)) * G + g;
                ml[it][p][j] = fetch_f32x2(a.part_ml + pg * 2);
                o01[it][p][j] = fetch_f32x2(a.part_o + pg * D + d);
                o23[it][p][j] = fetch_f32x2(a.part_o + pg * D + d + 2);
            }
        }
    };
#pragma unroll
    for (int it = 0; it < IT; ++it) {
        if (threadIdx.x + it * kThreads >= NC4) continue;
#pragma unroll
        for (int p = 0; p < kPend; ++p) {
            if (p >= n_pend || pend.role[p] == kRoleNone || pend.src_count[p] < 2) continue;
            fetch_batch(it, p, 0);
        }
    }
#pragma unroll
    for (int it = 0; it < IT; ++it) {
        const int idx = threadIdx.x + it * kThreads, g = idx / D4, d = (idx % D4) * 4;
        if (idx >= NC4) continue;
#pragma unroll
        for (int p = 0; p < kPend; ++p) {
            if (p >= n_pend || pend.role[p] == kRoleNone || pend.src_count[p] < 2) continue;
            const int nc = pend.src_count[p], p0 = pend.src_first[p], pair = pend.pair[p];
            float m_star = -INFINITY, l_star = 0.f, acc[4] = {0.f, 0.f, 0.f, 0.f};
            for (int c0 = 0; c0 < nc; c0 += MB) {
                if (c0 > 0) fetch_batch(it, p, c0);     // more than MB partials: the next batch
                float m_new = m_star;
#pragma unroll
                for (int j = 0; j < MB; ++j)
                    if (c0 + j < nc) m_new = fmaxf(m_new, ml[it][p][j].x);
                const float keep = m_star == -INFINITY ? 0.f : __builtin_amdgcn_exp2f(m_star - m_new);
                l_star *= keep;
#pragma unroll
                for (int e = 0; e < 4; ++e) acc[e] *= keep;
#pragma unroll
                for (int j = 0; j < MB; ++j) {
                    const bool live = c0 + j < nc && ml[it][p][j].x != -INFINITY;
                    const float f = live ? __builtin_amdgcn_exp2f(ml[it][p][j].x - m_new) : 0.f;
                    l_star = fmaf(ml[it][p][j].y, f, l_star);
                    acc[0] = fmaf(o01[it][p][j].x, f, acc[0]);
                    acc[1] = fmaf(o01[it][p][j].y, f, acc[1]);
                    acc[2] = fmaf(o23[it][p][j].x, f, acc[2]);
                    acc[3] = fmaf(o23[it][p][j].y, f, acc[3]);
                }
                m_star = m_new;
            }
            if (DEEP && pend.role[p] == kRoleGroup) {  // the group's partial, in the slot of its first piece
                const size_t pg = static_cast<size_t>(p0) * G + g;
                publish_f32x4(a.part_o + pg * D + d, make_float4(acc[0], acc[1], acc[2], acc[3]));
                if (d == 0) {
                    publish_f32(a.part_ml + pg * 2 + 0, m_star);
                    publish_f32(a.part_ml + pg * 2 + 1, l_star);
                }
                continue;
            }
            const int b = pair / a.Hkv, h = pair % a.Hkv;
            const size_t orow = out_row(a, b, h, g);
            const float inv = l_star > 0.f ? pend.v_mul[p] / l_star : 0.f;
            store_out4(a.out, a.out_dtype, orow * D + d, make_float4(acc[0] * inv, acc[1] * inv, acc[2] * inv, acc[3] * inv));
            if (d == 0 && a.lse)
                a.lse[orow] = l_star > 0.f ? (m_star + __builtin_amdgcn_logf(l_star)) * kLn2 : -INFINITY;
        }
    }
}

// Up to 256 float4 coordinates (G * D <= 1024) a thread owns at most one: the plain loop, whose code is the
// shorter (0.2 us per launch on the headline workload: this code runs cold, on the tail).  With more, all of
// a thread's coordinates are fetched together.
template <int D, int G, bool DEEP, bool TRACE = false>
__device__ __forceinline__ void merge_round(const DecodeArgs &a, PendingParts<D, G> &pend, int n_pend)
{
    if constexpr (G * D / 4 <= kThreads)
        merge_round_one<D, G, DEEP, TRACE>(a, pend, n_pend);
    else
        merge_round_many<D, G, DEEP>(a, pend, n_pend);
}

// DEEP: the plan has a pair in kDeepFrom pieces or more.  Without it the group code is not even compiled
// in: on the headline workload its mere presence cost 0.8 us per launch (longer cold code on the
// critical tail, more registers in the main loop).
template <int D, int G, bool DEEP, bool TRACE = false>
__device__ __forceinline__ void flush_pending(const DecodeArgs &a, PendingParts<D, G> &pend, int &n_pend)
{
    __syncthreads();
    if constexpr (TRACE) trace_stamp(a, kTraceFlushBegin, threadIdx.x == 0);
    for (int p = 0; p < n_pend; ++p) {
        const size_t base = static_cast<size_t>(pend.part[p]) * G;
        for (int idx = threadIdx.x; idx < G * D / 4; idx += kThreads)
            publish_f32x4(a.part_o + base * D + idx * 4, *reinterpret_cast<const float4 *>(&pend.o[p][idx * 4]));
        if (threadIdx.x < G * 2) publish_f32(a.part_ml + base * 2 + threadIdx.x, pend.ml[p][threadIdx.x]);
    }
    drain_vmem();                                      // this thread's stores have reached the shared level ...
    __syncthreads();                                   // ... and every other thread's, before the workgroup counts itself in
    if constexpr (TRACE) trace_stamp(a, kTraceFlushPublished, threadIdx.x == 0);
    // Round 0: every pending piece counts in (a piece of a deeply cut pair on its group's counter) and
    // the last arrivals merge.  Round 1, only if this workgroup merged a group: that group counts in on
    // the pair's counter.  One copy of the merge code serves both rounds: the hand-over runs once per
    // workgroup, on cold instruction-cache lines, so its length is paid for in full.
    for (int round = 0; round < (DEEP ? 2 : 1); ++round) {
        if (threadIdx.x < n_pend) {
            const int p = threadIdx.x;
            const int nc = pend.n_chunks[p], p0 = pend.first_part[p], chunk = pend.part[p] - p0;
            const bool ok = p0 >= 0 && chunk >= 0 && chunk < nc && p0 + nc <= a.n_parts;
            // two levels only if every group of the pair has a counter
            const bool deep = DEEP && nc >= kDeepFrom && static_cast<int64_t>(p0) + (nc - 1) / kGroup < a.n_group_counters;
            int role = kRoleNone;
            if (round == 0 && ok && !deep) {
                if (__hip_atomic_fetch_add(a.arrivals + pend.pair[p], 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) == nc - 1)
                    role = kRoleFinal;
                pend.src_first[p] = p0;
                pend.src_stride[p] = 1;
                pend.src_count[p] = nc;
            } else if (round == 0 && ok) {
                const int k = chunk / kGroup, gs = min(kGroup, nc - k * kGroup);
                if (__hip_atomic_fetch_add(a.group_arrivals + p0 + k, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) == gs - 1)
                    role = kRoleGroup;
                pend.src_first[p] = p0 + k * kGroup;
                pend.src_stride[p] = 1;
                pend.src_count[p] = gs;
            } else if (round == 1 && pend.role[p] == kRoleGroup) {
                const int ng = (nc + kGroup - 1) / kGroup;
                __hip_atomic_store(a.group_arrivals + p0 + chunk / kGroup, 0, __ATOMIC_RELAXED,
                                   __HIP_MEMORY_SCOPE_AGENT);      // the group's counter: ready for the next call
                if (__hip_atomic_fetch_add(a.arrivals + pend.pair[p], 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) == ng - 1)
                    role = kRoleFinal;
                pend.src_first[p] = p0;
                pend.src_stride[p] = kGroup;
                pend.src_count[p] = ng;
            }
            pend.role[p] = role;
        }
        __syncthreads();
        if constexpr (TRACE) trace_stamp(a, kTraceFlushCounted, threadIdx.x == 0);
        merge_round<D, G, DEEP, TRACE>(a, pend, n_pend);
        if constexpr (TRACE) trace_stamp(a, kTraceFlushMerged, threadIdx.x == 0);
        bool any_group = false;
        if (DEEP)
            for (int p = 0; p < n_pend; ++p) any_group |= pend.role[p] == kRoleGroup;
        if (threadIdx.x < n_pend && pend.role[threadIdx.x] == kRoleFinal)   // ready for the next call on this workspace
            __hip_atomic_store(a.arrivals + pend.pair[threadIdx.x], 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        if (!any_group) break;                             // uniform: the roles are in LDS
        drain_vmem();                                      // the group partials are acknowledged ...
        __syncthreads();                                   // ... all of them, before the groups count in
    }
    n_pend = 0;
    drain_vmem();     // the compiler stops tracking the loads above: no guard waits on their registers later on
    __syncthreads();
    if constexpr (TRACE) trace_stamp(a, kTraceFlushEnd, threadIdx.x == 0);
}

// End of one item, called by all threads of the workgroup after every wave has put its
// unnormalised output, running maximum (log2 units) and weight sum into st_o [kWaves][G][D]
// and st_ml [kWaves][G][2] in LDS.  Folds the waves:
//   m* = max_w m_w,  l* = sum_w l_w 2^(m_w - m*),  o* = sum_w o_w 2^(m_w - m*).
// An item that is a whole pair writes out = o*/l* and lse.  An item of a cut pair leaves its
// partial (m*, l*, o*) in `pend`.  Ends with a barrier, so st_o/st_ml may be reused at once.
template <int D, int G, bool DEEP, bool TRACE = false>
__device__ __forceinline__ void item_epilogue(const DecodeArgs &a, const fairkv_item &it, const float *st_o,
                                              const float *st_ml, PendingParts<D, G> &pend, int &n_pend, float v_mul)
{
    const int b = it.b, h = it.h;
    const bool whole_pair = it.n_chunks == 1;
    constexpr int D4 = D / 4;
    __syncthreads();
    // a thread owns four consecutive coordinates of one query head; all its LDS reads are issued together
    for (int idx = threadIdx.x; idx < G * D4; idx += kThreads) {
        const int g = idx / D4, d = (idx % D4) * 4;
        float2 ml[kWaves];
        float4 ow[kWaves];
#pragma unroll
        for (int w = 0; w < kWaves; ++w) {
            ml[w] = *reinterpret_cast<const float2 *>(st_ml + (w * G + g) * 2);
            ow[w] = *reinterpret_cast<const float4 *>(st_o + (w * G + g) * D + d);
        }
        float m_star = -INFINITY;
#pragma unroll
        for (int w = 0; w < kWaves; ++w) m_star = fmaxf(m_star, ml[w].x);
        float4 acc = make_float4(0.f, 0.f, 0.f, 0.f);
        float l_star = 0.f;
#pragma unroll
        for (int w = 0; w < kWaves; ++w) {
            const float f = ml[w].x == -INFINITY ? 0.f : __builtin_amdgcn_exp2f(ml[w].x - m_star);
            acc.x += ow[w].x * f;
            acc.y += ow[w].y * f;
            acc.z += ow[w].z * f;
            acc.w += ow[w].w * f;
            l_star += ml[w].y * f;
        }
        if (whole_pair) {
            const size_t orow = out_row(a, b, h, g);
            const float inv = l_star > 0.f ? v_mul / l_star : 0.f;
            store_out4(a.out, a.out_dtype, orow * D + d, make_float4(acc.x * inv, acc.y * inv, acc.z * inv, acc.w * inv));
            if (d == 0 && a.lse)
                a.lse[orow] = l_star > 0.f ? (m_star + __builtin_amdgcn_logf(l_star)) * kLn2 : -INFINITY;
        } else {
            *reinterpret_cast<float4 *>(&pend.o[n_pend][idx * 4]) = acc;
            if (d == 0) {
                pend.ml[n_pend][g * 2 + 0] = m_star;
                pend.ml[n_pend][g * 2 + 1] = l_star;
            }
        }
    }
    if (!whole_pair) {
        if (threadIdx.x == 0) {
            pend.pair[n_pend] = b * a.Hkv + h;
            pend.part[n_pend] = it.part;
            pend.first_part[n_pend] = it.part - it.chunk;   // the partials of a pair are consecutive
            pend.n_chunks[n_pend] = it.n_chunks;
            pend.v_mul[n_pend] = v_mul;
        }
        ++n_pend;
        if (n_pend == pend_slots(D, G)) {
            flush_pending<D, G, DEEP, TRACE>(a, pend, n_pend);
            return;
        }
    }
    __syncthreads();
}

}  // namespace fairkv

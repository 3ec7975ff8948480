// Building and growing the packed ragged cache on the GPU: gather of the kept rows of a dense
// K/V cache (what a per-head compressor leaves behind, Section 2) and the append of a decode
// step's new row per pair.  Pure data movement: rows travel as 16-byte pieces, a wave-wide
// access covers whole rows, so every read and write is a run of fully used cache lines.
#pragma once
#include <hip/hip_runtime.h>

#include <cstdint>

#include "fairkv.h"

namespace fairkv {

struct PackArgs {
    const char *k_dense, *v_dense;    // [B][Hkv][T][row bytes]
    char *k_out, *v_out;              // [n_rows][row bytes]
    const int64_t *keep_ptr;          // [B*Hkv+1]
    const int32_t *keep_t;            // [keep_ptr[B*Hkv]]
    const int64_t *off;               // [B*Hkv]
    const fairkv_item *items;         // work list: (row, tok_count, b, h) name runs of packed rows
    const int32_t *slot_ptr;          // [gridDim.x + 1]
    int32_t *bad;                     // rows and items skipped because they point outside; may be null
    int64_t n_rows;
    int32_t B, Hkv, T;
};

// One workgroup per slot of the work list.  An item is a run of rows of one pair; the workgroup
// moves kRowsPerPass rows per pass and keeps kUnroll passes in flight.
template <int ROWB>
__global__ __launch_bounds__(256) void fairkv_pack_kernel(PackArgs a)
{
    typedef __attribute__((ext_vector_type(4))) uint32_t u4;   // rows are read once and written once: non-temporal both ways
    constexpr int PPR = ROWB / 16;            // 16-byte pieces per row
    constexpr int kRowsPerPass = 256 / PPR;
    constexpr int kUnroll = 1;   // measured: 1 -> 36.7 us, 2 -> 42, 4 -> 48, 8 -> 61 for the 140 MB of the llama70b layer
    const int piece = threadIdx.x % PPR, sub = threadIdx.x / PPR;
    for (int i = a.slot_ptr[blockIdx.x]; i < a.slot_ptr[blockIdx.x + 1]; ++i) {
        const fairkv_item it = a.items[i];
        const int n = it.tok_count;
        if (n <= 0) continue;
        bool ok = it.b >= 0 && it.b < a.B && it.h >= 0 && it.h < a.Hkv && it.row >= 0 && it.row + n <= a.n_rows;
        int64_t pair = 0, begin = 0, first = 0;
        if (ok) {
            pair = static_cast<int64_t>(it.b) * a.Hkv + it.h;
            begin = it.row - a.off[pair];
            first = a.keep_ptr[pair];
            ok = begin >= 0 && first >= 0 && begin + n <= a.keep_ptr[pair + 1] - first;
        }
        if (!ok) {
            if (threadIdx.x == 0 && a.bad) atomicAdd(a.bad, 1);
            continue;
        }
        const int32_t *kt = a.keep_t + first + begin;
        const char *ksrc = a.k_dense + pair * a.T * ROWB + piece * 16;
        const char *vsrc = a.v_dense + pair * a.T * ROWB + piece * 16;
        char *kdst = a.k_out + it.row * ROWB + piece * 16;
        char *vdst = a.v_out + it.row * ROWB + piece * 16;
        // All indices of a round first, then all row loads, then the stores: nothing in a round waits
        // for an earlier load of the same round.  Rows past the end and rows with a bad index are
        // loaded from a clamped (valid) address and not stored.
        // The indices of the next round are requested before the rows of this one, so a round costs one
        // memory latency (the rows), not two (index, then rows).
        int32_t t_next[kUnroll];
#pragma unroll
        for (int u = 0; u < kUnroll; ++u) t_next[u] = kt[min(u * kRowsPerPass + sub, n - 1)];
        for (int r0 = 0; r0 < n; r0 += kRowsPerPass * kUnroll) {
            int32_t t[kUnroll];
#pragma unroll
            for (int u = 0; u < kUnroll; ++u) {
                t[u] = t_next[u];
                t_next[u] = kt[min(r0 + (kUnroll + u) * kRowsPerPass + sub, n - 1)];
            }
            u4 kk[kUnroll], vv[kUnroll];
#pragma unroll
            for (int u = 0; u < kUnroll; ++u) {
                const int64_t tc = min(max(t[u], 0), a.T - 1);
                kk[u] = __builtin_nontemporal_load(reinterpret_cast<const u4 *>(ksrc + tc * ROWB));
                vv[u] = __builtin_nontemporal_load(reinterpret_cast<const u4 *>(vsrc + tc * ROWB));
            }
#pragma unroll
            for (int u = 0; u < kUnroll; ++u) {
                const int r = r0 + u * kRowsPerPass + sub;
                if (r >= n) continue;
                if (t[u] < 0 || t[u] >= a.T) {
                    if (piece == 0 && a.bad) atomicAdd(a.bad, 1);
                    continue;
                }
                __builtin_nontemporal_store(kk[u], reinterpret_cast<u4 *>(kdst + static_cast<int64_t>(r) * ROWB));
                __builtin_nontemporal_store(vv[u], reinterpret_cast<u4 *>(vdst + static_cast<int64_t>(r) * ROWB));
            }
        }
    }
}

struct AppendArgs {
    const char *k_new, *v_new;   // [B*Hkv][row bytes]
    char *k, *v;                 // packed
    const int64_t *off;
    int32_t *len;                // in/out
    const int32_t *cap;
    int32_t *full;               // pairs found at capacity; may be null
    int64_t n_rows;
    int32_t n_pairs;
};

// A pair is served by PPR consecutive lanes of one wave (PPR divides 64): all of them read the
// pair's length with the same instruction, before the lane of piece 0 stores the new length.
template <int ROWB>
__global__ __launch_bounds__(256) void fairkv_append_kernel(AppendArgs a)
{
    constexpr int PPR = ROWB / 16;
    const int64_t idx = static_cast<int64_t>(blockIdx.x) * 256 + threadIdx.x;
    const int64_t pair = idx / PPR;
    const int piece = static_cast<int>(idx % PPR);
    if (pair >= a.n_pairs) return;
    const int32_t l = a.len[pair];
    const int64_t row = a.off[pair] + l;
    if (l < 0 || l >= a.cap[pair] || a.off[pair] < 0 || row >= a.n_rows) {
        if (piece == 0 && a.full) atomicAdd(a.full, 1);
        return;
    }
    const uint4 kk = *reinterpret_cast<const uint4 *>(a.k_new + pair * ROWB + piece * 16);
    const uint4 vv = *reinterpret_cast<const uint4 *>(a.v_new + pair * ROWB + piece * 16);
    *reinterpret_cast<uint4 *>(a.k + row * ROWB + piece * 16) = kk;
    *reinterpret_cast<uint4 *>(a.v + row * ROWB + piece * 16) = vv;
    if (piece == 0) a.len[pair] = l + 1;
}

}  // namespace fairkv

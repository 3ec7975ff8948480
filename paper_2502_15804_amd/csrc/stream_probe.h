// A reader with nothing to do: the K and V rows of a packed cache streamed HBM -> LDS through the
// same per-wave rings, with the same launch shape, as the decode kernel, split evenly over the
// workgroups; no item list, no arithmetic, nothing written.  What it achieves is the ceiling of this
// data path on this GPU for a given number of bytes, to set beside the decode kernel's time.
#pragma once
#include "decode_mfma.h"

namespace fairkv {

struct ProbeArgs {
    const char *k, *v;
    int64_t bytes_per_workgroup;   // from each of k and v; a multiple of the tile size
    uint32_t *sink;                // never written (the condition below cannot hold for real data)
};

// WAVES waves per workgroup, each with a ring of STAGES stages of (LPT KiB of K + LPT KiB of V): the decode kernel's
// shape is <kWaves, ring_stages(8), 4>; the others exist for the launch-shape sweep of fairkv_stream_probe_shape.
template <int WAVES, int STAGES, int LPT>
__global__ __launch_bounds__(WAVES * 64, 1) void fairkv_stream_probe_kernel(ProbeArgs a)
{
    constexpr int TILEB = LPT * 1024;
    constexpr int STAGEB = 2 * TILEB;
    constexpr int LOADS = 2 * LPT;
    static_assert(STAGES >= 2 && STAGES <= 4, "wait_all_but knows up to three tiles in flight behind the current one");
    extern __shared__ __attribute__((aligned(1024))) char lds[];      // WAVES * STAGES * STAGEB bytes
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const uint32_t ring = static_cast<uint32_t>(reinterpret_cast<uintptr_t>(FAIRKV_LDS_PTR(lds))) + wave * (STAGES * STAGEB);
    const char *kb = a.k + static_cast<int64_t>(blockIdx.x) * a.bytes_per_workgroup;
    const char *vb = a.v + static_cast<int64_t>(blockIdx.x) * a.bytes_per_workgroup;
    const int n_tiles = static_cast<int>(a.bytes_per_workgroup / TILEB);
    const int my_tiles = n_tiles > wave ? (n_tiles - wave + WAVES - 1) / WAVES : 0;
    int f_stage = 0, c_stage = 0, ahead = 0, f_t = 0;
    uint32_t acc = 0;
    for (int t = 0; t < my_tiles; ++t) {
        while (ahead < STAGES && f_t < my_tiles) {
            const uint32_t off = static_cast<uint32_t>((wave + f_t * WAVES) * TILEB + lane * 16);
#pragma unroll
            for (int i = 0; i < LPT; ++i) {
                load16_to_lds(kb, off + i * 1024, ring + f_stage * STAGEB + i * 1024);
                load16_to_lds(vb, off + i * 1024, ring + f_stage * STAGEB + TILEB + i * 1024);
            }
            f_stage = f_stage + 1 == STAGES ? 0 : f_stage + 1;
            ++f_t;
            ++ahead;
        }
        wait_all_but<LOADS, 1>(ahead - 1, 0);
        acc ^= *reinterpret_cast<const uint32_t *>(lds + wave * (STAGES * STAGEB) + c_stage * STAGEB + lane * 4);
        c_stage = c_stage + 1 == STAGES ? 0 : c_stage + 1;
        --ahead;
    }
    if (acc == 0x7fc01234u && a.bytes_per_workgroup < 0) a.sink[blockIdx.x] = acc;
}

}  // namespace fairkv

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

__global__ __launch_bounds__(kThreads, 1) void fairkv_stream_probe_kernel(ProbeArgs a)
{
    constexpr int kStages = ring_stages(8);      // the ring of the decode kernel for up to 8 columns
    constexpr int LPT = 4;                 // wave-wide loads per 4 KB K (or V) tile
    constexpr int TILEB = LPT * 1024;
    constexpr int STAGEB = 2 * TILEB;
    constexpr int LOADS = 2 * LPT;
    __shared__ __attribute__((aligned(1024))) char lds[kWaves * kStages * STAGEB];
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const uint32_t ring = static_cast<uint32_t>(reinterpret_cast<uintptr_t>(FAIRKV_LDS_PTR(lds))) + wave * (kStages * STAGEB);
    const char *kb = a.k + static_cast<int64_t>(blockIdx.x) * a.bytes_per_workgroup;
    const char *vb = a.v + static_cast<int64_t>(blockIdx.x) * a.bytes_per_workgroup;
    const int n_tiles = static_cast<int>(a.bytes_per_workgroup / TILEB);
    const int my_tiles = n_tiles > wave ? (n_tiles - wave + kWaves - 1) / kWaves : 0;
    int f_stage = 0, c_stage = 0, ahead = 0, f_t = 0;
    uint32_t acc = 0;
    for (int t = 0; t < my_tiles; ++t) {
        while (ahead < kStages && f_t < my_tiles) {
            const uint32_t off = static_cast<uint32_t>((wave + f_t * kWaves) * TILEB + lane * 16);
#pragma unroll
            for (int i = 0; i < LPT; ++i) {
                load16_to_lds(kb, off + i * 1024, ring + f_stage * STAGEB + i * 1024);
                load16_to_lds(vb, off + i * 1024, ring + f_stage * STAGEB + TILEB + i * 1024);
            }
            f_stage = f_stage + 1 == kStages ? 0 : f_stage + 1;
            ++f_t;
            ++ahead;
        }
        wait_all_but<LOADS, 1>(ahead - 1, 0);
        acc ^= *reinterpret_cast<const uint32_t *>(lds + wave * (kStages * STAGEB) + c_stage * STAGEB + lane * 4);
        c_stage = c_stage + 1 == kStages ? 0 : c_stage + 1;
        --ahead;
    }
    if (acc == 0x7fc01234u && a.bytes_per_workgroup < 0) a.sink[blockIdx.x] = acc;
}

}  // namespace fairkv

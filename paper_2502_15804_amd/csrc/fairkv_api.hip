// C ABI of the device side: argument checks, kernel selection and launches.
//
// The paper (Section 3.2) observes that decoding one token is bound by memory bandwidth
// and costs time linear in batch x retained tokens, so the job of the kernels is to stream
// every retained K and V row from HBM exactly once, at full rate, whatever the per-head
// lengths are.  One workgroup takes one work item of the plan (a token chunk of one
// (sequence, KV head) pair) and serves all G query heads of the group from the same K/V
// rows.  Heavy pairs arrive cut into several items (the single-GPU form of Fair-Copying,
// Section 4.2); their partial results are combined by the merge kernel.
#include <hip/hip_runtime.h>

#include <cmath>
#include <cstdint>
#include <cstdlib>

#include "decode_mfma.h"
#include "decode_valu.h"
#include "fairkv.h"
#include "merge.h"

namespace {

using namespace fairkv;

template <int IN_DT, int D>
hipError_t launch_valu(int G, const DecodeArgs &a, int n_items, hipStream_t st)
{
    const dim3 grid(static_cast<unsigned>(n_items)), block(kThreads);
    switch (G) {
    case 1: hipLaunchKernelGGL((fairkv_decode_valu_kernel<IN_DT, D, 1>), grid, block, 0, st, a); break;
    case 2: hipLaunchKernelGGL((fairkv_decode_valu_kernel<IN_DT, D, 2>), grid, block, 0, st, a); break;
    case 4: hipLaunchKernelGGL((fairkv_decode_valu_kernel<IN_DT, D, 4>), grid, block, 0, st, a); break;
    case 8: hipLaunchKernelGGL((fairkv_decode_valu_kernel<IN_DT, D, 8>), grid, block, 0, st, a); break;
    default: return hipErrorInvalidValue;
    }
    return hipGetLastError();
}

template <int D>
hipError_t launch_mfma(int G, const DecodeArgs &a, int n_items, hipStream_t st)
{
    const dim3 grid(static_cast<unsigned>(n_items)), block(kThreads);
    switch (G) {
    case 1: hipLaunchKernelGGL((fairkv_decode_mfma_kernel<D, 1>), grid, block, 0, st, a); break;
    case 2: hipLaunchKernelGGL((fairkv_decode_mfma_kernel<D, 2>), grid, block, 0, st, a); break;
    case 4: hipLaunchKernelGGL((fairkv_decode_mfma_kernel<D, 4>), grid, block, 0, st, a); break;
    case 8: hipLaunchKernelGGL((fairkv_decode_mfma_kernel<D, 8>), grid, block, 0, st, a); break;
    default: return hipErrorInvalidValue;
    }
    return hipGetLastError();
}

bool aligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

// FAIRKV_BF16_KERNEL=valu sends bf16 inputs through the vector-ALU kernel (for A/B
// measurements of the two kernels); anything else, or unset, uses the matrix-core kernel.
bool bf16_on_valu()
{
    static const bool v = [] {
        const char *e = std::getenv("FAIRKV_BF16_KERNEL");
        return e && e[0] == 'v';
    }();
    return v;
}

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
        if (in_dtype == FAIRKV_BF16 && !bf16_on_valu())
            e = D == 128 ? launch_mfma<128>(G, a, n_items, st) : launch_mfma<64>(G, a, n_items, st);
        else if (in_dtype == FAIRKV_BF16)
            e = D == 128 ? launch_valu<FAIRKV_BF16, 128>(G, a, n_items, st)
                         : launch_valu<FAIRKV_BF16, 64>(G, a, n_items, st);
        else
            e = D == 128 ? launch_valu<FAIRKV_F32, 128>(G, a, n_items, st)
                         : launch_valu<FAIRKV_F32, 64>(G, a, n_items, st);
        if (e != hipSuccess) return FAIRKV_EHIP;
    }
    hipLaunchKernelGGL(fairkv_merge_kernel, dim3(static_cast<unsigned>(B * Hkv)), dim3(kThreads), 0, st,
                       a.part_o, a.part_ml, part_base, out, lse, Hq, Hkv, G, D, out_dtype);
    if (hipGetLastError() != hipSuccess) return FAIRKV_EHIP;
    return FAIRKV_OK;
}

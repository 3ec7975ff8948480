// C ABI of the device side: argument checks, kernel selection and launches.
//
// The paper (Section 3.2) observes that decoding one token is bound by memory bandwidth
// and costs time linear in batch x retained tokens, so the job of the kernels is to stream
// every retained K and V row from HBM exactly once, at full rate, whatever the per-head
// lengths are.  A persistent workgroup per slot walks the work items the planner gave it
// (token chunks of (sequence, KV head) pairs) and serves all G query heads of a group from the same K/V
// rows.  Heavy pairs arrive cut into several items (the single-GPU form of Fair-Copying,
// Section 4.2); the workgroup that delivers the last partial result of a pair combines them.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <atomic>
#include <cmath>
#include <cstdint>
#include <cstdlib>
#include <vector>

#include "decode_mfma.h"
#include "decode_valu.h"
#include "pack.h"
#include "stream_probe.h"
#include "fairkv.h"
#include "fairkv_measure.h"

namespace {

using namespace fairkv;
static_assert(kTraceStamps == FAIRKV_TRACE_STAMPS, "the header's stamp count is the kernel's");

template <int IN_DT, int D>
hipError_t launch_valu(int G, const DecodeArgs &a, int n_slots, hipStream_t st)
{
    const dim3 grid(static_cast<unsigned>(n_slots)), block(kThreads);
    switch (G) {
    case 1: hipLaunchKernelGGL((fairkv_decode_valu_kernel<IN_DT, D, 1>), grid, block, 0, st, a); break;
    case 2: hipLaunchKernelGGL((fairkv_decode_valu_kernel<IN_DT, D, 2>), grid, block, 0, st, a); break;
    case 4: hipLaunchKernelGGL((fairkv_decode_valu_kernel<IN_DT, D, 4>), grid, block, 0, st, a); break;
    case 8: hipLaunchKernelGGL((fairkv_decode_valu_kernel<IN_DT, D, 8>), grid, block, 0, st, a); break;
    default: return hipErrorInvalidValue;
    }
    return hipGetLastError();
}

// The measurement instantiation exists for the shapes the benchmark traces: D = 128, bf16, 4 or 8 query heads per KV head.
hipError_t launch_mfma_trace(int G, bool deep, const DecodeArgs &a, int n_slots, hipStream_t st)
{
    const dim3 grid(static_cast<unsigned>(n_slots)), block(kThreads);
    if (G == 4 && !deep)
        hipLaunchKernelGGL((fairkv_decode_mfma_kernel<128, 4, false, false, true, true>), grid, block, 0, st, a);
    else if (G == 4)
        hipLaunchKernelGGL((fairkv_decode_mfma_kernel<128, 4, true, false, true, true>), grid, block, 0, st, a);
    else if (G == 8 && !deep)
        hipLaunchKernelGGL((fairkv_decode_mfma_kernel<128, 8, false, false, true, true>), grid, block, 0, st, a);
    else if (G == 8)
        hipLaunchKernelGGL((fairkv_decode_mfma_kernel<128, 8, true, false, true, true>), grid, block, 0, st, a);
    else
        return hipErrorInvalidValue;
    return hipGetLastError();
}

template <int D, bool DEEP, bool KV8, bool SOLO>
hipError_t launch_mfma_g(int G, const DecodeArgs &a, int n_slots, hipStream_t st)
{
    const dim3 grid(static_cast<unsigned>(n_slots)), block(kThreads);
    switch (G) {
    case 1: hipLaunchKernelGGL((fairkv_decode_mfma_kernel<D, 1, DEEP, KV8, SOLO>), grid, block, 0, st, a); break;
    case 2: hipLaunchKernelGGL((fairkv_decode_mfma_kernel<D, 2, DEEP, KV8, SOLO>), grid, block, 0, st, a); break;
    case 4: hipLaunchKernelGGL((fairkv_decode_mfma_kernel<D, 4, DEEP, KV8, SOLO>), grid, block, 0, st, a); break;
    case 8: hipLaunchKernelGGL((fairkv_decode_mfma_kernel<D, 8, DEEP, KV8, SOLO>), grid, block, 0, st, a); break;
    case 16: hipLaunchKernelGGL((fairkv_decode_mfma_kernel<D, 16, DEEP, KV8, SOLO>), grid, block, 0, st, a); break;
    default: return hipErrorInvalidValue;
    }
    return hipGetLastError();
}

// solo: the plan has short whole pairs behind the first item of a slot (the kernel gives those to single waves)
template <int D, bool DEEP, bool KV8>
hipError_t launch_mfma(int G, bool solo, const DecodeArgs &a, int n_slots, hipStream_t st)
{
    return solo ? launch_mfma_g<D, DEEP, KV8, true>(G, a, n_slots, st) : launch_mfma_g<D, DEEP, KV8, false>(G, a, n_slots, st);
}

bool aligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

}  // namespace

namespace {

size_t align256(size_t x) { return (x + 255) / 256 * 256; }

// Partial-result slots of a plan with n_parts items: one per item (a group partial of a pair cut very deeply
// takes the slot of the group's first piece).
size_t part_slots(int32_t n_parts) { return static_cast<size_t>(n_parts); }

}  // namespace

// Workspace layout: counters | part_ml [slots][G][2] f32 | part_o [slots][G][D] f32, each region
// starting on a 256-byte boundary, slots = part_slots(n_parts).  The counters come first so that their place
// does not depend on n_parts: calls with different plans may then share one workspace.  The counters are zero
// between calls.
// Counters of the hand-over: one per pair, then one per group of a pair cut into many pieces (indexed
// by the pair's first partial slot plus the group; a line cut has fewer partial slots than pairs plus
// slots, so n_pairs + FAIRKV_MAX_SLOTS counters serve every such plan).  Their number depends on the
// pairs alone, so that calls with different plans can share a workspace.
extern "C" size_t fairkv_workspace_counter_bytes(int32_t n_pairs)
{
    if (n_pairs < 1) return 0;
    return align256((2 * static_cast<size_t>(n_pairs) + FAIRKV_MAX_SLOTS) * sizeof(int32_t));
}

namespace {
__global__ __launch_bounds__(256) void fairkv_zero_words_kernel(uint32_t *p, size_t n_words)
{
    for (size_t i = static_cast<size_t>(blockIdx.x) * 256 + threadIdx.x; i < n_words; i += static_cast<size_t>(gridDim.x) * 256)
        p[i] = 0u;
}
}  // namespace

// A fill kernel, not a memset: a caller may record this call into a HIP graph, where memset nodes are best avoided.
extern "C" int fairkv_workspace_reset(void *workspace, size_t workspace_bytes, int32_t n_pairs, void *hip_stream)
{
    const size_t need = fairkv_workspace_counter_bytes(n_pairs);
    if (!workspace || need == 0 || (reinterpret_cast<uintptr_t>(workspace) & 15) != 0) return FAIRKV_EINVAL;
    if (workspace_bytes < need) return FAIRKV_EWORKSPACE;
    const size_t n_words = need / sizeof(uint32_t);
    const unsigned blocks = static_cast<unsigned>(std::min<size_t>((n_words + 255) / 256, 1024));
    hipLaunchKernelGGL(fairkv_zero_words_kernel, dim3(blocks), dim3(256), 0, static_cast<hipStream_t>(hip_stream),
                       static_cast<uint32_t *>(workspace), n_words);
    return hipGetLastError() == hipSuccess ? FAIRKV_OK : FAIRKV_EHIP;
}

extern "C" size_t fairkv_workspace_bytes(int32_t n_parts, int32_t n_pairs, int32_t G, int32_t D)
{
    if (n_parts < 0 || n_pairs < 1 || G < 1 || D < 1) return 0;
    return align256(part_slots(n_parts) * G * D * sizeof(float)) + align256(part_slots(n_parts) * G * 2 * sizeof(float)) +
           fairkv_workspace_counter_bytes(n_pairs);
}

namespace {

// Everything a decode call is given; the entry points differ in where the workspace comes from and in what they
// add (8-bit scales, a trace buffer).
struct DecodeCall {
    const void *q, *k, *v;
    int64_t n_rows;
    const fairkv_item *items, *items_host;
    int32_t n_items;
    const int32_t *slot_ptr;
    int32_t n_slots, n_parts;
    void *workspace;
    size_t workspace_bytes;
    void *out;
    float *lse;
    int32_t B, q_len, Hq, Hkv, D, in_dtype, out_dtype;
    float scale;
    bool kv8 = false;
    float k_scale = 1.f, v_scale = 1.f;
    const float *k_head = nullptr, *v_head = nullptr;
    unsigned long long *trace = nullptr;
    int32_t *count_scratch = nullptr;      // host, n_parts ints, for callers that must not allocate; else a vector is used
    bool static_workspace = false;         // the library's own array instead of `workspace`
    void *hip_stream;
};

int decode_common(const DecodeCall &c);

DecodeCall make_call(const void *q, const void *k, const void *v, int64_t n_rows, const fairkv_item *items,
                     const fairkv_item *items_host, int32_t n_items, const int32_t *slot_ptr, int32_t n_slots,
                     int32_t n_parts, void *workspace, size_t workspace_bytes, void *out, float *lse, int32_t B,
                     int32_t q_len, int32_t Hq, int32_t Hkv, int32_t D, int32_t in_dtype, int32_t out_dtype, float scale,
                     void *hip_stream)
{
    DecodeCall c{};
    c.q = q; c.k = k; c.v = v; c.n_rows = n_rows; c.items = items; c.items_host = items_host; c.n_items = n_items;
    c.slot_ptr = slot_ptr; c.n_slots = n_slots; c.n_parts = n_parts; c.workspace = workspace;
    c.workspace_bytes = workspace_bytes; c.out = out; c.lse = lse; c.B = B; c.q_len = q_len; c.Hq = Hq; c.Hkv = Hkv;
    c.D = D; c.in_dtype = in_dtype; c.out_dtype = out_dtype; c.scale = scale; c.hip_stream = hip_stream;
    return c;
}

bool finite(float x) { return x == x && !std::isinf(x); }

}  // namespace

extern "C" int fairkv_decode_attn(const void *q, const void *k, const void *v, int64_t n_rows, const fairkv_item *items,
                                  const fairkv_item *items_host, int32_t n_items, const int32_t *slot_ptr,
                                  int32_t n_slots,
                                  int32_t n_parts, void *workspace,
                                  size_t workspace_bytes, void *out, float *lse, int32_t B, int32_t Hq,
                                  int32_t Hkv, int32_t D, int32_t in_dtype, int32_t out_dtype, float scale,
                                  void *hip_stream)
{
    return decode_common(make_call(q, k, v, n_rows, items, items_host, n_items, slot_ptr, n_slots, n_parts, workspace,
                                   workspace_bytes, out, lse, B, 1, Hq, Hkv, D, in_dtype, out_dtype, scale, hip_stream));
}

extern "C" int fairkv_decode_attn_multi(const void *q, const void *k, const void *v, int64_t n_rows,
                                        const fairkv_item *items,
                                        const fairkv_item *items_host, int32_t n_items, const int32_t *slot_ptr,
                                        int32_t n_slots, int32_t n_parts, void *workspace, size_t workspace_bytes,
                                        void *out, float *lse, int32_t B, int32_t q_len, int32_t Hq, int32_t Hkv,
                                        int32_t D, int32_t in_dtype, int32_t out_dtype, float scale, void *hip_stream)
{
    return decode_common(make_call(q, k, v, n_rows, items, items_host, n_items, slot_ptr, n_slots, n_parts, workspace,
                                   workspace_bytes, out, lse, B, q_len, Hq, Hkv, D, in_dtype, out_dtype, scale, hip_stream));
}

extern "C" int fairkv_decode_attn_kv8(const void *q, const void *k8, const void *v8, int64_t n_rows, float k_scale,
                                      float v_scale, const fairkv_item *items, const fairkv_item *items_host,
                                      int32_t n_items, const int32_t *slot_ptr, int32_t n_slots, int32_t n_parts,
                                      void *workspace, size_t workspace_bytes, void *out, float *lse, int32_t B,
                                      int32_t q_len, int32_t Hq, int32_t Hkv, int32_t D, int32_t out_dtype, float scale,
                                      void *hip_stream)
{
    if (!finite(k_scale) || !finite(v_scale)) return FAIRKV_EINVAL;
    DecodeCall c = make_call(q, k8, v8, n_rows, items, items_host, n_items, slot_ptr, n_slots, n_parts, workspace,
                             workspace_bytes, out, lse, B, q_len, Hq, Hkv, D, FAIRKV_BF16, out_dtype, scale, hip_stream);
    c.kv8 = true;
    c.k_scale = k_scale;
    c.v_scale = v_scale;
    return decode_common(c);
}

extern "C" int fairkv_decode_attn_kv8_per_head(const void *q, const void *k8, const void *v8, int64_t n_rows,
                                               const float *k_scale, const float *v_scale, const fairkv_item *items,
                                               const fairkv_item *items_host, int32_t n_items, const int32_t *slot_ptr,
                                               int32_t n_slots, int32_t n_parts, void *workspace, size_t workspace_bytes,
                                               void *out, float *lse, int32_t B, int32_t q_len, int32_t Hq, int32_t Hkv,
                                               int32_t D, int32_t out_dtype, float scale, void *hip_stream)
{
    if (!k_scale || !v_scale || Hkv < 1) return FAIRKV_EINVAL;
    if (Hkv > kScaleHeads) return FAIRKV_EUNSUPPORTED;
    for (int32_t h = 0; h < Hkv; ++h)
        if (!finite(k_scale[h]) || !finite(v_scale[h])) return FAIRKV_EINVAL;
    DecodeCall c = make_call(q, k8, v8, n_rows, items, items_host, n_items, slot_ptr, n_slots, n_parts, workspace,
                             workspace_bytes, out, lse, B, q_len, Hq, Hkv, D, FAIRKV_BF16, out_dtype, scale, hip_stream);
    c.kv8 = true;
    c.k_head = k_scale;
    c.v_head = v_scale;
    return decode_common(c);
}

extern "C" int fairkv_decode_attn_trace(const void *q, const void *k, const void *v, int64_t n_rows,
                                        const fairkv_item *items, const fairkv_item *items_host, int32_t n_items,
                                        const int32_t *slot_ptr, int32_t n_slots, int32_t n_parts, void *workspace,
                                        size_t workspace_bytes, void *out, float *lse, int32_t B, int32_t Hq, int32_t Hkv,
                                        int32_t D, float scale, uint64_t *trace, size_t trace_bytes, void *hip_stream)
{
    if (!trace || n_slots < 1 || trace_bytes < static_cast<size_t>(n_slots) * kTraceStamps * sizeof(uint64_t)) return FAIRKV_EINVAL;
    if (D != 128 || Hkv < 1 || (Hq != 8 * Hkv && Hq != 4 * Hkv) || n_slots > FAIRKV_MAX_SLOTS) return FAIRKV_EUNSUPPORTED;
    DecodeCall c = make_call(q, k, v, n_rows, items, items_host, n_items, slot_ptr, n_slots, n_parts, workspace,
                             workspace_bytes, out, lse, B, 1, Hq, Hkv, D, FAIRKV_BF16, FAIRKV_F32, scale, hip_stream);
    c.trace = reinterpret_cast<unsigned long long *>(trace);
    return decode_common(c);
}

// ---- the entry point that allocates nothing ------------------------------------------------------
namespace {

// The workspace of fairkv_decode_attn_static: one array per GPU, part of the loaded code object and zero when
// that is loaded.  Only the arrival counters at its start need to be zero for a call, and every completed call
// leaves them zero, whatever its sizes (the counter region starts at offset 0 for every B * Hkv).
static __device__ __align__(256) unsigned char scratch[FAIRKV_STATIC_WORKSPACE_BYTES];

constexpr int kMaxDevices = 64;
constexpr int32_t kStaticMaxParts = FAIRKV_STATIC_WORKSPACE_BYTES / 256;   // a partial slot is at least 264 bytes

// Address of `scratch` on every device, looked up once per device with that device current.  In host code the
// array's name is only a handle for this lookup: the address it yields is what kernels and copies are given.
void *scratch_of_current_device()
{
    static std::atomic<void *> ptr[kMaxDevices];
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return nullptr;
    void *p = ptr[dev].load(std::memory_order_acquire);
    if (p) return p;
    if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) return nullptr;
    ptr[dev].store(p, std::memory_order_release);       // every thread that looks it up finds the same address
    return p;
}

}  // namespace

extern "C" int fairkv_decode_attn_static(const void *q, const void *k, const void *v, int64_t n_rows,
                                         const fairkv_item *items, const fairkv_item *items_host, int32_t n_items,
                                         const int32_t *slot_ptr, int32_t n_slots, int32_t n_parts, void *out, float *lse,
                                         int32_t B, int32_t q_len, int32_t Hq, int32_t Hkv, int32_t D, int32_t in_dtype,
                                         int32_t out_dtype, float scale, void *hip_stream)
{
    if (B < 1 || Hq < 1 || Hkv < 1 || D < 1 || q_len < 1 || n_parts < 0 || Hq % Hkv != 0) return FAIRKV_EINVAL;
    const int64_t cols = static_cast<int64_t>(Hq / Hkv) * q_len;
    if (static_cast<int64_t>(B) * Hkv > INT32_MAX || cols > 16 || D > 128) return FAIRKV_EUNSUPPORTED;
    if (n_parts > kStaticMaxParts ||
        fairkv_workspace_bytes(n_parts, B * Hkv, static_cast<int32_t>(cols), D) > FAIRKV_STATIC_WORKSPACE_BYTES)
        return FAIRKV_EWORKSPACE;       // this plan needs more than the built-in workspace holds
    static thread_local int32_t count_scratch[kStaticMaxParts];      // host side of the plan check, no heap
    DecodeCall c = make_call(q, k, v, n_rows, items, items_host, n_items, slot_ptr, n_slots, n_parts, nullptr,
                             FAIRKV_STATIC_WORKSPACE_BYTES, out, lse, B, q_len, Hq, Hkv, D, in_dtype, out_dtype, scale,
                             hip_stream);
    c.count_scratch = count_scratch;
    c.static_workspace = true;          // looked up after every check that needs no device has passed
    return decode_common(c);
}

namespace {
int decode_common(const DecodeCall &c)
{
    const int32_t B = c.B, Hq = c.Hq, Hkv = c.Hkv, D = c.D, q_len = c.q_len, n_items = c.n_items, n_slots = c.n_slots,
                  n_parts = c.n_parts;
    const fairkv_item *items_host = c.items_host;
    const int32_t *slot_ptr = c.slot_ptr;
    if (!c.q || !c.k || !c.v || !c.items || !items_host || !slot_ptr || !c.out) return FAIRKV_EINVAL;
    if (B < 1 || Hq < 1 || Hkv < 1 || D < 1 || n_items < 1 || n_slots < 1 || n_parts < 0 || q_len < 1 || c.n_rows < 0) return FAIRKV_EINVAL;
    if (Hq % Hkv != 0) return FAIRKV_EINVAL;
    if (n_parts < n_items) return FAIRKV_EINVAL;
    if (slot_ptr[0] != 0 || slot_ptr[n_slots] != n_items) return FAIRKV_EINVAL;
    for (int32_t j = 0; j < n_slots; ++j)
        if (slot_ptr[j] > slot_ptr[j + 1]) return FAIRKV_EINVAL;
    // Every cut pair must come with all its pieces, each exactly once: a piece that is missing would leave the
    // pair's arrival counter short for ever (no output, and a counter that is not zero for the next call); one
    // that comes twice would have two workgroups write one partial slot.  count[first slot of a pair] counts
    // that pair's pieces; a piece's own slot must be used once.
    std::vector<int32_t> count_own;
    int32_t *count = c.count_scratch;
    if (!count) {
        count_own.assign(static_cast<size_t>(n_parts), 0);
        count = count_own.data();
    } else {
        for (int32_t i = 0; i < n_parts; ++i) count[i] = 0;
    }
    bool deep = false;      // a pair in very many pieces: the kernel with the two-level merge
    bool solo = false;      // short whole pairs: the kernel that gives them to single waves
    for (int32_t i = 0; i < n_items; ++i) {
        const fairkv_item &it = items_host[i];
        deep |= it.n_chunks >= kDeepFrom;
        solo |= it.n_chunks == 1 && it.tok_count <= kSoloTokens;
        if (it.b < 0 || it.b >= B || it.h < 0 || it.h >= Hkv || it.row < 0 || it.tok_count < 0) return FAIRKV_EINVAL;
        if (it.row + it.tok_count > c.n_rows) return FAIRKV_EINVAL;      // the kernel reads exactly these rows of K and V
        if (it.n_chunks < 1 || it.chunk < 0 || it.chunk >= it.n_chunks) return FAIRKV_EINVAL;
        if (it.part < it.chunk || it.part - it.chunk + it.n_chunks > n_parts) return FAIRKV_EINVAL;
        // the rows new tokens hide from one another (the last q_len - 1 of a pair) must not reach
        // back beyond the pair's last chunk: the kernel masks inside that chunk only
        if (q_len > 1 && it.n_chunks > 1 && it.chunk == it.n_chunks - 1 && it.tok_count < q_len - 1) return FAIRKV_EINVAL;
        count[it.part - it.chunk] += 1 << 8;                 // pieces of the pair that starts at this slot
        count[it.part] += 1;                                 // uses of this slot
        if ((count[it.part] & 0xff) > 1 || (count[it.part - it.chunk] >> 8) > it.n_chunks) return FAIRKV_EINVAL;
    }
    for (int32_t i = 0; i < n_items; ++i) {
        const fairkv_item &it = items_host[i];
        if ((count[it.part - it.chunk] >> 8) != it.n_chunks) return FAIRKV_EINVAL;
    }
    if (!finite(c.scale)) return FAIRKV_EINVAL;
    const bool on_valu = c.in_dtype == FAIRKV_BF16_VALU;     // bf16 on the vector-ALU kernel: A/B measurements
    const int32_t in_dtype = on_valu ? FAIRKV_BF16 : c.in_dtype;
    if (in_dtype != FAIRKV_BF16 && in_dtype != FAIRKV_F32) return FAIRKV_EUNSUPPORTED;
    if (c.out_dtype != FAIRKV_BF16 && c.out_dtype != FAIRKV_F32) return FAIRKV_EUNSUPPORTED;
    const int G = Hq / Hkv;
    if (D != 64 && D != 128) return FAIRKV_EUNSUPPORTED;
    if (G != 1 && G != 2 && G != 4 && G != 8) return FAIRKV_EUNSUPPORTED;
    // columns of a pair: G heads times q_len new tokens; they share the 16 columns of one MFMA tile
    const int64_t cols = static_cast<int64_t>(G) * q_len;
    if (cols != 1 && cols != 2 && cols != 4 && cols != 8 && cols != 16) return FAIRKV_EUNSUPPORTED;
    if (q_len > 1 && (in_dtype != FAIRKV_BF16 || on_valu)) return FAIRKV_EUNSUPPORTED;
    if ((c.kv8 || c.trace) && on_valu) return FAIRKV_EUNSUPPORTED;
    if (!aligned16(c.k) || !aligned16(c.v) || !aligned16(c.q) || !aligned16(c.items) || !aligned16(c.out)) return FAIRKV_EINVAL;
    if (static_cast<int64_t>(B) * q_len * Hq * D > INT32_MAX) return FAIRKV_EINVAL;
    const size_t need = fairkv_workspace_bytes(n_parts, B * Hkv, static_cast<int32_t>(cols), D);
    if (c.workspace_bytes < need || (!c.static_workspace && !c.workspace)) return FAIRKV_EWORKSPACE;
    if (!c.static_workspace && !aligned16(c.workspace)) return FAIRKV_EINVAL;

    hipStream_t st = static_cast<hipStream_t>(c.hip_stream);
    char *ws = static_cast<char *>(c.static_workspace ? scratch_of_current_device() : c.workspace);
    if (!ws) return FAIRKV_EHIP;
    DecodeArgs a;
    a.q = c.q;
    a.k = c.k;
    a.v = c.v;
    a.items = c.items;
    // One workgroup per slot while the slot pointer fits the kernel arguments; beyond that, consecutive slots
    // share a workgroup (their items are consecutive in the list, and a workgroup walks a list of any length).
    const int32_t n_wg = n_slots < FAIRKV_MAX_SLOTS ? n_slots : FAIRKV_MAX_SLOTS;
    for (int32_t j = 0; j <= n_wg; ++j) a.slot_ptr[j] = slot_ptr[static_cast<int64_t>(j) * n_slots / n_wg];
    for (int32_t j = 0; j < n_wg; ++j) {
        a.first_row[j] = 0;
        a.first_np[j] = 0;
        if (a.slot_ptr[j] == a.slot_ptr[j + 1]) continue;
        const fairkv_item &it = items_host[a.slot_ptr[j]];
        const int64_t pair = static_cast<int64_t>(it.b) * Hkv + it.h;
        if (it.row > static_cast<int64_t>(UINT32_MAX) || pair >= (1 << 23)) continue;   // does not fit: normal start
        a.first_row[j] = static_cast<uint32_t>(it.row);
        a.first_np[j] = (static_cast<uint32_t>(pair) << 9) | static_cast<uint32_t>(it.tok_count < kEarlyTok ? it.tok_count : kEarlyTok);
    }
    a.arrivals = reinterpret_cast<int32_t *>(ws);
    a.group_arrivals = a.arrivals + static_cast<size_t>(B) * Hkv;
    a.n_group_counters = B * Hkv + FAIRKV_MAX_SLOTS;
    ws += fairkv_workspace_counter_bytes(B * Hkv);
    a.part_ml = reinterpret_cast<float *>(ws);
    ws += align256(part_slots(n_parts) * cols * 2 * sizeof(float));
    a.part_o = reinterpret_cast<float *>(ws);
    a.out = c.out;
    a.lse = c.lse;
    a.B = B;
    a.Hq = Hq;
    a.Hkv = Hkv;
    a.out_dtype = c.out_dtype;
    a.n_parts = n_parts;
    a.n_rows = c.n_rows;
    a.q_len = q_len;
    a.g_shift = G == 1 ? 0 : G == 2 ? 1 : G == 4 ? 2 : 3;
    a.scale_log2 = c.scale * kLog2e * c.k_scale;
    a.v_scale = c.v_scale;
    for (int h = 0; h < kScaleHeads; ++h) {     // a scale per KV head (at most kScaleHeads of them), else all 1
        a.k_head[h] = c.k_head ? c.k_head[h % Hkv] : 1.f;
        a.v_head[h] = c.v_head ? c.v_head[h % Hkv] : 1.f;
    }
    a.trace = c.trace;

    const bool kv8 = c.kv8;
    hipError_t e;
    if (c.trace)
        e = launch_mfma_trace(static_cast<int>(cols), deep, a, n_wg, st);
    else if (in_dtype == FAIRKV_BF16 && !on_valu)
        e = kv8 ? (D == 128 ? (deep ? launch_mfma<128, true, true>(static_cast<int>(cols), solo, a, n_wg, st)
                                    : launch_mfma<128, false, true>(static_cast<int>(cols), solo, a, n_wg, st))
                            : (deep ? launch_mfma<64, true, true>(static_cast<int>(cols), solo, a, n_wg, st)
                                    : launch_mfma<64, false, true>(static_cast<int>(cols), solo, a, n_wg, st)))
            : D == 128 ? (deep ? launch_mfma<128, true, false>(static_cast<int>(cols), solo, a, n_wg, st)
                               : launch_mfma<128, false, false>(static_cast<int>(cols), solo, a, n_wg, st))
                       : (deep ? launch_mfma<64, true, false>(static_cast<int>(cols), solo, a, n_wg, st)
                               : launch_mfma<64, false, false>(static_cast<int>(cols), solo, a, n_wg, st));
    else if (in_dtype == FAIRKV_BF16)
        e = D == 128 ? launch_valu<FAIRKV_BF16, 128>(G, a, n_wg, st) : launch_valu<FAIRKV_BF16, 64>(G, a, n_wg, st);
    else
        e = D == 128 ? launch_valu<FAIRKV_F32, 128>(G, a, n_wg, st) : launch_valu<FAIRKV_F32, 64>(G, a, n_wg, st);
    return e == hipSuccess ? FAIRKV_OK : FAIRKV_EHIP;
}
}  // namespace

// ---- packing and appending ------------------------------------------------------------------------
namespace {
int row_bytes_of(int32_t D, int32_t dtype)
{
    if (dtype != FAIRKV_BF16 && dtype != FAIRKV_F32 && dtype != FAIRKV_E4M3) return 0;
    const int64_t rb = static_cast<int64_t>(D) * (dtype == FAIRKV_E4M3 ? 1 : dtype == FAIRKV_BF16 ? 2 : 4);
    return (rb == 128 || rb == 256 || rb == 512) ? static_cast<int>(rb) : 0;
}
}  // namespace

extern "C" int fairkv_pack(const void *k_dense, const void *v_dense, int32_t B, int32_t Hkv, int32_t T, int32_t D,
                           int32_t dtype, const int64_t *keep_ptr, const int32_t *keep_t, const int64_t *off,
                           const fairkv_item *items, const int32_t *slot_ptr, int32_t n_slots, void *k_out,
                           void *v_out, int64_t n_rows, int32_t *bad, void *hip_stream)
{
    if (!k_dense || !v_dense || !keep_ptr || !keep_t || !off || !items || !slot_ptr || !k_out || !v_out) return FAIRKV_EINVAL;
    if (B < 1 || Hkv < 1 || T < 1 || D < 1 || n_slots < 1 || n_rows < 0) return FAIRKV_EINVAL;
    if (!aligned16(k_dense) || !aligned16(v_dense) || !aligned16(k_out) || !aligned16(v_out)) return FAIRKV_EINVAL;
    const int rb = row_bytes_of(D, dtype);
    if (rb == 0) return FAIRKV_EUNSUPPORTED;
    PackArgs a{static_cast<const char *>(k_dense), static_cast<const char *>(v_dense), static_cast<char *>(k_out),
               static_cast<char *>(v_out), keep_ptr, keep_t, off, items, slot_ptr, bad, n_rows, B, Hkv, T};
    hipStream_t st = static_cast<hipStream_t>(hip_stream);
    if (rb == 128)
        hipLaunchKernelGGL(fairkv_pack_kernel<128>, dim3(n_slots), dim3(256), 0, st, a);
    else if (rb == 256)
        hipLaunchKernelGGL(fairkv_pack_kernel<256>, dim3(n_slots), dim3(256), 0, st, a);
    else
        hipLaunchKernelGGL(fairkv_pack_kernel<512>, dim3(n_slots), dim3(256), 0, st, a);
    return hipGetLastError() == hipSuccess ? FAIRKV_OK : FAIRKV_EHIP;
}

extern "C" int fairkv_append(const void *k_new, const void *v_new, int32_t B, int32_t Hkv, int32_t D, int32_t dtype,
                             const int64_t *off, int32_t *len, const int32_t *cap, void *k, void *v, int64_t n_rows,
                             int32_t *full, void *hip_stream)
{
    if (!k_new || !v_new || !off || !len || !cap || !k || !v) return FAIRKV_EINVAL;
    if (B < 1 || Hkv < 1 || D < 1 || n_rows < 0) return FAIRKV_EINVAL;
    if (!aligned16(k_new) || !aligned16(v_new) || !aligned16(k) || !aligned16(v)) return FAIRKV_EINVAL;
    const int rb = row_bytes_of(D, dtype);
    if (rb == 0) return FAIRKV_EUNSUPPORTED;
    const int64_t n_pairs = static_cast<int64_t>(B) * Hkv;
    if (n_pairs > INT32_MAX) return FAIRKV_EINVAL;
    AppendArgs a{static_cast<const char *>(k_new), static_cast<const char *>(v_new), static_cast<char *>(k),
                 static_cast<char *>(v), off, len, cap, full, n_rows, static_cast<int32_t>(n_pairs)};
    const int64_t threads = n_pairs * (rb / 16);
    const dim3 grid(static_cast<unsigned>((threads + 255) / 256));
    hipStream_t st = static_cast<hipStream_t>(hip_stream);
    if (rb == 128)
        hipLaunchKernelGGL(fairkv_append_kernel<128>, grid, dim3(256), 0, st, a);
    else if (rb == 256)
        hipLaunchKernelGGL(fairkv_append_kernel<256>, grid, dim3(256), 0, st, a);
    else
        hipLaunchKernelGGL(fairkv_append_kernel<512>, grid, dim3(256), 0, st, a);
    return hipGetLastError() == hipSuccess ? FAIRKV_OK : FAIRKV_EHIP;
}

// ---- measurement aid ------------------------------------------------------------------------------
namespace {

template <int WAVES, int STAGES, int LPT>
int launch_probe(const ProbeArgs &a, int n_workgroups, hipStream_t st)
{
    constexpr size_t lds = static_cast<size_t>(WAVES) * STAGES * 2 * LPT * 1024;
    if constexpr (lds > 160 * 1024 || 3 * (2 * LPT + 1) >= 64) {
        return FAIRKV_EUNSUPPORTED;
    } else {
        static const hipError_t attr = hipFuncSetAttribute(reinterpret_cast<const void *>(&fairkv_stream_probe_kernel<WAVES, STAGES, LPT>),
                                                           hipFuncAttributeMaxDynamicSharedMemorySize, static_cast<int>(lds));
        if (attr != hipSuccess) return FAIRKV_EHIP;
        hipLaunchKernelGGL((fairkv_stream_probe_kernel<WAVES, STAGES, LPT>), dim3(n_workgroups), dim3(WAVES * 64), lds, st, a);
        return hipGetLastError() == hipSuccess ? FAIRKV_OK : FAIRKV_EHIP;
    }
}

template <int WAVES, int STAGES>
int launch_probe_t(int tile_kib, const ProbeArgs &a, int n, hipStream_t st)
{
    switch (tile_kib) {
    case 2: return launch_probe<WAVES, STAGES, 2>(a, n, st);
    case 4: return launch_probe<WAVES, STAGES, 4>(a, n, st);
    case 8: return launch_probe<WAVES, STAGES, 8>(a, n, st);
    default: return FAIRKV_EUNSUPPORTED;
    }
}

template <int WAVES>
int launch_probe_s(int stages, int tile_kib, const ProbeArgs &a, int n, hipStream_t st)
{
    switch (stages) {
    case 2: return launch_probe_t<WAVES, 2>(tile_kib, a, n, st);
    case 3: return launch_probe_t<WAVES, 3>(tile_kib, a, n, st);
    case 4: return launch_probe_t<WAVES, 4>(tile_kib, a, n, st);
    default: return FAIRKV_EUNSUPPORTED;
    }
}

}  // namespace

extern "C" int fairkv_stream_probe_shape(const void *k, const void *v, int64_t bytes_each, int32_t n_workgroups,
                                         int32_t waves, int32_t stages, int32_t tile_kib, void *sink, void *hip_stream)
{
    if (!k || !v || !sink || n_workgroups < 1 || bytes_each < 0 || !aligned16(k) || !aligned16(v)) return FAIRKV_EINVAL;
    if (tile_kib < 1 || tile_kib > 8) return FAIRKV_EUNSUPPORTED;
    ProbeArgs a{static_cast<const char *>(k), static_cast<const char *>(v),
                bytes_each / n_workgroups / (tile_kib * 1024) * (tile_kib * 1024), static_cast<uint32_t *>(sink)};
    if (a.bytes_per_workgroup * 16 > static_cast<int64_t>(UINT32_MAX)) return FAIRKV_EINVAL;   // 32-bit lane offsets
    hipStream_t st = static_cast<hipStream_t>(hip_stream);
    switch (waves) {
    case 4: return launch_probe_s<4>(stages, tile_kib, a, n_workgroups, st);
    case 8: return launch_probe_s<8>(stages, tile_kib, a, n_workgroups, st);
    case 16: return launch_probe_s<16>(stages, tile_kib, a, n_workgroups, st);
    default: return FAIRKV_EUNSUPPORTED;
    }
}

extern "C" int fairkv_stream_probe(const void *k, const void *v, int64_t bytes_each, int32_t n_workgroups,
                                   void *sink, void *hip_stream)
{
    return fairkv_stream_probe_shape(k, v, bytes_each, n_workgroups, kWaves, ring_stages(8), 4, sink, hip_stream);
}

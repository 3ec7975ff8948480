/*
 * fairkv.h - C ABI of the MI355X (gfx950) library for single-token grouped-query
 * decode attention over a KV cache compressed per head.
 *
 * Setting (paper: Introduction, "unfair head load"; Section 3.2; Section 4.2
 * Fair-Copying; Appendix A).  Per-head KV-cache compression leaves every
 * (sequence b, KV head h) pair with its own number len[b][h] of retained
 * tokens.  Decode attention is bandwidth bound and its cost is linear in the
 * retained tokens (Section 3.2), so unequal heads mean unequal work.  The
 * paper equalises per-GPU load by placing heads with care and by replicating
 * heavy heads so that each replica carries W/copies of the load (Algorithm 2;
 * objective eq. 4, cap on copies eq. 3, coverage eq. 2, efficiency eq. 5).
 * This library applies the same rule inside one GPU: the "devices" are
 * workgroup slots on compute units, a heavy pair is cut into equal token
 * chunks, and the chunks are scheduled longest first.
 *
 * Conventions for every entry point
 *   - returns FAIRKV_OK (0) or a negative fairkv_status; never throws, aborts or prints;
 *   - "host" pointers are ordinary process memory, "device" pointers are HIP device
 *     memory of the current device; the library never allocates or frees device memory
 *     and keeps no state between calls; all buffers are owned by the caller;
 *   - on error nothing is launched and no output buffer is written.
 *
 * Packed ragged KV layout.  K and V are two row-major buffers [n_rows][D] of the
 * same element type; the tokens of pair (b, h) are rows off[b][h] ... off[b][h] +
 * len[b][h] - 1 of both.  off is in rows (int64), len in tokens (int32), both
 * [B][Hkv] row-major.  Ranges of different pairs must not overlap; gaps are allowed.
 * A row is D * sizeof(element) bytes and the K and V base addresses must be 16-byte
 * aligned.  Query heads [h*G, (h+1)*G), G = Hq / Hkv, attend over KV head h.
 */
#ifndef FAIRKV_H
#define FAIRKV_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    FAIRKV_OK = 0,
    FAIRKV_EINVAL = -1,       /* null pointer, non-positive size, bad parameter combination */
    FAIRKV_ECAP = -2,         /* caller's items array is too small; summary.n_items says how big */
    FAIRKV_EWORKSPACE = -3,   /* workspace smaller than fairkv_workspace_bytes() */
    FAIRKV_EUNSUPPORTED = -4, /* element type / head_dim / group size without a kernel */
    FAIRKV_EHIP = -5          /* a HIP call failed; the HIP error is left for hipGetLastError */
} fairkv_status;

enum { FAIRKV_BF16 = 0, FAIRKV_F32 = 1 };

/* How the work list is built.
 *   NAIVE      one item per pair, dealt round-robin in (b, h) order: the analogue of the
 *              paper's static head allocation baseline (Figure 3 (1), Section 5.1 Baseline).
 *   LPT        load-aware order, no splitting: Best-effort Assignment only (Section 1.2).
 *   LPT_SPLIT  heavy pairs cut into equal chunks first: with Fair-Copying (Section 4.2). */
enum { FAIRKV_POLICY_NAIVE = 0, FAIRKV_POLICY_LPT = 1, FAIRKV_POLICY_LPT_SPLIT = 2 };

/* One unit of work: tokens [tok_begin, tok_begin + tok_count) of pair (b, h), for all G
 * query heads of the group.  chunk / n_chunks number the pieces of the pair; part is the
 * index of this item's partial result in the workspace; slot is the planner's predicted
 * placement (used for the summary; the kernels take items in list order). */
typedef struct {
    int32_t b, h, tok_begin, tok_count, chunk, n_chunks, slot, part;
} fairkv_item;

typedef struct {
    int32_t n_slots;         /* workgroup slots to balance over (compute units x resident groups) */
    int32_t tile;            /* chunk sizes are multiples of this many tokens (>= 1) */
    int32_t min_chunk;       /* no chunk target below this; positive multiple of tile */
    int32_t max_split;       /* most chunks one pair may be cut into: eq. 3's cap (>= 1) */
    int32_t oversub;         /* aim for about n_slots * oversub chunks in total (>= 1) */
    int32_t overhead_tokens; /* fixed cost of an item in token units: the offset of the
                                linear latency model of Section 3.2 (>= 0) */
    int32_t policy;          /* FAIRKV_POLICY_* */
    int32_t reserved;        /* must be 0 */
} fairkv_plan_params;

typedef struct {
    int64_t total_tokens;    /* sum of len */
    int64_t max_slot_load;   /* largest and smallest predicted slot load, in token units, */
    int64_t min_slot_load;   /*   over ALL n_slots (an idle slot counts 0): eq. 4 / Algorithm 2 */
    int32_t n_items;         /* items the plan has (also when it did not fit items_cap) */
    int32_t n_parts;         /* partial-result slots the workspace must hold */
} fairkv_plan_summary;

/* Defaults: n_slots = 2 * n_compute_units, tile 64, min_chunk 256, max_split 128,
 * oversub 2, overhead_tokens 64, policy LPT_SPLIT.  n_compute_units must be >= 1. */
int fairkv_default_params(fairkv_plan_params *p /*host, out*/, int32_t n_compute_units);

/*
 * Host-side planner (integer arithmetic only; deterministic).
 *
 *   target  = max(min_chunk, roundup_tile(ceil(sum len / (n_slots * oversub))))   [LPT_SPLIT]
 *   per pair with len > 0:  r = min(max_split, ceil(len / target)),  cs = roundup_tile(ceil(len / r)),
 *                           chunks of cs tokens, the last one shorter            (W / copies, Algorithm 2)
 *   order   = tok_count descending, then b, h, chunk ascending; each item goes to the slot
 *             with the smallest load so far (lowest index on ties); an item costs
 *             tok_count + overhead_tokens                                         (objective eq. 4)
 *   NAIVE and LPT never split; NAIVE keeps (b, h) order and deals slots round-robin.
 *
 * len        host [B*Hkv], every entry >= 0; pairs with len == 0 get no item.
 * items      host [items_cap], out, in execution order; may be NULL iff items_cap == 0.
 * slot_ptr   host [n_slots+1] or NULL, out: CSR pointer over items grouped by slot.
 * part_base  host [B*Hkv+1] or NULL, out: chunks before each pair; pair p owns partial slots
 *            part_base[p] ... part_base[p+1]-1, in chunk order.
 * summary    host, out, required; filled whenever the arguments are valid.
 *
 * Returns FAIRKV_ECAP (after filling summary, slot_ptr and part_base, writing no item)
 * when the plan has more items than items_cap: call once with items_cap = 0 to size.
 */
int fairkv_plan(const int32_t *len, int32_t B, int32_t Hkv, const fairkv_plan_params *p,
                fairkv_item *items, int32_t items_cap, int32_t *slot_ptr, int32_t *part_base,
                fairkv_plan_summary *summary);

/* Bytes of device workspace fairkv_decode_attn needs for n_parts partial results
 * (fp32 unnormalised outputs and softmax statistics per query head).  0 on bad arguments. */
size_t fairkv_workspace_bytes(int32_t n_parts, int32_t G, int32_t D);

/*
 * Decode attention for one layer: for every sequence b and query head hq (KV head
 * h = hq / G), out[b][hq] = softmax(scale * q[b][hq] . K_rows^T) V_rows over the
 * len[b][h] retained rows of pair (b, h), and lse[b][hq] = log sum exp of the scaled
 * scores.  Pairs with len == 0 give out = 0 and lse = -inf.  Accumulation is fp32.
 *
 * Enqueues a split-KV kernel over the work list (one workgroup per item; K/V rows are
 * read once and shared by the G query heads of the group) and a log-sum-exp merge of
 * the chunks of each pair on hip_stream, and returns without synchronising.
 *
 * q          device [B][Hq][D], element type in_dtype
 * k, v       device [n_rows][D], element type in_dtype, 16-byte aligned
 * off, len   device [B*Hkv] (int64 rows / int32 tokens), the layout above
 * items      device [n_items] and part_base device [B*Hkv+1]: a plan made by fairkv_plan
 *            from the same len (copied to the device by the caller).  Every item must
 *            satisfy tok_begin + tok_count <= len[b][h]; tokens past len are not read.
 * workspace  device, at least fairkv_workspace_bytes(n_parts, G, D) bytes, 16-byte aligned;
 *            n_parts = the plan's summary.n_parts
 * out        device [B][Hq][D], element type out_dtype (FAIRKV_F32, or FAIRKV_BF16 rounded
 *            to nearest even)
 * lse        device [B][Hq] float, or NULL
 * scale      multiplies the scores (1/sqrt(D) in the usual models)
 * hip_stream a hipStream_t (NULL = the default stream)
 *
 * Supported: D in {64, 128}; in_dtype BF16 or F32; G = Hq/Hkv in {1, 2, 4, 8}.
 * n_items == 0 is valid (every pair empty).  Calls that share a workspace must be
 * ordered on one stream.
 */
int fairkv_decode_attn(const void *q, const void *k, const void *v,
                       const int64_t *off, const int32_t *len,
                       const fairkv_item *items, int32_t n_items, const int32_t *part_base,
                       int32_t n_parts, void *workspace, size_t workspace_bytes,
                       void *out, float *lse,
                       int32_t B, int32_t Hq, int32_t Hkv, int32_t D,
                       int32_t in_dtype, int32_t out_dtype, float scale, void *hip_stream);

const char *fairkv_strerror(int code);
int fairkv_version(void);

#ifdef __cplusplus
}
#endif
#endif /* FAIRKV_H */

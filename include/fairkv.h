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
 * persistent workgroups, one per compute unit, and a heavy pair is shared by
 * several of them, each taking a token chunk.
 *
 * Conventions for every entry point
 *   - returns FAIRKV_OK (0) or a negative fairkv_status; never throws, aborts or prints;
 *   - "host" pointers are ordinary process memory, "device" pointers are HIP device
 *     memory of the current device; the library never allocates or frees device memory
 *     and keeps no state between calls (the only state, the arrival counters, lives in
 *     the caller's workspace); all buffers are owned by the caller;
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
    FAIRKV_ECAP = -2,         /* caller's output array is too small; the summary says how big */
    FAIRKV_EWORKSPACE = -3,   /* workspace smaller than fairkv_workspace_bytes() */
    FAIRKV_EUNSUPPORTED = -4, /* element type / head_dim / group size without a kernel */
    FAIRKV_EHIP = -5          /* a HIP call failed; the HIP error is left for hipGetLastError */
} fairkv_status;

enum { FAIRKV_BF16 = 0, FAIRKV_F32 = 1,
       FAIRKV_E4M3 = 2, /* one byte per element: fairkv_pack and fairkv_append only (they move bytes) */
       FAIRKV_BF16_VALU = 3 /* in_dtype of fairkv_decode_attn only: bf16 inputs through the vector-ALU kernel that
                               serves fp32 instead of the matrix-core kernel; for A/B measurements of the two */ };
enum { FAIRKV_SHORT_PAIR_TOKENS = 96 }; /* a whole pair of at most this many tokens is a "short pair": the bf16 and 8-bit
                                           kernels let one wave run it alone (four such pairs stream side by side,
                                           no fold across waves), and the planner may charge it its own overhead */
enum { FAIRKV_MAX_SLOTS = 320 };   /* most workgroups fairkv_decode_attn launches; a plan with more slots is run with
                                      consecutive slots sharing a workgroup */

/* How the work list is built; the four mirror the paper's ablation (Section 5.2.1).
 *   NAIVE      pairs dealt to slots round-robin in (b, h) order, unsplit: the analogue of the
 *              paper's static head allocation baseline (Figure 3 (1), Section 5.1 Baseline).
 *   LPT        load-aware placement of whole pairs, longest first onto the least loaded slot:
 *              Best-effort Assignment only (Section 1.2, Technique I).
 *   LPT_SPLIT  Fair-Copying as the paper states it (Section 4.2, Algorithm 2): a heavy pair
 *              becomes r equal chunks, each carrying len/r (the W/copies rule), then LPT.
 *   FAIR       Fair-Copying taken to its limit on one GPU, where a replica may take any share:
 *              all pairs are laid end to end and the line is cut into n_slots pieces of equal
 *              cost, so a pair is shared only by the slots whose boundary falls inside it.
 *              Reaches the lower bound of eq. 4 up to min_chunk and the per-item overhead. */
enum { FAIRKV_POLICY_NAIVE = 0, FAIRKV_POLICY_LPT = 1, FAIRKV_POLICY_LPT_SPLIT = 2, FAIRKV_POLICY_FAIR = 3 };

/* One unit of work: rows row ... row + tok_count - 1 of K and V, a chunk of pair (b, h),
 * for all G query heads of the group.  The pair was cut into n_chunks items, of which this
 * is number `chunk` (in token order: the first token of the chunk is row - off[b][h]);
 * part is the index of this item's partial result, and the partials of a pair are
 * consecutive: part - chunk ... part - chunk + n_chunks - 1.  A pair without tokens has
 * one item with tok_count == 0, so that some slot writes its zero output. */
typedef struct {
    int64_t row;
    int32_t tok_count;
    int32_t b, h;
    int32_t chunk;
    int32_t n_chunks;
    int32_t part;
} fairkv_item;          /* 32 bytes */

typedef struct {
    int32_t n_slots;         /* persistent workgroup slots to balance over (one per compute unit) */
    int32_t tile;            /* cuts inside a pair fall on multiples of this many tokens (>= 1) */
    int32_t min_chunk;       /* no piece of a cut pair is smaller; positive multiple of tile */
    int32_t max_split;       /* most items one pair may be cut into: eq. 3's cap (>= 1) */
    int32_t oversub;         /* LPT_SPLIT aims for about n_slots * oversub chunks in total (>= 1) */
    int32_t overhead_tokens; /* fixed cost of an item in token units: the offset of the
                                linear latency model of Section 3.2 (>= 0) */
    int32_t policy;          /* FAIRKV_POLICY_* */
    int32_t short_overhead_tokens; /* the same for an item that is a short pair (a whole pair of at most
                                FAIRKV_SHORT_PAIR_TOKENS tokens, empty pairs included); 0: overhead_tokens (>= 0) */
} fairkv_plan_params;

typedef struct {
    int64_t total_tokens;    /* sum of len */
    int64_t max_slot_load;   /* largest and smallest predicted slot load, in token units, */
    int64_t min_slot_load;   /*   over ALL n_slots (an idle slot counts 0): eq. 4 / Algorithm 2 */
    int32_t n_items;         /* items the plan has (also when it did not fit items_cap) */
    int32_t n_parts;         /* partial-result slots the workspace must hold (== n_items) */
} fairkv_plan_summary;

/* Defaults: n_slots = n_compute_units, tile 16, min_chunk 32, max_split 256, oversub 2,
 * overhead_tokens 160 (measured on MI355X: an extra item in a slot costs about as much as
 * streaming 120-160 tokens, and the time per launch is flat from 128 to 192), short_overhead_tokens 48
 * (a short pair costs a slot about a third of that), policy FAIR.  n_compute_units must be >= 1. */
int fairkv_default_params(fairkv_plan_params *p /*host, out*/, int32_t n_compute_units);

/*
 * Host-side planner (integer arithmetic only; deterministic).  An item costs
 * tok_count + ov, ov = short_overhead_tokens for a short pair (if that is not 0) and overhead_tokens
 * otherwise; the load of a slot is the sum over its items (objective: eq. 4).
 *
 * FAIR       pairs in (b, h) order fill slot 0, 1, ...  A slot opened as number j gets the budget
 *            ceil((tokens not yet placed + the ov of every pair not yet finished, taken whole +
 *            overhead_tokens * slots unopened) / slots unopened).  With fit = the whole tiles that still fit the slot's room: a pair
 *            (or its rest) that fits is placed whole; else it is cut at `fit` if both pieces are
 *            >= min_chunk; else it is placed whole anyway if the excess is <= fit; else the slot
 *            is closed and the next one opened.  After a cut the rest goes on in the next slot.
 *            The last slot, and the max_split-th piece of a pair, take all that is left.
 * LPT_SPLIT  target = max(min_chunk, roundup_tile(ceil(sum len / (n_slots * oversub)))); a pair is
 *            cut into r = min(max_split, ceil(len / target)) shares of roundup_tile(ceil(len / r))
 *            tokens, the last one shorter (W / copies, Algorithm 2); shares are sorted by
 *            tok_count descending, then pair and chunk ascending, and each goes to the slot with
 *            the smallest load so far (lowest index on ties).
 * LPT        the same with whole pairs.  NAIVE: whole pairs, pair i to slot i mod n_slots.
 *
 * len, off   host [B*Hkv]: tokens and first row of every pair; len >= 0, off >= 0 where len > 0.
 * items      host [items_cap], out, grouped by slot, inside a slot in the order the slot runs
 *            them; may be NULL iff items_cap == 0.
 * slot_ptr   host [n_slots+1] or NULL, out: slot j runs items[slot_ptr[j] .. slot_ptr[j+1]).
 * part_base  host [B*Hkv+1] or NULL, out: items before each pair; pair p owns partial slots
 *            part_base[p] ... part_base[p+1]-1, in chunk order.
 * summary    host, out, required; filled whenever the arguments are valid.
 *
 * Returns FAIRKV_ECAP (after filling summary, slot_ptr and part_base, writing no item)
 * when the plan has more items than items_cap: call once with items_cap = 0 to size.
 */
int fairkv_plan(const int32_t *len, const int64_t *off, int32_t B, int32_t Hkv, const fairkv_plan_params *p,
                fairkv_item *items, int32_t items_cap, int32_t *slot_ptr, int32_t *part_base,
                fairkv_plan_summary *summary);

/* Bytes of device workspace fairkv_decode_attn needs: fp32 partial outputs and softmax
 * statistics for n_parts items, plus the arrival counters of the hand-over.  0 on bad arguments.
 * Layout: the counters first (fairkv_workspace_counter_bytes(n_pairs) bytes: one per pair and
 * one per group of 8 pieces of a pair cut 32 ways or more; their number depends on n_pairs alone),
 * then statistics and partial outputs.  The counter bytes must be zero before the first use;
 * every completed call leaves them zero again, whatever its plan, so calls that are ordered on
 * one stream may share one workspace (the counter region of a smaller B * Hkv is a prefix of a
 * larger one's).  After a launch that did not complete (an aborted process, a device reset) zero
 * the counter bytes again: nothing else in the workspace carries state from call to call. */
size_t fairkv_workspace_counter_bytes(int32_t n_pairs);
size_t fairkv_workspace_bytes(int32_t n_parts, int32_t n_pairs, int32_t G, int32_t D);

/* Sets the counter bytes of a device workspace (the first fairkv_workspace_counter_bytes(n_pairs) bytes) to zero
 * with a small kernel on hip_stream, without synchronising: for a fresh workspace, and for one that a launch which
 * did not complete may have left with non-zero counters.  workspace: device, 16-byte aligned, at least that many
 * bytes (FAIRKV_EWORKSPACE otherwise).  Order it on the stream before the next decode call. */
int fairkv_workspace_reset(void *workspace, size_t workspace_bytes, int32_t n_pairs, void *hip_stream);

/*
 * Decode attention for one layer: for every sequence b and query head hq (KV head
 * h = hq / G), out[b][hq] = softmax(scale * q[b][hq] . K_rows^T) V_rows over the
 * len[b][h] retained rows of pair (b, h), and lse[b][hq] = log sum exp of the scaled
 * scores.  Pairs with len == 0 give out = 0 and lse = -inf.  Accumulation is fp32.
 *
 * Enqueues ONE kernel on hip_stream and returns without synchronising: n_slots persistent
 * workgroups, workgroup j streaming the K/V rows of its items from HBM exactly once (shared
 * by the G query heads of the group).  An item that is a whole pair writes out directly; the
 * items of a cut pair leave partial results in the workspace and the one that finishes last
 * combines them (log-sum-exp merge), so no second launch is needed.
 *
 * q          device [B][Hq][D], element type in_dtype, 16-byte aligned
 * k, v       device [n_rows][D], element type in_dtype, 16-byte aligned; every item must lie inside:
 *            row + tok_count <= n_rows (else FAIRKV_EINVAL)
 * items      device [n_items]: the items of a plan made by fairkv_plan from this cache's len
 *            and off, copied to the device by the caller.  The kernels read exactly the rows
 *            the items name.
 * items_host HOST [n_items]: the same array as the planner wrote it, and
 * slot_ptr   HOST [n_slots+1]: the plan's slot pointer.  The slot pointer and the first item
 *            of every slot travel to the GPU inside the kernel arguments, so that a workgroup
 *            requests its first K/V rows without first fetching its item list (two memory
 *            round trips less at the start of a 20 us kernel); with more than
 *            FAIRKV_MAX_SLOTS slots, consecutive slots share a workgroup.  items_host is also
 *            checked: every item must name a pair of this problem, rows >= 0 and a partial slot
 *            below n_parts, and a cut pair must come with every one of its n_chunks pieces, each
 *            once, in consecutive partial slots (else FAIRKV_EINVAL).
 * workspace  device, at least fairkv_workspace_bytes(n_parts, B*Hkv, G, D) bytes, 16-byte
 *            aligned, its counter bytes zero before the first use (see fairkv_workspace_bytes)
 * out        device [B][Hq][D], element type out_dtype (FAIRKV_F32, or FAIRKV_BF16 rounded
 *            to nearest even), 16-byte aligned
 * lse        device [B][Hq] float, or NULL
 * scale      multiplies the scores (1/sqrt(D) in the usual models)
 * hip_stream a hipStream_t (NULL = the default stream)
 *
 * Supported: D in {64, 128}; in_dtype BF16 or F32 (or BF16_VALU); G = Hq/Hkv in {1, 2, 4, 8}
 * (else FAIRKV_EUNSUPPORTED).
 * Calls that share a workspace must be ordered on one stream.
 */
int fairkv_decode_attn(const void *q, const void *k, const void *v, int64_t n_rows,
                       const fairkv_item *items, const fairkv_item *items_host, int32_t n_items,
                       const int32_t *slot_ptr, int32_t n_slots,
                       int32_t n_parts, void *workspace, size_t workspace_bytes,
                       void *out, float *lse,
                       int32_t B, int32_t Hq, int32_t Hkv, int32_t D,
                       int32_t in_dtype, int32_t out_dtype, float scale, void *hip_stream);

/* ---- placement over the GPUs of a tensor-parallel group (Section 4.3, Algorithms 1 and 2) -------
 *
 * Host only.  Which GPU holds which attention head of one layer, and which heads are replicated
 * so that their copies share the batch rows (Fair-Copying); with max_extra = 0 it is the
 * Best-effort Assignment (heads permuted over GPUs, no copies).  A copy of a head with c copies
 * weighs W / c (Algorithm 2's adjusted weights); the scheme kept is the first one, in the order of
 * the paper's two algorithms, with the smallest difference between the heaviest and the lightest
 * GPU (Algorithm 2's criterion).  Appendix A: every head is placed (eq. 2), at most max_copies
 * copies per head (eq. 3), efficiency = mean load / largest load (eq. 5).
 *
 * Readings: the extra copies of a scheme, sum over heads of (copies - 1), are at most max_extra
 * (Algorithm 1 declares such a bound and never uses it); the copies of a head sit on different
 * GPUs; GPUs may hold different numbers of heads; an idle GPU weighs 0; schemes are walked head
 * by head with 1 copy first, then 2, 3, ..., and splits in lexicographic order of the GPU of
 * (head 0 copy 0, head 0 copy 1, ..., head 1 copy 0, ...).
 *
 * FAIRKV_PLACE_EXACT walks all schemes (exponential: meant for the paper's handful of heads);
 * FAIRKV_PLACE_GREEDY places copies longest first on the least loaded GPU that does not hold
 * the head yet, then up to max_extra times gives one more copy to the heaviest copy on the
 * most loaded GPU while that lowers the largest load; FAIRKV_PLACE_AUTO is EXACT while
 * n_heads + max_extra <= 12, else GREEDY. */
enum { FAIRKV_PLACE_AUTO = 0, FAIRKV_PLACE_EXACT = 1, FAIRKV_PLACE_GREEDY = 2 };

typedef struct {
    int32_t tp;          /* GPUs of the group, >= 1 */
    int32_t max_extra;   /* m: extra copies in total, >= 0 */
    int32_t max_copies;  /* R_max of eq. 3: copies per head, 1..8 (and never more than tp) */
    int32_t mode;        /* FAIRKV_PLACE_* */
} fairkv_place_params;

/* One copy of a head: GPU `gpu` serves batch rows [row_begin, row_end) of head `head`.  The
 * copies of a head are numbered by ascending GPU and share the B rows contiguously; with c
 * copies the first B mod c of them take ceil(B / c) rows. */
typedef struct {
    int32_t head, gpu, copy, n_copies, row_begin, row_end;
} fairkv_share; /* 24 bytes */

typedef struct {
    int64_t den;           /* loads are in units of 1/den tokens, den = lcm(1..max_copies) */
    int64_t delta_num;     /* heaviest minus lightest GPU */
    int64_t max_load_num;
    int64_t min_load_num;
    double efficiency;     /* eq. 5 */
    int32_t n_shares;      /* copies in the scheme (also when they did not fit shares_cap) */
    int32_t exact;         /* 1: exhaustive walk, 0: greedy */
} fairkv_place_summary;

/* W         host [n_heads]: weight of every head (tokens it keeps, summed over the batch), 0..2^40
 * B         batch rows to share among the copies of a head, >= 1
 * shares    host [shares_cap], out, ordered by (head, copy); may be NULL iff shares_cap == 0
 * gpu_load  host [tp] or NULL, out: load of every GPU in units of 1/den
 * summary   host, out, required
 * Returns FAIRKV_ECAP (summary and gpu_load filled, no share written) when the scheme has more
 * copies than shares_cap; n_heads + max_extra always suffices. */
int fairkv_place(const int64_t *W, int32_t n_heads, int32_t B, const fairkv_place_params *p,
                 fairkv_share *shares, int32_t shares_cap, int64_t *gpu_load, fairkv_place_summary *summary);

/* Several new tokens per sequence in one call (a draft of q_len tokens being verified, or a short
 * chunk of prompt): not in the paper; the same path with the G heads of a group and the q_len new
 * tokens sharing the 16 columns of a matrix-core tile, so K and V are still streamed once.  The
 * caller has appended the new tokens' K/V first: they are the LAST q_len rows of every pair, and
 * new token i (0-based) attends rows [0, len - (q_len - 1 - i)) of the pair (causal among the new
 * tokens; nothing if that is not positive: out 0, lse -inf).  q and out are [B][q_len][Hq][D],
 * lse [B][q_len][Hq]; everything else as in fairkv_decode_attn, which is the case q_len = 1.
 * The workspace must hold fairkv_workspace_bytes(n_parts, B*Hkv, G * q_len, D) bytes.
 * The last chunk of a cut pair must hold at least q_len - 1 tokens (else FAIRKV_EINVAL): the rows
 * the new tokens hide from one another are masked inside that chunk only.  The FAIR policy makes
 * no chunk below min_chunk >= 16, so its plans always qualify.
 * Supported: bf16 inputs, G * q_len in {1, 2, 4, 8, 16} (else FAIRKV_EUNSUPPORTED). */
int fairkv_decode_attn_multi(const void *q, const void *k, const void *v, int64_t n_rows,
                             const fairkv_item *items, const fairkv_item *items_host, int32_t n_items,
                             const int32_t *slot_ptr, int32_t n_slots,
                             int32_t n_parts, void *workspace, size_t workspace_bytes,
                             void *out, float *lse,
                             int32_t B, int32_t q_len, int32_t Hq, int32_t Hkv, int32_t D,
                             int32_t in_dtype, int32_t out_dtype, float scale, void *hip_stream);

/* The same path over a cache stored as 8-bit floats: not in the paper (which fixes no storage
 * precision), an extension of its decode step.  Half the bytes per retained token, on a path bound
 * by HBM bandwidth.
 * k8, v8   device [n_rows][D] bytes: E4M3 in the finite-only encoding (1 sign, 4 exponent bits with
 *          bias 7, 3 mantissa bits; no infinities; S.1111.111 is NaN and must not occur).  A stored
 *          byte x stands for the value x * k_scale (x * v_scale): one scale per tensor.
 * q        device bf16 [B][q_len][Hq][D], D 64 or 128; out, lse, items, slot_ptr, workspace, n_rows,
 *          q_len as in fairkv_decode_attn_multi (q_len = 1: fairkv_decode_attn).
 * The bytes are widened to bf16 exactly and the products run as in the bf16 path, k_scale folded
 * into the softmax scale and v_scale into the final normalisation.
 * Returns FAIRKV_EINVAL for a scale that is not finite. */
int fairkv_decode_attn_kv8(const void *q, const void *k8, const void *v8, int64_t n_rows,
                           float k_scale, float v_scale,
                           const fairkv_item *items, const fairkv_item *items_host, int32_t n_items,
                           const int32_t *slot_ptr, int32_t n_slots,
                           int32_t n_parts, void *workspace, size_t workspace_bytes,
                           void *out, float *lse,
                           int32_t B, int32_t q_len, int32_t Hq, int32_t Hkv, int32_t D,
                           int32_t out_dtype, float scale, void *hip_stream);

/* The same with a scale per KV head: k_scale, v_scale host [Hkv], Hkv <= 8 (else FAIRKV_EUNSUPPORTED); a
 * stored byte of head h stands for byte * k_scale[h] (v_scale[h]).  The scales travel in the kernel
 * arguments; nothing else differs from fairkv_decode_attn_kv8. */
int fairkv_decode_attn_kv8_per_head(const void *q, const void *k8, const void *v8, int64_t n_rows,
                                    const float *k_scale, const float *v_scale,
                                    const fairkv_item *items, const fairkv_item *items_host, int32_t n_items,
                                    const int32_t *slot_ptr, int32_t n_slots,
                                    int32_t n_parts, void *workspace, size_t workspace_bytes,
                                    void *out, float *lse,
                                    int32_t B, int32_t q_len, int32_t Hq, int32_t Hkv, int32_t D,
                                    int32_t out_dtype, float scale, void *hip_stream);

/* For callers that cannot allocate device memory: code under HIP graph capture, tight serving loops,
 * harnesses that forbid hipMalloc.  fairkv_decode_attn_multi with the workspace inside the library: a device
 * array of FAIRKV_STATIC_WORKSPACE_BYTES that is part of the loaded library on every GPU (each GPU the library
 * runs on holds it until the process ends).  The call allocates and frees nothing, on the device or on the
 * host; inputs and outputs are the caller's as before.
 * Returns FAIRKV_EWORKSPACE when fairkv_workspace_bytes(n_parts, B*Hkv, G*q_len, D) exceeds
 * FAIRKV_STATIC_WORKSPACE_BYTES (8 MiB: about 1500 partial slots at G = 8, D = 128; the largest workload here,
 * 1024 pairs on 256 slots, needs 1279).  Everything else as fairkv_decode_attn_multi, same kernels.
 * All calls on one GPU share that GPU's array: calls that overlap in time on one GPU (different streams, or
 * different host threads without ordering) race; order them on one stream.  The array is zero when the
 * library is loaded; a call needs only the arrival counters at the array's start to be zero, and every
 * completed call leaves them zero, whatever its sizes (nothing else is read before it is written). */
enum { FAIRKV_STATIC_WORKSPACE_BYTES = 8 << 20 };
int fairkv_decode_attn_static(const void *q, const void *k, const void *v, int64_t n_rows,
                              const fairkv_item *items, const fairkv_item *items_host, int32_t n_items,
                              const int32_t *slot_ptr, int32_t n_slots, int32_t n_parts, void *out, float *lse,
                              int32_t B, int32_t q_len, int32_t Hq, int32_t Hkv, int32_t D,
                              int32_t in_dtype, int32_t out_dtype, float scale, void *hip_stream);

/* ---- building and growing the packed cache (the step before the path) ---------------------------
 *
 * fairkv_pack gathers the tokens a per-head compressor kept (Section 2: which entries a method
 * retains per head is its own business) out of a dense cache into the packed layout: for pair
 * p = b*Hkv + h and i < len, packed row off[p] + i = dense row keep_t[keep_ptr[p] + i] of
 * k_dense[b][h].  The rows to move are named by a work list in the format of fairkv_plan (made
 * from the same len and off: an item is a run of tok_count packed rows of pair (b, h) starting
 * at row; chunk fields are ignored), so that a ragged cache is gathered by evenly loaded
 * workgroups, one per slot.  Rows of no pair are left untouched.
 *
 * All pointers are DEVICE pointers.  k_dense, v_dense [B][Hkv][T][D] and k_out, v_out
 * [n_rows][D] of element type dtype, 16-byte aligned; keep_ptr int64 [B*Hkv+1]; keep_t int32;
 * off int64 [B*Hkv]; items [slot_ptr[n_slots]], slot_ptr int32 [n_slots+1]; bad: int32 counter or
 * NULL, incremented for every item or row that points outside its arrays (such rows are skipped,
 * nothing out of bounds is touched).  Supported: D * sizeof(element) in {128, 256, 512}.
 * Enqueues one kernel on hip_stream; no synchronisation. */
int fairkv_pack(const void *k_dense, const void *v_dense, int32_t B, int32_t Hkv, int32_t T, int32_t D,
                int32_t dtype, const int64_t *keep_ptr, const int32_t *keep_t, const int64_t *off,
                const fairkv_item *items, const int32_t *slot_ptr, int32_t n_slots, void *k_out, void *v_out,
                int64_t n_rows, int32_t *bad, void *hip_stream);

/* fairkv_append puts a decode step's new K and V row of every pair (k_new, v_new [B][Hkv][D])
 * behind the pair's last row, row off[p] + len[p], and adds one to len[p]; a pair with
 * len[p] >= cap[p] (its reserved rows are used up) is left alone and counted in *full.  All
 * pointers are DEVICE pointers; len is updated in place.  The caller re-plans (or grows the last
 * chunk of every pair in its plan) from the new lengths.  Enqueues one kernel; no synchronisation. */
int fairkv_append(const void *k_new, const void *v_new, int32_t B, int32_t Hkv, int32_t D, int32_t dtype,
                  const int64_t *off, int32_t *len, const int32_t *cap, void *k, void *v, int64_t n_rows,
                  int32_t *full, void *hip_stream);

/* Host mirror of fairkv_append for a plan that stays in use: the last chunk of every pair whose
 * len[p] < cap[p] covers one more row (tok_count + 1) and len[p] grows by one; pairs at capacity
 * are left alone.  items, len (in/out) and cap are HOST arrays; items must be a whole plan (one
 * last chunk per pair).  The plan stays valid and drifts from balance by at most one row per pair
 * and step; re-plan with fairkv_plan every few hundred steps. */
int fairkv_plan_grow(fairkv_item *items, int32_t n_items, int32_t B, int32_t Hkv, int32_t *len, const int32_t *cap);

/* The measurement aids (the decode kernel with wall-clock stamps, the reader that only streams) are declared in
 * fairkv_measure.h: they are in the library for the benchmark, not for callers of the method. */

const char *fairkv_strerror(int code);
int fairkv_version(void);

#ifdef __cplusplus
}
#endif
#endif /* FAIRKV_H */

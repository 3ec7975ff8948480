// Host-side work planner: balances (sequence, KV head) pairs of unequal retained-token
// counts over workgroup slots.
//
// The objective is the paper's (Appendix A, eq. 4): make the largest per-device load as
// small as possible, where a head replicated r times weighs W/r on each replica
// (Algorithm 2's adjusted weights) and r is capped (eq. 3).  The paper searches
// exhaustively over a few heads and GPUs (Algorithms 1 and 2); with hundreds of pairs
// and hundreds of slots that is out of reach, so this is the classical greedy for the
// same objective: cut heavy pairs into equal token chunks, then place chunks longest
// first on the least loaded slot.  Integer arithmetic only, so the plan is reproducible.
#include "fairkv.h"

#include <algorithm>
#include <cstdint>
#include <functional>
#include <limits>
#include <queue>
#include <utility>
#include <vector>

namespace {

inline int64_t ceil_div(int64_t a, int64_t b) { return (a + b - 1) / b; }

bool params_ok(const fairkv_plan_params &p)
{
    if (p.n_slots < 1 || p.tile < 1 || p.max_split < 1 || p.oversub < 1) return false;
    if (p.min_chunk < p.tile || p.min_chunk % p.tile != 0) return false;
    if (p.overhead_tokens < 0 || p.reserved != 0) return false;
    return p.policy == FAIRKV_POLICY_NAIVE || p.policy == FAIRKV_POLICY_LPT ||
           p.policy == FAIRKV_POLICY_LPT_SPLIT;
}

struct Piece {
    int32_t b, h, begin, count, chunk, n_chunks, part;
};

}  // namespace

extern "C" int fairkv_default_params(fairkv_plan_params *p, int32_t n_compute_units)
{
    if (!p || n_compute_units < 1 || n_compute_units > (1 << 20)) return FAIRKV_EINVAL;
    p->n_slots = 2 * n_compute_units;
    p->tile = 64;
    p->min_chunk = 256;
    p->max_split = 128;
    p->oversub = 2;
    p->overhead_tokens = 64;
    p->policy = FAIRKV_POLICY_LPT_SPLIT;
    p->reserved = 0;
    return FAIRKV_OK;
}

extern "C" int fairkv_plan(const int32_t *len, int32_t B, int32_t Hkv, const fairkv_plan_params *p,
                           fairkv_item *items, int32_t items_cap, int32_t *slot_ptr,
                           int32_t *part_base, fairkv_plan_summary *summary)
{
    if (!len || !p || !summary || B < 1 || Hkv < 1 || items_cap < 0) return FAIRKV_EINVAL;
    if (!items && items_cap != 0) return FAIRKV_EINVAL;
    if (!params_ok(*p)) return FAIRKV_EINVAL;
    const int64_t n_pairs = static_cast<int64_t>(B) * Hkv;
    if (n_pairs > std::numeric_limits<int32_t>::max() / 2) return FAIRKV_EINVAL;

    int64_t total = 0;
    for (int64_t i = 0; i < n_pairs; ++i) {
        if (len[i] < 0) return FAIRKV_EINVAL;
        total += len[i];
    }

    const int64_t tile = p->tile;
    auto round_up = [tile](int64_t x) { return ceil_div(x, tile) * tile; };

    // Chunk size every heavy pair is measured against: about n_slots * oversub chunks overall.
    const bool split = p->policy == FAIRKV_POLICY_LPT_SPLIT;
    int64_t target = 0;
    if (split) {
        const int64_t want = static_cast<int64_t>(p->n_slots) * p->oversub;
        target = std::max<int64_t>(p->min_chunk, round_up(ceil_div(total, want)));
    }

    std::vector<Piece> pieces;
    pieces.reserve(static_cast<size_t>(n_pairs) * 2);
    int64_t parts = 0;
    if (part_base) part_base[0] = 0;
    for (int64_t pair = 0; pair < n_pairs; ++pair) {
        const int64_t n = len[pair];
        if (n > 0) {
            const int64_t copies = split ? std::min<int64_t>(p->max_split, ceil_div(n, target)) : 1;
            const int64_t share = round_up(ceil_div(n, copies));   // W / copies, whole tiles
            const int64_t n_chunks = ceil_div(n, share);
            if (parts + n_chunks > std::numeric_limits<int32_t>::max()) return FAIRKV_EINVAL;
            for (int64_t c = 0; c < n_chunks; ++c) {
                Piece pc;
                pc.b = static_cast<int32_t>(pair / Hkv);
                pc.h = static_cast<int32_t>(pair % Hkv);
                pc.begin = static_cast<int32_t>(c * share);
                pc.count = static_cast<int32_t>(std::min<int64_t>(share, n - c * share));
                pc.chunk = static_cast<int32_t>(c);
                pc.n_chunks = static_cast<int32_t>(n_chunks);
                pc.part = static_cast<int32_t>(parts + c);
                pieces.push_back(pc);
            }
            parts += n_chunks;
        }
        if (part_base) part_base[pair + 1] = static_cast<int32_t>(parts);
    }

    const size_t n_items = pieces.size();
    std::vector<int32_t> slot_of(n_items);
    std::vector<int64_t> load(static_cast<size_t>(p->n_slots), 0);

    if (p->policy == FAIRKV_POLICY_NAIVE) {
        for (size_t i = 0; i < n_items; ++i) {
            const int32_t j = static_cast<int32_t>(i % static_cast<size_t>(p->n_slots));
            slot_of[i] = j;
            load[j] += static_cast<int64_t>(pieces[i].count) + p->overhead_tokens;
        }
    } else {
        std::sort(pieces.begin(), pieces.end(), [](const Piece &x, const Piece &y) {
            if (x.count != y.count) return x.count > y.count;
            if (x.b != y.b) return x.b < y.b;
            if (x.h != y.h) return x.h < y.h;
            return x.chunk < y.chunk;
        });
        // min-heap on (load, slot index): the pair order makes the least loaded slot with the
        // lowest index come out first, which is what a linear scan with "first minimum" gives.
        using Entry = std::pair<int64_t, int32_t>;
        std::priority_queue<Entry, std::vector<Entry>, std::greater<Entry>> heap;
        for (int32_t j = 0; j < p->n_slots; ++j) heap.emplace(0, j);
        for (size_t i = 0; i < n_items; ++i) {
            Entry e = heap.top();
            heap.pop();
            slot_of[i] = e.second;
            e.first += static_cast<int64_t>(pieces[i].count) + p->overhead_tokens;
            load[static_cast<size_t>(e.second)] = e.first;
            heap.push(e);
        }
    }

    summary->total_tokens = total;
    summary->max_slot_load = *std::max_element(load.begin(), load.end());
    summary->min_slot_load = *std::min_element(load.begin(), load.end());
    summary->n_items = static_cast<int32_t>(n_items);
    summary->n_parts = static_cast<int32_t>(parts);

    if (slot_ptr) {
        for (int32_t j = 0; j <= p->n_slots; ++j) slot_ptr[j] = 0;
        for (size_t i = 0; i < n_items; ++i) slot_ptr[slot_of[i] + 1] += 1;
        for (int32_t j = 0; j < p->n_slots; ++j) slot_ptr[j + 1] += slot_ptr[j];
    }

    if (n_items > static_cast<size_t>(items_cap)) return FAIRKV_ECAP;
    for (size_t i = 0; i < n_items; ++i) {
        const Piece &pc = pieces[i];
        fairkv_item &it = items[i];
        it.b = pc.b;
        it.h = pc.h;
        it.tok_begin = pc.begin;
        it.tok_count = pc.count;
        it.chunk = pc.chunk;
        it.n_chunks = pc.n_chunks;
        it.slot = slot_of[i];
        it.part = pc.part;
    }
    return FAIRKV_OK;
}

extern "C" const char *fairkv_strerror(int code)
{
    switch (code) {
    case FAIRKV_OK: return "ok";
    case FAIRKV_EINVAL: return "invalid argument";
    case FAIRKV_ECAP: return "items array too small";
    case FAIRKV_EWORKSPACE: return "workspace too small";
    case FAIRKV_EUNSUPPORTED: return "unsupported element type, head_dim or group size";
    case FAIRKV_EHIP: return "HIP call failed";
    default: return "unknown fairkv status";
    }
}

extern "C" int fairkv_version(void) { return 100; }

// Host-side work planner: balances (sequence, KV head) pairs of unequal retained-token
// counts over workgroup slots.
//
// The objective is the paper's (Appendix A, eq. 4): make the largest per-device load as
// small as possible, where a head replicated r times weighs W/r on each replica
// (Algorithm 2's adjusted weights) and r is capped (eq. 3).  The paper searches
// exhaustively over a few heads and GPUs (Algorithms 1 and 2); with hundreds of pairs
// and hundreds of slots that is out of reach, so this is the classical greedy for the
// same objective: either cut heavy pairs into equal token chunks and place chunks longest
// first on the least loaded slot, or (FAIR) cut the line of all pairs into pieces of equal
// cost.  Integer arithmetic only, so the plan is reproducible.
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
    if (p.overhead_tokens < 0 || p.short_overhead_tokens < 0) return false;
    return p.policy >= FAIRKV_POLICY_NAIVE && p.policy <= FAIRKV_POLICY_FAIR;
}

// A token chunk of one pair, before it is turned into a fairkv_item.
struct Piece {
    int32_t pair, begin, count, chunk, slot;
};

// Fixed cost of an item of `count` tokens: a whole pair of at most FAIRKV_SHORT_PAIR_TOKENS tokens is cheaper
// for the kernel (one wave runs it alone), if the parameters say by how much.
inline int64_t item_overhead(const fairkv_plan_params &p, int64_t count, bool whole_pair)
{
    return whole_pair && count <= FAIRKV_SHORT_PAIR_TOKENS && p.short_overhead_tokens > 0 ? p.short_overhead_tokens
                                                                                          : p.overhead_tokens;
}

// FAIR: lay the pairs end to end and cut the line into n_slots pieces of equal cost.
void cut_line(const int32_t *len, int64_t n_pairs, int64_t total, const fairkv_plan_params &p,
              std::vector<Piece> &pieces, std::vector<int32_t> &n_chunks)
{
    const int64_t S = p.n_slots, tile = p.tile;
    int64_t tokens_left = total;
    int64_t ov_left = 0;      // fixed costs of the pairs not yet finished, each taken as one whole item
    for (int64_t pair = 0; pair < n_pairs; ++pair) ov_left += item_overhead(p, len[pair], true);
    int64_t slot = 0;
    auto open_budget = [&](int64_t j) {
        const int64_t open_slots = S - j;
        return ceil_div(tokens_left + ov_left + p.overhead_tokens * open_slots, open_slots);
    };
    int64_t room = open_budget(0);
    for (int64_t pair = 0; pair < n_pairs; ++pair) {
        int64_t left = len[pair], begin = 0;
        int32_t copies = 0;
        if (left == 0) {   // an empty pair still needs someone to write its zero output
            const int64_t ov = item_overhead(p, 0, true);
            if (room < ov && slot < S - 1) room = open_budget(++slot);
            pieces.push_back({static_cast<int32_t>(pair), 0, 0, 0, static_cast<int32_t>(slot)});
            room -= ov;
            copies = 1;
        }
        while (left > 0) {
            const bool must_finish = slot == S - 1 || copies == p.max_split - 1;
            // ov_take_all: the fixed cost if this item takes all that is left of the pair (a short pair taken whole
            // has its own); a piece of a cut pair costs the full overhead.  fit: whole tiles that still fit.
            const int64_t ov_take_all = item_overhead(p, left, begin == 0), ov = p.overhead_tokens;
            const int64_t fit_all = std::max<int64_t>(0, (room - ov_take_all) / tile * tile);
            const int64_t fit = std::max<int64_t>(0, (room - ov) / tile * tile);
            int64_t take;
            if (must_finish || left <= fit_all)
                take = left;
            else if (fit >= p.min_chunk && left - fit >= p.min_chunk)
                take = fit;
            else if (left - fit <= fit)
                take = left;
            else {
                room = open_budget(++slot);
                continue;
            }
            pieces.push_back({static_cast<int32_t>(pair), static_cast<int32_t>(begin), static_cast<int32_t>(take),
                              copies, static_cast<int32_t>(slot)});
            room -= take + (take == left ? ov_take_all : ov);
            begin += take;
            left -= take;
            tokens_left -= take;
            ++copies;
            if (left > 0 && slot < S - 1) room = open_budget(++slot);
        }
        n_chunks[static_cast<size_t>(pair)] = copies;
        ov_left -= item_overhead(p, len[pair], true);
    }
}

}  // namespace

extern "C" int fairkv_default_params(fairkv_plan_params *p, int32_t n_compute_units)
{
    if (!p || n_compute_units < 1 || n_compute_units > (1 << 20)) return FAIRKV_EINVAL;
    p->n_slots = n_compute_units;
    p->tile = 16;
    p->min_chunk = 32;
    p->max_split = 256;
    p->oversub = 2;
    p->overhead_tokens = 160;
    p->policy = FAIRKV_POLICY_FAIR;
    p->short_overhead_tokens = 48;
    return FAIRKV_OK;
}

extern "C" int fairkv_plan(const int32_t *len, const int64_t *off, int32_t B, int32_t Hkv,
                           const fairkv_plan_params *p, fairkv_item *items, int32_t items_cap,
                           int32_t *slot_ptr, int32_t *part_base, fairkv_plan_summary *summary)
{
    if (!len || !off || !p || !summary || B < 1 || Hkv < 1 || items_cap < 0) return FAIRKV_EINVAL;
    if (!items && items_cap != 0) return FAIRKV_EINVAL;
    if (!params_ok(*p)) return FAIRKV_EINVAL;
    const int64_t n_pairs = static_cast<int64_t>(B) * Hkv;
    if (n_pairs > std::numeric_limits<int32_t>::max() / 2) return FAIRKV_EINVAL;

    int64_t total = 0;
    for (int64_t i = 0; i < n_pairs; ++i) {
        if (len[i] < 0 || (len[i] > 0 && off[i] < 0)) return FAIRKV_EINVAL;
        total += len[i];
    }

    const int64_t tile = p->tile;
    const int32_t S = p->n_slots;
    auto round_up = [tile](int64_t x) { return ceil_div(x, tile) * tile; };

    std::vector<Piece> pieces;
    pieces.reserve(static_cast<size_t>(n_pairs) + static_cast<size_t>(S));
    std::vector<int32_t> n_chunks(static_cast<size_t>(n_pairs), 0);

    if (p->policy == FAIRKV_POLICY_FAIR) {
        cut_line(len, n_pairs, total, *p, pieces, n_chunks);
    } else {
        // Equal shares of a heavy pair (W / copies), measured against about n_slots * oversub
        // chunks overall; NAIVE and LPT keep pairs whole.
        const bool split = p->policy == FAIRKV_POLICY_LPT_SPLIT;
        const int64_t target =
            split ? std::max<int64_t>(p->min_chunk, round_up(ceil_div(total, static_cast<int64_t>(S) * p->oversub))) : 0;
        for (int64_t pair = 0; pair < n_pairs; ++pair) {
            const int64_t n = len[pair];
            if (n == 0) {
                pieces.push_back({static_cast<int32_t>(pair), 0, 0, 0, 0});
                n_chunks[static_cast<size_t>(pair)] = 1;
                continue;
            }
            const int64_t copies = split ? std::min<int64_t>(p->max_split, ceil_div(n, target)) : 1;
            const int64_t share = round_up(ceil_div(n, copies));
            const int64_t made = ceil_div(n, share);
            for (int64_t c = 0; c < made; ++c)
                pieces.push_back({static_cast<int32_t>(pair), static_cast<int32_t>(c * share),
                                  static_cast<int32_t>(std::min<int64_t>(share, n - c * share)),
                                  static_cast<int32_t>(c), 0});
            n_chunks[static_cast<size_t>(pair)] = static_cast<int32_t>(made);
        }
        if (p->policy == FAIRKV_POLICY_NAIVE) {
            for (size_t i = 0; i < pieces.size(); ++i) pieces[i].slot = static_cast<int32_t>(i % static_cast<size_t>(S));
        } else {
            std::sort(pieces.begin(), pieces.end(), [](const Piece &x, const Piece &y) {
                if (x.count != y.count) return x.count > y.count;
                if (x.pair != y.pair) return x.pair < y.pair;
                return x.chunk < y.chunk;
            });
            // min-heap on (load, slot): pops the least loaded slot, lowest index on ties
            using Entry = std::pair<int64_t, int32_t>;
            std::priority_queue<Entry, std::vector<Entry>, std::greater<Entry>> heap;
            for (int32_t j = 0; j < S; ++j) heap.emplace(0, j);
            for (Piece &pc : pieces) {
                Entry e = heap.top();
                heap.pop();
                pc.slot = e.second;
                e.first += static_cast<int64_t>(pc.count) + item_overhead(*p, pc.count, n_chunks[static_cast<size_t>(pc.pair)] == 1);
                heap.push(e);
            }
        }
    }

    // chunks before each pair
    std::vector<int64_t> base(static_cast<size_t>(n_pairs) + 1, 0);
    for (int64_t pair = 0; pair < n_pairs; ++pair) base[pair + 1] = base[pair] + n_chunks[static_cast<size_t>(pair)];
    if (base[n_pairs] > std::numeric_limits<int32_t>::max()) return FAIRKV_EINVAL;
    if (part_base)
        for (int64_t i = 0; i <= n_pairs; ++i) part_base[i] = static_cast<int32_t>(base[i]);

    // group by slot, keeping the order in which a slot received its pieces
    std::vector<int32_t> start(static_cast<size_t>(S) + 1, 0);
    std::vector<int64_t> load(static_cast<size_t>(S), 0);
    for (const Piece &pc : pieces) {
        start[static_cast<size_t>(pc.slot) + 1] += 1;
        load[static_cast<size_t>(pc.slot)] += static_cast<int64_t>(pc.count) + item_overhead(*p, pc.count, n_chunks[static_cast<size_t>(pc.pair)] == 1);
    }
    for (int32_t j = 0; j < S; ++j) start[j + 1] += start[j];

    summary->total_tokens = total;
    summary->max_slot_load = *std::max_element(load.begin(), load.end());
    summary->min_slot_load = *std::min_element(load.begin(), load.end());
    summary->n_items = static_cast<int32_t>(pieces.size());
    summary->n_parts = static_cast<int32_t>(base[n_pairs]);
    if (slot_ptr)
        for (int32_t j = 0; j <= S; ++j) slot_ptr[j] = start[j];

    if (pieces.size() > static_cast<size_t>(items_cap)) return FAIRKV_ECAP;
    std::vector<int32_t> cursor(start.begin(), start.end() - 1);
    for (const Piece &pc : pieces) {
        fairkv_item &it = items[cursor[static_cast<size_t>(pc.slot)]++];
        it.row = off[pc.pair] + pc.begin;
        it.tok_count = pc.count;
        it.b = pc.pair / Hkv;
        it.h = pc.pair % Hkv;
        it.chunk = pc.chunk;
        it.n_chunks = n_chunks[static_cast<size_t>(pc.pair)];
        it.part = static_cast<int32_t>(base[pc.pair] + pc.chunk);
    }
    return FAIRKV_OK;
}

extern "C" int fairkv_plan_grow(fairkv_item *items, int32_t n_items, int32_t B, int32_t Hkv, int32_t *len,
                                const int32_t *cap)
{
    if (!items || !len || !cap || n_items < 0 || B < 1 || Hkv < 1) return FAIRKV_EINVAL;
    const int64_t n_pairs = static_cast<int64_t>(B) * Hkv;
    std::vector<char> seen(static_cast<size_t>(n_pairs), 0);
    for (int32_t i = 0; i < n_items; ++i) {
        const fairkv_item &it = items[i];
        if (it.b < 0 || it.b >= B || it.h < 0 || it.h >= Hkv || it.n_chunks < 1) return FAIRKV_EINVAL;
    }
    for (int32_t i = 0; i < n_items; ++i) {
        fairkv_item &it = items[i];
        if (it.chunk != it.n_chunks - 1) continue;
        const int64_t pair = static_cast<int64_t>(it.b) * Hkv + it.h;
        if (seen[pair]) return FAIRKV_EINVAL;      // two last chunks for one pair: not a plan
        seen[pair] = 1;
        if (len[pair] < cap[pair]) {
            ++it.tok_count;
            ++len[pair];
        }
    }
    return FAIRKV_OK;
}

extern "C" const char *fairkv_strerror(int code)
{
    switch (code) {
    case FAIRKV_OK: return "ok";
    case FAIRKV_EINVAL: return "invalid argument";
    case FAIRKV_ECAP: return "output array too small";
    case FAIRKV_EWORKSPACE: return "workspace too small";
    case FAIRKV_EUNSUPPORTED: return "unsupported element type, head_dim or group size";
    case FAIRKV_EHIP: return "HIP call failed";
    default: return "unknown fairkv status";
    }
}

extern "C" int fairkv_version(void) { return 100; }

// Multi-GPU head placement (Section 4.3, Algorithms 1 and 2; Appendix A): which GPU of a
// tensor-parallel group holds which attention head, and which heads are replicated and
// share their batch rows (Fair-Copying).
//
// The paper enumerates every replication scheme (Algorithm 1) and, for each, every split of
// the head copies into one group per GPU, keeping the split with the smallest difference
// between the heaviest and the lightest group, a copy weighing W / copies (Algorithm 2).
// That is the definition this file answers to.  The walk here is the same walk, in the same
// order, with two cuts that cannot change its answer:
//   * splits that differ from an earlier one only by renaming GPUs or by swapping copies of
//     one head are skipped (the earlier one has the same group weights and is kept anyway);
//   * a partial split is abandoned once no completion can beat the best difference so far:
//     the heaviest group only grows, and the lightest can end no higher than the mean, nor
//     higher than its present weight plus everything still to be placed.
// For layers too large for any exhaustive walk there is a greedy variant (copies longest first
// onto the least loaded GPU; then repeatedly one more copy for the heaviest copy on the most
// loaded GPU while that lowers the largest load).
#include "fairkv.h"

#include <algorithm>
#include <cstdint>
#include <vector>

namespace {

constexpr int kExactLimit = 12;   // FAIRKV_PLACE_AUTO walks exhaustively while heads + extra copies <= this

int64_t lcm_upto(int n)
{
    int64_t out = 1;
    for (int k = 2; k <= n; ++k) {
        int64_t a = out, b = k;
        while (b) {
            const int64_t t = a % b;
            a = b;
            b = t;
        }
        out = out / a * k;
    }
    return out;
}

struct Scheme {
    std::vector<int32_t> copies;   // per head
    std::vector<int32_t> gpu;      // per copy, heads in order, a head's copies on ascending GPUs
    std::vector<int64_t> load;     // per GPU, scaled by den
};

// ---- exhaustive walk ------------------------------------------------------------------------
class Walk {
  public:
    Walk(const std::vector<int64_t> &w, int tp, int m, int cap) : w_(w), tp_(tp), m_(m), cap_(cap), n_(static_cast<int>(w.size()))
    {
        for (int64_t x : w_) total_ += x;
        mean_floor_ = total_ / tp_;
        copies_.assign(n_, 1);
    }

    Scheme run()
    {
        schemes(0, m_);
        return best_;
    }

  private:
    // Algorithm 1: head by head, one copy first, then 2, 3, ... while extra copies remain.
    void schemes(int head, int extra_left)
    {
        if (done_) return;
        if (head == n_) {
            splits();
            return;
        }
        copies_[head] = 1;
        schemes(head + 1, extra_left);
        for (int k = 2; k <= std::min(cap_, 1 + extra_left) && !done_; ++k) {
            copies_[head] = k;
            schemes(head + 1, extra_left - (k - 1));
        }
        copies_[head] = 1;
    }

    // Algorithm 2 for the scheme in copies_: depth-first over the copies in order.
    void splits()
    {
        owner_.clear();
        weight_.clear();
        for (int i = 0; i < n_; ++i)
            for (int r = 0; r < copies_[i]; ++r) {
                owner_.push_back(i);
                weight_.push_back(w_[i] / copies_[i]);
            }
        const int K = static_cast<int>(owner_.size());
        suffix_.assign(K + 1, 0);
        for (int k = K - 1; k >= 0; --k) suffix_[k] = suffix_[k + 1] + weight_[k];
        gpu_.assign(K, 0);
        load_.assign(tp_, 0);
        descend(0, 0);
    }

    void descend(int k, int used)
    {
        if (done_) return;
        const int K = static_cast<int>(owner_.size());
        int64_t mx = 0, mn = load_[0];
        for (int j = 0; j < tp_; ++j) {
            mx = std::max(mx, load_[j]);
            mn = std::min(mn, load_[j]);
        }
        if (k == K) {
            const int64_t d = mx - mn;
            if (!have_ || d < best_delta_) {
                have_ = true;
                best_delta_ = d;
                best_.copies = copies_;
                best_.gpu = gpu_;
                best_.load = load_;
                if (d == 0) done_ = true;   // nothing later can be strictly better
            }
            return;
        }
        if (have_) {
            const int64_t min_at_best = std::min(mean_floor_, mn + suffix_[k]);
            if (mx - min_at_best >= best_delta_) return;
        }
        const int lo = (k > 0 && owner_[k - 1] == owner_[k]) ? gpu_[k - 1] + 1 : 0;
        const int hi = std::min(tp_, used + 1);
        for (int j = lo; j < hi && !done_; ++j) {
            gpu_[k] = j;
            load_[j] += weight_[k];
            descend(k + 1, std::max(used, j + 1));
            load_[j] -= weight_[k];
        }
    }

    const std::vector<int64_t> &w_;
    const int tp_, m_, cap_, n_;
    int64_t total_ = 0, mean_floor_ = 0;
    std::vector<int32_t> copies_, owner_, gpu_;
    std::vector<int64_t> weight_, suffix_, load_;
    Scheme best_;
    int64_t best_delta_ = 0;
    bool have_ = false, done_ = false;
};

// ---- greedy ----------------------------------------------------------------------------------
struct Placed {
    std::vector<std::vector<int32_t>> gpus_of_head;
    std::vector<int64_t> load;
};

Placed longest_first(const std::vector<int64_t> &w, const std::vector<int32_t> &copies, int tp)
{
    struct Copy {
        int64_t weight;
        int32_t head, index;
    };
    std::vector<Copy> all;
    for (int32_t i = 0; i < static_cast<int32_t>(w.size()); ++i)
        for (int32_t r = 0; r < copies[i]; ++r) all.push_back({w[i] / copies[i], i, r});
    std::sort(all.begin(), all.end(), [](const Copy &a, const Copy &b) {
        if (a.weight != b.weight) return a.weight > b.weight;
        if (a.head != b.head) return a.head < b.head;
        return a.index < b.index;
    });
    Placed out;
    out.gpus_of_head.assign(w.size(), {});
    out.load.assign(tp, 0);
    for (const Copy &cp : all) {
        int pick = -1;
        for (int j = 0; j < tp; ++j) {
            const auto &held = out.gpus_of_head[cp.head];
            if (std::find(held.begin(), held.end(), j) != held.end()) continue;
            if (pick < 0 || out.load[j] < out.load[pick]) pick = j;
        }
        out.load[pick] += cp.weight;
        out.gpus_of_head[cp.head].push_back(pick);
    }
    return out;
}

Scheme greedy(const std::vector<int64_t> &w, int tp, int m, int cap)
{
    std::vector<int32_t> copies(w.size(), 1);
    Placed cur = longest_first(w, copies, tp);
    for (int step = 0; step < m; ++step) {
        int top = 0;
        for (int j = 1; j < tp; ++j)
            if (cur.load[j] > cur.load[top]) top = j;
        int pick = -1;
        int64_t pick_w = -1;
        for (int32_t i = 0; i < static_cast<int32_t>(w.size()); ++i) {
            if (copies[i] >= cap) continue;
            const auto &held = cur.gpus_of_head[i];
            if (std::find(held.begin(), held.end(), top) == held.end()) continue;
            const int64_t wi = w[i] / copies[i];
            if (wi > pick_w) {
                pick_w = wi;
                pick = i;
            }
        }
        if (pick < 0) break;
        std::vector<int32_t> trial = copies;
        ++trial[pick];
        Placed next = longest_first(w, trial, tp);
        if (*std::max_element(next.load.begin(), next.load.end()) >= *std::max_element(cur.load.begin(), cur.load.end()))
            break;
        copies.swap(trial);
        cur = std::move(next);
    }
    Scheme s;
    s.copies = copies;
    s.load = cur.load;
    for (auto &held : cur.gpus_of_head) {
        std::sort(held.begin(), held.end());
        s.gpu.insert(s.gpu.end(), held.begin(), held.end());
    }
    return s;
}

}  // namespace

extern "C" int fairkv_place(const int64_t *W, int32_t n_heads, int32_t B, const fairkv_place_params *p,
                            fairkv_share *shares, int32_t shares_cap, int64_t *gpu_load,
                            fairkv_place_summary *summary)
{
    if (!W || !p || !summary || n_heads < 1 || B < 1) return FAIRKV_EINVAL;
    if (p->tp < 1 || p->max_extra < 0 || p->max_copies < 1 || p->max_copies > 8) return FAIRKV_EINVAL;
    if (p->mode != FAIRKV_PLACE_AUTO && p->mode != FAIRKV_PLACE_EXACT && p->mode != FAIRKV_PLACE_GREEDY) return FAIRKV_EINVAL;
    if (shares_cap < 0 || (shares_cap > 0 && !shares)) return FAIRKV_EINVAL;
    for (int32_t i = 0; i < n_heads; ++i)
        if (W[i] < 0 || W[i] > (int64_t{1} << 40)) return FAIRKV_EINVAL;

    const int64_t den = lcm_upto(p->max_copies);
    std::vector<int64_t> w(n_heads);
    for (int32_t i = 0; i < n_heads; ++i) w[i] = W[i] * den;
    const int cap = std::min(p->max_copies, p->tp);
    const bool exact = p->mode == FAIRKV_PLACE_EXACT || (p->mode == FAIRKV_PLACE_AUTO && n_heads + p->max_extra <= kExactLimit);
    const Scheme s = exact ? Walk(w, p->tp, p->max_extra, cap).run() : greedy(w, p->tp, p->max_extra, cap);

    int64_t mx = 0, mn = s.load[0], sum = 0;
    for (int64_t x : s.load) {
        mx = std::max(mx, x);
        mn = std::min(mn, x);
        sum += x;
    }
    summary->den = den;
    summary->delta_num = mx - mn;
    summary->max_load_num = mx;
    summary->min_load_num = mn;
    summary->efficiency = mx == 0 ? 1.0 : static_cast<double>(sum) / static_cast<double>(static_cast<int64_t>(p->tp) * mx);
    summary->n_shares = static_cast<int32_t>(s.gpu.size());
    summary->exact = exact ? 1 : 0;
    if (gpu_load)
        for (int j = 0; j < p->tp; ++j) gpu_load[j] = s.load[j];
    if (summary->n_shares > shares_cap) return FAIRKV_ECAP;

    int32_t k = 0;
    for (int32_t i = 0; i < n_heads; ++i) {
        const int32_t c = s.copies[i], base = B / c, rem = B % c;
        for (int32_t r = 0; r < c; ++r, ++k) {
            const int32_t begin = r * base + std::min(r, rem);
            shares[k] = {i, s.gpu[k], r, c, begin, begin + base + (r < rem ? 1 : 0)};
        }
    }
    return FAIRKV_OK;
}

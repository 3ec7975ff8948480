// Command-line driver for a host build of the planner, the placement search and the C oracle under
// AddressSanitizer and UndefinedBehaviorSanitizer (CPU only; see test_host_sanitizers.py).
//
// Reads one case per line from stdin and prints one result line per case:
//   plan  B Hkv n_slots tile min_chunk max_split oversub overhead policy short_overhead cap_mode  len[B*Hkv] off[B*Hkv]
//         -> "plan rc n_items n_parts max min | row tok b h chunk n_chunks part ... | slot_ptr ... | part_base ..."
//            cap_mode 0: sized exactly; 1: one record too few (must return the capacity error and write no item)
//   place n B tp max_extra max_copies mode  W[n]
//         -> "place rc den delta max min n_shares exact | head gpu copy n_copies row_begin row_end ... | load ..."
//   attn  B Hq Hkv D seed  len[B*Hkv]
//         -> "attn rc sum(out) sum(lse over non-empty heads)" on data drawn from a small generator below
//   grow  (a plan line's arguments) steps cap_slack
//         -> "grow rc tok_count ..." after `steps` calls of fairkv_plan_grow
#include <cmath>
#include <cstdint>
#include <cstdio>
#include <iostream>
#include <sstream>
#include <string>
#include <vector>

#include "fairkv.h"

extern "C" int fairkv_oracle_attn(const void *q, const void *k, const void *v, const int64_t *off, const int32_t *len,
                                  int B, int Hq, int Hkv, int D, int dtype, double scale, const int32_t *sel, int n_sel,
                                  double *out, double *lse, int n_threads);

namespace {

// the test regenerates the same numbers in Python: x_{n+1} = x_n * 6364136223846793005 + 1442695040888963407 (mod 2^64),
// value = ((x >> 11) / 2^53 - 0.5) * 4
struct Lcg {
    uint64_t x;
    double next()
    {
        x = x * 6364136223846793005ULL + 1442695040888963407ULL;
        return (static_cast<double>(x >> 11) / 9007199254740992.0 - 0.5) * 4.0;
    }
};

bool read_plan_args(std::istringstream &in, int32_t &B, int32_t &Hkv, fairkv_plan_params &p, int &cap_mode,
                    std::vector<int32_t> &len, std::vector<int64_t> &off)
{
    in >> B >> Hkv >> p.n_slots >> p.tile >> p.min_chunk >> p.max_split >> p.oversub >> p.overhead_tokens >> p.policy >>
        p.short_overhead_tokens >> cap_mode;
    if (!in || B < 1 || Hkv < 1 || B * Hkv > (1 << 20)) return false;
    len.resize(static_cast<size_t>(B) * Hkv);
    off.resize(len.size());
    for (auto &x : len) in >> x;
    for (auto &x : off) in >> x;
    return static_cast<bool>(in);
}

}  // namespace

int main()
{
    std::string line;
    while (std::getline(std::cin, line)) {
        std::istringstream in(line);
        std::string cmd;
        in >> cmd;
        if (cmd == "plan" || cmd == "grow") {
            int32_t B, Hkv;
            fairkv_plan_params p;
            int cap_mode;
            std::vector<int32_t> len;
            std::vector<int64_t> off;
            if (!read_plan_args(in, B, Hkv, p, cap_mode, len, off)) return 2;
            fairkv_plan_summary s{};
            const int n_slots = p.n_slots > 0 ? p.n_slots : 0;
            std::vector<int32_t> slot_ptr(static_cast<size_t>(n_slots) + 1, -7), part_base(len.size() + 1, -7);
            int rc = fairkv_plan(len.data(), off.data(), B, Hkv, &p, nullptr, 0, slot_ptr.data(), part_base.data(), &s);
            if (rc != FAIRKV_OK && rc != FAIRKV_ECAP) {
                std::printf("%s %d\n", cmd.c_str(), rc);
                continue;
            }
            const int cap = cap_mode == 1 && s.n_items > 0 ? s.n_items - 1 : s.n_items;
            // exactly `cap` records on the heap: a write past the capacity is an ASan report
            std::vector<fairkv_item> items(static_cast<size_t>(cap));
            for (auto &it : items) it.part = -99;
            rc = fairkv_plan(len.data(), off.data(), B, Hkv, &p, cap ? items.data() : nullptr, cap, slot_ptr.data(),
                             part_base.data(), &s);
            if (cmd == "grow" && rc == FAIRKV_OK) {
                int steps, slack;
                in >> steps >> slack;
                std::vector<int32_t> capv(len.size());
                for (size_t i = 0; i < len.size(); ++i) capv[i] = len[i] + slack + static_cast<int32_t>(i % 3);
                int grc = 0;
                for (int st = 0; st < steps && grc == 0; ++st)
                    grc = fairkv_plan_grow(items.data(), static_cast<int32_t>(items.size()), B, Hkv, len.data(), capv.data());
                std::printf("grow %d", grc);
                for (const auto &it : items) std::printf(" %d", it.tok_count);
                std::printf("\n");
                continue;
            }
            std::printf("plan %d %d %d %lld %lld |", rc, s.n_items, s.n_parts, static_cast<long long>(s.max_slot_load),
                        static_cast<long long>(s.min_slot_load));
            for (const auto &it : items)
                std::printf(" %lld %d %d %d %d %d %d", static_cast<long long>(it.row), it.tok_count, it.b, it.h, it.chunk,
                            it.n_chunks, it.part);
            std::printf(" |");
            for (int32_t x : slot_ptr) std::printf(" %d", x);
            std::printf(" |");
            for (int32_t x : part_base) std::printf(" %d", x);
            std::printf("\n");
        } else if (cmd == "place") {
            int32_t n, B;
            fairkv_place_params p;
            in >> n >> B >> p.tp >> p.max_extra >> p.max_copies >> p.mode;
            if (!in || n < 0 || n > 4096) return 2;
            std::vector<int64_t> W(static_cast<size_t>(n));
            for (auto &x : W) in >> x;
            const int cap = n + (p.max_extra > 0 ? p.max_extra : 0);
            std::vector<fairkv_share> shares(static_cast<size_t>(cap));
            std::vector<int64_t> load(static_cast<size_t>(p.tp > 0 ? p.tp : 1), -7);
            fairkv_place_summary s{};
            const int rc = fairkv_place(W.data(), n, B, &p, shares.data(), cap, load.data(), &s);
            std::printf("place %d", rc);
            if (rc == FAIRKV_OK) {
                std::printf(" %lld %lld %lld %lld %d %d |", static_cast<long long>(s.den), static_cast<long long>(s.delta_num),
                            static_cast<long long>(s.max_load_num), static_cast<long long>(s.min_load_num), s.n_shares, s.exact);
                for (int i = 0; i < s.n_shares; ++i)
                    std::printf(" %d %d %d %d %d %d", shares[i].head, shares[i].gpu, shares[i].copy, shares[i].n_copies,
                                shares[i].row_begin, shares[i].row_end);
                std::printf(" |");
                for (int64_t x : load) std::printf(" %lld", static_cast<long long>(x));
            }
            std::printf("\n");
        } else if (cmd == "attn") {
            int B, Hq, Hkv, D;
            uint64_t seed;
            in >> B >> Hq >> Hkv >> D >> seed;
            if (!in || B < 1 || Hkv < 1 || B * Hkv > 4096) return 2;
            std::vector<int32_t> len(static_cast<size_t>(B) * Hkv);
            for (auto &x : len) in >> x;
            std::vector<int64_t> off(len.size());
            int64_t rows = 0;
            for (size_t i = 0; i < len.size(); ++i) {
                off[i] = rows;
                rows += len[i] > 0 ? len[i] : 0;
            }
            Lcg g{seed};
            // buffers of exactly the rows the heads own: a read past a head's last row of the last head is a report
            std::vector<double> q(static_cast<size_t>(B) * Hq * D), k(static_cast<size_t>(rows) * D), v(k.size());
            for (auto &x : q) x = g.next();
            for (auto &x : k) x = g.next();
            for (auto &x : v) x = g.next();
            std::vector<double> out(q.size()), lse(static_cast<size_t>(B) * Hq);
            const int rc = fairkv_oracle_attn(q.data(), k.data(), v.data(), off.data(), len.data(), B, Hq, Hkv, D, 2,
                                              1.0 / std::sqrt(static_cast<double>(D)), nullptr, 0, out.data(), lse.data(), 0);
            double so = 0.0, sl = 0.0;
            for (double x : out) so += x;
            for (double x : lse)
                if (std::isfinite(x)) sl += x;
            std::printf("attn %d %.17g %.17g\n", rc, so, sl);
        } else if (!cmd.empty()) {
            return 2;
        }
    }
    return 0;
}

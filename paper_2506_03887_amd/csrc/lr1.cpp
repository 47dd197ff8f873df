// Canonical LR(1) construction with kernel item sets and lookahead bitsets.
//
// A state is identified by its kernel (items with the dot not at the left end, plus the
// start item), each kernel item carrying the set of its lookaheads.  The closure is never
// materialised item by item: for every nonterminal B that appears right after a dot, all
// closure items [B -> . gamma, b] share one lookahead set la[B], found by propagating
// FIRST(beta a) contributions to a fixpoint (App. A.2, "Closure Operation").
#include "lr1.hpp"

#include <algorithm>
#include <array>
#include <cstring>
#include <map>
#include <string>
#include <unordered_map>

#include "../../include/pre3.h"

namespace pre3 {
namespace {

struct TermSet {                       // subset of the 257 terminals
    std::array<uint64_t, 5> w{};
    bool add_all(const TermSet &o) {
        bool grew = false;
        for (int i = 0; i < 5; ++i) {
            uint64_t n = w[i] | o.w[i];
            grew |= n != w[i];
            w[i] = n;
        }
        return grew;
    }
    void set(int t) { w[t >> 6] |= 1ull << (t & 63); }
    bool test(int t) const { return (w[t >> 6] >> (t & 63)) & 1; }
    bool empty() const { return !(w[0] | w[1] | w[2] | w[3] | w[4]); }
};

struct KernelItem {
    int64_t core;                      // dotted-rule index: core_of[prod] + dot (64-bit: no padding, items are hashed as raw bytes)
    TermSet la;
};

struct Builder {
    const Grammar &g;
    std::vector<int> core_of;          // production -> index of its dot-0 rule
    std::vector<int> core_prod, core_dot;
    std::vector<TermSet> tail_first;   // per dotted rule: FIRST(rhs[dot..])
    std::vector<char> tail_nullable;   // per dotted rule: rhs[dot..] =>* empty
    std::vector<TermSet> first;        // per nonterminal
    std::vector<char> nullable;

    explicit Builder(const Grammar &gr) : g(gr) {
        for (size_t p = 0; p < g.prods.size(); ++p) {
            core_of.push_back((int)core_prod.size());
            for (size_t d = 0; d <= g.prods[p].rhs.size(); ++d) {
                core_prod.push_back((int)p);
                core_dot.push_back((int)d);
            }
        }
        first_sets();
        tail_first.resize(core_prod.size());
        tail_nullable.resize(core_prod.size());
        for (size_t p = 0; p < g.prods.size(); ++p) {
            const auto &rhs = g.prods[p].rhs;
            TermSet acc;
            char nul = 1;
            for (int d = (int)rhs.size(); d >= 0; --d) {
                if (d < (int)rhs.size()) {
                    int x = rhs[d];
                    if (x < kNtBase) { acc = TermSet(); acc.set(x); nul = 0; }
                    else if (nullable[x - kNtBase]) { acc.add_all(first[x - kNtBase]); }
                    else { acc = first[x - kNtBase]; nul = 0; }
                }
                tail_first[core_of[p] + d] = acc;
                tail_nullable[core_of[p] + d] = nul;
            }
        }
    }

    void first_sets() {
        first.assign(g.n_nt(), TermSet());
        nullable.assign(g.n_nt(), 0);
        for (bool changed = true; changed;) {
            changed = false;
            for (const auto &p : g.prods) {
                bool all_null = true;
                for (int x : p.rhs) {
                    if (x < kNtBase) {
                        if (!first[p.lhs].test(x)) { first[p.lhs].set(x); changed = true; }
                        all_null = false;
                        break;
                    }
                    changed |= first[p.lhs].add_all(first[x - kNtBase]);
                    if (!nullable[x - kNtBase]) { all_null = false; break; }
                }
                if (all_null && !nullable[p.lhs]) { nullable[p.lhs] = 1; changed = true; }
            }
        }
    }

    // lookahead contribution of an item whose dot stands before a nonterminal:
    // FIRST(beta a) for every a in `la`, beta = the rule's tail after that nonterminal
    TermSet follow_of(int core_after, const TermSet &la) const {
        TermSet s = tail_first[core_after];
        if (tail_nullable[core_after]) s.add_all(la);
        return s;
    }
};

std::string kernel_key(const std::vector<KernelItem> &k) {
    std::string s(k.size() * sizeof(KernelItem), '\0');
    if (!k.empty()) std::memcpy(&s[0], k.data(), s.size());
    return s;
}

// Cycles with the reduction problem (Sec. 3.2.3): a production  A -> X1..Xn A  whose states
// v1 = GOTO(vn, X1), .., vn = GOTO(v(n-1), Xn) close a cycle.  Each traversal leaves v1..vn on the
// stack and all of them are popped, one traversal per reduction by that production, when the
// list ends.  Dropping one traversal from under a top v1 is sound when every kernel item of v1 is
// an A-item with the dot after its first symbol: the only reductions that look below v1 then
// expose exactly the entry under it and go to A.  In a conflict-free canonical automaton that
// alone implies that r = GOTO(vn, A) holds nothing but the finished  A -> X1..Xn A .  in its
// kernel and reduces on every lookahead a kernel item of v1 carries (all A-items of vn's closure
// share one lookahead set, the cycle's own item carries it round the path into r, and any other
// item of vn with A after the dot would add a second action in r on part of that set), so the
// next move pops the whole traversal and repeats the goto one traversal lower: both stacks
// reach the same configuration before the next byte is consumed.
void find_reduction_cycles(const Grammar &g, const Builder &B, const std::vector<std::vector<KernelItem>> &kernels,
                           Lr1Automaton &out) {
    const int n_nt = g.n_nt();
    auto step = [&](int s, int x) -> int {
        if (x >= kNtBase) return out.go[(size_t)s * n_nt + (x - kNtBase)];
        const uint32_t a = out.action[(size_t)s * kNumTerminals + x];
        return (a & 3u) == kShift ? (int)(a >> 2) : -1;
    };
    for (size_t p = 1; p < g.prods.size(); ++p) {
        const auto &rhs = g.prods[p].rhs;
        const int n = (int)rhs.size() - 1, A = g.prods[p].lhs;
        if (n < 1 || n > kMaxCycleStates || rhs[n] != kNtBase + A) continue;
        const int64_t before_tail = B.core_of[p] + n;
        for (int u = 0; u < out.n_states; ++u) {
            bool has = false;
            for (const KernelItem &it : kernels[u]) has |= it.core == before_tail;
            if (!has) continue;
            std::vector<int32_t> path;
            int v = u;
            for (int i = 0; i < n && v >= 0; ++i) {
                v = step(v, rhs[i]);
                path.push_back(v);
            }
            if (v != u) continue;
            bool ok = true;
            for (const KernelItem &it : kernels[path[0]])
                ok &= B.core_dot[it.core] == 1 && g.prods[B.core_prod[it.core]].lhs == A;
            if (step(u, kNtBase + A) < 0) continue;
            if (ok) out.cycles.push_back(path);
        }
    }
    std::sort(out.cycles.begin(), out.cycles.end(), [](const std::vector<int32_t> &a, const std::vector<int32_t> &b) {
        return a.size() != b.size() ? a.size() < b.size() : a < b;
    });
    out.cycles.erase(std::unique(out.cycles.begin(), out.cycles.end()), out.cycles.end());
}

}  // namespace

Lr1Automaton build_lr1(const Grammar &g) {
    static_assert(sizeof(KernelItem) == 48, "kernel items are hashed as raw bytes");
    Builder B(g);
    const int n_nt = g.n_nt();

    std::vector<std::vector<KernelItem>> kernels;
    std::unordered_map<std::string, int> ids;
    {
        KernelItem start{};
        start.core = B.core_of[0];
        start.la.set(kEnd);
        kernels.push_back({start});
        ids.emplace(kernel_key(kernels[0]), 0);
    }

    Lr1Automaton out;
    out.n_nt = n_nt;
    for (const auto &p : g.prods) {
        out.prod_lhs.push_back(p.lhs);
        out.prod_len.push_back((int)p.rhs.size());
    }

    std::vector<TermSet> la(n_nt);
    std::vector<char> in_closure(n_nt);
    std::vector<int> work;

    for (size_t s = 0; s < kernels.size(); ++s) {
        // ---- closure: lookahead set of the dot-0 items of every reachable nonterminal
        std::fill(la.begin(), la.end(), TermSet());
        std::fill(in_closure.begin(), in_closure.end(), 0);
        work.clear();
        auto contribute = [&](int nt, const TermSet &add) {
            bool grew = la[nt].add_all(add);
            if (!in_closure[nt] || grew) {
                if (!in_closure[nt]) in_closure[nt] = 1;
                work.push_back(nt);
            }
        };
        for (const KernelItem &it : kernels[s]) {
            const auto &rhs = g.prods[B.core_prod[it.core]].rhs;
            int d = B.core_dot[it.core];
            if (d < (int)rhs.size() && rhs[d] >= kNtBase)
                contribute(rhs[d] - kNtBase, B.follow_of(it.core + 1, it.la));
        }
        while (!work.empty()) {
            int nt = work.back();
            work.pop_back();
            for (int q : g.prods_of[nt]) {
                const auto &rhs = g.prods[q].rhs;
                if (!rhs.empty() && rhs[0] >= kNtBase)
                    contribute(rhs[0] - kNtBase, B.follow_of(B.core_of[q] + 1, la[nt]));
            }
        }

        // ---- GOTO kernels, grouped by the symbol after the dot (std::map keeps terminals in
        //      ascending byte order, then nonterminals by index)
        std::map<int, std::vector<KernelItem>> moves;
        // complete items of this state: (production, lookaheads)
        std::vector<std::pair<int, const TermSet *>> complete;
        for (const KernelItem &it : kernels[s]) {
            int p = B.core_prod[it.core], d = B.core_dot[it.core];
            const auto &rhs = g.prods[p].rhs;
            if (d < (int)rhs.size()) moves[rhs[d]].push_back({it.core + 1, it.la});
            else complete.push_back({p, &it.la});
        }
        for (int nt = 0; nt < n_nt; ++nt) {
            if (!in_closure[nt]) continue;
            for (int q : g.prods_of[nt]) {
                const auto &rhs = g.prods[q].rhs;
                if (rhs.empty()) complete.push_back({q, &la[nt]});
                else moves[rhs[0]].push_back({B.core_of[q] + 1, la[nt]});
            }
        }

        out.action.resize((s + 1) * kNumTerminals, 0);
        out.go.resize((s + 1) * n_nt, -1);
        uint32_t *row = &out.action[s * kNumTerminals];
        auto put = [&](int a, uint32_t v) {
            if (row[a] != 0 && row[a] != v) {
                static const char *names[] = {"error", "shift", "reduce", "accept"};
                throw CompileError{PRE3_E_NOT_LR1,
                                   std::string("grammar is not LR(1): ") + names[row[a] & 3] + "/" +
                                       names[v & 3] + " conflict in state " + std::to_string(s) +
                                       " on terminal " + std::to_string(a)};
            }
            row[a] = v;
        };

        for (const auto &c : complete)
            for (int a = 0; a < kNumTerminals; ++a)
                if (c.second->test(a))
                    put(a, c.first == 0 ? (uint32_t)kAccept : (kReduce | ((uint32_t)c.first << 2)));
        // new kernels are appended last: `complete` points into kernels[s]
        for (auto &mv : moves) {
            auto &kern = mv.second;
            std::sort(kern.begin(), kern.end(),
                      [](const KernelItem &a, const KernelItem &b) { return a.core < b.core; });
            auto ins = ids.emplace(kernel_key(kern), (int)kernels.size());
            if (ins.second) kernels.push_back(kern);
            int target = ins.first->second;
            if (mv.first < kNtBase) put(mv.first, kShift | ((uint32_t)target << 2));
            else out.go[s * n_nt + (mv.first - kNtBase)] = target;
        }
    }
    out.n_states = (int)kernels.size();
    find_reduction_cycles(g, B, kernels, out);
    return out;
}

}  // namespace pre3

// Builds the per-symbol reduction edges with stack-matching conditions (see symbol_edges.hpp).
#include "symbol_edges.hpp"

#include <algorithm>
#include <deque>
#include <memory>

namespace pre3 {

namespace {

struct Pending {        // a symbol whose chain reached below the known stack entries
    int col;
    int need;           // the exposed state lies `need` entries below the deepest known one
    int nt;             // nonterminal pushed from it
    int rel;            // stack height after the pending pop, relative to the height before the symbol
    int peak;           // largest relative height seen just before a push so far
};

struct BuildNode {
    int known = 1;
    int floor = 0;
    std::vector<int32_t> suffix;                // the known entries, deepest first (suffix.back() = top state)
    std::vector<int32_t> eff;                   // per column: code or offset into the pool
    std::vector<Pending> pend;
    std::vector<std::pair<int32_t, std::unique_ptr<BuildNode>>> children;
};

struct Builder {
    const EdgeTables &T;
    const std::vector<std::vector<int32_t>> pred;
    const int ncol;
    const int max_known;
    int node_budget;
    std::vector<int32_t> pool;
    int64_t deepest = 0;

    Builder(const EdgeTables &t, int mk, int budget)
        : T(t), pred(predecessors(t)), ncol(t.n_classes + 1), max_known(mk), node_budget(budget) {}

    int goto_of(int state, int nt) const {
        int row = T.goto_row[state];
        return row < 0 ? -1 : T.goto_flat[row + nt];
    }

    // Runs the chain of column `col` on st (st[0] = deepest known state) and records the outcome.
    void run(BuildNode &nd, int col, std::vector<int32_t> &st, int rel, int peak) {
        for (;;) {
            uint32_t e = T.edge[(size_t)st.back() * ncol + col];
            uint32_t kind = e & kKindMask;
            if (kind == kError) { nd.eff[col] = kEffNone; return; }
            if (kind == kAccept) { nd.eff[col] = kEffAccept; return; }
            if (kind == kShift) {
                peak = std::max(peak, rel);
                st.push_back((int32_t)(e >> 2));
                while (pool.size() & 3) pool.push_back(0);          // records start on 16-byte boundaries
                nd.eff[col] = (int32_t)pool.size();
                // Self-similar edge: the stack keeps its height and all known entries except the top,
                // and the new top is of the same kind as the old one.  The next symbol then meets the
                // same condition node, which lets a run of such symbols be applied in one go.
                bool same_shape = st.size() == nd.suffix.size() &&
                                  T.state_kind[st.back()] == T.state_kind[nd.suffix.back()];
                for (size_t i = 1; same_shape && i + 1 < st.size(); ++i) same_shape = st[i] == nd.suffix[i];
                // Growing edge (right-recursive lists, one element per symbol): the node knows the top
                // and the entry x under it; the edge replaces the top by a second x and a new top of
                // the same kind.  The next symbol meets the same node again, so a run of such symbols
                // inserts one x each and replaces the top.
                const bool grow = nd.suffix.size() == 2 && st.size() == 3 && st[1] == st[0] &&
                                  T.state_kind[st.back()] == T.state_kind[nd.suffix.back()];
                pool.push_back(nd.known);
                pool.push_back(peak);
                pool.push_back(((int32_t)st.size() - 1) | (same_shape ? kEffSameShape : 0) | (grow ? kEffGrow : 0));
                pool.push_back(T.state_kind[st.back()]);
                pool.insert(pool.end(), st.begin() + 1, st.end());
                deepest = std::max<int64_t>(deepest, nd.known);
                return;
            }
            int n = (int)((e >> 2) & kMaxPop), nt = (int)(e >> kNtShift);
            rel -= n;
            if (n > (int)st.size() - 1) {
                nd.eff[col] = kEffDeeper;
                nd.pend.push_back({col, n - ((int)st.size() - 1), nt, rel, peak});
                return;
            }
            st.resize(st.size() - n);
            int t = goto_of(st.back(), nt);
            if (t < 0) { nd.eff[col] = kEffNone; return; }
            peak = std::max(peak, rel);
            st.push_back(t);
            ++rel;
        }
    }

    void resolve(int X, const std::vector<Pending> &in, BuildNode &out) {
        std::vector<int32_t> st;
        for (const Pending &u : in) {
            if (u.need > 1) {
                out.eff[u.col] = kEffDeeper;
                out.pend.push_back({u.col, u.need - 1, u.nt, u.rel, u.peak});
                continue;
            }
            int t = goto_of(X, u.nt);
            if (t < 0) { out.eff[u.col] = kEffNone; continue; }
            st.assign(1, X);
            st.push_back(t);
            run(out, u.col, st, u.rel + 1, std::max(u.peak, u.rel));
        }
    }

    void give_up(BuildNode &nd) {
        for (const Pending &u : nd.pend) nd.eff[u.col] = kEffStepwise;
        nd.pend.clear();
    }

    // Grows the tree under `root` breadth first: the node budget then cuts the deepest conditions
    // (right-recursive lists unroll without end) and never a shallow one that many stacks meet.
    void expand(BuildNode &root) {
        std::deque<BuildNode *> queue(1, &root);
        while (!queue.empty()) {
            BuildNode &nd = *queue.front();
            queue.pop_front();
            while (!nd.pend.empty()) {
                const std::vector<int32_t> &ps = pred[nd.floor];
                if (ps.empty()) {                               // the bottom of a stack is never popped
                    for (const Pending &u : nd.pend) nd.eff[u.col] = kEffNone;
                    nd.pend.clear();
                    break;
                }
                if (nd.known >= max_known) { give_up(nd); break; }
                if (ps.size() == 1) {                           // only one state can lie below: no test needed
                    std::vector<Pending> in;
                    in.swap(nd.pend);
                    nd.floor = ps[0];
                    nd.known++;
                    nd.suffix.insert(nd.suffix.begin(), ps[0]);
                    resolve(ps[0], in, nd);
                    continue;
                }
                if (node_budget < (int)ps.size()) { give_up(nd); break; }
                node_budget -= (int)ps.size();
                for (int X : ps) {
                    std::unique_ptr<BuildNode> ch(new BuildNode());
                    ch->known = nd.known + 1;
                    ch->floor = X;
                    ch->suffix = nd.suffix;
                    ch->suffix.insert(ch->suffix.begin(), X);
                    ch->eff.assign(ncol, kEffNone);
                    resolve(X, nd.pend, *ch);
                    queue.push_back(ch.get());
                    nd.children.emplace_back(X, std::move(ch));
                }
                nd.pend.clear();
            }
        }
    }
};

// children first get consecutive indices after all roots, breadth first per root
void flatten(const BuildNode &b, int idx, SymbolEdges &S, int ncol) {
    std::vector<std::pair<int32_t, const BuildNode *>> kids;
    for (const auto &ch : b.children) kids.push_back({ch.first, ch.second.get()});
    std::sort(kids.begin(), kids.end(), [](const auto &a, const auto &c) { return a.first < c.first; });
    // the children get consecutive node indices, so child j is node first_child + j
    SymbolNode n{b.known, (int32_t)S.child_state.size(), (int32_t)kids.size(), (int32_t)S.nodes.size()};
    std::vector<int> kid_idx;
    for (auto &k : kids) {
        kid_idx.push_back((int)S.nodes.size());
        S.nodes.push_back(SymbolNode{});
        S.eff.resize(S.nodes.size() * (size_t)ncol, kEffNone);
        S.child_state.push_back(k.first);
        S.child_node.push_back(kid_idx.back());
    }
    S.nodes[idx] = n;
    std::copy(b.eff.begin(), b.eff.end(), S.eff.begin() + (size_t)idx * ncol);
    for (size_t i = 0; i < kids.size(); ++i) flatten(*kids[i].second, kid_idx[i], S, ncol);
}

}  // namespace

std::vector<std::vector<int32_t>> predecessors(const EdgeTables &T) {
    std::vector<std::vector<int32_t>> pred(T.n_states);
    for (int g = 0; g < T.n_grammars; ++g) {
        const Lr1Automaton &A = T.automata[g];
        const int off = T.state_offset[g];
        for (int s = 0; s < A.n_states; ++s) {
            for (int a = 0; a < 256; ++a) {
                uint32_t act = A.action[(size_t)s * kNumTerminals + a];
                if ((act & 3u) == kShift) pred[off + (act >> 2)].push_back(off + s);
            }
            for (int nt = 0; nt < A.n_nt; ++nt) {
                int t = A.go[(size_t)s * A.n_nt + nt];
                if (t >= 0) pred[off + t].push_back(off + s);
            }
        }
    }
    for (auto &p : pred) {
        std::sort(p.begin(), p.end());
        p.erase(std::unique(p.begin(), p.end()), p.end());
    }
    return pred;
}

SymbolEdges build_symbol_edges(const EdgeTables &T, int max_known, int max_nodes) {
    SymbolEdges S;
    S.enabled = true;
    S.ncol = T.n_classes + 1;
    Builder B(T, max_known, 0);
    int remaining = max_nodes;
    S.nodes.assign(T.n_kinds, SymbolNode{});
    S.eff.assign((size_t)T.n_kinds * S.ncol, kEffNone);
    std::vector<int32_t> st;
    std::vector<char> done(T.n_kinds, 0);
    for (int s = 0; s < T.n_states; ++s) {
        const int kind = T.state_kind[s];
        if (done[kind]) continue;                               // one tree per kind, built from its first state
        done[kind] = 1;
        BuildNode root;
        root.known = 1;
        root.floor = s;
        root.suffix.assign(1, s);
        root.eff.assign(S.ncol, kEffNone);
        for (int col = 0; col < S.ncol; ++col) {
            st.assign(1, s);
            B.run(root, col, st, 0, -(1 << 30));
        }
        B.node_budget = std::min(remaining, 512);               // per-state share of the node budget
        const int granted = B.node_budget;
        B.expand(root);
        remaining -= granted - B.node_budget;
        flatten(root, kind, S, S.ncol);
    }
    while (B.pool.size() & 3) B.pool.push_back(0);
    B.pool.insert(B.pool.end(), 8, 0);                          // a record is read as two 16-byte halves
    S.pool.swap(B.pool);
    S.max_known = B.deepest;
    return S;
}

int host_feed(const EdgeTables &T, const SymbolEdges &S, std::vector<int32_t> &st, int col, int delta, int cap,
              bool use_merged) {
    const int ncol = T.n_classes + 1;
    int node = T.state_kind[st.back()];
    while (use_merged) {
        int code = S.eff[(size_t)node * ncol + col];
        if (code == kEffNone) return kHostRejected;
        if (code == kEffAccept) return kHostAccepted;
        if (code == kEffStepwise) break;
        if (code >= 0) {
            const int32_t *rec = &S.pool[code];
            int known = rec[0], peak = rec[1], np = rec[2] & kEffPushMask;
            if ((int)st.size() + peak >= cap) return kHostOverflow;
            st.resize(st.size() - (known - 1));
            for (int i = 0; i < np; ++i) st.push_back(rec[4 + i] + (i == np - 1 ? delta : 0));
            return kHostFed;
        }
        const SymbolNode &nd = S.nodes[node];
        if (nd.known >= (int)st.size()) break;
        int x = st[st.size() - 1 - nd.known], next = -1;
        for (int i = 0; i < nd.child_count; ++i)
            if (S.child_state[nd.child_begin + i] == x) next = S.child_node[nd.child_begin + i];
        if (next < 0) break;
        node = next;
    }
    for (;;) {                                                  // per-step edges
        uint32_t e = T.edge[(size_t)st.back() * ncol + col];
        uint32_t kind = e & kKindMask;
        if (kind == kError) return kHostRejected;
        if (kind == kAccept) return kHostAccepted;
        if (kind == kShift) {
            if ((int)st.size() >= cap) return kHostOverflow;
            st.push_back((int32_t)(e >> 2) + delta);
            return kHostFed;
        }
        int n = (int)((e >> 2) & kMaxPop), nt = (int)(e >> kNtShift);
        if ((int)st.size() - n >= cap) return kHostOverflow;
        if (n >= (int)st.size()) return kHostRejected;
        st.resize(st.size() - n);
        int row = T.goto_row[st.back()];
        int t = row < 0 ? -1 : T.goto_flat[row + nt];
        if (t < 0) return kHostRejected;
        st.push_back(t);
    }
}

}  // namespace pre3

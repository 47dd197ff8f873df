// Builds the condition tree of token-level prefix-conditioned edges (see token_edges.hpp).
#include "token_edges.hpp"

#include <algorithm>
#include <atomic>
#include <cstring>
#include <deque>
#include <map>
#include <exception>
#include <memory>
#include <mutex>
#include <numeric>
#include <thread>
#include <unordered_map>

namespace pre3 {

namespace {

// ------------------------------------------------------------------ vocabulary trie
struct Trie {
    struct Node {
        int32_t first_child = 0, n_children = 0;
        int32_t tok_begin = 0, tok_count = 0;   // token ids that end here
        int32_t col = 0, delta = 0;             // byte class column and target offset of the edge label
        int32_t sub_tokens = 0;                 // tokens in the whole subtree
    };
    std::vector<Node> nodes;                    // nodes[0] = root; nodes[1] = the end-of-input pseudo token
    std::vector<int32_t> tok_ids;
};

struct TrieBuilder {
    const EdgeTables &T;
    const VocabLayout &V;
    Trie trie;
    std::vector<int32_t> order;                 // token ids sorted by byte string

    const uint8_t *str(int t) const { return V.bytes.data() + V.offsets[t]; }
    int len(int t) const { return V.offsets[t + 1] - V.offsets[t]; }

    TrieBuilder(const EdgeTables &t, const VocabLayout &v) : T(t), V(v) {
        for (int t2 = 0; t2 < V.n_tokens; ++t2)
            if (t2 != V.eos_id && len(t2) > 0) order.push_back(t2);
        std::sort(order.begin(), order.end(), [&](int a, int b) {
            int la = len(a), lb = len(b);
            int r = std::memcmp(str(a), str(b), std::min(la, lb));
            if (r != 0) return r < 0;
            if (la != lb) return la < lb;
            return a < b;
        });
        trie.nodes.resize(2);
        // pseudo token: the single symbol '$', carried by the end-of-sequence token id
        trie.nodes[1].col = T.n_classes;
        trie.nodes[1].tok_begin = 0;
        trie.nodes[1].tok_count = 1;
        trie.nodes[1].sub_tokens = 1;
        trie.tok_ids.push_back(V.eos_id);
        build(0, 0, (int)order.size(), 0);
    }

    // tokens order[lo..hi) share their first `depth` bytes and belong below `node`
    void build(int node, int lo, int hi, int depth) {
        int p = lo;
        trie.nodes[node].tok_begin = (int)trie.tok_ids.size();
        while (p < hi && len(order[p]) == depth) trie.tok_ids.push_back(order[p++]);
        trie.nodes[node].tok_count = p - lo;
        trie.nodes[node].sub_tokens = hi - lo;
        std::vector<std::pair<int, int>> groups;        // [begin, end) per next byte
        while (p < hi) {
            int b = str(order[p])[depth], q = p;
            while (q < hi && str(order[q])[depth] == b) ++q;
            groups.push_back({p, q});
            p = q;
        }
        int first = (int)trie.nodes.size();
        trie.nodes[node].first_child = first;
        trie.nodes[node].n_children = (int)groups.size();
        trie.nodes.resize(first + groups.size());
        for (size_t i = 0; i < groups.size(); ++i) {
            int b = str(order[groups[i].first])[depth];
            trie.nodes[first + i].col = T.byte_class[b];
            trie.nodes[first + i].delta = T.byte_delta[b];
        }
        for (size_t i = 0; i < groups.size(); ++i) build(first + (int)i, groups[i].first, groups[i].second, depth + 1);
    }
};

// ------------------------------------------------------------- walking on a known suffix
enum FeedKind { kFedH, kRejectedH, kAcceptedH, kUnderflowH };
struct FeedOut {
    FeedKind kind;
    int need;       // kUnderflowH: the exposed state lies `need` entries below the deepest known one
    int nt;         // ... and this nonterminal is pushed from it
};

struct Pending {    // a trie subtree whose verdict depends on stack entries not known yet
    int32_t trie_node;
    int32_t need;
    int32_t nt;
    int32_t peak;   // highest the stack has been before a push so far in this token's walk (kNoPeak: no push yet)
};
constexpr int kNoPeak = -(1 << 24);

struct EffectBudget {   // shared by the workers: records written so far, and the switch that ends recording
    std::atomic<int64_t> records{0};
    std::atomic<bool> exceeded{false};
};

struct BuildNode {
    int known = 1;
    int floor = 0;                              // deepest known state
    std::vector<int32_t> accepted;              // token ids allowed under this node's condition
    std::vector<int32_t> eff;                   // their stack effects: token, k, peak, n_push, pushes (longer tokens only)
    std::vector<Pending> pend;
    std::vector<int32_t> path;                  // known states, top first (kept until the node is expanded)
    std::vector<std::pair<int32_t, std::unique_ptr<BuildNode>>> children;
};

struct Walker {
    const EdgeTables &T;
    const Trie &trie;
    const std::vector<std::vector<int32_t>> &pred;
    const TokenEdgeLimits &lim;
    const int ncol;
    std::vector<std::vector<int32_t>> pool;     // one scratch stack per trie depth
    const std::vector<int32_t> &tok_len;        // bytes of each token
    EffectBudget &budget;

    Walker(const EdgeTables &t, const Trie &tr, const std::vector<std::vector<int32_t>> &p,
           const TokenEdgeLimits &l, const std::vector<int32_t> &tl, EffectBudget &bud)
        : T(t), trie(tr), pred(p), lim(l), ncol(t.n_classes + 1), pool(300), tok_len(tl), budget(bud) {}

    int goto_of(int state, int nt) const {
        int row = T.goto_row[state];
        return row < 0 ? -1 : T.goto_flat[row + nt];
    }

    // st[0] is the deepest known state, the entry k - 1 below the top of the stack the walk started
    // from; consumes one symbol.  peak follows the height of the stack just before each push,
    // relative to the height before the token: st holds the entries from st[0] up, so that is |st| - k.
    FeedOut feed(std::vector<int32_t> &st, int col, int delta, int k, int &peak) const {
        for (;;) {
            uint32_t e = T.edge[(size_t)st.back() * ncol + col];
            switch (e & kKindMask) {
                case kError: return {kRejectedH, 0, 0};
                case kAccept: return {kAcceptedH, 0, 0};
                case kShift:
                    peak = std::max(peak, (int)st.size() - k);
                    st.push_back((int32_t)(e >> 2) + delta);
                    return {kFedH, 0, 0};
                default: break;
            }
            int n = (int)((e >> 2) & kMaxPop), nt = (int)(e >> kNtShift);
            if (n > (int)st.size() - 1) return {kUnderflowH, n - ((int)st.size() - 1), nt};
            st.resize(st.size() - n);
            int t = goto_of(st.back(), nt);
            if (t < 0) return {kRejectedH, 0, 0};
            peak = std::max(peak, (int)st.size() - k);
            st.push_back(t);
        }
    }

    // The stack operations of the merged edge of token `tok`, whose walk has just ended on `st`.
    void record_effect(BuildNode &out, int32_t tok, const std::vector<int32_t> &st, int k, int peak) {
        const int np = (int)st.size() - 1;
        if (lim.effect_min_len <= 0 || tok_len[tok] < lim.effect_min_len || budget.exceeded.load(std::memory_order_relaxed)) return;
        if (np < 1 || np > 255 || k > 255 || peak < -32768 || peak > 32767 || tok >= (1 << 21)) return;    // such a token keeps its byte-by-byte walk
        if (budget.records.fetch_add(1, std::memory_order_relaxed) >= lim.max_effect_records) {
            budget.exceeded.store(true, std::memory_order_relaxed);
            return;
        }
        out.eff.push_back(tok);
        out.eff.push_back(k);
        out.eff.push_back(peak);
        out.eff.push_back(np);
        out.eff.insert(out.eff.end(), st.begin() + 1, st.end());
    }

    // The edge into trie node `c` is fed from `st`; on success the subtree below is explored.
    void enter(int c, std::vector<int32_t> &st, int depth, BuildNode &out, int k, int peak) {
        const Trie::Node &N = trie.nodes[c];
        FeedOut r = feed(st, N.col, N.delta, k, peak);
        if (r.kind == kUnderflowH) { out.pend.push_back({c, r.need, r.nt, peak}); return; }
        if (r.kind == kRejectedH) return;
        // shifted (or, for the end-of-input pseudo token, accepted)
        for (int i = 0; i < N.tok_count; ++i) {
            const int32_t tok = trie.tok_ids[N.tok_begin + i];
            out.accepted.push_back(tok);
            if (r.kind == kFedH) record_effect(out, tok, st, k, peak);
        }
        if (r.kind == kAcceptedH) return;
        for (int i = 0; i < N.n_children; ++i) {
            std::vector<int32_t> &st2 = pool[depth + 1];
            st2 = st;
            enter(N.first_child + i, st2, depth + 1, out, k, peak);
        }
    }

    void walk_root(int state, BuildNode &out) {
        out.known = 1;
        out.floor = state;
        const Trie::Node &R = trie.nodes[0];
        std::vector<int32_t> &st = pool[0];
        st.assign(1, state);
        enter(1, st, 0, out, 1, kNoPeak);                       // '$'
        for (int i = 0; i < R.n_children; ++i) {
            st.assign(1, state);
            enter(R.first_child + i, st, 0, out, 1, kNoPeak);
        }
    }

    // One more stack entry X becomes known below the node that owned `in`: X is the entry k - 1 below the top.
    void resolve(int X, const std::vector<Pending> &in, BuildNode &out, int k) {
        for (const Pending &u : in) {
            if (u.need > 1) { out.pend.push_back({u.trie_node, u.need - 1, u.nt, u.peak}); continue; }
            int t = goto_of(X, u.nt);
            if (t < 0) continue;
            std::vector<int32_t> &st = pool[0];
            st.clear();
            st.push_back(X);
            st.push_back(t);                                    // pushed onto a stack cut down to X: height 1 - k before
            enter(u.trie_node, st, 0, out, k, std::max(u.peak, 1 - k));
        }
    }

    // With cycle-aware stacks no stack holds a complete traversal v1..vn of a reduction cycle right
    // below another v1: a condition state X that would complete one under the known entries cannot
    // occur, so its subtree is not built (a stack that was never compacted finds no child there and
    // falls back to the walk).  path = the known states, top first.
    bool excluded_by_compaction(const std::vector<int32_t> &path, int X) const {
        if (!lim.compacted_stacks) return false;
        const int size = (int)path.size();
        for (int at = T.cycle_head[X]; at >= 0; at = T.cycle_pool[at + 1]) {
            const int n = T.cycle_pool[at];
            if (size < n || path[size - n] != X) continue;
            bool same = true;
            for (int i = 1; i < n && same; ++i) same = path[size - i] == T.cycle_pool[at + 2 + i];
            if (same) return true;
        }
        return false;
    }

    // Expands the nodes waiting in `queue` breadth first until the queue is empty or `budget` nodes
    // have been created: the tree of one root grows level by level, so when the budget cuts it, it
    // cuts the deepest conditions (tokens that need them are left to the run-time walk) and never
    // a shallow one.  Returns the nodes created; a node that did not fit stays at the queue's head.
    int expand(std::deque<BuildNode *> &queue, int budget) {
        int used = 0;
        while (!queue.empty()) {
            BuildNode &nd = *queue.front();
            bool wait = false;
            while (!nd.pend.empty()) {
                const std::vector<int32_t> &ps = pred[nd.floor];
                if (ps.empty()) { nd.pend.clear(); break; }        // the bottom of a stack is never popped
                if (nd.known >= lim.max_known) break;               // left to the run-time walk
                if (ps.size() == 1) {                               // only one stack can lie below: no test needed
                    std::vector<Pending> in;
                    in.swap(nd.pend);
                    resolve(ps[0], in, nd, nd.known + 1);
                    nd.floor = ps[0];
                    nd.known++;
                    nd.path.push_back(ps[0]);
                    continue;
                }
                if (used + (int)ps.size() > budget) { wait = true; break; }
                used += (int)ps.size();
                for (int X : ps) {
                    if (excluded_by_compaction(nd.path, X)) continue;
                    std::unique_ptr<BuildNode> ch(new BuildNode());
                    ch->known = nd.known + 1;
                    ch->floor = X;
                    ch->path = nd.path;
                    ch->path.push_back(X);
                    resolve(X, nd.pend, *ch, ch->known);
                    queue.push_back(ch.get());
                    nd.children.emplace_back(X, std::move(ch));
                }
                nd.pend.clear();
                std::vector<int32_t>().swap(nd.path);               // only unexpanded nodes need theirs
                break;
            }
            if (wait) break;
            queue.pop_front();
        }
        return used;
    }
};

// ----------------------------------------------------------------------- flattening
struct Flattener {
    const Trie &trie;
    const TokenEdgeLimits &lim;
    TokenEdges &E;
    int dense_threshold;
    bool record_effects;

    void subtree_tokens(int c, std::vector<int32_t> &out) const {
        const Trie::Node &N = trie.nodes[c];
        for (int i = 0; i < N.tok_count; ++i) out.push_back(trie.tok_ids[N.tok_begin + i]);
        for (int i = 0; i < N.n_children; ++i) subtree_tokens(N.first_child + i, out);
    }

    // ---- materialised rows, each stored once.  A row is the base row plus tokens that are not in
    // it (a node only lists tokens no ancestor allows), so its content hash -- the sum of a mixed
    // value per token -- and its population follow from the base's in O(new tokens); a candidate with
    // the same hash is then verified exactly: same population, every new token present, and a
    // superset of the base (that last test is memoised per pair of rows).
    std::vector<uint64_t> row_hash;
    std::vector<int64_t> row_pop;
    std::unordered_multimap<uint64_t, int> row_index;
    std::unordered_map<uint64_t, bool> superset_memo;
    std::vector<uint32_t> seen;              // scratch bitmap, all zero between calls
    std::vector<int32_t> fresh_scratch;

    static uint64_t mix(uint64_t x) {
        x += 0x9E3779B97F4A7C15ull;
        x = (x ^ (x >> 30)) * 0xBF58476D1CE4E5B9ull;
        x = (x ^ (x >> 27)) * 0x94D049BB133111EBull;
        return x ^ (x >> 31);
    }

    bool is_superset(int cand, int base) {
        if (base < 0) return true;
        const uint64_t key = ((uint64_t)(uint32_t)cand << 32) | (uint32_t)base;
        auto it = superset_memo.find(key);
        if (it != superset_memo.end()) return it->second;
        const uint32_t *c = &E.dense_rows[(size_t)cand * E.n_words], *b = &E.dense_rows[(size_t)base * E.n_words];
        bool ok = true;
        for (int w = 0; w < E.n_words && ok; ++w) ok = (c[w] & b[w]) == b[w];
        superset_memo.emplace(key, ok);
        return ok;
    }

    // Index of the row  base + ids_a + ids_b.
    int row_of(int base, const std::vector<int32_t> &ids_a, const std::vector<int32_t> &ids_b) {
        auto has = [&](int row, int32_t t) { return (E.dense_rows[(size_t)row * E.n_words + (t >> 5)] >> (t & 31)) & 1u; };
        // the tokens that are really new (by construction all of them; made exact here because the
        // verification below counts on it)
        std::vector<int32_t> &fresh = fresh_scratch;
        fresh.clear();
        if (seen.empty()) seen.assign(E.n_words, 0);
        for (const std::vector<int32_t> *ids : {&ids_a, &ids_b})
            for (int32_t t : *ids) {
                if ((base >= 0 && has(base, t)) || ((seen[t >> 5] >> (t & 31)) & 1u)) continue;
                seen[t >> 5] |= 1u << (t & 31);
                fresh.push_back(t);
            }
        for (int32_t t : fresh) seen[t >> 5] = 0;
        if (fresh.empty() && base >= 0) return base;
        uint64_t h = base >= 0 ? row_hash[base] : 0;
        for (int32_t t : fresh) h += mix((uint64_t)t);
        const int64_t pop = (base >= 0 ? row_pop[base] : 0) + (int64_t)fresh.size();
        auto range = row_index.equal_range(h);
        for (auto it = range.first; it != range.second; ++it) {
            const int cand = it->second;
            if (row_pop[cand] != pop) continue;           // same size, contains base and the new tokens: equal
            bool ok = true;
            for (size_t i = 0; i < fresh.size() && ok; ++i) ok = has(cand, fresh[i]);
            if (ok && is_superset(cand, base)) return cand;
        }
        const int row = (int)(E.dense_rows.size() / E.n_words);
        E.dense_rows.resize(E.dense_rows.size() + E.n_words, 0);          // may move the rows: take pointers after it
        uint32_t *dst = &E.dense_rows[(size_t)row * E.n_words];
        if (base >= 0) std::memcpy(dst, &E.dense_rows[(size_t)base * E.n_words], sizeof(uint32_t) * E.n_words);
        for (int32_t t : fresh) dst[t >> 5] |= 1u << (t & 31);
        row_hash.push_back(h);
        row_pop.push_back(pop);
        row_index.emplace(h, row);
        E.n_dense++;
        return row;
    }

    // multiplicative hash over 4-byte words (every hashed object here is an array of int32/uint32)
    static uint64_t fnv(const void *data, size_t bytes, uint64_t h = 1469598103934665603ull) {
        const uint32_t *p = static_cast<const uint32_t *>(data);
        for (size_t i = 0; i < bytes / 4; ++i) h = (h ^ p[i]) * 1099511628211ull;
        return h;
    }

    // Appends `ids` to `pool` unless the same list is already there; returns where it starts.
    static int32_t intern_list(std::vector<int32_t> &pool, std::unordered_multimap<uint64_t, std::pair<int32_t, int32_t>> &index,
                               const std::vector<int32_t> &ids) {
        if (ids.empty()) return 0;
        const uint64_t h = fnv(ids.data(), ids.size() * sizeof(int32_t));
        auto range = index.equal_range(h);
        for (auto it = range.first; it != range.second; ++it)
            if (it->second.second == (int32_t)ids.size() &&
                std::memcmp(&pool[it->second.first], ids.data(), ids.size() * sizeof(int32_t)) == 0)
                return it->second.first;
        const int32_t begin = (int32_t)pool.size();
        pool.insert(pool.end(), ids.begin(), ids.end());
        index.emplace(h, std::make_pair(begin, (int32_t)ids.size()));
        return begin;
    }

    std::unordered_multimap<uint64_t, std::pair<int32_t, int32_t>> delta_index, walk_index, effect_index;
    // hash of a group of sibling records (with their condition states) -> (child_begin, count)
    std::unordered_multimap<uint64_t, std::pair<int32_t, int32_t>> group_index;

    // Stores a group of sibling nodes (records `recs`, told apart by `states`, ascending) unless an
    // identical group exists: equal subtrees under different parents share one copy, which turns the
    // trees into a DAG.  Returns the group's start in child_state / child_node; its nodes are
    // consecutive, beginning at child_node[start].
    int32_t intern_group(const std::vector<int32_t> &states, const std::vector<ConditionNode> &recs) {
        uint64_t h = fnv(states.data(), states.size() * sizeof(int32_t));
        h = fnv(recs.data(), recs.size() * sizeof(ConditionNode), h);
        auto range = group_index.equal_range(h);
        for (auto it = range.first; it != range.second; ++it) {
            const int32_t begin = it->second.first;
            if (it->second.second != (int32_t)states.size()) continue;
            if (std::memcmp(&E.child_state[begin], states.data(), states.size() * sizeof(int32_t)) != 0) continue;
            if (std::memcmp(&E.nodes[E.child_node[begin]], recs.data(), recs.size() * sizeof(ConditionNode)) == 0) return begin;
        }
        const int32_t begin = (int32_t)E.child_state.size(), first = (int32_t)E.nodes.size();
        for (size_t j = 0; j < states.size(); ++j) {
            E.child_state.push_back(states[j]);
            E.child_node.push_back(first + (int32_t)j);
        }
        E.nodes.insert(E.nodes.end(), recs.begin(), recs.end());
        group_index.emplace(h, std::make_pair(begin, (int32_t)states.size()));
        return begin;
    }

    // `base` = dense row of the nearest dense ancestor (or -1), `since` = ids accepted after it.
    // Returns the node's record; its children (and theirs) have been stored by then, consecutively
    // and in the order of their condition states, so that child j is node first_child + j.
    ConditionNode flatten(const BuildNode &b, int base, std::vector<int32_t> &since) {
        ConditionNode n{};
        n.known = b.known;
        n.dense_row = -1;
        E.max_known = std::max<int64_t>(E.max_known, b.known);
        size_t since_mark = since.size();
        // a row is materialised where the ids allowed since the last materialised row reach the
        // threshold (1 by default: wherever a node allows a token of its own), so that a descent
        // collects fewer than `dense_threshold` ids to OR in
        const bool dense = (int64_t)(since.size() + b.accepted.size()) >= dense_threshold &&
                           (int64_t)E.dense_rows.size() + E.n_words <= lim.max_dense_words;
        int own_row = base;
        if (dense) {
            own_row = row_of(base, since, b.accepted);
            n.dense_row = own_row;
        } else {
            n.delta_count = (int)b.accepted.size();
            n.delta_begin = intern_list(E.delta_ids, delta_index, b.accepted);
            since.insert(since.end(), b.accepted.begin(), b.accepted.end());
        }
        if (record_effects && !b.eff.empty()) {
            n.effect_words = (int)b.eff.size();
            n.effect_begin = intern_list(E.effects, effect_index, b.eff);
        }
        // tokens left undetermined when the tree ends here
        if (b.children.empty() && !b.pend.empty()) {
            int64_t total = 0;
            for (const Pending &u : b.pend) total += trie.nodes[u.trie_node].sub_tokens;
            if (total > lim.max_walk) {
                n.walk_count = -1;
            } else {
                std::vector<int32_t> ids;
                for (const Pending &u : b.pend) subtree_tokens(u.trie_node, ids);
                n.walk_count = (int)ids.size();
                n.walk_begin = intern_list(E.walk_ids, walk_index, ids);
            }
        }
        std::vector<std::pair<int32_t, const BuildNode *>> kids;
        for (const auto &ch : b.children) kids.push_back({ch.first, ch.second.get()});
        std::sort(kids.begin(), kids.end(), [](const auto &x, const auto &y) { return x.first < y.first; });
        std::vector<int32_t> states;
        std::vector<ConditionNode> recs;
        std::vector<int32_t> empty_since;
        for (const auto &kid : kids) {
            states.push_back(kid.first);
            if (dense) {
                empty_since.clear();
                recs.push_back(flatten(*kid.second, own_row, empty_since));
            } else {
                recs.push_back(flatten(*kid.second, base, since));
            }
        }
        n.child_count = (int)kids.size();
        n.child_begin = kids.empty() ? 0 : intern_group(states, recs);
        since.resize(since_mark);
        return n;
    }
};

}  // namespace

TokenEdges build_token_edges(const EdgeTables &T, const VocabLayout &V, const TokenEdgeLimits &lim) {
    TokenEdges E;
    E.enabled = true;
    E.n_words = V.n_words;
    TrieBuilder tb(T, V);
    const Trie &trie = tb.trie;
    const int ncol = T.n_classes + 1;

    const std::vector<std::vector<int32_t>> pred = predecessors(T);
    std::vector<int32_t> tok_len(V.n_tokens);
    for (int t = 0; t < V.n_tokens; ++t) tok_len[t] = V.offsets[t + 1] - V.offsets[t];
    EffectBudget budget;

    // states with identical edges, goto row and predecessors share one root
    std::map<std::tuple<std::vector<uint32_t>, int32_t, std::vector<int32_t>>, int> root_ids;
    std::vector<int> root_state;
    std::vector<int> root_index(T.n_states);
    for (int s = 0; s < T.n_states; ++s) {
        std::vector<uint32_t> row(T.edge.begin() + (size_t)s * ncol, T.edge.begin() + (size_t)(s + 1) * ncol);
        auto ins = root_ids.emplace(std::make_tuple(std::move(row), T.goto_row[s], pred[s]), (int)root_state.size());
        if (ins.second) root_state.push_back(s);
        root_index[s] = ins.first->second;
    }
    E.n_roots = (int64_t)root_state.size();

    // Every root first gets an equal share of the node budget (breadth first, see Walker::expand);
    // what the finished roots leave over goes, in further rounds, to the roots that were cut.
    std::vector<std::unique_ptr<BuildNode>> roots(root_state.size());
    std::vector<std::deque<BuildNode *>> queues(root_state.size());
    std::exception_ptr failure;                      // first exception of a worker, rethrown on the caller's thread
    std::mutex failure_lock;
    int64_t left = lim.max_nodes;
    std::vector<size_t> todo(roots.size());
    for (size_t i = 0; i < roots.size(); ++i) todo[i] = i;
    for (int round = 0; !todo.empty() && left > 0 && !failure; ++round) {
        const int share = (int)std::max<int64_t>(round == 0 ? 256 : 1, left / (int64_t)todo.size());
        std::atomic<size_t> next(0);
        std::atomic<int64_t> used(0);
        auto worker = [&]() {
            try {
                Walker w(T, trie, pred, lim, tok_len, budget);
                for (;;) {
                    const size_t k = next.fetch_add(1);
                    if (k >= todo.size()) return;
                    const size_t i = todo[k];
                    if (!roots[i]) {
                        roots[i].reset(new BuildNode());
                        w.walk_root(root_state[i], *roots[i]);
                        roots[i]->path.assign(1, root_state[i]);
                        queues[i].push_back(roots[i].get());
                    }
                    used += w.expand(queues[i], share);
                }
            } catch (...) {
                std::lock_guard<std::mutex> g(failure_lock);
                if (!failure) failure = std::current_exception();
                next.store(todo.size());                 // the other workers stop at their next root
            }
        };
        int n_threads = std::max(1, std::min<int>(lim.n_threads, (int)todo.size()));
        std::vector<std::thread> pool;
        for (int i = 1; i < n_threads; ++i) pool.emplace_back(worker);
        worker();
        for (auto &t : pool) t.join();
        left -= used.load();
        std::vector<size_t> cut;
        for (size_t i : todo)
            if (!queues[i].empty()) cut.push_back(i);
        if (used.load() == 0 && round > 0) break;        // the shares no longer buy a level anywhere
        todo.swap(cut);
    }
    if (failure) std::rethrow_exception(failure);
    queues.clear();

    // effect records are kept only if all of them fitted the budget (a partial set would make the speed
    // of an advance depend on which worker happened to write first)
    const bool keep_effects = lim.effect_min_len > 0 && !budget.exceeded.load();
    Flattener F{trie, lim, E, std::max(1, lim.max_path_ids), keep_effects};
    std::vector<int> root_node(roots.size());
    for (size_t i = 0; i < roots.size(); ++i) {
        std::vector<int32_t> since;
        const ConditionNode rec = F.flatten(*roots[i], -1, since);
        root_node[i] = (int)E.nodes.size();                  // a root is stored after its subtree
        E.nodes.push_back(rec);
        roots[i].reset();
    }
    E.root_of_state.resize(T.n_states);
    for (int s = 0; s < T.n_states; ++s) E.root_of_state[s] = root_node[root_index[s]];
    if (keep_effects && !E.effects.empty()) {
        E.effect_min_len = lim.effect_min_len;
        for (size_t i = 0; i < E.effects.size(); i += 4 + (size_t)E.effects[i + 3]) E.n_effect_records++;
    }
    return E;
}

EffectTable build_effect_table(const TokenEdges &E) {
    EffectTable X;
    if (E.effect_min_len <= 0) return X;
    // records per node (a list shared by several nodes is entered once per node)
    int64_t total = 0;
    for (const ConditionNode &n : E.nodes)
        for (int32_t at = n.effect_begin; at < n.effect_begin + n.effect_words; at += 4 + E.effects[at + 3]) ++total;
    uint64_t buckets = 1;
    while (buckets * 2 < (uint64_t)std::max<int64_t>(total, 1)) buckets <<= 1;       // about half full
    X.bucket_mask = (uint32_t)(buckets - 1);
    X.slots.assign((size_t)buckets * kEffectBucketSlots * 4, -1);
    std::vector<uint8_t> fill((size_t)buckets, 0);
    for (size_t node = 0; node < E.nodes.size(); ++node) {
        const ConditionNode &n = E.nodes[node];
        for (int32_t at = n.effect_begin; at < n.effect_begin + n.effect_words; at += 4 + E.effects[at + 3]) {
            const int32_t tok = E.effects[at], k = E.effects[at + 1], peak = E.effects[at + 2], np = E.effects[at + 3];
            uint32_t b1, b2;
            effect_buckets((uint32_t)node, (uint32_t)tok, X.bucket_mask, &b1, &b2);
            const uint32_t b = fill[b2] < fill[b1] ? b2 : b1;
            if (fill[b] >= kEffectBucketSlots) { ++X.dropped; continue; }
            int32_t *slot = &X.slots[((size_t)b * kEffectBucketSlots + fill[b]++) * 4];
            const bool inl = np <= 2 && E.effects[at + 4] < (1 << kEffectInlineStateBits) &&
                             (np == 1 || E.effects[at + 5] < (1 << kEffectInlineStateBits));
            const uint32_t s0 = (uint32_t)E.effects[at + 4], s1 = np == 2 ? (uint32_t)E.effects[at + 5] : 0u;
            slot[0] = (int32_t)node;
            slot[1] = (int32_t)((uint32_t)tok | ((uint32_t)k << 21) | ((inl ? (uint32_t)np : 0u) << 29));
            slot[2] = (int32_t)(((uint32_t)(peak + 32768) << 16) | (inl ? ((s1 >> 12) << 8) : 0u) | (uint32_t)np);
            if (inl) {
                slot[3] = (int32_t)(s0 | ((s1 & 0xFFFu) << 20));
            } else {
                slot[3] = (int32_t)X.pool.size();
                X.pool.insert(X.pool.end(), E.effects.begin() + at + 4, E.effects.begin() + at + 4 + np);
            }
            ++X.stored;
        }
    }
    return X;
}

bool find_effect(const TokenEdges &E, const EffectTable &X, const int32_t *stack, int len, int32_t token, int *k,
                 int *peak, std::vector<int32_t> *pushes) {
    if (X.slots.empty() || len < 1 || stack[len - 1] < 0 || stack[len - 1] >= (int)E.root_of_state.size()) return false;
    int node = E.root_of_state[stack[len - 1]];
    for (;;) {
        uint32_t b[2];
        effect_buckets((uint32_t)node, (uint32_t)token, X.bucket_mask, &b[0], &b[1]);
        for (int c = 0; c < 2; ++c)
            for (int s = 0; s < kEffectBucketSlots; ++s) {
                const int32_t *slot = &X.slots[((size_t)b[c] * kEffectBucketSlots + s) * 4];
                if (slot[0] < 0 || !effect_slot_matches((uint32_t)slot[0], (uint32_t)slot[1], (uint32_t)node, (uint32_t)token)) continue;
                const EffectFields f = effect_unpack((uint32_t)slot[1], (uint32_t)slot[2], (uint32_t)slot[3]);
                *k = f.k;
                *peak = f.peak;
                pushes->clear();
                if (f.inline_count >= 1) pushes->push_back(f.x0);
                if (f.inline_count == 2) pushes->push_back(f.x1);
                if (f.inline_count == 0) pushes->insert(pushes->end(), X.pool.begin() + f.x0, X.pool.begin() + f.x0 + f.np);
                return true;
            }
        const ConditionNode &n = E.nodes[node];
        if (n.child_count == 0 || n.known >= len) return false;
        const int x = stack[len - 1 - n.known];
        int next = -1;
        for (int i = 0; i < n.child_count; ++i)
            if (E.child_state[n.child_begin + i] == x) next = E.child_node[n.child_begin + i];
        if (next < 0) return false;
        node = next;
    }
}

bool resolve_row(const TokenEdges &E, const int32_t *stack, int len, uint32_t *row, std::vector<int32_t> &walk,
                 int32_t *info) {
    if (len < 1 || stack[len - 1] < 0 || stack[len - 1] >= (int)E.root_of_state.size()) return false;
    int node = E.root_of_state[stack[len - 1]];
    std::vector<int> path;
    for (;;) {
        path.push_back(node);
        const ConditionNode &n = E.nodes[node];
        if (n.child_count == 0) break;
        if (n.known >= len) return false;
        int x = stack[len - 1 - n.known], next = -1;
        for (int i = 0; i < n.child_count; ++i)
            if (E.child_state[n.child_begin + i] == x) next = E.child_node[n.child_begin + i];
        if (next < 0) return false;
        node = next;
    }
    int start = 0;
    for (int i = (int)path.size() - 1; i >= 0; --i)
        if (E.nodes[path[i]].dense_row >= 0) { start = i; break; }
    const ConditionNode &first = E.nodes[path[start]];
    if (first.dense_row >= 0)
        for (int w = 0; w < E.n_words; ++w) row[w] |= E.dense_rows[(size_t)first.dense_row * E.n_words + w];
    for (size_t i = start; i < path.size(); ++i) {
        const ConditionNode &n = E.nodes[path[i]];
        for (int k = 0; k < n.delta_count; ++k) {
            int t = E.delta_ids[n.delta_begin + k];
            row[t >> 5] |= 1u << (t & 31);
        }
    }
    const ConditionNode &last = E.nodes[path.back()];
    if (info) {
        info[0] = (int32_t)path.size();
        info[1] = start;
        info[2] = 0;
        for (size_t i = start; i < path.size(); ++i) info[2] += E.nodes[path[i]].delta_count;
        info[3] = last.known;
    }
    if (last.walk_count < 0) return false;
    for (int k = 0; k < last.walk_count; ++k) walk.push_back(E.walk_ids[last.walk_begin + k]);
    return true;
}

}  // namespace pre3

// From LR(1) automata to the flat DPDA edge tables the kernels walk (paper Sec. 3.1-3.3).
#include "tables.hpp"

#include <algorithm>
#include <cstring>
#include <map>
#include <numeric>

#include "../../include/pre3.h"

namespace pre3 {

namespace {

// Edge word of ACTION[s][a] of one automaton, with state ids made global.
uint32_t pack_edge(const Lr1Automaton &A, int state_offset, uint32_t action) {
    uint32_t kind = action & 3u, arg = action >> 2;
    switch (kind) {
        case kShift: return kShift | ((arg + (uint32_t)state_offset) << 2);
        case kReduce: {
            int n = A.prod_len[arg], lhs = A.prod_lhs[arg];
            if (n > kMaxPop)
                throw CompileError{PRE3_E_LIMIT, "a production has more than " + std::to_string(kMaxPop) +
                                                     " right-hand-side symbols"};
            return kReduce | ((uint32_t)n << 2) | ((uint32_t)lhs << kNtShift);
        }
        case kAccept: return kAccept;
        default: return 0;
    }
}

// H = 1 + the largest number of entries that the reductions and the shift of ONE input
// symbol can leave above the lowest stack position they touch.  Found by running, for every
// state u and class c, the deterministic chain of edges on the private stack [u] until the
// symbol is shifted, rejected, or a reduction reaches below u (from where the same bound
// applies again with the state pushed there as the new u).
int height_per_symbol(const EdgeTables &T) {
    const int ncol = T.n_classes + 1;
    int best = 1;
    std::vector<int32_t> st;
    for (int u = 0; u < T.n_states; ++u) {
        for (int c = 0; c < ncol; ++c) {
            st.assign(1, u);
            for (;;) {
                uint32_t e = T.edge[(size_t)st.back() * ncol + c];
                uint32_t kind = e & kKindMask;
                if (kind == kShift) { best = std::max(best, (int)st.size() + 1); break; }
                if (kind != kReduce) break;
                int n = (e >> 2) & kMaxPop, nt = e >> kNtShift;
                if (n >= (int)st.size()) break;            // would expose something below u
                st.resize(st.size() - n);
                int row = T.goto_row[st.back()];
                int t = row < 0 ? -1 : T.goto_flat[row + nt];
                if (t < 0) break;
                st.push_back(t);
                best = std::max(best, (int)st.size());
            }
        }
    }
    return best;
}

}  // namespace

// Multi-symbol edges for jump-forward (Sec. 3.3, merging of deterministic single-successor runs): a
// state whose ONLY edge is an acceptance edge on a byte class of one byte -- no reduction step on
// any class, nothing on '$' -- forces that byte whatever lies under it on the stack, and so does the
// state it leads to, and so on.  run_off[s] = offset of the run that starts at s (or -1), a run =
// its length (at most kMaxRun; a longer one continues with the run of the state it ends in), then
// per forced byte the word  target state << 8 | byte.
void build_forced_runs(EdgeTables &T) {
    std::vector<int32_t> *run_off = &T.run_off, *run_pool = &T.run_pool;
    const int ncol = T.n_classes + 1;
    std::vector<int> class_bytes(T.n_classes, 0), class_first(T.n_classes, -1);
    for (int b = 255; b >= 0; --b) {
        class_bytes[T.byte_class[b]]++;
        class_first[T.byte_class[b]] = b;
    }
    std::vector<int32_t> step(T.n_states, -1);             // target << 8 | byte of a state's forced byte, or -1
    for (int s = 0; s < T.n_states; ++s) {
        int edges = 0, col = -1;
        for (int c = 0; c < ncol; ++c)
            if ((T.edge[(size_t)s * ncol + c] & kKindMask) != kError) { ++edges; col = c; }
        if (edges != 1 || col >= T.n_classes || class_bytes[col] != 1) continue;
        const uint32_t e = T.edge[(size_t)s * ncol + col];
        if ((e & kKindMask) != kShift) continue;
        const int byte = class_first[col];
        step[s] = (int32_t)((((e >> 2) + (uint32_t)T.byte_delta[byte]) << 8) | (uint32_t)byte);
    }
    run_off->assign(T.n_states, -1);
    run_pool->clear();
    for (int s = 0; s < T.n_states; ++s) {
        if (step[s] < 0) continue;
        (*run_off)[s] = (int32_t)run_pool->size();
        run_pool->push_back(0);
        int len = 0;
        for (int at = s; len < kMaxRun && step[at] >= 0; at = step[at] >> 8, ++len) run_pool->push_back(step[at]);
        (*run_pool)[(*run_off)[s]] = len;
    }
    if (run_pool->empty()) run_pool->push_back(0);
}

EdgeTables build_edge_tables(const std::vector<Grammar> &grammars) {
    EdgeTables T;
    T.n_grammars = (int)grammars.size();
    T.state_offset.assign(1, 0);
    for (const Grammar &g : grammars) {
        T.automata.push_back(build_lr1(g));
        T.state_offset.push_back(T.state_offset.back() + T.automata.back().n_states);
    }
    T.n_states = T.state_offset.back();
    if (T.n_states >= (1 << 30)) throw CompileError{PRE3_E_LIMIT, "too many LR(1) states"};

    // Edge aggregation (Sec. 3.3): bytes whose edges agree in every state of every grammar form
    // one byte class.  Acceptance edges of two bytes "agree" when their targets differ by the
    // same constant in every state: a class such as [0-9], written as one production per byte,
    // shifts to ten item sets that were discovered, hence numbered, consecutively.  The
    // constant is kept per byte (byte_delta) and added to the class's target at run time.
    // Classes are numbered by their smallest byte.
    std::vector<std::vector<uint32_t>> column(256);
    std::vector<int64_t> first_target(256, -1);
    for (int b = 0; b < 256; ++b) {
        column[b].reserve(T.n_states);
        for (int g = 0; g < T.n_grammars; ++g) {
            const Lr1Automaton &A = T.automata[g];
            for (int s = 0; s < A.n_states; ++s) {
                uint32_t e = pack_edge(A, T.state_offset[g], A.action[(size_t)s * kNumTerminals + b]);
                if ((e & kKindMask) == kShift && first_target[b] < 0) first_target[b] = e >> 2;
                column[b].push_back(e);
            }
        }
    }
    // state kinds: identical per-byte edges (targets included), '$' edge, goto targets and predecessors
    {
        const std::vector<std::vector<int32_t>> pred = predecessors(T);
        std::map<std::vector<int64_t>, int> kinds;
        T.state_kind.resize(T.n_states);
        std::vector<int64_t> key;
        for (int g = 0; g < T.n_grammars; ++g) {
            const Lr1Automaton &A = T.automata[g];
            const int off = T.state_offset[g];
            for (int s = 0; s < A.n_states; ++s) {
                key.clear();
                key.push_back(g);
                for (int b = 0; b < 256; ++b) key.push_back(column[b][off + s]);
                key.push_back(pack_edge(A, off, A.action[(size_t)s * kNumTerminals + kEnd]));
                for (int nt = 0; nt < A.n_nt; ++nt) key.push_back(A.go[(size_t)s * A.n_nt + nt]);
                key.push_back(-7);
                for (int32_t p : pred[off + s]) key.push_back(p);
                T.state_kind[off + s] = kinds.emplace(key, (int)kinds.size()).first->second;
            }
        }
        T.n_kinds = (int)kinds.size();
    }
    std::map<std::vector<int64_t>, int> class_of_signature;
    T.byte_class.resize(256);
    T.byte_delta.assign(256, 0);
    std::vector<int> representative;
    std::vector<int64_t> sig;
    for (int b = 0; b < 256; ++b) {
        sig.clear();
        for (uint32_t e : column[b]) {
            if ((e & kKindMask) == kShift) {        // same target offset and same kind of target state
                sig.push_back((((int64_t)(e >> 2) - first_target[b]) << 2) | kShift);
                sig.push_back(T.state_kind[e >> 2]);
            } else {
                sig.push_back((int64_t)e);
            }
        }
        auto ins = class_of_signature.emplace(sig, (int)representative.size());
        if (ins.second) representative.push_back(b);
        T.byte_class[b] = (uint8_t)ins.first->second;
        int rep = representative[ins.first->second];
        T.byte_delta[b] = first_target[b] < 0 ? 0 : (int32_t)(first_target[b] - first_target[rep]);
    }
    T.n_classes = (int)representative.size();
    if (T.n_classes > 255) throw CompileError{PRE3_E_LIMIT, "more than 255 byte classes"};

    const int ncol = T.n_classes + 1;
    T.edge.assign((size_t)T.n_states * ncol, 0);
    for (int c = 0; c < T.n_classes; ++c)
        for (int s = 0; s < T.n_states; ++s) T.edge[(size_t)s * ncol + c] = column[representative[c]][s];
    for (int g = 0; g < T.n_grammars; ++g) {
        const Lr1Automaton &A = T.automata[g];
        for (int s = 0; s < A.n_states; ++s)
            T.edge[(size_t)(T.state_offset[g] + s) * ncol + T.n_classes] =
                pack_edge(A, T.state_offset[g], A.action[(size_t)s * kNumTerminals + kEnd]);
    }

    // Goto rows: the targets of reduction steps, selected by (exposed state, nonterminal).
    // Identical rows of one grammar are stored once; states without any target have no row.
    T.goto_row.assign(T.n_states, -1);
    int max_nt = 0;
    for (int g = 0; g < T.n_grammars; ++g) {
        const Lr1Automaton &A = T.automata[g];
        max_nt = std::max(max_nt, A.n_nt);
        std::map<std::vector<int32_t>, int> seen;
        for (int s = 0; s < A.n_states; ++s) {
            std::vector<int32_t> row(A.go.begin() + (size_t)s * A.n_nt, A.go.begin() + (size_t)(s + 1) * A.n_nt);
            bool any = false;
            for (auto &t : row)
                if (t >= 0) { t += T.state_offset[g]; any = true; }
            if (!any) continue;
            auto ins = seen.emplace(row, (int)T.goto_flat.size());
            if (ins.second) T.goto_flat.insert(T.goto_flat.end(), row.begin(), row.end());
            T.goto_row[T.state_offset[g] + s] = ins.first->second;
        }
    }
    // padding so that a nonterminal index of another grammar (possible only with a corrupted
    // stack) still reads inside the array
    T.goto_flat.insert(T.goto_flat.end(), (size_t)max_nt + 1, -1);

    T.height_per_byte = height_per_symbol(T);
    T.cycle_head.assign(T.n_states, -1);
    for (int g = 0; g < T.n_grammars; ++g) {
        const auto &cycles = T.automata[g].cycles;      // sorted by (length, states)
        for (size_t k = cycles.size(); k-- > 0;) {      // prepend, so that chains run shortest first
            const int head = T.state_offset[g] + cycles[k][0];
            const int at = (int)T.cycle_pool.size();
            T.cycle_pool.push_back((int32_t)cycles[k].size());
            T.cycle_pool.push_back(T.cycle_head[head]);
            for (int32_t v : cycles[k]) T.cycle_pool.push_back(T.state_offset[g] + v);
            T.cycle_head[head] = at;
            ++T.n_cycles;
        }
    }
    build_forced_runs(T);
    return T;
}

VocabLayout build_vocab_layout(const uint8_t *bytes, const int64_t *offsets, int n_tokens, int eos_id,
                               int max_token_len) {
    VocabLayout V;
    V.n_tokens = n_tokens;
    V.eos_id = eos_id;
    V.n_words = (n_tokens + 31) / 32;
    V.n_chunks = (n_tokens + kChunkIds - 1) / kChunkIds;
    V.n_padded = V.n_chunks * kChunkIds;
    for (int t = 0; t < n_tokens; ++t) {
        int64_t n = offsets[t + 1] - offsets[t];
        if (n < 0) throw CompileError{PRE3_E_BADARG, "vocabulary offsets must be non-decreasing"};
        if (t == eos_id) continue;
        if (n > max_token_len)
            throw CompileError{PRE3_E_TOKEN_TOO_LONG, "token " + std::to_string(t) + " has " + std::to_string(n) +
                                                          " bytes, more than max_token_len"};
        V.max_len = std::max(V.max_len, (int)n);
    }
    V.words_per_token = std::max(1, (V.max_len + 3) / 4);

    V.offsets.resize((size_t)n_tokens + 1);
    V.offsets[0] = 0;
    for (int t = 0; t < n_tokens; ++t) {
        int64_t n = t == eos_id ? 0 : offsets[t + 1] - offsets[t];
        V.bytes.insert(V.bytes.end(), bytes + offsets[t], bytes + offsets[t] + n);
        V.offsets[t + 1] = (int32_t)V.bytes.size();
    }
    V.bytes.resize(V.bytes.size() + 4, 0);

    V.tok_len.assign(V.n_padded, 0);
    V.tok_bit.assign(V.n_padded, 0);
    V.tok_words.assign((size_t)V.words_per_token * V.n_padded, 0);
    std::vector<int> order;
    for (int c = 0; c < V.n_chunks; ++c) {
        int lo = c * kChunkIds, hi = std::min(n_tokens, lo + kChunkIds);
        order.resize(hi - lo);
        std::iota(order.begin(), order.end(), lo);
        auto tok = [&](int t) {
            return std::make_pair(V.bytes.data() + V.offsets[t], (size_t)(V.offsets[t + 1] - V.offsets[t]));
        };
        std::sort(order.begin(), order.end(), [&](int a, int b) {
            auto x = tok(a), y = tok(b);
            int r = std::memcmp(x.first, y.first, std::min(x.second, y.second));
            if (r != 0) return r < 0;
            if (x.second != y.second) return x.second < y.second;
            return a < b;
        });
        for (int j = 0; j < (int)order.size(); ++j) {
            int t = order[j], pos = lo + j;
            auto x = tok(t);
            V.tok_bit[pos] = (uint16_t)(t - lo);
            V.tok_len[pos] = t == eos_id ? (uint8_t)kEosLen : (uint8_t)x.second;
            for (size_t k = 0; k < x.second; ++k)
                V.tok_words[(k / 4) * V.n_padded + pos] |= (uint32_t)x.first[k] << (8 * (k % 4));
        }
    }
    return V;
}

}  // namespace pre3

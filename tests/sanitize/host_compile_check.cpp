// CPU-only driver of the library's host compile path, built with AddressSanitizer and
// UndefinedBehaviorSanitizer by tests/test_sanitizers.py: grammar text -> canonical LR(1) ->
// DPDA edge tables -> merged reduction edges -> token-level condition trees, then one mask row per
// given stack from those tables (tree look-up, leftover tokens walked with the host mirror of the
// device step) and one advance per stack.  Prints one line per stack: a hash of the mask row and of
// the advanced stack.  No HIP: the sources under test are plain C++.
//
// usage: host_compile_check <dir> [compact] [max_known=N] [row_threshold=N] [stepwise] [no_token_edges]
//   <dir>/grammar_<i>.txt      grammar texts, i = 0, 1, ..
//   <dir>/vocab.bin            int32 n_tokens, int32 eos_id, int64 offsets[n_tokens + 1], bytes
//   <dir>/stacks.bin           int32 count, then per stack: int32 len, int32 entries[len], int32 token
#include <cstdint>
#include <cstdio>
#include <cstring>
#include <fstream>
#include <sstream>
#include <string>
#include <vector>

#include "../../paper_2506_03887_amd/csrc/symbol_edges.hpp"
#include "../../paper_2506_03887_amd/csrc/token_edges.hpp"

using namespace pre3;

static std::string slurp(const std::string &path, bool *ok) {
    std::ifstream f(path, std::ios::binary);
    *ok = (bool)f;
    std::ostringstream s;
    s << f.rdbuf();
    return s.str();
}

static uint64_t fnv(const void *data, size_t bytes) {
    const unsigned char *p = static_cast<const unsigned char *>(data);
    uint64_t h = 1469598103934665603ull;
    for (size_t i = 0; i < bytes; ++i) h = (h ^ p[i]) * 1099511628211ull;
    return h;
}

int main(int argc, char **argv) {
    if (argc < 2) return 2;
    const std::string dir = argv[1];
    bool compact = false, stepwise = false, token_edges = true;
    TokenEdgeLimits lim;
    lim.n_threads = 2;
    for (int i = 2; i < argc; ++i) {
        const std::string a = argv[i];
        if (a == "compact") compact = true;
        else if (a == "stepwise") stepwise = true;
        else if (a == "no_token_edges") token_edges = false;
        else if (a.rfind("max_known=", 0) == 0) lim.max_known = std::stoi(a.substr(10));
        else if (a.rfind("row_threshold=", 0) == 0) lim.max_path_ids = std::stoi(a.substr(14));
        else return 2;
    }
    lim.compacted_stacks = compact;
    try {
        std::vector<Grammar> gs;
        for (int i = 0;; ++i) {
            bool ok;
            const std::string text = slurp(dir + "/grammar_" + std::to_string(i) + ".txt", &ok);
            if (!ok) break;
            gs.push_back(parse_grammar(text));
        }
        if (gs.empty()) return 2;
        bool ok;
        const std::string vb = slurp(dir + "/vocab.bin", &ok);
        if (!ok || vb.size() < 8) return 2;
        int32_t n_tokens, eos;
        std::memcpy(&n_tokens, vb.data(), 4);
        std::memcpy(&eos, vb.data() + 4, 4);
        std::vector<int64_t> offsets((size_t)n_tokens + 1);
        std::memcpy(offsets.data(), vb.data() + 8, offsets.size() * 8);
        const uint8_t *bytes = reinterpret_cast<const uint8_t *>(vb.data()) + 8 + offsets.size() * 8;
        int max_len = 1;
        for (int t = 0; t < n_tokens; ++t) max_len = std::max<int>(max_len, (int)(offsets[t + 1] - offsets[t]));

        EdgeTables T = build_edge_tables(gs);
        VocabLayout V = build_vocab_layout(bytes, offsets.data(), n_tokens, eos, max_len);
        SymbolEdges S;
        if (!stepwise) S = build_symbol_edges(T);
        TokenEdges E;
        if (token_edges) E = build_token_edges(T, V, lim);
        const EffectTable X = build_effect_table(E);
        std::printf("tables states %d classes %d kinds %d cycles %d sym_nodes %zu tree_nodes %zu rows %lld effects %lld\n", T.n_states,
                    T.n_classes, T.n_kinds, T.n_cycles, S.nodes.size(), E.nodes.size(), (long long)E.n_dense, (long long)X.stored);

        const std::string sb = slurp(dir + "/stacks.bin", &ok);
        if (!ok) return 2;
        const int32_t *p = reinterpret_cast<const int32_t *>(sb.data());
        const int count = *p++;
        auto walk = [&](std::vector<int32_t> st, int t, int cap, std::vector<int32_t> *out) -> int {
            if (t == eos) return host_feed(T, S, st, T.n_classes, 0, cap, !stepwise) == kHostAccepted ? 0 : 1;
            const int lo = V.offsets[t], hi = V.offsets[t + 1];
            if (hi <= lo) return 1;
            for (int i = lo; i < hi; ++i) {
                const int r = host_feed(T, S, st, T.byte_class[V.bytes[i]], T.byte_delta[V.bytes[i]], cap, !stepwise);
                if (r != kHostFed) return r == kHostOverflow ? 2 : 1;
            }
            if (out) *out = st;
            return 0;
        };
        for (int k = 0; k < count; ++k) {
            const int len = *p++;
            std::vector<int32_t> st(p, p + len);
            p += len;
            const int token = *p++;
            std::vector<uint32_t> row(V.n_words, 0);
            std::vector<int32_t> left;
            bool resolved = token_edges && resolve_row(E, st.data(), len, row.data(), left);
            if (!resolved) {
                std::fill(row.begin(), row.end(), 0u);
                left.clear();
                for (int t = 0; t < n_tokens; ++t) left.push_back(t);
            }
            for (int t : left)
                if (walk(st, t, 1 << 30, nullptr) == 0) row[t >> 5] |= 1u << (t & 31);
            std::vector<int32_t> after = st;
            int rc = token >= 0 && token < n_tokens && token != eos ? walk(st, token, 1 << 30, &after) : -1;
            // the recorded stack operations of the token, where there are any, must give the walk's stack
            int fk = 0, fpeak = 0;
            std::vector<int32_t> pushes;
            if (rc == 0 && token_edges && find_effect(E, X, st.data(), len, token, &fk, &fpeak, &pushes) && fk <= len) {
                std::vector<int32_t> by_effect(st.begin(), st.begin() + (len - fk + 1));
                by_effect.insert(by_effect.end(), pushes.begin(), pushes.end());
                if (by_effect != after) std::printf("MISMATCH effect of token %d on stack %d\n", token, k);
            }
            std::printf("stack %d row %016llx resolved %d advance %d %016llx\n", k, (unsigned long long)fnv(row.data(), row.size() * 4),
                        (int)resolved, rc, (unsigned long long)fnv(after.data(), after.size() * 4));
        }
    } catch (const CompileError &e) {
        std::printf("compile error %d\n", e.status);
        return 0;
    }
    return 0;
}

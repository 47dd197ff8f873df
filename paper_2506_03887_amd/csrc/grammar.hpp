// Grammar text -> productions over byte terminals.
#pragma once
#include <cstdint>
#include <string>
#include <vector>

namespace pre3 {

// Symbol codes: 0..255 byte terminals, 256 end of input, kNtBase + i nonterminal i.
constexpr int kEnd = 256;
constexpr int kNumTerminals = 257;
constexpr int kNtBase = 257;

struct Production {
    int lhs;                    // nonterminal index
    std::vector<int> rhs;       // symbol codes
};

struct Grammar {
    std::vector<std::string> nt_names;      // index = nonterminal; the augmented start is last
    std::vector<Production> prods;          // prods[0] is  start' -> start
    std::vector<std::vector<int>> prods_of; // nonterminal -> production indices
    int n_nt() const { return (int)nt_names.size(); }
};

struct CompileError {
    int status;                 // pre3_status value
    std::string text;
};

// Parses one grammar text (format documented in pre3.h) and checks that every
// nonterminal is defined, productive and reachable.  Throws CompileError.
Grammar parse_grammar(const std::string &text);

}  // namespace pre3

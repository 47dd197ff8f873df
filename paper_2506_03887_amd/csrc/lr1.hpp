// Canonical LR(1) automaton of one grammar (paper App. A.2).
#pragma once
#include <cstdint>
#include <vector>

#include "grammar.hpp"

namespace pre3 {

enum ActionKind : uint32_t { kError = 0, kShift = 1, kReduce = 2, kAccept = 3 };

struct Lr1Automaton {
    int n_states = 0;
    int n_nt = 0;
    // action[s * kNumTerminals + a] = kind | (arg << 2); arg = shift target or production
    std::vector<uint32_t> action;
    // go[s * n_nt + A] = target state or -1
    std::vector<int32_t> go;
    std::vector<int32_t> prod_lhs, prod_len;
};

// States are numbered in breadth-first discovery order from the initial item set, trying
// terminals in ascending byte order and then nonterminals by index.  Throws CompileError
// (PRE3_E_NOT_LR1) on a shift/reduce or reduce/reduce conflict.
Lr1Automaton build_lr1(const Grammar &g);

}  // namespace pre3

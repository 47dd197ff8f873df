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
    // Cycles of right-recursive reductions (Sec. 3.2.3, Alg. 1 step 1): each entry lists the
    // states v1..vn of one cycle; a stack whose top is v1 with v1..vn right below it behaves
    // like the stack without those n entries.  Sorted by (length, states).
    std::vector<std::vector<int32_t>> cycles;
};

constexpr int kMaxCycleStates = 64;     // longer cycles are not registered

// States are numbered in breadth-first discovery order from the initial item set, trying
// terminals in ascending byte order and then nonterminals by index.  Throws CompileError
// (PRE3_E_NOT_LR1) on a shift/reduce or reduce/reduce conflict.
Lr1Automaton build_lr1(const Grammar &g);

}  // namespace pre3

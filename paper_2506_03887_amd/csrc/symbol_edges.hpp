// Reduction edges with their stack-matching conditions (paper Sec. 3.2.2, Alg. 1 step 3).
//
// For one input symbol the LR(1) parser may run a whole chain of reductions before it shifts.
// The paper replaces the chain by ONE reduction edge: match a stack prefix, pop, push the
// resulting states, accept the symbol.  Here the edges leaving a state form a small condition
// tree: the root is the state on top of the stack; a child fixes one more stack entry below the
// ones already known (chosen among the predecessors of the deepest known state; a unique
// predecessor needs no test).  For every input symbol class the tree holds, at the shallowest
// node where the chain is fully determined, the merged effect
//     truncate the stack to (len - known + 1) entries, then push p0 .. pk
// (the last push is the acceptance edge's target).  No chain is ever enumerated beyond the
// entries it really reads, so cyclic grammars need no special treatment.
#pragma once
#include <cstdint>
#include <vector>

#include "tables.hpp"

namespace pre3 {

enum SymbolEffectCode : int32_t {
    kEffNone = -1,        // no edge: the symbol is rejected
    kEffAccept = -2,      // '$' only: the text is a sentence
    kEffDeeper = -3,      // determined at a child: test the next stack entry
    kEffStepwise = -4     // not precomputed (limits reached): follow the per-step edges
};

// n_push field of an effect record: low bits = number of pushes, flags = self-similar edge (the
// stack keeps its shape) and growing edge (the stack gains one copy of the entry under the top)
constexpr int32_t kEffPushMask = 0xFFFF;
constexpr int32_t kEffSameShape = 1 << 16;
constexpr int32_t kEffGrow = 1 << 17;

struct SymbolNode {
    int32_t known;        // stack entries (from the top) fixed by this node
    int32_t child_begin;  // children in child_state/child_node[child_begin .. +child_count)
    int32_t child_count;
    int32_t first_child;  // children are the nodes first_child .. first_child + child_count - 1
};

struct SymbolEdges {
    bool enabled = false;
    int ncol = 0;
    std::vector<SymbolNode> nodes;              // nodes[k] is the root shared by the states of kind k
    std::vector<int32_t> child_state, child_node;
    std::vector<int32_t> eff;                   // [nodes * ncol]: SymbolEffectCode or offset into pool
    // effect record at pool[o] (16-byte aligned): known, peak, n_push, kind of the last pushed state,
    // push[0..n_push)
    //   peak = largest (stack height just before a push) - (height before the symbol), so that
    //   "a push would exceed cap" can be decided without replaying the chain
    std::vector<int32_t> pool;
    int64_t max_known = 0;
};

SymbolEdges build_symbol_edges(const EdgeTables &T, int max_known = 32, int max_nodes = 1 << 21);

enum HostFeed { kHostFed = 0, kHostRejected = 1, kHostOverflow = 2, kHostAccepted = 3 };

// Host mirror of the device step (tests and tools): consumes one symbol (column `col`, target
// offset `delta`) on `st` using the merged edges (use_merged) or the per-step edges.
int host_feed(const EdgeTables &T, const SymbolEdges &S, std::vector<int32_t> &st, int col, int delta, int cap,
              bool use_merged);

}  // namespace pre3

// Token-level prefix-conditioned edges (paper Sec. 3.1 and Sec. 3.3 "edge merging").
//
// Along the bytes of one vocabulary token the per-byte edges of the DPDA are merged into a
// single multi-byte "jump" edge.  Its stack-matching condition is the sequence of states that
// the walk would read from the sequence's stack: the top state, then deeper entries as
// reductions expose them.  Because every edge is known when the grammar is compiled, all
// feasible conditions can be enumerated ahead of time by following the automaton's
// transitions backwards from a state (Sec. 3.2.2: a reduction edge backtracks along the path
// it was reached by).  The result is a condition tree:
//
//   root  = a top state (states with identical edges and predecessors share a root)
//   child = one more known stack entry below the ones already known, chosen among the
//           predecessors of the deepest known state
//   node  = the tokens whose merged edge exists (token allowed) for EVERY stack that matches
//           the node's condition and that were still undetermined at the parent ("delta"),
//           and, where the tree was not expanded further, the tokens that are still
//           undetermined ("walk" list: the kernel walks those byte by byte).
//
// A token rejected for every matching stack simply appears nowhere.  At run time a sequence
// descends the tree by comparing its stack entries with the children's condition states,
// takes the materialised row of the deepest node that has one (a "dense" row holds everything
// allowed on the path so far), ORs the deltas of the nodes after it and walks the few tokens
// left.
//
// Storage: by default every node that allows a token of its own has a dense row, and identical
// rows are stored once; equal groups of sibling nodes (equal subtrees under different parents),
// equal delta lists and equal walk lists are stored once as well, so the trees form a DAG.
// Children of a node are consecutive records, sorted by condition state, and are stored before
// their parent.
#pragma once
#include <cstdint>
#include <vector>

#include "effect_hash.hpp"
#include "tables.hpp"

namespace pre3 {

struct ConditionNode {
    int32_t known;          // stack entries (from the top) fixed by this node's condition
    int32_t child_begin;    // children in child_state/child_node[child_begin .. +child_count); their nodes
                            // have consecutive indices in the order of their condition states
    int32_t child_count;    // they are told apart by the state at depth `known` below the top
    int32_t dense_row;      // >= 0: dense_rows[dense_row * n_words ..] holds every token allowed at
                            // this node or at an ancestor; -1: none
    int32_t delta_begin;    // token ids allowed here and not at an ancestor
    int32_t delta_count;
    int32_t walk_begin;     // token ids left undetermined if the descent ends here;
    int32_t walk_count;     // -1: too many, walk the whole vocabulary
    int32_t effect_begin;   // stack effects of the longer tokens allowed here (records in TokenEdges::effects)
    int32_t effect_words;
};

struct TokenEdges {
    bool enabled = false;
    int n_words = 0;
    std::vector<int32_t> root_of_state;       // [n_states]
    std::vector<ConditionNode> nodes;
    std::vector<int32_t> child_state, child_node;
    std::vector<uint32_t> dense_rows;
    std::vector<int32_t> delta_ids, walk_ids;
    // Stack effects (the merged edge's stack operations, Sec. 3.1: every edge carries its accepted
    // symbols, its stack-matching condition AND its stack operations).  For a token of at least
    // effect_min_len bytes that a node allows, one record
    //     token id, k, peak, n_push, push[0 .. n_push)
    // says what the token's walk does to ANY stack matching the node's condition: the top k - 1
    // entries are replaced by the n_push states (so the entry k - 1 below the top is the deepest one
    // the walk exposes, and it stays); peak = largest stack height just before a push, relative to the
    // height before the token (the walk overflows a capacity `cap` iff len + peak >= cap).
    // A node's records are effects[effect_begin .. effect_begin + effect_words).
    std::vector<int32_t> effects;
    int64_t n_effect_records = 0;
    int effect_min_len = 0;               // 0: no effects were recorded
    // statistics
    int64_t n_roots = 0, max_known = 0, n_dense = 0;
};

// (node, token) -> effect record: buckets of four 16-byte slots, two candidate buckets per key; a
// record that finds both full is left out (its token is then walked byte by byte, like every token
// without a record).  The slot layout is in effect_hash.hpp: one or two pushed states travel inside
// the slot, longer push lists in `pool`.
struct EffectTable {
    std::vector<int32_t> slots;           // 4 ints per slot, 4 slots per bucket; node = -1: empty
    std::vector<int32_t> pool;            // the pushes of records with more than one
    uint32_t bucket_mask = 0;
    int64_t stored = 0, dropped = 0;
};
EffectTable build_effect_table(const TokenEdges &E);
// Host mirror of the kernels' look-up (tests and tools): descends the condition tree for the stack,
// probes every node on the way for `token`.  Returns true and fills k, peak and the pushes on a hit.
bool find_effect(const TokenEdges &E, const EffectTable &X, const int32_t *stack, int len, int32_t token, int *k,
                 int *peak, std::vector<int32_t> *pushes);

struct TokenEdgeLimits {
    int max_nodes = 1 << 20;          // condition-tree nodes
    int max_known = 48;               // deepest stack entry a condition may test
    int max_path_ids = 1;             // token ids a descent may collect before a row is materialised
                                      // (1: every node that allows a token of its own has a row; rows
                                      // are shared, so this costs little; delta lists then only appear
                                      // once max_dense_words is exhausted)
    int max_walk = 2048;              // longest walk list kept per node (longer: whole vocabulary)
    int64_t max_dense_words = (int64_t)1 << 28;   // 1 GiB of dense rows
    int n_threads = 8;
    bool compacted_stacks = false;    // stacks hold no complete traversal of a reduction cycle (tables.hpp)
    int effect_min_len = 3;           // tokens of at least this many bytes get stack-effect records (0: none);
                                      // shorter ones are walked as fast as a record is found
    int64_t max_effect_records = (int64_t)12 << 20;   // beyond this no records are kept at all
};

TokenEdges build_token_edges(const EdgeTables &T, const VocabLayout &V, const TokenEdgeLimits &lim);

// Host-side evaluation of the condition tree for one stack (tests and tools): ORs into `row`
// (n_words words) every token the tree determines as allowed and appends to `walk` the tokens
// it leaves undetermined.  Returns false if the tree has no answer for this stack (the kernel
// then walks the whole vocabulary).
// info (optional, 4 ints): nodes on the path, index of the dense node used, delta ids ORed, deepest
// stack entry tested.
bool resolve_row(const TokenEdges &E, const int32_t *stack, int len, uint32_t *row, std::vector<int32_t> &walk,
                 int32_t *info = nullptr);

}  // namespace pre3

// Plain-pointer view of the uploaded tables, passed to kernels by value.
#pragma once
#include <hip/hip_runtime_api.h>

#include <cstdint>

namespace pre3 {

constexpr int32_t kCellInline = 1 << 30;
constexpr int32_t kCellSameShape = 1 << 18;
constexpr int32_t kCellGrow = 1 << 19;

constexpr int kTokInfoBytes = 31;

struct DevTables {
    // DPDA edges
    const int32_t *byte_info;      // [256] byte class | (acceptance-target offset << 8)
    const uint32_t *edge;          // [n_states * ncol], packed as in tables.hpp
    const int32_t *goto_row;       // [n_states]
    const int32_t *goto_flat;
    int n_states, ncol, end_col;   // end_col = column of '$'
    // merged reduction edges with stack-matching conditions (symbol_edges.hpp); null = not built
    const int4 *sym_nodes;         // (known, child_begin, child_count, first_child)
    const int2 *sym_pairs;         // (condition state, child node)
    // [nodes * ncol] one 16-byte cell per (condition node, symbol column).  x < 0: SymbolEffectCode;
    // x with kCellInline: the whole edge (x = known | (peak + 128) << 8 | n_push << 16 | same-shape
    // and growing flags, y = kind after the edge, z and w = the one or two states pushed); otherwise x is the
    // offset of the edge's record in sym_pool
    const int4 *sym_cell;
    const int32_t *sym_pool;       // effect records, 16-byte aligned
    const int32_t *state_kind;     // [n_states] root node of each state's condition tree
    const int32_t *class_info;     // [ncol] bytes in the class | (smallest byte of the class << 16)
    // vocabulary, chunk-sorted order
    const uint8_t *tok_len;        // [n_padded]
    const uint16_t *tok_bit;       // [n_padded]
    const uint32_t *tok_words;     // [words_per_token * n_padded]
    int n_padded, n_chunks, n_words, n_tokens, eos_id;
    // vocabulary, id order
    const uint8_t *vbytes;
    const int32_t *voffsets;       // [n_tokens + 1]
    // one 128-byte line per token: [0] = length in bytes (-1: longer than kTokInfoBytes, use vbytes),
    // [1 + i] = byte_info of byte i -- everything a walk needs to know about the token in one access
    const int32_t *tok_info;       // [n_tokens * 32]
    // runs of forced bytes (multi-symbol edges): run_off[s] = offset in run_pool of the run that starts at
    // state s, or -1; a run is its length L (1..64) followed by L words  target state << 8 | byte
    const int32_t *run_off;        // [n_states], null = none
    const int32_t *run_pool;
    int max_depth;                 // private stack entries a walk can need
    int cycle_pool_n;              // entries of the reduction-cycle records (cycle-aware stacks), 0 = none
    int32_t *fault;                // device counter: walks stopped by an internal guard (must stay 0)
    // the small tables every advance touches lie next to each other: idle waves pull them into L2
    const char *hot_begin;
    int32_t hot_bytes;             // 0 = no such region
};

// Condition tree of the token-level prefix-conditioned edges (see token_edges.hpp), device form.
// An inner node (child_count > 0) names its children: their condition states are
// child_state[a .. a + child_count), their records nodes[b .. b + child_count).
// A leaf names the tokens still undetermined there: walk_ids[a .. a + b), b = -1: all tokens.
struct DevConditionNode {
    int32_t known, child_count, a, b, dense_row, delta_begin, delta_count, pad;
};

struct DevTokenEdges {
    const DevConditionNode *root_nodes;    // [n_states] copy of each state's root record
    const DevConditionNode *nodes;
    const int32_t *child_state;            // condition states, sorted per node
    const uint32_t *dense_rows;            // [n_dense * stride], stride = n_words rounded up to 4
    const int32_t *delta_ids, *walk_ids;
    // stack effects of the longer tokens (token_edges.hpp): (node, token) -> record, null = none
    const int32_t *root_id;                // [n_states] index of each state's root in nodes[]
    const int4 *fx_slots;                  // buckets of kEffectBucketSlots slots
    const int32_t *fx_pool;                // pushes of records with more than one
    uint32_t fx_mask;
    int32_t fx_min_len;                    // tokens shorter than this have no record
};

}  // namespace pre3

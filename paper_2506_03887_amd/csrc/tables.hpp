// DPDA edge tables and vocabulary layout, as uploaded to the device.
#pragma once
#include <cstdint>
#include <string>
#include <vector>

#include "lr1.hpp"

namespace pre3 {

// Packed edge word, one per (state, byte class):
//   bits 0..1  kind: 0 no edge, 1 acceptance edge, 2 reduction step, 3 accept (only on '$')
//   acceptance edge: bits 2..31 = target state (global id) to push
//   reduction step : bits 2..11 = number of states to pop, bits 12..31 = nonterminal index
//                    (local to the grammar); the state exposed by the pop selects the target
//                    through the goto rows (the stack-matching condition of the edge)
constexpr uint32_t kKindMask = 3u;
constexpr int kPopBits = 10;
constexpr int kMaxPop = (1 << kPopBits) - 1;
constexpr int kNtShift = 2 + kPopBits;

constexpr int kChunkIds = 2048;            // token ids per vocabulary chunk (64 mask words)
constexpr int kChunkWords = kChunkIds / 32;
constexpr int kEosLen = 255;               // tok_len marker of the end-of-sequence token

struct EdgeTables {
    int n_grammars = 0;
    std::vector<int> state_offset;         // [n_grammars + 1]
    std::vector<Lr1Automaton> automata;    // kept for host-side introspection
    int n_states = 0;
    int n_classes = 0;                     // byte classes; column n_classes is '$'
    std::vector<uint8_t> byte_class;       // [256]
    std::vector<int32_t> byte_delta;       // [256] added to the target of an acceptance edge
    std::vector<uint32_t> edge;            // [n_states * (n_classes + 1)]
    std::vector<int32_t> goto_row;         // [n_states] offset into goto_flat, -1 = no row
    std::vector<int32_t> goto_flat;        // deduplicated rows of targets (global ids), -1 = none
    // States that behave identically as the top of a stack (same edges for every byte and '$', same
    // goto row, same predecessors) share a kind; bytes of one class shift to states of one kind.
    std::vector<int32_t> state_kind;       // [n_states]
    int n_kinds = 0;
    int height_per_byte = 1;               // H: most private entries one input symbol can add, plus 1
    // Reduction cycles of all grammars (global state ids).  cycle_head[v1] = offset of the first
    // record whose cycle starts with v1, or -1; a record is  n, offset of the next record with the
    // same head (or -1), v1..vn.  Records of one head are chained shortest first.
    std::vector<int32_t> cycle_head;       // [n_states]
    std::vector<int32_t> cycle_pool;
    int n_cycles = 0;
    // Runs of forced bytes (multi-symbol edges for jump-forward): run_off[s] = offset in run_pool of the
    // run that starts at state s, or -1; a run is its length (1 .. kMaxRun) followed by one word per
    // forced byte,  target state << 8 | byte.
    std::vector<int32_t> run_off;          // [n_states]
    std::vector<int32_t> run_pool;
};
constexpr int kMaxRun = 64;

struct VocabLayout {
    int n_tokens = 0, eos_id = 0;
    int n_words = 0;                       // ceil(n_tokens / 32)
    int n_chunks = 0, n_padded = 0;        // n_padded = n_chunks * kChunkIds
    int max_len = 0, words_per_token = 0;
    // chunk-sorted order: position pos = chunk * kChunkIds + rank of the token inside its chunk
    // when the chunk's tokens are sorted by bytes
    std::vector<uint8_t> tok_len;          // [n_padded] 0 = never allowed, kEosLen = EOS
    std::vector<uint16_t> tok_bit;         // [n_padded] id - chunk * kChunkIds
    std::vector<uint32_t> tok_words;       // [words_per_token * n_padded], 4 bytes per word, little endian
    // id order, for advance
    std::vector<uint8_t> bytes;
    std::vector<int32_t> offsets;          // [n_tokens + 1]
};

EdgeTables build_edge_tables(const std::vector<Grammar> &grammars);
// pred[s] = every state with a transition (acceptance edge or goto) into s, sorted
std::vector<std::vector<int32_t>> predecessors(const EdgeTables &T);
VocabLayout build_vocab_layout(const uint8_t *bytes, const int64_t *offsets, int n_tokens, int eos_id,
                               int max_token_len);

}  // namespace pre3

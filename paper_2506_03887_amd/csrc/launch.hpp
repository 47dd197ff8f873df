// Host-callable launchers of the kernels (defined in mask_kernels.hip, apply_kernels.hip, sampler_kernels.hip and
// advance_kernels.hip) and the sizes of the scratch areas they need.
#pragma once
#include <hip/hip_runtime_api.h>

#include <cstddef>
#include <cstdint>

#include "device_tables.hpp"

namespace pre3 {

int walk_grid_blocks(int n_compute_units);
size_t walk_spill_entries(int grid_blocks, int max_depth);          // int32 entries
size_t advance_scratch_entries(int batch, int max_depth);           // int32 entries

hipError_t launch_fill_mask_walk(const DevTables &T, const int32_t *states, const int32_t *data, const int32_t *len,
                                 int cap, int batch, uint32_t *bitmask, int32_t *spill, int grid_blocks,
                                 hipStream_t stream);
int edge_grid_blocks(int n_compute_units);
size_t edge_spill_entries(int grid_blocks, int max_depth);          // int32 entries
int edge_row_stride_words(int n_words);                             // stride of dense rows on the device
size_t edge_kernel_max_lds_words();                                 // largest bitmap row the kernel can hold
hipError_t launch_fill_mask_edges(const DevTables &T, const DevTokenEdges &E, const int32_t *states,
                                  const int32_t *data, const int32_t *len, int cap, int batch, uint32_t *bitmask,
                                  uint16_t *logits /* null: mask only */, int64_t row_stride, int32_t *spill,
                                  int grid_blocks, hipStream_t stream);
// One thread writes the device's wall clock (100 MHz) to *out.
hipError_t launch_timestamp(int64_t *out, hipStream_t stream);

hipError_t launch_apply_mask(uint16_t *logits, const uint32_t *bitmask, int batch, int vocab, int64_t row_stride,
                             hipStream_t stream);
// cycle_head / cycle_pool: the cycle tables for cycle-aware stacks (needs advance_fits_compact(cap)), or null;
// E: the token-level edges, whose stack-effect records apply longer tokens in one step (E.fx_slots null: every token is walked)
hipError_t launch_advance(const DevTables &T, const DevTokenEdges &E, const int32_t *tokens, int32_t *states, int32_t *data,
                          int32_t *len, int cap, int batch, int32_t *err, int32_t *scratch, int restart_on_eos,
                          const int32_t *cycle_head, const int32_t *cycle_pool, hipStream_t stream);
bool advance_fits_compact(int cap);                     // four staged stacks within the kernel's LDS
// The library's own spill area (a device array of kStaticScratchEntries int32 that is part of the
// loaded code object, 4 MiB per GPU): its address on the current device.  The first call on a
// device looks the address up; no call allocates.
constexpr size_t kStaticScratchEntries = (size_t)1 << 20;
hipError_t static_advance_scratch(int32_t **out);
hipError_t launch_masked_argmax(const uint16_t *logits, const uint32_t *bitmask, int batch, int vocab, int64_t row_stride,
                                int n_compute_units, unsigned long long *workspace, int32_t *out, hipStream_t stream);
size_t masked_argmax_workspace_bytes(int batch, int vocab, int n_compute_units);   // per-segment partial results
// The k largest allowed logits of every row (k <= kTopkMax), ids in out_ids[batch * k] (-1 padded),
// their bf16 patterns in out_vals (may be null; 0xFF80 padded).
constexpr int kTopkMax = 64;
bool masked_topk_fits(int vocab, int k);      // (chunks of 16,384 tokens) x k <= 1,024 candidates per row
size_t masked_topk_workspace_bytes(int batch, int vocab);
hipError_t launch_masked_topk(const uint16_t *logits, const uint32_t *bitmask, int batch, int vocab, int64_t row_stride,
                              int k, int n_compute_units, unsigned long long *workspace, int32_t *out_ids,
                              uint16_t *out_vals, hipStream_t stream);
size_t advance_fill_walk_spill_entries(int batch, int max_depth);   // int32 entries
// cycle_head / cycle_pool: the cycle tables for cycle-aware stacks (the call then needs
// advance_fill_fits_compact), or null.
hipError_t launch_advance_fill(const DevTables &T, const DevTokenEdges &E, const int32_t *tokens, int32_t *states,
                               int32_t *data, int32_t *len, int cap, int batch, int32_t *err, uint32_t *bitmask,
                               int restart_on_eos, int32_t *adv_scratch, int32_t *walk_spill,
                               const int32_t *cycle_head, const int32_t *cycle_pool, hipStream_t stream);
bool advance_fill_fits_compact(int n_words, int cap);   // row bitmap + staged stack within 64 KB of LDS
// The same followed by the masking of the logits with the new rows, as one kernel that fetches a
// sequence's logits while its token is still being walked.  Needs advance_fill_apply_fits, logits
// aligned to 16 bytes and a row stride that is a multiple of 8 and at least the vocabulary size.
// out_tokens null: the logits are masked in place; else they are only read and out_tokens[b] becomes
// the arg max of the allowed logits of row b (the greedy step).
// rows_per_launch: a batch of more rows goes as several launches of equal shares of at most that many
// (the number of compute units: a block fills one); 0: one launch.
bool advance_fill_apply_fits(int n_tokens, int n_words, int cap, bool cycles, bool greedy);   // greedy: the arg-max form
// The same kernel without the advance: mask rows of the stacks as they are, applied to the logits
// (walk_spill: advance_fill_walk_spill_entries(batch, ...) entries; same conditions on the logits).
hipError_t launch_fill_apply_rows(const DevTables &T, const DevTokenEdges &E, const int32_t *states, const int32_t *data,
                                  const int32_t *len, int cap, int batch, uint32_t *bitmask, int32_t *walk_spill,
                                  uint16_t *logits, int64_t row_stride, int rows_per_launch, hipStream_t stream);
hipError_t launch_advance_fill_apply(const DevTables &T, const DevTokenEdges &E, const int32_t *tokens, int32_t *states,
                                     int32_t *data, int32_t *len, int cap, int batch, int32_t *err, uint32_t *bitmask,
                                     int restart_on_eos, int32_t *adv_scratch, int32_t *walk_spill,
                                     const int32_t *cycle_head, const int32_t *cycle_pool, uint16_t *logits,
                                     int64_t row_stride, int32_t *out_tokens, int rows_per_launch, hipStream_t stream);
hipError_t launch_jump_forward(const DevTables &T, int32_t *states, int32_t *data, int32_t *len, int cap, int batch,
                               uint8_t *out_bytes, int32_t *out_len, int max_bytes, int32_t *adv_scratch,
                               int32_t *lane_spill, const int32_t *cycle_head, const int32_t *cycle_pool,
                               hipStream_t stream);
bool jump_forward_fits_compact(int cap);                // four staged stacks within the kernel's LDS

// The cycle records in device memory end with this many entries that match no state.
constexpr int kCyclePoolPad = 64;

// Stack compaction over registered reduction cycles; cap (entries per stack) at most kCompactMaxLen.
constexpr int kCompactMaxLen = 4096;
hipError_t launch_compact_stacks(const int32_t *cycle_head, const int32_t *cycle_pool, int pool_entries, int n_states,
                                 int32_t *data, int32_t *len, int cap, int batch, hipStream_t stream);

}  // namespace pre3

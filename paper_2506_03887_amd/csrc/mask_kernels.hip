// gfx950 kernels of the token mask (token walk + bitmask pack): from the token-level edges, and
// byte by byte.  Wave64; no matrix cores (gather/branch-bound table walking).
#include <hip/hip_runtime.h>

#include "launch.hpp"
#include "row_plan.hpp"

namespace pre3 {

namespace {

// One block per (sequence, vocabulary chunk) work item, grid-strided.  Every lane walks the
// tokens at its chunk-sorted positions (neighbouring lanes hold tokens with common prefixes,
// so they follow the same edges), sets the bit of the token's id in an LDS bitmap of the
// chunk, and the block stores the chunk's 64 mask words with coalesced writes.
__global__ __launch_bounds__(kBlock) void fill_mask_walk_kernel(DevTables T, const int32_t *__restrict__ states,
                                                                 const int32_t *__restrict__ data,
                                                                 const int32_t *__restrict__ len, int cap, int batch,
                                                                 uint32_t *__restrict__ bitmask, int32_t *spill,
                                                                 size_t spill_stride) {
    __shared__ uint32_t bits[kChunkWords];
    __shared__ int32_t lds_stack[kLdsDepth * kBlock];
    PrivateStack priv;
    priv.lds = lds_stack + threadIdx.x;
    priv.lds_stride = kBlock;
    priv.spill = spill + (size_t)blockIdx.x * kBlock + threadIdx.x;
    priv.spill_stride = spill_stride;

    const int n_items = batch * T.n_chunks;
    for (int item = blockIdx.x; item < n_items; item += gridDim.x) {
        const int b = item / T.n_chunks, chunk = item - b * T.n_chunks;
        const int32_t *row = data + (size_t)b * cap;
        const int n = len[b];
        const bool done = states[b] < 0;
        int top0 = -1;
        if (!done && n >= 1 && n <= cap) top0 = row[n - 1];
        const bool live = (unsigned)top0 < (unsigned)T.n_states;

        if (threadIdx.x < kChunkWords) bits[threadIdx.x] = 0;
        __syncthreads();
        for (int j = threadIdx.x; j < kChunkIds; j += kBlock) {
            const int pos = chunk * kChunkIds + j;
            const int nb = T.tok_len[pos];
            if (nb == 0) continue;
            bool ok;
            if (nb == kEosLen) ok = done || (live && walk_end(T, priv, row, n, top0));
            else ok = live && walk_token(T, priv, pos, nb, row, n, top0);
            if (ok) {
                const int bit = T.tok_bit[pos];
                atomicOr(&bits[bit >> 5], 1u << (bit & 31));
            }
        }
        __syncthreads();
        const int w = chunk * kChunkWords + threadIdx.x;
        if (threadIdx.x < kChunkWords && w < T.n_words) bitmask[(size_t)b * T.n_words + w] = bits[threadIdx.x];
        __syncthreads();
    }
}

constexpr int kEdgeBlock = 256;        // threads per block of the token-edge kernel
constexpr int kWalkLanes = 64;         // lanes of a block that may walk tokens byte by byte
constexpr uint32_t kNegInfPair = 0xFF80FF80u;

// Token mask from the precomputed token-level edges, optionally fused with the masking of the
// logits.  A work item is one segment (a run of mask words) of one sequence's row; blocks loop
// over items.  Per item:
//   1. wave 0 descends the condition tree.  Lane j holds the stack entry j below the top; each
//      node names the entry it tests, and all of the node's condition states are compared
//      with it at once (one lane per child, wave ballot).  The root is fetched from states[b]
//      while the stack is still loading and re-fetched if the stack's top disagrees;
//   2. the segment of the dense row of the deepest dense node on the path is copied into an
//      LDS bitmap;
//   3. the delta lists of the nodes after it are ORed in, one lane per token id;
//   4. tokens the tree leaves undetermined (rare) are walked byte by byte by one wave;
//   5. the bitmap segment is stored with coalesced writes and, when fused, applied to the
//      segment's logits straight from LDS (allowed groups untouched, masked groups
//      overwritten unread, mixed groups read, patched and written back).
// A stack the tree has no answer for falls back to walking every token of the segment.
// Items are numbered so that the segments of one row run on the same XCD (blocks are dealt
// round-robin to the 8 XCDs) and share that XCD's L2 for the row's table reads.
template <bool kApply>
__global__ __launch_bounds__(kEdgeBlock) void fill_mask_edges_kernel(
    DevTables T, DevTokenEdges E, const int32_t *__restrict__ states, const int32_t *__restrict__ data,
    const int32_t *__restrict__ len, int cap, int batch, uint32_t *__restrict__ bitmask,
    uint16_t *__restrict__ logits, int64_t row_stride, int n_seg, int seg_vec, int32_t *spill,
    size_t spill_stride) {
    extern __shared__ uint4 bits4[];                   // seg_vec
    uint32_t *bits = reinterpret_cast<uint32_t *>(bits4);
    __shared__ RowPlan plan;
    __shared__ int32_t s_win[kWindow];
    __shared__ int32_t lds_stack[kLdsDepth * kWalkLanes];
    const int tid = threadIdx.x;
    PrivateStack priv;
    priv.lds = lds_stack + (tid & (kWalkLanes - 1));
    priv.lds_stride = kWalkLanes;
    priv.spill = spill + (size_t)blockIdx.x * kWalkLanes + (tid & (kWalkLanes - 1));
    priv.spill_stride = spill_stride;
    const int n_vec = (T.n_words + 3) >> 2;
    const int rows_padded = (batch + 7) & ~7;
    const int n_items = rows_padded * n_seg;

    for (int item = blockIdx.x; item < n_items; item += gridDim.x) {
        // blocks i, i+8, i+16, ... share an XCD: give them the segments of the same rows
        const int xcd = item & 7, slot = item >> 3;
        const int seg = slot % n_seg, b = (slot / n_seg) * 8 + xcd;
        if (b >= batch) continue;                      // uniform for the block
        const int32_t *row = data + (size_t)b * cap;
        if (tid < 64) {                                // wave 0: descent, uniform across lanes
            const int st = states[b];
            const int n = len[b];
            int top = -1;
            if (st < 0) {
                if (tid == 0) plan.mode = kRowDone;
            } else if (n < 1 || n > cap) {
                if (tid == 0) plan.mode = kRowEmpty;
            } else {
                DevConditionNode nd{};
                const bool guess = (unsigned)st < (unsigned)T.n_states;
                if (guess) nd = E.root_nodes[st];      // overlaps the stack load below
                const int xj = n - 1 - tid >= 0 ? row[n - 1 - tid] : -1;
                s_win[tid] = xj;
                top = __shfl(xj, 0);
                if ((unsigned)top >= (unsigned)T.n_states) {
                    if (tid == 0) plan.mode = kRowEmpty;
                } else {
                    if (!guess || top != st) nd = E.root_nodes[top];
                    plan_row(E, nd, s_win, n, [&](int k) { return row[n - 1 - k]; }, &plan, tid);
                }
            }
            if (tid == 0) { plan.top = top; plan.len = n; }
        }
        __syncthreads();
        const int v_lo = seg * seg_vec;                                    // first uint4 of the segment
        const int v_cnt = min(seg_vec, n_vec - v_lo);                      // may be <= 0 for a trailing segment
        const int w_lo = v_lo * 4;
        const bool vector_ok = (T.n_words & 3) == 0 && (reinterpret_cast<uintptr_t>(bitmask) & 15) == 0;
        build_and_store_row<kEdgeBlock, false, !kApply>(T, E, plan, bits4, v_lo, v_cnt, row, priv, bitmask + (size_t)b * T.n_words,
                                        vector_ok, tid);
        if (kApply) {
            // group g = 8 logits = one byte of the LDS bitmap (little endian)
            const uint8_t *mbytes = reinterpret_cast<const uint8_t *>(bits);
            uint16_t *lrow = logits + (size_t)b * row_stride;
            const int g_lo = w_lo * 4, g_cnt = max(v_cnt, 0) * 16;
            for (int g0 = tid; g0 < g_cnt; g0 += kEdgeBlock * 4) {
                uint32_t m[4];
                bool line[4];
                uint4 v[4];
#pragma unroll
                for (int u = 0; u < 4; ++u) {
                    const int gl = g0 + u * kEdgeBlock;
                    m[u] = gl < g_cnt ? mbytes[gl] : 0xFFu;
                    const int t0 = (g_lo + gl) * 8;
                    if (t0 >= T.n_tokens) m[u] = 0xFFu;                   // padding beyond the vocabulary
                    // a 128-byte line (the groups of eight consecutive lanes) is written whole or not at all:
                    // lines written in part cost the memory system far more than the bytes saved
                    const unsigned long long changed = __ballot(m[u] != 0xFFu);
                    line[u] = ((changed >> (tid & 56)) & 0xFFull) != 0 && t0 < T.n_tokens && gl < g_cnt;
                    if (line[u] && m[u] != 0u && t0 + 8 <= T.n_tokens)
                        v[u] = *reinterpret_cast<const uint4 *>(lrow + t0);
                }
#pragma unroll
                for (int u = 0; u < 4; ++u) {
                    const uint32_t mu = m[u];
                    if (!line[u]) continue;
                    const int t0 = (g_lo + g0 + u * kEdgeBlock) * 8;
                    uint16_t *p = lrow + t0;
                    if (t0 + 8 <= T.n_tokens) {
                        if (mu == 0u) {
                            *reinterpret_cast<uint4 *>(p) = make_uint4(kNegInfPair, kNegInfPair, kNegInfPair, kNegInfPair);
                        } else {
                            uint32_t *x = reinterpret_cast<uint32_t *>(&v[u]);
#pragma unroll
                            for (int k = 0; k < 4; ++k) {
                                if (!((mu >> (2 * k)) & 1u)) x[k] = (x[k] & 0xFFFF0000u) | 0xFF80u;
                                if (!((mu >> (2 * k + 1)) & 1u)) x[k] = (x[k] & 0x0000FFFFu) | 0xFF800000u;
                            }
                            *reinterpret_cast<uint4 *>(p) = v[u];
                        }
                    } else {
                        for (int k = 0; t0 + k < T.n_tokens; ++k)
                            if (!((mu >> k) & 1u)) p[k] = 0xFF80;
                    }
                }
            }
        }
        __syncthreads();
    }
}

}  // namespace

int walk_grid_blocks(int n_compute_units) { return 4 * n_compute_units; }
int edge_grid_blocks(int n_compute_units) { return 4 * n_compute_units; }
size_t edge_spill_entries(int grid_blocks, int max_depth) {
    const int deep = max_depth > kLdsDepth ? max_depth - kLdsDepth : 0;
    return (size_t)grid_blocks * kWalkLanes * (size_t)deep;
}
size_t edge_kernel_max_lds_words() { return (size_t)(64 * 1024 - 8 * 1024) / 4; }
int edge_row_stride_words(int n_words) { return (n_words + 3) & ~3; }

hipError_t launch_fill_mask_edges(const DevTables &T, const DevTokenEdges &E, const int32_t *states,
                                  const int32_t *data, const int32_t *len, int cap, int batch, uint32_t *bitmask,
                                  uint16_t *logits, int64_t row_stride, int32_t *spill, int grid_blocks,
                                  hipStream_t stream) {
    if (batch == 0) return hipSuccess;
    // Segments per row: enough items to give every block of the grid one, but segments of at
    // least 64 uint4 (8 KiB of mask = 16 Ki logits) so that the redundant descents stay cheap.
    const int n_vec = (T.n_words + 3) / 4;
    const int rows_padded = (batch + 7) & ~7;
    int want = (grid_blocks + rows_padded - 1) / rows_padded;
    int max_seg = (n_vec + 63) / 64;
    int n_seg = want < 1 ? 1 : (want > max_seg ? max_seg : want);
    int seg_vec = (n_vec + n_seg - 1) / n_seg;
    n_seg = (n_vec + seg_vec - 1) / seg_vec;
    const long long n_items = (long long)rows_padded * n_seg;
    const int grid = (int)(n_items < grid_blocks ? n_items : grid_blocks);
    const size_t lds = (size_t)seg_vec * sizeof(uint4);
    const size_t stride = (size_t)grid_blocks * kWalkLanes;
    if (logits)
        hipLaunchKernelGGL(fill_mask_edges_kernel<true>, dim3(grid), dim3(kEdgeBlock), lds, stream, T, E, states, data,
                           len, cap, batch, bitmask, logits, row_stride, n_seg, seg_vec, spill, stride);
    else
        hipLaunchKernelGGL(fill_mask_edges_kernel<false>, dim3(grid), dim3(kEdgeBlock), lds, stream, T, E, states, data,
                           len, cap, batch, bitmask, logits, row_stride, n_seg, seg_vec, spill, stride);
    return hipGetLastError();
}

size_t walk_spill_entries(int grid_blocks, int max_depth) {
    const int deep = max_depth > kLdsDepth ? max_depth - kLdsDepth : 0;
    return (size_t)grid_blocks * kBlock * (size_t)deep;
}

hipError_t launch_fill_mask_walk(const DevTables &T, const int32_t *states, const int32_t *data, const int32_t *len,
                                 int cap, int batch, uint32_t *bitmask, int32_t *spill, int grid_blocks,
                                 hipStream_t stream) {
    const long long n_items = (long long)batch * T.n_chunks;
    if (n_items == 0) return hipSuccess;
    const int grid = (int)(n_items < grid_blocks ? n_items : grid_blocks);
    hipLaunchKernelGGL(fill_mask_walk_kernel, dim3(grid), dim3(kBlock), 0, stream, T, states, data, len, cap, batch,
                       bitmask, spill, (size_t)grid_blocks * kBlock);
    return hipGetLastError();
}

}  // namespace pre3

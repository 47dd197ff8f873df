// gfx950 kernels of the batched token-mask path: token walk + bitmask pack, logits
// masking, and stack advance.  Wave64; no matrix cores (gather/branch-bound table walking).
#include <hip/hip_runtime.h>

#include "device_tables.hpp"
#include "launch.hpp"
#include "tables.hpp"

namespace pre3 {

namespace {

constexpr int kBlock = 256;            // threads per block of the walk kernel
constexpr int kLdsDepth = 16;          // private stack entries kept in LDS per lane
constexpr int kMaxChain = 1 << 20;     // reduction steps per input symbol before a walk gives up

// Private stack of one walk: the states pushed above the part of the sequence's stack that
// is still untouched.  The first kLdsDepth entries live in LDS (one column per lane), deeper
// ones in a global spill area (one column per resident lane), both indexed [depth][lane] so
// that lanes of a wave touch consecutive addresses.
struct PrivateStack {
    int32_t *lds;                      // already offset to this lane's column
    int32_t *spill;                    // already offset to this lane's column
    int lds_stride;
    size_t spill_stride;
    __device__ int32_t get(int i) const {
        return i < kLdsDepth ? lds[i * lds_stride] : spill[(size_t)(i - kLdsDepth) * spill_stride];
    }
    __device__ void set(int i, int32_t v) {
        if (i < kLdsDepth) lds[i * lds_stride] = v;
        else spill[(size_t)(i - kLdsDepth) * spill_stride] = v;
    }
};

enum FeedResult { kFed = 0, kRejected = 1, kOverflow = 2, kAccepted = 3 };

// Consumes one input symbol (`info` = byte class column | target offset << 8) from the configuration
//   row[0 .. base) ++ priv[0 .. d),  top = last entry,
// following reduction steps until an acceptance edge shifts the symbol.  Each reduction step
// pops, reads the exposed state (its stack-matching condition) and pushes the goto target.
// With kCheckCap the walk reports kOverflow exactly when a push would exceed `cap` entries.
template <bool kCheckCap>
__device__ __forceinline__ int feed(const DevTables &T, PrivateStack &priv, int info, int &base, int &d,
                                    int &top, const int32_t *__restrict__ row, int cap) {
    const int col = info & 0xFF, delta = info >> 8;    // byte class and per-byte target offset
    // A chain of reduction steps on one symbol is finite for LR(1) tables; the counter only
    // guarantees that a lane also terminates on tables or stacks that are not.
    for (int guard = 0;; ++guard) {
        if (guard > kMaxChain) { atomicAdd(T.fault, 1); return kRejected; }
        const uint32_t e = T.edge[(size_t)top * T.ncol + col];
        const uint32_t kind = e & kKindMask;
        if (kind == kError) return kRejected;
        if (kind == kAccept) return kAccepted;
        if (kind == kShift) {
            if (kCheckCap && base + d >= cap) return kOverflow;
            if (d >= T.max_depth) { atomicAdd(T.fault, 1); return kRejected; }
            top = (int)(e >> 2) + delta;
            priv.set(d++, top);
            return kFed;
        }
        const int n = (int)((e >> 2) & kMaxPop), nt = (int)(e >> kNtShift);
        int exposed = top;
        if (n > 0) {
            if (n <= d) {
                d -= n;
            } else {
                base -= n - d;
                d = 0;
                if (base < 1) return kRejected;          // only with a corrupted stack
            }
            if (d > 0) {
                exposed = priv.get(d - 1);
            } else {
                exposed = row[base - 1];
                if ((unsigned)exposed >= (unsigned)T.n_states) return kRejected;
            }
        }
        if (kCheckCap && base + d >= cap) return kOverflow;
        const int r = T.goto_row[exposed];
        if (r < 0) return kRejected;
        const int t = T.goto_flat[r + nt];
        if (t < 0) return kRejected;
        if (d >= T.max_depth) { atomicAdd(T.fault, 1); return kRejected; }
        top = t;
        priv.set(d++, t);
    }
}

// Walks the token at chunk-sorted position `pos` from the stack row[0..len).
__device__ __forceinline__ bool walk_token(const DevTables &T, PrivateStack &priv, int pos, int n_bytes,
                                           const int32_t *__restrict__ row, int len, int top0) {
    int base = len, d = 0, top = top0;
    uint32_t w = 0;
    for (int i = 0; i < n_bytes; ++i) {
        if ((i & 3) == 0) w = T.tok_words[(size_t)(i >> 2) * T.n_padded + pos];
        const int info = T.byte_info[w & 0xFF];
        w >>= 8;
        if (feed<false>(T, priv, info, base, d, top, row, 0) != kFed) return false;
    }
    return true;
}

__device__ __forceinline__ bool walk_end(const DevTables &T, PrivateStack &priv, const int32_t *__restrict__ row,
                                         int len, int top0) {
    int base = len, d = 0, top = top0;
    return feed<false>(T, priv, T.end_col, base, d, top, row, 0) == kAccepted;
}

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


// Walks token id `t` (bytes in id order) from the stack row[0..len).
__device__ __forceinline__ bool walk_token_id(const DevTables &T, PrivateStack &priv, int t,
                                              const int32_t *__restrict__ row, int len, int top0) {
    if (t == T.eos_id) return walk_end(T, priv, row, len, top0);
    int base = len, d = 0, top = top0;
    const int lo = T.voffsets[t], hi = T.voffsets[t + 1];
    if (hi <= lo) return false;
    for (int i = lo; i < hi; ++i)
        if (feed<false>(T, priv, T.byte_info[T.vbytes[i]], base, d, top, row, 0) != kFed) return false;
    return true;
}

constexpr int kEdgeBlock = 1024;       // threads per block of the token-edge kernel (one row per block)
constexpr int kWalkLanes = 256;        // lanes of a block that may walk tokens byte by byte
constexpr int kMaxPath = 64;           // condition-tree nodes on one descent
constexpr int kStackWindow = 64;       // top-of-stack entries staged in LDS

// Token mask from the precomputed token-level edges.  One block owns one sequence:
//   1. the top of the sequence's stack is staged in LDS and wave 0 descends the condition tree,
//      comparing the stack entry each node asks for with all of the node's condition states
//      at once (one lane per child, wave ballot);
//   2. the dense row of the deepest dense node on the path is copied into an LDS bitmap;
//   3. the delta lists of the nodes after it are ORed in, one lane per token id;
//   4. tokens the tree leaves undetermined (rare) are walked byte by byte by up to 256 lanes;
//   5. the bitmap is stored with coalesced writes.
// A stack the tree has no answer for falls back to walking every token.
__global__ __launch_bounds__(kEdgeBlock) void fill_mask_edges_kernel(
    DevTables T, DevTokenEdges E, const int32_t *__restrict__ states, const int32_t *__restrict__ data,
    const int32_t *__restrict__ len, int cap, int batch, uint32_t *__restrict__ bitmask, int32_t *spill,
    size_t spill_stride) {
    extern __shared__ uint32_t bits[];                 // n_words
    __shared__ int32_t s_stack[kStackWindow];
    __shared__ int32_t s_path[kMaxPath];
    __shared__ int32_t s_npath, s_start, s_mode;
    __shared__ int32_t lds_stack[kLdsDepth * kWalkLanes];
    const int tid = threadIdx.x;
    PrivateStack priv;
    priv.lds = lds_stack + (tid & (kWalkLanes - 1));
    priv.lds_stride = kWalkLanes;
    priv.spill = spill + (size_t)blockIdx.x * kWalkLanes + (tid & (kWalkLanes - 1));
    priv.spill_stride = spill_stride;
    enum { kFast = 0, kWalkAll = 1, kEmpty = 2 };

    for (int b = blockIdx.x; b < batch; b += gridDim.x) {
        const int32_t *row = data + (size_t)b * cap;
        const int n = len[b];
        const bool done = states[b] < 0;
        const bool valid = !done && n >= 1 && n <= cap;
        if (tid < kStackWindow) s_stack[tid] = (valid && n - 1 - tid >= 0) ? row[n - 1 - tid] : -1;
        __syncthreads();
        if (tid < 64) {                                // wave 0: descent, uniform across lanes
            int mode = kFast, npath = 0, start = 0;
            const int top = s_stack[0];
            if (!valid || (unsigned)top >= (unsigned)T.n_states) {
                mode = kEmpty;
            } else {
                int node = E.root_of_state[top];
                for (;;) {
                    const DevConditionNode nd = E.nodes[node];
                    if (tid == 0) s_path[npath] = node;
                    if (nd.dense_row >= 0) start = npath;
                    ++npath;
                    if (nd.child_count == 0) {
                        if (nd.walk_count < 0) mode = kWalkAll;
                        break;
                    }
                    if (nd.known >= n || npath >= kMaxPath) { mode = kWalkAll; break; }
                    const int x = nd.known < kStackWindow ? s_stack[nd.known] : row[n - 1 - nd.known];
                    int next = -1;
                    for (int c0 = 0; c0 < nd.child_count; c0 += 64) {
                        const int i = c0 + tid;
                        const bool hit = i < nd.child_count && E.child_state[nd.child_begin + i] == x;
                        const unsigned long long m = __ballot(hit);
                        if (m) { next = E.child_node[nd.child_begin + c0 + __ffsll((long long)m) - 1]; break; }
                    }
                    if (next < 0) { mode = kWalkAll; break; }
                    node = next;
                }
            }
            if (tid == 0) { s_npath = npath; s_start = start; s_mode = mode; }
        }
        __syncthreads();
        const int mode = s_mode, npath = s_npath, start = s_start;
        int dense = -1;
        if (mode == kFast) dense = E.nodes[s_path[start]].dense_row;
        if (dense >= 0) {
            const uint32_t *src = E.dense_rows + (size_t)dense * T.n_words;
            for (int w = tid; w < T.n_words; w += kEdgeBlock) bits[w] = src[w];
        } else {
            for (int w = tid; w < T.n_words; w += kEdgeBlock) bits[w] = 0;
        }
        __syncthreads();
        const int top0 = s_stack[0];
        if (mode == kFast) {
            for (int i = start; i < npath; ++i) {
                const DevConditionNode nd = E.nodes[s_path[i]];
                for (int k = tid; k < nd.delta_count; k += kEdgeBlock) {
                    const int t = E.delta_ids[nd.delta_begin + k];
                    atomicOr(&bits[t >> 5], 1u << (t & 31));
                }
            }
            const DevConditionNode last = E.nodes[s_path[npath - 1]];
            if (tid < kWalkLanes)
                for (int k = tid; k < last.walk_count; k += kWalkLanes) {
                    const int t = E.walk_ids[last.walk_begin + k];
                    if (walk_token_id(T, priv, t, row, n, top0)) atomicOr(&bits[t >> 5], 1u << (t & 31));
                }
        } else if (mode == kWalkAll) {
            if (tid < kWalkLanes)
                for (int t = tid; t < T.n_tokens; t += kWalkLanes)
                    if (walk_token_id(T, priv, t, row, n, top0)) atomicOr(&bits[t >> 5], 1u << (t & 31));
        } else if (done && tid == 0) {
            bits[T.eos_id >> 5] = 1u << (T.eos_id & 31);
        }
        __syncthreads();
        uint32_t *dst = bitmask + (size_t)b * T.n_words;
        for (int w = tid; w < T.n_words; w += kEdgeBlock) dst[w] = bits[w];
        __syncthreads();
    }
}

// ---------------------------------------------------------------------------- apply

constexpr uint32_t kNegInfPair = 0xFF80FF80u;

// One lane per 8 consecutive logits (16 bytes) of one row: fully allowed groups are not
// touched, fully masked groups are overwritten without being read, mixed groups are patched.
__global__ __launch_bounds__(256) void apply_mask_vec8_kernel(uint16_t *__restrict__ logits,
                                                               const uint32_t *__restrict__ bitmask, int batch,
                                                               int vocab, int64_t row_stride, int n_words) {
    const int groups = (vocab + 7) >> 3;
    const int64_t total = (int64_t)batch * groups;
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < total;
         i += (int64_t)gridDim.x * blockDim.x) {
        const int b = (int)(i / groups), g = (int)(i - (int64_t)b * groups);
        const uint32_t m = (bitmask[(size_t)b * n_words + (g >> 2)] >> ((g & 3) * 8)) & 0xFFu;
        if (m == 0xFFu) continue;
        uint16_t *p = logits + (size_t)b * row_stride + (size_t)g * 8;
        if (g * 8 + 8 <= vocab) {
            uint4 *q = reinterpret_cast<uint4 *>(p);
            if (m == 0) {
                *q = make_uint4(kNegInfPair, kNegInfPair, kNegInfPair, kNegInfPair);
            } else {
                uint4 v = *q;
                uint32_t *x = reinterpret_cast<uint32_t *>(&v);
#pragma unroll
                for (int k = 0; k < 4; ++k) {
                    if (!((m >> (2 * k)) & 1u)) x[k] = (x[k] & 0xFFFF0000u) | 0xFF80u;
                    if (!((m >> (2 * k + 1)) & 1u)) x[k] = (x[k] & 0x0000FFFFu) | 0xFF800000u;
                }
                *q = v;
            }
        } else {
            for (int k = 0; g * 8 + k < vocab; ++k)
                if (!((m >> k) & 1u)) p[k] = 0xFF80;
        }
    }
}

// Fallback for rows that are not 16-byte aligned: one lane per logit.
__global__ __launch_bounds__(256) void apply_mask_scalar_kernel(uint16_t *__restrict__ logits,
                                                                 const uint32_t *__restrict__ bitmask, int batch,
                                                                 int vocab, int64_t row_stride, int n_words) {
    const int64_t total = (int64_t)batch * vocab;
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < total;
         i += (int64_t)gridDim.x * blockDim.x) {
        const int b = (int)(i / vocab), t = (int)(i - (int64_t)b * vocab);
        if (!((bitmask[(size_t)b * n_words + (t >> 5)] >> (t & 31)) & 1u))
            logits[(size_t)b * row_stride + t] = 0xFF80;
    }
}

// -------------------------------------------------------------------------- advance

// One lane per sequence.  The token is walked on a private overlay exactly like in the mask
// kernel; only a walk that succeeds is committed to the sequence's stack.
__global__ __launch_bounds__(64) void advance_kernel(DevTables T, const int32_t *__restrict__ tokens,
                                                     int32_t *__restrict__ states, int32_t *__restrict__ data,
                                                     int32_t *__restrict__ len, int cap, int batch,
                                                     int32_t *__restrict__ err, int32_t *scratch) {
    __shared__ int32_t lds_stack[kLdsDepth * 64];
    const int b = blockIdx.x * 64 + threadIdx.x;
    if (b >= batch) return;
    const int t = tokens[b];
    if (t < 0) { err[b] = 0; return; }
    int32_t *row = data + (size_t)b * cap;
    const int n = len[b];
    int top = -1;
    if (states[b] >= 0 && n >= 1 && n <= cap) top = row[n - 1];
    if (t >= T.n_tokens || (unsigned)top >= (unsigned)T.n_states) { err[b] = 1; return; }

    PrivateStack priv;
    priv.lds = lds_stack + threadIdx.x;
    priv.lds_stride = 64;
    priv.spill = scratch + b;
    priv.spill_stride = (size_t)batch;
    int base = n, d = 0;
    if (t == T.eos_id) {
        if (feed<false>(T, priv, T.end_col, base, d, top, row, 0) == kAccepted) { states[b] = -1; err[b] = 0; }
        else err[b] = 1;
        return;
    }
    const int lo = T.voffsets[t], hi = T.voffsets[t + 1];
    int rc = hi > lo ? kFed : kRejected;
    for (int i = lo; i < hi && rc == kFed; ++i)
        rc = feed<true>(T, priv, T.byte_info[T.vbytes[i]], base, d, top, row, cap);
    if (rc != kFed) { err[b] = rc == kOverflow ? 2 : 1; return; }
    for (int i = 0; i < d; ++i) row[base + i] = priv.get(i);
    len[b] = base + d;
    states[b] = top;
    err[b] = 0;
}

}  // namespace

int walk_grid_blocks(int n_compute_units) { return 4 * n_compute_units; }
int edge_grid_blocks(int n_compute_units) { return 2 * n_compute_units; }
size_t edge_spill_entries(int grid_blocks, int max_depth) {
    const int deep = max_depth > kLdsDepth ? max_depth - kLdsDepth : 0;
    return (size_t)grid_blocks * kWalkLanes * (size_t)deep;
}
size_t edge_kernel_max_lds_words() { return (size_t)(64 * 1024 - 24 * 1024) / 4; }

hipError_t launch_fill_mask_edges(const DevTables &T, const DevTokenEdges &E, const int32_t *states,
                                  const int32_t *data, const int32_t *len, int cap, int batch, uint32_t *bitmask,
                                  int32_t *spill, int grid_blocks, hipStream_t stream) {
    if (batch == 0) return hipSuccess;
    const int grid = batch < grid_blocks ? batch : grid_blocks;
    hipLaunchKernelGGL(fill_mask_edges_kernel, dim3(grid), dim3(kEdgeBlock), (size_t)T.n_words * sizeof(uint32_t),
                       stream, T, E, states, data, len, cap, batch, bitmask, spill, (size_t)grid_blocks * kWalkLanes);
    return hipGetLastError();
}
size_t walk_spill_entries(int grid_blocks, int max_depth) {
    const int deep = max_depth > kLdsDepth ? max_depth - kLdsDepth : 0;
    return (size_t)grid_blocks * kBlock * (size_t)deep;
}
size_t advance_scratch_entries(int batch, int max_depth) {
    const int deep = max_depth > kLdsDepth ? max_depth - kLdsDepth : 0;
    return (size_t)batch * (size_t)deep;
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

hipError_t launch_apply_mask(uint16_t *logits, const uint32_t *bitmask, int batch, int vocab, int64_t row_stride,
                             hipStream_t stream) {
    if (batch == 0 || vocab == 0) return hipSuccess;
    const int n_words = (vocab + 31) / 32;
    const bool aligned = (reinterpret_cast<uintptr_t>(logits) % 16 == 0) && (row_stride % 8 == 0);
    if (aligned) {
        const int64_t total = (int64_t)batch * ((vocab + 7) / 8);
        const int64_t want = (total + 255) / 256;
        const int grid = (int)(want < 65536 ? want : 65536);
        hipLaunchKernelGGL(apply_mask_vec8_kernel, dim3(grid), dim3(256), 0, stream, logits, bitmask, batch, vocab,
                           row_stride, n_words);
    } else {
        const int64_t total = (int64_t)batch * vocab;
        const int64_t want = (total + 255) / 256;
        const int grid = (int)(want < 65536 ? want : 65536);
        hipLaunchKernelGGL(apply_mask_scalar_kernel, dim3(grid), dim3(256), 0, stream, logits, bitmask, batch, vocab,
                           row_stride, n_words);
    }
    return hipGetLastError();
}

hipError_t launch_advance(const DevTables &T, const int32_t *tokens, int32_t *states, int32_t *data, int32_t *len,
                          int cap, int batch, int32_t *err, int32_t *scratch, hipStream_t stream) {
    if (batch == 0) return hipSuccess;
    hipLaunchKernelGGL(advance_kernel, dim3((batch + 63) / 64), dim3(64), 0, stream, T, tokens, states, data, len,
                       cap, batch, err, scratch);
    return hipGetLastError();
}

}  // namespace pre3

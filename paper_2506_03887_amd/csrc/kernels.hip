// gfx950 kernels of the batched token-mask path: token walk + bitmask pack, logits
// masking, and stack advance.  Wave64; no matrix cores (gather/branch-bound table walking).
#include <hip/hip_runtime.h>

#include "device_tables.hpp"
#include "launch.hpp"
#include "symbol_edges.hpp"
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

// Table look-ups.  In a wave that runs ONE walk (advance), every index is the same in all lanes:
// the index is moved to a scalar register and the read-only table is addressed through the
// constant address space, which lets the compiler use scalar loads served by the scalar cache
// (a chain of dependent look-ups then costs a fraction of the vector-memory latency).  The
// tables are never written by a kernel, so the scalar cache cannot hold stale data.
template <typename V>
using ConstPtr = const __attribute__((address_space(4))) V *;

typedef int NativeInt2 __attribute__((ext_vector_type(2)));
typedef int NativeInt4 __attribute__((ext_vector_type(4)));

template <bool kUniform, typename V>
__device__ __forceinline__ V table(const V *p, int i) {
    if (kUniform) return ((ConstPtr<V>)p)[__builtin_amdgcn_readfirstlane(i)];
    return p[i];
}
template <bool kUniform>
__device__ __forceinline__ int2 table(const int2 *p, int i) {
    if (kUniform) {
        const NativeInt2 v = ((ConstPtr<NativeInt2>)p)[__builtin_amdgcn_readfirstlane(i)];
        return make_int2(v.x, v.y);
    }
    return p[i];
}
template <bool kUniform>
__device__ __forceinline__ int4 table(const int4 *p, int i) {
    if (kUniform) {
        const NativeInt4 v = ((ConstPtr<NativeInt4>)p)[__builtin_amdgcn_readfirstlane(i)];
        return make_int4(v.x, v.y, v.z, v.w);
    }
    return p[i];
}
template <bool kUniform>
__device__ __forceinline__ int uni(int v) {
    return kUniform ? __builtin_amdgcn_readfirstlane(v) : v;
}

// The sequence's stack as the walk sees it: row[0..n), optionally with its top `kWindow` entries
// staged in LDS (win[k] = entry k below the top).
constexpr int kWindow = 64;
struct StackView {
    const int32_t *row;
    const int32_t *win;
    int n;
    __device__ int32_t at(int idx) const {
        const int k = n - 1 - idx;
        return (win && k < kWindow) ? win[k] : row[idx];
    }
};

// Consumes one input symbol (`info` = byte class column | target offset << 8) from the configuration
//   row[0 .. base) ++ priv[0 .. d),  top = last entry.
// First the merged reduction edge is looked up: starting at the top state's condition node, the
// stack entry each node names is matched against the node's condition states until a node holds
// the symbol's effect (truncate, push list ending in the acceptance edge's target).  Where no
// merged edge was precomputed the per-step edges are followed: each reduction step pops, reads
// the exposed state (its stack-matching condition) and pushes the goto target, until an
// acceptance edge shifts the symbol.
// With kCheckCap the walk reports kOverflow exactly when a push would exceed `cap` entries.
template <bool kCheckCap, bool kUniform = false>
__device__ __forceinline__ int feed(const DevTables &T, PrivateStack &priv, int info, int &base, int &d,
                                    int &top, int &tree, const StackView &row, int cap, int *run_node = nullptr) {
    const int col = info & 0xFF, delta = info >> 8;    // byte class and per-byte target offset
    // `tree` names the condition tree of the top state (states that behave alike share one, and all
    // bytes of a class shift to states of one kind, so the kind after an edge is stored with it)
    if (T.sym_cell) {
        int node = tree;
        int4 nd = table<kUniform>(T.sym_nodes, node);
        int4 cell = table<kUniform>(T.sym_cell, node * T.ncol + col);
        for (int level = 0; level < 64; ++level) {
            const int code = cell.x;
            if (code >= 0) {
                // the edge: truncate to (len - known + 1) entries, push np states (the last one is the
                // acceptance edge's target); `peak` bounds the height reached on the way
                int known, peak, np, same, after;
                int4 push4;
                if (code & kCellInline) {
                    known = code & 0xFF;
                    peak = ((code >> 8) & 0xFF) - 128;
                    np = (code >> 16) & 3;
                    same = code & kCellSameShape;
                    after = cell.y;
                    push4 = make_int4(cell.z, cell.w, 0, 0);
                } else {
                    // record in the pool: known, peak, n_push, kind after; push[0..3] ride along
                    const int4 hdr = table<kUniform>(reinterpret_cast<const int4 *>(T.sym_pool), code >> 2);
                    push4 = table<kUniform>(reinterpret_cast<const int4 *>(T.sym_pool), (code >> 2) + 1);
                    known = hdr.x;
                    peak = hdr.y;
                    np = hdr.z & kEffPushMask;
                    same = hdr.z & kEffSameShape;
                    after = hdr.w;
                }
                const int pops = known - 1;
                if (kCheckCap && base + d + peak >= cap) return kOverflow;
                if (pops <= d) {
                    d -= pops;
                } else {
                    base -= pops - d;
                    d = 0;
                    if (base < 1) return kRejected;              // only with a corrupted stack
                }
                if (d + np > T.max_depth) { if (!kUniform || (threadIdx.x & 63) == 0) atomicAdd(T.fault, 1); return kRejected; }
                for (int i = 0; i < np; ++i) {
                    int v;
                    if (i < 4) v = i == 0 ? push4.x : i == 1 ? push4.y : i == 2 ? push4.z : push4.w;
                    else v = table<kUniform>(T.sym_pool, code + 4 + i);
                    if (i == np - 1) v += delta;
                    priv.set(d++, v);
                    top = v;
                }
                if (run_node) *run_node = (same && after == tree) ? node : -1;
                tree = after;
                return kFed;
            }
            if (code == kEffNone) return kRejected;
            if (code == kEffAccept) return kAccepted;
            if (code == kEffStepwise) break;
            int x;                                             // the entry nd.x below the top
            if (nd.x < d) {
                x = priv.get(d - 1 - nd.x);
            } else {
                const int idx = base - 1 - (nd.x - d);
                if (idx < 0) break;
                x = row.at(idx);
            }
            x = uni<kUniform>(x);
            int next = -1;
            if (kUniform) {
                // all lanes run this walk: lane j fetches condition j together with child j's node
                // record and cell, so one round of loads both picks the child and enters it
                const int lane = threadIdx.x & 63;
                int4 cnd = make_int4(0, 0, 0, 0), ccell = make_int4(kEffStepwise, 0, 0, 0);
                int cstate = -2;
                for (int c0 = 0; c0 < nd.z && next < 0; c0 += 64) {
                    const int j = c0 + lane;
                    if (j < nd.z) {
                        cstate = T.sym_pairs[nd.y + j].x;
                        cnd = T.sym_nodes[nd.w + j];
                        ccell = T.sym_cell[(nd.w + j) * T.ncol + col];
                    }
                    const unsigned long long m = __ballot(j < nd.z && cstate == x);
                    if (m) {
                        const int src = __ffsll((long long)m) - 1;
                        next = nd.w + c0 + src;
                        nd = make_int4(uni<true>(__shfl(cnd.x, src)), uni<true>(__shfl(cnd.y, src)),
                                       uni<true>(__shfl(cnd.z, src)), uni<true>(__shfl(cnd.w, src)));
                        cell = make_int4(uni<true>(__shfl(ccell.x, src)), uni<true>(__shfl(ccell.y, src)),
                                         uni<true>(__shfl(ccell.z, src)), uni<true>(__shfl(ccell.w, src)));
                    }
                }
                if (next < 0) break;
                node = next;
            } else {
                for (int i = 0; i < nd.z; ++i) {
                    const int2 pr = T.sym_pairs[nd.y + i];
                    if (pr.x == x) next = pr.y;
                }
                if (next < 0) break;
                node = next;
                nd = T.sym_nodes[node];
                cell = T.sym_cell[node * T.ncol + col];
            }
        }
    }
    // A chain of reduction steps on one symbol is finite for LR(1) tables; the counter only
    // guarantees that a lane also terminates on tables or stacks that are not.
    for (int guard = 0;; ++guard) {
        if (guard > kMaxChain) { atomicAdd(T.fault, 1); return kRejected; }
        const uint32_t e = table<kUniform>(T.edge, top * T.ncol + col);
        const uint32_t kind = e & kKindMask;
        if (kind == kError) return kRejected;
        if (kind == kAccept) return kAccepted;
        if (kind == kShift) {
            if (kCheckCap && base + d >= cap) return kOverflow;
            if (d >= T.max_depth) { atomicAdd(T.fault, 1); return kRejected; }
            top = (int)(e >> 2) + delta;
            priv.set(d++, top);
            if (T.state_kind) tree = table<kUniform>(T.state_kind, top);
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
                exposed = row.at(base - 1);
                if ((unsigned)exposed >= (unsigned)T.n_states) return kRejected;
            }
            exposed = uni<kUniform>(exposed);
        }
        if (kCheckCap && base + d >= cap) return kOverflow;
        const int r = table<kUniform>(T.goto_row, exposed);
        if (r < 0) return kRejected;
        const int t = table<kUniform>(T.goto_flat, r + nt);
        if (t < 0) return kRejected;
        if (d >= T.max_depth) { atomicAdd(T.fault, 1); return kRejected; }
        top = t;
        priv.set(d++, t);
    }
}

// After a self-similar edge found at condition node `node` (the stack kept its shape and the kind
// of its top), every following symbol whose edge at the same node is again self-similar merely
// replaces the top of the stack.  Each of the 64 lanes examines one upcoming byte
// (infos[first + lane], staged in LDS); the run ends at the first byte that is not such an edge.
// Returns the number of bytes consumed; the last one's target becomes the new top.
template <bool kCheckCap>
__device__ __forceinline__ int apply_run(const DevTables &T, PrivateStack &priv, const int32_t *infos, int first,
                                         int n_bytes, int node, int tree, int base, int d, int &top, int cap) {
    const int i = first + (threadIdx.x & 63);
    bool ok = i < n_bytes && i < 64;
    int new_top = 0;
    if (ok) {
        const int info = infos[i];
        const int4 cell = T.sym_cell[node * T.ncol + (info & 0xFF)];
        const int code = cell.x;
        ok = code >= 0;
        if (ok && (code & kCellInline)) {
            ok = (code & kCellSameShape) && cell.y == tree && (!kCheckCap || base + d + ((code >> 8) & 0xFF) - 128 < cap);
            new_top = (((code >> 16) & 3) == 1 ? cell.z : cell.w) + (info >> 8);
        } else if (ok) {
            const int4 hdr = *reinterpret_cast<const int4 *>(T.sym_pool + code);
            ok = (hdr.z & kEffSameShape) && hdr.w == tree && (!kCheckCap || base + d + hdr.y < cap);
            if (ok) new_top = T.sym_pool[code + 4 + (hdr.z & kEffPushMask) - 1] + (info >> 8);
        }
    }
    const unsigned long long bad = __ballot(!ok);
    const int run = bad ? __ffsll((long long)bad) - 1 : 64;
    if (run > 0) {
        top = __builtin_amdgcn_readfirstlane(__shfl(new_top, run - 1));
        priv.set(d - 1, top);
    }
    return run;
}

// Walks the token at chunk-sorted position `pos` from the stack row[0..len).
__device__ __forceinline__ bool walk_token(const DevTables &T, PrivateStack &priv, int pos, int n_bytes,
                                           const int32_t *__restrict__ row, int len, int top0) {
    int base = len, d = 0, top = top0, kind = T.state_kind ? T.state_kind[top0] : 0;
    uint32_t w = 0;
    for (int i = 0; i < n_bytes; ++i) {
        if ((i & 3) == 0) w = T.tok_words[(size_t)(i >> 2) * T.n_padded + pos];
        const int info = T.byte_info[w & 0xFF];
        w >>= 8;
        if (feed<false>(T, priv, info, base, d, top, kind, StackView{row, nullptr, len}, 0) != kFed) return false;
    }
    return true;
}

__device__ __forceinline__ bool walk_end(const DevTables &T, PrivateStack &priv, const int32_t *__restrict__ row,
                                         int len, int top0) {
    int base = len, d = 0, top = top0, kind = T.state_kind ? T.state_kind[top0] : 0;
    return feed<false>(T, priv, T.end_col, base, d, top, kind, StackView{row, nullptr, len}, 0) == kAccepted;
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
    int base = len, d = 0, top = top0, kind = T.state_kind ? T.state_kind[top0] : 0;
    const int lo = T.voffsets[t], hi = T.voffsets[t + 1];
    if (hi <= lo) return false;
    for (int i = lo; i < hi; ++i)
        if (feed<false>(T, priv, T.byte_info[T.vbytes[i]], base, d, top, kind, StackView{row, nullptr, len}, 0) != kFed) return false;
    return true;
}

constexpr int kMaxPath = 64;           // delta lists ORed on one descent
enum RowMode { kRowFast = 0, kRowWalkAll = 1, kRowEmpty = 2, kRowDone = 3 };

// How one sequence's mask row is assembled; lives in LDS, written by the wave that descends.
struct RowPlan {
    int32_t seg_begin[kMaxPath], seg_count[kMaxPath];   // delta lists to OR in
    int32_t nseg;
    int32_t dense;            // dense row to start from, or -1 (start from zero)
    int32_t mode;             // RowMode
    int32_t walk_begin, walk_count;                     // tokens left to the byte-by-byte walk
    int32_t top, len;         // the stack the row belongs to
};

// Descent of the condition tree of the token-level edges, run by all 64 lanes of one wave with
// identical values.  `win[k]` (LDS) is the stack entry k below the top for k < kWindow, deeper(k)
// any entry below that; `n` the stack length; `nd` the root record of the top state.  Each node
// names the entry it tests; lane j fetches condition state j TOGETHER with child j's record
// (children are stored consecutively), so one round of loads both verifies all of the node's
// stack-matching conditions at once (wave ballot) and enters the matching child.
template <typename Deeper>
__device__ __forceinline__ void plan_row(const DevTokenEdges &E, DevConditionNode nd, const int32_t *win, int n,
                                         Deeper deeper, RowPlan *plan, int lane) {
    int mode = kRowFast, nseg = 0, dense = -1, walk_begin = 0, walk_count = 0;
    for (;;) {
        if (nd.dense_row >= 0) {               // holds everything allowed so far on this path
            dense = nd.dense_row;
            nseg = 0;
        } else if (nd.delta_count > 0) {
            if (lane == 0) { plan->seg_begin[nseg] = nd.delta_begin; plan->seg_count[nseg] = nd.delta_count; }
            ++nseg;
        }
        if (nd.child_count == 0) {
            walk_begin = nd.a;
            walk_count = nd.b;
            if (walk_count < 0) mode = kRowWalkAll;
            break;
        }
        if (nd.known >= n || nseg >= kMaxPath) { mode = kRowWalkAll; break; }
        const int x = nd.known < kWindow ? win[nd.known] : deeper(nd.known);
        bool found = false;
        for (int c0 = 0; c0 < nd.child_count && !found; c0 += 64) {
            const int j = c0 + lane;
            int cstate = -2;
            DevConditionNode c{};
            if (j < nd.child_count) {
                cstate = E.child_state[nd.a + j];
                c = E.nodes[nd.b + j];
            }
            const unsigned long long m = __ballot(cstate == x);
            if (m) {
                const int src = __ffsll((long long)m) - 1;
                nd.known = __shfl(c.known, src);
                nd.child_count = __shfl(c.child_count, src);
                nd.a = __shfl(c.a, src);
                nd.b = __shfl(c.b, src);
                nd.dense_row = __shfl(c.dense_row, src);
                nd.delta_begin = __shfl(c.delta_begin, src);
                nd.delta_count = __shfl(c.delta_count, src);
                found = true;
            }
        }
        if (!found) { mode = kRowWalkAll; break; }
    }
    if (lane == 0) {
        plan->nseg = nseg;
        plan->dense = dense;
        plan->mode = mode;
        plan->walk_begin = walk_begin;
        plan->walk_count = walk_count;
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
        const int mode = plan.mode;
        const int v_lo = seg * seg_vec;                                    // first uint4 of the segment
        const int v_cnt = min(seg_vec, n_vec - v_lo);                      // may be <= 0 for a trailing segment
        const int w_lo = v_lo * 4, w_hi = w_lo + max(v_cnt, 0) * 4;        // mask words [w_lo, w_hi)
        if (mode == kRowFast && plan.dense >= 0) {
            const uint4 *src = reinterpret_cast<const uint4 *>(E.dense_rows) + (size_t)plan.dense * n_vec + v_lo;
            for (int w = tid; w < v_cnt; w += kEdgeBlock) bits4[w] = src[w];
        } else {
            for (int w = tid; w < v_cnt; w += kEdgeBlock) bits4[w] = make_uint4(0, 0, 0, 0);
        }
        __syncthreads();
        if (mode == kRowFast) {
            const int nseg = plan.nseg;
            for (int i = 0; i < nseg; ++i) {
                const int32_t *ids = E.delta_ids + plan.seg_begin[i];
                const int cnt = plan.seg_count[i];
                for (int k = tid; k < cnt; k += kEdgeBlock) {
                    const int t = ids[k], w = t >> 5;
                    if (w >= w_lo && w < w_hi) atomicOr(&bits[w - w_lo], 1u << (t & 31));
                }
            }
            const int wc = plan.walk_count;
            if (wc > 0 && tid < kWalkLanes) {
                const int n = plan.len, top0 = plan.top;
                for (int k = tid; k < wc; k += kWalkLanes) {
                    const int t = E.walk_ids[plan.walk_begin + k], w = t >> 5;
                    if (w >= w_lo && w < w_hi && walk_token_id(T, priv, t, row, n, top0))
                        atomicOr(&bits[w - w_lo], 1u << (t & 31));
                }
            }
        } else if (mode == kRowWalkAll) {
            if (tid < kWalkLanes) {
                const int n = plan.len, top0 = plan.top;
                const int t_hi = min(T.n_tokens, w_hi * 32);
                for (int t = w_lo * 32 + tid; t < t_hi; t += kWalkLanes)
                    if (walk_token_id(T, priv, t, row, n, top0)) atomicOr(&bits[(t >> 5) - w_lo], 1u << (t & 31));
            }
        } else if (mode == kRowDone && tid == 0) {
            const int w = T.eos_id >> 5;
            if (w >= w_lo && w < w_hi) bits[w - w_lo] = 1u << (T.eos_id & 31);
        }
        __syncthreads();
        uint32_t *dst = bitmask + (size_t)b * T.n_words;
        if ((T.n_words & 3) == 0 && (reinterpret_cast<uintptr_t>(bitmask) & 15) == 0) {
            uint4 *dst4 = reinterpret_cast<uint4 *>(dst) + v_lo;
            for (int w = tid; w < v_cnt; w += kEdgeBlock) dst4[w] = bits4[w];
        } else {
            for (int w = w_lo + tid; w < min(w_hi, T.n_words); w += kEdgeBlock) dst[w] = bits[w - w_lo];
        }
        if (kApply) {
            // group g = 8 logits = one byte of the LDS bitmap (little endian)
            const uint8_t *mbytes = reinterpret_cast<const uint8_t *>(bits);
            uint16_t *lrow = logits + (size_t)b * row_stride;
            const int g_lo = w_lo * 4, g_cnt = max(v_cnt, 0) * 16;
            for (int g0 = tid; g0 < g_cnt; g0 += kEdgeBlock * 4) {
                uint32_t m[4];
                uint4 v[4];
#pragma unroll
                for (int u = 0; u < 4; ++u) {
                    const int gl = g0 + u * kEdgeBlock;
                    m[u] = gl < g_cnt ? mbytes[gl] : 0xFFu;
                    const int t0 = (g_lo + gl) * 8;
                    if (t0 >= T.n_tokens) m[u] = 0xFFu;                   // padding beyond the vocabulary
                    if (m[u] != 0xFFu && m[u] != 0u && t0 + 8 <= T.n_tokens)
                        v[u] = *reinterpret_cast<const uint4 *>(lrow + t0);
                }
#pragma unroll
                for (int u = 0; u < 4; ++u) {
                    const uint32_t mu = m[u];
                    if (mu == 0xFFu) continue;
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

// ---------------------------------------------------------------------------- apply

// 16-byte accesses marked non-temporal: the logits pass through once, and lines marked this way
// are the first to leave L2, so the automaton's tables survive the pass for the next kernel.
typedef unsigned int NativeUint4 __attribute__((ext_vector_type(4)));
__device__ __forceinline__ uint4 stream_load(const uint16_t *p) {
    const NativeUint4 x = __builtin_nontemporal_load(reinterpret_cast<const NativeUint4 *>(p));
    return make_uint4(x.x, x.y, x.z, x.w);
}
__device__ __forceinline__ void stream_store(uint4 v, uint16_t *p) {
    const NativeUint4 x = {v.x, v.y, v.z, v.w};
    __builtin_nontemporal_store(x, reinterpret_cast<NativeUint4 *>(p));
}

constexpr int kApplyBlock = 256;
constexpr int kApplyUnroll = 1;        // 16-byte groups per lane (measured: more waves beat more loads per lane)
constexpr int kApplySpan = kApplyBlock * kApplyUnroll * 8;   // logits per block

// blockIdx.y = row, blockIdx.x = span of kApplySpan logits.  A lane owns kApplyUnroll groups of 8
// consecutive logits (16 bytes), one per pass, so that every pass of a wave is one contiguous
// 1 KiB access.  Fully allowed groups are not touched, fully masked groups are overwritten
// without being read, mixed groups are read, patched and written back.  In-place
// read-modify-write of the logits streams at about 5.4 TB/s on MI355X whatever the unroll or
// block size; one group per lane was the fastest.
__global__ __launch_bounds__(kApplyBlock) void apply_mask_vec8_kernel(uint16_t *__restrict__ logits,
                                                                     const uint32_t *__restrict__ bitmask,
                                                                     int vocab, int64_t row_stride, int n_words) {
    const int b = blockIdx.y;
    const int groups = (vocab + 7) >> 3;
    const int g0 = blockIdx.x * (kApplyBlock * kApplyUnroll) + threadIdx.x;
    const uint8_t *mrow = reinterpret_cast<const uint8_t *>(bitmask + (size_t)b * n_words);
    uint16_t *lrow = logits + (size_t)b * row_stride;
    uint32_t m[kApplyUnroll];
    uint4 v[kApplyUnroll];
#pragma unroll
    for (int u = 0; u < kApplyUnroll; ++u) {
        const int g = g0 + u * kApplyBlock;
        m[u] = g < groups ? mrow[g] : 0xFFu;            // little endian: byte g of the row = bits of group g
    }
#pragma unroll
    for (int u = 0; u < kApplyUnroll; ++u) {                // all loads of the lane are in flight together
        const int g = g0 + u * kApplyBlock;
        if (m[u] != 0xFFu && m[u] != 0u && g * 8 + 8 <= vocab) v[u] = stream_load(lrow + (size_t)g * 8);
    }
#pragma unroll
    for (int u = 0; u < kApplyUnroll; ++u) {
        const int g = g0 + u * kApplyBlock;
        const uint32_t mu = m[u];
        if (mu == 0xFFu) continue;
        uint16_t *p = lrow + (size_t)g * 8;
        if (g * 8 + 8 <= vocab) {
            if (mu == 0u) {
                stream_store(make_uint4(kNegInfPair, kNegInfPair, kNegInfPair, kNegInfPair), p);
            } else {
                uint32_t *x = reinterpret_cast<uint32_t *>(&v[u]);
#pragma unroll
                for (int k = 0; k < 4; ++k) {
                    if (!((mu >> (2 * k)) & 1u)) x[k] = (x[k] & 0xFFFF0000u) | 0xFF80u;
                    if (!((mu >> (2 * k + 1)) & 1u)) x[k] = (x[k] & 0x0000FFFFu) | 0xFF800000u;
                }
                stream_store(v[u], p);
            }
        } else {
            for (int k = 0; g * 8 + k < vocab; ++k)
                if (!((mu >> k) & 1u)) p[k] = 0xFF80;
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


// ------------------------------------------------------------------- masked argmax

// Order-preserving map of a non-NaN binary32 pattern to an unsigned key (-0 counts as +0).
__device__ __forceinline__ uint32_t float_key(float f) {
    uint32_t u = __float_as_uint(f);
    if (u == 0x80000000u) u = 0;
    return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}

__device__ __forceinline__ unsigned long long shfl_xor_u64(unsigned long long v, int mask) {
    const uint32_t lo = __shfl_xor((uint32_t)v, mask), hi = __shfl_xor((uint32_t)(v >> 32), mask);
    return ((unsigned long long)hi << 32) | lo;
}

__device__ __forceinline__ unsigned long long wave_max_u64(unsigned long long v) {
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) {
        const unsigned long long o = shfl_xor_u64(v, off);
        v = o > v ? o : v;
    }
    return v;
}

// Greedy choice among the allowed tokens without writing the masked logits back: a row's logits
// are read once (groups of 8 whose mask byte is zero are not read at all).  blockIdx.x = row,
// blockIdx.y = segment of the row.  A lane keeps the largest value it has seen among allowed
// entries and its id (ids ascend within a lane, so `>` keeps the first of equal values; a NaN
// never compares greater; an allowed -inf, which can only win if nothing else is allowed, is
// remembered separately by lanes that have seen nothing larger); lanes and waves are then
// combined through the packed word
//   key(value) << 32 | ~id,
// whose maximum is the largest value and, among equal values, the smallest id; 0 = no candidate.  With one segment
// per row the block writes out[b] itself; otherwise it stores its word in partial[b][segment]
// and masked_argmax_finish_kernel combines the segments.  (Combining them inside this kernel
// with device-scope atomics and a last-arrival counter was measured: rows that finish early
// then cost tens of microseconds per launch.)  The mask bytes of the next pass are fetched
// while the logits of the current one are in flight.
constexpr int kArgBlock = 1024;
constexpr int kArgUnroll = 4;
__global__ __launch_bounds__(kArgBlock) void masked_argmax_kernel(
    const uint16_t *__restrict__ logits, const uint32_t *__restrict__ bitmask, int vocab, int64_t row_stride,
    int n_words, int groups_per_seg, int vec_ok, unsigned long long *__restrict__ partial, int32_t *__restrict__ out) {
    __shared__ unsigned long long s_part[kArgBlock / 64];
    const int b = blockIdx.x, seg = blockIdx.y, n_seg = gridDim.y, tid = threadIdx.x;
    const int groups = (vocab + 7) >> 3;
    const int g_lo = seg * groups_per_seg, g_hi = min(groups, g_lo + groups_per_seg);
    const uint8_t *mrow = reinterpret_cast<const uint8_t *>(bitmask + (size_t)b * n_words);
    const uint16_t *lrow = logits + (size_t)b * row_stride;
    float best_v = -INFINITY;
    int best_t = -1, ninf_t = -1;                       // ninf_t: first allowed entry that is exactly -inf
    uint32_t m[kArgUnroll], m_next[kArgUnroll];
#pragma unroll
    for (int u = 0; u < kArgUnroll; ++u) {
        const int g = g_lo + tid + u * kArgBlock;
        m[u] = g < g_hi ? mrow[g] : 0u;
    }
    for (int g0 = g_lo + tid; g0 < g_hi; g0 += kArgBlock * kArgUnroll) {
        uint4 v[kArgUnroll];
#pragma unroll
        for (int u = 0; u < kArgUnroll; ++u) {
            const int g = g0 + u * kArgBlock;
            if (m[u] != 0u && vec_ok && g * 8 + 8 <= vocab) v[u] = stream_load(lrow + (size_t)g * 8);
        }
#pragma unroll
        for (int u = 0; u < kArgUnroll; ++u) {
            const int g = g0 + kArgBlock * kArgUnroll + u * kArgBlock;
            m_next[u] = g < g_hi ? mrow[g] : 0u;
        }
#pragma unroll
        for (int u = 0; u < kArgUnroll; ++u) {
            const uint32_t mu = m[u];
            if (mu == 0u) continue;
            const int t0 = (g0 + u * kArgBlock) * 8;
            if (vec_ok && t0 + 8 <= vocab) {
                const uint32_t x[4] = {v[u].x, v[u].y, v[u].z, v[u].w};
#pragma unroll
                for (int k = 0; k < 4; ++k) {
                    const float f0 = (mu >> (2 * k)) & 1u ? __uint_as_float(x[k] << 16) : -INFINITY;
                    const float f1 = (mu >> (2 * k + 1)) & 1u ? __uint_as_float(x[k] & 0xFFFF0000u) : -INFINITY;
                    if (f0 > best_v) { best_v = f0; best_t = t0 + 2 * k; }
                    if (f1 > best_v) { best_v = f1; best_t = t0 + 2 * k + 1; }
                }
                if (best_t < 0 && ninf_t < 0) {
#pragma unroll
                    for (int k = 7; k >= 0; --k) {     // descending: the smallest k is assigned last
                        const uint32_t h = (k & 1) ? (x[k >> 1] >> 16) : (x[k >> 1] & 0xFFFFu);
                        if (((mu >> k) & 1u) && h == 0xFF80u) ninf_t = t0 + k;
                    }
                }
            } else {                                   // ragged tail or unaligned rows: one logit at a time
                for (int k = 0; k < 8 && t0 + k < vocab; ++k) {
                    const uint32_t h = lrow[t0 + k];
                    const float f = (mu >> k) & 1u ? __uint_as_float(h << 16) : -INFINITY;
                    if (f > best_v) { best_v = f; best_t = t0 + k; }
                    if (best_t < 0 && ninf_t < 0 && ((mu >> k) & 1u) && h == 0xFF80u) ninf_t = t0 + k;
                }
            }
        }
#pragma unroll
        for (int u = 0; u < kArgUnroll; ++u) m[u] = m_next[u];
    }
    unsigned long long mine = 0ull;
    if (best_t >= 0) mine = ((unsigned long long)float_key(best_v) << 32) | (0xFFFFFFFFu - (uint32_t)best_t);
    else if (ninf_t >= 0) mine = ((unsigned long long)float_key(-INFINITY) << 32) | (0xFFFFFFFFu - (uint32_t)ninf_t);
    mine = wave_max_u64(mine);
    if ((tid & 63) == 0) s_part[tid >> 6] = mine;
    __syncthreads();
    if (tid < 64) {
        mine = wave_max_u64(tid < kArgBlock / 64 ? s_part[tid] : 0ull);
        if (tid == 0) s_part[0] = mine;
    }
    __syncthreads();
    mine = s_part[0];
    if (n_seg > 1) {
        if (tid == 0) partial[(size_t)b * n_seg + seg] = mine;
        return;
    }
    if (tid == 0) out[b] = mine != 0ull ? (int32_t)(0xFFFFFFFFu - (uint32_t)mine) : -1;
}

// One wave per row: combines the row's segments.
constexpr int kArgFinishRows = 4;
__global__ __launch_bounds__(64 * kArgFinishRows) void masked_argmax_finish_kernel(
    int batch, int n_seg, const unsigned long long *__restrict__ partial, int32_t *__restrict__ out) {
    const int lane = threadIdx.x & 63, b = blockIdx.x * kArgFinishRows + (threadIdx.x >> 6);
    if (b >= batch) return;
    unsigned long long mine = 0ull;
    for (int i = lane; i < n_seg; i += 64) {
        const unsigned long long p = partial[(size_t)b * n_seg + i];
        mine = p > mine ? p : mine;
    }
    mine = wave_max_u64(mine);
    if (lane == 0) out[b] = mine != 0ull ? (int32_t)(0xFFFFFFFFu - (uint32_t)mine) : -1;
}

// -------------------------------------------------------------------------- advance

// One wave per sequence: the walk of a single token is a chain of dependent table look-ups, so
// giving every sequence its own wave keeps control flow uniform (lanes of a shared wave would
// serialise each other's reduction chains) and lets the chip overlap the chains of all
// sequences.  Lane 0 walks the token on a private overlay exactly like in the mask kernels;
// only a walk that succeeds is committed, by all lanes, to the sequence's stack.
constexpr int kAdvSeqPerBlock = 4;
__global__ __launch_bounds__(64 * kAdvSeqPerBlock) void advance_kernel(
    DevTables T, const int32_t *__restrict__ tokens, int32_t *__restrict__ states, int32_t *__restrict__ data,
    int32_t *__restrict__ len, int cap, int batch, int32_t *__restrict__ err, int32_t *scratch, int restart_on_eos) {
    __shared__ int32_t lds_stack[kLdsDepth * kAdvSeqPerBlock];
    __shared__ int32_t s_win[kAdvSeqPerBlock][kWindow], s_info[kAdvSeqPerBlock][64];
    __shared__ int32_t s_base[kAdvSeqPerBlock], s_depth[kAdvSeqPerBlock];
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int b = blockIdx.x * kAdvSeqPerBlock + wave;
    if (b >= batch) return;
    int32_t *row = data + (size_t)b * cap;
    PrivateStack priv;
    priv.lds = lds_stack + wave;
    priv.lds_stride = kAdvSeqPerBlock;
    priv.spill = scratch + b;
    priv.spill_stride = (size_t)batch;
    // every lane: the sequence's inputs, then (in parallel across lanes) the top of the stack and
    // the byte classes of the token, so that lane 0's walk finds them in LDS
    const int t = tokens[b];
    const int n = len[b];
    const int st = states[b];
    const bool live = t >= 0 && t < T.n_tokens && st >= 0 && n >= 1 && n <= cap;
    int lo = 0, hi = 0;
    if (live) {
        s_win[wave][lane] = n - 1 - lane >= 0 ? row[n - 1 - lane] : -1;
        if (t != T.eos_id) {
            const int32_t *rec = T.tok_info + (size_t)t * 32;       // the token's line: length and byte infos
            const int n_bytes = rec[0];
            if (n_bytes >= 0) {
                hi = n_bytes;
                if (lane < n_bytes) s_info[wave][lane] = rec[1 + lane];
            } else {
                lo = T.voffsets[t];
                hi = T.voffsets[t + 1];
                if (lo + lane < hi) s_info[wave][lane] = T.byte_info[T.vbytes[lo + lane]];
            }
        }
    }
    __builtin_amdgcn_wave_barrier();
    // The walk itself runs on all 64 lanes with identical values (scalar table loads, LDS
    // broadcast reads); lane 0 alone writes the results.
    int commit = -1, out_err = 0, out_state = st, out_len = n;
    if (t >= 0) {
        int top = live ? __builtin_amdgcn_readfirstlane(s_win[wave][0]) : -1;
        if (!live || (unsigned)top >= (unsigned)T.n_states) {
            out_err = 1;
        } else {
            const StackView view{row, s_win[wave], n};
            int base = n, d = 0;
            int kind = T.state_kind ? table<true>(T.state_kind, top) : 0;
            if (t == T.eos_id) {
                if (feed<false, true>(T, priv, T.end_col, base, d, top, kind, view, 0) == kAccepted) {
                    out_state = -1;
                    if (restart_on_eos) { out_state = row[0]; out_len = 1; }   // slot reuse: back to the initial state
                } else {
                    out_err = 1;
                }
            } else {
                int rc = hi > lo ? kFed : kRejected;
                for (int i = 0; i < hi - lo && rc == kFed; ++i) {
                    const int info = __builtin_amdgcn_readfirstlane(i < 64 ? s_info[wave][i] : T.byte_info[T.vbytes[lo + i]]);
                    int run_node = -1;
                    rc = feed<true, true>(T, priv, info, base, d, top, kind, view, cap, &run_node);
                    if (rc == kFed && run_node >= 0 && i + 1 < hi - lo)
                        i += apply_run<true>(T, priv, s_info[wave], i + 1, hi - lo, run_node, kind, base, d, top, cap);
                }
                if (rc != kFed) {
                    out_err = rc == kOverflow ? 2 : 1;
                } else {
                    commit = d;
                    out_len = base + d;
                    out_state = top;
                    s_base[wave] = base;
                }
            }
        }
        if (lane == 0) {
            err[b] = out_err;
            if (out_err == 0) { states[b] = out_state; len[b] = out_len; }
        }
    } else if (lane == 0) {
        err[b] = 0;
    }
    s_depth[wave] = commit;
    __builtin_amdgcn_wave_barrier();
    // LDS operations of one wave complete in order; entries that spilled to global memory are
    // copied by lane 0
    const int d = s_depth[wave];
    if (d > 0) {
        const int base = s_base[wave];
        const int in_lds = d < kLdsDepth ? d : kLdsDepth;
        if (lane < in_lds) row[base + lane] = priv.get(lane);
        if (lane == 0)
            for (int i = kLdsDepth; i < d; ++i) row[base + i] = priv.get(i);
    }
}

// Advance and next mask in one launch: one block per sequence.  Wave 0 walks the sampled token
// exactly like advance_kernel (scalar table loads), commits the new stack, stages the NEW top
// of the stack in LDS and descends the condition tree of the token-level edges with it; then the
// whole block builds the sequence's next mask row (dense row copy, delta lists, leftover walks)
// and stores it.  The sequence's inputs are loaded once, no kernel boundary separates the two
// halves, and the long walks of a few sequences overlap the mask building of all others.
constexpr int kAfBlock = 256;
__global__ __launch_bounds__(kAfBlock) void advance_fill_kernel(
    DevTables T, DevTokenEdges E, const int32_t *__restrict__ tokens, int32_t *__restrict__ states,
    int32_t *__restrict__ data, int32_t *__restrict__ len, int cap, int batch, int32_t *__restrict__ err,
    uint32_t *__restrict__ bitmask, int restart_on_eos, int32_t *adv_scratch, int32_t *walk_spill,
    size_t walk_spill_stride) {
    extern __shared__ uint4 bits4[];                   // whole row: n_words rounded up to a multiple of 4
    uint32_t *bits = reinterpret_cast<uint32_t *>(bits4);
    __shared__ int32_t s_win[kWindow], s_new[kWindow], s_info[64];
    __shared__ int32_t s_adv_stack[kLdsDepth], s_walk_stack[kLdsDepth * 64];
    __shared__ RowPlan plan;
    const int tid = threadIdx.x, lane = tid & 63;
    const int b = blockIdx.x;
    const int n_vec = (T.n_words + 3) >> 2;
    int32_t *row = data + (size_t)b * cap;

    if (tid >= 64) {
        // The waves that wait for the walk pull the small tables it reads into this XCD's L2 (a
        // streaming kernel that ran in between has evicted them): one 128-byte line per lane,
        // the lines dealt out over the blocks of the XCD (blocks go round-robin to the 8 XCDs).
        const int per_xcd = (gridDim.x + 7) >> 3, idle = kAfBlock - 64;
        int acc = 0;
        for (int off = ((blockIdx.x >> 3) * idle + (tid - 64)) * 128; off < T.hot_bytes; off += per_xcd * idle * 128)
            acc |= *reinterpret_cast<const volatile int *>(T.hot_begin + off);
        if (acc == 0x7ff1234f && T.fault) atomicAdd(T.fault, 0);   // keeps the loads alive; no effect
    }
    if (tid < 64) {
        PrivateStack priv;
        priv.lds = s_adv_stack;
        priv.lds_stride = 1;
        priv.spill = adv_scratch + b;
        priv.spill_stride = (size_t)batch;
        const int t = tokens[b];
        const int n = len[b];
        const int st = states[b];
        const bool shape_ok = n >= 1 && n <= cap;
        const bool live = t >= 0 && t < T.n_tokens && st >= 0 && shape_ok;
        int lo = 0, hi = 0;
        s_win[lane] = (shape_ok && n - 1 - lane >= 0) ? row[n - 1 - lane] : -1;
        if (live && t != T.eos_id) {
            const int32_t *rec = T.tok_info + (size_t)t * 32;       // the token's line: length and byte infos
            const int n_bytes = rec[0];
            if (n_bytes >= 0) {
                hi = n_bytes;
                if (lane < n_bytes) s_info[lane] = rec[1 + lane];
            } else {
                lo = T.voffsets[t];
                hi = T.voffsets[t + 1];
                if (lo + lane < hi) s_info[lane] = T.byte_info[T.vbytes[lo + lane]];
            }
        }
        __builtin_amdgcn_wave_barrier();
        // ---- advance (all lanes hold identical values)
        int out_err = 0, out_state = st, out_len = n, base = n, d = 0;
        bool restarted = false;
        if (t >= 0) {
            int top = live ? __builtin_amdgcn_readfirstlane(s_win[0]) : -1;
            if (!live || (unsigned)top >= (unsigned)T.n_states) {
                out_err = 1;
            } else {
                const StackView view{row, s_win, n};
                int kind = T.state_kind ? table<true>(T.state_kind, top) : 0;
                if (t == T.eos_id) {
                    if (feed<false, true>(T, priv, T.end_col, base, d, top, kind, view, 0) == kAccepted) {
                        out_state = -1;
                        if (restart_on_eos) { out_state = row[0]; out_len = 1; restarted = true; }   // slot reuse
                    } else {
                        out_err = 1;
                    }
                    base = n;
                    d = 0;                               // the '$' walk never changes the stack
                } else {
                    int rc = hi > lo ? kFed : kRejected;
                    for (int i = 0; i < hi - lo && rc == kFed; ++i) {
                        const int info = __builtin_amdgcn_readfirstlane(i < 64 ? s_info[i] : T.byte_info[T.vbytes[lo + i]]);
                        int run_node = -1;
                        rc = feed<true, true>(T, priv, info, base, d, top, kind, view, cap, &run_node);
                        if (rc == kFed && run_node >= 0 && i + 1 < hi - lo)
                            i += apply_run<true>(T, priv, s_info, i + 1, hi - lo, run_node, kind, base, d, top, cap);
                    }
                    if (rc != kFed) {
                        out_err = rc == kOverflow ? 2 : 1;
                        base = n;
                        d = 0;
                    } else {
                        out_len = base + d;
                        out_state = top;
                    }
                }
            }
        }
        if (lane == 0) {
            err[b] = out_err;
            if (out_err == 0 && t >= 0) { states[b] = out_state; len[b] = out_len; }
        }
        // ---- the new stack is  row[0 .. base) ++ priv[0 .. d)  (or just its bottom after a restart):
        //      stage its top in LDS and commit the private part
        const int nl = out_len;
        auto new_at = [&](int k) -> int32_t {           // entry k below the new top
            if (restarted) return k == 0 ? row[0] : -1;
            if (k < d) return priv.get(d - 1 - k);
            const int idx = base - 1 - (k - d);
            return idx >= 0 ? StackView{row, s_win, n}.at(idx) : -1;
        };
        s_new[lane] = (shape_ok && lane < nl) ? new_at(lane) : -1;
        {
            const int in_lds = d < kLdsDepth ? d : kLdsDepth;
            if (lane < in_lds) row[base + lane] = priv.get(lane);
            if (lane == 0)
                for (int i = kLdsDepth; i < d; ++i) row[base + i] = priv.get(i);
        }
        __builtin_amdgcn_wave_barrier();
        // ---- descent of the condition tree with the new stack
        const int top = s_new[0];
        if (out_state < 0) {
            if (lane == 0) plan.mode = kRowDone;
        } else if (!shape_ok || (unsigned)top >= (unsigned)T.n_states) {
            if (lane == 0) plan.mode = kRowEmpty;
        } else {
            plan_row(E, E.root_nodes[top], s_new, nl, new_at, &plan, lane);
        }
        if (lane == 0) { plan.top = top; plan.len = nl; }
    }
    __syncthreads();
    // ---- the next mask row
    const int mode = plan.mode;
    if (mode == kRowFast && plan.dense >= 0) {
        const uint4 *src = reinterpret_cast<const uint4 *>(E.dense_rows) + (size_t)plan.dense * n_vec;
        for (int w = tid; w < n_vec; w += kAfBlock) bits4[w] = src[w];
    } else {
        for (int w = tid; w < n_vec; w += kAfBlock) bits4[w] = make_uint4(0, 0, 0, 0);
    }
    __syncthreads();
    if (mode == kRowFast || mode == kRowWalkAll) {
        if (mode == kRowFast) {
            const int nseg = plan.nseg;
            for (int i = 0; i < nseg; ++i) {
                const int32_t *ids = E.delta_ids + plan.seg_begin[i];
                const int cnt = plan.seg_count[i];
                for (int k = tid; k < cnt; k += kAfBlock) {
                    const int t = ids[k];
                    atomicOr(&bits[t >> 5], 1u << (t & 31));
                }
            }
        }
        const int wc = mode == kRowWalkAll ? T.n_tokens : plan.walk_count;
        if (wc > 0 && tid < 64) {                       // leftovers: walked on the committed stack
            PrivateStack wp;
            wp.lds = s_walk_stack + lane;
            wp.lds_stride = 64;
            wp.spill = walk_spill + (size_t)b * 64 + lane;
            wp.spill_stride = walk_spill_stride;
            const int n = plan.len, top0 = plan.top;
            for (int k = lane; k < wc; k += 64) {
                const int t = mode == kRowWalkAll ? k : E.walk_ids[plan.walk_begin + k];
                if (walk_token_id(T, wp, t, row, n, top0)) atomicOr(&bits[t >> 5], 1u << (t & 31));
            }
        }
    } else if (mode == kRowDone && tid == 0) {
        bits[T.eos_id >> 5] = 1u << (T.eos_id & 31);
    }
    __syncthreads();
    uint32_t *dst = bitmask + (size_t)b * T.n_words;
    if ((T.n_words & 3) == 0 && (reinterpret_cast<uintptr_t>(bitmask) & 15) == 0) {
        uint4 *dst4 = reinterpret_cast<uint4 *>(dst);
        for (int w = tid; w < n_vec; w += kAfBlock) dst4[w] = bits4[w];
    } else {
        for (int w = tid; w < T.n_words; w += kAfBlock) dst[w] = bits[w];
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

size_t advance_fill_walk_spill_entries(int batch, int max_depth) {
    const int deep = max_depth > kLdsDepth ? max_depth - kLdsDepth : 0;
    return (size_t)batch * 64 * (size_t)deep;
}

hipError_t launch_advance_fill(const DevTables &T, const DevTokenEdges &E, const int32_t *tokens, int32_t *states,
                               int32_t *data, int32_t *len, int cap, int batch, int32_t *err, uint32_t *bitmask,
                               int restart_on_eos, int32_t *adv_scratch, int32_t *walk_spill, hipStream_t stream) {
    if (batch == 0) return hipSuccess;
    const size_t lds = (size_t)edge_row_stride_words(T.n_words) * sizeof(uint32_t);
    hipLaunchKernelGGL(advance_fill_kernel, dim3(batch), dim3(kAfBlock), lds, stream, T, E, tokens, states, data, len, cap,
                       batch, err, bitmask, restart_on_eos, adv_scratch, walk_spill, (size_t)batch * 64);
    return hipGetLastError();
}

hipError_t launch_apply_mask(uint16_t *logits, const uint32_t *bitmask, int batch, int vocab, int64_t row_stride,
                             hipStream_t stream) {
    if (batch == 0 || vocab == 0) return hipSuccess;
    const int n_words = (vocab + 31) / 32;
    const bool aligned = (reinterpret_cast<uintptr_t>(logits) % 16 == 0) && (row_stride % 8 == 0);
    if (aligned && batch <= 65535) {
        const dim3 grid((vocab + kApplySpan - 1) / kApplySpan, batch);
        hipLaunchKernelGGL(apply_mask_vec8_kernel, grid, dim3(kApplyBlock), 0, stream, logits, bitmask, vocab, row_stride,
                           n_words);
    } else {
        const int64_t total = (int64_t)batch * vocab;
        const int64_t want = (total + 255) / 256;
        const int grid = (int)(want < 65536 ? want : 65536);
        hipLaunchKernelGGL(apply_mask_scalar_kernel, dim3(grid), dim3(256), 0, stream, logits, bitmask, batch, vocab,
                           row_stride, n_words);
    }
    return hipGetLastError();
}

// blocks per row of the argmax kernel: enough blocks to fill the chip, and every block at least
// one full pass wide
static int masked_argmax_segments(int batch, int vocab, int n_compute_units) {
    const int groups = (vocab + 7) / 8;
    const int max_seg = (groups + kArgBlock * kArgUnroll - 1) / (kArgBlock * kArgUnroll);
    int n_seg = batch > 0 ? (n_compute_units + batch - 1) / batch : 1;
    n_seg = n_seg > max_seg ? max_seg : n_seg;
    return n_seg < 1 ? 1 : n_seg;
}

size_t masked_argmax_workspace_bytes(int batch, int vocab, int n_compute_units) {
    return (size_t)batch * masked_argmax_segments(batch, vocab, n_compute_units) * sizeof(unsigned long long);
}

hipError_t launch_masked_argmax(const uint16_t *logits, const uint32_t *bitmask, int batch, int vocab, int64_t row_stride,
                                int n_compute_units, unsigned long long *workspace, int32_t *out, hipStream_t stream) {
    if (batch == 0) return hipSuccess;
    const int n_words = (vocab + 31) / 32, groups = (vocab + 7) / 8;
    const int n_seg = masked_argmax_segments(batch, vocab, n_compute_units);
    const int groups_per_seg = (groups + n_seg - 1) / n_seg;
    const int vec_ok = (reinterpret_cast<uintptr_t>(logits) % 16 == 0) && (row_stride % 8 == 0);
    hipLaunchKernelGGL(masked_argmax_kernel, dim3(batch, n_seg), dim3(kArgBlock), 0, stream, logits, bitmask, vocab,
                       row_stride, n_words, groups_per_seg, vec_ok, workspace, out);
    if (n_seg > 1)
        hipLaunchKernelGGL(masked_argmax_finish_kernel, dim3((batch + kArgFinishRows - 1) / kArgFinishRows),
                           dim3(64 * kArgFinishRows), 0, stream, batch, n_seg, workspace, out);
    return hipGetLastError();
}

hipError_t launch_advance(const DevTables &T, const int32_t *tokens, int32_t *states, int32_t *data, int32_t *len,
                          int cap, int batch, int32_t *err, int32_t *scratch, int restart_on_eos, hipStream_t stream) {
    if (batch == 0) return hipSuccess;
    hipLaunchKernelGGL(advance_kernel, dim3((batch + kAdvSeqPerBlock - 1) / kAdvSeqPerBlock), dim3(64 * kAdvSeqPerBlock),
                       0, stream, T, tokens, states, data, len, cap, batch, err, scratch, restart_on_eos);
    return hipGetLastError();
}

}  // namespace pre3

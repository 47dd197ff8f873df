// Device-side walk of the DPDA: private stacks, table look-ups, the step that consumes one input
// symbol (merged reduction edges with their stack-matching conditions, per-step edges as the
// fallback), self-similar runs, and whole-token walks.  Included by the kernel files.
#pragma once
#include <hip/hip_runtime.h>

#include "device_tables.hpp"
#include "symbol_edges.hpp"
#include "tables.hpp"

namespace pre3 {

namespace {

constexpr int kBlock = 256;            // threads per block of the walk kernel
constexpr int kRunGrows = 1 << 30;      // flag on a run's condition node: the run's edges grow the stack
constexpr int kLdsDepth = 16;          // private stack entries kept in LDS per lane
constexpr int kMaxChain = 1 << 20;     // reduction steps per input symbol before a walk gives up

// Reads that name their address space.  Where the source chooses between an LDS and a global address
// the compiler otherwise forms ONE load from the chosen generic address, a flat load, and a wave
// waits for a flat load as for a vector-memory load -- in order behind whatever its compute unit
// has in flight there -- even when the address turns out to be in LDS.
__device__ __forceinline__ int32_t lds_read(const int32_t *p) {
    return *(const __attribute__((address_space(3))) int32_t *)p;
}
__device__ __forceinline__ int32_t global_read(const int32_t *p) {
    return *(const __attribute__((address_space(1))) int32_t *)p;
}

// Block barrier that orders the block's LDS accesses only.  __syncthreads also makes a wave wait until
// its global stores are acknowledged, which takes microseconds while the memory system is saturated.
__device__ __forceinline__ void lds_barrier() {
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup", "local");
    __builtin_amdgcn_s_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup", "local");
}

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
        int32_t v = lds_read(lds + (i < kLdsDepth ? i : kLdsDepth - 1) * lds_stride);
        if (i >= kLdsDepth) v = global_read(spill + (size_t)(i - kLdsDepth) * spill_stride);
        return v;
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

// Wider scalar loads for a wave that must stay off the vector-memory path (its block's other waves
// have a long queue of loads in flight there, and vector loads return in order): 8 or 16 consecutive
// 32-bit words at a wave-uniform, 4-byte aligned address of a read-only table.  A 16-word load may
// reach up to 60 bytes past the entries the caller wants: every uploaded table ends with that much
// padding.
typedef int NativeInt8 __attribute__((ext_vector_type(8)));
typedef int NativeInt16 __attribute__((ext_vector_type(16)));
typedef NativeInt8 __attribute__((aligned(4))) NativeInt8U;
typedef NativeInt16 __attribute__((aligned(4))) NativeInt16U;
__device__ __forceinline__ NativeInt8 scalar_load8(const void *p) { return *(ConstPtr<NativeInt8U>)p; }
__device__ __forceinline__ NativeInt16 scalar_load16(const void *p) { return *(ConstPtr<NativeInt16U>)p; }

// Position of `x` among the `count` ascending values that start at list[0], or -1; values at a stride
// of kStride words (1: plain list, 2: the first halves of pairs).  All arguments wave-uniform.
template <int kStride>
__device__ __forceinline__ int scalar_find(const int32_t *list, int count, int x) {
    constexpr int kPer = 16 / kStride;
    for (int c0 = 0; c0 < count; c0 += kPer) {
        const NativeInt16 v = scalar_load16(list + (size_t)c0 * kStride);
        int found = -1;
#pragma unroll
        for (int k = 0; k < kPer; ++k)
            if (c0 + k < count && v[k * kStride] == x) found = c0 + k;
        if (found >= 0) return found;
        if (v[(kPer - 1) * kStride] > x && c0 + kPer <= count) return -1;      // ascending: x cannot follow
    }
    return -1;
}

// The sequence's stack as the walk sees it: row[0..n), optionally with its top `kWindow` entries
// staged in LDS (win[k] = entry k below the top).
constexpr int kWindow = 64;
struct StackView {
    const int32_t *row;
    const int32_t *win;
    int n;
    __device__ int32_t at(int idx) const {
        if (!win) return row[idx];
        const int k = n - 1 - idx;
        int32_t v = lds_read(win + (k < kWindow ? k : kWindow - 1));
        if (k >= kWindow) v = global_read(row + idx);
        return v;
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
template <bool kCheckCap, bool kUniform = false, bool kScalarOnly = false>
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
                int known, peak, np, same, grow, after;
                int4 push4;
                if (code & kCellInline) {
                    known = code & 0xFF;
                    peak = ((code >> 8) & 0xFF) - 128;
                    np = (code >> 16) & 3;
                    same = code & kCellSameShape;
                    grow = code & kCellGrow;
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
                    grow = hdr.z & kEffGrow;
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
                if (run_node) *run_node = ((same || grow) && after == tree) ? (node | (grow ? kRunGrows : 0)) : -1;
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
            if (kUniform && kScalarOnly) {
                // the same search through the scalar cache: the condition states first, then the child's record and cell
                const int j = scalar_find<2>(reinterpret_cast<const int32_t *>(T.sym_pairs + nd.y), nd.z, x);
                if (j < 0) break;
                next = nd.w + j;
                node = next;
                nd = table<true>(T.sym_nodes, node);
                cell = table<true>(T.sym_cell, node * T.ncol + col);
            } else if (kUniform) {
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
// replaces the top of the stack; after a growing edge (`node` carries kRunGrows: the stack gained a
// second copy of the entry under its top) every following growing edge at the same node inserts one
// more copy and replaces the top.  Each of the 64 lanes examines one upcoming byte
// (infos[first + lane], staged in LDS); the run ends at the first byte that is not such an edge.
// Returns the number of bytes consumed; the last one's target becomes the new top, and a growing
// run adds one private entry per byte (d grows).
template <bool kCheckCap>
__device__ __forceinline__ int apply_run(const DevTables &T, PrivateStack &priv, const int32_t *infos, int first,
                                         int n_bytes, int node, int tree, int base, int &d, int &top, int cap) {
    const bool grows = (node & kRunGrows) != 0;
    node &= ~kRunGrows;
    const int lane = threadIdx.x & 63, i = first + lane;
    const int gain = grows ? lane : 0;                  // entries added by the run's earlier bytes
    bool ok = i < n_bytes && i < 64;
    int new_top = 0, copy = 0;
    if (ok) {
        const int info = infos[i];
        const int4 cell = T.sym_cell[node * T.ncol + (info & 0xFF)];
        const int code = cell.x;
        ok = code >= 0;
        if (ok && (code & kCellInline)) {
            ok = (code & (grows ? kCellGrow : kCellSameShape)) && cell.y == tree &&
                 (!kCheckCap || base + d + gain + ((code >> 8) & 0xFF) - 128 < cap);
            new_top = (((code >> 16) & 3) == 1 ? cell.z : cell.w) + (info >> 8);
            copy = cell.z;
        } else if (ok) {
            const int4 hdr = *reinterpret_cast<const int4 *>(T.sym_pool + code);
            ok = (hdr.z & (grows ? kEffGrow : kEffSameShape)) && hdr.w == tree && (!kCheckCap || base + d + gain + hdr.y < cap);
            if (ok) {
                new_top = T.sym_pool[code + 4 + (hdr.z & kEffPushMask) - 1] + (info >> 8);
                copy = T.sym_pool[code + 4];
            }
        }
    }
    const unsigned long long bad = __ballot(!ok);
    int run = bad ? __ffsll((long long)bad) - 1 : 64;
    if (grows && d + run > T.max_depth) run = T.max_depth > d ? T.max_depth - d : 0;    // cannot happen: see the depth bound
    if (run > 0) {
        top = __builtin_amdgcn_readfirstlane(__shfl(new_top, run - 1));
        if (grows) {
            const int x = __builtin_amdgcn_readfirstlane(copy);       // the same entry for every byte of the run
            for (int j = 0; j < run; ++j) priv.set(d - 1 + j, x);
            d += run;
        }
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

}  // namespace

}  // namespace pre3

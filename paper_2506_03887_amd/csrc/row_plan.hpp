// Descent of the condition tree of the token-level edges and the assembly of one sequence's mask
// row from what the descent found.  Shared by the mask kernel and the advance+mask kernel.
#pragma once
#include "effect_hash.hpp"
#include "stream_access.hpp"
#include "walk.hpp"

namespace pre3 {

namespace {

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
        int x = lds_read(win + (nd.known < kWindow ? nd.known : kWindow - 1));
        if (nd.known >= kWindow) x = deeper(nd.known);
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

// A node record of the condition tree through the scalar cache (all lanes get the same record).
__device__ __forceinline__ DevConditionNode scalar_node(const DevConditionNode *p) {
    const NativeInt8 v = scalar_load8(p);
    DevConditionNode nd;
    nd.known = v[0]; nd.child_count = v[1]; nd.a = v[2]; nd.b = v[3];
    nd.dense_row = v[4]; nd.delta_begin = v[5]; nd.delta_count = v[6]; nd.pad = v[7];
    return nd;
}

// plan_row with scalar loads only (see scalar_load16): per level one round for the condition states,
// one for the child's record.
template <typename Deeper>
__device__ __forceinline__ void plan_row_scalar(const DevTokenEdges &E, DevConditionNode nd, const int32_t *win, int n,
                                                Deeper deeper, RowPlan *plan, int lane) {
    int mode = kRowFast, nseg = 0, dense = -1, walk_begin = 0, walk_count = 0;
    for (;;) {
        if (nd.dense_row >= 0) {
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
        int x = lds_read(win + (nd.known < kWindow ? nd.known : kWindow - 1));
        if (nd.known >= kWindow) x = deeper(nd.known);
        x = __builtin_amdgcn_readfirstlane(x);
        const int j = scalar_find<1>(E.child_state + nd.a, nd.child_count, x);
        if (j < 0) { mode = kRowWalkAll; break; }
        nd = scalar_node(E.nodes + nd.b + j);
    }
    if (lane == 0) {
        plan->nseg = nseg;
        plan->dense = dense;
        plan->mode = mode;
        plan->walk_begin = walk_begin;
        plan->walk_count = walk_count;
    }
}

// What the merged edge of a token does to the stack (the stack operations that every prefix-conditioned
// edge carries, Sec. 3.1): the top k - 1 entries are replaced by np states; peak = highest the stack
// gets just before a push, relative to its height before the token.
struct EffectHit {
    int found, k, peak, np, inline_count, x0, x1;   // x0, x1: the states pushed when inline_count > 0, else x0 = their offset in fx_pool
};

// Looks the effect of token `tok` up for the stack whose top state has the root `node` (its record:
// `nd`): descends the condition tree like plan_row and probes every node on the way.  One round of
// loads per level: lanes 0..7 fetch the eight slots of the key's two buckets, lanes 8..63 the
// condition states and records of the node's first 56 children (more children take further rounds);
// a ballot finds the record, another the child.  Run by all 64 lanes of a wave with identical
// values; a miss means "walk the token".
template <typename Deeper>
__device__ __forceinline__ EffectHit find_effect(const DevTokenEdges &E, int node, DevConditionNode nd, const int32_t *win,
                                                 int n, Deeper deeper, int tok, int lane) {
    EffectHit r{0, 0, 0, 0, 0, 0, 0};
    for (int level = 0; level < 256; ++level) {
        uint32_t b1, b2;
        effect_buckets((uint32_t)node, (uint32_t)tok, E.fx_mask, &b1, &b2);
        int4 slot = make_int4(-1, 0, 0, 0);
        if (lane < 2 * kEffectBucketSlots)
            slot = E.fx_slots[(size_t)(lane < kEffectBucketSlots ? b1 : b2) * kEffectBucketSlots + (lane & (kEffectBucketSlots - 1))];
        const bool inner = nd.child_count > 0 && nd.known < n;
        int x = -3;
        if (inner) {
            x = lds_read(win + (nd.known < kWindow ? nd.known : kWindow - 1));
            if (nd.known >= kWindow) x = deeper(nd.known);
        }
        int cstate = -2;
        DevConditionNode c{};
        int j = lane - 2 * kEffectBucketSlots;
        if (inner && j >= 0 && j < nd.child_count) {
            cstate = E.child_state[nd.a + j];
            c = E.nodes[nd.b + j];
        }
        const unsigned long long hit = __ballot(lane < 2 * kEffectBucketSlots && slot.x >= 0 &&
                                                effect_slot_matches((uint32_t)slot.x, (uint32_t)slot.y, (uint32_t)node, (uint32_t)tok));
        if (hit) {
            const int src = __ffsll((long long)hit) - 1;
            const EffectFields f = effect_unpack((uint32_t)__shfl(slot.y, src), (uint32_t)__shfl(slot.z, src), (uint32_t)__shfl(slot.w, src));
            r.found = 1;
            r.k = f.k;
            r.peak = f.peak;
            r.np = f.np;
            r.inline_count = f.inline_count;
            r.x0 = f.x0;
            r.x1 = f.x1;
            return r;
        }
        if (!inner) return r;
        unsigned long long m = __ballot(cstate == x);
        int child = -1;
        if (m) child = __ffsll((long long)m) - 1 - 2 * kEffectBucketSlots;
        for (int c0 = 64 - 2 * kEffectBucketSlots; !m && c0 < nd.child_count; c0 += 64) {
            j = c0 + lane;
            cstate = -2;
            if (j < nd.child_count) {
                cstate = E.child_state[nd.a + j];
                c = E.nodes[nd.b + j];
            }
            m = __ballot(cstate == x);
            if (m) child = c0 + __ffsll((long long)m) - 1;
        }
        if (!m) return r;
        const int src = __ffsll((long long)m) - 1;
        node = nd.b + child;
        nd.known = __shfl(c.known, src);
        nd.child_count = __shfl(c.child_count, src);
        nd.a = __shfl(c.a, src);
        nd.b = __shfl(c.b, src);
    }
    return r;
}

// find_effect with scalar loads only (see scalar_load16): per level one round for the two buckets and
// the node's first sixteen condition states, one for the child's record.
template <typename Deeper>
__device__ __forceinline__ EffectHit find_effect_scalar(const DevTokenEdges &E, int node, DevConditionNode nd, const int32_t *win,
                                                        int n, Deeper deeper, int tok) {
    EffectHit r{0, 0, 0, 0, 0, 0, 0};
    for (int level = 0; level < 256; ++level) {
        uint32_t b1, b2;
        effect_buckets((uint32_t)node, (uint32_t)tok, E.fx_mask, &b1, &b2);
        const bool inner = nd.child_count > 0 && nd.known < n;
        const NativeInt16 s1 = scalar_load16(E.fx_slots + (size_t)b1 * kEffectBucketSlots);
        const NativeInt16 s2 = scalar_load16(E.fx_slots + (size_t)b2 * kEffectBucketSlots);
        const int32_t *kids = E.child_state + (inner ? nd.a : 0);
        const NativeInt16 first = scalar_load16(kids);
        int x = -3;
        if (inner) {
            x = lds_read(win + (nd.known < kWindow ? nd.known : kWindow - 1));
            if (nd.known >= kWindow) x = deeper(nd.known);
            x = __builtin_amdgcn_readfirstlane(x);
        }
        bool hit = false;
        uint32_t w1 = 0, w2 = 0, w3 = 0;
#pragma unroll
        for (int k = 0; k < 2 * kEffectBucketSlots; ++k) {
            const NativeInt16 &s = k < kEffectBucketSlots ? s1 : s2;
            const int o = (k & (kEffectBucketSlots - 1)) * 4;
            if (!hit && s[o] >= 0 && effect_slot_matches((uint32_t)s[o], (uint32_t)s[o + 1], (uint32_t)node, (uint32_t)tok)) {
                hit = true;
                w1 = (uint32_t)s[o + 1]; w2 = (uint32_t)s[o + 2]; w3 = (uint32_t)s[o + 3];
            }
        }
        if (hit) {
            const EffectFields f = effect_unpack(w1, w2, w3);
            r.found = 1;
            r.k = f.k;
            r.peak = f.peak;
            r.np = f.np;
            r.inline_count = f.inline_count;
            r.x0 = f.x0;
            r.x1 = f.x1;
            return r;
        }
        if (!inner) return r;
        int j = -1;
#pragma unroll
        for (int k = 0; k < 16; ++k)
            if (k < nd.child_count && first[k] == x) j = k;
        if (j < 0 && nd.child_count > 16) {
            j = scalar_find<1>(kids + 16, nd.child_count - 16, x);
            if (j >= 0) j += 16;
        }
        if (j < 0) return r;
        node = nd.b + j;
        nd = scalar_node(E.nodes + node);
    }
    return r;
}

// Assembles mask words [4 * v_lo, 4 * (v_lo + v_cnt)) of the row that `plan` describes in the LDS
// bitmap bits4[0 .. v_cnt) and stores them to dst_row (the row's first word in the bitmask):
//   1. the segment of the materialised row the descent ended on (or zeros);
//   2. the token ids collected after it, ORed in one lane per id (LDS atomics);
//   3. tokens the tree leaves undetermined, walked byte by byte on `row` by the first 64 threads
//      (each with its own private stack `priv`); a stack the tree has no answer for walks every
//      token of the segment; a finished sequence gets the EOS bit only.
// Called by all kThreads threads of the block after a barrier that made `plan` visible; contains
// two block barriers; on return the bitmap still holds the segment.  kWholeRow: the segment is the
// whole row (v_lo = 0), so no id needs a range test.
template <int kThreads, bool kWholeRow = false, bool kDirect = false>
__device__ __forceinline__ void build_and_store_row(const DevTables &T, const DevTokenEdges &E, const RowPlan &plan,
                                                    uint4 *bits4, int v_lo, int v_cnt, const int32_t *row,
                                                    PrivateStack &priv, uint32_t *dst_row, bool dst_vector_ok, int tid) {
    uint32_t *bits = reinterpret_cast<uint32_t *>(bits4);
    const int n_vec = (T.n_words + 3) >> 2;
    const int mode = plan.mode;
    const int w_lo = v_lo * 4, w_hi = w_lo + max(v_cnt, 0) * 4;
    if (kDirect && mode == kRowFast && plan.dense >= 0 && plan.nseg == 0 && plan.walk_count == 0 && dst_vector_ok) {
        // the row is exactly a materialised row: copy it without staging it in LDS
        const uint4 *src = reinterpret_cast<const uint4 *>(E.dense_rows) + (size_t)plan.dense * n_vec + v_lo;
        uint4 *dst4 = reinterpret_cast<uint4 *>(dst_row) + v_lo;
        for (int w = tid; w < v_cnt; w += kThreads) stream_store(src[w], dst4 + w);
        return;
    }
    if (mode == kRowFast && plan.dense >= 0) {
        const uint4 *src = reinterpret_cast<const uint4 *>(E.dense_rows) + (size_t)plan.dense * n_vec + v_lo;
        for (int w = tid; w < v_cnt; w += kThreads) bits4[w] = src[w];
    } else {
        for (int w = tid; w < v_cnt; w += kThreads) bits4[w] = make_uint4(0, 0, 0, 0);
    }
    __syncthreads();
    if (mode == kRowFast) {
        const int nseg = plan.nseg;
        for (int i = 0; i < nseg; ++i) {
            const int32_t *ids = E.delta_ids + plan.seg_begin[i];
            const int cnt = plan.seg_count[i];
            for (int k = tid; k < cnt; k += kThreads) {
                const int t = ids[k], w = t >> 5;
                if (kWholeRow || (w >= w_lo && w < w_hi)) atomicOr(&bits[w - w_lo], 1u << (t & 31));
            }
        }
        const int wc = plan.walk_count;
        if (wc > 0 && tid < 64) {
            const int n = plan.len, top0 = plan.top;
            for (int k = tid; k < wc; k += 64) {
                const int t = E.walk_ids[plan.walk_begin + k], w = t >> 5;
                if (w >= w_lo && w < w_hi && walk_token_id(T, priv, t, row, n, top0))
                    atomicOr(&bits[w - w_lo], 1u << (t & 31));
            }
        }
    } else if (mode == kRowWalkAll) {
        if (tid < 64) {
            const int n = plan.len, top0 = plan.top;
            const int t_hi = min(T.n_tokens, w_hi * 32);
            for (int t = w_lo * 32 + tid; t < t_hi; t += 64)
                if (walk_token_id(T, priv, t, row, n, top0)) atomicOr(&bits[(t >> 5) - w_lo], 1u << (t & 31));
        }
    } else if (mode == kRowDone && tid == 0) {
        const int w = T.eos_id >> 5;
        if (w >= w_lo && w < w_hi) bits[w - w_lo] = 1u << (T.eos_id & 31);
    }
    __syncthreads();
    if (dst_vector_ok) {
        uint4 *dst4 = reinterpret_cast<uint4 *>(dst_row) + v_lo;
        for (int w = tid; w < v_cnt; w += kThreads) stream_store(bits4[w], dst4 + w);
    } else {
        for (int w = w_lo + tid; w < min(w_hi, T.n_words); w += kThreads) dst_row[w] = bits[w - w_lo];
    }
}

}  // namespace

}  // namespace pre3

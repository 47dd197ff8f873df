// Descent of the condition tree of the token-level edges: how one sequence's mask row is
// assembled.  Shared by the mask kernel and the advance+mask kernel.
#pragma once
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

}  // namespace

}  // namespace pre3

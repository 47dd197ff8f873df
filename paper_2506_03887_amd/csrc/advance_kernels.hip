// gfx950 kernels of the stack advance: one sampled token per sequence walked on the sequence's
// own stack, alone or followed by the next step's mask row in the same launch.
#include <hip/hip_runtime.h>

#include <mutex>

#include "argmax.hpp"
#include "launch.hpp"
#include "row_plan.hpp"

// Spill area of the private stacks for pre3_advance_static, the entry point that allocates
// nothing: device memory that belongs to the loaded library itself (every GPU the library runs
// on holds its own copy until the process ends).  Host code never passes this name to a kernel:
// the device address is taken once per device with hipGetSymbolAddress (static_advance_scratch).
static __device__ __align__(256) int32_t pre3_static_scratch[pre3::kStaticScratchEntries];

namespace pre3 {

namespace {

// -------------------------------------------------------------------------- advance

// The bytes of a sampled token as the walk needs them: hi - lo bytes; the class/offset word of
// byte i < 64 is staged in LDS, later ones are read through the id-ordered vocabulary at lo + i.
struct StagedToken {
    int lo, hi;
};

// All 64 lanes of the wave call this with the same token id: lane i fetches byte i.
__device__ __forceinline__ StagedToken stage_token(const DevTables &T, int t, int lane, int32_t *s_info) {
    StagedToken tok{0, 0};
    const int32_t *rec = T.tok_info + (size_t)t * 32;           // the token's line: length and byte infos
    const int n_bytes = rec[0];
    if (n_bytes >= 0) {
        tok.hi = n_bytes;
        if (lane < n_bytes) s_info[lane] = rec[1 + lane];
    } else {
        tok.lo = T.voffsets[t];
        tok.hi = T.voffsets[t + 1];
        if (tok.lo + lane < tok.hi) s_info[lane] = T.byte_info[T.vbytes[tok.lo + lane]];
    }
    return tok;
}

// Lanes kLane0 .. kLane0 + kCount of `w` replaced by the wave-uniform words v[kSrc0 ..] (one v_writelane
// each; the lane is an immediate, the instruction takes one scalar register only).
template <int kLane0, int kSrc0, int kCount, int kI = 0>
__device__ __forceinline__ int32_t deal_to_lanes(int32_t w, const NativeInt16 &v) {
    if constexpr (kI < kCount) {
        asm("v_writelane_b32 %0, %1, %2" : "+v"(w) : "s"(v[kSrc0 + kI]), "n"(kLane0 + kI));
        return deal_to_lanes<kLane0, kSrc0, kCount, kI + 1>(w, v);
    } else {
        return w;
    }
}

// stage_token through the scalar cache: the token's 128-byte line comes as two 16-word loads, whose words
// are dealt out to the lanes (lane i gets byte i's word) and stored with one LDS write.  Tokens longer
// than the line holds take the vector path.
__device__ __forceinline__ StagedToken stage_token_scalar(const DevTables &T, int t, int lane, int32_t *s_info) {
    const int32_t *rec = T.tok_info + (size_t)t * 32;
    const NativeInt16 a = scalar_load16(rec), b = scalar_load16(rec + 16);
    const int n_bytes = a[0];
    if (n_bytes < 0) return stage_token(T, t, lane, s_info);
    static_assert(kTokInfoBytes == 31, "two 16-word loads hold the length and 31 bytes");
    int32_t w = 0;
    w = deal_to_lanes<0, 1, 15>(w, a);
    w = deal_to_lanes<15, 0, 16>(w, b);
    if (lane < n_bytes) s_info[lane] = w;
    return StagedToken{0, n_bytes};
}

// The top 64 entries of a stack (win[k] = entry k below the top, -1 beyond the bottom) through the scalar
// cache: four 16-entry loads that end at the top -- each moved to where it lies wholly inside the row's
// cap entries, cap >= 16 --, dealt out to the lanes and stored with one LDS write.
__device__ __forceinline__ void stage_window_scalar(const int32_t *row, int n, int cap, bool shape_ok, int lane, int32_t *win) {
    win[lane] = -1;
    if (!shape_ok) return;
    int32_t w = 0;
    int my_lo = 0;
    auto chunk_begin = [&](int c) {
        int lo = n - 16 * (c + 1);
        lo = lo < 0 ? 0 : lo;
        return lo > cap - 16 ? cap - 16 : lo;
    };
    // one chunk at a time, and only the chunks the stack reaches (few scalar registers live; the later loads
    // find their cache lines where the first one brought them)
    const int lo0 = chunk_begin(0);
    w = deal_to_lanes<0, 0, 16>(w, scalar_load16(row + lo0));
    my_lo = lo0;
    int dealt = 16;                                     // lanes that hold an entry
    if (n > 16) {
        const int lo1 = chunk_begin(1);
        w = deal_to_lanes<16, 0, 16>(w, scalar_load16(row + lo1));
        if (lane >= 16) my_lo = lo1;
        dealt = 32;
        if (n > 32) {
            const int lo2 = chunk_begin(2);
            w = deal_to_lanes<32, 0, 16>(w, scalar_load16(row + lo2));
            if (lane >= 32) my_lo = lo2;
            dealt = 48;
            if (n > 48) {
                const int lo3 = chunk_begin(3);
                w = deal_to_lanes<48, 0, 16>(w, scalar_load16(row + lo3));
                if (lane >= 48) my_lo = lo3;
                dealt = 64;
            }
        }
    }
    const int idx = my_lo + (lane & 15), k = n - 1 - idx;
    if (lane < dealt && idx < n && k >= 0 && k < kWindow) win[k] = w;
}

constexpr int kScalarRunMin = 8;       // bytes left in a token before a scalar-only walk looks for a run

// Walks a staged token from the configuration  view ++ priv[0..d)  with capacity checks.  Runs on
// all 64 lanes with identical values (scalar table loads, LDS broadcast reads); a run of
// self-similar edges is applied in one step.  Returns kFed, kRejected or kOverflow.
template <bool kScalar = false>
__device__ __forceinline__ int walk_staged_token(const DevTables &T, PrivateStack &priv, const int32_t *s_info,
                                                 StagedToken tok, const StackView &view, int cap, int &base, int &d,
                                                 int &top, int &kind) {
    const int n_bytes = tok.hi - tok.lo;
    int rc = n_bytes > 0 ? kFed : kRejected;
    for (int i = 0; i < n_bytes && rc == kFed; ++i) {
        int info = lds_read(s_info + (i < 64 ? i : 63));
        if (i >= 64) info = T.byte_info[T.vbytes[tok.lo + i]];
        info = __builtin_amdgcn_readfirstlane(info);
        int run_node = -1;
        rc = feed<true, true, kScalar>(T, priv, info, base, d, top, kind, view, cap, &run_node);
        // (a run is examined with one vector load per lane: a wave that keeps to scalar loads takes short tails byte by byte)
        if (rc == kFed && run_node >= 0 && i + 1 < n_bytes && (!kScalar || n_bytes - (i + 1) >= kScalarRunMin))
            i += apply_run<true>(T, priv, s_info, i + 1, n_bytes, run_node, kind, base, d, top, cap);
    }
    return rc;
}

// Writes the d private entries of a finished walk above row[0..base): the first kLdsDepth by one
// lane each, entries that spilled to global memory by lane 0.
__device__ __forceinline__ void commit_overlay(int32_t *row, const PrivateStack &priv, int base, int d, int lane) {
    const int in_lds = d < kLdsDepth ? d : kLdsDepth;
    if (lane < in_lds) row[base + lane] = priv.get(lane);
    if (lane == 0)
        for (int i = kLdsDepth; i < d; ++i) row[base + i] = priv.get(i);
}

// Cycle-aware stack compaction (Sec. 3.2.3; Alg. 1 step 1) of a stack staged in LDS, s[0 .. n): a
// complete traversal v1..vn of a registered reduction cycle that lies right below another v1 carries
// no information and is taken out.  The stack is rebuilt entry by entry from the bottom; after each
// entry that is the head of a cycle, the n entries under it are compared with the cycle's states
// and dropped on a match (then the check repeats).  Run by the 64 lanes of one wave in lockstep:
// lanes look up cycle_head for 64 entries at a time, a ballot finds the heads, lane i compares
// entry i of a traversal, segments between heads are moved down as blocks.  `pool` = the cycle
// records in their device layout (states last first, kCyclePoolPad entries of padding at the end),
// in LDS or global memory.  Returns the new length; *first_moved = lowest index whose
// content changed (= the new length if only the top was cut, n if nothing changed).
__device__ __forceinline__ int fold_cycles(int32_t *s, int n, const int32_t *cycle_head, const int32_t *pool,
                                           int n_states, int lane, int *first_moved) {
    // Where can the first traversal end?  Until one is dropped the stack has its original layout, and
    // a traversal of length k under the entry at position p needs s[p - k] == s[p] (both are the
    // cycle's first state): every lane tests that for one position and the cycles of its state, and
    // the rebuilding starts at the lowest position that passes -- in a stack that was compacted
    // before the call, that is inside the entries the call added.
    int start = n;
    for (int r0 = 0; r0 < n && start == n; r0 += 64) {
        const int p = r0 + lane;
        bool candidate = false;
        if (p < n) {
            const int x = s[p];
            for (int at = (unsigned)x < (unsigned)n_states ? cycle_head[x] : -1; at >= 0 && !candidate; at = pool[at + 1]) {
                const int k = pool[at];
                candidate = p - k >= 0 && s[p - k] == x;
            }
        }
        const unsigned long long c = __ballot(candidate);
        if (c) start = r0 + __ffsll((long long)c) - 1;
    }
    if (start == n) { *first_moved = n; return n; }
    int w = start, moved = n;
    for (int r0 = start; r0 < n; r0 += 64) {
        const int cnt = n - r0 < 64 ? n - r0 : 64;
        const int x = lane < cnt ? s[r0 + lane] : -1;
        const int hd = (unsigned)x < (unsigned)n_states ? cycle_head[x] : -1;
        unsigned long long heads = __ballot(hd >= 0);
        if (heads == 0 && w == r0) { w += cnt; continue; }
        int prev = 0;                                   // entries of this chunk already moved
        for (;;) {
            const int j = heads ? __ffsll((long long)heads) - 1 : cnt - 1;   // the segment prev..j ends at a head or at the chunk's end
            const int seg = j - prev + 1;
            if (seg > 0) {
                if (w != r0 + prev) {                   // all lanes read, then all lanes write: the ranges may overlap
                    const int v = lane < seg ? s[r0 + prev + lane] : 0;
                    __builtin_amdgcn_wave_barrier();
                    if (lane < seg) s[w + lane] = v;
                    __builtin_amdgcn_wave_barrier();
                    moved = w < moved ? w : moved;
                }
                w += seg;
            }
            if (!heads) break;
            heads &= heads - 1;
            prev = j + 1;
            const int first = __builtin_amdgcn_readlane(hd, j);   // s[w - 1] is the head of these cycles
            int h = first;
            while (h >= 0) {
                // one round of loads per record: its header, its states (stored last first and
                // padded, so no address depends on the length) and the entries under the head
                const int header = pool[h + (lane & 1)];
                const int want = pool[h + 2 + lane];
                const int have = w - 2 - lane >= 0 ? s[w - 2 - lane] : -1;
                const int k = __builtin_amdgcn_readlane(header, 0), next = __builtin_amdgcn_readlane(header, 1);
                const bool match = __all(lane >= k || have == want);   // an entry below the bottom (-1) matches no state
                if (match) {
                    w -= k;                             // the top stays: s[w - 1] held the same state
                    moved = w < moved ? w : moved;
                    // The new top failed every check when it was put there, over the same entries:
                    // no need to try its records again.  And the k entries just dropped, s[w .. w + k),
                    // took the stack from this very content back to it without any drop on the way, so
                    // every further copy of them that follows in the input does the same: skip those
                    // copies (as far as they lie in this chunk) at once.
                    const int left = cnt - prev;
                    if (left >= k) {
                        const bool same = lane < left && s[r0 + prev + lane] == s[w + lane % k];
                        const unsigned long long differs = ~__ballot(same);
                        const int run = differs ? __ffsll((long long)differs) - 1 : 64;
                        prev += run / k * k;
                        heads = prev >= 64 ? 0ull : heads & (~0ull << prev);
                    }
                    h = -1;
                } else {
                    h = next;
                }
            }
        }
    }
    *first_moved = moved;
    return w;
}

// The cycle tables (cycle_head[n_states], then the records) are small for most grammars: the threads
// given here copy them into LDS (`lds`, n_states + pool_n entries) so that fold_cycles, whose look-ups
// depend on one another, does not go to global memory for each.  The caller puts a block barrier
// between this copy and the first use.
constexpr int kStageCycleStates = 4096, kStageCyclePool = 1024;
__host__ __device__ inline bool cycles_fit_lds(int n_states, int pool_n) {
    return n_states <= kStageCycleStates && pool_n <= kStageCyclePool;
}
__device__ __forceinline__ void copy_cycle_tables(int32_t *lds, int n_states, int pool_n, const int32_t *head,
                                                  const int32_t *pool, int first, int step) {
    for (int i = first; i < n_states; i += step) lds[i] = head[i];
    for (int i = first; i < pool_n; i += step) lds[n_states + i] = pool[i];
}

// One wave per sequence: the walk of a single token is a chain of dependent table look-ups, so
// giving every sequence its own wave keeps control flow uniform (lanes of a shared wave would
// serialise each other's reduction chains) and lets the chip overlap the chains of all
// sequences.  The walk runs on a private overlay exactly like in the mask kernels; only a walk
// that succeeds is committed to the sequence's stack.
// kCompact (cycle-aware stacks): instead of committing the private entries, the wave puts the new
// stack together in LDS (cap entries per sequence), takes complete traversals of reduction cycles
// out of it (fold_cycles) and writes back what changed.
constexpr int kAdvSeqPerBlock = 4;
template <bool kCompact>
__global__ __launch_bounds__(64 * kAdvSeqPerBlock) void advance_kernel(
    DevTables T, DevTokenEdges E, const int32_t *__restrict__ tokens, int32_t *__restrict__ states,
    int32_t *__restrict__ data, int32_t *__restrict__ len, int cap, int batch, int32_t *__restrict__ err, int32_t *scratch,
    int restart_on_eos, const int32_t *cycle_head, const int32_t *cycle_pool, int stage_cycles) {
    extern __shared__ int32_t adv_stage[];             // kCompact: kAdvSeqPerBlock x (cap stack entries [+ cycle tables])
    __shared__ int32_t lds_stack[kLdsDepth * kAdvSeqPerBlock];
    __shared__ int32_t s_win[kAdvSeqPerBlock][kWindow], s_info[kAdvSeqPerBlock][64];
    __shared__ int32_t s_base[kAdvSeqPerBlock], s_depth[kAdvSeqPerBlock];
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int b = blockIdx.x * kAdvSeqPerBlock + wave;
    // kCompact with small cycle tables: the block copies them into LDS behind the staged stacks; every
    // wave passes exactly one block barrier (a wave without a sequence right here, the others once
    // their own input loads are under way)
    int32_t *cycle_lds = adv_stage + kAdvSeqPerBlock * cap;
    if (kCompact && stage_cycles) {
        copy_cycle_tables(cycle_lds, T.n_states, T.cycle_pool_n, cycle_head, cycle_pool, threadIdx.x, 64 * kAdvSeqPerBlock);
        cycle_head = cycle_lds;
        cycle_pool = cycle_lds + T.n_states;
    }
    if (b >= batch) {
        if (kCompact && stage_cycles) __syncthreads();
        return;
    }
    int32_t *row = data + (size_t)b * cap;
    PrivateStack priv;
    priv.lds = lds_stack + wave;
    priv.lds_stride = kAdvSeqPerBlock;
    priv.spill = scratch + b;
    priv.spill_stride = (size_t)batch;
    // every lane: the sequence's inputs, then (in parallel across lanes) the top of the stack and
    // the byte classes of the token, so that the walk finds them in LDS
    const int t = tokens[b];
    const int n = len[b];
    const int st = states[b];
    const bool live = t >= 0 && t < T.n_tokens && st >= 0 && n >= 1 && n <= cap;
    StagedToken tok{0, 0};
    // the root of the condition tree of the stack's top (states[b] names it) is fetched together with
    // the stack window and the token's bytes: the look-up of the token's stack operations starts from it
    int fx_root = -1;
    DevConditionNode fx_nd{};
    if (E.fx_slots && live && t != T.eos_id && (unsigned)st < (unsigned)T.n_states) {
        fx_root = E.root_id[st];
        fx_nd = E.root_nodes[st];
    }
    if (live) {
        s_win[wave][lane] = n - 1 - lane >= 0 ? row[n - 1 - lane] : -1;
        if (t != T.eos_id) tok = stage_token(T, t, lane, s_info[wave]);
    }
    if (kCompact && stage_cycles) __syncthreads();
    __builtin_amdgcn_wave_barrier();
    // all lanes hold identical values from here on; lane 0 alone writes the results
    int commit = -1, out_err = 0, out_state = st, out_len = n;
    int new_base = n, new_d = 0;                        // the new stack is  row[0 .. new_base) ++ priv[0 .. new_d)
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
                // a longer token whose merged edge carries its stack operations is applied in one step
                // (look-up, truncate, push), as in advance_fill_kernel; every other token is walked
                EffectHit fx{0, 0, 0, 0, 0, 0, 0};
                if (fx_root >= 0 && top == st && tok.hi - tok.lo >= E.fx_min_len)
                    fx = find_effect(E, __builtin_amdgcn_readfirstlane(fx_root), fx_nd, s_win[wave], n,
                                     [&](int k2) { return global_read(row + (n - 1 - k2)); }, t, lane);
                int rc;
                if (fx.found && fx.k <= n && fx.np <= T.max_depth) {
                    if (n + fx.peak >= cap) {
                        rc = kOverflow;
                    } else {
                        base = n - fx.k + 1;
                        if (fx.inline_count > 0) {
                            priv.set(0, fx.x0);
                            top = fx.x0;
                            if (fx.inline_count == 2) { priv.set(1, fx.x1); top = fx.x1; }
                        } else {
                            for (int i = 0; i < fx.np; ++i) {
                                top = table<true>(E.fx_pool, fx.x0 + i);
                                priv.set(i, top);
                            }
                        }
                        d = fx.np;
                        rc = kFed;
                    }
                } else {
                    rc = walk_staged_token(T, priv, s_info[wave], tok, view, cap, base, d, top, kind);
                }
                if (rc != kFed) {
                    out_err = rc == kOverflow ? 2 : 1;
                } else {
                    commit = d;
                    out_len = base + d;
                    out_state = top;
                    s_base[wave] = base;
                    new_base = base;
                    new_d = d;
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
    if (kCompact && n >= 1 && n <= cap) {
        int32_t *stack = adv_stage + wave * cap;
        int nl = out_len;                               // 1 after a restart: only the bottom entry stays
        for (int i = lane; i < nl; i += 64) stack[i] = i < new_base ? row[i] : priv.get(i - new_base);
        __builtin_amdgcn_wave_barrier();
        int first_moved = nl;
        if (nl >= 2) nl = fold_cycles(stack, nl, cycle_head, cycle_pool, T.n_states, lane, &first_moved);
        const int from = first_moved < new_base ? first_moved : new_base;
        for (int i = from + lane; i < nl; i += 64) row[i] = stack[i];
        if (lane == 0 && nl != out_len) len[b] = nl;    // the top, hence states[b], is the same
        return;
    }
    s_depth[wave] = commit;
    __builtin_amdgcn_wave_barrier();
    const int d = s_depth[wave];
    if (d > 0) commit_overlay(row, priv, s_base[wave], d, lane);
}

// The work of the wave that advances one sequence (all 64 lanes with identical values): walks the
// sampled token (or applies its stack-effect record), commits the new stack, stages the new top of
// the stack in s_new and descends the condition tree of the token-level edges with it; the result is
// `plan`.  kCompact: the new stack is put together at after_row (LDS, cap entries), folded and only
// then written back and looked up; stage_cycles: the block's other waves copy the cycle tables to
// after_row + cap meanwhile and meet this wave at one block barrier.
template <bool kCompact, bool kScalar = false>
__device__ __forceinline__ void advance_and_plan(const DevTables &T, const DevTokenEdges &E, const int32_t *__restrict__ tokens,
                                                 int32_t *__restrict__ states, int32_t *row, int32_t *__restrict__ len,
                                                 int cap, int batch, int32_t *__restrict__ err, int restart_on_eos,
                                                 int32_t *adv_scratch, const int32_t *cycle_head, const int32_t *cycle_pool,
                                                 int stage_cycles, int32_t *after_row, int32_t *s_win, int32_t *s_new,
                                                 int32_t *s_info, int32_t *s_adv_stack, RowPlan &plan, int b, int lane) {
    PrivateStack priv;
    priv.lds = s_adv_stack;
    priv.lds_stride = 1;
    priv.spill = adv_scratch + b;
    priv.spill_stride = (size_t)batch;
    const int t = kScalar ? table<true>(tokens, b) : tokens[b];
    const int n = kScalar ? table<true>(const_cast<const int32_t *>(len), b) : len[b];
    const int st = kScalar ? table<true>(const_cast<const int32_t *>(states), b) : states[b];
    const bool shape_ok = n >= 1 && n <= cap;
    const bool live = t >= 0 && t < T.n_tokens && st >= 0 && shape_ok;
    StagedToken tok{0, 0};
    // the root of the condition tree of the stack's top (states[b] names it) is fetched together
    // with the stack window and the token's bytes: the effect look-up starts from it
    int fx_root = -1;
    DevConditionNode fx_nd{};
    if (E.fx_slots && live && t != T.eos_id && (unsigned)st < (unsigned)T.n_states) {
        fx_root = kScalar ? table<true>(E.root_id, st) : E.root_id[st];
        fx_nd = kScalar ? scalar_node(E.root_nodes + __builtin_amdgcn_readfirstlane(st)) : E.root_nodes[st];
    }
    if (kScalar && cap >= 16) {
        stage_window_scalar(row, n, cap, shape_ok, lane, s_win);
        if (live && t != T.eos_id) tok = stage_token_scalar(T, __builtin_amdgcn_readfirstlane(t), lane, s_info);
    } else {
        s_win[lane] = (shape_ok && n - 1 - lane >= 0) ? row[n - 1 - lane] : -1;
        if (live && t != T.eos_id) tok = stage_token(T, t, lane, s_info);
    }
    if (kCompact && stage_cycles) {                 // the other waves have copied the cycle tables meanwhile
        __syncthreads();
        int32_t *cycle_lds = after_row + cap;
        cycle_head = cycle_lds;
        cycle_pool = cycle_lds + T.n_states;
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
                if (feed<false, true, kScalar>(T, priv, T.end_col, base, d, top, kind, view, 0) == kAccepted) {
                    out_state = -1;
                    if (restart_on_eos) { out_state = row[0]; out_len = 1; restarted = true; }   // slot reuse
                } else {
                    out_err = 1;
                }
                base = n;
                d = 0;                               // the '$' walk never changes the stack
            } else {
                // a longer token whose merged edge carries its stack operations is applied in one
                // step (look-up, truncate, push); every other token is walked byte by byte
                EffectHit fx{0, 0, 0, 0, 0, 0, 0};
                if (fx_root >= 0 && top == st && tok.hi - tok.lo >= E.fx_min_len) {
                    if (kScalar)
                        fx = find_effect_scalar(E, __builtin_amdgcn_readfirstlane(fx_root), fx_nd, s_win, n,
                                                [&](int k2) { return global_read(row + (n - 1 - k2)); }, __builtin_amdgcn_readfirstlane(t));
                    else
                        fx = find_effect(E, __builtin_amdgcn_readfirstlane(fx_root), fx_nd, s_win, n,
                                         [&](int k2) { return global_read(row + (n - 1 - k2)); }, t, lane);
                }
                int rc;
                if (fx.found && fx.k <= n && fx.np <= T.max_depth) {
                    if (n + fx.peak >= cap) {
                        rc = kOverflow;
                    } else {
                        base = n - fx.k + 1;
                        if (fx.inline_count > 0) {
                            priv.set(0, fx.x0);
                            top = fx.x0;
                            if (fx.inline_count == 2) { priv.set(1, fx.x1); top = fx.x1; }
                        } else {
                            for (int i = 0; i < fx.np; ++i) {
                                top = table<true>(E.fx_pool, fx.x0 + i);
                                priv.set(i, top);
                            }
                        }
                        d = fx.np;
                        rc = kFed;
                    }
                } else {
                    rc = walk_staged_token<kScalar>(T, priv, s_info, tok, view, cap, base, d, top, kind);
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
    // ---- the new stack is  row[0 .. base) ++ priv[0 .. d)  (or just its bottom after a restart).
    // Its top is staged and the condition tree descended BEFORE anything is stored: a wave that has
    // stores in flight waits for them wherever it next waits for a load, and in the one-launch step
    // kernel they complete only behind the row loads of the block's other waves.
    int nl = out_len;
    if (kCompact && shape_ok) {
        // put it together in LDS, compact it, write back what changed
        int32_t *stack = after_row;
        for (int i = lane; i < nl; i += 64)
            stack[i] = i < base ? StackView{row, s_win, n}.at(i) : priv.get(i - base);
        __builtin_amdgcn_wave_barrier();
        int first_moved = nl;
        if (nl >= 2) nl = fold_cycles(stack, nl, cycle_head, cycle_pool, T.n_states, lane, &first_moved);
        auto new_at = [&](int k) -> int32_t { return k < nl ? stack[nl - 1 - k] : -1; };
        s_new[lane] = lane < nl ? stack[nl - 1 - lane] : -1;
        __builtin_amdgcn_wave_barrier();
        const int top = s_new[0];
        if (out_state < 0) {
            if (lane == 0) plan.mode = kRowDone;
        } else if ((unsigned)top >= (unsigned)T.n_states) {
            if (lane == 0) plan.mode = kRowEmpty;
        } else {
            if (kScalar) plan_row_scalar(E, scalar_node(E.root_nodes + __builtin_amdgcn_readfirstlane(top)), s_new, nl, new_at, &plan, lane);
            else plan_row(E, E.root_nodes[top], s_new, nl, new_at, &plan, lane);
        }
        if (lane == 0) { plan.top = top; plan.len = nl; }
        const int from = restarted ? nl : (first_moved < base ? first_moved : base);
        for (int i = from + lane; i < nl; i += 64) row[i] = stack[i];
        if (lane == 0) {
            err[b] = out_err;
            if ((out_err == 0 && t >= 0) || nl != n) { states[b] = out_state; len[b] = nl; }
        }
    } else {
        auto new_at = [&](int k) -> int32_t {           // entry k below the new top
            if (restarted) return k == 0 ? (kScalar ? table<true>(const_cast<const int32_t *>(row), 0) : row[0]) : -1;
            if (k < d) return priv.get(d - 1 - k);
            const int idx = base - 1 - (k - d);
            return idx >= 0 ? StackView{row, s_win, n}.at(idx) : -1;
        };
        s_new[lane] = (shape_ok && lane < nl) ? new_at(lane) : -1;
        __builtin_amdgcn_wave_barrier();
        // ---- descent of the condition tree with the new stack
        const int top = s_new[0];
        if (out_state < 0) {
            if (lane == 0) plan.mode = kRowDone;
        } else if (!shape_ok || (unsigned)top >= (unsigned)T.n_states) {
            if (lane == 0) plan.mode = kRowEmpty;
        } else {
            if (kScalar) plan_row_scalar(E, scalar_node(E.root_nodes + __builtin_amdgcn_readfirstlane(top)), s_new, nl, new_at, &plan, lane);
            else plan_row(E, E.root_nodes[top], s_new, nl, new_at, &plan, lane);
        }
        if (lane == 0) { plan.top = top; plan.len = nl; }
        // ---- commit the private part
        commit_overlay(row, priv, base, d, lane);
        if (lane == 0) {
            err[b] = out_err;
            if (out_err == 0 && t >= 0) { states[b] = out_state; len[b] = out_len; }
        }
    }
}

// Advance and next mask in one launch: one block per sequence.  Wave 0 walks the sampled token
// exactly like advance_kernel (scalar table loads), commits the new stack, stages the NEW top
// of the stack in LDS and descends the condition tree of the token-level edges with it; then the
// whole block builds the sequence's next mask row (dense row copy, delta lists, leftover walks)
// and stores it.  The sequence's inputs are loaded once, no kernel boundary separates the two
// halves, and the long walks of a few sequences overlap the mask building of all others.
// kCompact (cycle-aware stacks): the new stack is put together in LDS, complete traversals of reduction
// cycles are taken out of it (fold_cycles) and only then is it written back and looked up, so the call
// leaves compacted stacks and the mask of exactly those stacks.
constexpr int kAfBlock = 512;
// LDS the kernel declares statically (stack windows, token bytes, private stacks, the row plan),
// rounded up: what is left of the 64 KB for the dynamic part (mask row, staged stack)
constexpr size_t kAfStaticLdsBytes =
    ((sizeof(int32_t) * (2 * kWindow + 64 + kLdsDepth + kLdsDepth * 64) + sizeof(RowPlan)) + 1023) & ~(size_t)1023;
constexpr size_t kAfDynamicLdsMax = 65536 - kAfStaticLdsBytes;
template <bool kCompact>
__global__ __launch_bounds__(kAfBlock) void advance_fill_kernel(
    DevTables T, DevTokenEdges E, const int32_t *__restrict__ tokens, int32_t *__restrict__ states,
    int32_t *__restrict__ data, int32_t *__restrict__ len, int cap, int batch, int32_t *__restrict__ err,
    uint32_t *__restrict__ bitmask, int restart_on_eos, int32_t *adv_scratch, int32_t *walk_spill,
    size_t walk_spill_stride, const int32_t *cycle_head, const int32_t *cycle_pool, int stage_cycles) {
    extern __shared__ uint4 bits4[];                   // whole row: n_words rounded up to a multiple of 4;
                                                       // kCompact: followed by cap stack entries [+ cycle tables]
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
        const int64_t per_xcd = (gridDim.x + 7) >> 3, idle = kAfBlock - 64;
        int acc = 0;
        for (int64_t off = ((int64_t)(blockIdx.x >> 3) * idle + (tid - 64)) * 128; off < T.hot_bytes; off += per_xcd * idle * 128)
            acc |= *(const volatile __attribute__((address_space(1))) int *)(T.hot_begin + off);
        if (acc == 0x7ff1234f && T.fault) atomicAdd(T.fault, 0);   // keeps the loads alive; no effect
        if (kCompact && stage_cycles) {                 // ... and copy the cycle tables into LDS for wave 0
            int32_t *cycle_lds = reinterpret_cast<int32_t *>(bits4 + ((T.n_words + 3) >> 2)) + cap;
            copy_cycle_tables(cycle_lds, T.n_states, T.cycle_pool_n, cycle_head, cycle_pool, tid - 64, kAfBlock - 64);
            __syncthreads();
        }
    }
    if (tid < 64) {
        advance_and_plan<kCompact>(T, E, tokens, states, row, len, cap, batch, err, restart_on_eos, adv_scratch, cycle_head,
                                   cycle_pool, stage_cycles, reinterpret_cast<int32_t *>(bits4 + ((T.n_words + 3) >> 2)), s_win,
                                   s_new, s_info, s_adv_stack, plan, b, lane);
    }
    __syncthreads();
    // ---- the next mask row, by the whole block
    PrivateStack wp;                                    // leftovers are walked on the committed stack
    wp.lds = s_walk_stack + lane;
    wp.lds_stride = 64;
    wp.spill = walk_spill + (size_t)b * 64 + lane;
    wp.spill_stride = walk_spill_stride;
    const bool vector_ok = (T.n_words & 3) == 0 && (reinterpret_cast<uintptr_t>(bitmask) & 15) == 0;
    build_and_store_row<kAfBlock, true, true>(T, E, plan, bits4, 0, n_vec, row, wp, bitmask + (size_t)b * T.n_words, vector_ok, tid);
}

// The part of advance_and_plan that is left when there is no token: the top of the stack as it stands is
// staged in s_new and the condition tree descended with it, through scalar loads (the step kernel's
// wave 0 when the kernel is asked for mask + masking only).
__device__ __forceinline__ void plan_only_scalar(const DevTables &T, const DevTokenEdges &E, const int32_t *states,
                                                 const int32_t *row, const int32_t *len, int cap, int32_t *s_new,
                                                 RowPlan &plan, int b, int lane) {
    const int n = table<true>(len, b);
    const int st = table<true>(states, b);
    const bool shape_ok = n >= 1 && n <= cap;
    if (cap >= 16) stage_window_scalar(row, n, cap, shape_ok, lane, s_new);
    else s_new[lane] = (shape_ok && n - 1 - lane >= 0) ? row[n - 1 - lane] : -1;
    __builtin_amdgcn_wave_barrier();
    const int top = s_new[0];
    if (st < 0) {
        if (lane == 0) plan.mode = kRowDone;
    } else if (!shape_ok || (unsigned)top >= (unsigned)T.n_states) {
        if (lane == 0) plan.mode = kRowEmpty;
    } else {
        plan_row_scalar(E, scalar_node(E.root_nodes + __builtin_amdgcn_readfirstlane(top)), s_new, n,
                        [&](int k) { return global_read(row + (n - 1 - k)); }, &plan, lane);
    }
    if (lane == 0) { plan.top = top; plan.len = n; }
}

// The whole decode step in one launch: advance, next mask row, and that row applied to the
// sequence's logits.  One 1,024-thread block per sequence.  Wave 0 advances and descends the
// condition tree as in advance_fill_kernel, but through scalar loads only (vector loads return in order
// per compute unit: behind the row loads of this block each of them would wait microseconds).  The
// other fifteen waves meanwhile fetch the
// sequence's whole row of logits -- the fetch does not depend on the mask -- into registers (kHeld
// groups of 8 bf16 per lane, lane j of the 960 holding groups j, j + 960, ...), so the read half of
// the masking pass runs under the advance instead of after it; once the plan is there they put the
// mask row together in LDS (materialised row, id lists; wave 0 walks what the tree left open),
// store it, and patch and store the logits they hold.  The two halves are separate branches of the
// kernel with the same number of block barriers, so the registers that hold the logits are not live
// in wave 0's code.  Masked logits are exactly those of apply_mask_vec8_kernel (-inf where a bit is
// clear, 128-byte lines written whole or not at all).
// kArgmax: the greedy decode step.  The logits are not written back; instead every lane takes the arg max
// of the allowed logits among the groups it holds (the order keys of masked_argmax_kernel, the same rules:
// largest value, first of equal values, +0 = -0, NaN never), the block combines the lanes, and out_tokens[b]
// is the sequence's next token (-1 if nothing is allowed).  out_tokens may be the tokens buffer: block b
// reads tokens[b] before anything else and writes out_tokens[b] last.
// tokens == nullptr: no advance -- the mask of the stacks as they are, and the masking (states, data and
// len are then only read).
constexpr int kStepBlock = 1024, kStepData = kStepBlock - 64;
static_assert(kStepBlock == kArgBlock, "the step kernel combines its lanes with argmax_block_max");
template <bool kCompact, int kHeld, bool kArgmax>
__global__ __launch_bounds__(kStepBlock) void advance_fill_apply_kernel(
    DevTables T, DevTokenEdges E, const int32_t *tokens, int32_t *__restrict__ states,
    int32_t *__restrict__ data, int32_t *__restrict__ len, int cap, int batch, int32_t *__restrict__ err,
    uint32_t *__restrict__ bitmask, int restart_on_eos, int32_t *adv_scratch, int32_t *walk_spill,
    size_t walk_spill_stride, const int32_t *cycle_head, const int32_t *cycle_pool, int stage_cycles,
    uint16_t *__restrict__ logits, int64_t row_stride, int32_t *out_tokens, int first_row) {
    extern __shared__ uint4 bits4[];                   // the mask row; kCompact: then cap stack entries [+ cycle tables]
    __shared__ int32_t s_win[kWindow], s_new[kWindow], s_info[64];
    __shared__ int32_t s_adv_stack[kLdsDepth], s_walk_stack[kLdsDepth * 64];
    __shared__ RowPlan plan;
    const int tid = threadIdx.x, lane = tid & 63;
    const int b = first_row + blockIdx.x;          // (a large batch comes as several launches of one row per compute unit)
    const int n_vec = (T.n_words + 3) >> 2;
    int32_t *row = data + (size_t)b * cap;
    uint32_t *bits = reinterpret_cast<uint32_t *>(bits4);
    uint32_t *dst_row = bitmask + (size_t)b * T.n_words;
    const bool vector_ok = (T.n_words & 3) == 0 && (reinterpret_cast<uintptr_t>(bitmask) & 15) == 0;
    uint16_t *lrow = logits + (size_t)b * row_stride;
    unsigned long long mine = 0ull;                    // kArgmax: this lane's candidate
    // kArgmax: half a mask byte -> AND masks of two registers.  Sixteen entries: lanes that read the same entry are
    // served together and different entries lie in different banks (a 256-entry table of whole bytes cost 4-way
    // bank conflicts on every read: 5.1 us for the arg max of a block instead of the 3.3 us it takes now)
    __shared__ uint2 s_expand[kArgmax ? 16 : 1];
    __shared__ unsigned long long s_part[kArgmax ? kStepBlock / 64 + 1 : 1];

    if (tid < 64) {
        if (tokens)
            advance_and_plan<kCompact, true>(T, E, tokens, states, row, len, cap, batch, err, restart_on_eos, adv_scratch,
                                             cycle_head, cycle_pool, stage_cycles, reinterpret_cast<int32_t *>(bits4 + n_vec),
                                             s_win, s_new, s_info, s_adv_stack, plan, b, lane);
        else
            plan_only_scalar(T, E, states, row, len, cap, s_new, plan, b, lane);
        // (barriers that order LDS only: this wave's stores of the new stack are still on their way, and
        // nothing in this block reads them before the launch ends -- except the walks below, which wait)
        lds_barrier();                                 // the plan is there
        lds_barrier();                                 // the materialised row (or zeros) is in LDS
        // tokens the tree leaves undetermined are walked on the committed stack, one lane per token
        PrivateStack wp;
        wp.lds = s_walk_stack + lane;
        wp.lds_stride = 64;
        wp.spill = walk_spill + (size_t)b * 64 + lane;
        wp.spill_stride = walk_spill_stride;
        const int mode = plan.mode, n = plan.len, top0 = plan.top;
        if (mode == kRowWalkAll || (mode == kRowFast && plan.walk_count > 0))
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");      // the walks read the committed stack
        if (mode == kRowFast) {
            const int wc = plan.walk_count;
            for (int k = lane; k < wc; k += 64) {
                const int t = E.walk_ids[plan.walk_begin + k];
                if (walk_token_id(T, wp, t, row, n, top0)) atomicOr(&bits[t >> 5], 1u << (t & 31));
            }
        } else if (mode == kRowWalkAll) {
            for (int t = lane; t < T.n_tokens; t += 64)
                if (walk_token_id(T, wp, t, row, n, top0)) atomicOr(&bits[t >> 5], 1u << (t & 31));
        } else if (mode == kRowDone && lane == 0) {
            bits[T.eos_id >> 5] = 1u << (T.eos_id & 31);
        }
        lds_barrier();                                 // the row is complete
        if (kArgmax) mine = argmax_block_max(0ull, s_part, tid);
    } else {
        const int j = tid - 64;
        if (kCompact && stage_cycles) {
            int32_t *cycle_lds = reinterpret_cast<int32_t *>(bits4 + n_vec) + cap;
            copy_cycle_tables(cycle_lds, T.n_states, T.cycle_pool_n, cycle_head, cycle_pool, j, kStepData);
            __syncthreads();
        }
        // the row of logits: every group of 8 that lies wholly inside the vocabulary
        const int whole = T.n_tokens >> 3;
        uint4 held[kHeld];
#pragma unroll
        for (int i = 0; i < kHeld; ++i) {
            const int g = i * kStepData + j;
            held[i] = make_uint4(0u, 0u, 0u, 0u);
            // (a wave-uniform base per i plus one 32-bit lane offset: no 64-bit address register per group)
            if (g < whole) held[i] = stream_load(lrow + (size_t)i * (kStepData * 8) + (uint32_t)(j * 8));
        }
        if (kArgmax) {
            if (j < 16) {
                uint32_t am[2];
#pragma unroll
                for (int q = 0; q < 2; ++q) am[q] = (((j >> (2 * q)) & 1) ? 0x0000FFFFu : 0u) | (((j >> (2 * q + 1)) & 1) ? 0xFFFF0000u : 0u);
                s_expand[j] = make_uint2(am[0], am[1]);
            }
            // the patterns become order keys as the groups arrive, under the loads still in flight
#pragma unroll
            for (int i = 0; i < kHeld; ++i)
                held[i] = make_uint4(bf16_order_keys(held[i].x), bf16_order_keys(held[i].y), bf16_order_keys(held[i].z),
                                     bf16_order_keys(held[i].w));
        }
        lds_barrier();                                 // the plan is there
        const int mode = plan.mode;
        if (mode == kRowFast && plan.dense >= 0) {
            const uint4 *src = reinterpret_cast<const uint4 *>(E.dense_rows) + (size_t)plan.dense * n_vec;
            for (int w = j; w < n_vec; w += kStepData) bits4[w] = src[w];
        } else {
            for (int w = j; w < n_vec; w += kStepData) bits4[w] = make_uint4(0, 0, 0, 0);
        }
        lds_barrier();                                 // the materialised row (or zeros) is in LDS
        if (mode == kRowFast) {
            const int nseg = plan.nseg;
            for (int i = 0; i < nseg; ++i) {
                const int32_t *ids = E.delta_ids + plan.seg_begin[i];
                const int cnt = plan.seg_count[i];
                for (int k = j; k < cnt; k += kStepData) {
                    const int t = ids[k];
                    atomicOr(&bits[t >> 5], 1u << (t & 31));
                }
            }
        }
        lds_barrier();                                 // the row is complete
        if (vector_ok) {
            uint4 *dst4 = reinterpret_cast<uint4 *>(dst_row);
            for (int w = j; w < n_vec; w += kStepData) stream_store(bits4[w], dst4 + w);
        } else {
            for (int w = j; w < T.n_words; w += kStepData) dst_row[w] = bits[w];
        }
        const uint8_t *mask_bytes = reinterpret_cast<const uint8_t *>(bits4);     // byte g = bits of group g
        if (kArgmax) {
            // Per group: the AND masks of the two halves of the mask byte come from the LDS table, masked halves
            // get the lowest key, three packed maxima fold the group, and only the best key and the slot of its
            // group are kept (a lane's groups ascend, so `>` keeps the first of equal values).  The block is
            // combined on (key, group): groups are disjoint runs of ascending ids, so the first of equal values
            // lies in the smallest group.  Only the one lane that holds the winning group then picks that
            // group out of its registers and finds the token inside it.
            int best = kOrderNegInf - 1, best_i = -1;   // only a valid value (or a positive NaN pattern) beats the start
            auto group_best = [&](uint4 v, uint32_t mu) {        // v: the group's order keys
                const uint2 lo = s_expand[mu & 15u], hi = s_expand[mu >> 4];
                const uint32_t k01 = packed_max_s16(mask_order_keys(v.x, lo.x), mask_order_keys(v.y, lo.y));
                const uint32_t k23 = packed_max_s16(mask_order_keys(v.z, hi.x), mask_order_keys(v.w, hi.y));
                const uint32_t kk = packed_max_s16(k01, k23);
                return max((int)(int16_t)(kk & 0xFFFFu), (int)kk >> 16);
            };
#pragma unroll
            for (int i = 0; i < kHeld; ++i) {
                // no branches: a group outside the row or without an allowed token gets the lowest key in every
                // half, which is below the start value, and the LDS reads of the groups can overlap (the row's
                // LDS area is at least kHeld * kStepData bytes, so the byte is read at a fixed offset)
                const int g = i * kStepData + j;
                const uint32_t mu = mask_bytes[g];
                const int gb = group_best(held[i], g < whole ? mu : 0u);
                best_i = gb > best ? i : best_i;
                best = max(gb, best);
            }
            int best_g = best_i >= 0 ? best_i * kStepData + j : -1;
            uint4 tail_keys = make_uint4(0, 0, 0, 0);
            uint32_t tail_m = 0u;
            const int tail = T.n_tokens & 7;
            if (tail > 0 && j == 0) {                   // the last, partial group: its logits one at a time
                uint32_t x[4] = {0u, 0u, 0u, 0u};
#pragma unroll
                for (int k = 0; k < 7; ++k)
                    if (k < tail) x[k >> 1] |= (uint32_t)lrow[whole * 8 + k] << (16 * (k & 1));
                const uint32_t mu = mask_bytes[whole] & ((1u << tail) - 1u);
                if (mu != 0u) {
                    const uint4 v = make_uint4(bf16_order_keys(x[0]), bf16_order_keys(x[1]), bf16_order_keys(x[2]), bf16_order_keys(x[3]));
                    const int gb = group_best(v, mu);
                    if (gb > best) { best = gb; best_g = whole; tail_keys = v; tail_m = mu; }
                }
            }
            const unsigned long long word = best_g >= 0 ? argmax_word(best, best_g) : 0ull;
            mine = argmax_block_max(word, s_part, tid);
            const int top = (int)(uint32_t)(mine >> 32) - 32768;
            if (word != 0ull && word == mine && !(top > kOrderPosInf || top == 0)) {
                uint4 keys = tail_keys;                 // the winning lane: its group's keys and mask byte
                uint32_t m = tail_m;
                if (best_g != whole || tail_m == 0u) {
#pragma unroll
                    for (int i = 0; i < kHeld; ++i)
                        if (best_i == i) keys = held[i];
                    m = mask_bytes[best_g];
                }
                const uint32_t x[4] = {keys.x, keys.y, keys.z, keys.w};
                int first = 0;
#pragma unroll
                for (int k = 7; k >= 0; --k) {          // descending: the smallest k is assigned last
                    const int key = (k & 1) ? ((int)x[k >> 1] >> 16) : (int)(int16_t)(x[k >> 1] & 0xFFFFu);
                    if (((m >> k) & 1u) && key == best) first = k;
                }
                out_tokens[b] = best_g * 8 + first;
            }
        } else {
#pragma unroll
        for (int i = 0; i < kHeld; ++i) {
            const int g = i * kStepData + j;
            // a group that needs no change is still written if one of the eight groups of its 128-byte line
            // does: lines written in part cost the memory system far more than the bytes saved
            const uint32_t mu = g < whole ? mask_bytes[g] : 0xFFu;
            const unsigned long long changed = __ballot(mu != 0xFFu);
            if (g < whole) {
                if ((changed >> (lane & 56)) & 0xFFull) {
                    uint4 v = held[i];
                    uint32_t *x = reinterpret_cast<uint32_t *>(&v);
#pragma unroll
                    for (int k = 0; k < 4; ++k) {
                        const uint32_t lo = (uint32_t)__builtin_amdgcn_sbfe((int)mu, 2 * k, 1);
                        const uint32_t hi = (uint32_t)__builtin_amdgcn_sbfe((int)mu, 2 * k + 1, 1);
                        const uint32_t allow = __builtin_amdgcn_perm(hi, lo, 0x05040100u);
                        x[k] = (x[k] & allow) | (~allow & kNegInfPair);
                    }
                    stream_store(v, lrow + (size_t)i * (kStepData * 8) + (uint32_t)(j * 8));
                }
            }
        }
        // the last, partial group of a vocabulary that is not a multiple of 8
        const int tail = T.n_tokens & 7;
        if (j < tail) {
            const int t = whole * 8 + j;
            if (!((bits[t >> 5] >> (t & 31)) & 1u)) lrow[t] = 0xFF80;
        }
        }
    }
    if (kArgmax) {
        // `mine` is the block's best (key, group) word in every thread.  The lane that holds it has written the
        // token unless the keys cannot decide: a positive NaN pattern or a zero on top are compared as numbers.
        const int top = (int)(uint32_t)(mine >> 32) - 32768;
        if (mine == 0ull) {
            if (tid == 0) out_tokens[b] = -1;
        } else if (top > kOrderPosInf || top == 0) {
            mine = argmax_block_max(argmax_segment_by_compare_inline(lrow, reinterpret_cast<const uint8_t *>(bits4), 0,
                                                                     (T.n_tokens + 7) >> 3, T.n_tokens, tid), s_part, tid);
            if (tid == 0) out_tokens[b] = mine != 0ull ? (int32_t)(0xFFFFFFFFu - (uint32_t)mine) : -1;
        }
    }
}

// Jump-forward: while a sequence's text is not a sentence and exactly one byte keeps it a viable
// prefix, that byte is forced; it is emitted and the stack is advanced by it.  One wave per
// sequence.  At every position lane c tries byte class c (and one lane the end-of-input symbol)
// from the current stack on a private overlay of its own -- the walk of a one-byte token --, the
// wave adds up the BYTES of the viable classes, and if that is one (and '$' is not accepted) the
// forced byte is walked on the real stack by all lanes together, exactly like in advance_kernel.
// kCompact (cycle-aware stacks): at the end the wave stages its stack in LDS (cap entries per
// sequence), takes complete traversals of reduction cycles out of it and writes back what changed.
constexpr int kJfSeqPerBlock = 4;
template <bool kCompact>
__global__ __launch_bounds__(64 * kJfSeqPerBlock) void jump_forward_kernel(
    DevTables T, int32_t *__restrict__ states, int32_t *__restrict__ data, int32_t *__restrict__ len, int cap,
    int batch, uint8_t *__restrict__ out_bytes, int32_t *__restrict__ out_len, int max_bytes, int32_t *adv_scratch,
    int32_t *lane_spill, size_t lane_spill_stride, const int32_t *cycle_head, const int32_t *cycle_pool,
    int stage_cycles) {
    extern __shared__ int32_t jf_stage[];              // kCompact: kJfSeqPerBlock x (cap stack entries [+ cycle tables])
    __shared__ int32_t s_trial[kJfSeqPerBlock][kLdsDepth * 64];
    __shared__ int32_t s_adv[kJfSeqPerBlock][kLdsDepth];
    __shared__ int32_t s_win[kJfSeqPerBlock][kWindow], s_new[kJfSeqPerBlock][kWindow];
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int b = blockIdx.x * kJfSeqPerBlock + wave;
    if (kCompact && stage_cycles) {                     // small cycle tables: copied into LDS by the whole block
        int32_t *cycle_lds = jf_stage + kJfSeqPerBlock * cap;
        copy_cycle_tables(cycle_lds, T.n_states, T.cycle_pool_n, cycle_head, cycle_pool, threadIdx.x, 64 * kJfSeqPerBlock);
        cycle_head = cycle_lds;
        cycle_pool = cycle_lds + T.n_states;
        __syncthreads();
    }
    if (b >= batch) return;
    int32_t *row = data + (size_t)b * cap;
    int n = len[b];
    const int st = states[b];
    int count = 0;
    if (st >= 0 && n >= 1 && n <= cap && max_bytes > 0) {
        s_win[wave][lane] = n - 1 - lane >= 0 ? row[n - 1 - lane] : -1;
        __builtin_amdgcn_wave_barrier();
        int top = __builtin_amdgcn_readfirstlane(s_win[wave][0]);
        if ((unsigned)top < (unsigned)T.n_states) {
            int kind = T.state_kind ? table<true>(T.state_kind, top) : 0;
            PrivateStack trial;                        // one column per lane
            trial.lds = s_trial[wave] + lane;
            trial.lds_stride = 64;
            trial.spill = lane_spill + (size_t)b * 64 + lane;
            trial.spill_stride = lane_spill_stride;
            PrivateStack adv;                          // the wave's own walk of a forced byte
            adv.lds = s_adv[wave];
            adv.lds_stride = 1;
            adv.spill = adv_scratch + b;
            adv.spill_stride = (size_t)batch;
            int new_top = top;
            while (count < max_bytes) {
                // a state whose only edge shifts one byte starts a run of forced bytes known since the
                // tables were compiled: emitted and pushed in one step (the byte-by-byte search below
                // would find the same bytes one at a time)
                const int run = T.run_off ? table<true>(T.run_off, top) : -1;
                if (run >= 0) {
                    int take = table<true>(T.run_pool, run);
                    take = take < max_bytes - count ? take : max_bytes - count;
                    take = take < cap - n ? take : cap - n;
                    if (take <= 0) break;                  // the stack is full
                    const int word = lane < take ? T.run_pool[run + 1 + lane] : 0;
                    if (lane < take) {
                        row[n + lane] = word >> 8;
                        out_bytes[(size_t)b * max_bytes + count + lane] = (uint8_t)(word & 0xFF);
                    }
                    // the new top of the stack: the run's states, then what was the top before
                    const int from_run = __shfl(word, take - 1 - lane < 0 ? 0 : take - 1 - lane) >> 8;
                    const int below = lane >= take ? s_win[wave][lane - take] : -1;
                    __builtin_amdgcn_wave_barrier();
                    s_win[wave][lane] = lane < take ? from_run : below;
                    __builtin_amdgcn_wave_barrier();
                    n += take;
                    top = __builtin_amdgcn_readfirstlane(s_win[wave][0]);
                    kind = T.state_kind ? table<true>(T.state_kind, top) : 0;
                    count += take;
                    continue;
                }
                const StackView view{row, s_win[wave], n};
                int viable_bytes = 0, only = -1;
                bool at_end = false;
                for (int c0 = 0; c0 < T.ncol; c0 += 64) {
                    const int c = c0 + lane;
                    int res = kRejected;
                    if (c < T.ncol) {
                        int base = n, d = 0, tp = top, tr = kind;
                        res = feed<false, false>(T, trial, c, base, d, tp, tr, view, 0);
                    }
                    if (__ballot(c == T.end_col && res == kAccepted)) at_end = true;
                    int bytes_here = (c < T.end_col && res == kFed) ? (T.class_info[c] & 0xFFFF) : 0;
                    const unsigned long long m = __ballot(bytes_here > 0);
                    if (m) only = c0 + __ffsll((long long)m) - 1;
#pragma unroll
                    for (int off = 32; off >= 1; off >>= 1) bytes_here += __shfl_xor(bytes_here, off);
                    viable_bytes += bytes_here;
                }
                if (at_end || viable_bytes != 1) break;
                const int byte = __builtin_amdgcn_readfirstlane(T.class_info[only] >> 16);
                const int info = __builtin_amdgcn_readfirstlane(T.byte_info[byte]);
                int base = n, d = 0;
                new_top = top;
                int new_kind = kind;
                if (feed<true, true>(T, adv, info, base, d, new_top, new_kind, view, cap) != kFed) break;   // would exceed cap
                // commit: stage the new top of the stack, then write the pushed entries
                int entry = -1;
                if (lane < base + d) {
                    if (lane < d) {
                        entry = adv.get(d - 1 - lane);
                    } else {
                        const int idx = base - 1 - (lane - d);
                        entry = idx >= 0 ? view.at(idx) : -1;
                    }
                }
                s_new[wave][lane] = entry;
                commit_overlay(row, adv, base, d, lane);
                if (lane == 0) out_bytes[(size_t)b * max_bytes + count] = (uint8_t)byte;
                __builtin_amdgcn_wave_barrier();
                s_win[wave][lane] = s_new[wave][lane];
                __builtin_amdgcn_wave_barrier();
                n = base + d;
                top = new_top;
                kind = new_kind;
                ++count;
            }
            if (lane == 0 && count > 0) {
                len[b] = n;
                states[b] = top;
            }
        }
    }
    if (lane == 0) out_len[b] = count;
    if (kCompact && n >= 2 && n <= cap) {
        // n is the current length (the entries committed above are this wave's own stores)
        __threadfence_block();
        int32_t *stack = jf_stage + wave * cap;
        for (int i = lane; i < n; i += 64) stack[i] = row[i];
        __builtin_amdgcn_wave_barrier();
        int first_moved = n;
        const int w = fold_cycles(stack, n, cycle_head, cycle_pool, T.n_states, lane, &first_moved);
        if (w != n) {
            for (int i = first_moved + lane; i < w; i += 64) row[i] = stack[i];
            if (lane == 0) len[b] = w;
        }
    }
}


// Stack compaction as a kernel of its own (after advance_kernel and jump_forward_kernel): one wave
// per sequence, the stack staged in LDS (cap entries per wave) next to a copy of the cycle records
// (pool_n entries; 0 = read them from global memory).  A stack without any cycle head costs one
// pass over its entries and writes nothing.
__global__ __launch_bounds__(256) void compact_stacks_kernel(const int32_t *__restrict__ cycle_head,
                                                             const int32_t *__restrict__ cycle_pool, int pool_n,
                                                             int n_states, int32_t *__restrict__ data,
                                                             int32_t *__restrict__ len, int cap, int batch) {
    extern __shared__ int32_t compact_lds[];
    for (int i = threadIdx.x; i < pool_n; i += blockDim.x) compact_lds[i] = cycle_pool[i];
    __syncthreads();
    const int32_t *pool = pool_n > 0 ? compact_lds : cycle_pool;
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int b = blockIdx.x * (blockDim.x >> 6) + wave;
    if (b >= batch) return;
    const int n = len[b];
    if (n < 2 || n > cap) return;
    int32_t *s = compact_lds + pool_n + wave * cap;
    int32_t *row = data + (size_t)b * cap;
    bool any = false;
    for (int i = lane; i < n; i += 64) {
        const int x = row[i];
        s[i] = x;
        any |= (unsigned)x < (unsigned)n_states && cycle_head[x] >= 0;
    }
    if (!__any(any)) return;
    __builtin_amdgcn_wave_barrier();
    int first_moved;
    const int w = fold_cycles(s, n, cycle_head, pool, n_states, lane, &first_moved);
    if (w != n) {
        for (int i = first_moved + lane; i < w; i += 64) row[i] = s[i];
        if (lane == 0) len[b] = w;
    }
}

}  // namespace

hipError_t static_advance_scratch(int32_t **out) {
    constexpr int kMaxDevices = 64;
    static std::mutex lock;
    static int32_t *address[kMaxDevices] = {};
    int device = -1;
    hipError_t e = hipGetDevice(&device);
    if (e != hipSuccess) return e;
    if (device < 0 || device >= kMaxDevices) return hipErrorInvalidDevice;
    std::lock_guard<std::mutex> guard(lock);
    if (!address[device]) {
        void *p = nullptr;
        e = hipGetSymbolAddress(&p, HIP_SYMBOL(pre3_static_scratch));
        if (e != hipSuccess) return e;
        if (!p) return hipErrorInvalidSymbol;
        address[device] = static_cast<int32_t *>(p);
    }
    *out = address[device];
    return hipSuccess;
}

size_t advance_scratch_entries(int batch, int max_depth) {
    const int deep = max_depth > kLdsDepth ? max_depth - kLdsDepth : 0;
    return (size_t)batch * (size_t)deep;
}

size_t advance_fill_walk_spill_entries(int batch, int max_depth) {
    const int deep = max_depth > kLdsDepth ? max_depth - kLdsDepth : 0;
    return (size_t)batch * 64 * (size_t)deep;
}

hipError_t launch_advance_fill(const DevTables &T, const DevTokenEdges &E, const int32_t *tokens, int32_t *states,
                               int32_t *data, int32_t *len, int cap, int batch, int32_t *err, uint32_t *bitmask,
                               int restart_on_eos, int32_t *adv_scratch, int32_t *walk_spill,
                               const int32_t *cycle_head, const int32_t *cycle_pool, hipStream_t stream) {
    if (batch == 0) return hipSuccess;
    const size_t row_bytes = (size_t)edge_row_stride_words(T.n_words) * sizeof(uint32_t);
    if (cycle_head) {                                  // cycle-aware stacks: the new stack is staged in LDS too
        size_t lds = row_bytes + (size_t)cap * sizeof(int32_t);
        if (cap > kCompactMaxLen || lds > kAfDynamicLdsMax) return hipErrorInvalidValue;
        const size_t tables = (size_t)(T.n_states + T.cycle_pool_n) * sizeof(int32_t);
        const int stage = cycles_fit_lds(T.n_states, T.cycle_pool_n) && lds + tables <= kAfDynamicLdsMax;
        if (stage) lds += tables;
        hipLaunchKernelGGL(advance_fill_kernel<true>, dim3(batch), dim3(kAfBlock), lds, stream, T, E, tokens, states, data,
                           len, cap, batch, err, bitmask, restart_on_eos, adv_scratch, walk_spill, (size_t)batch * 64,
                           cycle_head, cycle_pool, stage);
    } else {
        if (row_bytes > kAfDynamicLdsMax) return hipErrorInvalidValue;
        hipLaunchKernelGGL(advance_fill_kernel<false>, dim3(batch), dim3(kAfBlock), row_bytes, stream, T, E, tokens, states,
                           data, len, cap, batch, err, bitmask, restart_on_eos, adv_scratch, walk_spill, (size_t)batch * 64,
                           nullptr, nullptr, 0);
    }
    return hipGetLastError();
}

// (27 groups per lane, 207,360 tokens, is what fits the 128 vector registers of a 1,024-thread block beside the
// masking code; the greedy fold needs more registers and stops at 20 groups, 153,600 tokens)
constexpr int kStepHeldMax = 27, kStepHeldMaxGreedy = 20;
// Largest vocabulary the fused step kernel can hold in registers, and the choice of its variant.
bool advance_fill_apply_fits(int n_tokens, int n_words, int cap, bool cycles, bool greedy) {
    const size_t row_bytes = (size_t)edge_row_stride_words(n_words) * sizeof(uint32_t);
    if ((n_tokens >> 3) > (greedy ? kStepHeldMaxGreedy : kStepHeldMax) * kStepData) return false;
    if (cycles) return cap <= kCompactMaxLen && row_bytes + (size_t)cap * sizeof(int32_t) <= kAfDynamicLdsMax;
    return row_bytes <= kAfDynamicLdsMax;
}

template <bool kCompact, bool kArgmax>
static void launch_step_variant(int held, dim3 grid, size_t lds, hipStream_t stream, const DevTables &T, const DevTokenEdges &E,
                                const int32_t *tokens, int32_t *states, int32_t *data, int32_t *len, int cap, int batch,
                                int32_t *err, uint32_t *bitmask, int restart_on_eos, int32_t *adv_scratch, int32_t *walk_spill,
                                const int32_t *cycle_head, const int32_t *cycle_pool, int stage, uint16_t *logits,
                                int64_t row_stride, int32_t *out_tokens, int first_row) {
#define PRE3_STEP(H)                                                                                                        \
    hipLaunchKernelGGL((advance_fill_apply_kernel<kCompact, H, kArgmax>), grid, dim3(kStepBlock), lds, stream, T, E, tokens,  \
                       states, data, len, cap, batch, err, bitmask, restart_on_eos, adv_scratch, walk_spill,                 \
                       (size_t)batch * 64, cycle_head, cycle_pool, stage, logits, row_stride, out_tokens, first_row)
    if (held <= 9) PRE3_STEP(9);
    else if (held <= 17) PRE3_STEP(17);
    else if (held <= kStepHeldMaxGreedy || kArgmax) PRE3_STEP(20);
    else if constexpr (!kArgmax) PRE3_STEP(27);
#undef PRE3_STEP
}

// A block holds its row in the registers of a whole compute unit, so a grid of more blocks than units runs in
// rounds whose blocks start as others end, out of step with each other (62.5 us per step at 512 x 152,064).  A
// large batch goes as several launches of at most rows_per_launch rows instead, in equal shares (320 rows on
// 256 units as 160 + 160: 32.2 us against 36.7 us as 256 + 64), each launch a front of its own (47.2 us at 512).
static int step_rows_per_launch(int batch, int rows_per_launch) {
    if (rows_per_launch <= 0 || rows_per_launch >= batch) return batch;
    const int launches = (batch + rows_per_launch - 1) / rows_per_launch;
    return (batch + launches - 1) / launches;
}

hipError_t launch_advance_fill_apply(const DevTables &T, const DevTokenEdges &E, const int32_t *tokens, int32_t *states,
                                     int32_t *data, int32_t *len, int cap, int batch, int32_t *err, uint32_t *bitmask,
                                     int restart_on_eos, int32_t *adv_scratch, int32_t *walk_spill,
                                     const int32_t *cycle_head, const int32_t *cycle_pool, uint16_t *logits,
                                     int64_t row_stride, int32_t *out_tokens, int rows_per_launch, hipStream_t stream) {
    if (batch == 0) return hipSuccess;
    if (!advance_fill_apply_fits(T.n_tokens, T.n_words, cap, cycle_head != nullptr, out_tokens != nullptr)) return hipErrorInvalidValue;
    if ((reinterpret_cast<uintptr_t>(logits) & 15) != 0 || (row_stride & 7) != 0 || row_stride < T.n_tokens)
        return hipErrorInvalidValue;
    const int held = ((T.n_tokens >> 3) + kStepData - 1) / kStepData;
    const int held_variant = held <= 9 ? 9 : held <= 17 ? 17 : kStepHeldMaxGreedy;
    size_t lds = (size_t)edge_row_stride_words(T.n_words) * sizeof(uint32_t);
    int stage = 0;
    if (cycle_head) {
        lds += (size_t)cap * sizeof(int32_t);
        const size_t tables = (size_t)(T.n_states + T.cycle_pool_n) * sizeof(int32_t);
        stage = cycles_fit_lds(T.n_states, T.cycle_pool_n) && lds + tables <= kAfDynamicLdsMax;
        if (stage) lds += tables;
    }
    // the greedy fold reads a mask byte for every group slot of a lane, also those past the row's end
    if (out_tokens && lds < (size_t)held_variant * kStepData + 16) lds = (size_t)held_variant * kStepData + 16;
#define PRE3_STEP_ARGS held, dim3(rows), lds, stream, T, E, tokens, states, data, len, cap, batch, err, bitmask, restart_on_eos, \
                       adv_scratch, walk_spill, cycle_head, cycle_pool, stage, logits, row_stride, out_tokens, first
    const int share = step_rows_per_launch(batch, rows_per_launch);
    for (int first = 0; first < batch; first += share) {
        const int rows = batch - first < share ? batch - first : share;
        if (cycle_head) {
            if (out_tokens) launch_step_variant<true, true>(PRE3_STEP_ARGS);
            else launch_step_variant<true, false>(PRE3_STEP_ARGS);
        } else {
            if (out_tokens) launch_step_variant<false, true>(PRE3_STEP_ARGS);
            else launch_step_variant<false, false>(PRE3_STEP_ARGS);
        }
    }
#undef PRE3_STEP_ARGS
    return hipGetLastError();
}

hipError_t launch_fill_apply_rows(const DevTables &T, const DevTokenEdges &E, const int32_t *states, const int32_t *data,
                                  const int32_t *len, int cap, int batch, uint32_t *bitmask, int32_t *walk_spill,
                                  uint16_t *logits, int64_t row_stride, int rows_per_launch, hipStream_t stream) {
    if (batch == 0) return hipSuccess;
    if (!advance_fill_apply_fits(T.n_tokens, T.n_words, cap, false, false)) return hipErrorInvalidValue;
    if ((reinterpret_cast<uintptr_t>(logits) & 15) != 0 || (row_stride & 7) != 0 || row_stride < T.n_tokens)
        return hipErrorInvalidValue;
    const int held = ((T.n_tokens >> 3) + kStepData - 1) / kStepData;
    const size_t lds = (size_t)edge_row_stride_words(T.n_words) * sizeof(uint32_t);
    const int share = step_rows_per_launch(batch, rows_per_launch);
    // no tokens: the kernel only reads the states and the stacks
    for (int first = 0; first < batch; first += share)
        launch_step_variant<false, false>(held, dim3(batch - first < share ? batch - first : share), lds, stream, T, E, nullptr,
                                          const_cast<int32_t *>(states), const_cast<int32_t *>(data), const_cast<int32_t *>(len),
                                          cap, batch, nullptr, bitmask, 0, nullptr, walk_spill, nullptr, nullptr, 0, logits,
                                          row_stride, nullptr, first);
    return hipGetLastError();
}

bool advance_fill_fits_compact(int n_words, int cap) {
    return cap <= kCompactMaxLen &&
           (size_t)edge_row_stride_words(n_words) * sizeof(uint32_t) + (size_t)cap * sizeof(int32_t) <= kAfDynamicLdsMax;
}

bool advance_fits_compact(int cap) {
    return cap <= kCompactMaxLen && (size_t)kAdvSeqPerBlock * cap * sizeof(int32_t) + 4096 <= 65536;
}

hipError_t launch_advance(const DevTables &T, const DevTokenEdges &E, const int32_t *tokens, int32_t *states, int32_t *data,
                          int32_t *len, int cap, int batch, int32_t *err, int32_t *scratch, int restart_on_eos,
                          const int32_t *cycle_head, const int32_t *cycle_pool, hipStream_t stream) {
    if (batch == 0) return hipSuccess;
    const dim3 grid((batch + kAdvSeqPerBlock - 1) / kAdvSeqPerBlock), block(64 * kAdvSeqPerBlock);
    if (cycle_head) {                                  // cycle-aware stacks: the new stack is staged in LDS
        if (!advance_fits_compact(cap)) return hipErrorInvalidValue;
        const size_t tables = (size_t)(T.n_states + T.cycle_pool_n) * sizeof(int32_t);
        const int stage = cycles_fit_lds(T.n_states, T.cycle_pool_n) &&
                          (size_t)kAdvSeqPerBlock * cap * sizeof(int32_t) + tables + 4096 <= 65536;
        const size_t lds = (size_t)kAdvSeqPerBlock * cap * sizeof(int32_t) + (stage ? tables : 0);
        hipLaunchKernelGGL(advance_kernel<true>, grid, block, lds, stream, T, E, tokens, states, data, len, cap, batch, err,
                           scratch, restart_on_eos, cycle_head, cycle_pool, stage);
    } else {
        hipLaunchKernelGGL(advance_kernel<false>, grid, block, 0, stream, T, E, tokens, states, data, len, cap, batch, err,
                           scratch, restart_on_eos, nullptr, nullptr, 0);
    }
    return hipGetLastError();
}

bool jump_forward_fits_compact(int cap) {
    return cap <= kCompactMaxLen && (size_t)kJfSeqPerBlock * cap * sizeof(int32_t) + 20480 <= 65536;
}

hipError_t launch_jump_forward(const DevTables &T, int32_t *states, int32_t *data, int32_t *len, int cap, int batch,
                               uint8_t *out_bytes, int32_t *out_len, int max_bytes, int32_t *adv_scratch,
                               int32_t *lane_spill, const int32_t *cycle_head, const int32_t *cycle_pool,
                               hipStream_t stream) {
    if (batch == 0) return hipSuccess;
    const dim3 grid((batch + kJfSeqPerBlock - 1) / kJfSeqPerBlock), block(64 * kJfSeqPerBlock);
    if (cycle_head) {                                  // cycle-aware stacks: compacted before the kernel ends
        if (!jump_forward_fits_compact(cap)) return hipErrorInvalidValue;
        const size_t tables = (size_t)(T.n_states + T.cycle_pool_n) * sizeof(int32_t);
        const int stage = cycles_fit_lds(T.n_states, T.cycle_pool_n) &&
                          (size_t)kJfSeqPerBlock * cap * sizeof(int32_t) + tables + 20480 <= 65536;
        const size_t lds = (size_t)kJfSeqPerBlock * cap * sizeof(int32_t) + (stage ? tables : 0);
        hipLaunchKernelGGL(jump_forward_kernel<true>, grid, block, lds, stream, T, states, data, len, cap, batch, out_bytes,
                           out_len, max_bytes, adv_scratch, lane_spill, (size_t)batch * 64, cycle_head, cycle_pool, stage);
    } else {
        hipLaunchKernelGGL(jump_forward_kernel<false>, grid, block, 0, stream, T, states, data, len, cap, batch, out_bytes,
                           out_len, max_bytes, adv_scratch, lane_spill, (size_t)batch * 64, nullptr, nullptr, 0);
    }
    return hipGetLastError();
}

hipError_t launch_compact_stacks(const int32_t *cycle_head, const int32_t *cycle_pool, int pool_entries, int n_states,
                                 int32_t *data, int32_t *len, int cap, int batch, hipStream_t stream) {
    if (batch == 0) return hipSuccess;
    if (cap > kCompactMaxLen) return hipErrorInvalidValue;
    const int pool_n = pool_entries <= 1024 ? pool_entries : 0;         // small record pools are staged in LDS
    int waves = 4;                                                      // sequences per block, within 64 KB of LDS
    while (waves > 1 && (size_t)(pool_n + waves * cap) * sizeof(int32_t) > 65536) waves >>= 1;
    const size_t lds = (size_t)(pool_n + waves * cap) * sizeof(int32_t);
    hipLaunchKernelGGL(compact_stacks_kernel, dim3((batch + waves - 1) / waves), dim3(64 * waves), lds, stream, cycle_head,
                       cycle_pool, pool_n, n_states, data, len, cap, batch);
    return hipGetLastError();
}

}  // namespace pre3

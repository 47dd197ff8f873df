// C ABI of the library (declared in include/pre3.h): argument checks, table upload, launches.
#include <hip/hip_runtime_api.h>

#include <algorithm>
#include <cstring>
#include <exception>
#include <new>
#include <string>
#include <thread>
#include <vector>

#include "../../include/pre3.h"
#include "device_tables.hpp"
#include "grammar.hpp"
#include "launch.hpp"
#include "symbol_edges.hpp"
#include "tables.hpp"
#include "token_edges.hpp"

using namespace pre3;

struct pre3_handle {
    std::string error;
    bool compiled = false;
    bool host_only = false;
    int stack_cap = 1024;
    EdgeTables T;
    VocabLayout V;
    TokenEdges E;
    EffectTable X;                       // (condition node, token) -> stack effect, built from E
    SymbolEdges S;
    int max_depth = 0;

    std::vector<void *> allocations;     // device memory owned by the handle (arena chunks)
    char *arena = nullptr;               // current chunk: tables are packed into few large
    size_t arena_left = 0;               // allocations so that they share address translations
    DevTables dev{};
    int grid_blocks = 0;
    int32_t *spill = nullptr;
    DevTokenEdges dev_edges{};
    bool use_edges = false;
    int edge_blocks = 0;
    int32_t *edge_spill = nullptr;

    // binding used by pre3_advance
    int32_t *b_states = nullptr, *b_err = nullptr;
    pre3_stacks b_stacks{};
    // per-batch workspaces (pre3_bind_state): device allocations of their own, outside the arena
    struct Workspace { void *p = nullptr; size_t bytes = 0; };
    Workspace ws_adv, ws_argmax, ws_topk, ws_af_spill;
    int32_t *adv_scratch = nullptr;              // private-stack spill of the advance
    int32_t *af_walk_spill = nullptr;            // ... of per-lane walks beside an advance
    unsigned long long *argmax_best = nullptr;   // per-segment partial results of pre3_apply_mask_argmax
    unsigned long long *topk_cand = nullptr;     // per-segment candidates of pre3_apply_mask_topk
    bool topk_ready = false;
    int n_compute_units = 0;
    bool bound_empty = false;
    // stack compaction over reduction cycles (PRE3_FLAG_COMPACT_CYCLES)
    bool compact = false;
    const int32_t *cycle_head = nullptr, *cycle_pool = nullptr;
};

namespace {

int fail(pre3_handle *h, int status, const std::string &text) {
    if (h) h->error = text;
    return status;
}

int hip_fail(pre3_handle *h, hipError_t e, const char *what) {
    return fail(h, PRE3_E_HIP, std::string(what) + ": " + hipGetErrorString(e));
}

// Sub-allocates from large chunks (256-byte aligned): the many small tables of a handle end up
// next to each other instead of each in its own mapping.
hipError_t arena_alloc(pre3_handle *h, size_t bytes, void **out) {
    const size_t kChunk = (size_t)64 << 20;
    bytes = (bytes + 255) & ~(size_t)255;
    if (bytes == 0) bytes = 256;
    if (bytes > h->arena_left) {
        const size_t chunk = bytes > kChunk ? bytes : kChunk;
        void *p = nullptr;
        hipError_t e = hipMalloc(&p, chunk);
        if (e != hipSuccess) return e;
        h->allocations.push_back(p);
        if (bytes >= kChunk) { *out = p; return hipSuccess; }   // a chunk of its own; keep the current one
        h->arena = static_cast<char *>(p);
        h->arena_left = chunk;
    }
    *out = h->arena;
    h->arena += bytes;
    h->arena_left -= bytes;
    return hipSuccess;
}

// The reduction-cycle records as the kernels read them: same offsets as in EdgeTables::cycle_pool
// ([length, next record of the same head, states]), but every record's states last first, so that
// the lane that looks at the entry i below a head compares it with entry 2 + i of the record
// whatever the record's length; kCyclePoolPad entries that match no state follow the last record,
// so that all 64 lanes can load.
std::vector<int32_t> device_cycle_pool(const EdgeTables &T) {
    std::vector<int32_t> pool = T.cycle_pool;
    for (size_t at = 0; at + 2 <= pool.size(); at += 2 + (size_t)pool[at])
        std::reverse(pool.begin() + at + 2, pool.begin() + at + 2 + pool[at]);
    pool.insert(pool.end(), kCyclePoolPad, -2);
    return pool;
}

template <typename T>
hipError_t upload(pre3_handle *h, const std::vector<T> &src, const T **dst) {
    void *p = nullptr;
    size_t bytes = src.size() * sizeof(T);
    hipError_t e = arena_alloc(h, bytes + 64, &p);        // the scalar 16-word loads of the kernels may reach 60 bytes past a table
    if (e != hipSuccess) return e;
    if (bytes) {
        e = hipMemcpy(p, src.data(), bytes, hipMemcpyHostToDevice);
        if (e != hipSuccess) return e;
    }
    *dst = static_cast<const T *>(p);
    return hipSuccess;
}

hipError_t device_alloc(pre3_handle *h, size_t bytes, void **out, bool zero) {
    hipError_t e = arena_alloc(h, bytes, out);
    if (e != hipSuccess) return e;
    if (zero) e = hipMemset(*out, 0, bytes ? bytes : 16);
    return e;
}

// Makes `w` hold at least `need` bytes: kept if large enough, else freed and allocated anew, so a
// handle holds one workspace of each kind, sized for the largest batch bound so far.
hipError_t grow_workspace(pre3_handle::Workspace &w, size_t need, void **out) {
    if (need > w.bytes || !w.p) {
        if (w.p) { (void)hipFree(w.p); w.p = nullptr; w.bytes = 0; }
        const size_t bytes = need < 256 ? 256 : need;
        hipError_t e = hipMalloc(&w.p, bytes);
        if (e != hipSuccess) { w.p = nullptr; return e; }
        w.bytes = bytes;
    }
    *out = w.p;
    return hipSuccess;
}

constexpr ptrdiff_t kHotBytesMax = 2 << 20;   // half of one XCD's L2

int upload_tables(pre3_handle *h) {
    hipError_t e;
    DevTables &D = h->dev;
#define PRE3_UP(vec, field)                                               \
    if ((e = upload(h, vec, &D.field)) != hipSuccess) return hip_fail(h, e, "upload " #field)
    std::vector<int32_t> byte_info(256);
    for (int b = 0; b < 256; ++b) byte_info[b] = (int32_t)h->T.byte_class[b] | (h->T.byte_delta[b] * 256);
    // first the tables a walk of one token touches, so that they form one contiguous region
    PRE3_UP(byte_info, byte_info);
    const size_t chunks_before = h->allocations.size();
    {
        std::vector<int32_t> class_info(h->T.n_classes + 1, 0);
        for (int b = 255; b >= 0; --b) {
            int32_t &ci = class_info[h->T.byte_class[b]];
            ci = ((ci & 0xFFFF) + 1) | (b << 16);
        }
        PRE3_UP(class_info, class_info);
    }
    D.sym_nodes = nullptr; D.sym_pairs = nullptr; D.sym_cell = nullptr; D.sym_pool = nullptr; D.state_kind = nullptr;
    if (h->S.enabled) {
        std::vector<int4> sn(h->S.nodes.size());
        for (size_t i = 0; i < sn.size(); ++i)
            sn[i] = make_int4(h->S.nodes[i].known, h->S.nodes[i].child_begin, h->S.nodes[i].child_count,
                              h->S.nodes[i].first_child);
        std::vector<int2> sp(h->S.child_state.size());
        for (size_t i = 0; i < sp.size(); ++i) sp[i] = make_int2(h->S.child_state[i], h->S.child_node[i]);
        if ((e = upload(h, sn, &D.sym_nodes)) != hipSuccess) return hip_fail(h, e, "upload sym_nodes");
        if ((e = upload(h, sp, &D.sym_pairs)) != hipSuccess) return hip_fail(h, e, "upload sym_pairs");
        // edges with at most two pushes travel inside their cell: one look-up per input symbol
        if (h->S.pool.size() >= (size_t)kCellInline) return fail(h, PRE3_E_LIMIT, "reduction-edge records exceed 2^30 words");
        std::vector<int4> cells(h->S.eff.size());
        for (size_t i = 0; i < cells.size(); ++i) {
            const int32_t code = h->S.eff[i];
            int4 c = make_int4(code, 0, 0, 0);
            if (code >= 0) {
                const int32_t *r = &h->S.pool[code];
                const int32_t known = r[0], peak = r[1], np = r[2] & kEffPushMask;
                if (known < 256 && peak >= -128 && peak < 128 && np >= 1 && np <= 2)
                    c = make_int4(kCellInline | known | ((peak + 128) << 8) | (np << 16) |
                                      ((r[2] & kEffSameShape) ? kCellSameShape : 0) | ((r[2] & kEffGrow) ? kCellGrow : 0),
                                  r[3], r[4], np == 2 ? r[5] : 0);
            }
            cells[i] = c;
        }
        if ((e = upload(h, cells, &D.sym_cell)) != hipSuccess) return hip_fail(h, e, "upload sym_cell");
        if ((e = upload(h, h->S.pool, &D.sym_pool)) != hipSuccess) return hip_fail(h, e, "upload sym_pool");
        if ((e = upload(h, h->T.state_kind, &D.state_kind)) != hipSuccess) return hip_fail(h, e, "upload state_kind");
    }
    // the condition trees of the token-level edges (shared subtrees make them small) belong to the same hot region
    const bool with_token_edges = h->E.enabled && (size_t)h->V.n_words <= edge_kernel_max_lds_words();
    std::vector<DevConditionNode> nodes;
    if (with_token_edges) {
        nodes.resize(h->E.nodes.size());
        for (size_t i = 0; i < nodes.size(); ++i) {
            const ConditionNode &n = h->E.nodes[i];
            DevConditionNode d{};
            d.known = n.known;
            d.child_count = n.child_count;
            if (n.child_count > 0) {
                d.a = n.child_begin;
                d.b = h->E.child_node[n.child_begin];            // first child; the others follow it
            } else {
                d.a = n.walk_begin;
                d.b = n.walk_count;
            }
            d.dense_row = n.dense_row;
            d.delta_begin = n.delta_begin;
            d.delta_count = n.delta_count;
            nodes[i] = d;
        }
        std::vector<DevConditionNode> roots(h->E.root_of_state.size());
        for (size_t i = 0; i < roots.size(); ++i) roots[i] = nodes[h->E.root_of_state[i]];
        if ((e = upload(h, roots, &h->dev_edges.root_nodes)) != hipSuccess) return hip_fail(h, e, "upload root_nodes");
        if ((e = upload(h, h->E.child_state, &h->dev_edges.child_state)) != hipSuccess)
            return hip_fail(h, e, "upload child_state");
        if ((e = upload(h, nodes, &h->dev_edges.nodes)) != hipSuccess) return hip_fail(h, e, "upload nodes");
        if ((e = upload(h, h->E.root_of_state, &h->dev_edges.root_id)) != hipSuccess) return hip_fail(h, e, "upload root_id");
    }
    {
        const ptrdiff_t span = h->arena - reinterpret_cast<const char *>(D.byte_info);
        const bool one_chunk = h->allocations.size() == chunks_before;
        D.hot_begin = reinterpret_cast<const char *>(D.byte_info);
        D.hot_bytes = one_chunk && span > 0 ? (int32_t)std::min<ptrdiff_t>(span, kHotBytesMax) : 0;
    }
    PRE3_UP(h->T.edge, edge);
    PRE3_UP(h->T.goto_row, goto_row);
    PRE3_UP(h->T.goto_flat, goto_flat);
    PRE3_UP(h->T.run_off, run_off);
    PRE3_UP(h->T.run_pool, run_pool);
    PRE3_UP(h->V.tok_len, tok_len);
    PRE3_UP(h->V.tok_bit, tok_bit);
    PRE3_UP(h->V.tok_words, tok_words);
    PRE3_UP(h->V.bytes, vbytes);
    PRE3_UP(h->V.offsets, voffsets);
    {
        std::vector<int32_t> info((size_t)h->V.n_tokens * 32, 0);
        for (int t = 0; t < h->V.n_tokens; ++t) {
            const int lo = h->V.offsets[t], n = h->V.offsets[t + 1] - lo;
            int32_t *rec = &info[(size_t)t * 32];
            rec[0] = n <= kTokInfoBytes ? n : -1;
            for (int i = 0; i < n && i < kTokInfoBytes; ++i) rec[1 + i] = byte_info[h->V.bytes[lo + i]];
        }
        PRE3_UP(info, tok_info);
    }
#undef PRE3_UP
    D.n_states = h->T.n_states;
    D.ncol = h->T.n_classes + 1;
    D.end_col = h->T.n_classes;
    D.n_padded = h->V.n_padded;
    D.n_chunks = h->V.n_chunks;
    D.n_words = h->V.n_words;
    D.n_tokens = h->V.n_tokens;
    D.eos_id = h->V.eos_id;
    D.max_depth = h->max_depth;
    D.cycle_pool_n = h->compact ? (int)h->T.cycle_pool.size() + kCyclePoolPad : 0;

    int device = 0;
    hipDeviceProp_t prop;
    if ((e = hipGetDevice(&device)) != hipSuccess) return hip_fail(h, e, "hipGetDevice");
    if ((e = hipGetDeviceProperties(&prop, device)) != hipSuccess) return hip_fail(h, e, "hipGetDeviceProperties");
    h->n_compute_units = prop.multiProcessorCount;
    {   // the spill area of pre3_advance_static: its address on this device is looked up here, once
        int32_t *unused = nullptr;
        if ((e = static_advance_scratch(&unused)) != hipSuccess) return hip_fail(h, e, "address of the static scratch");
    }
    h->grid_blocks = walk_grid_blocks(prop.multiProcessorCount);
    void *p = nullptr;
    if ((e = device_alloc(h, walk_spill_entries(h->grid_blocks, h->max_depth) * sizeof(int32_t), &p, false)) != hipSuccess)
        return hip_fail(h, e, "allocate walk spill area");
    h->spill = static_cast<int32_t *>(p);
    if ((e = device_alloc(h, sizeof(int32_t), &p, true)) != hipSuccess) return hip_fail(h, e, "allocate fault counter");
    D.fault = static_cast<int32_t *>(p);

    // token-level edges; a vocabulary whose mask row does not fit the kernel's LDS bitmap keeps
    // the byte-by-byte path
    if (with_token_edges) {
        DevTokenEdges &X = h->dev_edges;
#define PRE3_UPE(vec, field)                                              \
    if ((e = upload(h, vec, &X.field)) != hipSuccess) return hip_fail(h, e, "upload " #field)
        const int stride = edge_row_stride_words(h->V.n_words);
        std::vector<uint32_t> dense((size_t)h->E.n_dense * stride, 0);
        for (int64_t r = 0; r < h->E.n_dense; ++r)
            std::memcpy(&dense[(size_t)r * stride], &h->E.dense_rows[(size_t)r * h->V.n_words],
                        sizeof(uint32_t) * h->V.n_words);
        PRE3_UPE(dense, dense_rows);
        PRE3_UPE(h->E.delta_ids, delta_ids);
        PRE3_UPE(h->E.walk_ids, walk_ids);
#undef PRE3_UPE
        X.fx_slots = nullptr; X.fx_pool = nullptr; X.fx_mask = 0; X.fx_min_len = 0;   // X = h->dev_edges
        if (!h->X.slots.empty()) {
            const int32_t *slots = nullptr;
            if ((e = upload(h, h->X.slots, &slots)) != hipSuccess) return hip_fail(h, e, "upload effect slots");
            std::vector<int32_t> pool = h->X.pool;
            if (pool.empty()) pool.push_back(0);
            if ((e = upload(h, pool, &X.fx_pool)) != hipSuccess) return hip_fail(h, e, "upload effect pool");
            X.fx_slots = reinterpret_cast<const int4 *>(slots);
            X.fx_mask = h->X.bucket_mask;
            X.fx_min_len = h->E.effect_min_len;
        }
        h->edge_blocks = edge_grid_blocks(prop.multiProcessorCount);
        if ((e = device_alloc(h, edge_spill_entries(h->edge_blocks, h->max_depth) * sizeof(int32_t), &p, false)) != hipSuccess)
            return hip_fail(h, e, "allocate edge-kernel spill area");
        h->edge_spill = static_cast<int32_t *>(p);
        h->use_edges = true;
    }
    if (h->compact) {
        if ((e = upload(h, h->T.cycle_head, &h->cycle_head)) != hipSuccess) return hip_fail(h, e, "upload cycle_head");
        if ((e = upload(h, device_cycle_pool(h->T), &h->cycle_pool)) != hipSuccess) return hip_fail(h, e, "upload cycle_pool");
    }
    return PRE3_OK;
}

bool usable(const pre3_handle *h) { return h && h->compiled && !h->host_only; }

// Batch sizes at which the one-kernel step is chosen unasked.  It keeps a sequence's logits in the registers of one
// compute unit while the token is walked: below a quarter of the units too much of the chip idles.  A batch larger
// than the chip goes as equal launches of at most one row per unit; against the two launches that wins where most
// of the logits have to be read anyway (JSON at 128,256 tokens: 10 % at 320 rows on 256 units, 8 % at 512, 3 % at
// 1,024, none at 2,048) and loses where the masks are sparse (a fixed schema at 512 x 152,064: 55.4 against 53.7 us),
// because the masking kernel does not read lines that are masked as a whole and this kernel fetches the row before
// it knows the mask.  The library cannot tell which it will be, so beyond the chip the caller asks for it.
bool step_kernel_batch(const pre3_handle *h, int batch) {
    return batch * 4 >= h->n_compute_units && batch <= h->n_compute_units;
}

// The token-level edges for pre3_advance: only their stack-effect records are used there.
DevTokenEdges effect_edges(const pre3_handle *h) { return h->use_edges ? h->dev_edges : DevTokenEdges{}; }

// After a call that changed the bound stacks: take complete traversals of reduction cycles out
// again (only with PRE3_FLAG_COMPACT_CYCLES and a grammar that has such cycles).
hipError_t compact_stacks(pre3_handle *h, const pre3_stacks &st, hipStream_t s) {
    if (!h->compact || h->T.n_cycles == 0) return hipSuccess;
    return launch_compact_stacks(h->cycle_head, h->cycle_pool, h->dev.cycle_pool_n, h->T.n_states,
                                 st.data, st.len, st.cap, st.batch, s);
}
hipError_t compact_bound_stacks(pre3_handle *h, hipStream_t s) { return compact_stacks(h, h->b_stacks, s); }

// (grammar, local state) of a global state id
bool locate(const pre3_handle *h, int state, int *g, int *local) {
    if (!h || !h->compiled || state < 0 || state >= h->T.n_states) return false;
    for (int i = 0; i < h->T.n_grammars; ++i)
        if (state < h->T.state_offset[i + 1]) { *g = i; *local = state - h->T.state_offset[i]; return true; }
    return false;
}

}  // namespace

extern "C" {

int pre3_compile(const char *const *grammars, int32_t n_grammars, const pre3_vocab *vocab, const pre3_options *opt,
                 pre3_handle **out) {
    if (!out) return PRE3_E_BADARG;
    *out = nullptr;
    pre3_handle *h = new (std::nothrow) pre3_handle();
    if (!h) return PRE3_E_NOMEM;
    *out = h;
    if (!grammars || n_grammars < 1 || !vocab) return fail(h, PRE3_E_BADARG, "null or empty argument");
    if (!vocab->bytes || !vocab->offsets || vocab->n_tokens < 1 || vocab->eos_id < 0 ||
        vocab->eos_id >= vocab->n_tokens)
        return fail(h, PRE3_E_BADARG, "bad vocabulary");
    int max_token_len = opt && opt->max_token_len ? opt->max_token_len : 64;
    h->stack_cap = opt && opt->stack_cap ? opt->stack_cap : 1024;
    h->host_only = opt && (opt->flags & PRE3_FLAG_HOST_ONLY);
    h->compact = opt && (opt->flags & PRE3_FLAG_COMPACT_CYCLES);
    if (opt && (opt->flags & ~(PRE3_FLAG_HOST_ONLY | PRE3_FLAG_NO_TOKEN_EDGES | PRE3_FLAG_STEPWISE_REDUCTIONS |
                               PRE3_FLAG_COMPACT_CYCLES | PRE3_FLAG_NO_TOKEN_EFFECTS)))
        return fail(h, PRE3_E_BADARG, "unknown flag in options");
    if (h->compact && h->stack_cap > kCompactMaxLen)
        return fail(h, PRE3_E_BADARG, "stack compaction handles stacks of at most " + std::to_string(kCompactMaxLen) +
                                          " entries: lower stack_cap");
    if (max_token_len < 1 || max_token_len > 254 || h->stack_cap < 1)
        return fail(h, PRE3_E_BADARG, "max_token_len must be in 1..254 and stack_cap positive");
    try {
        std::vector<Grammar> gs;
        for (int i = 0; i < n_grammars; ++i) {
            if (!grammars[i]) return fail(h, PRE3_E_BADARG, "null grammar text");
            try {
                gs.push_back(parse_grammar(grammars[i]));
            } catch (CompileError &e) {
                if (n_grammars > 1) e.text = "grammar " + std::to_string(i) + ": " + e.text;
                throw;
            }
        }
        h->T = build_edge_tables(gs);
        h->V = build_vocab_layout(vocab->bytes, vocab->offsets, vocab->n_tokens, vocab->eos_id, max_token_len);
        // every input symbol adds at most height_per_byte - 1 private entries (see tables.cpp)
        h->max_depth = std::max(1, h->V.max_len) * (h->T.height_per_byte - 1) + 1;
        if (!(opt && (opt->flags & PRE3_FLAG_STEPWISE_REDUCTIONS))) h->S = build_symbol_edges(h->T);
        // token-level edges serve the kernels that keep a whole mask row in LDS: a vocabulary
        // beyond that size keeps the byte-by-byte path and needs no such tables
        if (!(opt && (opt->flags & PRE3_FLAG_NO_TOKEN_EDGES)) && (size_t)h->V.n_words <= edge_kernel_max_lds_words()) {
            TokenEdgeLimits lim;
            if (opt && opt->max_condition_depth > 0) lim.max_known = opt->max_condition_depth;
            if (opt && opt->row_threshold > 0) lim.max_path_ids = opt->row_threshold;
            lim.compacted_stacks = h->compact;
            lim.n_threads = (int)std::max(1u, std::min(16u, std::thread::hardware_concurrency()));
            if (opt && opt->effect_min_len > 0) lim.effect_min_len = opt->effect_min_len;
            if (opt && (opt->flags & PRE3_FLAG_NO_TOKEN_EFFECTS)) lim.effect_min_len = 0;
            h->E = build_token_edges(h->T, h->V, lim);
            h->X = build_effect_table(h->E);
        }
    } catch (const CompileError &e) {
        return fail(h, e.status, e.text);
    } catch (const std::bad_alloc &) {
        return fail(h, PRE3_E_NOMEM, "out of host memory");
    } catch (const std::exception &e) {            // nothing may cross the C boundary
        return fail(h, PRE3_E_LIMIT, std::string("internal error: ") + e.what());
    } catch (...) {
        return fail(h, PRE3_E_LIMIT, "internal error");
    }
    h->compiled = true;
    if (!h->host_only) {
        int rc = upload_tables(h);
        if (rc != PRE3_OK) { h->compiled = false; return rc; }
    }
    return PRE3_OK;
}

int pre3_free(pre3_handle *h) {
    if (!h) return PRE3_OK;
    for (void *p : h->allocations) (void)hipFree(p);
    for (pre3_handle::Workspace *w : {&h->ws_adv, &h->ws_argmax, &h->ws_topk, &h->ws_af_spill})
        if (w->p) (void)hipFree(w->p);
    delete h;
    return PRE3_OK;
}

const char *pre3_last_error(const pre3_handle *h) { return h ? h->error.c_str() : "null handle"; }

int32_t pre3_initial_state(const pre3_handle *h, int32_t g) {
    if (!h || !h->compiled || g < 0 || g >= h->T.n_grammars) return PRE3_E_BADARG;
    return h->T.state_offset[g];
}

int pre3_bind_state(pre3_handle *h, int32_t *states, pre3_stacks stacks, int32_t *err) {
    if (!usable(h)) return PRE3_E_BADARG;
    if (stacks.batch == 0) {                 // an empty batch has no buffers to point at
        h->b_states = nullptr; h->b_err = nullptr; h->b_stacks = stacks; h->bound_empty = true;
        return PRE3_OK;
    }
    h->bound_empty = false;
    if (!states || !err || !stacks.data || !stacks.len || stacks.batch < 0 || stacks.cap < 1 ||
        stacks.cap > h->stack_cap)
        return fail(h, PRE3_E_BADARG, "bind_state: null buffer, negative batch or cap outside 1..stack_cap");
    // per-batch workspaces: each is an allocation of its own that grows with the largest batch bound
    // so far; a superseded one is freed (hipFree waits until the device no longer uses it)
    hipError_t e;
    void *p = nullptr;
    if ((e = grow_workspace(h->ws_adv, advance_scratch_entries(stacks.batch, h->max_depth) * sizeof(int32_t), &p)) != hipSuccess)
        return hip_fail(h, e, "allocate advance scratch");
    h->adv_scratch = static_cast<int32_t *>(p);
    if ((e = grow_workspace(h->ws_argmax, masked_argmax_workspace_bytes(stacks.batch, h->V.n_tokens, h->n_compute_units), &p)) != hipSuccess)
        return hip_fail(h, e, "allocate argmax workspace");
    h->argmax_best = static_cast<unsigned long long *>(p);
    // the top-k candidates: batch x segments x 64 words; a batch so large that this passes 1 GiB goes
    // without (pre3_apply_mask_topk then reports PRE3_E_LIMIT)
    const size_t need_topk = masked_topk_workspace_bytes(stacks.batch, h->V.n_tokens);
    h->topk_ready = need_topk <= ((size_t)1 << 30);
    if (h->topk_ready) {
        if ((e = grow_workspace(h->ws_topk, need_topk, &p)) != hipSuccess) return hip_fail(h, e, "allocate top-k workspace");
        h->topk_cand = static_cast<unsigned long long *>(p);
    }
    // private stacks of per-lane walks beside an advance (leftover tokens, jump-forward trials)
    if ((e = grow_workspace(h->ws_af_spill, advance_fill_walk_spill_entries(stacks.batch, h->max_depth) * sizeof(int32_t), &p)) != hipSuccess)
        return hip_fail(h, e, "allocate advance+fill spill area");
    h->af_walk_spill = static_cast<int32_t *>(p);
    h->b_states = states;
    h->b_stacks = stacks;
    h->b_err = err;
    return PRE3_OK;
}

int pre3_fill_mask(pre3_handle *h, const int32_t *states, pre3_stacks stacks, uint32_t *bitmask, pre3_stream stream) {
    if (!usable(h)) return PRE3_E_BADARG;
    if (stacks.batch == 0) return PRE3_OK;
    if (!states || !stacks.data || !stacks.len || !bitmask || stacks.batch < 0 || stacks.cap < 1 ||
        stacks.cap > h->stack_cap)
        return fail(h, PRE3_E_BADARG, "fill_mask: null buffer, negative batch or cap outside 1..stack_cap");
    hipError_t e =
        h->use_edges
            ? launch_fill_mask_edges(h->dev, h->dev_edges, states, stacks.data, stacks.len, stacks.cap, stacks.batch,
                                     bitmask, nullptr, 0, h->edge_spill, h->edge_blocks,
                                     static_cast<hipStream_t>(stream))
            : launch_fill_mask_walk(h->dev, states, stacks.data, stacks.len, stacks.cap, stacks.batch, bitmask,
                                    h->spill, h->grid_blocks, static_cast<hipStream_t>(stream));
    return e == hipSuccess ? PRE3_OK : hip_fail(h, e, "launch fill_mask");
}

int pre3_fill_apply_mask(pre3_handle *h, const int32_t *states, pre3_stacks stacks, uint32_t *bitmask,
                         uint16_t *logits, int64_t row_stride, pre3_stream stream) {
    if (!usable(h)) return PRE3_E_BADARG;
    if (stacks.batch == 0) return PRE3_OK;
    if (!states || !stacks.data || !stacks.len || !bitmask || !logits || stacks.batch < 0 || stacks.cap < 1 ||
        stacks.cap > h->stack_cap || row_stride < h->V.n_tokens)
        return fail(h, PRE3_E_BADARG, "fill_apply_mask: null buffer, negative batch, bad cap or row_stride < vocabulary");
    if (reinterpret_cast<uintptr_t>(logits) % 2 != 0) return fail(h, PRE3_E_BADARG, "fill_apply_mask: misaligned logits");
    hipStream_t s = static_cast<hipStream_t>(stream);
    const bool fused = h->use_edges && reinterpret_cast<uintptr_t>(logits) % 16 == 0 && row_stride % 8 == 0;
    // A batch that suits the one-launch step kernel (a row of logits per compute unit, fetched while the mask is
    // looked up) runs through it, without the advance; its walks spill into the workspace of the bound batch.
    if (fused && h->af_walk_spill && stacks.batch <= h->b_stacks.batch && step_kernel_batch(h, stacks.batch) &&
        advance_fill_apply_fits(h->V.n_tokens, h->V.n_words, stacks.cap, false, false)) {
        hipError_t e = launch_fill_apply_rows(h->dev, h->dev_edges, states, stacks.data, stacks.len, stacks.cap, stacks.batch,
                                              bitmask, h->af_walk_spill, logits, row_stride, h->n_compute_units, s);
        return e == hipSuccess ? PRE3_OK : hip_fail(h, e, "launch fill_apply_mask");
    }
    // The kernel that masks each row segment as it leaves LDS saves a launch and the read of the mask, which decides
    // below one sequence per compute unit; beyond, its few hundred blocks stream the logits more slowly than the flat
    // grid of the masking kernel (66.3 against 49.4 us at 512 x 128,256, 78.6 against 51.9 us at 512 x 152,064).
    if (fused && stacks.batch <= h->n_compute_units) {
        hipError_t e = launch_fill_mask_edges(h->dev, h->dev_edges, states, stacks.data, stacks.len, stacks.cap,
                                              stacks.batch, bitmask, logits, row_stride, h->edge_spill, h->edge_blocks, s);
        return e == hipSuccess ? PRE3_OK : hip_fail(h, e, "launch fill_apply_mask");
    }
    int rc = pre3_fill_mask(h, states, stacks, bitmask, stream);
    if (rc != PRE3_OK) return rc;
    return pre3_apply_mask(logits, bitmask, stacks.batch, h->V.n_tokens, row_stride, stream);
}

int pre3_apply_mask(uint16_t *logits, const uint32_t *bitmask, int32_t batch, int32_t vocab, int64_t row_stride,
                    pre3_stream stream) {
    if (batch == 0 || vocab == 0) return PRE3_OK;
    if (!logits || !bitmask || batch < 0 || vocab < 0 || row_stride < vocab) return PRE3_E_BADARG;
    if (reinterpret_cast<uintptr_t>(logits) % 2 != 0 || reinterpret_cast<uintptr_t>(bitmask) % 4 != 0)
        return PRE3_E_BADARG;
    hipError_t e = launch_apply_mask(logits, bitmask, batch, vocab, row_stride, static_cast<hipStream_t>(stream));
    return e == hipSuccess ? PRE3_OK : PRE3_E_HIP;
}

int pre3_advance(pre3_handle *h, const int32_t *tokens, pre3_stream stream) {
    if (!usable(h)) return PRE3_E_BADARG;
    if (h->bound_empty) return PRE3_OK;
    if (!h->b_states) return fail(h, PRE3_E_BADARG, "advance: no state bound");
    if (!tokens) return fail(h, PRE3_E_BADARG, "advance: null tokens");
    // cycle-aware stacks: compacted inside the kernel when four staged stacks fit its LDS, else by a kernel of its own
    const bool fused = h->compact && h->T.n_cycles > 0 && advance_fits_compact(h->b_stacks.cap);
    hipError_t e = launch_advance(h->dev, effect_edges(h), tokens, h->b_states, h->b_stacks.data, h->b_stacks.len, h->b_stacks.cap,
                                  h->b_stacks.batch, h->b_err, h->adv_scratch, 0, fused ? h->cycle_head : nullptr,
                                  fused ? h->cycle_pool : nullptr, static_cast<hipStream_t>(stream));
    if (e == hipSuccess && !fused) e = compact_bound_stacks(h, static_cast<hipStream_t>(stream));
    return e == hipSuccess ? PRE3_OK : hip_fail(h, e, "launch advance");
}

int pre3_advance_static(pre3_handle *h, const int32_t *tokens, int32_t *states, pre3_stacks stacks, int32_t *err,
                        pre3_stream stream) {
    if (!usable(h)) return PRE3_E_BADARG;
    if (stacks.batch == 0) return PRE3_OK;
    if (!tokens || !states || !err || !stacks.data || !stacks.len || stacks.batch < 0 || stacks.cap < 1 ||
        stacks.cap > h->stack_cap)
        return fail(h, PRE3_E_BADARG, "advance_static: null buffer, negative batch or cap outside 1..stack_cap");
    const size_t need = advance_scratch_entries(stacks.batch, h->max_depth);
    if (need > kStaticScratchEntries)
        return fail(h, PRE3_E_LIMIT, "advance_static: batch " + std::to_string(stacks.batch) + " x " +
                                         std::to_string(need / (size_t)stacks.batch) + " spill entries per sequence exceeds the static scratch of " +
                                         std::to_string(kStaticScratchEntries) + " entries: use pre3_bind_state + pre3_advance");
    int32_t *scratch = nullptr;
    hipError_t e = static_advance_scratch(&scratch);
    if (e != hipSuccess) return hip_fail(h, e, "advance_static: address of the static scratch");
    hipStream_t s = static_cast<hipStream_t>(stream);
    const bool fused = h->compact && h->T.n_cycles > 0 && advance_fits_compact(stacks.cap);
    e = launch_advance(h->dev, effect_edges(h), tokens, states, stacks.data, stacks.len, stacks.cap, stacks.batch, err, scratch, 0,
                       fused ? h->cycle_head : nullptr, fused ? h->cycle_pool : nullptr, s);
    if (e == hipSuccess && !fused) e = compact_stacks(h, stacks, s);
    return e == hipSuccess ? PRE3_OK : hip_fail(h, e, "launch advance_static");
}

int pre3_advance_fill_mask(pre3_handle *h, const int32_t *tokens, uint32_t *bitmask, int32_t flags,
                           pre3_stream stream) {
    if (!usable(h)) return PRE3_E_BADARG;
    if (h->bound_empty) return PRE3_OK;
    if (!h->b_states) return fail(h, PRE3_E_BADARG, "advance_fill_mask: no state bound");
    if (!tokens || !bitmask) return fail(h, PRE3_E_BADARG, "advance_fill_mask: null tokens or bitmask");
    if (flags & ~PRE3_ADVANCE_RESTART_ON_EOS) return fail(h, PRE3_E_BADARG, "advance_fill_mask: unknown flag");
    const int restart = (flags & PRE3_ADVANCE_RESTART_ON_EOS) ? 1 : 0;
    hipStream_t s = static_cast<hipStream_t>(stream);
    hipError_t e;
    // With cycle-aware stacks the kernel compacts the new stack before it looks the mask up (the
    // condition trees are built for compacted stacks); if the stack does not fit the kernel's LDS
    // next to the mask row, the call takes the three launches below.
    const bool cycles = h->compact && h->T.n_cycles > 0;
    if (h->use_edges && (!cycles || advance_fill_fits_compact(h->V.n_words, h->b_stacks.cap))) {
        e = launch_advance_fill(h->dev, h->dev_edges, tokens, h->b_states, h->b_stacks.data, h->b_stacks.len,
                                h->b_stacks.cap, h->b_stacks.batch, h->b_err, bitmask, restart, h->adv_scratch,
                                h->af_walk_spill, cycles ? h->cycle_head : nullptr, cycles ? h->cycle_pool : nullptr, s);
        return e == hipSuccess ? PRE3_OK : hip_fail(h, e, "launch advance_fill_mask");
    }
    e = launch_advance(h->dev, effect_edges(h), tokens, h->b_states, h->b_stacks.data, h->b_stacks.len, h->b_stacks.cap,
                       h->b_stacks.batch, h->b_err, h->adv_scratch, restart, nullptr, nullptr, s);
    if (e == hipSuccess) e = compact_bound_stacks(h, s);
    if (e != hipSuccess) return hip_fail(h, e, "launch advance");
    return pre3_fill_mask(h, h->b_states, h->b_stacks, bitmask, stream);
}

namespace {
// Whether the step call takes its one-kernel form: asked for or a suitable batch size, and the kernel's conditions.
bool step_takes_one_kernel(const pre3_handle *h, const uint16_t *logits_bf16, int64_t row_stride, int32_t flags, bool greedy) {
    const int batch = h->b_stacks.batch;
    const bool cycles = h->compact && h->T.n_cycles > 0;
    const bool wanted = (flags & PRE3_STEP_ONE_KERNEL) || step_kernel_batch(h, batch);
    return wanted && h->use_edges && reinterpret_cast<uintptr_t>(logits_bf16) % 16 == 0 && row_stride % 8 == 0 &&
           row_stride >= h->V.n_tokens && advance_fill_apply_fits(h->V.n_tokens, h->V.n_words, h->b_stacks.cap, cycles, greedy);
}
}  // namespace

int32_t pre3_step_is_one_kernel(const pre3_handle *h, const uint16_t *logits_bf16, int64_t row_stride, int32_t flags) {
    if (!usable(h) || (!h->b_states && !h->bound_empty)) return PRE3_E_BADARG;
    if (h->bound_empty || !step_takes_one_kernel(h, logits_bf16, row_stride, flags, false)) return 0;
    // launches of equal shares, counted as the launcher deals them out
    const int batch = h->b_stacks.batch, most = (batch + h->n_compute_units - 1) / h->n_compute_units;
    const int share = (batch + most - 1) / most;
    return (batch + share - 1) / share;
}

int pre3_advance_fill_apply_mask(pre3_handle *h, const int32_t *tokens, uint32_t *bitmask, uint16_t *logits_bf16,
                                 int64_t row_stride, int32_t flags, pre3_stream stream) {
    if (!usable(h)) return PRE3_E_BADARG;
    if (h->bound_empty) return PRE3_OK;
    if (!h->b_states) return fail(h, PRE3_E_BADARG, "advance_fill_apply_mask: no state bound");
    if (!tokens || !bitmask || !logits_bf16) return fail(h, PRE3_E_BADARG, "advance_fill_apply_mask: null pointer");
    if (flags & ~(PRE3_ADVANCE_RESTART_ON_EOS | PRE3_STEP_ONE_KERNEL)) return fail(h, PRE3_E_BADARG, "advance_fill_apply_mask: unknown flag");
    if (row_stride < h->V.n_tokens) return fail(h, PRE3_E_BADARG, "advance_fill_apply_mask: row stride below vocabulary size");
    if (reinterpret_cast<uintptr_t>(logits_bf16) % 2 != 0) return fail(h, PRE3_E_BADARG, "advance_fill_apply_mask: misaligned logits");
    const bool cycles = h->compact && h->T.n_cycles > 0;
    if (step_takes_one_kernel(h, logits_bf16, row_stride, flags, false)) {
        const int restart = (flags & PRE3_ADVANCE_RESTART_ON_EOS) ? 1 : 0;
        hipError_t e = launch_advance_fill_apply(h->dev, h->dev_edges, tokens, h->b_states, h->b_stacks.data, h->b_stacks.len,
                                                 h->b_stacks.cap, h->b_stacks.batch, h->b_err, bitmask, restart, h->adv_scratch,
                                                 h->af_walk_spill, cycles ? h->cycle_head : nullptr,
                                                 cycles ? h->cycle_pool : nullptr, logits_bf16, row_stride, nullptr,
                                                 h->n_compute_units, static_cast<hipStream_t>(stream));
        return e == hipSuccess ? PRE3_OK : hip_fail(h, e, "launch advance_fill_apply_mask");
    }
    const int rc = pre3_advance_fill_mask(h, tokens, bitmask, flags & PRE3_ADVANCE_RESTART_ON_EOS, stream);
    if (rc != PRE3_OK) return rc;
    hipError_t e = launch_apply_mask(logits_bf16, bitmask, h->b_stacks.batch, h->V.n_tokens, row_stride,
                                     static_cast<hipStream_t>(stream));
    return e == hipSuccess ? PRE3_OK : hip_fail(h, e, "launch apply_mask");
}

int pre3_advance_fill_argmax(pre3_handle *h, const int32_t *tokens, uint32_t *bitmask, const uint16_t *logits_bf16,
                             int64_t row_stride, int32_t *out_tokens, int32_t flags, pre3_stream stream) {
    if (!usable(h)) return PRE3_E_BADARG;
    if (h->bound_empty) return PRE3_OK;
    if (!h->b_states) return fail(h, PRE3_E_BADARG, "advance_fill_argmax: no state bound");
    if (!tokens || !bitmask || !logits_bf16 || !out_tokens) return fail(h, PRE3_E_BADARG, "advance_fill_argmax: null pointer");
    if (flags & ~(PRE3_ADVANCE_RESTART_ON_EOS | PRE3_STEP_ONE_KERNEL)) return fail(h, PRE3_E_BADARG, "advance_fill_argmax: unknown flag");
    if (row_stride < h->V.n_tokens) return fail(h, PRE3_E_BADARG, "advance_fill_argmax: row stride below vocabulary size");
    if (reinterpret_cast<uintptr_t>(logits_bf16) % 2 != 0) return fail(h, PRE3_E_BADARG, "advance_fill_argmax: misaligned logits");
    if (step_takes_one_kernel(h, logits_bf16, row_stride, flags, true)) {
        const bool cycles = h->compact && h->T.n_cycles > 0;
        const int restart = (flags & PRE3_ADVANCE_RESTART_ON_EOS) ? 1 : 0;
        // the kernel only reads the logits in this form
        hipError_t e = launch_advance_fill_apply(h->dev, h->dev_edges, tokens, h->b_states, h->b_stacks.data, h->b_stacks.len,
                                                 h->b_stacks.cap, h->b_stacks.batch, h->b_err, bitmask, restart, h->adv_scratch,
                                                 h->af_walk_spill, cycles ? h->cycle_head : nullptr,
                                                 cycles ? h->cycle_pool : nullptr, const_cast<uint16_t *>(logits_bf16), row_stride,
                                                 out_tokens, h->n_compute_units, static_cast<hipStream_t>(stream));
        return e == hipSuccess ? PRE3_OK : hip_fail(h, e, "launch advance_fill_argmax");
    }
    const int rc = pre3_advance_fill_mask(h, tokens, bitmask, flags & PRE3_ADVANCE_RESTART_ON_EOS, stream);
    if (rc != PRE3_OK) return rc;
    return pre3_apply_mask_argmax(h, logits_bf16, row_stride, bitmask, out_tokens, stream);
}

int pre3_apply_mask_argmax(pre3_handle *h, const uint16_t *logits_bf16, int64_t row_stride, const uint32_t *bitmask,
                           int32_t *out_tokens, pre3_stream stream) {
    if (!usable(h)) return PRE3_E_BADARG;
    if (h->bound_empty) return PRE3_OK;
    if (!h->b_states) return fail(h, PRE3_E_BADARG, "apply_mask_argmax: no state bound");
    if (!logits_bf16 || !bitmask || !out_tokens) return fail(h, PRE3_E_BADARG, "apply_mask_argmax: null pointer");
    if (row_stride < h->V.n_tokens) return fail(h, PRE3_E_BADARG, "apply_mask_argmax: row stride below vocabulary size");
    hipError_t e = launch_masked_argmax(logits_bf16, bitmask, h->b_stacks.batch, h->V.n_tokens, row_stride,
                                        h->n_compute_units, h->argmax_best, out_tokens,
                                        static_cast<hipStream_t>(stream));
    return e == hipSuccess ? PRE3_OK : hip_fail(h, e, "launch apply_mask_argmax");
}

int pre3_apply_mask_topk(pre3_handle *h, const uint16_t *logits_bf16, int64_t row_stride, const uint32_t *bitmask,
                         int32_t k, int32_t *out_tokens, uint16_t *out_logits, pre3_stream stream) {
    if (!usable(h)) return PRE3_E_BADARG;
    if (h->bound_empty) return PRE3_OK;
    if (!h->b_states) return fail(h, PRE3_E_BADARG, "apply_mask_topk: no state bound");
    if (!logits_bf16 || !bitmask || !out_tokens) return fail(h, PRE3_E_BADARG, "apply_mask_topk: null pointer");
    if (row_stride < h->V.n_tokens) return fail(h, PRE3_E_BADARG, "apply_mask_topk: row stride below vocabulary size");
    if (k < 1 || k > PRE3_TOPK_MAX) return fail(h, PRE3_E_BADARG, "apply_mask_topk: k outside 1..PRE3_TOPK_MAX");
    if (!h->topk_ready) return fail(h, PRE3_E_LIMIT, "apply_mask_topk: batch x vocabulary too large for the candidate workspace (1 GiB)");
    if (!masked_topk_fits(h->V.n_tokens, k))
        return fail(h, PRE3_E_LIMIT, "apply_mask_topk: ceil(n_tokens / 16384) * k must not exceed 1024");
    hipError_t e = launch_masked_topk(logits_bf16, bitmask, h->b_stacks.batch, h->V.n_tokens, row_stride, k, h->n_compute_units,
                                      h->topk_cand, out_tokens, out_logits, static_cast<hipStream_t>(stream));
    return e == hipSuccess ? PRE3_OK : hip_fail(h, e, "launch apply_mask_topk");
}

int pre3_jump_forward(pre3_handle *h, uint8_t *out_bytes, int32_t *out_len, int32_t max_bytes, pre3_stream stream) {
    if (!usable(h)) return PRE3_E_BADARG;
    if (h->bound_empty) return PRE3_OK;
    if (!h->b_states) return fail(h, PRE3_E_BADARG, "jump_forward: no state bound");
    if (!out_len || max_bytes < 0 || (max_bytes > 0 && !out_bytes))
        return fail(h, PRE3_E_BADARG, "jump_forward: null pointer or negative max_bytes");
    const bool fused = h->compact && h->T.n_cycles > 0 && jump_forward_fits_compact(h->b_stacks.cap);
    hipError_t e = launch_jump_forward(h->dev, h->b_states, h->b_stacks.data, h->b_stacks.len, h->b_stacks.cap,
                                       h->b_stacks.batch, out_bytes, out_len, max_bytes, h->adv_scratch,
                                       h->af_walk_spill, fused ? h->cycle_head : nullptr, fused ? h->cycle_pool : nullptr,
                                       static_cast<hipStream_t>(stream));
    if (e == hipSuccess && !fused) e = compact_bound_stacks(h, static_cast<hipStream_t>(stream));
    return e == hipSuccess ? PRE3_OK : hip_fail(h, e, "launch jump_forward");
}

int32_t pre3_n_grammars(const pre3_handle *h) { return h && h->compiled ? h->T.n_grammars : PRE3_E_BADARG; }
int32_t pre3_n_states(const pre3_handle *h) { return h && h->compiled ? h->T.n_states : PRE3_E_BADARG; }
int32_t pre3_n_byte_classes(const pre3_handle *h) { return h && h->compiled ? h->T.n_classes : PRE3_E_BADARG; }
int32_t pre3_byte_class(const pre3_handle *h, int32_t byte) {
    if (!h || !h->compiled || byte < 0 || byte > 255) return PRE3_E_BADARG;
    return h->T.byte_class[byte];
}

int32_t pre3_edge(const pre3_handle *h, int32_t state, int32_t symbol, int32_t *arg0, int32_t *arg1) {
    int g, local;
    if (!locate(h, state, &g, &local) || symbol < 0 || symbol > 256 || !arg0 || !arg1) return PRE3_E_BADARG;
    int col = symbol == 256 ? h->T.n_classes : h->T.byte_class[symbol];
    uint32_t e = h->T.edge[(size_t)state * (h->T.n_classes + 1) + col];
    *arg0 = *arg1 = 0;
    switch (e & kKindMask) {
        case kShift: *arg0 = (int32_t)(e >> 2) + (symbol < 256 ? h->T.byte_delta[symbol] : 0); return 1;
        case kReduce: *arg0 = (int32_t)((e >> 2) & kMaxPop); *arg1 = (int32_t)(e >> kNtShift); return 2;
        case kAccept: return 3;
        default: return 0;
    }
}

int32_t pre3_goto_target(const pre3_handle *h, int32_t state, int32_t nt) {
    int g, local;
    if (!locate(h, state, &g, &local) || nt < 0 || nt >= h->T.automata[g].n_nt) return PRE3_E_BADARG;
    int row = h->T.goto_row[state];
    return row < 0 ? -1 : h->T.goto_flat[row + nt];
}

int32_t pre3_forced_run(const pre3_handle *h, int32_t state, uint8_t *out_bytes, int32_t *out_states, int32_t out_cap) {
    if (!h || !h->compiled || state < 0 || state >= h->T.n_states || !out_bytes || !out_states) return PRE3_E_BADARG;
    const int at = h->T.run_off[state];
    if (at < 0) return 0;
    const int n = h->T.run_pool[at];
    if (n > out_cap) return PRE3_E_BADARG;
    for (int i = 0; i < n; ++i) {
        out_bytes[i] = (uint8_t)(h->T.run_pool[at + 1 + i] & 0xFF);
        out_states[i] = h->T.run_pool[at + 1 + i] >> 8;
    }
    return n;
}

int32_t pre3_n_reduction_cycles(const pre3_handle *h) { return h && h->compiled ? h->T.n_cycles : PRE3_E_BADARG; }

int32_t pre3_reduction_cycle(const pre3_handle *h, int32_t index, int32_t *out_states, int32_t out_cap) {
    if (!h || !h->compiled || index < 0 || index >= h->T.n_cycles || !out_states) return PRE3_E_BADARG;
    int i = 0;                                  // records in head order, each chain shortest first
    for (int head = 0; head < h->T.n_states; ++head)
        for (int at = h->T.cycle_head[head]; at >= 0; at = h->T.cycle_pool[at + 1], ++i)
            if (i == index) {
                const int n = h->T.cycle_pool[at];
                if (n > out_cap) return PRE3_E_BADARG;
                for (int k = 0; k < n; ++k) out_states[k] = h->T.cycle_pool[at + 2 + k];
                return n;
            }
    return PRE3_E_BADARG;
}

int32_t pre3_debug_compact(const pre3_handle *h, int32_t *stack, int32_t len) {
    if (!h || !h->compiled || !stack || len < 1) return PRE3_E_BADARG;
    int w = 0;
    for (int r = 0; r < len; ++r) {
        const int x = stack[r];
        stack[w++] = x;
        if (x < 0 || x >= h->T.n_states) continue;
        for (int at = h->T.cycle_head[x]; at >= 0;) {
            const int n = h->T.cycle_pool[at];
            bool match = w - 1 - n >= 0;
            for (int k = 0; match && k < n; ++k) match = stack[w - 1 - n + k] == h->T.cycle_pool[at + 2 + k];
            if (match) { w -= n; at = h->T.cycle_head[x]; }
            else at = h->T.cycle_pool[at + 1];
        }
    }
    return w;
}

int32_t pre3_walk_depth_bound(const pre3_handle *h) { return h && h->compiled ? h->max_depth : PRE3_E_BADARG; }

int pre3_debug_timestamp(int64_t *out, pre3_stream stream) {
    if (!out) return PRE3_E_BADARG;
    return launch_timestamp(out, static_cast<hipStream_t>(stream)) == hipSuccess ? PRE3_OK : PRE3_E_HIP;
}

int pre3_debug_fault_count(pre3_handle *h, int64_t *out) {
    if (!usable(h) || !out) return PRE3_E_BADARG;
    int32_t n = 0;
    hipError_t e = hipMemcpy(&n, h->dev.fault, sizeof(n), hipMemcpyDeviceToHost);
    if (e != hipSuccess) return hip_fail(h, e, "read fault counter");
    *out = n;
    return PRE3_OK;
}

int pre3_token_edge_stats(const pre3_handle *h, int64_t out[8]) {
    if (!h || !h->compiled || !out) return PRE3_E_BADARG;
    const TokenEdges &E = h->E;
    out[0] = E.enabled;
    out[1] = E.n_roots;
    out[2] = (int64_t)E.nodes.size();
    out[3] = E.n_dense;
    out[4] = (int64_t)E.delta_ids.size();
    out[5] = (int64_t)E.walk_ids.size();
    out[6] = E.max_known;
    out[7] = (int64_t)(E.dense_rows.size() * 4 + (E.delta_ids.size() + E.walk_ids.size() + E.child_state.size() * 2 +
                                                   E.root_of_state.size()) * 4 + E.nodes.size() * sizeof(ConditionNode));
    return PRE3_OK;
}

int pre3_token_effect_stats(const pre3_handle *h, int64_t out[4]) {
    if (!h || !h->compiled || !out) return PRE3_E_BADARG;
    out[0] = h->E.n_effect_records;
    out[1] = h->X.stored;
    out[2] = h->X.dropped;
    out[3] = (int64_t)((h->X.slots.size() + h->X.pool.size()) * sizeof(int32_t));
    return PRE3_OK;
}

int32_t pre3_debug_token_effect(const pre3_handle *h, const int32_t *stack, int32_t len, int32_t token, int32_t *out,
                                int32_t out_cap, int32_t *info) {
    if (!h || !h->compiled || !stack || len < 1 || !out || token < 0 || token >= h->V.n_tokens) return PRE3_E_BADARG;
    int k = 0, peak = 0;
    std::vector<int32_t> pushes;
    if (h->E.effect_min_len <= 0 || h->V.offsets[token + 1] - h->V.offsets[token] < h->E.effect_min_len) return 0;
    if (!find_effect(h->E, h->X, stack, len, token, &k, &peak, &pushes) || k > len) return 0;
    const int new_len = len - k + 1 + (int)pushes.size();
    if (new_len > out_cap) return PRE3_E_BADARG;
    std::copy(stack, stack + (len - k + 1), out);
    std::copy(pushes.begin(), pushes.end(), out + (len - k + 1));
    if (info) { info[0] = k; info[1] = peak; info[2] = (int32_t)pushes.size(); }
    return new_len;
}

int pre3_symbol_edge_stats(const pre3_handle *h, int64_t out[4]) {
    if (!h || !h->compiled || !out) return PRE3_E_BADARG;
    out[0] = h->S.enabled;
    out[1] = (int64_t)h->S.nodes.size();
    out[2] = h->S.max_known;
    // device form: 16-byte node records, 16-byte cells, records pool, (condition state, child) pairs
    out[3] = (int64_t)(h->S.nodes.size() * 16 + h->S.eff.size() * 16 + h->S.pool.size() * 4 +
                       h->S.child_state.size() * 8);
    return PRE3_OK;
}

// Every index a kernel follows in the compiled tables must stay inside its table: the kernels
// themselves do not range-check table contents.  Returns the number of violations found.
int pre3_debug_validate_tables(const pre3_handle *h) {
    if (!h || !h->compiled) return PRE3_E_BADARG;
    int64_t bad = 0;
    auto need = [&](bool ok) { if (!ok) ++bad; };
    const EdgeTables &T = h->T;
    const int ncol = T.n_classes + 1;
    need((int)T.state_kind.size() == T.n_states && (int)T.goto_row.size() == T.n_states);
    need((int64_t)T.edge.size() == (int64_t)T.n_states * ncol);
    for (int b = 0; b < 256; ++b) need(T.byte_class[b] < T.n_classes);
    for (int s = 0; s < T.n_states && bad == 0; ++s) {
        need(T.state_kind[s] >= 0 && T.state_kind[s] < T.n_kinds);
        for (int c = 0; c < ncol; ++c) {
            const uint32_t e = T.edge[(size_t)s * ncol + c];
            if ((e & kKindMask) == kShift) {
                // the per-byte offsets of the class must keep the target inside the state range
                for (int b = 0; b < 256; ++b)
                    if (T.byte_class[b] == c) need((int64_t)(e >> 2) + T.byte_delta[b] >= 0 && (int64_t)(e >> 2) + T.byte_delta[b] < T.n_states);
            }
        }
        const int r = T.goto_row[s];
        need(r < (int)T.goto_flat.size());
    }
    for (int32_t t : T.goto_flat) need(t < T.n_states);
    // reduction cycles: chains of records inside the pool, states in range, every record headed by its chain's state
    need((int)T.cycle_head.size() == T.n_states);
    int64_t records = 0;
    for (int s = 0; s < T.n_states && bad == 0; ++s)
        for (int at = T.cycle_head[s], guard = 0; at >= 0 && bad == 0; at = T.cycle_pool[at + 1]) {
            need(at + 2 < (int)T.cycle_pool.size() && ++guard <= T.n_cycles);
            if (bad) break;
            const int n = T.cycle_pool[at];
            need(n >= 1 && n <= kMaxCycleStates && at + 2 + n <= (int)T.cycle_pool.size() && T.cycle_pool[at + 1] < (int)T.cycle_pool.size());
            if (bad) break;
            need(T.cycle_pool[at + 2] == s);
            for (int k = 0; k < n; ++k) need(T.cycle_pool[at + 2 + k] >= 0 && T.cycle_pool[at + 2 + k] < T.n_states);
            ++records;
        }
    need(records == T.n_cycles);
    // merged reduction edges
    const SymbolEdges &S = h->S;
    if (S.enabled) {
        need((int)S.nodes.size() >= T.n_kinds && (int64_t)S.eff.size() == (int64_t)S.nodes.size() * ncol);
        need(S.child_state.size() == S.child_node.size());
        for (size_t i = 0; i < S.nodes.size(); ++i) {
            const SymbolNode &n = S.nodes[i];
            need(n.known >= 1 && n.child_count >= 0 && n.child_begin >= 0 &&
                 (size_t)n.child_begin + n.child_count <= S.child_state.size());
            for (int j = 0; j < n.child_count; ++j) {
                need(S.child_node[n.child_begin + j] == n.first_child + j);          // children are consecutive
                need(S.child_state[n.child_begin + j] >= 0 && S.child_state[n.child_begin + j] < T.n_states);
            }
            need(n.child_count == 0 || (n.first_child > (int)i && (size_t)n.first_child + n.child_count <= S.nodes.size()));
        }
        for (int32_t code : S.eff) {
            if (code < 0) { need(code >= kEffStepwise); continue; }
            need((code & 3) == 0 && (size_t)code + 4 <= S.pool.size());
            if ((size_t)code + 4 > S.pool.size()) continue;
            const int32_t *r = &S.pool[code];
            const int np = r[2] & kEffPushMask;
            need(r[0] >= 1 && np >= 1 && (size_t)code + 4 + np <= S.pool.size() && r[3] >= 0 && r[3] < T.n_kinds);
            if ((size_t)code + 4 + np <= S.pool.size())
                for (int k = 0; k < np; ++k) need(r[4 + k] >= 0 && r[4 + k] < T.n_states);
        }
    }
    // token-level edges
    const TokenEdges &E = h->E;
    if (E.enabled) {
        const int64_t n_dense = E.n_words ? (int64_t)E.dense_rows.size() / E.n_words : 0;
        need((int)E.root_of_state.size() == T.n_states && E.n_words == h->V.n_words);
        for (int32_t r : E.root_of_state) need(r >= 0 && r < (int)E.nodes.size());
        need(E.child_state.size() == E.child_node.size());
        for (size_t i = 0; i < E.nodes.size(); ++i) {
            const ConditionNode &n = E.nodes[i];
            need(n.known >= 1 && n.child_count >= 0 && n.child_begin >= 0 &&
                 (size_t)n.child_begin + n.child_count <= E.child_state.size());
            for (int j = 0; j < n.child_count; ++j) {
                const int32_t c = E.child_node[n.child_begin + j];
                need(c == E.child_node[n.child_begin] + j && c >= 0 && c < (int)i);   // children are stored before their parents
                need(j == 0 || E.child_state[n.child_begin + j] > E.child_state[n.child_begin + j - 1]);
            }
            need(n.dense_row >= -1 && n.dense_row < n_dense);
            need(n.delta_count >= 0 && n.delta_begin >= 0 && (size_t)n.delta_begin + n.delta_count <= E.delta_ids.size());
            need(n.walk_count >= -1 && n.walk_begin >= 0 &&
                 (n.walk_count < 0 || (size_t)n.walk_begin + n.walk_count <= E.walk_ids.size()));
        }
        // stack-effect records and their look-up table
        for (const ConditionNode &n : E.nodes) {
            need(n.effect_words >= 0 && n.effect_begin >= 0 && (size_t)n.effect_begin + n.effect_words <= E.effects.size());
            if (bad) break;
            for (int32_t at = n.effect_begin; at < n.effect_begin + n.effect_words;) {
                need(at + 4 <= n.effect_begin + n.effect_words);
                if (bad) break;
                const int32_t np = E.effects[at + 3];
                need(E.effects[at] >= 0 && E.effects[at] < h->V.n_tokens && E.effects[at + 1] >= 1 && E.effects[at + 1] <= 255 && np >= 1 &&
                     np <= 255 && at + 4 + np <= n.effect_begin + n.effect_words);
                if (bad) break;
                for (int i = 0; i < np; ++i) need(E.effects[at + 4 + i] >= 0 && E.effects[at + 4 + i] < T.n_states);
                at += 4 + np;
            }
        }
        const EffectTable &X = h->X;
        need(X.slots.size() == (X.slots.empty() ? 0 : ((size_t)X.bucket_mask + 1) * kEffectBucketSlots * 4));
        for (size_t i = 0; i + 3 < X.slots.size() && bad == 0; i += 4) {
            if (X.slots[i] < 0) continue;
            const EffectFields f = effect_unpack((uint32_t)X.slots[i + 1], (uint32_t)X.slots[i + 2], (uint32_t)X.slots[i + 3]);
            const int32_t tok = X.slots[i + 1] & 0x1FFFFF;
            need(X.slots[i] < (int)E.nodes.size() && tok < h->V.n_tokens && f.np >= 1 && f.k >= 1);
            if (f.inline_count > 0) need(f.inline_count == f.np && f.x0 < T.n_states && (f.np == 1 || f.x1 < T.n_states));
            else need(f.x0 >= 0 && (size_t)f.x0 + f.np <= X.pool.size());
        }
        for (int32_t v : X.pool) need(v >= 0 && v < T.n_states);
        for (int32_t t : E.delta_ids) need(t >= 0 && t < h->V.n_tokens);
        for (int32_t t : E.walk_ids) need(t >= 0 && t < h->V.n_tokens);
    }
    // vocabulary
    need((int)h->V.offsets.size() == h->V.n_tokens + 1);
    for (int t = 0; t < h->V.n_tokens; ++t) need(h->V.offsets[t] <= h->V.offsets[t + 1]);
    need(h->V.offsets.empty() || (size_t)h->V.offsets.back() + 4 <= h->V.bytes.size());
    return (int)std::min<int64_t>(bad, 1 << 30);
}

int pre3_debug_advance(const pre3_handle *h, int32_t *stack, int32_t *len, int32_t cap, const uint8_t *bytes,
                       int32_t n_bytes, int32_t use_merged) {
    if (!h || !h->compiled || !stack || !len || *len < 1 || *len > cap || (n_bytes > 0 && !bytes)) return PRE3_E_BADARG;
    if (use_merged && !h->S.enabled) return PRE3_E_BADARG;
    if (stack[*len - 1] < 0 || stack[*len - 1] >= h->T.n_states) return PRE3_E_BADARG;
    std::vector<int32_t> st(stack, stack + *len);
    if (n_bytes < 0)                                            // end of input
        return host_feed(h->T, h->S, st, h->T.n_classes, 0, 1 << 30, use_merged != 0) == kHostAccepted ? 0 : 1;
    if (n_bytes == 0) return 1;
    for (int i = 0; i < n_bytes; ++i) {
        int r = host_feed(h->T, h->S, st, h->T.byte_class[bytes[i]], h->T.byte_delta[bytes[i]], cap, use_merged != 0);
        if (r != kHostFed) return r == kHostOverflow ? 2 : 1;
    }
    std::copy(st.begin(), st.end(), stack);
    *len = (int32_t)st.size();
    return 0;
}

int pre3_debug_resolve_row(const pre3_handle *h, const int32_t *stack, int32_t len, uint32_t *row, int32_t *walk,
                           int32_t walk_cap, int32_t *n_walk, int32_t *info) {
    if (!h || !h->compiled || !h->E.enabled || !stack || !row || !walk || !n_walk) return PRE3_E_BADARG;
    std::vector<int32_t> w;
    std::memset(row, 0, sizeof(uint32_t) * h->V.n_words);
    bool ok = resolve_row(h->E, stack, len, row, w, info);
    *n_walk = (int32_t)w.size();
    if (!ok) return 0;
    if ((int32_t)w.size() > walk_cap) return PRE3_E_BADARG;
    std::copy(w.begin(), w.end(), walk);
    return 1;
}

}  // extern "C"

/*
 * pre3.h -- C ABI of the MI355X (gfx950) batched token-mask path of Pre^3
 * (arXiv 2506.03887: constrained LLM decoding with a deterministic pushdown automaton
 * built from a canonical LR(1) grammar).
 *
 * Per decode step, for every (sequence, vocabulary token) pair the token's bytes are
 * walked through the DPDA from the sequence's stack; the verdicts are packed into a
 * vocabulary bitmask, the bitmask is applied to the logits, and each sequence's stack is
 * advanced by its sampled token.  All per-step work runs in HIP kernels; the host only
 * compiles the grammar once.
 *
 * Conventions
 *   - "host" / "device" says where a pointer must live.  Device pointers are plain
 *     hipMalloc-style addresses (e.g. torch tensor data_ptr()); the library never frees
 *     or reallocates caller memory.
 *   - Every function returns PRE3_OK (0) or a negative pre3_status.  Nothing throws.
 *   - Device calls only enqueue work on `stream` (a hipStream_t, NULL = default stream)
 *     and return; they do not synchronise and do not allocate.  pre3_compile and
 *     pre3_bind_state are the calls that allocate device memory (tables; scratch sized by
 *     the bound batch).  Device calls that take the handle share that scratch: enqueue
 *     them so that calls on one handle do not run concurrently (one stream, or ordered
 *     by events); different handles are independent.  A handle's tables live on the
 *     device that was current in pre3_compile: later calls on it need that device current.
 *   - Terminals are single bytes; a parse stack holds LR(1) state ids only, bottom first
 *     (Sec. 3.2.2: an acceptance edge pushes the target node's state).
 *   - State ids: canonical LR(1) item sets (App. A.2) numbered in breadth-first discovery
 *     order from the initial set, trying terminals in ascending byte order and then
 *     nonterminals in order of first appearance on a left-hand side; with several
 *     grammars, the ids of grammar g are shifted by the number of states of grammars
 *     0..g-1 (disjoint union), so a stack identifies its grammar by itself.
 */
#ifndef PRE3_H
#define PRE3_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    PRE3_OK = 0,
    PRE3_E_BADARG = -1,          /* null pointer, bad size, misaligned buffer, wrong handle kind */
    PRE3_E_PARSE = -2,           /* malformed grammar text, undefined or useless nonterminal     */
    PRE3_E_NOT_LR1 = -3,         /* shift/reduce or reduce/reduce conflict in the canonical table */
    PRE3_E_TOKEN_TOO_LONG = -4,  /* a vocabulary token exceeds options.max_token_len             */
    PRE3_E_NOMEM = -5,
    PRE3_E_HIP = -6,             /* a HIP runtime call failed; text in pre3_last_error           */
    PRE3_E_LIMIT = -7            /* grammar exceeds an internal table limit                      */
} pre3_status;

/* per-sequence error codes written by pre3_advance into err[b] */
#define PRE3_SEQ_OK 0
#define PRE3_SEQ_NOT_ALLOWED 1   /* token not allowed (also: any token on a finished sequence)  */
#define PRE3_SEQ_OVERFLOW 2      /* the stack would exceed `cap` entries during the walk         */

#define PRE3_STATE_DONE (-1)     /* states[b] of a sequence that has taken the EOS token         */

#define PRE3_FLAG_HOST_ONLY 1    /* build the tables but upload nothing (no GPU needed);         */
                                 /* device calls on such a handle return PRE3_E_BADARG           */
#define PRE3_FLAG_STEPWISE_REDUCTIONS 4 /* do not merge reduction chains into single reduction   */
                                 /* edges: walks follow one reduction step at a time             */
#define PRE3_FLAG_NO_TOKEN_EDGES 2 /* do not precompute token-level edges: pre3_fill_mask then     */
                                 /* walks every (sequence, token) pair byte by byte              */
#define PRE3_FLAG_NO_TOKEN_EFFECTS 16 /* do not record the stack operations of the token-level edges:     */
                                 /* pre3_advance_fill_mask then walks every sampled token byte by byte   */
#define PRE3_FLAG_COMPACT_CYCLES 8 /* cycle-aware stacks (Sec. 3.2.3; Alg. 1 step 1): every call that */
                                 /* changes the bound stacks (pre3_advance, pre3_advance_fill_mask,  */
                                 /* pre3_jump_forward) afterwards takes complete traversals of       */
                                 /* reduction cycles out of them, see pre3_n_reduction_cycles.       */
                                 /* Needs stack_cap <= 4096.  The token-level edges are then built   */
                                 /* for compacted stacks: pre3_fill_mask stays exact on any valid     */
                                 /* stack, but one that was never compacted takes the slow walk       */

typedef struct pre3_handle pre3_handle;     /* opaque; owns host and device tables */
typedef void *pre3_stream;                  /* hipStream_t */

/* Vocabulary, host memory, borrowed for the duration of pre3_compile only.
 * Token t is bytes[offsets[t] .. offsets[t+1]).  The bytes of eos_id are ignored.
 * Tokens of length 0 are never allowed.  Equal byte strings get equal mask bits. */
typedef struct {
    const uint8_t *bytes;
    const int64_t *offsets;      /* [n_tokens + 1], non-decreasing, offsets[0] >= 0 */
    int32_t n_tokens;
    int32_t eos_id;              /* in [0, n_tokens) */
} pre3_vocab;

typedef struct {
    int32_t max_token_len;       /* 0 = default 64; longer tokens -> PRE3_E_TOKEN_TOO_LONG */
    int32_t stack_cap;           /* 0 = default 1024; largest `cap` accepted in pre3_stacks */
    int32_t flags;               /* PRE3_FLAG_* */
    int32_t max_condition_depth; /* 0 = default 48: deepest stack entry (below the top) that the    */
                                 /* stack-matching condition of a token-level edge may test; tokens */
                                 /* that would need more are walked byte by byte at run time        */
    int32_t row_threshold;       /* 0 = default 1: a node of a token-level condition tree holds a whole   */
                                 /* mask row once this many token ids have been allowed since the last   */
                                 /* such row on its path (identical rows are stored once); below the     */
                                 /* threshold the node lists the ids and the kernel ORs them in.  Larger */
                                 /* values trade table size for work at run time                         */
    int32_t effect_min_len;      /* 0 = default 5: tokens of at least this many bytes get a stack-effect     */
                                 /* record (see pre3_token_effect_stats); shorter ones are always walked     */
} pre3_options;

/* Parse stacks of a batch, device memory, caller-owned.
 * Row b is data[b*cap .. b*cap + len[b]); data[b*cap] is the initial state of the
 * sequence's grammar and data[b*cap + len[b] - 1] its current top.  len[b] >= 1. */
typedef struct {
    int32_t *data;               /* device [batch, cap] row-major */
    int32_t *len;                /* device [batch] */
    int32_t cap;
    int32_t batch;
} pre3_stacks;

/* Builds, on the host, the canonical LR(1) automaton of each grammar (App. A.2) and from
 * it the DPDA edge tables of Sec. 3.1-3.3: acceptance edges (shift: push the target state),
 * reduction edges keyed by the exposed stack state (the stack-matching condition), byte
 * classes that aggregate bytes with identical edges (Sec. 3.3, edge aggregation), and the
 * byte-sorted vocabulary layout; then uploads them to the current HIP device.
 *
 * grammars: host array of n_grammars NUL-terminated texts (n_grammars >= 1).  Format:
 *     Name ::= alt | alt ...      a following line starting with '|' continues the rule
 *     alt  = sequence of Names and "quoted byte strings" ("" = empty string)
 *          | [class]              a byte class must be a whole alternative (sugar for one
 *                                 production per byte; '^' negates, a-b is a range)
 *     escapes: \n \r \t \\ \" \] \- \^ \[ \xHH ; '#' starts a comment; first rule = start.
 * opt: host, may be NULL (defaults).
 * out: receives the handle; on error *out is still a valid handle holding only the error
 *      text (free it with pre3_free) or NULL if even that allocation failed.
 * Errors: BADARG, PARSE, NOT_LR1, TOKEN_TOO_LONG, LIMIT, NOMEM, HIP. */
int pre3_compile(const char *const *grammars, int32_t n_grammars, const pre3_vocab *vocab,
                 const pre3_options *opt, pre3_handle **out);

/* Releases host and device tables.  NULL is allowed.  The caller must have synchronised
 * every stream that still runs work of this handle. */
int pre3_free(pre3_handle *h);

/* Host text of the last error recorded on this handle ("" if none).  Never NULL. */
const char *pre3_last_error(const pre3_handle *h);

/* Initial LR(1) state of grammar g (the value to put in data[b*cap] with len[b] = 1 and
 * states[b]), or PRE3_E_BADARG. */
int32_t pre3_initial_state(const pre3_handle *h, int32_t grammar_idx);

/* Binds the per-sequence buffers that pre3_advance mutates (all device memory, caller-owned,
 * must outlive the binding): states [batch] (top state of each stack, or PRE3_STATE_DONE),
 * the stacks, and err [batch].  Rebinding replaces the previous binding.
 * This is the call that allocates the per-batch workspaces (private-stack spill areas, partial
 * results of the arg max and the top-k): one allocation of each kind per handle, sized for the
 * largest batch bound so far.  Binding a batch that needs no more reuses them; binding a larger
 * one frees the superseded workspace (hipFree: waits for the device to go idle) and allocates the
 * larger one, so a server that resizes its batch does not accumulate device memory.  Work that was
 * recorded into a HIP graph before such a growing rebind points at the freed workspace and must be
 * recorded again.  Errors: BADARG, HIP (allocation failed). */
int pre3_bind_state(pre3_handle *h, int32_t *states, pre3_stacks stacks, int32_t *err);

/* Token mask of one decode step (Sec. 1: every token whose bytes leave the language of
 * viable prefixes is excluded; Sec. 3.1-3.2: the walk follows acceptance and reduction
 * edges, each selected by input byte and stack-matching condition, never backtracking).
 * For each sequence b and token t: bit (t mod 32), least significant first, of word
 * bitmask[b*W + t/32], W = ceil(n_tokens/32), is 1 iff t is allowed after b's stack; the
 * EOS bit is 1 iff the text so far is a sentence; padding bits are 0.  A sequence with
 * states[b] == PRE3_STATE_DONE gets only the EOS bit.  Reads states/stacks (which may be
 * the bound buffers or any snapshot of the same shape), writes all batch*W words.
 * states, stacks.*, bitmask: device.  Errors: BADARG (null, cap > stack_cap, batch < 0). */
int pre3_fill_mask(pre3_handle *h, const int32_t *states, pre3_stacks stacks, uint32_t *bitmask,
                   pre3_stream stream);

/* Applies a token mask to bf16 logits in place (Sec. 1: the mask removes the sampling
 * probability of excluded tokens): logits[b*row_stride + t] becomes -inf (bit pattern
 * 0xFF80) where the token's bit is 0 and keeps its value, bit for bit, where it is 1 (the kernel
 * writes 128-byte lines whole: an allowed logit next to a masked one is stored back unchanged).
 * logits_bf16: device, [batch, >= vocab] with row_stride elements between rows;
 * bitmask: device [batch, ceil(vocab/32)].  Needs no handle.  Errors: BADARG. */
int pre3_apply_mask(uint16_t *logits_bf16, const uint32_t *bitmask, int32_t batch, int32_t vocab,
                    int64_t row_stride, pre3_stream stream);

/* pre3_fill_mask followed by pre3_apply_mask on the same rows, as one call: the mask of each
 * row segment is applied to the logits while it is still on chip, so the bitmask is not read
 * back from memory (Sec. 1: mask computation and masking belong to the same decode step).
 * Results are exactly those of the two calls in sequence: bitmask as pre3_fill_mask writes it,
 * logits (device, [batch, >= n_tokens], row_stride elements between rows) as pre3_apply_mask
 * leaves them.  A batch between a quarter of the GPU's compute units and all of them, no larger
 * than the bound batch, with logits as pre3_advance_fill_apply_mask's one-kernel form needs them,
 * runs through that kernel without the advance: each sequence's logits are fetched while its
 * mask row is looked up; a batch of more sequences than compute units runs as the two calls,
 * which are then the faster form.  Errors: BADARG. */
int pre3_fill_apply_mask(pre3_handle *h, const int32_t *states, pre3_stacks stacks, uint32_t *bitmask,
                         uint16_t *logits_bf16, int64_t row_stride, pre3_stream stream);

/* Advances every bound sequence by its sampled token (Sec. 3.2.2: acceptance edges push,
 * reduction edges match, pop and push).  tokens: device [batch]; tokens[b] < 0 skips b.
 * The EOS token, where allowed, sets states[b] = PRE3_STATE_DONE and leaves the stack
 * untouched.  A token that is not allowed, any token on a finished sequence, or an id
 * >= n_tokens sets err[b] = PRE3_SEQ_NOT_ALLOWED; a walk that would grow the stack
 * beyond cap sets err[b] = PRE3_SEQ_OVERFLOW; in both cases the sequence is left
 * unchanged.  Otherwise err[b] = 0, the stack holds the LR(1) stack after the token's
 * last byte (reductions that wait for the next byte are not applied) and states[b] its
 * top.  Errors: BADARG (nothing bound, null tokens). */
int pre3_advance(pre3_handle *h, const int32_t *tokens, pre3_stream stream);

/* pre3_advance for callers that cannot allocate device memory at all: code under HIP graph capture,
 * tight serving loops, harnesses that forbid hipMalloc.  Same results as pre3_advance, but on the
 * buffers passed in (nothing needs to be bound, so pre3_bind_state, which allocates the per-batch
 * workspaces, is never needed), and the spill area of the walks' private stacks is a fixed array
 * of 2^20 int32 (4 MiB) inside the library's own device code instead of an allocation.  The call
 * allocates nothing on the device and frees nothing; it only enqueues kernels on `stream`.
 * tokens [batch], states [batch], stacks, err [batch]: device, as for pre3_bind_state / pre3_advance.
 * Limit: batch * max(0, pre3_walk_depth_bound(h) - 16) <= 2^20, else PRE3_E_LIMIT (text in
 * pre3_last_error) and nothing is enqueued.  Every call on one GPU, from any handle or stream, uses
 * that GPU's one array: calls that overlap in time on one GPU race and must be ordered by the
 * caller (one stream, or events).  The array keeps the last call's contents; a walk writes each
 * spilled entry before it reads it, so nothing has to be cleared between calls.
 * Errors: BADARG (null pointer, cap > stack_cap, batch < 0), LIMIT, HIP. */
int pre3_advance_static(pre3_handle *h, const int32_t *tokens, int32_t *states, pre3_stacks stacks, int32_t *err,
                        pre3_stream stream);

#define PRE3_ADVANCE_RESTART_ON_EOS 1  /* slot reuse: a sequence that takes the EOS token (where allowed) */
                                      /* goes back to its initial state (len = 1) instead of DONE         */

/* pre3_advance followed by pre3_fill_mask on the bound buffers, as one call (the natural shape of
 * a decode loop: once the token is sampled, advance and prepare the next step's mask, which can
 * run under the model's next forward pass).  Results are exactly those of the two calls in
 * sequence: states, stacks and err as pre3_advance leaves them (with flag
 * PRE3_ADVANCE_RESTART_ON_EOS a sequence that takes EOS restarts from data[b*cap] with len 1),
 * bitmask (device, [batch, ceil(n_tokens/32)]) as pre3_fill_mask then writes it for the new
 * stacks.  A sequence whose advance fails keeps its stack and gets the mask of that stack.
 * (With PRE3_FLAG_COMPACT_CYCLES the stacks are compacted before the mask is looked up.)
 * Errors: BADARG (nothing bound, null pointer, unknown flag). */
int pre3_advance_fill_mask(pre3_handle *h, const int32_t *tokens, uint32_t *bitmask, int32_t flags,
                           pre3_stream stream);

/* One whole decode step as one call (Alg. 1 per step: advance by the sampled token, compute the
 * mask of the new stacks, mask the logits): pre3_advance_fill_mask followed by pre3_apply_mask of
 * the new rows on logits_bf16 (device, [batch, >= n_tokens] bf16 patterns, row_stride elements
 * between rows, masked in place).  Results are exactly those of the two calls in sequence --
 * states, stacks, err and bitmask as pre3_advance_fill_mask leaves them, logits as pre3_apply_mask
 * then leaves them.
 * The step can run as ONE kernel in which every sequence's logits are fetched while its token is
 * still being walked.  That form needs: logits aligned to 16 bytes, row_stride a multiple of 8, at
 * most 207,360 tokens (a row has to fit the registers of one compute unit), token-level edges in
 * use, and the mask row and -- with cycle-aware stacks -- the stack within the kernel's LDS.
 * It holds one sequence's logits in the registers of one compute unit; a batch larger than the
 * number of compute units goes as several launches of that kernel, each an equal share of the
 * batch of at most one sequence per unit.  The call chooses that form when the batch is between a
 * quarter of the GPU's compute units and all of them (64..256 sequences on 256 units: 23.5 against
 * 30.7 us per step at 256 x 128,256) and is the two calls otherwise.  PRE3_STEP_ONE_KERNEL asks
 * for the one kernel at any batch size where the conditions above hold (the call is still the two
 * calls where not): on larger batches it wins where the masks leave most lines of the logits to
 * be read (JSON, 512 x 128,256: 47.2 against 51.6 us) and loses where they are sparse (a fixed
 * schema, 512 x 152,064: 55.4 against 53.7 us), since it fetches a row before its mask is known
 * and pre3_apply_mask does not read what is masked as a whole.
 * flags: PRE3_ADVANCE_RESTART_ON_EOS as for pre3_advance_fill_mask, PRE3_STEP_ONE_KERNEL.
 * Errors: BADARG (nothing bound, null pointer, unknown flag, row_stride < n_tokens, logits not
 * 2-byte aligned), HIP. */
#define PRE3_STEP_ONE_KERNEL 2
int pre3_advance_fill_apply_mask(pre3_handle *h, const int32_t *tokens, uint32_t *bitmask, uint16_t *logits_bf16,
                                 int64_t row_stride, int32_t flags, pre3_stream stream);
/* One whole greedy decode step as one call: pre3_advance_fill_mask followed by
 * pre3_apply_mask_argmax of the new rows on logits_bf16 (device, [batch, >= n_tokens], row_stride
 * elements between rows; only read).  Results are exactly those of the two calls in sequence:
 * states, stacks, err and bitmask as pre3_advance_fill_mask leaves them, out_tokens[b] (device,
 * [batch]) the arg max of the allowed logits of row b under the rules of pre3_apply_mask_argmax.
 * out_tokens may be the tokens buffer itself (a greedy loop then needs no copy between steps).
 * The call takes its one-kernel form -- the logits are fetched while the token is walked and the
 * arg max is taken from the registers that hold them -- under the conditions and for the batch
 * sizes of pre3_advance_fill_apply_mask, except that the vocabulary may have at most 153,600 tokens
 * (the fold needs registers of its own), and is the two calls otherwise; flags as there.
 * Errors: BADARG (nothing bound, null pointer, unknown flag, row_stride < n_tokens, logits not
 * 2-byte aligned), HIP. */
int pre3_advance_fill_argmax(pre3_handle *h, const int32_t *tokens, uint32_t *bitmask, const uint16_t *logits_bf16,
                             int64_t row_stride, int32_t *out_tokens, int32_t flags, pre3_stream stream);

/* Which form pre3_advance_fill_apply_mask takes for the bound batch and these logits: 0 = the two
 * calls, n >= 1 = the one kernel, launched n times on equal shares of the batch (n = 1 up to one
 * sequence per compute unit); BADARG if nothing is bound.  pre3_advance_fill_argmax takes the same
 * form for vocabularies of at most 153,600 tokens.  Host call, launches nothing. */
int32_t pre3_step_is_one_kernel(const pre3_handle *h, const uint16_t *logits_bf16, int64_t row_stride, int32_t flags);

/* Greedy sampling fused behind the mask (Sec. 1: invalid tokens are excluded, then a token is
 * sampled; here the sampler is the arg max).  For every bound sequence b:
 *   out_tokens[b] = the token t with bit t of bitmask row b set whose bf16 logit is the largest
 *   number; among equal values (+0 and -0 are equal) the smallest id; NaN logits are never
 *   chosen; -1 if no token is both allowed and not NaN.
 * This is the arg max of what pre3_apply_mask would leave in the row, but the logits are only
 * read (groups of 8 masked tokens are not even read) and nothing is written back.
 * logits_bf16: device, [batch, row_stride] bf16 bit patterns, row_stride >= n_tokens (16-byte
 * aligned rows take the vector path, any other layout a slower one); bitmask: device, [batch,
 * ceil(n_tokens/32)] as pre3_fill_mask writes it; out_tokens: device [batch], ready to be
 * passed to pre3_advance.  batch is that of the bound buffers (pre3_bind_state), which also
 * sized the call's workspace inside the handle: calls on one handle must not overlap.
 * Errors: BADARG (nothing bound, null pointer, row_stride < n_tokens). */
int pre3_apply_mask_argmax(pre3_handle *h, const uint16_t *logits_bf16, int64_t row_stride, const uint32_t *bitmask,
                           int32_t *out_tokens, pre3_stream stream);

#define PRE3_TOPK_MAX 64

/* Top-k behind the mask (Sec. 1: invalid tokens are excluded, then a token is sampled; a top-k or
 * nucleus sampler only needs the k most probable of what is left).  For every bound sequence b and
 * j < k:  out_tokens[b*k + j] = the allowed token with the (j+1)-th largest bf16 logit as a number,
 * equal values (+0 and -0 are equal) in ascending order of id; NaN logits are never listed;
 * out_logits[b*k + j] (if not null) = that token's bf16 pattern as stored.  Rows with fewer than k
 * such tokens are padded with -1 and 0xFF80.  out_tokens[b*k] equals the choice of
 * pre3_apply_mask_argmax.  The logits are read once and not modified (groups of 8 masked tokens
 * are not read).  1 <= k <= PRE3_TOPK_MAX; layouts and the workspace rule as for
 * pre3_apply_mask_argmax.  Errors: BADARG (nothing bound, null pointer, row_stride < n_tokens, k out
 * of range), LIMIT (ceil(n_tokens / 16384) * k above 1024: k = 64 serves up to 262,144 tokens; or a
 * bound batch whose candidate workspace, batch * ceil(n_tokens / 16384) * 512 bytes, would pass 1 GiB). */
int pre3_apply_mask_topk(pre3_handle *h, const uint16_t *logits_bf16, int64_t row_stride, const uint32_t *bitmask,
                         int32_t k, int32_t *out_tokens, uint16_t *out_logits, pre3_stream stream);

/* Jump-forward (Sec. 3.3: runs of edges with a single successor merge into one jump): for every
 * bound, unfinished sequence, the bytes that every continuation of its text must start with.
 * While the end-of-sequence token is not allowed and exactly one of the 256 bytes keeps the text
 * a viable prefix, that byte is forced: it is stored in out_bytes[b * max_bytes + i] and the
 * sequence's stack is advanced by it (states, len and the stack entries change as under
 * pre3_advance; err is not touched).  A sequence stops at the first position with no or several
 * viable bytes, where EOS is allowed, after max_bytes bytes, or before a byte whose walk would
 * grow the stack beyond cap.  out_len[b] = number of forced bytes (0 for a finished sequence).
 * A server appends the bytes to the output (re-tokenising them as it likes) without running the
 * model, then asks for the next mask.  out_bytes: device [batch, max_bytes] (may be null when
 * max_bytes is 0); out_len: device [batch].  Errors: BADARG (nothing bound, null pointer,
 * negative max_bytes). */
int pre3_jump_forward(pre3_handle *h, uint8_t *out_bytes, int32_t *out_len, int32_t max_bytes, pre3_stream stream);

/* ---- host-side introspection of the compiled tables (used by tests and tools) ---- */

/* Reduction cycles (Sec. 3.2.3: cycles with the reduction problem; Alg. 1 step 1).  A cycle is
 * registered for a right-recursive production  A -> X1..Xn A  (1 <= n <= 64) and states
 * v1 = GOTO(vn, X1), v2 = GOTO(v1, X2), .., vn = GOTO(v(n-1), Xn) when every kernel item of v1 is
 * an item of A with the dot after its first symbol.  (In a conflict-free canonical automaton the
 * kernel of r = GOTO(vn, A) then holds only the finished item  A -> X1..Xn A .  and r reduces on
 * every lookahead that a kernel item of v1 carries.)
 * Then a stack  .. v1 .. vn v1 rest  accepts exactly the continuations of  .. v1 rest : whatever
 * looks below the upper v1 goes to r, pops the traversal and repeats one traversal lower before
 * the next byte is consumed.  With PRE3_FLAG_COMPACT_CYCLES the stacks are kept in the normal
 * form that results from rebuilding them bottom-up and, after each entry v1, dropping the n
 * entries below it while they equal v1..vn of a cycle headed by v1 (cycles of one head tried
 * shortest first, then in ascending order of their states, from the first again after a match).
 * Masks, err and DONE are those of the uncompacted stacks; len and the entries differ, and a
 * right-recursive list of any length keeps a bounded stack.  (The paper pops the traversal on the
 * cycle's back-edge; for cycles that are not of this shape, such as nesting, dropping a traversal
 * would forget the depth, so none is registered.)
 * pre3_n_reduction_cycles: number of registered cycles over all grammars.
 * pre3_reduction_cycle: writes the states v1..vn (global ids) of cycle `index` (ordered by v1,
 * then as tried) to out_states[0..out_cap) and returns n; BADARG if n > out_cap. */
int32_t pre3_n_reduction_cycles(const pre3_handle *h);
int32_t pre3_reduction_cycle(const pre3_handle *h, int32_t index, int32_t *out_states, int32_t out_cap);

/* Multi-symbol edges for jump-forward (Sec. 3.3, merging of deterministic single-successor runs):
 * the run of forced bytes that starts at `state`, i.e. while a state's only edge is an acceptance
 * edge on one byte.  out_bytes[i] / out_states[i] (host, out_cap entries each) = the i-th forced
 * byte and the state it is shifted to; at most 64 per entry (a longer run continues with the run of
 * its last state).  Returns the length, 0 if the state forces nothing; BADARG if out_cap is too small. */
int32_t pre3_forced_run(const pre3_handle *h, int32_t state, uint8_t *out_bytes, int32_t *out_states, int32_t out_cap);

/* Host evaluation of the normal form on the uploaded cycle tables: compacts stack[0..len) in place
 * and returns the new length (tests check the tables with it; the device path is the kernel). */
int32_t pre3_debug_compact(const pre3_handle *h, int32_t *stack, int32_t len);


int32_t pre3_n_grammars(const pre3_handle *h);
int32_t pre3_n_states(const pre3_handle *h);            /* total over all grammars */
int32_t pre3_n_byte_classes(const pre3_handle *h);      /* aggregated input symbols, without '$' */
int32_t pre3_byte_class(const pre3_handle *h, int32_t byte);
/* Edge leaving global state `state` on input `symbol` (0..255 a byte, 256 = end of input):
 * returns 0 none, 1 acceptance edge (*arg0 = target state), 2 reduction step (*arg0 = number
 * of states popped, *arg1 = nonterminal index local to the state's grammar), 3 accept. */
int32_t pre3_edge(const pre3_handle *h, int32_t state, int32_t symbol, int32_t *arg0, int32_t *arg1);
/* Target of the reduction step that exposes `state` and pushes nonterminal `nt` (the
 * stack-matching condition of a reduction edge), or -1. */
int32_t pre3_goto_target(const pre3_handle *h, int32_t state, int32_t nt);
/* Largest number of private stack entries a walk of one token can need. */
int32_t pre3_walk_depth_bound(const pre3_handle *h);
/* Number of token walks, since pre3_compile, that a kernel stopped at one of its internal guards
 * (a private stack deeper than pre3_walk_depth_bound, a reduction chain longer than the tables
 * allow) and therefore reported as "not allowed".  The bounds are derived from the grammar at
 * compile time, so the count is 0 unless the tables or the bound are wrong: tests and the
 * benchmark assert that.  Host call; copies one device counter back (synchronise the streams that
 * run the handle's work first, so that their walks are counted).  out: host.  Errors: BADARG, HIP. */
int pre3_debug_fault_count(pre3_handle *h, int64_t *out);
/* Measurement aid (no passage of the paper: it serves the benchmark): enqueues a one-thread kernel
 * that writes the device's 100 MHz wall clock to *out (device, 8 bytes).  Recorded between the
 * calls of a captured step it gives each kernel's duration in its real place, which HIP events
 * cannot give inside a graph; two stamps with nothing between them give the cost of a stamp.
 * Asynchronous on `stream`.  Errors: BADARG, HIP. */
int pre3_debug_timestamp(int64_t *out, pre3_stream stream);
/* Sizes of the token-level prefix-conditioned edge tables (Sec. 3.3, edge merging along the
 * bytes of each token): out[0] built?, [1] distinct root conditions, [2] condition-tree nodes,
 * [3] dense rows, [4] token ids in delta lists, [5] token ids in walk lists, [6] deepest stack
 * entry tested, [7] bytes of device memory they take. */
int pre3_token_edge_stats(const pre3_handle *h, int64_t out[8]);
/* Stack operations of the token-level edges (Sec. 3.1: an edge carries its accepted symbols, its
 * stack-matching condition and its stack operations): for every token of at least 5 bytes that a
 * node of a condition tree allows, what the token's walk does to any stack matching the node's
 * condition (how many entries it replaces, the states it pushes, the highest the stack gets on
 * the way).  pre3_advance_fill_mask applies such a token with one look-up instead of a walk; tokens
 * without a record (short ones, records that found their two hash buckets full, grammars whose
 * records would pass 12 Mi) are walked.  out[0] records, [1] records in the look-up table, [2] records
 * left out of it, [3] bytes of device memory. */
int pre3_token_effect_stats(const pre3_handle *h, int64_t out[4]);
/* Host mirror of that look-up (tests and tools): stack[0..len) (host, global state ids, bottom
 * first) and a token id.  On a hit writes the stack after the token to out[0..return value) and,
 * if info is not NULL, k (entries from the top that the record covers), peak (the walk overflows a
 * capacity cap iff len + peak >= cap) and the number of states pushed; returns the new length, 0 if
 * no record covers (stack, token), or PRE3_E_BADARG (also when out_cap is too small). */
int32_t pre3_debug_token_effect(const pre3_handle *h, const int32_t *stack, int32_t len, int32_t token, int32_t *out,
                                int32_t out_cap, int32_t *info);
/* Sizes of the merged reduction edges (Sec. 3.2.2; Alg. 1 step 3): out[0] built?, [1] condition
 * nodes, [2] deepest stack entry tested, [3] bytes of device memory. */
int pre3_symbol_edge_stats(const pre3_handle *h, int64_t out[4]);
/* Consistency check of the compiled tables on the host (tests and tools): every index that a
 * kernel follows (edge targets, goto rows, condition children, record offsets, token ids, dense
 * rows, vocabulary offsets) must stay inside its table.  Returns the number of violations (0 for
 * a handle that pre3_compile built), or PRE3_E_BADARG. */
int pre3_debug_validate_tables(const pre3_handle *h);
/* Host mirror of one sequence's advance, for checking the compiled edge tables without a GPU
 * (tests and tools; never used by the device calls): walks bytes[0..n_bytes) (n_bytes < 0: the
 * end-of-input symbol) on stack[0..*len) (host memory, capacity cap) with the merged reduction
 * edges (use_merged != 0) or one reduction step at a time.  Returns 0 (stack and *len updated;
 * for end of input: accepted, stack untouched), 1 not allowed, 2 overflow, or PRE3_E_BADARG. */
int pre3_debug_advance(const pre3_handle *h, int32_t *stack, int32_t *len, int32_t cap, const uint8_t *bytes,
                       int32_t n_bytes, int32_t use_merged);
/* Table lookup only, on the host: evaluates the condition tree for one stack (host memory,
 * global state ids, bottom first).  row (ceil(n_tokens/32) words) receives the tokens whose
 * merged edge matches the stack; walk[0..*n_walk) the token ids the tables leave to a
 * byte-by-byte walk; info (may be NULL) 4 ints: condition-tree nodes on the path, index of the
 * node whose dense row is used, delta ids ORed, deepest stack entry tested.  Returns 1, or 0 if the tables hold no answer for this stack (then the
 * kernels walk every token), or PRE3_E_BADARG (also when walk_cap is too small). */
int pre3_debug_resolve_row(const pre3_handle *h, const int32_t *stack, int32_t len, uint32_t *row,
                           int32_t *walk, int32_t walk_cap, int32_t *n_walk, int32_t *info);

#ifdef __cplusplus
}
#endif
#endif /* PRE3_H */

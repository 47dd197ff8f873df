/*
 * pre3_oracle.c -- TEST INFRASTRUCTURE, NOT PRODUCT CODE.
 *
 * A plain, slow, obviously-correct CPU statement of what the constrained-decoding
 * hot path of Pre^3 (arXiv 2506.03887) computes.  Only tests, the smoke check and
 * the benchmark's CPU-baseline leg may use it.  It shares no code with the GPU
 * library and knows nothing about prefix-conditioned edges, tries or caches: it is
 * the textbook canonical LR(1) construction (paper App. A.2, "Detailed
 * Construction Procedure of the Canonical LR(1) Automaton") followed by the
 * textbook stack-based parse loop (App. A.2, "Stack-based Parsing Mechanism")
 * run once per (sequence, token) pair.
 *
 * The result it defines: token t (bytes t1..tn, n >= 1) is ALLOWED after the
 * emitted text p iff p.t is a prefix of some sentence of the grammar; the
 * end-of-sequence token is allowed iff p itself is a sentence.  For a canonical
 * LR(1) parser over a grammar without useless symbols the parse loop decides
 * exactly this (an item [A -> alpha., a] is in a state only if a can follow in
 * that context, because lookaheads propagate through FIRST(beta a), App. A.2
 * "Closure Operation"), so "no Error action before the byte is shifted" is the
 * test.  Section 1 of the paper states the mask semantics ("excludes invalid
 * tokens ... probability mask").
 *
 * Conventions fixed here where the paper is silent (each is listed in the design
 * notes of the repository):
 *   - terminals are single bytes 0..255; '$' (end of input) is terminal 256;
 *   - a character class in the grammar text is sugar for one production per byte;
 *   - the parse stack holds state ids only (Sec. 3.2.2: an acceptance edge pushes
 *     the target node's state); stack[0] is the initial state;
 *   - states are numbered in breadth-first discovery order from I0, trying the
 *     terminals in ascending byte order and then the nonterminals in order of
 *     first appearance on a left-hand side;
 *   - no reduction is performed after the last byte of a token: pending
 *     reductions wait for the next lookahead byte (or for '$');
 *   - several grammars form a disjoint union: state ids of grammar g are shifted
 *     by the total number of states of grammars 0..g-1.
 *
 * Pinned by tests/test_oracle_*.py: hand-derived canonical collections of small
 * textbook grammars, conflict detection, brute-force enumeration of all strings
 * up to length 8 with an independent (non-LR) recogniser, Dyck == counter,
 * right-linear grammar == DFA, JSON grammar == the json module of the Python
 * standard library, and the prefix/concatenation/EOS invariants; the greedy choice
 * (masked arg max) against numpy's argmax over the candidates and hand cases, the
 * top-k list against numpy's stable sort of the candidates and hand cases; the
 * jump-forward bytes against the forced bytes read off the brute-force sets of
 * viable prefixes; seeded random grammars against the brute-force recogniser
 * (tests/test_random_grammars.py); the statements of the paper that can be checked
 * mechanically (tests/golden/paper_statements.txt, tests/test_golden.py); the
 * cycle-aware stacks of Sec. 3.2.3 (which cycles are registered: hand-derived cases;
 * soundness: compacted stacks against the brute-force recogniser on every split of
 * every short string, curated and seeded random grammars; right-recursive JSON with
 * compaction against left-recursive JSON: tests/test_oracle_cycles.py).  No function
 * here is unpinned.
 */
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>
#include <stdarg.h>

#define N_TERM 257          /* bytes 0..255 and '$' = 256 */
#define T_END 256
#define NT_BASE 257         /* symbol code of nonterminal i is NT_BASE + i */

enum { A_ERROR = 0, A_SHIFT = 1, A_REDUCE = 2, A_ACCEPT = 3 };

typedef struct {
    int lhs;                /* nonterminal index */
    int len;
    int *rhs;               /* symbol codes */
} prod_t;

typedef struct { int prod, dot, la; } item_t;

typedef struct {
    int n_nt;               /* includes the augmented start symbol (last index) */
    char **nt_name;
    int n_prod;
    prod_t *prod;           /* prod[0] is S' -> S */
    int n_states;
    uint8_t *act_kind;      /* [n_states][N_TERM] */
    int *act_arg;           /* [n_states][N_TERM]: shift target or production */
    int *go;                /* [n_states][n_nt], -1 = none */
    int *n_items;           /* [n_states] size of each closed item set */
    /* reduction cycles (Sec. 3.2.3): cycle k has cyc_len[k] states cyc_state[cyc_off[k] ..],
     * local ids, ordered by (first state, length, states) */
    int n_cycles;
    int *cyc_len, *cyc_off, *cyc_state;
} grammar_t;

typedef struct {
    int n_grammars;
    grammar_t **g;
    int *offset;            /* [n_grammars+1] running state offsets */
} oracle_t;

/* ------------------------------------------------------------------ errors */

static void set_err(char *err, int errlen, const char *fmt, ...) {
    if (!err || errlen <= 0) return;
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(err, (size_t)errlen, fmt, ap);
    va_end(ap);
}

/* ------------------------------------------------ grammar text -> productions
 * Text format (one grammar):
 *   Name ::= alt | alt ...        a following line that starts with '|' continues
 *   alt  = sequence of Names and "quoted byte strings"; "" is the empty string
 *        | [class]                a class must be the whole alternative
 *   escapes inside "..." and [...]:  \n \r \t \\ \" \] \- \^ \xHH
 *   '#' starts a comment.  The first rule defines the start symbol.
 */
enum { TK_EOF, TK_IDENT, TK_ASSIGN, TK_BAR, TK_STRING, TK_CLASS, TK_NEWLINE };

typedef struct {
    int kind;
    char *text;             /* identifier name, or string bytes */
    int len;                /* string length */
    uint8_t set[256];       /* class membership */
} token_t;

typedef struct { token_t *t; int n, cap; } toklist_t;

static void tok_push(toklist_t *L, token_t tk) {
    if (L->n == L->cap) {
        L->cap = L->cap ? 2 * L->cap : 64;
        L->t = (token_t *)realloc(L->t, sizeof(token_t) * (size_t)L->cap);
    }
    L->t[L->n++] = tk;
}

static int hexval(int c) {
    if (c >= '0' && c <= '9') return c - '0';
    if (c >= 'a' && c <= 'f') return c - 'a' + 10;
    if (c >= 'A' && c <= 'F') return c - 'A' + 10;
    return -1;
}

/* Reads one possibly escaped byte at s[*i]; returns the byte value or -1. */
static int read_escaped(const char *s, int *i) {
    int c = (unsigned char)s[*i];
    if (c == 0) return -1;
    if (c != '\\') { (*i)++; return c; }
    int d = (unsigned char)s[*i + 1];
    if (d == 0) return -1;
    if (d == 'x') {
        int h1 = hexval((unsigned char)s[*i + 2]);
        if (h1 < 0) return -1;
        int h2 = hexval((unsigned char)s[*i + 3]);
        if (h2 < 0) return -1;
        *i += 4;
        return h1 * 16 + h2;
    }
    *i += 2;
    switch (d) {
        case 'n': return '\n';
        case 'r': return '\r';
        case 't': return '\t';
        case '\\': case '"': case ']': case '-': case '^': case '[': return d;
        default: return -1;
    }
}

static int tokenize(const char *s, toklist_t *L, char *err, int errlen) {
    int i = 0, line = 1;
    for (;;) {
        int c = (unsigned char)s[i];
        token_t tk;
        memset(&tk, 0, sizeof tk);
        if (c == 0) { tk.kind = TK_EOF; tok_push(L, tk); return 0; }
        if (c == '\n') { tk.kind = TK_NEWLINE; tok_push(L, tk); i++; line++; continue; }
        if (c == ' ' || c == '\t' || c == '\r') { i++; continue; }
        if (c == '#') { while (s[i] && s[i] != '\n') i++; continue; }
        if (c == '|') { tk.kind = TK_BAR; tok_push(L, tk); i++; continue; }
        if (c == ':' && s[i + 1] == ':' && s[i + 2] == '=') {
            tk.kind = TK_ASSIGN; tok_push(L, tk); i += 3; continue;
        }
        if ((c >= 'A' && c <= 'Z') || (c >= 'a' && c <= 'z') || c == '_') {
            int j = i;
            while ((s[j] >= 'A' && s[j] <= 'Z') || (s[j] >= 'a' && s[j] <= 'z') ||
                   (s[j] >= '0' && s[j] <= '9') || s[j] == '_') j++;
            tk.kind = TK_IDENT;
            tk.text = (char *)malloc((size_t)(j - i + 1));
            memcpy(tk.text, s + i, (size_t)(j - i));
            tk.text[j - i] = 0;
            tok_push(L, tk);
            i = j;
            continue;
        }
        if (c == '"') {
            i++;
            tk.kind = TK_STRING;
            tk.text = (char *)malloc(strlen(s + i) + 1);
            tk.len = 0;
            while (s[i] != '"') {
                if (s[i] == 0 || s[i] == '\n') {
                    set_err(err, errlen, "line %d: unterminated string", line);
                    free(tk.text);
                    return -1;
                }
                int b = read_escaped(s, &i);
                if (b < 0) { set_err(err, errlen, "line %d: bad escape in string", line); free(tk.text); return -1; }
                tk.text[tk.len++] = (char)b;
            }
            i++;
            tok_push(L, tk);
            continue;
        }
        if (c == '[') {
            i++;
            tk.kind = TK_CLASS;
            int neg = 0;
            if (s[i] == '^') { neg = 1; i++; }
            while (s[i] != ']') {
                if (s[i] == 0 || s[i] == '\n') {
                    set_err(err, errlen, "line %d: unterminated class", line);
                    return -1;
                }
                int lo = read_escaped(s, &i);
                if (lo < 0) { set_err(err, errlen, "line %d: bad escape in class", line); return -1; }
                int hi = lo;
                if (s[i] == '-' && s[i + 1] != ']') {
                    i++;
                    hi = read_escaped(s, &i);
                    if (hi < 0 || hi < lo) {
                        set_err(err, errlen, "line %d: bad range in class", line);
                        return -1;
                    }
                }
                for (int b = lo; b <= hi; b++) tk.set[b] = 1;
            }
            i++;
            if (neg) for (int b = 0; b < 256; b++) tk.set[b] = (uint8_t)!tk.set[b];
            tok_push(L, tk);
            continue;
        }
        set_err(err, errlen, "line %d: unexpected character '%c'", line, c);
        return -1;
    }
}

static void add_prod(grammar_t *G, int lhs, const int *rhs, int len) {
    G->prod = (prod_t *)realloc(G->prod, sizeof(prod_t) * (size_t)(G->n_prod + 1));
    prod_t *p = &G->prod[G->n_prod++];
    p->lhs = lhs;
    p->len = len;
    p->rhs = (int *)malloc(sizeof(int) * (size_t)(len > 0 ? len : 1));
    if (len > 0) memcpy(p->rhs, rhs, sizeof(int) * (size_t)len);
}

static int find_nt(const grammar_t *G, const char *name) {
    for (int i = 0; i < G->n_nt; i++)
        if (strcmp(G->nt_name[i], name) == 0) return i;
    return -1;
}

/* The rules of a tokenised grammar text; `buf` has room for every symbol of the text. */
static int parse_rules(toklist_t L, int *buf, grammar_t *G, char *err, int errlen) {
    /* pass 1: left-hand sides in order of first appearance */
    for (int k = 0; k + 1 < L.n; k++) {
        if (L.t[k].kind == TK_IDENT && L.t[k + 1].kind == TK_ASSIGN) {
            if (find_nt(G, L.t[k].text) < 0) {
                G->nt_name = (char **)realloc(G->nt_name, sizeof(char *) * (size_t)(G->n_nt + 1));
                G->nt_name[G->n_nt++] = strdup(L.t[k].text);
            }
        }
    }
    if (G->n_nt == 0) { set_err(err, errlen, "grammar has no rules"); return -1; }
    /* the augmented start symbol S' gets the last index; production 0 is S' -> S */
    int start = 0;
    G->nt_name = (char **)realloc(G->nt_name, sizeof(char *) * (size_t)(G->n_nt + 1));
    G->nt_name[G->n_nt] = strdup("$accept");
    int aug = G->n_nt++;
    int rhs0 = NT_BASE + start;
    add_prod(G, aug, &rhs0, 1);

    /* pass 2: rules */
    int k = 0;
    while (L.t[k].kind != TK_EOF) {
        if (L.t[k].kind == TK_NEWLINE) { k++; continue; }
        if (L.t[k].kind != TK_IDENT || L.t[k + 1].kind != TK_ASSIGN) {
            set_err(err, errlen, "expected 'Name ::=' at token %d", k);
            return -1;
        }
        int lhs = find_nt(G, L.t[k].text);
        k += 2;
        for (;;) {                         /* one alternative per iteration */
            int n = 0, is_class = 0, n_items = 0;
            while (L.t[k].kind == TK_IDENT || L.t[k].kind == TK_STRING || L.t[k].kind == TK_CLASS) {
                if (L.t[k].kind == TK_IDENT && L.t[k + 1].kind == TK_ASSIGN) break;
                n_items++;
                if (L.t[k].kind == TK_IDENT) {
                    int nt = find_nt(G, L.t[k].text);
                    if (nt < 0) {
                        set_err(err, errlen, "undefined nonterminal '%s'", L.t[k].text);
                        return -1;
                    }
                    buf[n++] = NT_BASE + nt;
                } else if (L.t[k].kind == TK_STRING) {
                    for (int j = 0; j < L.t[k].len; j++) buf[n++] = (unsigned char)L.t[k].text[j];
                } else {
                    is_class = 1;
                    if (n_items != 1) {
                        set_err(err, errlen, "rule '%s': a class must be a whole alternative",
                                G->nt_name[lhs]);
                        return -1;
                    }
                    for (int b = 0; b < 256; b++)
                        if (L.t[k].set[b]) { int sym = b; add_prod(G, lhs, &sym, 1); }
                }
                k++;
                if (is_class) break;
            }
            if (is_class) {
                if (L.t[k].kind == TK_IDENT && L.t[k + 1].kind != TK_ASSIGN) {
                    set_err(err, errlen, "rule '%s': a class must be a whole alternative",
                            G->nt_name[lhs]);
                    return -1;
                }
                if (L.t[k].kind == TK_STRING || L.t[k].kind == TK_CLASS) {
                    set_err(err, errlen, "rule '%s': a class must be a whole alternative",
                            G->nt_name[lhs]);
                    return -1;
                }
            } else {
                if (n_items == 0) {
                    set_err(err, errlen, "rule '%s': empty alternative must be written \"\"",
                            G->nt_name[lhs]);
                    return -1;
                }
                add_prod(G, lhs, buf, n);
            }
            /* continue with '| alt', possibly on a following line */
            int kk = k;
            while (L.t[kk].kind == TK_NEWLINE) kk++;
            if (L.t[kk].kind == TK_BAR) { k = kk + 1; continue; }
            break;
        }
        if (L.t[k].kind != TK_NEWLINE && L.t[k].kind != TK_EOF) {
            set_err(err, errlen, "rule '%s': unexpected token after alternative", G->nt_name[lhs]);
            return -1;
        }
    }
    return 0;
}

static int parse_grammar(const char *text, grammar_t *G, char *err, int errlen) {
    toklist_t L = {0, 0, 0};
    int rc = tokenize(text, &L, err, errlen);
    if (rc == 0) {
        int *buf = (int *)malloc(sizeof(int) * (strlen(text) + 4));
        rc = parse_rules(L, buf, G, err, errlen);
        free(buf);
    }
    for (int i = 0; i < L.n; i++) free(L.t[i].text);
    free(L.t);
    return rc;
}

/* -------------------------------------------- useless symbols (must be none) */

static int check_reduced(const grammar_t *G, char *err, int errlen) {
    int n = G->n_nt;
    uint8_t *productive = (uint8_t *)calloc((size_t)n, 1);
    uint8_t *reach = (uint8_t *)calloc((size_t)n, 1);
    int changed = 1;
    while (changed) {
        changed = 0;
        for (int p = 0; p < G->n_prod; p++) {
            const prod_t *P = &G->prod[p];
            if (productive[P->lhs]) continue;
            int ok = 1;
            for (int j = 0; j < P->len; j++)
                if (P->rhs[j] >= NT_BASE && !productive[P->rhs[j] - NT_BASE]) { ok = 0; break; }
            if (ok) { productive[P->lhs] = 1; changed = 1; }
        }
    }
    reach[G->prod[0].lhs] = 1;
    changed = 1;
    while (changed) {
        changed = 0;
        for (int p = 0; p < G->n_prod; p++) {
            const prod_t *P = &G->prod[p];
            if (!reach[P->lhs]) continue;
            for (int j = 0; j < P->len; j++)
                if (P->rhs[j] >= NT_BASE && !reach[P->rhs[j] - NT_BASE]) {
                    reach[P->rhs[j] - NT_BASE] = 1;
                    changed = 1;
                }
        }
    }
    int rc = 0;
    for (int i = 0; i < n && rc == 0; i++) {
        if (!productive[i]) { set_err(err, errlen, "nonterminal '%s' derives no string", G->nt_name[i]); rc = -1; }
        else if (!reach[i]) { set_err(err, errlen, "nonterminal '%s' is unreachable", G->nt_name[i]); rc = -1; }
    }
    free(productive);
    free(reach);
    return rc;
}

/* ------------------------------------------------------------- FIRST sets */

typedef struct {
    uint8_t *nullable;      /* [n_nt] */
    uint8_t *first;         /* [n_nt][N_TERM] */
} first_t;

static void compute_first(const grammar_t *G, first_t *F) {
    F->nullable = (uint8_t *)calloc((size_t)G->n_nt, 1);
    F->first = (uint8_t *)calloc((size_t)G->n_nt * N_TERM, 1);
    int changed = 1;
    while (changed) {
        changed = 0;
        for (int p = 0; p < G->n_prod; p++) {
            const prod_t *P = &G->prod[p];
            uint8_t *fa = F->first + (size_t)P->lhs * N_TERM;
            int all_nullable = 1;
            for (int j = 0; j < P->len; j++) {
                int x = P->rhs[j];
                if (x < NT_BASE) {
                    if (!fa[x]) { fa[x] = 1; changed = 1; }
                    all_nullable = 0;
                    break;
                }
                const uint8_t *fb = F->first + (size_t)(x - NT_BASE) * N_TERM;
                for (int t = 0; t < N_TERM; t++)
                    if (fb[t] && !fa[t]) { fa[t] = 1; changed = 1; }
                if (!F->nullable[x - NT_BASE]) { all_nullable = 0; break; }
            }
            if (all_nullable && !F->nullable[P->lhs]) { F->nullable[P->lhs] = 1; changed = 1; }
        }
    }
}

/* FIRST(beta a) where beta = rhs[from..len) of production P: writes a 0/1 vector. */
static void first_of_tail(const grammar_t *G, const first_t *F, const prod_t *P, int from, int a,
                          uint8_t *out) {
    (void)G;
    memset(out, 0, N_TERM);
    for (int j = from; j < P->len; j++) {
        int x = P->rhs[j];
        if (x < NT_BASE) { out[x] = 1; return; }
        const uint8_t *fb = F->first + (size_t)(x - NT_BASE) * N_TERM;
        for (int t = 0; t < N_TERM; t++) if (fb[t]) out[t] = 1;
        if (!F->nullable[x - NT_BASE]) return;
    }
    out[a] = 1;
}

/* ---------------------------------------------- item sets, CLOSURE and GOTO */

typedef struct { item_t *it; int n, cap; } itemset_t;

static void iset_push(itemset_t *S, item_t x) {
    if (S->n == S->cap) {
        S->cap = S->cap ? 2 * S->cap : 256;
        S->it = (item_t *)realloc(S->it, sizeof(item_t) * (size_t)S->cap);
    }
    S->it[S->n++] = x;
}

static int item_cmp(const void *pa, const void *pb) {
    const item_t *a = (const item_t *)pa, *b = (const item_t *)pb;
    if (a->prod != b->prod) return a->prod < b->prod ? -1 : 1;
    if (a->dot != b->dot) return a->dot < b->dot ? -1 : 1;
    if (a->la != b->la) return a->la < b->la ? -1 : 1;
    return 0;
}

typedef struct {
    const grammar_t *G;
    const first_t *F;
    int *prod_off;          /* [n_prod] offset of (prod, dot=0) among all dotted rules */
    uint8_t *seen;          /* [n_dotted][N_TERM] membership flags of the set being closed */
} closure_ctx_t;

static size_t seen_index(const closure_ctx_t *C, item_t x) {
    return ((size_t)(C->prod_off[x.prod] + x.dot)) * N_TERM + (size_t)x.la;
}

/* CLOSURE(I): smallest superset of I that, for every [A -> alpha . B beta, a] in it,
 * every production B -> gamma and every b in FIRST(beta a), holds [B -> . gamma, b]. */
static void closure(closure_ctx_t *C, itemset_t *S) {
    const grammar_t *G = C->G;
    uint8_t fb[N_TERM];
    for (int i = 0; i < S->n; i++) C->seen[seen_index(C, S->it[i])] = 1;
    for (int i = 0; i < S->n; i++) {          /* S grows while we scan it */
        item_t x = S->it[i];
        const prod_t *P = &G->prod[x.prod];
        if (x.dot >= P->len) continue;
        int B = P->rhs[x.dot];
        if (B < NT_BASE) continue;
        first_of_tail(G, C->F, P, x.dot + 1, x.la, fb);
        for (int q = 0; q < G->n_prod; q++) {
            if (G->prod[q].lhs != B - NT_BASE) continue;
            for (int b = 0; b < N_TERM; b++) {
                if (!fb[b]) continue;
                item_t y = {q, 0, b};
                size_t idx = seen_index(C, y);
                if (!C->seen[idx]) { C->seen[idx] = 1; iset_push(S, y); }
            }
        }
    }
    for (int i = 0; i < S->n; i++) C->seen[seen_index(C, S->it[i])] = 0;
    qsort(S->it, (size_t)S->n, sizeof(item_t), item_cmp);
}

/* GOTO(I, X) = CLOSURE({[A -> alpha X . beta, a] : [A -> alpha . X beta, a] in I}) */
static void goto_set(closure_ctx_t *C, const itemset_t *I, int X, itemset_t *J) {
    J->n = 0;
    for (int i = 0; i < I->n; i++) {
        item_t x = I->it[i];
        const prod_t *P = &C->G->prod[x.prod];
        if (x.dot < P->len && P->rhs[x.dot] == X) {
            item_t y = {x.prod, x.dot + 1, x.la};
            iset_push(J, y);
        }
    }
    if (J->n > 0) closure(C, J);
}

static int same_set(const itemset_t *a, const itemset_t *b) {
    return a->n == b->n && memcmp(a->it, b->it, sizeof(item_t) * (size_t)a->n) == 0;
}

static uint64_t set_hash(const itemset_t *a) {
    uint64_t h = 1469598103934665603ull;
    for (int i = 0; i < a->n; i++) {
        h = (h ^ (uint64_t)a->it[i].prod) * 1099511628211ull;
        h = (h ^ (uint64_t)a->it[i].dot) * 1099511628211ull;
        h = (h ^ (uint64_t)a->it[i].la) * 1099511628211ull;
    }
    return h;
}

/* Sets one ACTION cell; a second, different entry is an LR(1) conflict. */
static int set_action(grammar_t *G, int s, int a, int kind, int arg, char *err, int errlen) {
    size_t c = (size_t)s * N_TERM + (size_t)a;
    if (G->act_kind[c] == A_ERROR) { G->act_kind[c] = (uint8_t)kind; G->act_arg[c] = arg; return 0; }
    if (G->act_kind[c] == kind && G->act_arg[c] == arg) return 0;
    const char *names[] = {"error", "shift", "reduce", "accept"};
    set_err(err, errlen, "grammar is not LR(1): %s/%s conflict in state %d on terminal %d",
            names[G->act_kind[c]], names[kind], s, a);
    return -1;
}

/* Canonical collection (App. A.2 "Construction Algorithm") and the ACTION / GOTO
 * tables (App. A.2 "Parsing with the Canonical LR(1) Automaton"). */
/* ---------------------------------------------------------- reduction cycles */

/* Sec. 3.2.3 and Alg. 1 step 1 pop a complete traversal of a cycle "with the reduction
 * problem" that "corresponds to recursive reduction of a nonterminal A".  The reading taken
 * here (the paper does not define the terms): a production  A -> X1 .. Xn A  and item sets
 * v1 .. vn with  GOTO(vn, X1) = v1, GOTO(v1, X2) = v2, .., GOTO(v(n-1), Xn) = vn,  such that
 * every kernel item (dot not at the left end) of v1 is [A -> Y . delta, a]: an item of A with
 * the dot after one symbol.
 * In a conflict-free canonical LR(1) automaton two more facts follow, with r = GOTO(vn, A):
 *   (i)  every kernel item of r is the finished [A -> X1 .. Xn A ., a];
 *   (ii) for every kernel item [.., a] of v1 the item [A -> X1 .. Xn A ., a] is in r.
 * (The kernel of v1 stems from closure items [A -> . X1 delta, a] of vn; the closure gives all
 * productions of A the same lookaheads L, the union of FIRST(beta b) over the items
 * [C -> alpha . A beta, b] of vn; the item of the cycle's own production carries L from v1 along
 * the path to vn, which gives (ii); an item of vn with A after the dot other than that one
 * would put FIRST(beta b), a part of L, on a second action of r: a conflict, hence (i).)
 * Why a stack  .. v1 .. vn v1 rest  then accepts the same continuations as  .. v1 rest : the
 * parser looks below the upper v1 only by finishing a kernel item of it, which pops down to the
 * entry under v1 and goes to A from there: from vn that is r, where by (i) and (ii) the same
 * lookahead reduces A -> X1..Xn A, pops r and the traversal v1..vn and goes to A again from the
 * entry below -- the very configuration the shorter stack reached directly. */
static int cycle_cmp(const int *a, int na, const int *b, int nb) {
    if (a[0] != b[0]) return a[0] < b[0] ? -1 : 1;
    if (na != nb) return na < nb ? -1 : 1;
    for (int i = 0; i < na; i++)
        if (a[i] != b[i]) return a[i] < b[i] ? -1 : 1;
    return 0;
}

#define MAX_CYCLE_STATES 64      /* longer cycles are not registered */

static void find_cycles(grammar_t *G, const itemset_t *states, int n_states, const int *delta, int n_sym) {
    int cap = 16, total = 0;
    G->n_cycles = 0;
    G->cyc_len = (int *)malloc(sizeof(int) * (size_t)cap);
    G->cyc_off = (int *)malloc(sizeof(int) * (size_t)cap);
    G->cyc_state = (int *)malloc(sizeof(int) * (size_t)cap * MAX_CYCLE_STATES);
    for (int p = 1; p < G->n_prod; p++) {
        const prod_t *P = &G->prod[p];
        int n = P->len - 1;
        if (n < 1 || n > MAX_CYCLE_STATES || P->rhs[n] != NT_BASE + P->lhs) continue;
        for (int vn = 0; vn < n_states; vn++) {
            int found = 0;
            for (int k = 0; k < states[vn].n && !found; k++)
                found = states[vn].it[k].prod == p && states[vn].it[k].dot == n;
            if (!found) continue;
            int path[MAX_CYCLE_STATES], v = vn;
            for (int i = 0; i < n && v >= 0; i++) { v = delta[(size_t)v * n_sym + P->rhs[i]]; path[i] = v; }
            if (v != vn) continue;
            const itemset_t *V1 = &states[path[0]];
            if (delta[(size_t)vn * n_sym + NT_BASE + P->lhs] < 0) continue;
            int ok = 1;
            for (int k = 0; k < V1->n && ok; k++) {
                item_t x = V1->it[k];
                if (x.dot == 0) continue;                              /* closure item */
                ok = G->prod[x.prod].lhs == P->lhs && x.dot == 1;
            }
            if (!ok) continue;
            /* insert in order, skipping a duplicate */
            int at = 0, dup = 0;
            while (at < G->n_cycles) {
                int c = cycle_cmp(G->cyc_state + G->cyc_off[at], G->cyc_len[at], path, n);
                if (c == 0) dup = 1;
                if (c >= 0) break;
                at++;
            }
            if (dup) continue;
            if (G->n_cycles == cap) {
                cap *= 2;
                G->cyc_len = (int *)realloc(G->cyc_len, sizeof(int) * (size_t)cap);
                G->cyc_off = (int *)realloc(G->cyc_off, sizeof(int) * (size_t)cap);
                G->cyc_state = (int *)realloc(G->cyc_state, sizeof(int) * (size_t)cap * MAX_CYCLE_STATES);
            }
            for (int k = G->n_cycles; k > at; k--) { G->cyc_len[k] = G->cyc_len[k - 1]; G->cyc_off[k] = G->cyc_off[k - 1]; }
            G->cyc_len[at] = n;
            G->cyc_off[at] = total;
            memcpy(G->cyc_state + total, path, sizeof(int) * (size_t)n);
            total += n;
            G->n_cycles++;
        }
    }
}

static int build_tables(grammar_t *G, char *err, int errlen) {
    first_t F;
    compute_first(G, &F);
    closure_ctx_t C;
    C.G = G;
    C.F = &F;
    C.prod_off = (int *)malloc(sizeof(int) * (size_t)G->n_prod);
    int n_dotted = 0;
    for (int p = 0; p < G->n_prod; p++) { C.prod_off[p] = n_dotted; n_dotted += G->prod[p].len + 1; }
    C.seen = (uint8_t *)calloc((size_t)n_dotted * N_TERM, 1);

    int cap = 64, n = 0;
    itemset_t *states = (itemset_t *)calloc((size_t)cap, sizeof(itemset_t));
    uint64_t *hashes = (uint64_t *)malloc(sizeof(uint64_t) * (size_t)cap);
    /* transitions recorded as they are found: delta[s][X] with X a symbol code */
    int n_sym = NT_BASE + G->n_nt;
    int *delta = (int *)malloc(sizeof(int) * (size_t)cap * (size_t)n_sym);

    item_t start = {0, 0, T_END};
    iset_push(&states[0], start);
    closure(&C, &states[0]);
    hashes[0] = set_hash(&states[0]);
    n = 1;

    itemset_t J = {0, 0, 0};
    uint8_t *after_dot = (uint8_t *)malloc((size_t)n_sym);
    for (int i = 0; i < n; i++) {             /* queue = states in discovery order */
        for (int X = 0; X < n_sym; X++) delta[(size_t)i * n_sym + X] = -1;
        memset(after_dot, 0, (size_t)n_sym);
        for (int k = 0; k < states[i].n; k++) {
            item_t x = states[i].it[k];
            const prod_t *P = &G->prod[x.prod];
            if (x.dot < P->len) after_dot[P->rhs[x.dot]] = 1;
        }
        /* terminals in ascending byte order, then nonterminals by index */
        for (int X = 0; X < n_sym; X++) {
            if (!after_dot[X]) continue;      /* GOTO(I, X) is empty */
            goto_set(&C, &states[i], X, &J);
            uint64_t h = set_hash(&J);
            int j = -1;
            for (int k = 0; k < n; k++)
                if (hashes[k] == h && same_set(&states[k], &J)) { j = k; break; }
            if (j < 0) {
                if (n == cap) {
                    cap *= 2;
                    states = (itemset_t *)realloc(states, sizeof(itemset_t) * (size_t)cap);
                    memset(states + n, 0, sizeof(itemset_t) * (size_t)(cap - n));
                    hashes = (uint64_t *)realloc(hashes, sizeof(uint64_t) * (size_t)cap);
                    delta = (int *)realloc(delta, sizeof(int) * (size_t)cap * (size_t)n_sym);
                }
                j = n++;
                states[j].n = 0;
                for (int k = 0; k < J.n; k++) iset_push(&states[j], J.it[k]);
                hashes[j] = h;
            }
            delta[(size_t)i * n_sym + X] = j;
        }
    }

    G->n_states = n;
    G->act_kind = (uint8_t *)calloc((size_t)n * N_TERM, 1);
    G->act_arg = (int *)calloc((size_t)n * N_TERM, sizeof(int));
    G->go = (int *)malloc(sizeof(int) * (size_t)n * (size_t)G->n_nt);
    G->n_items = (int *)malloc(sizeof(int) * (size_t)n);
    int rc = 0;
    for (int s = 0; s < n && rc == 0; s++) {
        G->n_items[s] = states[s].n;
        for (int A = 0; A < G->n_nt; A++)
            G->go[(size_t)s * G->n_nt + A] = delta[(size_t)s * n_sym + NT_BASE + A];
        for (int k = 0; k < states[s].n && rc == 0; k++) {
            item_t x = states[s].it[k];
            const prod_t *P = &G->prod[x.prod];
            if (x.dot < P->len) {
                int X = P->rhs[x.dot];
                if (X < NT_BASE)
                    rc = set_action(G, s, X, A_SHIFT, delta[(size_t)s * n_sym + X], err, errlen);
            } else if (x.prod == 0) {
                rc = set_action(G, s, x.la, A_ACCEPT, 0, err, errlen);   /* [S' -> S., $] */
            } else {
                rc = set_action(G, s, x.la, A_REDUCE, x.prod, err, errlen);
            }
        }
    }

    if (rc == 0) find_cycles(G, states, n, delta, n_sym);
    for (int i = 0; i < cap; i++) free(states[i].it);
    free(states); free(hashes); free(delta); free(J.it); free(after_dot);
    free(C.prod_off); free(C.seen); free(F.nullable); free(F.first);
    return rc;
}

static void free_grammar(grammar_t *G) {
    if (!G) return;
    for (int i = 0; i < G->n_nt; i++) free(G->nt_name[i]);
    free(G->nt_name);
    for (int p = 0; p < G->n_prod; p++) free(G->prod[p].rhs);
    free(G->prod);
    free(G->act_kind); free(G->act_arg); free(G->go); free(G->n_items);
    free(G->cyc_len); free(G->cyc_off); free(G->cyc_state);
    free(G);
}

/* ------------------------------------------------------------ public: build */

void pre3o_free(oracle_t *O) {
    if (!O) return;
    for (int i = 0; i < O->n_grammars; i++) free_grammar(O->g[i]);
    free(O->g);
    free(O->offset);
    free(O);
}

oracle_t *pre3o_build(const char *const *texts, int n_grammars, char *err, int errlen) {
    if (err && errlen > 0) err[0] = 0;
    if (n_grammars <= 0) { set_err(err, errlen, "no grammar given"); return NULL; }
    oracle_t *O = (oracle_t *)calloc(1, sizeof(oracle_t));
    O->g = (grammar_t **)calloc((size_t)n_grammars, sizeof(grammar_t *));
    O->offset = (int *)calloc((size_t)n_grammars + 1, sizeof(int));
    for (int i = 0; i < n_grammars; i++) {
        grammar_t *G = (grammar_t *)calloc(1, sizeof(grammar_t));
        O->g[i] = G;
        O->n_grammars = i + 1;
        if (parse_grammar(texts[i], G, err, errlen) != 0 || check_reduced(G, err, errlen) != 0 ||
            build_tables(G, err, errlen) != 0) {
            pre3o_free(O);
            return NULL;
        }
        O->offset[i + 1] = O->offset[i] + G->n_states;
    }
    return O;
}

/* ---------------------------------------------------------- public: queries */

int pre3o_n_grammars(const oracle_t *O) { return O->n_grammars; }
int pre3o_n_states(const oracle_t *O, int g) { return O->g[g]->n_states; }
int pre3o_n_states_total(const oracle_t *O) { return O->offset[O->n_grammars]; }
int pre3o_n_productions(const oracle_t *O, int g) { return O->g[g]->n_prod; }
int pre3o_n_nonterminals(const oracle_t *O, int g) { return O->g[g]->n_nt; }
int pre3o_initial_state(const oracle_t *O, int g) { return O->offset[g]; }
int pre3o_n_items(const oracle_t *O, int g, int s) { return O->g[g]->n_items[s]; }
int pre3o_production_lhs(const oracle_t *O, int g, int p) { return O->g[g]->prod[p].lhs; }
int pre3o_production_len(const oracle_t *O, int g, int p) { return O->g[g]->prod[p].len; }
const char *pre3o_nonterminal_name(const oracle_t *O, int g, int a) { return O->g[g]->nt_name[a]; }
/* ACTION[s][a] with local state ids: kind in the return value, argument in *arg */
int pre3o_action(const oracle_t *O, int g, int s, int a, int *arg) {
    const grammar_t *G = O->g[g];
    *arg = G->act_arg[(size_t)s * N_TERM + (size_t)a];
    return G->act_kind[(size_t)s * N_TERM + (size_t)a];
}
int pre3o_goto(const oracle_t *O, int g, int s, int A) {
    return O->g[g]->go[(size_t)s * O->g[g]->n_nt + A];
}

/* grammar that owns global state id s, or -1 */
static int grammar_of(const oracle_t *O, int s) {
    for (int g = 0; g < O->n_grammars; g++)
        if (s >= O->offset[g] && s < O->offset[g + 1]) return g;
    return -1;
}

/* ------------------------------------------------- the stack-based parse loop
 * One lookahead symbol `a` against the work stack `st` (global state ids, *len live
 * entries, capacity cap): reductions until the symbol is shifted.
 * Returns 0 shifted (or, for a = '$', accepted), 1 Error action, 2 stack overflow. */
static int feed(const oracle_t *O, int g, int *st, int *len, int cap, int a) {
    const grammar_t *G = O->g[g];
    int off = O->offset[g];
    for (;;) {
        int top = st[*len - 1] - off;
        size_t c = (size_t)top * N_TERM + (size_t)a;
        int kind = G->act_kind[c], arg = G->act_arg[c];
        if (kind == A_ERROR) return 1;
        if (kind == A_ACCEPT) return 0;
        if (kind == A_SHIFT) {
            if (*len >= cap) return 2;
            st[(*len)++] = arg + off;
            return 0;
        }
        /* reduce A -> beta: pop |beta| states, push GOTO[exposed state][A].
           Capacity is checked before anything changes, so the caller may enlarge
           the stack and call again with the same lookahead. */
        const prod_t *P = &G->prod[arg];
        if (*len - P->len >= cap) return 2;
        *len -= P->len;
        int exposed = st[*len - 1] - off;
        st[(*len)++] = G->go[(size_t)exposed * G->n_nt + P->lhs] + off;
    }
}

/* Is the byte string allowed after `stack`?  Works on a copy; no reduction after
 * the last byte.  An empty string is never allowed. */
int pre3o_allowed(const oracle_t *O, const int32_t *stack, int len, const uint8_t *bytes, int n) {
    if (n <= 0 || len <= 0) return 0;
    int g = grammar_of(O, stack[0]);
    if (g < 0) return 0;
    int cap = len + 64;                  /* private work copy, enlarged on demand */
    int *st = (int *)malloc(sizeof(int) * (size_t)cap);
    for (int i = 0; i < len; i++) st[i] = stack[i];
    int ok = 1;
    for (int i = 0; i < n && ok; i++) {
        int r;
        while ((r = feed(O, g, st, &len, cap, bytes[i])) == 2) {
            cap *= 2;
            st = (int *)realloc(st, sizeof(int) * (size_t)cap);
        }
        if (r == 1) ok = 0;
    }
    free(st);
    return ok;
}

/* Is the end-of-sequence token allowed, i.e. is the emitted text a sentence? */
int pre3o_eos_allowed(const oracle_t *O, const int32_t *stack, int len) {
    if (len <= 0) return 0;
    int g = grammar_of(O, stack[0]);
    if (g < 0) return 0;
    int cap = len + 64;
    int *st = (int *)malloc(sizeof(int) * (size_t)cap);
    for (int i = 0; i < len; i++) st[i] = stack[i];
    int r;
    while ((r = feed(O, g, st, &len, cap, T_END)) == 2) {
        cap *= 2;
        st = (int *)realloc(st, sizeof(int) * (size_t)cap);
    }
    free(st);
    return r == 0;
}

/* Advance the real stack by a token.  0 ok; 1 token not allowed; 2 the stack would
 * exceed `cap` entries at some point of the walk.  On 1 and 2 the stack is unchanged. */
int pre3o_advance(const oracle_t *O, int32_t *stack, int32_t *len, int cap, const uint8_t *bytes,
                  int n) {
    if (n <= 0 || *len <= 0) return 1;
    int g = grammar_of(O, stack[0]);
    if (g < 0) return 1;
    int *st = (int *)malloc(sizeof(int) * (size_t)cap);
    int l = *len;
    for (int i = 0; i < l; i++) st[i] = stack[i];
    int r = 0;
    for (int i = 0; i < n && r == 0; i++) r = feed(O, g, st, &l, cap, bytes[i]);
    if (r == 0) {
        for (int i = 0; i < l; i++) stack[i] = st[i];
        *len = l;
    }
    free(st);
    return r;
}

/* ------------------------------------------------------- batched mask / apply
 * Vocabulary: token t = bytes[offsets[t] .. offsets[t+1]); eos_id's bytes are ignored.
 * Sequence b: stack row data[b*cap .. b*cap+len[b]), states[b] = top state or -1 when
 * the sequence has finished (then only the end-of-sequence bit is set).
 * Bit (t mod 32) of word (t div 32) of row b, least significant bit first; padding 0. */

void pre3o_mask_row(const oracle_t *O, const int32_t *stack, int len, int done, const uint8_t *bytes,
                    const int64_t *offsets, int n_tokens, int eos_id, uint32_t *row) {
    int W = (n_tokens + 31) / 32;
    memset(row, 0, sizeof(uint32_t) * (size_t)W);
    for (int t = 0; t < n_tokens; t++) {
        int ok;
        if (t == eos_id) ok = done ? 1 : pre3o_eos_allowed(O, stack, len);
        else if (done) ok = 0;
        else ok = pre3o_allowed(O, stack, len, bytes + offsets[t], (int)(offsets[t + 1] - offsets[t]));
        if (ok) row[t >> 5] |= 1u << (t & 31);
    }
}

void pre3o_fill_mask(const oracle_t *O, const int32_t *states, const int32_t *data,
                     const int32_t *len, int cap, int batch, const uint8_t *bytes,
                     const int64_t *offsets, int n_tokens, int eos_id, uint32_t *bitmask) {
    int W = (n_tokens + 31) / 32;
    /* plain threads over (sequence, 32-token word): every word has one owner */
#pragma omp parallel for collapse(2) schedule(dynamic, 64)
    for (int b = 0; b < batch; b++) {
        for (int w = 0; w < W; w++) {
            const int32_t *stack = data + (size_t)b * cap;
            int done = states[b] < 0;
            uint32_t word = 0;
            for (int i = 0; i < 32; i++) {
                int t = w * 32 + i;
                if (t >= n_tokens) break;
                int ok;
                if (t == eos_id) ok = done ? 1 : pre3o_eos_allowed(O, stack, len[b]);
                else if (done) ok = 0;
                else ok = pre3o_allowed(O, stack, len[b], bytes + offsets[t],
                                        (int)(offsets[t + 1] - offsets[t]));
                if (ok) word |= 1u << i;
            }
            bitmask[(size_t)b * W + w] = word;
        }
    }
}

/* Which of `n` given token ids are allowed after one stack (no EOS handling here). */
void pre3o_allowed_many(const oracle_t *O, const int32_t *stack, int len, const uint8_t *bytes,
                        const int64_t *offsets, const int32_t *ids, int n, uint8_t *out) {
    for (int i = 0; i < n; i++) {
        int t = ids[i];
        out[i] = (uint8_t)pre3o_allowed(O, stack, len, bytes + offsets[t],
                                        (int)(offsets[t + 1] - offsets[t]));
    }
}

/* logits[b][t] keeps its bf16 bit pattern where bit t of row b is 1 and becomes
 * -inf (0xFF80) where it is 0 (Sec. 1: the mask removes the token's probability). */
void pre3o_apply_mask(uint16_t *logits, const uint32_t *bitmask, int batch, int n_tokens,
                      int64_t row_stride) {
    int W = (n_tokens + 31) / 32;
    for (int b = 0; b < batch; b++)
        for (int t = 0; t < n_tokens; t++)
            if (!((bitmask[(size_t)b * W + (t >> 5)] >> (t & 31)) & 1u))
                logits[(size_t)b * (size_t)row_stride + (size_t)t] = 0xFF80;
}

/* Greedy choice among the allowed tokens (Sec. 1: the mask removes the invalid tokens before
 * a token is sampled; the greedy sampler takes the most probable of what is left):
 * out[b] = the allowed token whose bf16 logit is largest as a number; among equal values
 * (+0 and -0 are equal) the smallest id; NaN logits are never chosen; -1 if no token is both
 * allowed and not NaN.  The logits are not modified. */
void pre3o_masked_argmax(const uint16_t *logits, const uint32_t *bitmask, int batch, int n_tokens,
                         int64_t row_stride, int32_t *out) {
    int W = (n_tokens + 31) / 32;
    for (int b = 0; b < batch; b++) {
        int best = -1;
        float best_value = 0.0f;
        for (int t = 0; t < n_tokens; t++) {
            if (!((bitmask[(size_t)b * W + (t >> 5)] >> (t & 31)) & 1u)) continue;
            uint32_t bits = (uint32_t)logits[(size_t)b * (size_t)row_stride + (size_t)t] << 16;
            float value;                      /* a bf16 number is the upper half of a binary32 */
            memcpy(&value, &bits, sizeof value);
            if (value != value) continue;     /* NaN */
            if (best < 0 || value > best_value) { best = t; best_value = value; }
        }
        out[b] = best;
    }
}

/* Top-k behind the mask (Sec. 1: invalid tokens are excluded, then a token is sampled; a top-k
 * sampler draws among the k most probable of what is left): for every row the allowed,
 * non-NaN tokens ordered by logit as a number, largest first, equal values (+0 = -0) by
 * ascending id; the first k of them.  out_ids[b][j] = token id, out_vals[b][j] = its bf16
 * pattern as stored; rows with fewer than k candidates are padded with id -1 and 0xFF80.
 * Written as the definition: collect the candidates, sort them, cut. */
typedef struct { float value; int32_t id; } cand_t;

static int cand_cmp(const void *pa, const void *pb) {
    const cand_t *a = (const cand_t *)pa, *b = (const cand_t *)pb;
    if (a->value > b->value) return -1;
    if (a->value < b->value) return 1;
    return a->id < b->id ? -1 : (a->id > b->id ? 1 : 0);
}

void pre3o_masked_topk(const uint16_t *logits, const uint32_t *bitmask, int batch, int n_tokens,
                       int64_t row_stride, int k, int32_t *out_ids, uint16_t *out_vals) {
    int W = (n_tokens + 31) / 32;
#pragma omp parallel
    {
        cand_t *c = (cand_t *)malloc(sizeof(cand_t) * (size_t)(n_tokens > 0 ? n_tokens : 1));
#pragma omp for schedule(dynamic, 1)
        for (int b = 0; b < batch; b++) {
            const uint16_t *row = logits + (size_t)b * (size_t)row_stride;
            int n = 0;
            for (int t = 0; t < n_tokens; t++) {
                if (!((bitmask[(size_t)b * W + (t >> 5)] >> (t & 31)) & 1u)) continue;
                uint32_t bits = (uint32_t)row[t] << 16;
                float value;
                memcpy(&value, &bits, sizeof value);
                if (value != value) continue;     /* NaN */
                c[n].value = value;
                c[n].id = t;
                n++;
            }
            qsort(c, (size_t)n, sizeof(cand_t), cand_cmp);
            for (int j = 0; j < k; j++) {
                out_ids[(size_t)b * k + j] = j < n ? c[j].id : -1;
                out_vals[(size_t)b * k + j] = j < n ? row[c[j].id] : 0xFF80;
            }
        }
        free(c);
    }
}

/* Jump-forward (Sec. 3.3: runs of edges with a single successor can be merged into one jump):
 * the bytes every continuation of the text must start with.  While the text is not a sentence
 * (the end-of-sequence token is not allowed) and exactly ONE of the 256 bytes keeps it a viable
 * prefix, that byte is forced: it is appended to out[] and the stack is advanced by it.  Stops
 * at the first position with no or several viable bytes, where EOS is allowed, after max_bytes
 * bytes, or before a byte whose walk would exceed cap.  Returns the number of forced bytes;
 * stack / *len hold the advanced stack. */
int pre3o_jump_forward(const oracle_t *O, int32_t *stack, int32_t *len, int cap, int max_bytes, uint8_t *out) {
    int n = 0;
    while (n < max_bytes) {
        if (pre3o_eos_allowed(O, stack, *len)) break;
        int viable = 0, which = -1;
        for (int c = 0; c < 256 && viable < 2; c++) {
            uint8_t byte = (uint8_t)c;
            if (pre3o_allowed(O, stack, *len, &byte, 1)) { viable++; which = c; }
        }
        if (viable != 1) break;
        uint8_t byte = (uint8_t)which;
        if (pre3o_advance(O, stack, len, cap, &byte, 1) != 0) break;
        out[n++] = byte;
    }
    return n;
}

/* The same for a batch, mirroring the device call: finished sequences (states[b] < 0) get no
 * bytes; states[b] follows the top of the advanced stack. */
void pre3o_jump_forward_batch(const oracle_t *O, int32_t *states, int32_t *data, int32_t *len, int cap, int batch,
                              int max_bytes, uint8_t *out_bytes, int32_t *out_len) {
    for (int b = 0; b < batch; b++) {
        out_len[b] = 0;
        if (states[b] < 0) continue;
        int32_t *stack = data + (size_t)b * cap;
        out_len[b] = pre3o_jump_forward(O, stack, &len[b], cap, max_bytes, out_bytes + (size_t)b * max_bytes);
        states[b] = stack[len[b] - 1];
    }
}

/* Batched advance mirroring the device call: tokens[b] < 0 skips the sequence;
 * the end-of-sequence token marks it finished (states[b] = -1, stack untouched);
 * err[b] = 1 for a token that is not allowed (also any token on a finished
 * sequence, and EOS where it is not allowed), 2 for stack overflow; a failing
 * sequence is left unchanged. */
void pre3o_advance_batch(const oracle_t *O, int32_t *states, int32_t *data, int32_t *len, int cap,
                         int batch, const int32_t *tokens, const uint8_t *bytes,
                         const int64_t *offsets, int n_tokens, int eos_id, int32_t *err) {
    for (int b = 0; b < batch; b++) {
        int t = tokens[b];
        err[b] = 0;
        if (t < 0) continue;
        int32_t *stack = data + (size_t)b * cap;
        if (t >= n_tokens || states[b] < 0) { err[b] = 1; continue; }
        if (t == eos_id) {
            if (pre3o_eos_allowed(O, stack, len[b])) states[b] = -1;
            else err[b] = 1;
            continue;
        }
        int r = pre3o_advance(O, stack, &len[b], cap, bytes + offsets[t],
                              (int)(offsets[t + 1] - offsets[t]));
        if (r != 0) { err[b] = r; continue; }
        states[b] = stack[len[b] - 1];
    }
}

/* ----------------------------------------------------- cycle-aware stacks */

int pre3o_n_cycles(const oracle_t *O, int g) { return O->g[g]->n_cycles; }

/* Copies the states (local ids) of cycle k of grammar g to out; returns their number. */
int pre3o_cycle(const oracle_t *O, int g, int k, int32_t *out) {
    const grammar_t *G = O->g[g];
    for (int i = 0; i < G->cyc_len[k]; i++) out[i] = G->cyc_state[G->cyc_off[k] + i];
    return G->cyc_len[k];
}

/* The stack in normal form (Sec. 3.2.3: the stack never keeps a complete traversal of a
 * cycle under the state that starts the next one).  The stack is rebuilt from the bottom, one
 * push at a time; after a push of v1, while the entries under it spell v1 .. vn of a cycle that
 * starts with v1 (cycles tried in their stored order, from the first again after a match), those
 * n entries are popped and v1 pushed back -- the modified back-edge of Alg. 1 step 1.
 * Returns the new length. */
int pre3o_compact(const oracle_t *O, int32_t *stack, int len) {
    if (len < 1) return len;
    int g = grammar_of(O, stack[0]);
    if (g < 0) return len;
    const grammar_t *G = O->g[g];
    int off = O->offset[g], w = 0;
    for (int r = 0; r < len; r++) {
        int32_t x = stack[r];
        stack[w++] = x;                                  /* push */
        int k = 0;
        while (k < G->n_cycles) {
            const int *c = G->cyc_state + G->cyc_off[k];
            int n = G->cyc_len[k], match = c[0] + off == x && w - 1 - n >= 0;
            for (int i = 0; match && i < n; i++) match = stack[w - 1 - n + i] == c[i] + off;
            if (match) { w -= n; k = 0; }                /* pop v1..vn and the top, push v1 */
            else k++;
        }
    }
    return w;
}

/* Normal form of every stack of a batch (finished sequences included: their stacks are kept). */
void pre3o_compact_batch(const oracle_t *O, int32_t *data, int32_t *len, int cap, int batch) {
    for (int b = 0; b < batch; b++)
        if (len[b] >= 1 && len[b] <= cap) len[b] = pre3o_compact(O, data + (size_t)b * cap, len[b]);
}

"""An LR-free recogniser for tiny context-free grammars, used to pin the oracle.

For every nonterminal A it computes, by fixpoint iteration over *sets of strings*,
  L[A] = { w : A =>* w, |w| <= N }            (sentences of A up to length N)
  P[A] = { w : w is a prefix of some string derived from A, |w| <= N }
straight from the productions: L of a right-hand side is the concatenation of the L sets
of its symbols (truncated at N); a prefix of X1..Xk is a sentence of X1..X(m-1) followed
by a prefix of Xm (every nonterminal derives some string, so the rest can always be
completed).  Nothing here knows about items, states, lookaheads or stacks.
"""
import re


def parse_tiny(text):
    """Productions of a grammar text that uses only Names and quoted strings (no classes,
    no escapes).  Returns (start, {A: [rhs, ...]}) with rhs a list of ('t', char)/('n', name)."""
    prods, start = {}, None
    for line in text.strip().splitlines():
        line = line.strip()
        if not line:
            continue
        lhs, rhs = line.split("::=")
        lhs = lhs.strip()
        start = start or lhs
        for alt in rhs.split("|"):
            syms = []
            for m in re.finditer(r'"([^"]*)"|([A-Za-z_][A-Za-z0-9_]*)', alt):
                if m.group(2):
                    syms.append(("n", m.group(2)))
                else:
                    syms.extend(("t", c) for c in m.group(1))
            prods.setdefault(lhs, []).append(syms)
    return start, prods


def _cat(a, b, n):
    return {x + y for x in a for y in b if len(x) + len(y) <= n}


def languages(text, n):
    start, prods = parse_tiny(text)
    L = {A: set() for A in prods}
    changed = True
    while changed:
        changed = False
        for A, alts in prods.items():
            for rhs in alts:
                cur = {""}
                for kind, x in rhs:
                    cur = _cat(cur, {x} if kind == "t" else L[x], n)
                    if not cur:
                        break
                if not cur <= L[A]:
                    L[A] |= cur
                    changed = True
    P = {A: {""} for A in prods}
    changed = True
    while changed:
        changed = False
        for A, alts in prods.items():
            for rhs in alts:
                head = {""}                      # sentences of X1..X(m-1)
                for kind, x in rhs:
                    pre = {"", x} if kind == "t" else P[x]
                    new = _cat(head, pre, n)
                    if not new <= P[A]:
                        P[A] |= new
                        changed = True
                    head = _cat(head, {x} if kind == "t" else L[x], n)
                    if not head:
                        break
    return L[start], P[start]

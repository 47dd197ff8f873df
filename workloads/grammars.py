"""Grammar texts of the synthetic workloads (inputs only: no automaton arithmetic here).

Text format, understood independently by the CPU oracle and by the GPU library:
  Name ::= alt | alt ...      a following line that starts with '|' continues the rule
  alt  = sequence of Names and "quoted byte strings" ("" is the empty string)
       | [class]              a byte class must be a whole alternative
  escapes in "..." and [...]: \\n \\r \\t \\\\ \\" \\] \\- \\^ \\[ \\xHH ; '#' starts a comment.
The first rule is the start symbol.  Terminals are single bytes.
"""
from __future__ import annotations

import numpy as np

# E -> E+T | T, T -> T*F | F, F -> (E) | a   over the alphabet {a,+,*,(,)}
ARITHMETIC = r'''
E ::= E "+" T | T
T ::= T "*" F | F
F ::= "(" E ")" | "a"
'''

# Byte-level JSON in the shape of RFC 8259.  Optional white space is attached after
# every value and after every separator (and once at the start) so that one byte of
# lookahead always decides; lists are left-recursive; numbers end by lookahead.
_JSON_VALUE_RULES = r'''
object   ::= "{" ws "}" | "{" ws members "}"
members  ::= member | members "," ws member
member   ::= string ws ":" ws value
array    ::= "[" ws "]" | "[" ws elements "]"
elements ::= value | elements "," ws value
'''

_JSON_LEXICAL_RULES = r'''
string   ::= "\"" chars "\""
chars    ::= "" | chars char
char     ::= plain | "\\" escape
plain    ::= [^"\\\x00-\x1f]
escape   ::= simple | "u" hex hex hex hex
simple   ::= ["\\/bfnrt]
hex      ::= [0-9a-fA-F]
number   ::= sign int frac exp
sign     ::= "" | "-"
int      ::= "0" | onenine | onenine digits
digits   ::= digit | digits digit
digit    ::= [0-9]
onenine  ::= [1-9]
frac     ::= "" | "." digits
exp      ::= "" | e esign digits
e        ::= [eE]
esign    ::= "" | [+\-]
ws       ::= "" | ws wsc
wsc      ::= [ \t\n\r]
'''

JSON = (
    r'''
json     ::= ws value
value    ::= object ws | array ws | string ws | number ws | "true" ws | "false" ws | "null" ws
'''
    + _JSON_VALUE_RULES
    + _JSON_LEXICAL_RULES
)

# Free text, then JSON: one to three lines of unconstrained text (any byte from 0x20 up), each
# opened by a space and closed by a line feed, then the answer as a JSON value.  After a line
# feed one byte decides: a space opens another line, "A" opens the answer.
THOUGHT_THEN_JSON = (
    r'''
doc      ::= "Thought:" lines "Answer: " value
lines    ::= line | line line | line line line
line     ::= " " text "\n"
text     ::= tchar | text tchar
tchar    ::= [^\x00-\x1f]
value    ::= object ws | array ws | string ws | number ws | "true" ws | "false" ws | "null" ws
'''
    + _JSON_VALUE_RULES
    + _JSON_LEXICAL_RULES
)
THOUGHT_THEN_JSON_MARKER = b"\nA"      # the first bytes that cannot belong to the free text

# The same JSON language with every list written right-recursively (members, elements, string
# characters, digits, white space): the LR stack then grows with the length of each list until
# the list ends -- the shape that the cycle-aware stacks of Sec. 3.2.3 are for.
JSON_RIGHT_RECURSIVE = r'''
json     ::= ws value
value    ::= object ws | array ws | string ws | number ws | "true" ws | "false" ws | "null" ws
object   ::= "{" ws "}" | "{" ws members "}"
members  ::= member | member "," ws members
member   ::= string ws ":" ws value
array    ::= "[" ws "]" | "[" ws elements "]"
elements ::= value | value "," ws elements
string   ::= "\"" chars "\""
chars    ::= "" | char chars
char     ::= plain | "\\" escape
plain    ::= [^"\\\x00-\x1f]
escape   ::= simple | "u" hex hex hex hex
simple   ::= ["\\/bfnrt]
hex      ::= [0-9a-fA-F]
number   ::= sign int frac exp
sign     ::= "" | "-"
int      ::= "0" | onenine | onenine digits
digits   ::= digit | digit digits
digit    ::= [0-9]
onenine  ::= [1-9]
frac     ::= "" | "." digits
exp      ::= "" | e esign digits
e        ::= [eE]
esign    ::= "" | [+\-]
ws       ::= "" | wsc ws
wsc      ::= [ \t\n\r]
'''

# Small grammars used by the oracle's pins.
DRAGON_CC = r'''
S ::= C C
C ::= "c" C | "d"
'''
DYCK = r'''
S ::= "" | S "(" S ")"
'''
ANBN = r'''
S ::= "a" S "b" | "a" "b"
'''
RIGHT_LIST = r'''
L ::= "x" | "x" "," L
'''
EPSILON_MIX = r'''
S ::= A B "c"
A ::= "" | "a" A
B ::= "" | "b"
'''
# right-linear: (ab|c)*d
RIGHT_LINEAR = r'''
S ::= "a" T | "c" S | "d"
T ::= "b" S
'''
AMBIGUOUS = r'''
E ::= E "+" E | "a"
'''
PALINDROME = r'''
S ::= "a" S "a" | "b" S "b" | ""
'''


def _ident(rng: np.random.Generator, lo=3, hi=10) -> str:
    n = int(rng.integers(lo, hi + 1))
    return "".join(chr(ord("a") + int(c)) for c in rng.integers(0, 26, size=n))


def _unique_idents(rng, k, first_letters=None):
    """k lowercase identifiers with pairwise distinct first letters when k <= 26, so that
    one byte of lookahead separates alternatives that start with them."""
    out, used = [], set()
    while len(out) < k:
        s = _ident(rng)
        key = s[0] if k <= 26 else s
        if key in used or s in out:
            continue
        used.add(key)
        out.append(s)
    return out


class SchemaGrammar:
    """A JSON-schema-like grammar: objects with fixed keys in fixed order and typed values."""

    def __init__(self, text: str, n_alternatives: int, description: dict):
        self.text = text
        self.n_alternatives = n_alternatives      # productions as written (a class counts once)
        self.description = description


def schema_grammar(seed: int, n_keys: int = 12, depth: int = 3, n_enum: int = 8,
                   extra_objects: int = 0) -> SchemaGrammar:
    """Seeded synthetic schema: `n_keys` fixed keys at the top level with value types cycling
    through int, float, enum of `n_enum` strings, bool, free string, nested object
    (`depth` levels deep) and array of objects; `extra_objects` adds further sibling object
    types (each with its own keys and enums) to scale the number of productions."""
    rng = np.random.default_rng(seed)
    rules = []
    counter = {"obj": 0, "enum": 0, "arr": 0}
    n_alt = 0

    def new_enum():
        counter["enum"] += 1
        name = f"enum{counter['enum']}"
        members = _unique_idents(rng, n_enum)
        alts = " | ".join('"\\"%s\\""' % m for m in members)
        rules.append(f"{name} ::= {alts}")
        return name, len(members)

    def new_object(level: int, keys: int):
        nonlocal n_alt
        counter["obj"] += 1
        name = f"obj{counter['obj']}"
        kinds = ["int", "float", "enum", "bool", "str"]
        if level < depth:
            kinds.append("obj")
        if level < depth:
            kinds.append("arr")
        key_names = _unique_idents(rng, keys)
        parts = []
        for i, k in enumerate(key_names):
            kind = kinds[i % len(kinds)]
            if kind == "int":
                v = "intv"
            elif kind == "float":
                v = "number"
            elif kind == "enum":
                v, c = new_enum()
                n_alt += c
            elif kind == "bool":
                v = "boolv"
            elif kind == "str":
                v = "string"
            elif kind == "obj":
                v = new_object(level + 1, max(3, keys // 2))
            else:
                inner = new_object(level + 1, max(2, keys // 3))
                counter["arr"] += 1
                v = f"arr{counter['arr']}"
                rules.append(f'{v} ::= "[" ws "]" | "[" ws items{counter["arr"]} "]"')
                rules.append(f'items{counter["arr"]} ::= {inner} ws | items{counter["arr"]} "," ws {inner} ws')
                n_alt += 4
            kv = f"{name}_kv{i}"
            rules.append(f'{kv} ::= "\\"{k}\\"" ws ":" ws {v} ws')
            n_alt += 1
            parts.append(kv)
        body = ' "," ws '.join(parts)
        rules.append(f'{name} ::= "{{" ws {body} "}}"')
        n_alt += 1
        return name

    top = new_object(1, n_keys)
    extras = [new_object(2, max(3, n_keys // 2)) for _ in range(extra_objects)]
    head = [f"root ::= ws {top} ws" if not extras else "root ::= ws rootv ws"]
    n_alt += 1
    if extras:
        # a top-level array-free choice would need distinct first bytes; wrap the extra object
        # types as further keys of a synthetic outer object instead
        outer_keys = _unique_idents(rng, len(extras) + 1)
        parts = []
        for i, (k, o) in enumerate(zip(outer_keys, [top] + extras)):
            kv = f"rootv_kv{i}"
            rules.append(f'{kv} ::= "\\"{k}\\"" ws ":" ws {o} ws')
            parts.append(kv)
            n_alt += 1
        rules.append('rootv ::= "{" ws ' + ' "," ws '.join(parts) + ' "}"')
        n_alt += 1
    shared = r'''
intv     ::= sign int
boolv    ::= "true" | "false"
''' + _JSON_LEXICAL_RULES
    # alternatives as written in the shared part: intv 1, boolv 2, lexical 30
    n_alt += 3 + 30
    text = "\n".join(head + rules) + "\n" + shared
    return SchemaGrammar(text, n_alt, dict(seed=seed, n_keys=n_keys, depth=depth, n_enum=n_enum,
                                           extra_objects=extra_objects, objects=counter["obj"],
                                           enums=counter["enum"], arrays=counter["arr"]))

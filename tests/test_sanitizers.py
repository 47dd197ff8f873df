"""The library's host compile path (grammar.cpp, lr1.cpp, tables.cpp, symbol_edges.cpp,
token_edges.cpp) and the C oracle, each built into a CPU-only program with AddressSanitizer and
UndefinedBehaviorSanitizer (tests/sanitize/) and run over the grammar corpus of the other CPU
tests and the compile of workload configurations 1-5.  Both programs must finish without a
sanitizer report; since they print, per stack, a hash of the mask row and of the advanced stack
computed from their own tables, the outputs are also compared line by line."""
import os
import random
import struct
import subprocess

import numpy as np
import pytest

from oracle import GrammarError, Oracle
from test_oracle_cycles import CURATED, _random_right_recursive_grammar
from test_random_grammars import _vocab as tiny_vocab, random_grammar
from workloads import configs, grammars as G, trajectory
from workloads.vocab import BASE_SEED, bpe_like_vocab

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(ROOT, "paper_2506_03887_amd", "csrc")
SAN = ["-fsanitize=address,undefined", "-fno-sanitize-recover=all", "-fno-omit-frame-pointer", "-g", "-O1", "-static-libasan"]
ENV = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0:verify_asan_link_order=0", UBSAN_OPTIONS="print_stacktrace=1")


@pytest.fixture(scope="session")
def programs(tmp_path_factory):
    out = tmp_path_factory.mktemp("sanitize")
    lib_exe, ora_exe = str(out / "host_compile_check"), str(out / "oracle_check")
    srcs = [os.path.join(CSRC, f) for f in ("grammar.cpp", "lr1.cpp", "tables.cpp", "symbol_edges.cpp", "token_edges.cpp")]
    jobs = [subprocess.Popen(["g++", "-std=c++17", "-pthread", *SAN, "-o", lib_exe, os.path.join(HERE, "sanitize", "host_compile_check.cpp"), *srcs],
                             stderr=subprocess.PIPE, text=True),
            subprocess.Popen(["gcc", *SAN, "-o", ora_exe, os.path.join(HERE, "sanitize", "oracle_check.c"),
                              os.path.join(ROOT, "oracle", "pre3_oracle.c"), "-lm"], stderr=subprocess.PIPE, text=True)]
    for j in jobs:
        err = j.communicate()[1]
        assert j.returncode == 0, err
    return lib_exe, ora_exe


def _write_case(path, grammars, vocab, stacks):
    """stacks: list of (entries, token id or -1)."""
    os.makedirs(path, exist_ok=True)
    for i, g in enumerate(grammars):
        with open(os.path.join(path, f"grammar_{i}.txt"), "wb") as f:
            f.write(g.encode("latin-1"))
    with open(os.path.join(path, "vocab.bin"), "wb") as f:
        f.write(struct.pack("<ii", vocab.n_tokens, vocab.eos_id))
        f.write(np.ascontiguousarray(vocab.offsets, dtype=np.int64).tobytes())
        f.write(np.ascontiguousarray(vocab.bytes, dtype=np.uint8).tobytes())
    with open(os.path.join(path, "stacks.bin"), "wb") as f:
        f.write(struct.pack("<i", len(stacks)))
        for st, tok in stacks:
            f.write(struct.pack("<i", len(st)))
            f.write(np.asarray(st, dtype=np.int32).tobytes())
            f.write(struct.pack("<i", int(tok)))


def _run(exe, case, *options):
    r = subprocess.run([exe, case, *options], capture_output=True, text=True, env=ENV, timeout=600)
    report = r.stderr + r.stdout
    assert r.returncode == 0 and "runtime error" not in report and "Sanitizer" not in report, \
        f"{os.path.basename(exe)} {options}: exit {r.returncode}\n{report[-3000:]}"
    assert "MISMATCH" not in r.stdout, r.stdout[-2000:]
    return r.stdout.splitlines()


def _rows(lines):
    """per stack: (mask row hash, advance status, advanced stack hash)"""
    out = []
    for l in lines:
        if l.startswith("stack "):
            w = l.split()
            out.append((w[3], w[w.index("advance") + 1], w[w.index("advance") + 2]))
    return out


def _compare(programs, case, *options):
    lib_exe, ora_exe = programs
    lib_lines, ora_lines = _run(lib_exe, case, *options), _run(ora_exe, case)
    assert _rows(lib_lines) == _rows(ora_lines) and len(_rows(ora_lines)) > 0, (case, options)
    return lib_lines[0]


def _trajectory_stacks(cfg, o, n_seq, steps):
    """Stacks (and the token taken from each) of the first sequences over the first steps of the
    configuration's seeded trajectory."""
    gi, depths = configs.sequence_setup(cfg)
    gi = gi[:n_seq]
    depths = None if depths is None else depths[:n_seq]
    traj = trajectory.generate(o, cfg.vocab, n_seq, steps, cfg.cap, cfg.seed, gi, cfg.nest_cap, None, cfg.json_strings, depths,
                               marker=cfg.marker, p_line_feed=cfg.p_line_feed)
    data, length = traj.init_data.copy(), traj.init_len.copy()
    states = data[np.arange(n_seq), length - 1].copy()
    out = []
    for s in range(steps):
        for b in np.flatnonzero(traj.reset[s]):
            data[b, 0] = o.initial_state(int(gi[b]))
            length[b], states[b] = 1, data[b, 0]
        for b in range(n_seq):
            out.append((data[b, : length[b]].copy(), traj.tokens[s][b]))
        o.advance_batch(states, data, length, traj.tokens[s], cfg.vocab)
    return out


@pytest.mark.parametrize("idx,n_seq,steps", [(1, 4, 6), (2, 6, 4), (3, 5, 3), (4, 5, 3), (5, 12, 2)])
def test_compile_of_the_workload_configurations(programs, tmp_path, idx, n_seq, steps):
    cfg = configs.get(idx)
    o = Oracle(cfg.grammars)
    case = str(tmp_path / f"cfg{idx}")
    _write_case(case, cfg.grammars, cfg.vocab, _trajectory_stacks(cfg, o, n_seq, steps))
    head = _compare(programs, case)
    assert f"states {o.n_states_total()} " in head


def test_every_merging_level_and_cycle_aware_tables(programs, tmp_path):
    cfg = configs.get(2)
    o = Oracle(cfg.grammars)
    case = str(tmp_path / "json")
    _write_case(case, cfg.grammars, cfg.vocab, _trajectory_stacks(cfg, o, 4, 3))
    for options in (["stepwise"], ["no_token_edges"], ["max_known=2"], ["max_known=1"], ["row_threshold=64"], ["row_threshold=4000"]):
        _compare(programs, case, *options)
    # right-recursive JSON, compacted stacks, tables built for them
    v = bpe_like_vocab(4000, 12, BASE_SEED + 85)
    oc = Oracle([G.JSON_RIGHT_RECURSIVE], compact_cycles=True)
    stacks = []
    for text in (b'[1,2,3,4,[5,6,"abc', b'{"k":[1,2,{"l":"x', b'[[[],[],[', b'"abcdef', b"[1 , 2 ,\n 3"):
        rc, st = oc.advance(oc.initial_stack(), text)
        assert rc == 0
        stacks.append((st, v.tokens.index(b"1")))
    case = str(tmp_path / "rr")
    _write_case(case, [G.JSON_RIGHT_RECURSIVE], v, stacks)
    head = _compare(programs, case, "compact")
    assert "cycles 20" in head
    _compare(programs, case, "compact", "max_known=3")


def test_grammar_corpus(programs, tmp_path):
    """Seeded random grammars (accepted ones: every viable prefix up to length 4 as a stack; refused ones
    must be refused by both programs), the curated right-recursive grammars and the textbook ones."""
    lib_exe, ora_exe = programs
    rnd = random.Random(2506_03887 + 21)
    v = tiny_vocab()
    texts, n_ok, n_bad = [], 0, 0
    while n_ok < 30:                                      # mostly refused: keep 30 accepted and 20 refused ones
        text = random_grammar(rnd) if len(texts) % 2 else _random_right_recursive_grammar(rnd)
        try:
            Oracle(text)
            n_ok += 1
        except GrammarError:
            n_bad += 1
            if n_bad > 20:
                continue
        texts.append(text)
    texts += list(CURATED.values()) + [G.ARITHMETIC, G.DRAGON_CC, G.DYCK, G.ANBN, G.RIGHT_LIST, G.EPSILON_MIX, G.RIGHT_LINEAR]
    texts += ['S ::= "a" S "a" | "b" S "b" | ""', 'S ::= S "+" S | "a"', 'S ::= A\nA ::= A', 'S ::= "a', "S ::= [z-a]", ""]
    accepted = refused = 0
    for i, text in enumerate(texts):
        case = str(tmp_path / f"g{i}")
        try:
            o = Oracle(text)
        except GrammarError:
            o = None
        stacks = []
        if o is not None:
            seen = set()
            frontier = [b""]
            while frontier and len(stacks) < 24:
                p = frontier.pop(0)
                rc, st = (0, o.initial_stack()) if not p else o.advance(o.initial_stack(), p)
                if rc != 0 or tuple(st) in seen:
                    continue
                seen.add(tuple(st))
                stacks.append((st, rnd.randrange(v.n_tokens - 1)))
                if len(p) < 4:
                    frontier += [p + c.encode() for c in "abc"]
        _write_case(case, [text], v, stacks)
        lib_lines, ora_lines = _run(lib_exe, case), _run(ora_exe, case)
        if o is None:
            assert lib_lines[0].startswith("compile error") and ora_lines[0].startswith("compile error"), text
            refused += 1
        else:
            assert _rows(lib_lines) == _rows(ora_lines), text
            options = [["stepwise"], ["max_known=1"], ["no_token_edges"]][i % 3]
            assert _rows(_run(lib_exe, case, *options)) == _rows(ora_lines), (text, options)
            accepted += 1
    assert accepted >= 40 and refused >= 20, (accepted, refused)

"""The C ABI without Python in the loop: tests/c_abi/check (plain C, gcc-built, HIP runtime for
device memory only) replays one step of a seeded JSON workload from a fixture holding the inputs
and the oracle's expected outputs, and must match bit for bit."""
import os
import subprocess

import numpy as np
import pytest

from oracle import Oracle, apply_mask as oracle_apply_mask, masked_argmax as oracle_masked_argmax
from workloads import grammars as G
from workloads import trajectory
from workloads.vocab import BASE_SEED, bf16_logits, bpe_like_vocab

pytestmark = pytest.mark.gpu
HERE = os.path.dirname(os.path.abspath(__file__))
BINARY = os.path.join(HERE, "c_abi", "check")


def test_plain_c_program_matches_the_oracle(tmp_path):
    if not os.path.exists(BINARY):                 # normally built beforehand with everything else; gcc, under a second
        import importlib.util
        spec = importlib.util.spec_from_file_location("c_abi_build", os.path.join(HERE, "c_abi", "build.py"))
        mod = importlib.util.module_from_spec(spec)
        spec.loader.exec_module(mod)
        mod.build()
    text = G.schema_grammar(11, 6, 2, 4).text
    v = bpe_like_vocab(5000, 12, BASE_SEED + 81)
    o = Oracle([text])
    B, cap, V, max_jump = 48, 128, v.n_tokens, 24
    drv = trajectory.Driver(o, v, B, cap, 23, None, 5, None, True)
    for _ in range(9):
        drv.step(last_step=False)
    states, data, length = drv.states.copy(), drv.data.copy(), drv.len.copy()
    rng = np.random.default_rng(4)
    mask = o.fill_mask(states, data, length, v)
    logits = bf16_logits(rng, B, V)
    masked = logits.copy()
    oracle_apply_mask(masked, mask, V)
    argmax = oracle_masked_argmax(logits, mask, V)
    tokens = argmax.copy()
    tokens[::7] = rng.integers(0, V, size=len(tokens[::7]))      # some arbitrary tokens: err paths
    tokens[3] = -1
    s1, d1, l1 = states.copy(), data.copy(), length.copy()
    err = o.advance_batch(s1, d1, l1, tokens, v)
    mask1 = o.fill_mask(s1, d1, l1, v)
    s2, d2, l2 = s1.copy(), d1.copy(), l1.copy()
    jb, jn = o.jump_forward_batch(s2, d2, l2, max_jump)
    gram = text.encode("latin-1")
    header = np.array([len(gram), len(v.bytes), V, v.eos_id, B, cap, max_jump, 0], dtype=np.int32)
    parts = [header, np.frombuffer(gram, dtype=np.uint8), np.asarray(v.bytes, dtype=np.uint8),
             np.asarray(v.offsets, dtype=np.int64), states, data, length, mask, logits, masked, argmax,
             tokens.astype(np.int32), err.astype(np.int32), s1, l1, d1, mask1,
             np.ascontiguousarray(jb, dtype=np.uint8), jn.astype(np.int32), s2, l2]
    path = tmp_path / "fixture.bin"
    with open(path, "wb") as f:
        for a in parts:
            f.write(np.ascontiguousarray(a).tobytes())
    proc = subprocess.run([BINARY, str(path)], capture_output=True, text=True, timeout=120)
    assert proc.returncode == 0 and "C ABI OK" in proc.stdout, (proc.returncode, proc.stdout, proc.stderr)
    assert int(jn.sum()) > 0 and (err != 0).any() and (err == 0).any()

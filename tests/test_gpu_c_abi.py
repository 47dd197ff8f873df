"""The C ABI without Python in the loop: tests/c_abi/check (plain C, gcc-built, HIP runtime for
device memory only) replays one step of a seeded JSON workload from a fixture holding the inputs
and the oracle's expected outputs -- call by call, then as the one-call step and the one-call greedy
step -- and must match bit for bit."""
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
    masked1 = logits.copy()
    oracle_apply_mask(masked1, mask1, V)
    argmax1 = oracle_masked_argmax(logits, mask1, V)
    gram = text.encode("latin-1")
    header = np.array([len(gram), len(v.bytes), V, v.eos_id, B, cap, max_jump, 0], dtype=np.int32)
    parts = [header, np.frombuffer(gram, dtype=np.uint8), np.asarray(v.bytes, dtype=np.uint8),
             np.asarray(v.offsets, dtype=np.int64), states, data, length, mask, logits, masked, argmax,
             tokens.astype(np.int32), err.astype(np.int32), s1, l1, d1, mask1,
             np.ascontiguousarray(jb, dtype=np.uint8), jn.astype(np.int32), s2, l2, masked1, argmax1]
    path = tmp_path / "fixture.bin"
    with open(path, "wb") as f:
        for a in parts:
            f.write(np.ascontiguousarray(a).tobytes())
    proc = subprocess.run([BINARY, str(path)], capture_output=True, text=True, timeout=120)
    assert proc.returncode == 0 and "C ABI OK" in proc.stdout, (proc.returncode, proc.stdout, proc.stderr)
    assert int(jn.sum()) > 0 and (err != 0).any() and (err == 0).any()


def test_device_timestamps_follow_stream_order_and_time_a_kernel():
    """pre3_debug_timestamp: stamps recorded around a masking launch, eagerly and inside a captured graph,
    increase in stream order, and the launch they bracket takes a plausible time (the clock runs at 100 MHz)."""
    import torch
    from paper_2506_03887_amd import apply_mask
    from paper_2506_03887_amd.binding import Pre3Error, device_timestamp, load
    dev = torch.device("cuda:0")
    B, V = 64, 32000
    W = (V + 31) // 32
    logits = torch.randn((B, V), device=dev).to(torch.bfloat16)
    mask = torch.full((B, W), 0x55555555, dtype=torch.int32, device=dev)
    stamps = torch.zeros(6, dtype=torch.int64, device=dev)

    def bracket(first):
        device_timestamp(stamps, first)
        device_timestamp(stamps, first + 1)
        apply_mask(logits, mask, V)
        device_timestamp(stamps, first + 2)

    bracket(0)
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        bracket(3)
    g.replay()
    torch.cuda.synchronize()
    t = stamps.cpu().numpy()
    assert (np.diff(t[:3]) > 0).all() and (np.diff(t[3:]) > 0).all() and t[3] > t[2], t
    for first in (0, 3):
        launch_us = ((t[first + 2] - t[first + 1]) - (t[first + 1] - t[first])) * 0.01
        assert -2.0 < launch_us < 200.0, (first, launch_us, t)
    assert load().pre3_debug_timestamp(None, None) < 0          # a null pointer is refused, nothing is launched

"""Benchmark of the batched token-mask path on one MI355X.

One step = fill_mask -> apply_mask -> advance over one batch (B=256 sequences, V=128,256
tokens, byte-level JSON grammar: workload "json-B256-V128256"), replaying a seeded
trajectory; all inputs are resident in HBM before the timed region.  Prints ONE JSON line.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

BYTES_PER_PAIR = 4.25          # algorithmic HBM bytes per (sequence, token) pair of mask+apply
HBM_PEAK_GBS = 8000.0


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=128)
    ap.add_argument("--warmup", type=int, default=16)
    ap.add_argument("--config", type=int, default=3)
    ap.add_argument("--cpu-steps", type=int, default=2, help="steps of the workload timed on the CPU oracle")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py: this path runs on one GPU (sequences are independent; see DESIGN.md on sharding); use --gpus 1")

    import numpy as np
    import torch

    from oracle import Oracle, apply_mask as oracle_apply_mask
    from paper_2506_03887_amd import Pre3, apply_mask
    from workloads import configs, trajectory
    from workloads.vocab import bf16_logits

    cfg = configs.get(args.config)
    v = cfg.vocab
    B, V, W, cap = cfg.batch, v.n_tokens, v.words, cfg.cap
    K, Wm = args.steps, args.warmup
    total = K + Wm

    # ---- inputs: oracle-driven seeded trajectory (host), then everything uploaded
    o = Oracle(cfg.grammars)
    gi, depths = configs.sequence_setup(cfg)
    traj = trajectory.generate(o, v, B, total, cap, cfg.seed, gi, cfg.nest_cap, None, cfg.json_strings, depths)
    s0 = np.array([o.initial_state(int(g)) for g in gi], dtype=np.int32)

    dev = torch.device("cuda:0")
    lib = Pre3(cfg.grammars, v.bytes, v.offsets, v.eos_id, max_token_len=max(1, v.max_len), stack_cap=cap)
    data_h, len_h = traj.init_data.copy(), traj.init_len.copy()
    states_h = data_h[np.arange(B), len_h - 1].copy()
    data_d = torch.from_numpy(data_h).to(dev)
    len_d = torch.from_numpy(len_h).to(dev)
    states_d = torch.from_numpy(states_h).to(dev)
    err_d = torch.zeros(B, dtype=torch.int32, device=dev)
    mask_d = torch.empty((B, W), dtype=torch.int32, device=dev)
    lib.bind_state(states_d, data_d, len_d, err_d)
    tokens_d = torch.from_numpy(traj.tokens).to(dev)
    reset_d = torch.from_numpy(traj.reset).to(dev)
    any_reset = traj.reset.any(axis=1)
    s0_d = torch.from_numpy(s0).to(dev)
    one_d = torch.ones(B, dtype=torch.int32, device=dev)
    n_pool = 4
    gen = torch.Generator(device=dev)
    gen.manual_seed(cfg.seed)
    logits = [torch.randn((B, V), generator=gen, device=dev, dtype=torch.float32).to(torch.bfloat16)
              for _ in range(n_pool)]

    def step(s, ev=None):
        if any_reset[s]:          # slot reuse: a finished sequence restarts (bottom of its stack is kept)
            torch.where(reset_d[s], one_d, len_d, out=len_d)
            torch.where(reset_d[s], s0_d, states_d, out=states_d)
        if ev:
            ev[0].record()
        lib.fill_mask(states_d, data_d, len_d, mask_d)
        if ev:
            ev[1].record()
        apply_mask(logits[s % n_pool], mask_d, V)
        if ev:
            ev[2].record()
        lib.advance(tokens_d[s])
        if ev:
            ev[3].record()

    for s in range(Wm):
        step(s)
    torch.cuda.synchronize()
    events = [[torch.cuda.Event(enable_timing=True) for _ in range(4)] for _ in range(K)]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for s in range(K):
        step(Wm + s, events[s])
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0

    fill_us = np.array([e[0].elapsed_time(e[1]) for e in events]) * 1e3
    apply_us = np.array([e[1].elapsed_time(e[2]) for e in events]) * 1e3
    adv_us = np.array([e[2].elapsed_time(e[3]) for e in events]) * 1e3

    # ---- the timed run must have done the real work: final state == oracle's replay
    for s in range(total):
        rs = np.flatnonzero(traj.reset[s])
        data_h[rs, 0], len_h[rs], states_h[rs] = s0[rs], 1, s0[rs]
        err = o.advance_batch(states_h, data_h, len_h, traj.tokens[s], v)
        assert not err.any()
    assert (states_d.cpu().numpy() == states_h).all() and (len_d.cpu().numpy() == len_h).all(), \
        "device state after the timed run differs from the oracle's replay"
    assert int(err_d.abs().sum().item()) == 0

    # ---- CPU baseline: the oracle's fill + apply on the first steps of the same workload
    n_cpu = max(1, args.cpu_steps)
    data_c, len_c = traj.init_data.copy(), traj.init_len.copy()
    states_c = data_c[np.arange(B), len_c - 1].copy()
    rng = np.random.default_rng(cfg.seed + 1)
    cpu_logits = bf16_logits(rng, B, V)
    cpu_t = 0.0
    for s in range(n_cpu):
        rs = np.flatnonzero(traj.reset[s])
        data_c[rs, 0], len_c[rs], states_c[rs] = s0[rs], 1, s0[rs]
        t1 = time.perf_counter()
        m = o.fill_mask(states_c, data_c, len_c, v)
        oracle_apply_mask(cpu_logits, m, V)
        cpu_t += time.perf_counter() - t1
        o.advance_batch(states_c, data_c, len_c, traj.tokens[s], v)
    cores = min(os.cpu_count() or 1, int(os.environ.get("OMP_NUM_THREADS", os.cpu_count() or 1)))

    pairs = float(B) * V
    mask_apply_us = float(np.mean(fill_us + apply_us))
    dominant = "fill_mask" if fill_us.mean() >= apply_us.mean() else "apply_mask"
    achieved = BYTES_PER_PAIR * pairs / (mask_apply_us * 1e-6) / 1e9
    out = {
        "metric": "masked (seq x vocab) tokens/sec",
        "value": pairs * K / elapsed,
        "unit": "tokens/s",
        "n_gpus": 1, "steps": K, "warmup": Wm,
        "ms_per_step": elapsed / K * 1e3,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "u32 bitmask / bf16 logits / i32 states",
        "data": "synthetic",
        "config": {"workload": cfg.name, "batch": B, "vocab": V, "grammar": "byte-level JSON, canonical LR(1)",
                   "stack_cap": cap, "resets_in_timed_steps": int(traj.reset[Wm:].sum())},
        "mask_apply_us_per_step": mask_apply_us,
        "kernels_us": {"fill_mask": {"mean": float(fill_us.mean()), "p50": float(np.median(fill_us)),
                                     "p99": float(np.percentile(fill_us, 99))},
                       "apply_mask": {"mean": float(apply_us.mean()), "p50": float(np.median(apply_us)),
                                      "p99": float(np.percentile(apply_us, 99))},
                       "advance": {"mean": float(adv_us.mean()), "p50": float(np.median(adv_us)),
                                   "p99": float(np.percentile(adv_us, 99))}},
        "mask_apply_tokens_per_s": pairs / (mask_apply_us * 1e-6),
        "roofline": {"bound": "hbm", "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": achieved / HBM_PEAK_GBS, "traffic": None,
                     "kernel": "fill_mask + apply_mask (one step)", "dominant": dominant,
                     "algorithmic_bytes_per_step": BYTES_PER_PAIR * pairs},
        "cpu_baseline": {"value": pairs * n_cpu / cpu_t, "unit": "tokens/s", "cores": cores, "kind": "oracle",
                         "sample": f"fill_mask+apply_mask of the first {n_cpu} steps of the same workload "
                                   f"({cpu_t:.1f} s wall, OpenMP over (sequence, mask word))",
                         "us_per_step": cpu_t / n_cpu * 1e6},
    }
    print(json.dumps(out))


if __name__ == "__main__":
    main()

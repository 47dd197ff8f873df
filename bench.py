"""Benchmark of the batched token-mask path on one MI355X.

One step = stack advance + token mask of the new stacks + logits masking over one batch (B=256
sequences, V=128,256 tokens, byte-level JSON grammar: workload "json-B256-V128256"), replaying
a seeded trajectory; all inputs are resident in HBM before the timed region.  By default the step
is one call, pre3_advance_fill_apply_mask (one kernel launch where the batch size allows, else
pre3_apply_mask + pre3_advance_fill_mask).  The K timed steps are captured into one HIP graph
(kernel launches only) and replayed between two HIP events, so the GPU runs the kernels back to
back as a serving loop would: that replay gives `value`.
Per-call durations (`kernels_us`) come from a second, eager pass over the same K steps with a
HIP event before and after every launch; the pass is queued behind a device-side delay so the
events are processed back to back on the GPU.  The launch duration behind `roofline` is taken
inside the timed steps: they are captured once more with one-thread kernels that write the
device clock before and after every launch; the rocprofv3 summaries under profiles/ hold the
profiler's durations of the same kernels.  After the timed runs the device state and the last mask are checked against the CPU
oracle's replay.  Prints ONE JSON line.

The headline fields (`value`, `ms_per_step`, `config`, `dtype`, `roofline`, `cpu_baseline`) are
measured first; every further leg (per-call brackets, greedy decoding, top-k, jump-forward, the
byte-by-byte mask, the state checks) is guarded: if it fails, its entry of the line holds an
"error" string and the line is still printed.  A failed check of the device state against the
oracle is reported under "checks" and makes the process exit with status 1 after the line.
"""
import argparse
import hashlib
import json
import os
import re
import sys
import time
import traceback

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

BYTES_PER_PAIR = 4.25          # algorithmic HBM bytes per (sequence, token) pair of mask+apply
APPLY_BYTES_PER_PAIR = 4.125   # logits read + written (2 + 2 B) and one mask bit read per 4 B word / 32 tokens
HBM_PEAK_GBS = 8000.0
GRAMMAR_LABEL = {7: "byte-level JSON, every list right-recursive", 1: "arithmetic expressions", 2: "byte-level JSON", 3: "byte-level JSON",
                 4: "schema JSON (12 typed keys)", 5: "8 schema-JSON grammars, mixed",
                 6: "free text, then byte-level JSON"}

def plan_steps(steps: int, warmup: int, cpu_steps: int) -> dict:
    """How many steps of the trajectory each leg uses.  K timed steps follow Wm warm-up steps on the
    GPU; the CPU baseline replays the first n_cpu steps of the same trajectory, so the trajectory
    is generated for n_traj = max(K + Wm, n_cpu) steps and every index any leg uses is below n_traj."""
    K = max(1, int(steps))
    Wm = max(0, int(warmup))
    n_cpu = max(1, int(cpu_steps))
    total = K + Wm
    return {"K": K, "Wm": Wm, "total": total, "n_cpu": n_cpu, "n_traj": max(total, n_cpu)}


def cpu_model() -> str:
    try:
        with open("/proc/cpuinfo") as f:
            for line in f:
                if line.lower().startswith("model name"):
                    return line.split(":", 1)[1].strip()
    except OSError:
        pass
    import platform
    return platform.processor() or platform.machine() or "unknown"


def source_hash(rel_path: str) -> str:
    with open(os.path.join(ROOT, rel_path), "rb") as f:
        return hashlib.sha256(f.read()).hexdigest()[:16]


def profile_traffic(kernel: str, workload: str, profiles_dir: str = None):
    """(bytes per launch or None, note).  Reads `traffic_bytes_per_launch:` from the rocprofv3 summary
    profiles/<kernel>__<workload>.txt; the figure is void (None) when the summary is missing, does not
    state it, or was taken with another version of the kernel's source file (`kernel_source_sha256:`)."""
    path = os.path.join(profiles_dir or os.path.join(ROOT, "profiles"), f"{kernel}__{workload}.txt")
    rel = os.path.relpath(path, ROOT)
    if not os.path.exists(path):
        return None, f"no counter summary {rel}"
    text = open(path).read()
    m = re.search(r"^traffic_bytes_per_launch:\s*([0-9.eE+]+)", text, re.M)
    h = re.search(r"^kernel_source_sha256:\s*(\S+)\s+(\S+)", text, re.M)
    if not m or not h:
        return None, f"{rel} states no traffic figure"
    try:
        now = source_hash(h.group(1))
    except OSError:
        return None, f"{rel}: source file {h.group(1)} not found"
    if now != h.group(2):
        return None, f"{rel} was taken with another version of {h.group(1)}: counters void"
    return float(m.group(1)), f"FETCH_SIZE + WRITE_SIZE per launch, calibrated on a plain copy, from {rel}"


def guarded(fn, *a, **kw):
    """Result of fn, or {"error": ...} if it raises: an auxiliary leg must not take the headline down."""
    try:
        return fn(*a, **kw)
    except Exception as e:                     # noqa: BLE001 - anything: the line is still printed
        tb = traceback.extract_tb(e.__traceback__)
        where = f"{os.path.basename(tb[-1].filename)}:{tb[-1].lineno}" if tb else "?"
        return {"error": f"{type(e).__name__}: {e} ({where})"}


def parse_args(argv=None):
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=128)
    ap.add_argument("--warmup", type=int, default=16)
    ap.add_argument("--config", type=int, default=3)
    ap.add_argument("--cpu-steps", type=int, default=96, help="most steps of the workload timed on the CPU oracle")
    ap.add_argument("--cpu-seconds", type=float, default=25.0,
                    help="the CPU oracle stops after the step that brings its timed work past this many seconds")
    ap.add_argument("--repeats", type=int, default=3, help="replays of each graph (the fastest is reported)")
    ap.add_argument("--eager", action="store_true",
                    help="no HIP graphs: time the eager pass only (for counter collection with rocprofv3 --pmc)")
    ap.add_argument("--headline-only", action="store_true", help="skip the auxiliary legs (greedy, top-k, jump-forward, byte-by-byte)")
    ap.add_argument("--calibrate-copy", type=int, default=0, metavar="MIB",
                    help="only run 20 plain device copies of MIB mebibytes (known traffic, to scale HBM counters)")
    ap.add_argument("--no-token-edges", action="store_true",
                    help="compile without token-level edges: fill_mask walks every (sequence, token) pair")
    ap.add_argument("--max-condition-depth", type=int, default=0,
                    help="limit the token-level conditions to this many stack entries (0 = the library's default of 48): "
                         "a probe that leaves tokens to the run-time walk")
    ap.add_argument("--row-latency", action="store_true",
                    help="also time pre3_fill_mask one sequence at a time (hundreds of one-row launches)")
    ap.add_argument("--effect-min-len", type=int, default=0,
                    help="shortest token that gets a stack-effect record (0 = the library's default; -1 = no records)")
    ap.add_argument("--batch", type=int, default=0,
                    help="override the workload's batch size (a scaling probe: the JSON line names the workload with the new size)")
    ap.add_argument("--step", choices=["two-call", "fused", "advance-fill", "one-call"], default="one-call",
                    help="fill_mask + apply_mask + advance | fill_apply_mask + advance | "
                         "apply_mask + advance_fill_mask (advance and next mask in one launch, slot reuse on EOS) | "
                         "advance_fill_apply_mask (the whole step in one launch)")
    return ap.parse_args(argv)


def main(argv=None):
    args = parse_args(argv)
    if args.gpus != 1:
        sys.exit("bench.py: this path runs on one GPU (sequences are independent: shard the batch across processes, one handle each); use --gpus 1")

    import numpy as np
    import torch

    if args.calibrate_copy:
        n = args.calibrate_copy << 20
        src = torch.zeros(n, dtype=torch.uint8, device="cuda:0")
        dst = torch.empty_like(src)
        dst.copy_(src)
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(20):
            dst.copy_(src)
        e1.record()
        torch.cuda.synchronize()
        us = e0.elapsed_time(e1) * 1e3 / 20
        # buffers beyond the 256 MB Infinity Cache give the chip's practical read+write HBM rate
        print(json.dumps({"calibrate_copy_bytes_read": n, "calibrate_copy_bytes_written": n, "copies": 21,
                          "us_per_copy": us, "read_plus_write_GBs": 2.0 * n / (us * 1e-6) / 1e9}))
        return 0

    from oracle import Oracle, apply_mask as oracle_apply_mask, masked_argmax as oracle_masked_argmax, masked_topk as oracle_masked_topk
    from paper_2506_03887_amd import Pre3, apply_mask
    from workloads import configs, trajectory
    from workloads.vocab import bf16_logits

    cfg = configs.get(args.config)
    if args.batch > 0 and args.batch != cfg.batch:
        import dataclasses
        cfg = dataclasses.replace(cfg, batch=args.batch, name=re.sub(r"-B\d+-", f"-B{args.batch}-", cfg.name))
    v = cfg.vocab
    B, V, W, cap = cfg.batch, v.n_tokens, v.words, cfg.cap
    plan = plan_steps(args.steps, args.warmup, args.cpu_steps)
    K, Wm, total, n_traj = plan["K"], plan["Wm"], plan["total"], plan["n_traj"]
    pairs = float(B) * V

    # ---- inputs: oracle-driven seeded trajectory (host), then everything uploaded
    compact = cfg.compact
    o = Oracle(cfg.grammars, compact_cycles=compact)
    gi, depths = configs.sequence_setup(cfg)
    traj = trajectory.generate(o, v, B, n_traj, cap, cfg.seed, gi, cfg.nest_cap, None, cfg.json_strings, depths, marker=cfg.marker, p_line_feed=cfg.p_line_feed)
    assert traj.tokens.shape[0] == traj.reset.shape[0] == n_traj >= total
    s0 = np.array([o.initial_state(int(g)) for g in gi], dtype=np.int32)

    dev = torch.device("cuda:0")
    t_compile = time.perf_counter()
    lib = Pre3(cfg.grammars, v.bytes, v.offsets, v.eos_id, max_token_len=max(1, v.max_len), stack_cap=cap,
               token_edges=not args.no_token_edges, compact_cycles=compact, max_condition_depth=args.max_condition_depth,
               token_effects=args.effect_min_len >= 0, effect_min_len=max(0, args.effect_min_len))
    t_compile = time.perf_counter() - t_compile
    data_h, len_h = traj.init_data.copy(), traj.init_len.copy()
    states_h = data_h[np.arange(B), len_h - 1].copy()
    data_d = torch.from_numpy(data_h).to(dev)
    # len and states share one [2, B] tensor so that slot reuse is a single small kernel
    ls_d = torch.from_numpy(np.stack([len_h, states_h])).to(dev)
    len_d, states_d = ls_d[0], ls_d[1]
    err_d = torch.zeros(B, dtype=torch.int32, device=dev)
    mask_d = torch.empty((B, W), dtype=torch.int32, device=dev)
    lib.bind_state(states_d, data_d, len_d, err_d)
    tokens_d = torch.from_numpy(traj.tokens[:total]).to(dev)
    reset_d = torch.from_numpy(np.repeat(traj.reset[:total, None, :], 2, axis=1)).to(dev)      # [steps, 2, B]
    any_reset = traj.reset.any(axis=1)
    fresh_d = torch.from_numpy(np.stack([np.ones(B, dtype=np.int32), s0])).to(dev)        # len = 1, state = s0
    n_pool = 4
    gen = torch.Generator(device=dev)
    gen.manual_seed(cfg.seed)
    logits = [torch.randn((B, V), generator=gen, device=dev, dtype=torch.float32).to(torch.bfloat16)
              for _ in range(n_pool)]

    def resets(s):
        if any_reset[s]:          # slot reuse: a finished sequence restarts (bottom of its stack is kept)
            torch.where(reset_d[s], fresh_d, ls_d, out=ls_d)

    def step(s, kind):
        if kind == "one-call":         # advance by this step's tokens, next mask, and that mask on the next logits
            lib.advance_fill_apply_mask(tokens_d[s], mask_d, logits[(s + 1) % n_pool], restart_on_eos=True)
            return
        if kind == "one-call-asked":   # the same call asked for its one-kernel form whatever the batch size
            lib.advance_fill_apply_mask(tokens_d[s], mask_d, logits[(s + 1) % n_pool], restart_on_eos=True, one_kernel=True)
            return
        if kind == "advance-fill":     # mask_d already holds this step's mask (from the previous call)
            apply_mask(logits[s % n_pool], mask_d, V)
            lib.advance_fill_mask(tokens_d[s], mask_d, restart_on_eos=True)
            return
        resets(s)
        if kind == "fused":
            lib.fill_apply_mask(states_d, data_d, len_d, mask_d, logits[s % n_pool])
        if kind in ("fill", "fill+apply"):
            lib.fill_mask(states_d, data_d, len_d, mask_d)
        if kind == "fill+apply":
            apply_mask(logits[s % n_pool], mask_d, V)
        if kind != "resets":
            lib.advance(tokens_d[s])

    # every kernel runs once before anything is captured or timed, whatever the warm-up count
    # (a token id of -1 leaves a sequence untouched)
    skip_d = torch.full((B,), -1, dtype=torch.int32, device=dev)
    lib.fill_mask(states_d, data_d, len_d, mask_d)
    lib.fill_apply_mask(states_d, data_d, len_d, mask_d, logits[0])
    apply_mask(logits[0], mask_d, V)
    lib.advance(skip_d)
    lib.advance_fill_mask(skip_d, mask_d, restart_on_eos=True)
    lib.advance_fill_apply_mask(skip_d, mask_d, logits[0], restart_on_eos=True)
    for s in range(Wm):
        step(s, "fused" if s % 2 else "fill+apply")
    torch.cuda.synchronize()
    snap = (data_d.clone(), ls_d.clone())

    def restore():
        data_d.copy_(snap[0]); ls_d.copy_(snap[1])
        # the advance-fill pipeline enters a step with that step's mask already computed
        resets(Wm)
        lib.fill_mask(states_d, data_d, len_d, mask_d)

    def replay_best(g, before=None):
        best = float("inf")
        for _ in range(max(1, args.repeats) + 1):          # the first replay also warms the graph
            if before:
                before()
            torch.cuda.synchronize()
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            g.replay()
            e1.record()
            torch.cuda.synchronize()
            best = min(best, e0.elapsed_time(e1))
        return best

    def timed_graph(kind):
        """Captures the K timed steps with the given kernels and returns the fastest replay (ms)."""
        restore()
        torch.cuda.synchronize()
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g):
            for s in range(K):
                step(Wm + s, kind)
        return replay_best(g, restore)

    def eager_pass(kind):
        """The same K steps launched eagerly with a HIP event before and after every library call.
        Returns {call name: microseconds per step} and the wall time of the pass (ms)."""
        restore()
        torch.cuda.synchronize()
        ev = [[torch.cuda.Event(enable_timing=True) for _ in range(4)] for _ in range(K)]
        if not args.eager:
            # keep the GPU busy while the host enqueues the K steps, so that the events are taken back
            # to back on the device and bracket kernel time rather than the host's launch latency
            torch.cuda._sleep(int(60e6))
        t0 = time.perf_counter()
        for s in range(K):
            lg = logits[(Wm + s) % n_pool]
            if kind == "one-call":
                ev[s][0].record()
                lib.advance_fill_apply_mask(tokens_d[Wm + s], mask_d, logits[(Wm + s + 1) % n_pool], restart_on_eos=True)
                ev[s][1].record()
                continue
            if kind == "advance-fill":
                ev[s][0].record()
                apply_mask(lg, mask_d, V)
                ev[s][1].record()
                lib.advance_fill_mask(tokens_d[Wm + s], mask_d, restart_on_eos=True)
                ev[s][2].record()
                continue
            resets(Wm + s)
            ev[s][0].record()
            if kind == "fused":
                lib.fill_apply_mask(states_d, data_d, len_d, mask_d, lg)
                ev[s][1].record()
            else:
                lib.fill_mask(states_d, data_d, len_d, mask_d)
                ev[s][1].record()
                apply_mask(lg, mask_d, V)
            ev[s][2].record()
            lib.advance(tokens_d[Wm + s])
            ev[s][3].record()
        torch.cuda.synchronize()
        wall = (time.perf_counter() - t0) * 1e3
        d = lambda i, j: np.array([e[i].elapsed_time(e[j]) for e in ev]) * 1e3
        if kind == "one-call":
            return {"advance_fill_apply_mask": d(0, 1)}, wall
        if kind == "advance-fill":
            return {"apply_mask": d(0, 1), "advance_fill_mask": d(1, 2)}, wall
        if kind == "fused":
            return {"fill_apply_mask": d(0, 1), "advance": d(2, 3)}, wall
        return {"fill_mask": d(0, 1), "apply_mask": d(1, 2), "advance": d(2, 3)}, wall

    def apply_launch_us():
        """Average duration of one apply_mask launch: K launches (rotating logits buffers, so every
        launch streams from HBM) replayed as one graph between two HIP events."""
        restore()
        torch.cuda.synchronize()
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g):
            for s in range(K):
                apply_mask(logits[s % n_pool], mask_d, V)
        return replay_best(g) * 1e3 / K

    def in_step_us(kind):
        """Durations of the kernels of the step (advance-fill: two, one-call: one) where they run: the K timed steps are
        captured once more with a one-thread kernel between the calls that writes the device's
        100 MHz clock (HIP events cannot be recorded inside a graph here).  A stamp kernel sits between
        every two kernels, so a difference of two stamps is one kernel plus one stamp launch; that
        cost is the difference of two stamps with nothing between them (taken once per step)."""
        from paper_2506_03887_amd.binding import device_timestamp
        restore()
        torch.cuda.synchronize()
        stamps = torch.zeros(4 * K, dtype=torch.int64, device=dev)
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g):
            for s in range(K):
                device_timestamp(stamps, 4 * s)
                device_timestamp(stamps, 4 * s + 1)
                if kind == "one-call":
                    lib.advance_fill_apply_mask(tokens_d[Wm + s], mask_d, logits[(s + 1) % n_pool], restart_on_eos=True)
                    device_timestamp(stamps, 4 * s + 2)
                    continue
                apply_mask(logits[s % n_pool], mask_d, V)
                device_timestamp(stamps, 4 * s + 2)
                lib.advance_fill_mask(tokens_d[Wm + s], mask_d, restart_on_eos=True)
                device_timestamp(stamps, 4 * s + 3)
        best = None
        for _ in range(max(1, args.repeats) + 1):
            restore()
            torch.cuda.synchronize()
            g.replay()
            torch.cuda.synchronize()
            t = stamps.cpu().numpy().reshape(K, 4).astype(np.float64) * 0.01        # microseconds
            cost = np.median(t[:, 1] - t[:, 0])
            if kind == "one-call":
                cur = {"advance_fill_apply_mask": float(np.mean(t[:, 2] - t[:, 1]) - cost), "stamp_cost": float(cost)}
            else:
                cur = {"apply_mask": float(np.mean(t[:, 2] - t[:, 1]) - cost),
                       "advance_fill_mask": float(np.mean(t[:, 3] - t[:, 2]) - cost), "stamp_cost": float(cost)}
            total_us = lambda r: sum(x for k_, x in r.items() if k_ != "stamp_cost")
            if best is None or total_us(cur) < total_us(best):
                best = cur
        return best

    _snaps = []

    def recorded_stacks():
        """(len/states, stack data) of the batch at each of the K timed steps of the trajectory."""
        if not _snaps:
            restore()
            for s in range(K):
                resets(Wm + s)
                _snaps.append((ls_d.clone(), data_d.clone()))
                lib.advance(tokens_d[Wm + s])
            torch.cuda.synchronize()
        return _snaps

    def mask_apply_graph_us():
        """fill_mask + apply_mask alone, K steps in one graph: the stacks of the K timed steps are
        recorded first (fill_mask reads a snapshot, the bound buffers stay untouched), so every
        step computes a different batch of rows, as in the real loop, but no advance or reset
        kernel and no event bracket sits between the two calls that are timed."""
        snaps = recorded_stacks()
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g):
            for s in range(K):
                ls, da = snaps[s]
                lib.fill_mask(ls[1], da, ls[0], mask_d)
                apply_mask(logits[s % n_pool], mask_d, V)
        return replay_best(g) * 1e3 / K

    def fill_apply_graph_us():
        """pre3_fill_apply_mask (mask + masking as one call; one launch where the batch size allows) on the recorded
        stacks of the K timed steps, one graph between two events."""
        snaps = recorded_stacks()
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g):
            for s in range(K):
                ls, da = snaps[s]
                lib.fill_apply_mask(ls[1], da, ls[0], mask_d, logits[s % n_pool])
        return replay_best(g) * 1e3 / K

    # =========================== headline: the step, then the dominant kernel ===========================
    step_kind = {"two-call": "fill+apply", "fused": "fused", "advance-fill": "advance-fill", "one-call": "one-call"}[args.step]
    step_launches = lib.step_kernel_launches(logits[0]) if step_kind == "one-call" else 0
    if step_kind == "one-call" and step_launches == 0:
        # outside the batch sizes (or vocabulary) of the one kernel the call is pre3_advance_fill_mask + pre3_apply_mask:
        # time and label those
        step_kind = "advance-fill"
    step_text = {"fill+apply": "pre3_fill_mask + pre3_apply_mask + pre3_advance (+ slot-reuse resets by the caller)",
                 "fused": "pre3_fill_apply_mask + pre3_advance (+ slot-reuse resets by the caller)",
                 "advance-fill": "pre3_apply_mask + pre3_advance_fill_mask (advance and next mask in one launch, "
                                 "slot reuse on EOS)",
                 "one-call": "pre3_advance_fill_apply_mask (advance, next mask and masked logits in one launch, "
                             "slot reuse on EOS)" if step_launches <= 1 else
                             f"pre3_advance_fill_apply_mask (advance, next mask and masked logits in one kernel, {step_launches} "
                             "launches on equal shares of the batch, slot reuse on EOS)"}
    step_us = None
    if args.eager:
        step_us, t_step = eager_pass(step_kind)
        apply_us = float(step_us["apply_mask"].mean()) if "apply_mask" in step_us else float("nan")
        if step_kind == "one-call":
            apply_us = float(step_us["advance_fill_apply_mask"].mean())
    else:
        t_step = timed_graph(step_kind)
    # the device now holds the state after all K timed steps of `step_kind`: kept for the check below
    final_states_d, final_len_d, final_err_d = states_d.clone(), len_d.clone(), err_d.clone()
    apply_alone_us, in_step = None, None
    if not args.eager:
        apply_alone_us = apply_launch_us()
        apply_us = apply_alone_us
        if step_kind == "advance-fill":
            in_step = in_step_us(step_kind)
            apply_us = in_step["apply_mask"]
        if step_kind == "one-call":
            in_step = in_step_us(step_kind)
            apply_us = in_step["advance_fill_apply_mask"]

    out = {
        "metric": "masked (seq x vocab) tokens/sec",
        "value": pairs * K / (t_step * 1e-3),
        "unit": "tokens/s",
        "n_gpus": 1, "steps": K, "warmup": Wm,
        "ms_per_step": t_step / K,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "i32 (integer and bit work: i32 states, u32 bitmask words; the bf16 logits are selected, not computed on)",
        "data": "synthetic",
        "config": {"workload": cfg.name, "batch": B, "vocab": V, "grammar": GRAMMAR_LABEL.get(cfg.idx, cfg.name) + ", canonical LR(1)",
                   "stack_cap": cap, **({"max_condition_depth": args.max_condition_depth} if args.max_condition_depth else {}),
                   "sequences_restarted_in_timed_steps": int(traj.reset[Wm:total].sum()),
                   "step": step_text[step_kind] + (", K eager steps" if args.eager else ", K steps in one HIP graph")},
    }

    # the logits-masking kernel dominates: it reads and writes the bf16 logits (4 B/pair) and reads the mask
    if step_kind == "one-call":
        # the one kernel of the step reads and writes the logits (4 B/pair) and writes the mask (one bit per pair)
        # (a batch beyond one sequence per compute unit goes as several launches of equal shares: the figures are per launch)
        dom_name, dom_bytes, dom_us = "advance_fill_apply_kernel", APPLY_BYTES_PER_PAIR * pairs / step_launches, apply_us / step_launches
        dom_timing = ("HIP events around every launch of an eager pass over the timed steps" if args.eager else
                      "inside the K timed steps replayed as one HIP graph: device clock stamps (one-thread kernels) before and "
                      "after every launch, minus the cost of a stamp")
    elif step_kind != "fused":
        dom_name, dom_bytes, dom_us = "apply_mask_vec8_kernel", APPLY_BYTES_PER_PAIR * pairs, apply_us
        dom_timing = ("HIP events around every launch of an eager pass over the timed steps" if args.eager else
                      "inside the K timed steps replayed as one HIP graph: device clock stamps (one-thread kernels) before and "
                      "after every launch, minus the cost of a stamp" if in_step else
                      "K launches on rotating logits buffers replayed as one HIP graph between two HIP events, divided by K")
    else:
        fused_us, _ = eager_pass("fused")
        # the call takes one of three forms by the batch size (the figures below are those of the whole call)
        units = torch.cuda.get_device_properties(0).multi_processor_count
        dom_name = ("advance_fill_apply_kernel (without the advance)" if lib.step_kernel_launches(logits[0]) == 1 else
                    "fill_mask_edges_kernel<false> + apply_mask_vec8_kernel" if B > units else "fill_mask_edges_kernel<true>")
        dom_bytes = BYTES_PER_PAIR * pairs
        dom_us = float(fused_us["fill_apply_mask"].mean())
        dom_timing = "HIP events around every launch of an eager pass over the timed steps"
    traffic, traffic_note = (None, "batch size differs from the profiled workload") if args.batch not in (0, configs.get(args.config).batch) \
        else profile_traffic(dom_name.split("<")[0].split(" ")[0], cfg.name) if step_kind != "fused" else (None, "no counters for this form")
    achieved = dom_bytes / (dom_us * 1e-6) / 1e9
    out["roofline"] = {"bound": "hbm", "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                       "frac": achieved / HBM_PEAK_GBS, "traffic": traffic,
                       "kernel": dom_name, "algorithmic_bytes_per_launch": dom_bytes, "launch_us": dom_us,
                       "timing": dom_timing, "traffic_source": traffic_note,
                       "frac_on_traffic": None if traffic is None else traffic / (dom_us * 1e-6) / 1e9 / HBM_PEAK_GBS}
    if in_step and step_kind == "advance-fill":
        # the same kernel launched K times back to back finds its mask bytes in L2 and runs faster than in the step
        out["roofline"]["launch_us_back_to_back"] = apply_alone_us
        out["roofline"]["frac_back_to_back"] = dom_bytes / (apply_alone_us * 1e-6) / 1e9 / HBM_PEAK_GBS
    if in_step:
        out["in_step_kernel_us"] = in_step
    if step_kind == "one-call":
        out["apply_mask_alone_us"] = apply_alone_us
        out["roofline"]["launches_per_step"] = step_launches

    # ---- CPU baseline: the oracle's fill + apply on the first steps of the same workload
    def cpu_baseline():
        data_c, len_c = traj.init_data.copy(), traj.init_len.copy()
        states_c = data_c[np.arange(B), len_c - 1].copy()
        rng = np.random.default_rng(cfg.seed + 1)
        cpu_logits = bf16_logits(rng, B, V)
        cpu_t, done = 0.0, 0
        for s in range(min(plan["n_cpu"], traj.reset.shape[0])):
            rs = np.flatnonzero(traj.reset[s])
            data_c[rs, 0], len_c[rs], states_c[rs] = s0[rs], 1, s0[rs]
            t1 = time.perf_counter()
            m = o.fill_mask(states_c, data_c, len_c, v)
            oracle_apply_mask(cpu_logits, m, V)
            cpu_t += time.perf_counter() - t1
            done += 1
            if cpu_t >= args.cpu_seconds:
                break
            o.advance_batch(states_c, data_c, len_c, traj.tokens[s], v)
        cores = min(os.cpu_count() or 1, int(os.environ.get("OMP_NUM_THREADS", os.cpu_count() or 1)))
        return {"value": pairs * done / cpu_t, "unit": "tokens/s", "cores": cores, "kind": "oracle",
                "cpu": cpu_model(),
                "sample": f"fill_mask+apply_mask of the first {done} steps of the same workload "
                          f"({cpu_t:.1f} s wall, OpenMP over (sequence, mask word))",
                "us_per_step": cpu_t / done * 1e6}

    out["cpu_baseline"] = guarded(cpu_baseline)

    # =========================== everything below is auxiliary and guarded ===========================
    stat = lambda x: {"mean": float(x.mean()), "p50": float(np.median(x)), "p99": float(np.percentile(x, 99))}

    def per_call_leg():
        """Three-call step in a graph, fill+apply alone in a graph, and per-call event brackets."""
        r = {}
        two_call_us, wall_two = eager_pass("fill+apply")
        kernels = {k: stat(x) for k, x in two_call_us.items()}
        if step_kind != "fill+apply":
            su = step_us if step_us is not None else eager_pass(step_kind)[0]
            kernels.update({k: stat(x) for k, x in su.items()})
        r["kernels_us"] = kernels
        brackets = float((two_call_us["fill_mask"] + two_call_us["apply_mask"]).mean())
        if args.eager:
            t_two, mask_apply_us = wall_two, brackets
        else:
            t_two = t_step if step_kind == "fill+apply" else timed_graph("fill+apply")
            mask_apply_us = mask_apply_graph_us()
        r["fill_mask_tokens_per_s"] = pairs / (float(two_call_us["fill_mask"].mean()) * 1e-6)
        r["mask_apply_us_per_step"] = mask_apply_us
        r["mask_apply_timing"] = ("pre3_fill_mask + pre3_apply_mask on the recorded stacks of the K timed steps, one HIP graph "
                                  "between two HIP events, divided by K; with a pair of events around every launch the two "
                                  f"calls read {brackets:.1f} us")
        r["mask_apply_tokens_per_s"] = pairs / (mask_apply_us * 1e-6)
        if not args.eager:
            fa_us = fill_apply_graph_us()
            r["fill_apply_one_call_us_per_step"] = fa_us
            r["fill_apply_one_call_frac_of_hbm_peak"] = BYTES_PER_PAIR * pairs / (fa_us * 1e-6) / 1e9 / HBM_PEAK_GBS
        r["mask_apply_frac_of_hbm_peak"] = BYTES_PER_PAIR * pairs / (mask_apply_us * 1e-6) / 1e9 / HBM_PEAK_GBS
        r["step_frac_of_hbm_peak"] = BYTES_PER_PAIR * pairs / (t_step / K * 1e-3) / 1e9 / HBM_PEAK_GBS
        r["graph_ms_per_step"] = {step_text[step_kind]: t_step / K, step_text["fill+apply"]: t_two / K}
        if step_kind == "one-call" and not args.eager:
            r["graph_ms_per_step"][step_text["advance-fill"]] = timed_graph("advance-fill") / K
        asked = lib.step_kernel_launches(logits[0], one_kernel=True)
        if step_kind == "advance-fill" and args.step == "one-call" and asked > 0 and not args.eager:
            # a batch beyond one sequence per compute unit: the one kernel only runs on request (PRE3_STEP_ONE_KERNEL)
            r["graph_ms_per_step"][f"pre3_advance_fill_apply_mask asked for its one-kernel form ({asked} launches on equal shares "
                                   "of the batch)"] = timed_graph("one-call-asked") / K
        return r

    def state_check():
        """The timed run must have done the real work: final state == the oracle's replay."""
        d_h, l_h, s_h = traj.init_data.copy(), traj.init_len.copy(), None
        s_h = d_h[np.arange(B), l_h - 1].copy()
        for s in range(total):
            rs = np.flatnonzero(traj.reset[s])
            d_h[rs, 0], l_h[rs], s_h[rs] = s0[rs], 1, s0[rs]
            err = o.advance_batch(s_h, d_h, l_h, traj.tokens[s], v)
            assert not err.any()
        if step_kind in ("advance-fill", "one-call"):            # slot reuse happened inside the last call
            fin = s_h < 0
            s_h[fin], l_h[fin] = s0[fin], 1
        assert (final_states_d.cpu().numpy() == s_h).all() and (final_len_d.cpu().numpy() == l_h).all(), \
            "device state after the timed run differs from the oracle's replay"
        assert int(final_err_d.abs().sum().item()) == 0, "err flags set during the timed run"
        return {"ok": True, "len_after_timed_steps": {"mean": float(l_h.mean()), "max": int(l_h.max())},
                "stacks": (d_h, l_h, s_h)}

    def mask_check():
        """The last mask on the device is the oracle's mask of the last timed step's input state."""
        restore()
        for s in range(K - 1):
            step(Wm + s, "advance")
        resets(total - 1)
        lib.fill_mask(states_d, data_d, len_d, mask_d)
        d_c, l_c = traj.init_data.copy(), traj.init_len.copy()
        s_c = d_c[np.arange(B), l_c - 1].copy()
        for s in range(total - 1):
            rs = np.flatnonzero(traj.reset[s])
            d_c[rs, 0], l_c[rs], s_c[rs] = s0[rs], 1, s0[rs]
            o.advance_batch(s_c, d_c, l_c, traj.tokens[s], v)
        rs = np.flatnonzero(traj.reset[total - 1])
        d_c[rs, 0], l_c[rs], s_c[rs] = s0[rs], 1, s0[rs]
        assert (mask_d.cpu().numpy().view(np.uint32) == o.fill_mask(s_c, d_c, l_c, v)).all(), "final mask differs"
        return {"ok": True}

    def lookup_stats(stacks):
        """What one mask look-up touches (host evaluation of the same condition trees on the final stacks)."""
        d_h, l_h, s_h = stacks
        tree_nodes = deepest = leftover = 0
        if not args.no_token_edges and lib.token_edge_stats()["built"]:
            for b in range(B):
                if s_h[b] < 0:
                    continue
                ok, _, walk = lib.debug_resolve_row(d_h[b, : l_h[b]].copy())
                tree_nodes += lib.last_resolve_info["path_nodes"]
                deepest = max(deepest, lib.last_resolve_info["deepest_entry"])
                leftover += len(walk) if ok else V
        return {"condition_nodes_visited_per_step": tree_nodes,
                "deepest_stack_entry_tested": deepest, "tokens_left_to_the_walk_per_step": leftover,
                "note": "host evaluation of the device's condition trees on the stacks after the timed steps; "
                        "the kernel is latency-bound: a descent of dependent loads per row, then a row copy"}

    def jump_forward_leg(n_calls=32, max_bytes=32):
        """pre3_jump_forward on the recorded stacks of the first steps (on copies: it advances the
        stacks), one call per step with a HIP event on either side; checked against the oracle."""
        snaps = recorded_stacks()
        n_calls = min(n_calls, K)
        ls2, da2 = snaps[0][0].clone(), snaps[0][1].clone()
        err2 = torch.zeros(B, dtype=torch.int32, device=dev)
        out_b = torch.zeros((B, max_bytes), dtype=torch.uint8, device=dev)
        out_n = torch.zeros(B, dtype=torch.int32, device=dev)
        lib.bind_state(ls2[1], da2, ls2[0], err2)
        try:
            times, forced = [], 0
            for s in range(n_calls):
                ls2.copy_(snaps[s][0]); da2.copy_(snaps[s][1])
                if s == 0:                                            # check one call against the oracle
                    l_h, s_h = (x.copy() for x in ls2.cpu().numpy())
                    d_h = da2.cpu().numpy().copy()
                    wb, wn = o.jump_forward_batch(s_h, d_h, l_h, max_bytes)
                torch.cuda.synchronize()
                e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                e0.record()
                lib.jump_forward(out_b, out_n)
                e1.record()
                torch.cuda.synchronize()
                times.append(e0.elapsed_time(e1) * 1e3)
                forced += int(out_n.sum().item())
                if s == 0:
                    assert (out_n.cpu().numpy() == wn).all() and (ls2[0].cpu().numpy() == l_h).all(), "jump_forward differs from the oracle"
                    gb = out_b.cpu().numpy()
                    assert all(gb[b, : wn[b]].tobytes() == wb[b, : wn[b]].tobytes() for b in range(B))
        finally:
            lib.bind_state(states_d, data_d, len_d, err_d)
        timed = times[1:] if len(times) > 1 else times
        return {"us_per_call": float(np.mean(timed)), "calls": len(timed), "max_bytes": max_bytes,
                "forced_bytes_per_call": forced / n_calls,
                "timing": "one eager call per recorded step between two HIP events (the bracket adds a few us)"}

    def byte_by_byte_leg(n_calls=6):
        """The same masks without token-level edges: every (sequence, token) pair walked byte by byte
        (the path the token-level edges replace), on the recorded stacks of the first steps."""
        snaps = recorded_stacks()
        plain = Pre3(cfg.grammars, v.bytes, v.offsets, v.eos_id, max_token_len=max(1, v.max_len), stack_cap=cap,
                     token_edges=False, compact_cycles=compact)
        m2 = torch.empty_like(mask_d)
        times = []
        for s in range(min(n_calls, K)):
            ls, da = snaps[s]
            torch.cuda.synchronize()
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            plain.fill_mask(ls[1], da, ls[0], m2)
            e1.record()
            torch.cuda.synchronize()
            times.append(e0.elapsed_time(e1) * 1e3)
            if s == 0:
                lib.fill_mask(ls[1], da, ls[0], mask_d)
                assert torch.equal(m2, mask_d), "byte-by-byte mask differs from the token-edge mask"
        t = float(np.mean(times[1:])) if len(times) > 1 else float(times[0])
        return {"us_per_launch": t, "tokens_per_s": pairs / (t * 1e-6),
                "vocab_bytes_times_batch_per_s": float(B) * float(v.offsets[-1]) / (t * 1e-6),
                "note": "fill_mask_walk_kernel; a walk stops at its first rejected byte, so the byte rate is an upper bound on byte steps"}

    def row_latency_leg(max_rows=256, launches=16):
        """pre3_fill_mask on ONE sequence at a time (the stacks of the first timed step, and rows of the first 32
        steps whose look-up leaves tokens to the run-time walk): per row, `launches` calls in one HIP graph
        between two events.  Shows what the rows that leave tokens to the run-time
        walk cost next to the rows that are a pure look-up (the launch itself is part of every figure)."""
        snaps = recorded_stacks()
        # every row of the first timed step, plus up to 128 rows of the other steps that leave tokens to the walk
        todo = []
        for si, (ls, da) in enumerate(snaps):
            l_h, s_h = ls.cpu().numpy()
            d_h = da.cpu().numpy()
            for b in range(B):
                n_walk = 0
                if not args.no_token_edges and s_h[b] >= 0:
                    ok, _, walk = lib.debug_resolve_row(d_h[b, : l_h[b]].copy())
                    n_walk = len(walk) if ok else V
                if (si == 0 and b < max_rows) or (si > 0 and n_walk > 0 and len(todo) < max_rows + 128):
                    todo.append((si, b, n_walk))
            if si >= 31:
                break
        us, walked = [], []
        for si, b, n_walk in todo:
            ls, da = snaps[si]
            walked.append(n_walk)
            st1, da1, ln1, m1 = ls[1][b:b + 1], da[b:b + 1], ls[0][b:b + 1], mask_d[b:b + 1]
            lib.fill_mask(st1, da1, ln1, m1)
            torch.cuda.synchronize()
            g = torch.cuda.CUDAGraph()
            with torch.cuda.graph(g):
                for _ in range(launches):
                    lib.fill_mask(st1, da1, ln1, m1)
            best = float("inf")
            for _ in range(2):
                torch.cuda.synchronize()
                e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                e0.record()
                g.replay()
                e1.record()
                torch.cuda.synchronize()
                best = min(best, e0.elapsed_time(e1))
            us.append(best * 1e3 / launches)
        rows = todo
        us, walked = np.array(us), np.array(walked)
        r = {"rows": len(rows), "us_per_row_launch": stat(us), "max": float(us.max()),
             "rows_with_tokens_left_to_the_walk": int((walked > 0).sum()), "most_tokens_walked_in_a_row": int(walked.max()),
             "timing": f"per row: {launches} one-row pre3_fill_mask launches in one HIP graph between two events, divided by {launches}"}
        if (walked > 0).any() and (walked == 0).any():
            r["us_rows_pure_lookup_mean"] = float(us[walked == 0].mean())
            r["us_rows_with_walk_mean"] = float(us[walked > 0].mean())
        return r

    # ---- greedy decoding: the sampler fused behind the mask (pre3_apply_mask_argmax reads the logits once
    #      and writes nothing back), tokens fed straight to pre3_advance_fill_mask
    def fresh_logits():
        for x in logits:                          # the timed passes above have masked these in place
            x.copy_(torch.randn((B, V), generator=gen, device=dev, dtype=torch.float32))
        return [x.view(torch.int16).cpu().numpy().view(np.uint16) for x in logits]

    def graph_us(fn):
        restore()
        torch.cuda.synchronize()
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g):
            for s in range(K):
                fn(s)
        return replay_best(g, restore) * 1e3 / K

    def greedy_leg():
        tok_d = torch.empty(B, dtype=torch.int32, device=dev)
        host_logits = fresh_logits()
        restore()
        torch.cuda.synchronize()
        d_g, ls_g = data_d.cpu().numpy().copy(), ls_d.cpu().numpy().copy()
        l_g, s_g = ls_g[0].copy(), ls_g[1].copy()
        n_check = 6
        for s in range(n_check):                  # both sides choose their own tokens and must agree
            want = oracle_masked_argmax(host_logits[s % n_pool], o.fill_mask(s_g, d_g, l_g, v), V)
            lib.apply_mask_argmax(logits[s % n_pool], mask_d, tok_d)
            lib.advance_fill_mask(tok_d, mask_d, restart_on_eos=True)
            assert (tok_d.cpu().numpy() == want).all(), "greedy tokens differ from the oracle's"
            e = o.advance_batch(s_g, d_g, l_g, want, v)
            fin = s_g < 0
            s_g[fin], l_g[fin] = s0[fin], 1
            assert (err_d.cpu().numpy() == e).all()
        assert (states_d.cpu().numpy() == s_g).all() and (len_d.cpu().numpy() == l_g).all()

        # the same loop with one call per step: pre3_advance_fill_argmax takes the token buffer in and out
        def first_token():
            restore()
            lib.apply_mask_argmax(logits[0], mask_d, tok_d)
        first_token()
        torch.cuda.synchronize()
        d_g, ls_g = data_d.cpu().numpy().copy(), ls_d.cpu().numpy().copy()
        l_g, s_g = ls_g[0].copy(), ls_g[1].copy()
        want = oracle_masked_argmax(host_logits[0], o.fill_mask(s_g, d_g, l_g, v), V)
        for s in range(n_check):
            lib.advance_fill_argmax(tok_d, mask_d, logits[(s + 1) % n_pool], tok_d, restart_on_eos=True)
            e = o.advance_batch(s_g, d_g, l_g, want, v)
            fin = s_g < 0
            s_g[fin], l_g[fin] = s0[fin], 1
            want = oracle_masked_argmax(host_logits[(s + 1) % n_pool], o.fill_mask(s_g, d_g, l_g, v), V)
            assert (err_d.cpu().numpy() == e).all() and (tok_d.cpu().numpy() == want).all(), "one-call greedy step differs from the oracle's"
        if args.eager:                            # counter collection: the checked eager steps are enough
            return {"checked_steps_against_oracle": n_check}

        def greedy_step(s):
            lib.apply_mask_argmax(logits[s % n_pool], mask_d, tok_d)
            lib.advance_fill_mask(tok_d, mask_d, restart_on_eos=True)

        argmax_us = graph_us(lambda s: lib.apply_mask_argmax(logits[s % n_pool], mask_d, tok_d))
        step_us_g = graph_us(greedy_step)
        nbytes = 2.0 * pairs + 4.0 * B * W

        first_token()
        torch.cuda.synchronize()
        g1 = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g1):
            for s in range(K):
                lib.advance_fill_argmax(tok_d, mask_d, logits[(s + 1) % n_pool], tok_d, restart_on_eos=True)
        one_call_us = replay_best(g1, first_token) * 1e3 / K
        return {"step": "pre3_apply_mask_argmax + pre3_advance_fill_mask, K steps in one HIP graph, tokens chosen on the device",
                "one_call_step": "pre3_advance_fill_argmax (one launch per step where the batch size allows), K steps in one HIP graph",
                "one_call_us_per_step": one_call_us, "one_call_tokens_per_s": pairs / (one_call_us * 1e-6),
                "one_call_kernel_launches": lib.step_kernel_launches(logits[0]),
                "us_per_step": step_us_g, "tokens_per_s": pairs / (step_us_g * 1e-6),
                "argmax_launch_us": argmax_us, "argmax_algorithmic_bytes": nbytes,
                "argmax_achieved_GBs": nbytes / (argmax_us * 1e-6) / 1e9,
                "argmax_frac_of_hbm_peak": nbytes / (argmax_us * 1e-6) / 1e9 / HBM_PEAK_GBS,
                "checked_steps_against_oracle": n_check}

    def topk_leg(topk_k=50):
        """top-k behind the mask: same read-once traffic as the arg max; one call checked against the oracle."""
        host_logits = fresh_logits()
        restore()
        topk_ids = torch.empty((B, topk_k), dtype=torch.int32, device=dev)
        topk_vals = torch.empty((B, topk_k), dtype=torch.int16, device=dev)
        lib.apply_mask_topk(logits[0], mask_d, topk_ids, topk_vals)
        want_ids, want_vals = oracle_masked_topk(host_logits[0], mask_d.cpu().numpy().view(np.uint32), V, topk_k)
        assert (topk_ids.cpu().numpy() == want_ids).all() and (topk_vals.cpu().numpy().view(np.uint16) == want_vals).all(), \
            "top-k differs from the oracle's"
        for s in range(1, 4):
            lib.apply_mask_topk(logits[s % n_pool], mask_d, topk_ids, topk_vals)
        if args.eager:
            return {"k": topk_k, "checked_calls_against_oracle": 1}
        topk_us = graph_us(lambda s: lib.apply_mask_topk(logits[s % n_pool], mask_d, topk_ids, topk_vals))
        nbytes = 2.0 * pairs + 4.0 * B * W
        return {"k": topk_k, "launch_us": topk_us, "achieved_GBs": nbytes / (topk_us * 1e-6) / 1e9,
                "frac_of_hbm_peak": nbytes / (topk_us * 1e-6) / 1e9 / HBM_PEAK_GBS,
                "note": "pre3_apply_mask_topk, K calls in one HIP graph; same algorithmic bytes as the arg max"}

    def auxiliary(out, checks):
        sc = guarded(state_check)
        stacks = sc.pop("stacks", None)
        checks["final_state_vs_oracle"] = sc
        r = guarded(per_call_leg)
        out.update({"per_call": r} if "error" in r else r)
        checks["last_mask_vs_oracle"] = guarded(mask_check)
        checks["device_fault_count"] = guarded(lambda: {"ok": lib.fault_count() == 0, "count": lib.fault_count()})
        if stacks is not None:
            out["fill_mask_lookup"] = guarded(lookup_stats, stacks)
            if "kernels_us" in out and "error" not in out["fill_mask_lookup"]:
                out["fill_mask_lookup"]["condition_nodes_per_s"] = (
                    out["fill_mask_lookup"]["condition_nodes_visited_per_step"] / (out["kernels_us"]["fill_mask"]["mean"] * 1e-6))
            out["stacks"] = {"cycle_aware": bool(compact), "reduction_cycles": len(lib.reduction_cycles()),
                             "len_after_timed_steps": sc.get("len_after_timed_steps")}
        out["initial_stack_depths"] = ({"min": int(traj.init_len.min() - 1), "mean": float(traj.init_len.mean() - 1),
                                        "max": int(traj.init_len.max() - 1)} if cfg.mixed else None)
        if not args.headline_only:
            out["greedy"] = guarded(greedy_leg)
            out["topk"] = guarded(topk_leg)
            if not args.eager:
                if args.row_latency:
                    out["fill_mask_row_latency"] = guarded(row_latency_leg)
                out["jump_forward"] = guarded(jump_forward_leg)
                if not args.no_token_edges:
                    out["fill_mask_byte_by_byte"] = guarded(byte_by_byte_leg)
        out["token_edges"] = guarded(lib.token_edge_stats)

    checks = {}
    try:
        auxiliary(out, checks)
    except Exception as e:                     # noqa: BLE001 - the headline above is still printed
        out["auxiliary_error"] = f"{type(e).__name__}: {e}"
    out["checks"] = checks
    out["compile_s"] = t_compile
    print(json.dumps(out))
    sys.stdout.flush()
    bad = [k for k, c in checks.items() if not c.get("ok")]
    if bad:
        print("bench.py: check(s) failed: " + ", ".join(f"{k}: {checks[k]}" for k in bad), file=sys.stderr)
        return 1
    return 0


if __name__ == "__main__":
    sys.exit(main())

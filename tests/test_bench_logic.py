"""The benchmark's host-side arithmetic (no GPU): which trajectory steps each leg indexes, the
guard around auxiliary legs, and the reading of counter traffic from a profile summary."""
import os
import sys

import numpy as np
import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
sys.path.insert(0, ROOT)
import bench  # noqa: E402


@pytest.mark.parametrize("steps,warmup,cpu_steps", [(20, 5, 96), (1, 0, 96), (128, 16, 96), (20, 5, 3), (20, 5, 25),
                                                   (20, 5, 26), (0, 0, 0), (1, 0, 1), (512, 64, 8)])
def test_every_leg_indexes_inside_the_trajectory(steps, warmup, cpu_steps):
    p = bench.plan_steps(steps, warmup, cpu_steps)
    K, Wm, total, n_cpu, n_traj = p["K"], p["Wm"], p["total"], p["n_cpu"], p["n_traj"]
    assert K >= 1 and Wm >= 0 and total == K + Wm and n_cpu >= 1
    tokens = np.zeros((n_traj, 4), dtype=np.int32)         # what trajectory.generate returns for n_traj steps
    reset = np.zeros((n_traj, 4), dtype=bool)
    # GPU legs: warm-up steps 0..Wm-1, timed steps Wm..total-1, the checks replay 0..total-1
    for s in list(range(Wm)) + [Wm + k for k in range(K)] + list(range(total)) + [total - 1]:
        tokens[s], reset[s]
    # the device copies hold the first `total` steps only
    assert tokens[:total].shape[0] == total
    # CPU baseline: steps 0..n_cpu-1
    for s in range(min(n_cpu, reset.shape[0])):
        tokens[s], reset[s]
    assert n_cpu <= n_traj


def test_driver_command_line_parses_to_the_failing_case_of_old():
    a = bench.parse_args(["--gpus", "1", "--steps", "20", "--warmup", "5"])
    p = bench.plan_steps(a.steps, a.warmup, a.cpu_steps)
    assert p["total"] == 25 and p["n_cpu"] == 96 and p["n_traj"] == 96     # the CPU leg no longer runs off the end


def test_more_than_one_gpu_is_refused_with_a_message():
    with pytest.raises(SystemExit) as e:
        bench.main(["--gpus", "2"])
    assert "one GPU" in str(e.value)


def test_guarded_turns_an_exception_into_an_error_entry():
    assert bench.guarded(lambda: {"x": 1}) == {"x": 1}
    r = bench.guarded(lambda: [][3])
    assert set(r) == {"error"} and "IndexError" in r["error"]


def test_profile_traffic_is_void_unless_the_summary_matches_the_source(tmp_path):
    src = "paper_2506_03887_amd/csrc/apply_kernels.hip"
    h = bench.source_hash(src)
    t, note = bench.profile_traffic("k", "w", str(tmp_path))
    assert t is None and "no counter summary" in note
    f = tmp_path / "k__w.txt"
    f.write_text("some summary\n")
    assert bench.profile_traffic("k", "w", str(tmp_path))[0] is None
    f.write_text(f"x\nkernel_source_sha256: {src} {h}\ntraffic_bytes_per_launch: 130630000\n")
    t, note = bench.profile_traffic("k", "w", str(tmp_path))
    assert t == 130630000.0
    f.write_text(f"x\nkernel_source_sha256: {src} 0000000000000000\ntraffic_bytes_per_launch: 130630000\n")
    t, note = bench.profile_traffic("k", "w", str(tmp_path))
    assert t is None and "another version" in note


def test_cpu_model_is_a_nonempty_string():
    assert isinstance(bench.cpu_model(), str) and bench.cpu_model()

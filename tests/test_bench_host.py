"""Host-side checks of the benchmark script (no GPU): it refuses more than one
GPU with a message, and its per-stage algorithmic byte counts add up to the
42 U of the kernels and bracket the 29 U floor of the path."""
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_more_than_one_gpu_is_refused_with_a_message():
    r = subprocess.run([sys.executable, "bench.py", "--gpus", "2"], cwd=ROOT, capture_output=True, text=True)
    assert r.returncode == 2 and "one GPU" in r.stderr and r.stdout.strip() == ""


def test_stage_bytes_add_up():
    sys.path.insert(0, ROOT)
    import bench
    n, C, T, e = 4, 4096, 32768, 2
    U = C * e
    per_token = [bench.stage_bytes(s, n, C, T, e) // T for s in (1, 2, 3, 4, 5)]
    assert per_token == [n * U, (n + 1) * U, (2 * n + 1) * U, (2 * n + 2) * U, (3 * n + 2) * U]
    assert sum(per_token) == 42 * U                    # what the five streaming kernels move
    floor = (3 * n + 2) * U + (3 * n + 3) * U          # every stream tensor once: forward + backward
    assert floor == 29 * U == 237568 and sum(per_token) > floor


def test_measured_traffic_comes_from_the_tracked_profile_and_is_tied_to_the_sources():
    sys.path.insert(0, ROOT)
    import bench
    digest, table = bench.profile_traffic("n4_c4096")
    assert len(digest) == 16 and any(k.startswith("bwd_out_gw_kernel") for k in table)
    # the figures are the ones tabulated in profiles/n4_c4096_bench_step.md (read + written MiB)
    text = open(os.path.join(ROOT, "profiles", "n4_c4096_bench_step.md")).read()
    for name, nbytes in table.items():
        row = next(l for l in text.splitlines() if l.startswith(f"| {name} |") and l.count("|") == 6)
        cells = [c.strip() for c in row.strip("|").split("|")]
        assert nbytes == int((float(cells[3]) + float(cells[4])) * 2**20)
    got = bench.measured_traffic("n4_c4096", 5)
    want = next(v for k, v in table.items() if k.startswith("bwd_out_gw_kernel"))
    assert got == (want if digest == bench.csrc_digest() else None)   # None once the sources have changed
    assert bench.measured_traffic("no_such_workload", 5) is None

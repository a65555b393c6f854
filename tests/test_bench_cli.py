"""bench.py's command line, without a GPU: defaults, the refusal of more than one GPU, and that the
variant runs of the default line only set flags the parser knows."""
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
sys.path.insert(0, ROOT)

import bench  # noqa: E402


def test_defaults_name_the_largest_configuration():
    args = bench.build_parser().parse_args([])
    assert args.gpus == 1 and args.workload == "c4" and args.size == "full" and args.stage == "hit"
    assert args.steps is None and args.warmup is None and args.secondary is None and args.extras is None
    a = bench.with_defaults(args, "c4", "config", 20, 5, None)
    assert (a.steps, a.warmup, a.variants, a.kernel_timing) == (20, 5, 1, 1)
    c1 = bench.with_defaults(args, "c1", "paper", None, None, None, cpu=False)
    assert (c1.steps, c1.warmup, c1.variants, c1.kernel_timing, c1.cdc, c1.no_cpu_baseline) == (200, 20, 8, 4, "paper", True)
    assert args.steps is None                                   # the caller's namespace is left alone


def test_variant_runs_only_set_known_flags():
    known = set(vars(bench.build_parser().parse_args([])))
    for flags in bench.EXTRAS:
        assert "what" in flags and set(flags) - {"what"} <= known, flags
        assert flags.get("workload", "c2") in bench.DEFAULTS


def test_more_than_one_gpu_is_refused():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True)
    assert r.returncode == 2 and "ONE GPU" in r.stderr and r.stdout == ""


def test_stored_traffic_profiles_have_what_the_bench_line_reads():
    import glob
    import json
    files = sorted(glob.glob(os.path.join(ROOT, "profiles", "*_traffic.json")))
    assert files, "the bench line's roofline.traffic comes from these"
    for f in files:
        t = json.load(open(f))
        assert t["kernel"].startswith("reattach_rows"), f
        ratio = t["hbm_bytes_per_launch"] / t["algorithmic_bytes_per_launch"]
        assert 0.99 < ratio < 1.03 and abs(ratio - t["traffic_over_algorithmic"]) < 1e-9, (f, ratio)
        assert 1.9 < t["fetch_scale"] < 2.1 and 0.99 < t["write_scale"] < 1.01, f     # the plain copy's yardstick

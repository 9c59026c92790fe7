"""CPU checks of the shared input generators and of bench.py's command-line contract."""
import os
import subprocess
import sys

import numpy as np

import workloads as W

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_counter_fill_is_the_same_stream_everywhere():
    import torch

    ref = W.fills.counter_bytes_numpy(7, 0, 5000)
    # any slice, any gather, and the chunked torch builder give the same bytes
    assert np.array_equal(W.fills.counter_bytes_numpy(7, 123, 777), ref[123:900])
    idx = np.array([0, 1, 7, 8, 9, 4095, 4999])
    assert np.array_equal(W.fills.counter_byte_at(7, idx), ref[idx])
    assert np.array_equal(W.fills.counter_bytes_torch(7, 5000, "cpu", chunk_words=37).numpy(), ref)
    assert not np.array_equal(W.fills.counter_bytes_numpy(8, 0, 5000), ref)
    # roughly uniform bytes
    counts = np.bincount(W.fills.counter_bytes_numpy(7, 0, 1 << 20), minlength=256)
    assert counts.min() > 3500 and counts.max() < 4700


def test_sweep_shapes_follow_the_stated_rule():
    # packed size fixed; a1 >= a2, both powers of two, a1 <= 512; the allocation grows with a2
    for packed in (1 << 20, 1 << 26):
        for p in W.configs.cfg2_sweep(packed):
            a0, a1, a2 = p["a"]
            assert a0 * a1 * a2 == packed == p["packed_bytes"]
            assert a1 >= a2 or a1 == 512
            assert a1 <= 512 and a1 & (a1 - 1) == 0 and a2 & (a2 - 1) == 0
            assert p["e"] == (512, 512, max(512, a2)) and p["alloc_bytes"] == 512 * 512 * max(512, a2)
    assert [p["a"] for p in W.configs.cfg2_sweep(1 << 20)][:5] == [
        (1, 512, 2048), (2, 512, 1024), (4, 512, 512), (8, 512, 256), (16, 256, 256)]
    assert W.configs.cfg2_point(1, 1 << 26)["alloc_bytes"] == 32 << 30
    assert W.configs.cfg2_point(16, 1 << 26, a1_cap=256)["a"] == (16, 256, 16384)


def test_halo_regions_tile_the_ghost_shell():
    c = W.configs.cfg3(16, 2)
    n = 16
    seen = np.zeros((n, n, n), dtype=np.int32)
    for reg in c["ghost_region_for_send"]:
        seen[tuple(slice(a, b) for a, b in reg)] += 1
    shell = np.ones((n, n, n), dtype=bool)
    shell[2:-2, 2:-2, 2:-2] = False
    assert (seen[shell] == 1).all() and (seen[~shell] == 0).all()      # 26 ghost regions = the shell, once
    sent = np.zeros((n, n, n), dtype=np.int32)
    for reg in c["send_region"]:
        sent[tuple(slice(a, b) for a, b in reg)] += 1
    assert (sent[shell] == 0).all() and sent.max() == 7                 # interior only; corners go 7 ways
    assert len(W.configs.halo_directions()) == 26


def test_bench_refuses_more_than_one_gpu():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True,
                       text=True, timeout=120)
    assert r.returncode == 2
    assert "one GPU" in r.stderr and r.stdout.strip() == ""


def test_bench_final_line_is_compact_and_complete():
    """The line the benchmark ends with must survive a reader that keeps only a few KB of stdout:
    a result with everything long in it still formats to less than 2000 characters with the contract's keys."""
    import json

    import bench

    long_plan = " + ".join(["4 x [tile W=1 ux=1 ur=1 nt=6 bx=1 n0=1 back=0 rows=16777216 nrd=1 blocks=65536 grid=256]"] * 6)
    out = {
        "metric": "pack/unpack GB/s (read+write) and % of MI355X HBM peak; canonicalize us/type", "value": 392.11,
        "unit": "GB/s", "n_gpus": 1, "steps": 30, "warmup": 5, "ms_per_step": 6.8412, "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": "u8", "data": "synthetic",
        "config": {"workload": "3D strided-block sweep, a0 in {1..512}, 64 MiB packed per point, "
                               "512x512xE2 byte allocation, pack+unpack of all 10 points per step",
                   "packed_bytes_per_point": 1 << 26, "points": 10, "overrides": [], "bytes_per_step": 2684354560,
                   "frac_of_hbm_peak": 0.049},
        "roofline": {"bound": "hbm", "kernel": "prefetch_kernel + tile_kernel<0,1,1,true,1,6> (unpack a0=1)",
                     "achieved": 75.6, "peak": 8000.0, "unit": "GB/s", "frac": 0.0095, "avg_launch_us": 1774.9,
                     "algorithmic_bytes_per_launch": 134217728, "launches_per_call": 8, "traffic": 2280238262,
                     "traffic_rate_gbs": 1284.7, "limit": "x" * 200, "plan": long_plan, "note": "y" * 3000},
        "kernels": [{"plan": long_plan}] * 20, "extras": {"z": "w" * 20000}, "other_workloads": {"q": ["r" * 100] * 100},
        "cpu_baseline": {"value": 4.012, "unit": "GB/s", "cores": 16, "cpu_model": "AMD EPYC 9575F 64-Core Processor",
                         "kind": "oracle", "single_thread_value": 0.42, "sample": "s" * 180},
        "detail": "gpurun_out/bench_detail.json",
    }
    line = bench.final_line(out)
    assert len(line) < 2000 and "\n" not in line
    got = json.loads(line)
    for key in ("metric", "value", "unit", "n_gpus", "steps", "warmup", "ms_per_step", "higher_is_better", "scaling",
                "vs_baseline", "dtype", "data", "config", "roofline", "cpu_baseline"):
        assert key in got, key
    assert got["config"]["workload"].startswith("3D strided-block sweep")
    for key in ("bound", "kernel", "achieved", "peak", "unit", "frac", "avg_launch_us", "algorithmic_bytes_per_launch",
                "launches_per_call", "traffic"):
        assert key in got["roofline"], key
    for key in ("value", "unit", "cores", "cpu_model", "kind", "sample"):
        assert key in got["cpu_baseline"], key
    assert "kernels" not in got and "extras" not in got and "other_workloads" not in got
    assert abs(got["roofline"]["frac"] - got["roofline"]["achieved"] / got["roofline"]["peak"]) < 1e-3
    # free text far beyond anything the benchmark writes is shortened, never fatal
    out["roofline"]["limit"] = "x" * 5000
    out["cpu_baseline"]["sample"] = "s" * 5000
    out["config"]["overrides"] = ["nt=3"] * 400
    line = bench.final_line(out)
    assert len(line) < 2000 and json.loads(line)["roofline"]["frac"] == 0.0095


def test_bench_names_the_kernel_a_plan_line_runs():
    import bench

    assert bench.kernel_name("tile W=1 ux=1 ur=1 nt=6 bx=1 n0=1 back=0 rows=16777216 nrd=1 blocks=65536 grid=256",
                             "unpack") == "tile_kernel<0,1,1,true,1,6>"
    assert bench.kernel_name("tile W=16 ux=4 ur=1 nt=3 bx=256 n0=4194304 back=0 rows=1 nrd=0 blocks=4096",
                             "pack") == "tile_kernel<4,4,1,false,1,3>"
    assert bench.kernel_name("tile W=4 ux=1 ur=4 nt=3 bx=8 n0=6 back=0 rows=45 nrd=3 blocks=1", "pack") == \
        "tile_kernel<2,1,4,false,0,3>"
    assert bench.kernels_of("prefetch bytes=16777216 tile=256 blocks=65536 grid=2048\n"
                            "tile W=1 ux=1 ur=1 nt=6 bx=1 n0=1 back=0 rows=16777216 nrd=1 blocks=65536 grid=256\n"
                            "prefetch bytes=16777216 tile=256 blocks=65536 grid=2048\n", "unpack") == \
        "prefetch_kernel + tile_kernel<0,1,1,true,1,6>"


def test_bench_override_defaults_are_values_the_library_takes():
    # bench.py puts a call's own overrides back to these after the call: each must be a key and value
    # tp_set_override accepts, and the planner's own default for it
    import bench
    from paper_2012_14363_amd import binding as tp

    for key, value in bench.OVERRIDE_DEFAULTS.items():
        tp.set_override(key, value)
    assert bench.OVERRIDE_DEFAULTS["stage_bytes"] == 16 << 20 and bench.OVERRIDE_DEFAULTS["stage"] == -1
    args = bench.parse_args(["--points", "pack:32,unpack:1@stage=0@unpack_rule=0", "--steps", "3"])
    assert args.points == "pack:32,unpack:1@stage=0@unpack_rule=0" and args.steps == 3 and args.gpus == 1

#!/usr/bin/env python3
"""Benchmark of the pack/unpack hot path on one MI355X.

Workload (config.workload): the 3D strided-block sweep - a0 x a1 x a2 byte
sub-blocks of a 512 x 512 x e2 byte allocation, a0 in {1,...,512}, 64 MiB packed
per point.  One step = for every one of the 10 points: build and commit the
datatype (translate, canonicalize, StridedBlock, plan), pack it, and - after all
packs - unpack every point back into its typed buffer; the a0 = 512 point is the
fully dense 1D path.  Calls are enqueued with the *_async entry points and the
step ends with one stream synchronize.  Inputs are resident in HBM before the
timed region.  value = bytes read + bytes written by the method (2 x packed
bytes per pack or unpack) / wall time.

The last line of stdout is ONE compact JSON object (below 2 KB): metric, value,
ms_per_step, config, `roofline` for the call that takes most of the step, and
`cpu_baseline`, the CPU oracle on a bounded sample of the same sweep.  Everything
else (every sweep point, the secondary workloads) goes to the file --detail names.
"""
from __future__ import annotations

import argparse
import json
import os
import subprocess
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0
PACKED_BYTES = 1 << 26


def parse_args(argv=None):
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=30)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--packed-bytes", type=int, default=PACKED_BYTES, help="packed bytes per sweep point")
    ap.add_argument("--override", action="append", default=[], metavar="KEY=VALUE",
                    help="planner override passed to tp_set_override (ablations), e.g. nt=0 or word=4")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-extras", action="store_true", help="skip the secondary measurements")
    ap.add_argument("--detail", default=os.path.join(ROOT, "gpurun_out", "bench_detail.json"),
                    help="file that receives the full result (per-point table, secondary workloads)")
    ap.add_argument("--verbose", action="store_true", help="print the stage the run is in to stderr")
    ap.add_argument("--points", default="", metavar="OP:A0[@KEY=VALUE...],...",
                    help="run only these calls of the sweep in the step, in this order, e.g. pack:32,unpack:1,unpack:1@stage=0 "
                         "(profiling and ablation runs; a call's @overrides hold for that call only; the printed value "
                         "then is not the benchmark's)")
    return ap.parse_args(argv)


def summarise_plan(text: str):
    """A call's plan as one line: equal launches (a staged unpack repeats a read-only pass and a store pass
    per 16 MiB chunk) are counted instead of repeated.  Returns (summary, number of launches)."""
    lines = text.strip().splitlines()
    order, count = [], {}
    for ln in lines:
        if ln not in count:
            order.append(ln)
        count[ln] = count.get(ln, 0) + 1
    return " + ".join(ln if count[ln] == 1 else f"{count[ln]} x [{ln}]" for ln in order), len(lines)


def sector_bound_fraction(run: int, granule: int = 128) -> float:
    """Reachable fraction of peak for the algorithmic metric when every run of `run` bytes on the
    strided side costs whole `granule`-byte memory transactions: 2r / (g*ceil(r/g) + r).
    Measured on MI355X (FETCH_SIZE): a strided read brings in whole 128-byte lines."""
    g = granule
    return 2.0 * run / (g * ((run + g - 1) // g) + run)


# HBM bytes per call of the sweep's points at 64 MiB packed, from rocprofv3 --pmc FETCH_SIZE and WRITE_SIZE
# runs of this script (profiles/tile_kernel_strided_block_sweep_64MiB_hbm_traffic.md): counter KiB x 1024 x the
# factor a plain 64 MiB copy calibrates (FETCH_SIZE reads half the known bytes: x2; WRITE_SIZE: x1).
# Keyed by (op, a0): the plan the call had when the counters were read (tp_last_plan, summarised), bytes
# fetched, bytes written.  A point whose plan differs today reports no traffic rather than a stale one.
MEASURED_TRAFFIC = {
    ('pack', 1): {"plan": 'tile W=1 ux=1 ur=4 nt=3 bx=1 n0=1 back=0 rows=67108864 nrd=1 blocks=65536',
                   "fetch": 8585916908, "write": 72429112},
    ('pack', 2): {"plan": 'tile W=1 ux=1 ur=4 nt=3 bx=2 n0=2 back=0 rows=33554432 nrd=1 blocks=65536',
                   "fetch": 4293019034, "write": 72044646},
    ('pack', 4): {"plan": 'tile W=1 ux=1 ur=4 nt=3 bx=4 n0=4 back=0 rows=16777216 nrd=1 blocks=65536',
                   "fetch": 2146530243, "write": 70420976},
    ('pack', 8): {"plan": 'tile W=2 ux=1 ur=4 nt=3 bx=4 n0=4 back=0 rows=8388608 nrd=1 blocks=32768',
                   "fetch": 1073278299, "write": 67045053},
    ('pack', 16): {"plan": 'tile W=4 ux=1 ur=4 nt=3 bx=4 n0=4 back=0 rows=4194304 nrd=1 blocks=16384',
                   "fetch": 536656485, "write": 67083416},
    ('pack', 32): {"plan": 'tile W=4 ux=1 ur=4 nt=3 bx=8 n0=8 back=0 rows=2097152 nrd=1 blocks=16384',
                   "fetch": 268343084, "write": 67062956},
    ('pack', 64): {"plan": 'tile W=16 ux=1 ur=4 nt=3 bx=4 n0=4 back=0 rows=1048576 nrd=1 blocks=4096',
                   "fetch": 134187918, "write": 67143391},
    ('pack', 128): {"plan": 'tile W=16 ux=1 ur=4 nt=3 bx=8 n0=8 back=0 rows=524288 nrd=1 blocks=4096',
                   "fetch": 67110143, "write": 67115769},
    ('pack', 256): {"plan": 'tile W=16 ux=1 ur=4 nt=3 bx=16 n0=16 back=0 rows=262144 nrd=1 blocks=4096',
                   "fetch": 67109888, "write": 67113595},
    ('pack', 512): {"plan": 'tile W=16 ux=4 ur=1 nt=3 bx=256 n0=4194304 back=0 rows=1 nrd=0 blocks=4096',
                   "fetch": 67108864, "write": 67108864},
    ('unpack', 1): {"plan": '4 x [prefetch bytes=16777216 tile=256 blocks=65536 grid=1536] + 4 x [tile W=1 ux=1 ur=1 nt=6 bx=1 n0=1 back=0 rows=16777216 nrd=1 blocks=65536 grid=192]',
                   "fetch": 134391726, "write": 2145441687},
    ('unpack', 2): {"plan": '4 x [prefetch bytes=16777216 tile=512 blocks=32768 grid=1536] + 4 x [tile W=2 ux=1 ur=1 nt=6 bx=1 n0=1 back=0 rows=8388608 nrd=1 blocks=32768 grid=192]',
                   "fetch": 134391726, "write": 1072720844},
    ('unpack', 4): {"plan": '4 x [prefetch bytes=16777216 tile=1024 blocks=16384 grid=1536] + 4 x [tile W=4 ux=1 ur=1 nt=6 bx=1 n0=1 back=0 rows=4194304 nrd=1 blocks=16384 grid=192]',
                   "fetch": 134391726, "write": 536360422},
    ('unpack', 8): {"plan": '4 x [prefetch bytes=16777216 tile=2048 blocks=8192 grid=1536] + 4 x [tile W=8 ux=1 ur=1 nt=6 bx=1 n0=1 back=0 rows=2097152 nrd=1 blocks=8192 grid=192]',
                   "fetch": 134391726, "write": 268180211},
    ('unpack', 16): {"plan": '4 x [prefetch bytes=16777216 tile=4096 blocks=4096 grid=1536] + 4 x [tile W=16 ux=1 ur=1 nt=6 bx=1 n0=1 back=0 rows=1048576 nrd=1 blocks=4096 grid=192]',
                   "fetch": 134334409, "write": 134090105},
    ('unpack', 32): {"plan": 'tile W=4 ux=1 ur=1 nt=7 bx=8 n0=8 back=0 rows=2097152 nrd=1 blocks=65536',
                   "fetch": 67102723, "write": 67045053},
    ('unpack', 64): {"plan": 'tile W=8 ux=1 ur=1 nt=7 bx=8 n0=8 back=0 rows=1048576 nrd=1 blocks=32768',
                   "fetch": 67096582, "write": 67045053},
    ('unpack', 128): {"plan": 'tile W=16 ux=1 ur=4 nt=3 bx=8 n0=8 back=0 rows=524288 nrd=1 blocks=4096',
                   "fetch": 67104770, "write": 67144926},
    ('unpack', 256): {"plan": 'tile W=16 ux=1 ur=4 nt=3 bx=16 n0=16 back=0 rows=262144 nrd=1 blocks=4096',
                   "fetch": 67104898, "write": 67110910},
    ('unpack', 512): {"plan": 'tile W=16 ux=4 ur=1 nt=3 bx=256 n0=4194304 back=0 rows=1 nrd=0 blocks=4096',
                   "fetch": 67100676, "write": 67120117},
}


# what tp_set_override keys are reset to after a call that ran under its own overrides (--points ...@key=value)
OVERRIDE_DEFAULTS = {"stage": -1, "unpack_rule": 1, "nt": -1, "word": 0, "ur": -1, "xpose": 1, "narrow_partial_rows": 1,
                     "stage_bytes": 16 << 20, "stage_grid": 0, "grid": 0}


def kernel_name(plan_line: str, op: str) -> str:
    """The kernel instantiation a line of tp_last_plan() names, as rocprofv3 prints it (short form)."""
    if plan_line.startswith("prefetch"):
        return "prefetch_kernel"
    if plan_line.startswith("xpose"):
        return "xpose_kernel"
    f = dict(kv.split("=") for kv in plan_line.split()[1:] if "=" in kv)
    wlog2 = int(f["W"]).bit_length() - 1
    nrd = int(f["nrd"])
    nrd = 1 if nrd <= 1 else 2 if nrd == 2 else 0
    return f"tile_kernel<{wlog2},{f['ux']},{f['ur']},{'true' if op == 'unpack' else 'false'},{nrd},{f['nt']}>"


def kernels_of(plan_text: str, op: str) -> str:
    names = []
    for ln in plan_text.strip().splitlines():
        n = kernel_name(ln, op)
        if n not in names:
            names.append(n)
    return " + ".join(names)


def cpu_model_string() -> str:
    try:
        with open("/proc/cpuinfo") as f:
            for ln in f:
                if ln.lower().startswith("model name"):
                    return ln.split(":", 1)[1].strip()
    except OSError:
        pass
    return "unknown"


FINAL_KEYS = ("metric", "value", "unit", "n_gpus", "steps", "warmup", "ms_per_step", "higher_is_better", "scaling",
              "vs_baseline", "dtype", "data", "config", "roofline", "cpu_baseline", "canonicalize_us_per_type")
ROOFLINE_KEYS = ("bound", "kernel", "achieved", "peak", "unit", "frac", "avg_launch_us", "algorithmic_bytes_per_launch",
                 "launches_per_call", "traffic", "traffic_rate_gbs", "rows_per_ns", "copy_write_requests_per_ns",
                 "frac_of_copy_request_rate", "limit")
CPU_KEYS = ("value", "unit", "cores", "cpu_model", "kind", "single_thread_value", "sample")


def final_line(out: dict) -> str:
    """The one line the benchmark ends with: the contract's keys only, everything long left to the detail file."""
    line = {k: out[k] for k in FINAL_KEYS if k in out}
    line["roofline"] = {k: out["roofline"][k] for k in ROOFLINE_KEYS if k in out["roofline"]}
    if "cpu_baseline" in out:
        line["cpu_baseline"] = {k: out["cpu_baseline"][k] for k in CPU_KEYS if k in out["cpu_baseline"]}
    if "detail" in out:
        line["detail"] = out["detail"]
    text = json.dumps(line, separators=(",", ":"))
    # never lose the line to its length: shorten the free-text fields first, then drop them
    for cut in (160, 60, 0):
        if len(text) < 2000:
            break
        for obj, key in ((line["roofline"], "limit"), (line.get("cpu_baseline", {}), "sample"), (line["config"], "overrides"),
                         (line["config"], "only")):
            if key in obj:
                if cut and isinstance(obj[key], str):
                    obj[key] = obj[key][:cut]
                else:
                    del obj[key]
        text = json.dumps(line, separators=(",", ":"))
    return text


def main(argv=None):
    args = parse_args(argv)
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only; --gpus N with N > 1 is not supported "
              "(no collectives or sharding in this path).", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch

    import workloads as W
    from paper_2012_14363_amd import binding as tp

    assert torch.cuda.is_available(), "bench.py needs a GPU"

    def stage(text):
        if args.verbose:
            print(f"bench.py: {text}", file=sys.stderr, flush=True)
    if args.points:
        args.no_extras = True   # the secondary workloads live in the full arena
    tp.lib()
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    stream = torch.cuda.current_stream()

    # ---------------------------------------------------------------- the step's calls
    points = W.configs.cfg2_sweep(args.packed_bytes)
    # one call = (op, index of the sweep point, overrides in force for that call only)
    if args.points:
        calls = []
        for item in args.points.split(","):
            head, *ovr = item.split("@")
            op, _, a0 = head.partition(":")
            assert op in ("pack", "unpack") and int(a0) in W.configs.A0_SWEEP, item
            assert all(kv.partition("=")[0] in OVERRIDE_DEFAULTS for kv in ovr), item
            calls.append((op, W.configs.A0_SWEEP.index(int(a0)), tuple(kv.partition("=")[::2] for kv in ovr)))
    else:
        calls = [("pack", i, ()) for i in range(len(points))] + [("unpack", i, ()) for i in range(len(points))]
    used = sorted({i for _, i, _ in calls})

    # ---------------------------------------------------------------- inputs, resident in HBM
    align = 1 << 21
    bases, total = {}, 0
    for i in used:
        bases[i] = total
        total += (points[i]["alloc_bytes"] + align - 1) // align * align
    stage(f"filling {total >> 20} MiB of typed buffers")
    arena = W.fills.counter_bytes_torch(W.configs.SEED_BASE + 1, total, dev)
    packed = {i: torch.zeros(points[i]["packed_bytes"], dtype=torch.uint8, device=dev) for i in used}
    torch.cuda.synchronize()
    for kv in args.override:
        key, _, val = kv.partition("=")
        tp.set_override(key, val)

    def one_call(op, i, ovr, h, synchronous=False):
        for key, val in ovr:
            tp.set_override(key, val)
        p = points[i]
        if op == "pack":
            (tp.pack if synchronous else tp.pack_async)(arena.data_ptr() + bases[i], 1, h, packed[i], p["packed_bytes"], 0, stream)
        else:
            (tp.unpack if synchronous else tp.unpack_async)(packed[i], p["packed_bytes"], 0, arena.data_ptr() + bases[i], 1, h, stream)
        for key, _ in ovr:
            tp.set_override(key, OVERRIDE_DEFAULTS[key])

    def run_step(events=None):
        handles = {}
        for c, (op, i, ovr) in enumerate(calls):
            if i not in handles:   # construct + commit, when the step first needs the type
                handles[i] = tp.type_from_recipe(points[i]["recipe"])
            if events is not None:
                events[c][0].record(stream)
            one_call(op, i, ovr, handles[i])
            if events is not None:
                events[c][1].record(stream)
        stream.synchronize()                               # completion
        for h in handles.values():
            if h >= 12:
                tp.type_free(h)

    stage("warm-up steps")
    for _ in range(args.warmup):
        run_step()
    stage("plans")
    handles = {i: tp.type_from_recipe(points[i]["recipe"]) for i in used}
    if not args.points:
        for i in used:   # every unpack restores the bytes its pack took
            one_call("pack", i, (), handles[i], synchronous=True)
    plans = []
    for op, i, ovr in calls:
        one_call(op, i, ovr, handles[i], synchronous=True)
        plans.append(tp.last_plan().strip())

    def new_events():
        return [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in calls]

    all_events = [new_events() for _ in range(args.steps)]
    torch.cuda.synchronize()
    stage("timed steps")
    t0 = time.perf_counter()
    for k in range(args.steps):
        run_step(all_events[k])
    torch.cuda.synchronize()
    t1 = time.perf_counter()

    step_s = (t1 - t0) / args.steps

    # reference: a dense 1 GiB copy through the library (the 1D path), large enough for launch and event
    # overhead to vanish; a dense copy leaves L2 as one 64-byte write request per 64 bytes
    gib = 1 << 30
    stage("1 GiB reference copy")
    ref_src = [torch.empty(gib, dtype=torch.uint8, device=dev).fill_(i + 1) for i in range(2)]
    ref_dst = torch.empty(gib, dtype=torch.uint8, device=dev)
    ref_t = tp.type_from_recipe(W.contiguous(gib, W.BYTE))
    ref_ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(6)]
    for j, (e0, e1) in enumerate(ref_ev):
        e0.record(stream)
        tp.pack_async(ref_src[j % 2], 1, ref_t, ref_dst, gib, 0, stream)
        e1.record(stream)
    torch.cuda.synchronize()
    ref_us = sorted(e0.elapsed_time(e1) for e0, e1 in ref_ev[2:])[1] * 1e3
    copy_1gib = {"us": round(ref_us, 1), "gbs": round(2 * gib / ref_us / 1e3, 1), "write_requests_per_ns": gib / 64 / ref_us / 1e3}
    tp.type_free(ref_t)
    del ref_src, ref_dst
    stage("results")
    bytes_per_step = sum(2 * points[i]["packed_bytes"] for _, i, _ in calls)   # read + write
    value = bytes_per_step / step_s / 1e9

    # per-call device times from the HIP events recorded inside the timed region
    use_traffic = args.packed_bytes == PACKED_BYTES and not args.override
    kernels = []
    for c, (op, i, ovr) in enumerate(calls):
        p = points[i]
        ms = [all_events[k][c][0].elapsed_time(all_events[k][c][1]) for k in range(args.steps)]
        avg_us = 1e3 * sum(ms) / len(ms)
        srt = sorted(ms)
        alg = 2 * p["packed_bytes"]
        plan, nlaunch = summarise_plan(plans[c])
        run = p["a"][0] if p["a"][0] < 512 else p["packed_bytes"]
        k = {
            "op": op, "a": list(p["a"]), "kernel": kernels_of(plans[c], op), "plan": plan,
            "launches_per_call": nlaunch, "avg_us": round(avg_us, 2),
            "median_us": round(1e3 * srt[len(srt) // 2], 2), "min_us": round(1e3 * srt[0], 2),
            "algorithmic_bytes": alg, "gbs": round(alg / avg_us / 1e3, 1),
            "frac_of_peak": round(alg / avg_us / 1e3 / HBM_PEAK_GBS, 4),
            "sector_bound_frac_g128": round(sector_bound_fraction(run), 4),
        }
        if ovr:
            k["overrides"] = ["=".join(kv) for kv in ovr]
        m = MEASURED_TRAFFIC.get((op, p["a"][0]))
        if m and use_traffic and not ovr and m["plan"] == plan:   # HBM bytes actually moved, next to the algorithmic rate
            k["hbm_traffic_fetch_write"] = [m["fetch"], m["write"]]
            k["hbm_traffic_gbs"] = round((m["fetch"] + m["write"]) / avg_us / 1e3, 1)
            k["hbm_traffic_frac_of_peak"] = round((m["fetch"] + m["write"]) / avg_us / 1e3 / HBM_PEAK_GBS, 4)
        kernels.append(k)
    # the same-size plain copy through the same kernel (the dense a0 = 512 point) is the copy ceiling
    ceiling = {k["op"]: k["gbs"] for k in kernels if k["a"][0] == 512 and "overrides" not in k}
    for k in kernels:
        if k["op"] in ceiling:
            k["frac_of_copy_ceiling"] = round(k["gbs"] / ceiling[k["op"]], 4)
    dominant = max(kernels, key=lambda k: k["avg_us"])
    roofline = {
        "bound": "hbm", "kernel": f"{dominant['kernel']} ({dominant['op']} a0={dominant['a'][0]})",
        "achieved": dominant["gbs"], "peak": HBM_PEAK_GBS, "unit": "GB/s",
        "frac": round(dominant["gbs"] / HBM_PEAK_GBS, 4),
        "avg_launch_us": dominant["avg_us"], "algorithmic_bytes_per_launch": dominant["algorithmic_bytes"],
        "launches_per_call": dominant["launches_per_call"],
        "traffic": None,
        "sector_bound_frac_g128": dominant["sector_bound_frac_g128"],
        "plan": dominant["plan"],
    }
    if dominant["launches_per_call"] > 1:
        roofline["limit"] = "avg_launch_us, achieved and traffic are per call, all of its launches included"
    if dominant["op"] == "unpack" and dominant["a"][0] < 64:
        # Rows below 64 bytes cost one masked 32-byte write request each, so the call is bound by the write
        # requests per second the memory path takes, not by bytes: compare its rows/ns with the 64-byte
        # write requests/ns of a dense 1 GiB copy through the same library, timed in this same run.
        rows = dominant["algorithmic_bytes"] // 2 // dominant["a"][0]
        roofline["rows_per_ns"] = round(rows / dominant["avg_us"] / 1e3, 2)
        roofline["copy_write_requests_per_ns"] = round(copy_1gib["write_requests_per_ns"], 2)
        roofline["frac_of_copy_request_rate"] = round(roofline["rows_per_ns"] / copy_1gib["write_requests_per_ns"], 3)
        roofline["limit"] = ("one masked 32-byte write request per row: bound by the write requests/s of the memory path "
                             "(see frac_of_copy_request_rate), 1 useful byte of 32 per request; figures are per call, all launches included")
    if "hbm_traffic_fetch_write" in dominant:
        roofline["traffic"] = sum(dominant["hbm_traffic_fetch_write"])
        roofline["traffic_fetch_write"] = dominant["hbm_traffic_fetch_write"]
        roofline["traffic_rate_gbs"] = dominant["hbm_traffic_gbs"]

    out = {
        "metric": "pack/unpack GB/s (read+write) and % of MI355X HBM peak; canonicalize us/type", "value": round(value, 2), "unit": "GB/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(step_s * 1e3, 4),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "u8", "data": "synthetic",
        "config": {"workload": "3D strided-block sweep, a0 in {1..512}, 64 MiB packed per point, "
                               "512x512xE2 byte allocation, pack+unpack of all 10 points per step",
                   "packed_bytes_per_point": args.packed_bytes, "points": len(points),
                   "overrides": args.override, "bytes_per_step": bytes_per_step, "frac_of_hbm_peak": round(value / HBM_PEAK_GBS, 4)},
        "roofline": roofline,
        "copy_1GiB": copy_1gib,
        "kernels": kernels,
    }
    if args.points:
        out["config"]["only"] = args.points

    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(W, np)
    if not args.no_extras:
        out["extras"] = extras(W, tp, torch, np, dev, stream)
        out["other_workloads"] = other_workloads(W, tp, torch, arena, dev, stream)
    # the metric's second half in the final line: commit (translate + canonicalize + StridedBlock) per type
    rows = out.get("extras", {}).get("canonicalize_us_per_type")
    if isinstance(rows, list) and rows:
        commits = sorted(r["commit_us"] for r in rows)
        out["canonicalize_us_per_type"] = {"median": commits[len(commits) // 2], "max": commits[-1], "types": len(rows),
                                           "statistic": "trimean of 30000 commits per type"}
    try:
        os.makedirs(os.path.dirname(os.path.abspath(args.detail)), exist_ok=True)
        with open(args.detail, "w") as f:
            json.dump(out, f, indent=1)
        out["detail"] = os.path.relpath(args.detail, ROOT)
    except OSError as e:   # the detail file is a convenience; the line below is the result
        print(f"bench.py: detail file not written: {e}", file=sys.stderr)
    print(final_line(out), flush=True)


def cpu_baseline(W, np):
    """The CPU oracle (C twin) on a bounded sample of the same sweep: 8 MiB packed per point
    (the outermost dimension cut to 1/8), pack + unpack of all 10 points, all host cores."""
    from oracle import typemap_c as cc

    cores = len(os.sched_getaffinity(0))
    sample_bytes = 1 << 23
    pts = W.configs.cfg2_sweep(sample_bytes)
    biggest = max(p["alloc_bytes"] for p in pts)
    src = np.empty(biggest, dtype=np.uint8)
    src.view(np.uint64)[:] = np.arange(biggest // 8, dtype=np.uint64) * np.uint64(0x9E3779B97F4A7C15)
    outs = [np.zeros(p["packed_bytes"], np.uint8) for p in pts]
    for p, o in zip(pts[-2:], outs[-2:]):  # warm the code path
        cc.pack(src, 0, 1, p["recipe"], o, 0, nthreads=cores)
    t0 = time.perf_counter()
    reps = 0
    while True:
        for p, o in zip(pts, outs):
            cc.pack(src, 0, 1, p["recipe"], o, 0, nthreads=cores)
        for p, o in zip(pts, outs):
            cc.unpack(o, 0, src, 0, 1, p["recipe"], nthreads=cores)
        reps += 1
        if time.perf_counter() - t0 > 8.0:
            break
    dt = time.perf_counter() - t0
    moved = reps * sum(2 * p["packed_bytes"] for p in pts) * 2
    t0 = time.perf_counter()
    for p, o in zip(pts, outs):
        cc.pack(src, 0, 1, p["recipe"], o, 0, nthreads=1)
    for p, o in zip(pts, outs):
        cc.unpack(o, 0, src, 0, 1, p["recipe"], nthreads=1)
    single = sum(2 * p["packed_bytes"] for p in pts) * 2 / (time.perf_counter() - t0) / 1e9
    return {"value": round(moved / dt / 1e9, 3), "unit": "GB/s", "cores": cores, "cpu_model": cpu_model_string(),
            "kind": "oracle", "single_thread_value": round(single, 3),
            "sample": f"same sweep at 8 MiB packed per point (outermost dimension / 8), {reps} passes of "
                      f"pack+unpack over all 10 points, {cores} threads over the outermost loop"}


def extras(W, tp, torch, np, dev, stream):
    """Secondary measurements: copy ceiling, synchronous-call latency, commit time per type."""
    res = {}

    def timed(fn, n=20, warm=3):
        for _ in range(warm):
            fn()
        torch.cuda.synchronize()
        ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(n)]
        for a, b in ev:
            a.record(stream)
            fn()
            b.record(stream)
        torch.cuda.synchronize()
        ts = sorted(a.elapsed_time(b) for a, b in ev)
        return ts[len(ts) // 2] * 1e3  # median, us

    # copy ceiling: torch's device-to-device copy of 64 MiB, rotating over 1.5 GiB so caches do not help
    n = 1 << 26
    srcs = [torch.empty(n, dtype=torch.uint8, device=dev).fill_(i) for i in range(12)]
    dsts = [torch.empty(n, dtype=torch.uint8, device=dev) for _ in range(12)]
    k = [0]

    def copy():
        dsts[k[0] % 12].copy_(srcs[k[0] % 12])
        k[0] += 1
    us = timed(copy, n=24)
    res["copy_ceiling_torch_64MiB"] = {"us": round(us, 2), "gbs": round(2 * n / us / 1e3, 1)}

    byte_t = tp.type_from_recipe(W.contiguous(n, W.BYTE))

    def own_copy():
        tp.pack_async(srcs[k[0] % 12], 1, byte_t, dsts[k[0] % 12], n, 0, stream)
        k[0] += 1
    us = timed(own_copy, n=24)
    res["copy_ceiling_tp_1d_64MiB"] = {"us": round(us, 2), "gbs": round(2 * n / us / 1e3, 1)}
    # the same copy without rotation: source and destination stay in the 256 MiB Infinity Cache
    us = timed(lambda: tp.pack_async(srcs[0], 1, byte_t, dsts[0], n, 0, stream), n=24)
    res["copy_64MiB_same_buffers_cache_assisted"] = {"us": round(us, 2), "gbs": round(2 * n / us / 1e3, 1)}
    # the same 64 MiB copy between odd addresses (source + 1, destination + 3), of an odd length:
    # unaligned 16-byte words against the byte-wide words that natural alignment would force
    odd = n - 65

    def unaligned():
        tp.pack_async(srcs[k[0] % 12].data_ptr() + 1, 1, odd_t, dsts[k[0] % 12].data_ptr() + 3, odd, 0, stream)
        k[0] += 1
    odd_t = tp.type_from_recipe(W.contiguous(odd, W.BYTE))
    us = timed(unaligned, n=24)
    res["copy_64MiB_odd_addresses"] = {"us": round(us, 2), "gbs": round(2 * odd / us / 1e3, 1),
                                      "plan": tp.last_plan().strip()}
    tp.set_override("word", 1)
    us = timed(unaligned, n=12)
    tp.set_override("word", 0)
    res["copy_64MiB_odd_addresses_bytewise"] = {"us": round(us, 2), "gbs": round(2 * odd / us / 1e3, 1)}
    # rows at odd addresses (typed + 1, packed + 3): 200-, 67- and 24-byte runs at 512-byte pitch; the unpack
    # also as it was planned before stores were written through (override unpack_rule = 0)
    for run in (200, 67, 24):
        rows_o = (48 << 20) // run
        t_o = tp.type_from_recipe(W.vector(rows_o, run, 512, W.BYTE))
        typed_o = [torch.empty(rows_o * 512 + 64, dtype=torch.uint8, device=dev).fill_(i + 1) for i in range(2)]
        entry = {}
        for label, toff, poff in (("aligned", 0, 0), ("typed+1_packed+3", 1, 3)):
            def pk(toff=toff, poff=poff):
                j = k[0] % 12
                tp.pack_async(typed_o[j % 2].data_ptr() + toff, 1, t_o, dsts[j].data_ptr() + poff, rows_o * run, 0, stream)
                k[0] += 1

            def un(toff=toff, poff=poff):
                j = k[0] % 12
                tp.unpack_async(dsts[j].data_ptr() + poff, rows_o * run, 0, typed_o[j % 2].data_ptr() + toff, 1, t_o, stream)
                k[0] += 1
            entry[label] = {"pack_us": round(timed(pk, n=12), 1), "unpack_us": round(timed(un, n=12), 1)}
            tp.set_override("unpack_rule", 0)
            try:
                entry[label]["unpack_us_nt_stores_four_rows_per_thread"] = round(timed(un, n=12), 1)
            finally:
                tp.set_override("unpack_rule", 1)
        res[f"rows_of_{run}B_at_512B_pitch_48MiB"] = entry
        del typed_o
    # unpack of 2^24 tiny rows at 512-byte pitch from twelve rotating sources: as planned (staged: packed bytes
    # brought into L2 per 16 MiB, stores written through, rows 512 bytes apart), written through but not
    # staged, and with plain streaming stores, four rows per thread
    rows_t = 1 << 24
    typed_t = torch.empty(rows_t * 512, dtype=torch.uint8, device=dev).fill_(1)
    entry = {}
    for run in (1, 4):
        t_t = tp.type_from_recipe(W.vector(rows_t, run, 512, W.BYTE))

        def un_t():
            j = k[0] % 12
            tp.unpack_async(dsts[j], rows_t * run, 0, typed_t, 1, t_t, stream)
            k[0] += 1
        one = {"staged_us": round(timed(un_t, n=10), 1)}
        try:
            tp.set_override("stage", 0)
            one["written_through_us"] = round(timed(un_t, n=10), 1)
            tp.set_override("unpack_rule", 0)
            one["streaming_stores_us"] = round(timed(un_t, n=10), 1)
        finally:
            tp.set_override("stage", -1)
            tp.set_override("unpack_rule", 1)
        one["staged_rows_per_ns"] = round(rows_t / one["staged_us"] / 1e3, 2)
        entry[f"{run}B_rows"] = one
    res["unpack_2p24_tiny_rows_at_512B_pitch"] = entry
    del typed_t
    del srcs, dsts

    # the runtime's own 2D copy (the DMA-engine route the paper lists as future work, Sec. 8) on the
    # same 2D shape as a sweep point: 64 MiB in 128-byte runs at 512-byte pitch, against this library
    try:
        import ctypes
        hip = ctypes.CDLL(os.path.join(os.path.dirname(torch.__file__), "lib", "libamdhip64.so"))
        hip.hipMemcpy2DAsync.argtypes = [ctypes.c_void_p, ctypes.c_size_t, ctypes.c_void_p, ctypes.c_size_t,
                                         ctypes.c_size_t, ctypes.c_size_t, ctypes.c_int, ctypes.c_void_p]
        hip.hipMemcpy2DAsync.restype = ctypes.c_int
        rows2d, width2d, pitch2d = 1 << 19, 128, 512
        src2d = [torch.empty(rows2d * pitch2d, dtype=torch.uint8, device=dev).fill_(i + 1) for i in range(4)]
        dst2d = [torch.empty(rows2d * width2d, dtype=torch.uint8, device=dev) for _ in range(4)]
        D2D = 3  # hipMemcpyDeviceToDevice

        def dma2d():
            j = k[0] % 4
            rc = hip.hipMemcpy2DAsync(dst2d[j].data_ptr(), width2d, src2d[j].data_ptr(), pitch2d, width2d, rows2d, D2D,
                                      stream.cuda_stream)
            assert rc == 0, rc
            k[0] += 1
        us_dma = timed(dma2d, n=12)
        t2d = tp.type_from_recipe(W.vector(rows2d, width2d, pitch2d, W.BYTE))

        def ours2d():
            j = k[0] % 4
            tp.pack_async(src2d[j], 1, t2d, dst2d[j], rows2d * width2d, 0, stream)
            k[0] += 1
        us_ours = timed(ours2d, n=12)
        same = bool(torch.equal(dst2d[0], src2d[0].view(rows2d, pitch2d)[:, :width2d].reshape(-1)))
        res["pack_2d_64MiB_128B_runs_vs_hipMemcpy2DAsync"] = {
            "hipMemcpy2DAsync_us": round(us_dma, 1), "tp_pack_us": round(us_ours, 1), "outputs_equal": same}
        del src2d, dst2d
    except Exception as e:  # a comparison point only
        res["pack_2d_64MiB_128B_runs_vs_hipMemcpy2DAsync"] = f"not measured: {e}"

    # an independent implementation of the narrowest sweep pattern (one byte per 512-byte row):
    # PyTorch's strided copy kernels on views of the same buffers.  If the masked-write rate were a
    # property of this library's kernel, another kernel would not share it.
    rows1, pitch1 = 1 << 24, 512
    typed1 = [torch.empty(rows1 * pitch1, dtype=torch.uint8, device=dev).fill_(7) for _ in range(2)]
    packed1 = torch.empty(rows1, dtype=torch.uint8, device=dev).fill_(9)
    t1 = tp.type_from_recipe(W.vector(rows1, 1, pitch1, W.BYTE))
    ops = {
        "torch_gather": lambda j: packed1.copy_(typed1[j].view(rows1, pitch1)[:, 0]),
        "tp_pack": lambda j: tp.pack_async(typed1[j], 1, t1, packed1, rows1, 0, stream),
        "torch_scatter": lambda j: typed1[j].view(rows1, pitch1)[:, 0].copy_(packed1),
        "tp_unpack": lambda j: tp.unpack_async(packed1, rows1, 0, typed1[j], 1, t1, stream),
    }
    narrow = {"rows": rows1, "pitch": pitch1, "run_bytes": 1}
    for name, op in ops.items():
        def rotating(op=op):
            op(k[0] % 2)
            k[0] += 1
        us = timed(rotating, n=8, warm=2)
        narrow[name + "_us"] = round(us, 1)
        narrow[name + "_rows_per_ns"] = round(rows1 / us / 1e3, 2)
    res["one_byte_rows_vs_torch_strided_copy"] = narrow
    del typed1, packed1

    # synchronous-call latency (launch + kernel + synchronize, the paper's timed region) on the small 2D vector
    c1 = W.configs.cfg1()
    buf = torch.zeros(c1["buffer_bytes"], dtype=torch.uint8, device=dev)
    out = torch.zeros(512, dtype=torch.uint8, device=dev)
    h = tp.type_from_recipe(c1["recipes"]["vector"])
    lat = []
    for _ in range(200):
        t0 = time.perf_counter()
        tp.pack(buf, 1, h, out, 512, 0, stream)
        lat.append(time.perf_counter() - t0)
    lat.sort()
    res["sync_pack_latency_us_2d_vector_512B"] = round(lat[len(lat) // 2] * 1e6, 2)

    # commit time per type: the plain-C program timing create and commit through the C ABI,
    # trimean of 30000 cycles per type (the statistic of the paper's Sec. 6.1)
    import tempfile

    # measured performance model (paper Sec. 4 / 6.3): measure the system, keep the table, and ask it
    # which way packed data should reach the host for a few shapes
    model_path = os.path.join(tempfile.mkdtemp(prefix="tp_model_"), "model.txt")
    t0 = time.perf_counter()
    tp.model_measure(stream)
    measure_s = time.perf_counter() - t0
    tp.model_save(model_path)
    # the saved table is plain text: "sizes n ...", "blocks m ...", then one line per primitive
    lines = {ln.split()[0]: ln.split()[1:] for ln in open(model_path).read().splitlines()}
    sizes = [float(v) for v in lines["sizes"][1:]]
    blocks = [float(v) for v in lines["blocks"][1:]]
    model = {"measure_seconds": round(measure_s, 2), "sizes": sizes, "blocks": blocks}
    for name in ("gpu_pack", "gpu_unpack", "host_pack", "host_unpack"):
        vals = np.array([float(v) for v in lines[name]]).reshape(len(sizes), len(blocks))
        model[name + "_us"] = np.round(vals * 1e6, 2).tolist()
    for name in ("d2h", "h2d"):
        model[name + "_us"] = np.round(np.array([float(v) for v in lines[name]]) * 1e6, 2).tolist()
    picks = []
    for label, recipe, count in (("64 KiB in 8-byte runs", W.vector(8192, 8, 512, W.BYTE), 1),
                                 ("4 MiB in 64-byte runs", W.vector(65536, 64, 512, W.BYTE), 1),
                                 ("4 MiB in 4 KiB runs", W.vector(1024, 4096, 8192, W.BYTE), 1),
                                 ("64 MiB in 4 KiB runs", W.vector(16384, 4096, 8192, W.BYTE), 1)):
        hh = tp.type_from_recipe(recipe)
        q = tp.model_query(hh, count)
        picks.append({"object": label, "host_pack_us": round(q["host_pack"] * 1e6, 1),
                      "gpu_pack_plus_d2h_us": round((q["gpu_pack"] + q["d2h"]) * 1e6, 1),
                      "to_host": "staged" if q["gpu_pack"] + q["d2h"] < q["host_pack"] else "one-shot"})
    model["to_host_choice"] = picks
    res["model"] = model

    exe = os.path.join(ROOT, "paper_2012_14363_amd", "commit_timing")
    if os.path.exists(exe):
        try:
            rows = json.loads(subprocess.run([exe, "30000", model_path], capture_output=True, text=True, timeout=120,
                                             check=True).stdout)
            select = [r for r in rows if r["type"].startswith("tp_model_select")]
            rows = [r for r in rows if not r["type"].startswith("tp_model_select")]
            if select:
                res["model"]["select_ns_per_query_memoised"] = select[0]["ns_per_query"]
            res["canonicalize_us_per_type"] = [
                {"type": r["type"], "shape": r["shape"], "canonical_dims": r["canonical_dims"],
                 "create_us": round(r["create_trimean_ns"] / 1e3, 3),
                 "commit_us": round(r["commit_trimean_ns"] / 1e3, 3)} for r in rows]
        except Exception as e:  # reported, never fatal for the benchmark line
            res["canonicalize_us_per_type"] = f"commit_timing failed: {e}"
    else:
        res["canonicalize_us_per_type"] = "commit_timing not built"
    res["resource_cache"] = resource_cache_timing(W, tp, torch, dev, stream)
    return res


def resource_cache_timing(W, tp, torch, dev, stream):
    """Paper Sec. 5: what a repeated request for a buffer, stream or event costs from the library's
    cache against what the runtime takes to create one, and what a pack call saves on buffers the
    cache knows (no memory-residency query)."""
    res = {}
    exe = os.path.join(ROOT, "paper_2012_14363_amd", "resource_timing")
    if os.path.exists(exe):
        try:
            rows = json.loads(subprocess.run([exe, "500000", "16"], capture_output=True, text=True, timeout=120,
                                             check=True).stdout)
            res["per_kind"] = [{"kind": r["kind"], "create_us": round(r["create_median_ns"] / 1e3, 2),
                                "cached_acquire_release_ns": r["cached_pair_ns"]} for r in rows]
        except Exception as e:  # reported, never fatal for the benchmark line
            res["per_kind"] = f"resource_timing failed: {e}"
    else:
        res["per_kind"] = "resource_timing not built"

    # host time of an enqueue-only pack call: both buffers leased from the cache vs. both torch's
    h = tp.type_from_recipe(W.vector(64, 8, 512, W.BYTE))
    size, ex = tp.type_size(h), tp.type_get_extent(h)[1]
    calls = 20000

    def per_call_us(src, dst):
        for _ in range(200):
            tp.pack_async(src, 1, h, dst, size, 0, stream)
        stream.synchronize()
        t0 = time.perf_counter()
        for _ in range(calls):
            tp.pack_async(src, 1, h, dst, size, 0, stream)
        dt = time.perf_counter() - t0
        stream.synchronize()
        return dt / calls * 1e6

    src_t = torch.zeros(ex, dtype=torch.uint8, device=dev)
    dst_t = torch.zeros(size, dtype=torch.uint8, device=dev)
    src_l = tp.resource_acquire(tp.TP_RES_DEVICE, ex)
    dst_l = tp.resource_acquire(tp.TP_RES_DEVICE, size)
    try:
        res["pack_async_host_us_per_call"] = {
            "queried_buffers": round(per_call_us(src_t.data_ptr(), dst_t.data_ptr()), 2),
            "leased_buffers": round(per_call_us(src_l, dst_l), 2),
            "calls": calls,
            "note": "512-byte object; the loop is Python + ctypes, equal on both sides; the difference is the "
                    "memory queries (one attribute and one bounds query per buffer)",
        }
    finally:
        tp.resource_release(tp.TP_RES_DEVICE, src_l)
        tp.resource_release(tp.TP_RES_DEVICE, dst_l)
        tp.resource_trim()
    return res


def other_workloads(W, tp, torch, arena, dev, stream):
    """The remaining workloads, timed the same way (HIP events on the launch stream, median), with the
    typed side taken from regions of the resident arena that rotate between repetitions so that no
    repetition finds its lines in the 256 MiB Infinity Cache.  Reported, not part of `value`."""
    res = {}
    GiB = 1 << 30

    def median_event_us(fn, reps):
        ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(reps)]
        for k, (a, b) in enumerate(ev):
            a.record(stream)
            fn(k)
            b.record(stream)
        torch.cuda.synchronize()
        ts = sorted(a.elapsed_time(b) for a, b in ev)
        return ts[len(ts) // 2] * 1e3

    def median_wall_us(fn, reps):
        ts = []
        for k in range(reps):
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            fn(k)
            ts.append(time.perf_counter() - t0)
        ts.sort()
        return ts[len(ts) // 2] * 1e6

    # ---- 3D sweep at 1 MiB packed: latency regime (launch + kernel + synchronize per call)
    rows = []
    out1 = [torch.zeros(1 << 20, dtype=torch.uint8, device=dev) for _ in range(8)]
    for p in W.configs.cfg2_sweep(1 << 20):
        h = tp.type_from_recipe(p["recipe"])
        span = p["alloc_bytes"]
        nreg = max(1, min(16, (8 * GiB) // span))
        pk = median_wall_us(lambda k: tp.pack(arena.data_ptr() + (k % nreg) * span, 1, h, out1[k % 8], 1 << 20, 0, stream), 30)
        up = median_wall_us(lambda k: tp.unpack(out1[k % 8], 1 << 20, 0, arena.data_ptr() + (k % nreg) * span, 1, h, stream), 30)
        pk_ev = median_event_us(lambda k: tp.pack_async(arena.data_ptr() + (k % nreg) * span, 1, h, out1[k % 8], 1 << 20, 0, stream), 30)
        up_ev = median_event_us(lambda k: tp.unpack_async(out1[k % 8], 1 << 20, 0, arena.data_ptr() + (k % nreg) * span, 1, h, stream), 30)
        rows.append({"a": list(p["a"]), "pack_sync_call_us": round(pk, 1), "unpack_sync_call_us": round(up, 1),
                     "pack_event_us": round(pk_ev, 1), "unpack_event_us": round(up_ev, 1),
                     "pack_gbs_event": round(2 * (1 << 20) / pk_ev / 1e3, 1)})
    res["sweep_1MiB"] = rows

    # ---- the 64 MiB sweep with a1 held at 256 so the canonical form stays 3D (the main sweep's
    # points all flatten to 2D because a1 reaches the 512-byte-pitch plane height)
    rows = []
    out64 = [torch.zeros(1 << 26, dtype=torch.uint8, device=dev) for _ in range(4)]
    for a0 in (16, 64, 256):
        p = W.configs.cfg2_point(a0, 1 << 26, a1_cap=256)
        h = tp.type_from_recipe(p["recipe"])
        span = p["alloc_bytes"]
        nreg = max(1, min(8, (16 * GiB) // span))
        pk = median_event_us(lambda k: tp.pack_async(arena.data_ptr() + (k % nreg) * span, 1, h, out64[k % 4], 1 << 26, 0, stream), 12)
        plan = tp.last_plan().strip()
        up = median_event_us(lambda k: tp.unpack_async(out64[k % 4], 1 << 26, 0, arena.data_ptr() + (k % nreg) * span, 1, h, stream), 12)
        rows.append({"a": list(p["a"]), "pack_us": round(pk, 1), "unpack_us": round(up, 1),
                     "pack_gbs": round(2 * (1 << 26) / pk / 1e3, 1), "unpack_gbs": round(2 * (1 << 26) / up / 1e3, 1),
                     "plan": plan})
    res["sweep_64MiB_3d_a1_256"] = rows
    del out64

    # ---- 2D objects of 512-byte pitch: construction (vector or subarray) and object count must not
    # matter (the paper's pack figure, Sec. 6.2): 4 MiB in total, runs of 64 bytes
    rows = []
    out4 = [torch.zeros(1 << 22, dtype=torch.uint8, device=dev) for _ in range(8)]
    for count in (1, 16, 256):
        nrows = (1 << 22) // 64 // count
        variants = {
            "vector": W.vector(nrows, 64, 512, W.BYTE),
            "subarray": W.subarray((nrows, 512), (nrows, 64), (0, 0), "C", W.BYTE),
        }
        for name, recipe in variants.items():
            h = tp.type_from_recipe(recipe)
            span = 1 << 25
            pk = median_event_us(lambda k: tp.pack_async(arena.data_ptr() + (k % 16) * span, count, h, out4[k % 8], 1 << 22, 0, stream), 20)
            block = tp.type_get_strided_block(h)
            rows.append({"construction": name, "incount": count, "object_bytes": (1 << 22) // count,
                         "canonical": [block[1], block[2]], "extent": tp.type_get_extent(h)[1],
                         "pack_event_us": round(pk, 1), "pack_gbs": round(2 * (1 << 22) / pk / 1e3, 1)})
    res["objects_2d_4MiB_vector_vs_subarray"] = rows
    del out4

    # ---- halo: 26 regions of a 512^3 float64 grid, ghost width 3
    c3 = W.configs.cfg3()
    send = [tp.type_from_recipe(r) for r in c3["send"]]
    ghost = [tp.type_from_recipe(r) for r in c3["ghost_for_send"]]
    sizes = [tp.type_size(h) for h in send]
    total = sum(sizes)
    bufs = [torch.zeros(total, dtype=torch.uint8, device=dev) for _ in range(8)]
    grid_at = lambda k: arena.data_ptr() + (k % 8) * GiB   # noqa: E731

    def halo(k, types, unpack, sync_each):
        pos = 0
        for h in types:
            if unpack:
                f = tp.unpack if sync_each else tp.unpack_async
                pos = f(bufs[k % 8], total, pos, grid_at(k), 1, h, stream)
            else:
                f = tp.pack if sync_each else tp.pack_async
                pos = f(grid_at(k), 1, h, bufs[k % 8], total, pos, stream)
        if not sync_each:
            stream.synchronize()
    halo_res = {"packed_bytes": total}
    for name, types, unpack in (("pack", send, False), ("unpack", ghost, True)):
        t_sync = median_wall_us(lambda k: halo(k, types, unpack, True), 12)
        t_async = median_wall_us(lambda k: halo(k, types, unpack, False), 12)
        halo_res[name] = {"26_sync_calls_us": round(t_sync, 1), "26_async_calls_one_sync_us": round(t_async, 1),
                          "gbs_async": round(2 * total / t_async / 1e3, 1)}
        # the same 26 requests as one batched launch
        def batched(k, types=types, unpack=unpack):
            b = batches[(name, k % 8)]
            if unpack:
                tp.unpack_batch_async(bufs[k % 8], total, 0, b, stream)
            else:
                tp.pack_batch_async(b, bufs[k % 8], total, 0, stream)
        batches = {(name, j): tp.Batch([grid_at(j)] * 26, [1] * 26, types) for j in range(8)}
        t_b_ev = median_event_us(batched, 16)
        t_b_wall = median_wall_us(lambda k: (batched(k), stream.synchronize()), 12)
        halo_res[name].update({"batched_one_launch_event_us": round(t_b_ev, 1),
                               "batched_one_launch_call_and_sync_us": round(t_b_wall, 1),
                               "gbs_batched_event": round(2 * total / t_b_ev / 1e3, 1),
                               "gbs_batched_call_and_sync": round(2 * total / t_b_wall / 1e3, 1)})
    # the 26 pack calls captured once in a HIP graph (what an iterative application would replay)
    side = torch.cuda.Stream()
    graph = torch.cuda.CUDAGraph()
    torch.cuda.synchronize()
    with torch.cuda.graph(graph, stream=side):
        pos = 0
        for h in send:
            pos = tp.pack_async(grid_at(0), 1, h, bufs[0], total, pos, torch.cuda.current_stream())
    t_graph = median_wall_us(lambda k: (graph.replay(), torch.cuda.synchronize()), 12)
    halo_res["pack"]["26_calls_hip_graph_replay_and_sync_us"] = round(t_graph, 1)
    del graph
    # per class: one x-face (24-byte runs), one y-face, one z-face (4048-byte runs)
    dirs = c3["directions"]
    for label, d in (("x_face", (0, 0, -1)), ("y_face", (0, -1, 0)), ("z_face", (-1, 0, 0))):
        i = dirs.index(d)
        h, g = send[i], ghost[i]
        n = sizes[i]
        pk = median_event_us(lambda k: tp.pack_async(grid_at(k), 1, h, bufs[k % 8], total, 0, stream), 16)
        plan = tp.last_plan().strip()
        up = median_event_us(lambda k: tp.unpack_async(bufs[k % 8], total, 0, grid_at(k), 1, g, stream), 16)
        halo_res[label] = {"bytes": n, "pack_us": round(pk, 1), "pack_gbs": round(2 * n / pk / 1e3, 1),
                           "unpack_us": round(up, 1), "unpack_gbs": round(2 * n / up / 1e3, 1), "plan": plan}
    res["halo_26_regions"] = halo_res
    del bufs

    # ---- tiny runs: 2^24 runs of bl bytes at 64-byte stride (1 GiB footprint)
    rows = []
    outs = [torch.zeros((8 << 24) + 64, dtype=torch.uint8, device=dev) for _ in range(4)]
    for bl in W.configs.CFG4_BLOCKLENGTHS:
        p = W.configs.cfg4_point(bl)
        h = tp.type_from_recipe(p["recipe"])
        n = p["packed_bytes"]
        for off in W.configs.CFG4_OFFSETS:
            src = lambda k: arena.data_ptr() + (k % 8) * 2 * GiB + off   # noqa: E731
            pk = median_event_us(lambda k: tp.pack_async(src(k), 1, h, outs[k % 4], n, 0, stream), 12)
            plan = tp.last_plan().strip()
            up = median_event_us(lambda k: tp.unpack_async(outs[k % 4], n, 0, src(k), 1, h, stream), 12)
            rows.append({"blocklength": bl, "offset": off, "pack_us": round(pk, 1), "unpack_us": round(up, 1),
                         "pack_gbs": round(2 * n / pk / 1e3, 1), "unpack_gbs": round(2 * n / up / 1e3, 1),
                         "pack_footprint_gbs": round((GiB + n) / pk / 1e3, 1), "plan": plan})
    # the same runs with the offset inside the datatype (a 2D byte subarray's start) and the packed
    # side at an odd position
    extra = []
    srcs = lambda k: arena.data_ptr() + (k % 8) * 2 * GiB   # noqa: E731
    for bl, off, pos in ((3, 5, 0), (3, 0, 1), (8, 3, 1)):
        h = tp.type_from_recipe(W.subarray([1 << 24, 64], [1 << 24, bl], [0, off], "C", W.BYTE))
        n = (1 << 24) * bl
        pk = median_event_us(lambda k: tp.pack_async(srcs(k), 1, h, outs[k % 4], n + pos, pos, stream), 8)
        plan = tp.last_plan().strip()
        up = median_event_us(lambda k: tp.unpack_async(outs[k % 4], n + pos, pos, srcs(k), 1, h, stream), 8)
        extra.append({"blocklength": bl, "subarray_start": off, "position": pos, "pack_us": round(pk, 1),
                      "unpack_us": round(up, 1), "plan": plan})
    res["tiny_runs_2p24_stride64"] = rows
    res["tiny_runs_offset_in_type_and_odd_position"] = extra
    del outs

    # ---- a matrix walked column by column (a transpose as a datatype): one-word elements adjacent in
    # the typed buffer along the outer dimension.  The transposing kernel (tiles through LDS) against
    # the row-by-row kernel and against PyTorch's transposing copy of the same matrix.
    xp = []
    for label, elem, esz in (("float32", W.FLOAT, 4), ("float64", W.DOUBLE, 8)):
        n = 4096
        h = tp.type_from_recipe(W.hvector(n, 1, esz, W.vector(n, 1, n, elem)))
        size = n * n * esz
        outs = [torch.empty(size, dtype=torch.uint8, device=dev) for _ in range(3)]
        mats = lambda k: arena.data_ptr() + (k % 8) * 2 * GiB   # noqa: E731
        row = {"matrix": f"{n} x {n} {label}", "bytes": size}
        for mode in ("tiles_through_lds", "row_by_row"):
            tp.set_override("xpose", 1 if mode == "tiles_through_lds" else 0)
            pk = median_event_us(lambda k: tp.pack_async(mats(k), 1, h, outs[k % 3], size, 0, stream), 9)
            plan = tp.last_plan().strip()
            up = median_event_us(lambda k: tp.unpack_async(outs[k % 3], size, 0, mats(k), 1, h, stream), 9)
            row[mode] = {"pack_us": round(pk, 1), "unpack_us": round(up, 1), "pack_gbs": round(2 * size / pk / 1e3, 1),
                         "unpack_gbs": round(2 * size / up / 1e3, 1), "plan": plan}
        tp.set_override("xpose", 1)
        a = torch.empty(n * n * esz, dtype=torch.uint8, device=dev).view(n, n, esz)
        b = torch.empty(n, n, esz, dtype=torch.uint8, device=dev)
        row["torch_transposing_copy_us"] = round(median_event_us(lambda k: b.copy_(a.transpose(0, 1)), 9), 1)
        xp.append(row)
        del outs, a, b
    res["matrix_walked_by_columns"] = xp

    # ---- nested 4-level type, 1000 objects of 2 MiB packed
    c5 = W.configs.cfg5()
    h = tp.type_from_recipe(c5["recipe"])
    ex, size, nobj = tp.type_get_extent(h)[1], tp.type_size(h), c5["objects"]
    out = torch.zeros(nobj * size, dtype=torch.uint8, device=dev)
    base = lambda k: arena.data_ptr() + (k % 4) * 10 * GiB   # noqa: E731
    one = median_event_us(lambda k: tp.pack_async(base(k), nobj, h, out, nobj * size, 0, stream), 8)
    plan = tp.last_plan().strip()

    def many_async(k):
        pos = 0
        for i in range(nobj):
            pos = tp.pack_async(base(k) + i * ex, 1, h, out, nobj * size, pos, stream)
        stream.synchronize()

    def many_sync(k):
        pos = 0
        for i in range(100):
            pos = tp.pack(base(k) + i * ex, 1, h, out, nobj * size, pos, stream)
    t_async = median_wall_us(many_async, 5)
    t_sync = median_wall_us(many_sync, 5)
    nested = {"objects": nobj, "packed_bytes_per_object": size, "plan": plan,
              "one_call_incount_1000_us": round(one, 1), "one_call_us_per_object": round(one / nobj, 3),
              "one_call_gbs": round(2 * nobj * size / one / 1e3, 1),
              "1000_async_calls_one_sync_us_per_object": round(t_async / nobj, 2),
              "1000_async_calls_gbs": round(2 * nobj * size / t_async / 1e3, 1),
              "sync_call_us_per_object": round(t_sync / 100, 2)}
    bb = [tp.Batch([base(j) + i * ex for i in range(nobj)], [1] * nobj, [h] * nobj) for j in range(4)]
    t_batch = median_wall_us(lambda k: (tp.pack_batch_async(bb[k % 4], out, nobj * size, 0, stream),
                                        stream.synchronize()), 5)
    nested["1000_objects_batched_us_per_object"] = round(t_batch / nobj, 3)
    nested["1000_objects_batched_gbs"] = round(2 * nobj * size / t_batch / 1e3, 1)
    npin = 128
    pinned = torch.zeros(npin * size, dtype=torch.uint8).pin_memory()
    t_pin = median_wall_us(lambda k: tp.pack(base(k), npin, h, pinned, npin * size, 0, stream), 5)
    nested["zero_copy_pinned_host"] = {"objects": npin, "us_per_object": round(t_pin / npin, 2),
                                       "packed_gbs_over_pcie": round(npin * size / t_pin / 1e3, 1)}
    res["nested_4level"] = nested
    return res


if __name__ == "__main__":
    main()

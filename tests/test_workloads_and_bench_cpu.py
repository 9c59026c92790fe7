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

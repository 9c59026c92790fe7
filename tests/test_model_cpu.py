"""CPU tests of the measured performance model (paper Sec. 4 Eq. 1-3, Sec. 6.3): the oracle's
interpolation against scipy's and against closed forms, then the library against the oracle."""
import math
import os
import random

import numpy as np
import pytest
from scipy.interpolate import RegularGridInterpolator

import workloads as W
from workloads import BYTE, contiguous, vector
from oracle import model as om
from paper_2012_14363_amd import binding as tp


def synthetic_table_text(seed=1, ns=5, nb=7):
    rng = np.random.default_rng(seed)
    sizes = 64.0 * 16.0 ** np.arange(ns)
    blocks = 4.0 ** np.arange(nb)
    lines = ["tp_model 1", "sizes %d " % ns + " ".join(repr(float(v)) for v in sizes),
             "blocks %d " % nb + " ".join(repr(float(v)) for v in blocks)]
    for name in om.PRIMITIVES[:4]:
        g = 5e-6 + sizes[:, None] / (1e9 * (1 + rng.random((ns, nb)) * blocks[None, :]))
        lines.append(name + " " + " ".join(repr(float(v)) for v in g.reshape(-1)))
    for name in om.PRIMITIVES[4:]:
        v = 8e-6 + sizes / (50e9 * (0.5 + rng.random(ns)))
        lines.append(name + " " + " ".join(repr(float(x)) for x in v))
    return "\n".join(lines) + "\n"


def test_oracle_interpolation_matches_scipy_and_grid_points():
    table = om.parse(synthetic_table_text())
    sizes, blocks = table["sizes"], table["blocks"]
    # on the grid the table itself comes back
    for i, s in enumerate(sizes):
        for j, b in enumerate(blocks):
            q = om.query(table, s, b)
            for name in om.PRIMITIVES[:4]:
                assert q[name] == pytest.approx(table[name][i, j], rel=1e-14)
            assert q["d2h"] == pytest.approx(table["d2h"][i], rel=1e-14)
    # inside: scipy's multilinear interpolation on log2 coordinates is the same thing
    rng = random.Random(5)
    for name in om.PRIMITIVES[:4]:
        rgi = RegularGridInterpolator((np.log2(sizes), np.log2(blocks)), table[name], method="linear")
        for _ in range(200):
            s = 2 ** rng.uniform(math.log2(sizes[0]), math.log2(sizes[-1]))
            b = 2 ** rng.uniform(math.log2(blocks[0]), math.log2(blocks[-1]))
            assert om.query(table, s, b)[name] == pytest.approx(float(rgi([[math.log2(s), math.log2(b)]])[0]), rel=1e-12)
    # outside: clamped block, clamped small size, proportional large size
    q_in = om.query(table, sizes[-1], blocks[-1])
    assert om.query(table, sizes[-1], blocks[-1] * 100) == q_in
    assert om.query(table, sizes[0] / 8, blocks[0] / 2) == om.query(table, sizes[0], blocks[0])
    big = om.query(table, sizes[-1] * 8, blocks[2])
    ref = om.query(table, sizes[-1], blocks[2])
    assert all(big[k] == pytest.approx(8 * ref[k], rel=1e-14) for k in ref)


def test_oracle_exact_on_a_log_linear_table():
    # T = a + b*log2(size) + c*log2(block) is reproduced exactly by bilinear interpolation in log space
    sizes, blocks = [64.0, 1024.0, 65536.0], [1.0, 16.0, 256.0, 4096.0]
    f = lambda s, b: 3.0 + 0.25 * math.log2(s) + 0.5 * math.log2(b)  # noqa: E731
    lines = ["tp_model 1", "sizes 3 64 1024 65536", "blocks 4 1 16 256 4096"]
    for name in om.PRIMITIVES[:4]:
        lines.append(name + " " + " ".join(repr(f(s, b)) for s in sizes for b in blocks))
    for name in om.PRIMITIVES[4:]:
        lines.append(name + " " + " ".join(repr(f(s, 1.0)) for s in sizes))
    table = om.parse("\n".join(lines))
    for s, b in ((100.0, 3.0), (5000.0, 77.0), (64.0, 4096.0), (40000.0, 1.0)):
        assert om.query(table, s, b)["host_pack"] == pytest.approx(f(s, b), rel=1e-13)


def test_oracle_selection_is_eq_1_to_3():
    t = {"gpu_pack": 1.0, "gpu_unpack": 2.0, "host_pack": 4.0, "host_unpack": 8.0, "d2h": 16.0, "h2d": 32.0}
    m, totals = om.select(t, t_cpu_cpu=100.0, t_gpu_gpu=1000.0)
    assert totals == [1003.0, 112.0, 151.0] and m == om.ONESHOT
    assert om.select(t)[0] == om.DEVICE
    assert om.select(t, t_cpu_cpu=0.0, t_gpu_gpu=60.0)[0] == om.ONESHOT
    t2 = dict(t, host_pack=400.0)
    assert om.select(t2, t_cpu_cpu=0.0, t_gpu_gpu=60.0)[0] == om.STAGED


def test_library_model_matches_oracle(tmp_path):
    text = synthetic_table_text(seed=9)
    path = tmp_path / "model.txt"
    path.write_text(text)
    tp.model_load(str(path))
    table = om.parse(text)
    # save -> load round trip keeps every digit
    out = tmp_path / "model2.txt"
    tp.model_save(str(out))
    t2 = om.parse(out.read_text())
    assert all(np.array_equal(table[k], t2[k]) for k in table)
    rng = random.Random(11)
    for _ in range(300):
        bl = rng.choice((1, 2, 3, 8, 24, 100, 512, 4048, 20000))
        count = rng.choice((1, 2, 7, 64, 1000, 100000))
        incount = rng.choice((1, 1, 3))
        h = tp.type_from_recipe(vector(count, bl, bl + rng.choice((1, 8, 512)), BYTE))
        nbytes = tp.type_size(h) * incount
        block = tp.type_get_strided_block(h)[1][0]
        want = om.query(table, nbytes, block if len(tp.type_get_strided_block(h)[1]) > 1 else nbytes)
        got = tp.model_query(h, incount)
        for k in want:
            assert got[k] == pytest.approx(want[k], rel=1e-12), (k, count, bl)
        cc, gg = rng.choice((0.0, 5e-6, 1e-3)), rng.choice((0.0, 20e-6, 1e-3))
        method, totals = tp.model_select(h, incount, cc, gg)
        wm, wt = om.select(want, cc, gg)
        assert method == wm and totals == pytest.approx(wt, rel=1e-12)
        tp.type_free(h)
    # a dense type is keyed by its whole size
    h = tp.type_from_recipe(contiguous(5000, BYTE))
    assert tp.model_query(h, 3)["d2h"] == pytest.approx(om.query(table, 15000, 15000)["d2h"], rel=1e-12)


def test_model_errors(tmp_path):
    bad = tmp_path / "bad.txt"
    bad.write_text("tp_model 1\nsizes 2 64 32\nblocks 1 1\n")
    with pytest.raises(tp.TpError) as e:
        tp.model_load(str(bad))
    assert e.value.code == tp.TP_ERR_ARG
    with pytest.raises(tp.TpError):
        tp.model_load(str(tmp_path / "missing.txt"))
    h = tp.type_vector(3, 2, 4, tp.TP_BYTE)
    with pytest.raises(tp.TpError) as e:   # not committed
        tp.model_query(h, 1)
    assert e.value.code == tp.TP_ERR_TYPE

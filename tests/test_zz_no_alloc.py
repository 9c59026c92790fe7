"""The entry point that allocates nothing (tp_pack_host_static: staged host delivery through a fixed
device array inside the library) against the existing entry point it is a variant of (tp_pack_host,
staged through a caller's buffer) and against the oracle, byte for byte.  Two calls in a row, the
second smaller, so that bytes the first call left in the shared array would show.  Collected last:
a failure here must not hide the other GPU tests."""
import numpy as np
import pytest

import workloads as W
from workloads import BYTE, DOUBLE, hvector, subarray, vector
from oracle import typemap_c as cc
from paper_2012_14363_amd import binding as tp

torch = pytest.importorskip("torch")


@pytest.mark.gpu
def test_static_staging_equals_staged_host_delivery():
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    tp.lib()
    dev = torch.device("cuda:0")
    # first a message that fills most of the array, of short ragged rows, then a much smaller one of
    # another type at another position: 3 objects of 7 x 19 doubles out of a 3D array
    calls = [
        (vector(29000, 131, 512, BYTE), 1, 5),
        (hvector(3, 1, 40000, subarray((9, 7, 32), (1, 7, 19), (4, 0, 6), "C", DOUBLE)), 3, 0),
    ]
    sizes = []
    for k, (recipe, count, position) in enumerate(calls):
        h = tp.type_from_recipe(recipe)
        size = tp.type_size(h) * count
        extent = tp.type_get_extent(h)[1]
        sizes.append(size)
        assert size <= tp.TP_STATIC_STAGING_BYTES
        print("static staging call", k, "bytes", size, flush=True)
        typed_h = W.random_bytes(900 + k, extent * count + 64)
        typed = torch.from_numpy(typed_h).to(dev)
        total = position + size + 32
        got = torch.full((total,), 0xEE, dtype=torch.uint8).pin_memory()
        ref = torch.full((total,), 0xEE, dtype=torch.uint8).pin_memory()
        staging = torch.zeros(size, dtype=torch.uint8, device=dev)
        assert tp.pack_host_static(typed, count, h, got, total, position) == position + size
        plan = tp.last_plan()
        new_pos, used = tp.pack_host(typed, count, h, ref, total, position, staging=staging, staging_size=size,
                                     method=tp.TP_METHOD_STAGED)
        assert (new_pos, used) == (position + size, tp.TP_METHOD_STAGED)
        assert np.array_equal(got.numpy(), ref.numpy()), plan
        expect = np.full(total, 0xEE, np.uint8)
        cc.pack(typed_h, 0, count, recipe, expect, position)
        assert np.array_equal(got.numpy(), expect), plan
        tp.type_free(h)
    assert sizes[1] < sizes[0] // 100
    # a message larger than the array is refused before anything runs
    big = tp.type_from_recipe(vector(tp.TP_STATIC_STAGING_BYTES // 64 + 1, 64, 128, BYTE))
    src = torch.zeros(tp.type_get_extent(big)[1], dtype=torch.uint8, device=dev)
    out = torch.full((tp.type_size(big),), 0x11, dtype=torch.uint8).pin_memory()
    with pytest.raises(tp.TpError) as e:
        tp.pack_host_static(src, 1, big, out, out.numel(), 0)
    assert e.value.code == tp.TP_ERR_RANGE
    assert (out.numpy() == 0x11).all()
    tp.type_free(big)


def test_static_staging_checks_sizes_before_touching_a_device():
    import ctypes

    L = tp.lib()
    fake = ctypes.c_void_p(4096)
    big = tp.type_from_recipe(vector(tp.TP_STATIC_STAGING_BYTES // 64 + 1, 64, 128, BYTE))
    pos = ctypes.c_int64(3)
    assert L.tp_pack_host_static(fake, 1, big, fake, 1 << 40, ctypes.byref(pos), None) == tp.TP_ERR_RANGE
    assert L.tp_pack_host_static(fake, -1, big, fake, 1 << 40, ctypes.byref(pos), None) == tp.TP_ERR_COUNT
    assert L.tp_pack_host_static(fake, 1, big, fake, 1 << 40, None, None) == tp.TP_ERR_ARG
    assert L.tp_pack_host_static(fake, 1, 999999, fake, 1 << 40, ctypes.byref(pos), None) == tp.TP_ERR_TYPE
    small = tp.type_from_recipe(vector(4, 8, 16, BYTE))
    assert L.tp_pack_host_static(fake, 1, small, fake, 34, ctypes.byref(pos), None) == tp.TP_ERR_TRUNCATE
    assert L.tp_pack_host_static(fake, 1, small, None, 64, ctypes.byref(pos), None) == tp.TP_ERR_BUFFER
    assert pos.value == 3
    tp.type_free(big)
    tp.type_free(small)

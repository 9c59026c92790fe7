"""The resource cache's bookkeeping (paper Sec. 5), run over the host heap: size classes, reuse,
per-device and per-kind separation, trimming, the retry after a failed creation, lookup of leased
ranges, misuse, and concurrent holders.  No GPU."""
import pytest

from tests import host_emul

DEVICE, PINNED, STREAM, EVENT = 0, 1, 2, 3
OK, ERR_ARG, ERR_OTHER, ERR_RANGE = 0, 3, 6, 7


@pytest.fixture()
def cache():
    host_emul.cache_set_device(0)
    host_emul.cache_fail_next(0)
    c = host_emul.Cache()
    yield c
    c.close()


def test_capacity_classes():
    cap = host_emul.cache_capacity
    assert cap(0) == cap(1) == cap(4096) == 4096
    assert cap(4097) == 5120 and cap(5120) == 5120 and cap(5121) == 6144
    assert cap(8192) == 8192 and cap(8193) == 10240
    assert cap(-1) == 0 and cap(1 << 62) == 0
    # never smaller than asked, never more than a quarter larger (beyond the 4 KiB floor), and
    # idempotent, so a released buffer is found again by any request that rounds to it
    for n in list(range(4096, 70000, 37)) + [(1 << 30) + 1, (3 << 33) - 5, (1 << 40) + 12345]:
        c = cap(n)
        assert n <= c <= n + n // 4 + 1, n
        assert cap(c) == c
        assert c % 1024 == 0


def test_reuse_within_a_class_only(cache):
    rc, a = cache.acquire(DEVICE, 5000)
    assert rc == OK and a
    assert cache.counts(DEVICE) == dict(hits=0, misses=1, idle=0, leased=1, idle_bytes=0, leased_bytes=5120)
    assert cache.release(DEVICE, a) == OK
    assert cache.counts(DEVICE) == dict(hits=0, misses=1, idle=1, leased=0, idle_bytes=5120, leased_bytes=0)
    rc, b = cache.acquire(DEVICE, 4200)  # same class: the same buffer comes back
    assert rc == OK and b == a
    assert cache.counts(DEVICE)["hits"] == 1
    rc, c = cache.acquire(DEVICE, 5000)  # same class, but the only buffer is out
    assert rc == OK and c != a
    rc, d = cache.acquire(DEVICE, 100000)  # another class
    assert rc == OK and d not in (a, c)
    assert cache.counts(DEVICE)["misses"] == 3
    for h in (b, c, d):
        assert cache.release(DEVICE, h) == OK
    # a smaller request does not take the larger idle buffer (classes are exact)
    rc, e = cache.acquire(DEVICE, 10)
    assert rc == OK and e not in (a, c, d)
    assert cache.release(DEVICE, e) == OK


def test_kinds_and_devices_do_not_mix(cache):
    rc, dev = cache.acquire(DEVICE, 8000)
    assert cache.release(DEVICE, dev) == OK
    rc, pin = cache.acquire(PINNED, 8000)
    assert rc == OK and pin != dev and cache.counts(PINNED)["misses"] == 1
    assert cache.release(PINNED, pin) == OK
    host_emul.cache_set_device(1)
    rc, other = cache.acquire(DEVICE, 8000)
    assert rc == OK and other != dev and cache.counts(DEVICE)["misses"] == 2
    assert cache.release(DEVICE, other) == OK
    host_emul.cache_set_device(0)
    rc, again = cache.acquire(DEVICE, 8000)
    assert rc == OK and again == dev
    assert cache.release(DEVICE, again) == OK


def test_streams_and_events(cache):
    rc, s1 = cache.acquire(STREAM, 0)
    rc2, s2 = cache.acquire(STREAM, 123456)  # bytes are ignored
    assert rc == OK and rc2 == OK and s1 != s2
    assert cache.release(STREAM, s1) == OK
    rc, s3 = cache.acquire(STREAM, 0)
    assert s3 == s1
    rc, e1 = cache.acquire(EVENT, 0)
    assert rc == OK and e1 not in (s1, s2)
    assert cache.release(STREAM, e1) == ERR_ARG  # wrong kind
    assert cache.release(EVENT, e1) == OK
    n = cache.counts(STREAM)
    assert (n["hits"], n["misses"], n["leased"], n["idle_bytes"], n["leased_bytes"]) == (1, 2, 2, 0, 0)
    assert cache.release(STREAM, s2) == OK and cache.release(STREAM, s3) == OK


def test_misuse_is_refused(cache):
    assert cache.acquire(4, 10)[0] == ERR_ARG and cache.acquire(-1, 10)[0] == ERR_ARG
    assert cache.acquire(DEVICE, -5)[0] == ERR_ARG
    assert cache.acquire(PINNED, 1 << 62)[0] == ERR_RANGE
    rc, a = cache.acquire(DEVICE, 100)
    assert cache.release(DEVICE, a + 8) == ERR_ARG  # not the handle
    assert cache.release(PINNED, a) == ERR_ARG
    assert cache.release(DEVICE, None) == ERR_ARG
    assert cache.release(DEVICE, a) == OK
    assert cache.release(DEVICE, a) == ERR_ARG  # twice
    assert cache.counts(DEVICE)["idle"] == 1  # and the failed calls changed nothing


def test_trim_and_teardown_destroy_exactly_the_idle():
    host_emul.cache_set_device(0)
    host_emul.cache_fail_next(0)
    made0, gone0, live0 = host_emul.cache_backend(DEVICE)
    c = host_emul.Cache()
    handles = [c.acquire(DEVICE, n)[1] for n in (100, 5000, 70000, 70000)]
    assert host_emul.cache_backend(DEVICE)[0] - made0 == 4
    assert host_emul.cache_backend(DEVICE)[2] - live0 == 4096 + 5120 + 2 * 81920
    for h in handles[:3]:
        assert c.release(DEVICE, h) == OK
    assert c.trim() == 4096 + 5120 + 81920
    assert host_emul.cache_backend(DEVICE)[1] - gone0 == 3
    n = c.counts(DEVICE)
    assert (n["idle"], n["idle_bytes"], n["leased"], n["leased_bytes"]) == (0, 0, 1, 81920)
    assert c.trim() == 0
    # the leased buffer is still valid and comes back into the cache afterwards
    assert c.find(handles[3]) is not None
    assert c.release(DEVICE, handles[3]) == OK
    c.close()  # teardown destroys what is idle
    made, gone, live = host_emul.cache_backend(DEVICE)
    assert made - made0 == 4 and gone - gone0 == 4 and live == live0


def test_failed_creation_trims_and_retries(cache):
    rc, a = cache.acquire(DEVICE, 1 << 20)
    assert cache.release(DEVICE, a) == OK
    gone0 = host_emul.cache_backend(DEVICE)[1]
    host_emul.cache_fail_next(1)  # first try fails: idle memory is given back, second try succeeds
    rc, b = cache.acquire(DEVICE, 1 << 21)
    assert rc == OK and b
    assert host_emul.cache_backend(DEVICE)[1] - gone0 == 1
    assert cache.counts(DEVICE)["idle"] == 0
    host_emul.cache_fail_next(2)  # both tries fail
    rc, c = cache.acquire(DEVICE, 1 << 22)
    assert rc == ERR_OTHER and not c
    n = cache.counts(DEVICE)
    assert (n["leased"], n["misses"]) == (1, 2)
    assert cache.release(DEVICE, b) == OK


def test_find_leased_ranges(cache):
    rc, a = cache.acquire(DEVICE, 10000)  # capacity 10240
    rc, p = cache.acquire(PINNED, 6000)  # capacity 6144
    assert cache.find(a) == (DEVICE, 0, 10240)
    assert cache.find(a + 10239) == (DEVICE, 0, 1)
    for outside in (a + 10240, a - 1):  # one past either end: not this buffer (the heap may put p there)
        hit = cache.find(outside)
        assert hit is None or hit[0] == PINNED
    # the pinned backend places the GPU view 2^40 above the host address
    assert cache.find(p + 100) == (PINNED, 1 << 40, 6044)
    assert cache.release(DEVICE, a) == OK
    assert cache.find(a) is None  # idle buffers are nobody's
    assert cache.release(PINNED, p) == OK
    assert cache.find(p) is None


def test_concurrent_holders(cache):
    assert cache.hammer(8, 20000) == 0
    for kind in range(4):
        n = cache.counts(kind)
        assert n["leased"] == 0 and n["leased_bytes"] == 0
        assert n["hits"] + n["misses"] > 0 and n["hits"] > 10 * n["misses"]
        assert n["idle"] == n["misses"]


# ------------------------------------------------------------------ per-call buffer map
def test_buffer_map_asks_once_per_allocation():
    BUF = 5  # TP_ERR_BUFFER
    allocs = [(0x1000, 0x2000, False), (0x2000, 0x2800, False), (0x9000, 0xA000, True)]
    ops = [(0x1800, False), (0x1000, False), (0x1FFF, False),   # one allocation: one query
           (0x2000, False),                                     # its neighbour: a second query
           (0x0FFF, False), (0x2800, False),                    # just outside either: refused, and asked each time
           (0x2800, False),
           (0x9800, True), (0x9000, True), (0x9FFF, False),     # mapped host memory: only where allowed
           (0x17FF, True)]
    q, got = host_emul.buffer_map_run(allocs, ops)
    assert got == [(0, 0)] * 4 + [(BUF, 0)] * 3 + [(0, 1 << 40), (0, 1 << 40), (BUF, 0), (0, 0)]
    assert q == 2 + 3 + 1
    # a runtime that does not tell the bounds: every new address is asked, repeated ones are not
    q, got = host_emul.buffer_map_run(allocs, ops[:4] + [(0x1800, False)], bounds_known=False)
    assert [g[0] for g in got] == [0] * 5 and q == 4
    # checks switched off: nothing is asked, everything passes as device memory
    q, got = host_emul.buffer_map_run(allocs, ops, checked=False)
    assert q == 0 and got == [(0, 0)] * len(ops)


# ------------------------------------------------------------------ the library's own entry points, without a GPU
def test_library_resource_calls_reject_bad_arguments():
    import ctypes

    from paper_2012_14363_amd import binding as tp
    L = tp.lib()
    h = ctypes.c_void_p()
    assert L.tp_resource_acquire(7, 100, ctypes.byref(h)) == tp.TP_ERR_ARG
    assert L.tp_resource_acquire(tp.TP_RES_DEVICE, -1, ctypes.byref(h)) == tp.TP_ERR_ARG
    assert L.tp_resource_acquire(tp.TP_RES_DEVICE, 100, None) == tp.TP_ERR_ARG
    assert L.tp_resource_release(tp.TP_RES_DEVICE, None) == tp.TP_ERR_ARG
    assert L.tp_resource_release(tp.TP_RES_PINNED, 0x1000) == tp.TP_ERR_ARG     # never leased
    assert L.tp_resource_stats(9, ctypes.byref(tp.ResourceCounts())) == tp.TP_ERR_ARG
    assert L.tp_resource_stats(tp.TP_RES_EVENT, None) == tp.TP_ERR_ARG
    for kind in range(4):
        c = tp.resource_stats(kind)
        assert c["leased"] >= 0 and c["idle"] >= 0 and c["leased_bytes"] >= 0
    assert tp.resource_trim() >= 0
    assert L.tp_resource_trim(None) == tp.TP_SUCCESS

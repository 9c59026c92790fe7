"""Thin ctypes binding over libtp_pack.so: same names as include/tp_pack.h, argument
marshalling only.  Every step of the path runs inside the library; without the
built library (or, for pack/unpack, without a GPU) calls fail loudly.
"""
from __future__ import annotations

import ctypes
import os

_PKG_DIR = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_PKG_DIR, "libtp_pack.so")

TP_TYPE_NULL = -1
TP_BYTE, TP_CHAR, TP_INT8, TP_UINT8, TP_INT16, TP_UINT16 = 0, 1, 2, 3, 4, 5
TP_INT32, TP_UINT32, TP_INT64, TP_UINT64, TP_FLOAT, TP_DOUBLE = 6, 7, 8, 9, 10, 11
TP_ORDER_C, TP_ORDER_FORTRAN = 0, 1
TP_MAX_DIMS = 16

TP_SUCCESS, TP_ERR_TYPE, TP_ERR_COUNT, TP_ERR_ARG = 0, 1, 2, 3
TP_ERR_TRUNCATE, TP_ERR_BUFFER, TP_ERR_OTHER, TP_ERR_RANGE = 4, 5, 6, 7

PREDEFINED = {
    "BYTE": TP_BYTE, "CHAR": TP_CHAR, "INT8": TP_INT8, "UINT8": TP_UINT8, "INT16": TP_INT16,
    "UINT16": TP_UINT16, "INT32": TP_INT32, "UINT32": TP_UINT32, "INT64": TP_INT64,
    "UINT64": TP_UINT64, "FLOAT": TP_FLOAT, "DOUBLE": TP_DOUBLE,
}

# every symbol include/tp_pack.h declares
EXPORTS = (
    "tp_type_contiguous", "tp_type_vector", "tp_type_create_hvector", "tp_type_create_subarray",
    "tp_type_commit", "tp_type_free", "tp_type_size", "tp_type_get_extent", "tp_pack_size",
    "tp_pack", "tp_unpack", "tp_pack_async", "tp_unpack_async",
    "tp_pack_batch", "tp_unpack_batch", "tp_pack_batch_async", "tp_unpack_batch_async",
    "tp_model_measure", "tp_model_save", "tp_model_load", "tp_model_query", "tp_model_select",
    "tp_pack_host", "tp_unpack_host", "tp_pack_host_static",
    "tp_resource_acquire", "tp_resource_release", "tp_resource_trim", "tp_resource_stats",
    "tp_type_get_strided_block", "tp_set_override", "tp_last_plan", "tp_error_string",
)


TP_METHOD_AUTO, TP_METHOD_DEVICE, TP_METHOD_ONESHOT, TP_METHOD_STAGED = -1, 0, 1, 2
TP_RES_DEVICE, TP_RES_PINNED, TP_RES_STREAM, TP_RES_EVENT = 0, 1, 2, 3


class ResourceCounts(ctypes.Structure):
    """tp_resource_counts"""
    _fields_ = [(n, ctypes.c_int64) for n in ("hits", "misses", "idle", "leased", "idle_bytes", "leased_bytes")]

    def as_dict(self):
        return {n: getattr(self, n) for n, _ in self._fields_}


class ModelTimes(ctypes.Structure):
    """tp_model_times: seconds per operation."""
    _fields_ = [(n, ctypes.c_double) for n in ("gpu_pack", "gpu_unpack", "host_pack", "host_unpack", "d2h", "h2d")]

    def as_dict(self):
        return {n: getattr(self, n) for n, _ in self._fields_}


class TpError(RuntimeError):
    def __init__(self, code: int, where: str):
        self.code = code
        super().__init__(f"{where}: error {code} ({error_string(code)})")


_lib = None


def lib() -> ctypes.CDLL:
    """The loaded library.  Raises if it has not been built (no fallback exists)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(
                f"{LIB_PATH} is missing: build it with `python -m paper_2012_14363_amd.build` "
                "(there is no CPU or PyTorch fallback for the pack/unpack path)")
        # One HIP runtime per process: PyTorch ships its own libamdhip64.  Import it first so the
        # loader resolves this library's dependency to that already-loaded runtime; loaded the
        # other way round the process would hold two runtimes that cannot see each other's memory.
        try:
            import torch  # noqa: F401
        except ImportError:
            pass
        L = ctypes.CDLL(LIB_PATH)
        i32, i64, vp = ctypes.c_int32, ctypes.c_int64, ctypes.c_void_p
        pi32, pi64, pint = ctypes.POINTER(i32), ctypes.POINTER(i64), ctypes.POINTER(ctypes.c_int)
        pvp = ctypes.POINTER(vp)
        sig = {
            "tp_type_contiguous": [ctypes.c_int, i32, pi32],
            "tp_type_vector": [ctypes.c_int, ctypes.c_int, ctypes.c_int, i32, pi32],
            "tp_type_create_hvector": [ctypes.c_int, ctypes.c_int, i64, i32, pi32],
            "tp_type_create_subarray": [ctypes.c_int, pint, pint, pint, ctypes.c_int, i32, pi32],
            "tp_type_commit": [pi32],
            "tp_type_free": [pi32],
            "tp_type_size": [i32, pi64],
            "tp_type_get_extent": [i32, pi64, pi64],
            "tp_pack_size": [ctypes.c_int, i32, pi64],
            "tp_pack": [vp, ctypes.c_int, i32, vp, i64, pi64, vp],
            "tp_unpack": [vp, i64, pi64, vp, ctypes.c_int, i32, vp],
            "tp_pack_async": [vp, ctypes.c_int, i32, vp, i64, pi64, vp],
            "tp_unpack_async": [vp, i64, pi64, vp, ctypes.c_int, i32, vp],
            "tp_pack_batch": [ctypes.c_int, pvp, pint, pi32, vp, i64, pi64, vp],
            "tp_unpack_batch": [ctypes.c_int, vp, i64, pi64, pvp, pint, pi32, vp],
            "tp_pack_batch_async": [ctypes.c_int, pvp, pint, pi32, vp, i64, pi64, vp],
            "tp_unpack_batch_async": [ctypes.c_int, vp, i64, pi64, pvp, pint, pi32, vp],
            "tp_model_measure": [vp],
            "tp_model_save": [ctypes.c_char_p],
            "tp_model_load": [ctypes.c_char_p],
            "tp_model_query": [i32, ctypes.c_int, ctypes.POINTER(ModelTimes)],
            "tp_model_select": [i32, ctypes.c_int, ctypes.c_double, ctypes.c_double, pint,
                                ctypes.POINTER(ctypes.c_double)],
            "tp_pack_host": [vp, ctypes.c_int, i32, vp, i64, pi64, vp, i64, ctypes.c_int, vp, pint],
            "tp_pack_host_static": [vp, ctypes.c_int, i32, vp, i64, pi64, vp],
            "tp_unpack_host": [vp, i64, pi64, vp, ctypes.c_int, i32, vp, i64, ctypes.c_int, vp, pint],
            "tp_resource_acquire": [ctypes.c_int, i64, pvp],
            "tp_resource_release": [ctypes.c_int, vp],
            "tp_resource_trim": [pi64],
            "tp_resource_stats": [ctypes.c_int, ctypes.POINTER(ResourceCounts)],
            "tp_type_get_strided_block": [i32, pint, pi64, pi64, pi64],
            "tp_set_override": [ctypes.c_char_p, ctypes.c_char_p],
        }
        for name, argtypes in sig.items():
            fn = getattr(L, name)
            fn.argtypes = argtypes
            fn.restype = ctypes.c_int
        L.tp_last_plan.argtypes = []
        L.tp_last_plan.restype = ctypes.c_char_p
        L.tp_error_string.argtypes = [ctypes.c_int]
        L.tp_error_string.restype = ctypes.c_char_p
        _lib = L
    return _lib


def error_string(code: int) -> str:
    return lib().tp_error_string(int(code)).decode()


def _check(rc: int, where: str):
    if rc != TP_SUCCESS:
        raise TpError(rc, where)


# ------------------------------------------------------------------ constructors
def type_contiguous(count: int, old: int) -> int:
    new = ctypes.c_int32(TP_TYPE_NULL)
    _check(lib().tp_type_contiguous(count, old, ctypes.byref(new)), "tp_type_contiguous")
    return new.value


def type_vector(count: int, blocklength: int, stride: int, old: int) -> int:
    new = ctypes.c_int32(TP_TYPE_NULL)
    _check(lib().tp_type_vector(count, blocklength, stride, old, ctypes.byref(new)), "tp_type_vector")
    return new.value


def type_create_hvector(count: int, blocklength: int, stride_bytes: int, old: int) -> int:
    new = ctypes.c_int32(TP_TYPE_NULL)
    _check(lib().tp_type_create_hvector(count, blocklength, stride_bytes, old, ctypes.byref(new)),
           "tp_type_create_hvector")
    return new.value


def type_create_subarray(sizes, subsizes, starts, order: int, old: int) -> int:
    n = len(sizes)
    arr = ctypes.c_int * n
    new = ctypes.c_int32(TP_TYPE_NULL)
    _check(lib().tp_type_create_subarray(n, arr(*sizes), arr(*subsizes), arr(*starts), order, old,
                                         ctypes.byref(new)), "tp_type_create_subarray")
    return new.value


def type_commit(t: int) -> None:
    h = ctypes.c_int32(t)
    _check(lib().tp_type_commit(ctypes.byref(h)), "tp_type_commit")


def type_free(t: int) -> None:
    h = ctypes.c_int32(t)
    _check(lib().tp_type_free(ctypes.byref(h)), "tp_type_free")


def type_size(t: int) -> int:
    v = ctypes.c_int64()
    _check(lib().tp_type_size(t, ctypes.byref(v)), "tp_type_size")
    return v.value


def type_get_extent(t: int):
    lb, ex = ctypes.c_int64(), ctypes.c_int64()
    _check(lib().tp_type_get_extent(t, ctypes.byref(lb), ctypes.byref(ex)), "tp_type_get_extent")
    return lb.value, ex.value


def pack_size(incount: int, t: int) -> int:
    v = ctypes.c_int64()
    _check(lib().tp_pack_size(incount, t, ctypes.byref(v)), "tp_pack_size")
    return v.value


def type_get_strided_block(t: int):
    """(start, counts, strides) of a committed type's canonical StridedBlock."""
    nd, start = ctypes.c_int(), ctypes.c_int64()
    counts = (ctypes.c_int64 * TP_MAX_DIMS)()
    strides = (ctypes.c_int64 * TP_MAX_DIMS)()
    _check(lib().tp_type_get_strided_block(t, ctypes.byref(nd), ctypes.byref(start), counts, strides),
           "tp_type_get_strided_block")
    return start.value, list(counts[:nd.value]), list(strides[:nd.value])


def set_override(key: str, value) -> None:
    _check(lib().tp_set_override(key.encode(), str(value).encode()), "tp_set_override")


def last_plan() -> str:
    return lib().tp_last_plan().decode()


# ------------------------------------------------------------------ pack / unpack
def _ptr(buf) -> int:
    """Address of a torch tensor (device or pinned host), or a raw integer address."""
    if isinstance(buf, int):
        return buf
    return buf.data_ptr()


def _stream(stream) -> int:
    if stream is None:
        import torch
        return torch.cuda.current_stream().cuda_stream
    if isinstance(stream, int):
        return stream
    return stream.cuda_stream


def _pack_call(fn_name, inbuf, incount, t, outbuf, outsize, position, stream):
    pos = ctypes.c_int64(position)
    rc = getattr(lib(), fn_name)(_ptr(inbuf), incount, t, _ptr(outbuf), outsize, ctypes.byref(pos), _stream(stream))
    _check(rc, fn_name)
    return pos.value


def _unpack_call(fn_name, inbuf, insize, position, outbuf, outcount, t, stream):
    pos = ctypes.c_int64(position)
    rc = getattr(lib(), fn_name)(_ptr(inbuf), insize, ctypes.byref(pos), _ptr(outbuf), outcount, t, _stream(stream))
    _check(rc, fn_name)
    return pos.value


def pack(inbuf, incount: int, t: int, outbuf, outsize: int, position: int, stream=None) -> int:
    """tp_pack; returns the new position."""
    return _pack_call("tp_pack", inbuf, incount, t, outbuf, outsize, position, stream)


def pack_async(inbuf, incount: int, t: int, outbuf, outsize: int, position: int, stream=None) -> int:
    """tp_pack_async (enqueue only); returns the new position."""
    return _pack_call("tp_pack_async", inbuf, incount, t, outbuf, outsize, position, stream)


def unpack(inbuf, insize: int, position: int, outbuf, outcount: int, t: int, stream=None) -> int:
    """tp_unpack; returns the new position."""
    return _unpack_call("tp_unpack", inbuf, insize, position, outbuf, outcount, t, stream)


def unpack_async(inbuf, insize: int, position: int, outbuf, outcount: int, t: int, stream=None) -> int:
    """tp_unpack_async (enqueue only); returns the new position."""
    return _unpack_call("tp_unpack_async", inbuf, insize, position, outbuf, outcount, t, stream)


class Batch:
    """Marshalled argument arrays of a batched call, reusable across calls (the arrays are built once)."""

    def __init__(self, typed_bufs, counts, types):
        n = len(types)
        assert len(typed_bufs) == len(counts) == n
        self.n = n
        self.ptrs = (ctypes.c_void_p * n)(*[_ptr(b) for b in typed_bufs])
        self.counts = (ctypes.c_int * n)(*counts)
        self.types = (ctypes.c_int32 * n)(*types)


def _batch(fn_name, batch, packed, packed_size, position, stream):
    pos = ctypes.c_int64(position)
    fn = getattr(lib(), fn_name)
    if "unpack" in fn_name:
        rc = fn(batch.n, _ptr(packed), packed_size, ctypes.byref(pos), batch.ptrs, batch.counts, batch.types,
                _stream(stream))
    else:
        rc = fn(batch.n, batch.ptrs, batch.counts, batch.types, _ptr(packed), packed_size, ctypes.byref(pos),
                _stream(stream))
    _check(rc, fn_name)
    return pos.value


def pack_batch(batch: Batch, outbuf, outsize: int, position: int, stream=None) -> int:
    """tp_pack_batch; returns the new position."""
    return _batch("tp_pack_batch", batch, outbuf, outsize, position, stream)


def pack_batch_async(batch: Batch, outbuf, outsize: int, position: int, stream=None) -> int:
    return _batch("tp_pack_batch_async", batch, outbuf, outsize, position, stream)


def unpack_batch(inbuf, insize: int, position: int, batch: Batch, stream=None) -> int:
    """tp_unpack_batch; returns the new position."""
    return _batch("tp_unpack_batch", batch, inbuf, insize, position, stream)


def unpack_batch_async(inbuf, insize: int, position: int, batch: Batch, stream=None) -> int:
    return _batch("tp_unpack_batch_async", batch, inbuf, insize, position, stream)


# ------------------------------------------------------------------ model and host delivery
def model_measure(stream=None) -> None:
    _check(lib().tp_model_measure(_stream(stream)), "tp_model_measure")


def model_save(path: str) -> None:
    _check(lib().tp_model_save(path.encode()), "tp_model_save")


def model_load(path: str) -> None:
    _check(lib().tp_model_load(path.encode()), "tp_model_load")


def model_query(t: int, count: int) -> dict:
    m = ModelTimes()
    _check(lib().tp_model_query(t, count, ctypes.byref(m)), "tp_model_query")
    return m.as_dict()


def model_select(t: int, count: int, t_cpu_cpu: float = 0.0, t_gpu_gpu: float = 0.0):
    """(method, [T_device, T_oneshot, T_staged])"""
    method = ctypes.c_int(-9)
    times = (ctypes.c_double * 3)()
    _check(lib().tp_model_select(t, count, t_cpu_cpu, t_gpu_gpu, ctypes.byref(method), times), "tp_model_select")
    return method.value, list(times)


def pack_host(inbuf, incount, t, host_outbuf, outsize, position, staging=None, staging_size=0,
              method=TP_METHOD_AUTO, stream=None):
    """tp_pack_host; returns (new position, method used)."""
    pos, used = ctypes.c_int64(position), ctypes.c_int(-9)
    rc = lib().tp_pack_host(_ptr(inbuf), incount, t, _ptr(host_outbuf), outsize, ctypes.byref(pos),
                            _ptr(staging) if staging is not None else None, staging_size, method, _stream(stream),
                            ctypes.byref(used))
    _check(rc, "tp_pack_host")
    return pos.value, used.value


TP_STATIC_STAGING_BYTES = 4 << 20


def pack_host_static(inbuf, incount, t, host_outbuf, outsize, position, stream=None) -> int:
    """tp_pack_host_static (staged through the library's fixed device array; allocates nothing); returns the new position."""
    pos = ctypes.c_int64(position)
    rc = lib().tp_pack_host_static(_ptr(inbuf), incount, t, _ptr(host_outbuf), outsize, ctypes.byref(pos), _stream(stream))
    _check(rc, "tp_pack_host_static")
    return pos.value


def unpack_host(host_inbuf, insize, position, outbuf, outcount, t, staging=None, staging_size=0,
                method=TP_METHOD_AUTO, stream=None):
    """tp_unpack_host; returns (new position, method used)."""
    pos, used = ctypes.c_int64(position), ctypes.c_int(-9)
    rc = lib().tp_unpack_host(_ptr(host_inbuf), insize, ctypes.byref(pos), _ptr(outbuf), outcount, t,
                              _ptr(staging) if staging is not None else None, staging_size, method, _stream(stream),
                              ctypes.byref(used))
    _check(rc, "tp_unpack_host")
    return pos.value, used.value


# ------------------------------------------------------------------ resource cache
def resource_acquire(kind: int, nbytes: int = 0) -> int:
    """tp_resource_acquire; returns the handle (buffer address, hipStream_t or hipEvent_t) as an int."""
    h = ctypes.c_void_p()
    _check(lib().tp_resource_acquire(kind, nbytes, ctypes.byref(h)), "tp_resource_acquire")
    return h.value


def resource_release(kind: int, handle: int) -> None:
    _check(lib().tp_resource_release(kind, handle), "tp_resource_release")


def resource_trim() -> int:
    """tp_resource_trim; returns the buffer bytes freed."""
    freed = ctypes.c_int64()
    _check(lib().tp_resource_trim(ctypes.byref(freed)), "tp_resource_trim")
    return freed.value


def resource_stats(kind: int) -> dict:
    c = ResourceCounts()
    _check(lib().tp_resource_stats(kind, ctypes.byref(c)), "tp_resource_stats")
    return c.as_dict()


# ------------------------------------------------------------------ recipes -> handles
def type_from_recipe(recipe, commit: bool = True) -> int:
    """Builds (and by default commits) the datatype a `workloads` recipe names, by
    calling the constructors; intermediate handles are freed."""
    kind = recipe[0]
    if kind == "named":
        return PREDEFINED[recipe[1]]
    old = type_from_recipe(recipe[-1], commit=False)
    if kind == "contiguous":
        new = type_contiguous(recipe[1], old)
    elif kind == "vector":
        new = type_vector(recipe[1], recipe[2], recipe[3], old)
    elif kind == "hvector":
        new = type_create_hvector(recipe[1], recipe[2], recipe[3], old)
    elif kind == "subarray":
        _, sizes, subs, starts, order, _old = recipe
        new = type_create_subarray(sizes, subs, starts, TP_ORDER_C if order == "C" else TP_ORDER_FORTRAN, old)
    else:
        raise ValueError(kind)
    if old >= 12:
        type_free(old)
    if commit:
        type_commit(new)
    return new

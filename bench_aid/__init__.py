"""ctypes loader of the benchmark's measurement aid (bench_aid/stream_probe.h).  Used by bench.py and by the
tests of the aid itself; the MG-WFBP library does not know about it."""
from __future__ import annotations

import ctypes as C
import os
from typing import Optional, Sequence

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB: Optional[C.CDLL] = None
_vp = C.c_void_p


class BenchAidError(RuntimeError):
    pass


def library_path() -> str:
    return os.path.join(_HERE, "libmgwfbp_bench_aid.so")


def lib() -> C.CDLL:
    global _LIB
    if _LIB is None:
        path = library_path()
        if not os.path.exists(path):
            raise BenchAidError(f"{path} is not built; run `python -m paper_1912_09268_amd.build`")
        h = C.CDLL(path)
        h.bench_aid_stream_probe.restype = C.c_int
        h.bench_aid_stream_probe.argtypes = [C.POINTER(_vp), C.c_int32, C.POINTER(_vp), C.c_int32, C.POINTER(_vp),
                                             C.c_int32, C.c_uint64, _vp]
        h.bench_aid_paced_probe.restype = C.c_int
        h.bench_aid_paced_probe.argtypes = [C.POINTER(_vp), C.c_int32, C.POINTER(_vp), C.c_int32, C.POINTER(_vp),
                                            C.c_int32, C.c_uint64, C.c_int32, C.c_int32, C.c_uint32, _vp]
        h.bench_aid_cache_scrub.restype = C.c_int
        h.bench_aid_cache_scrub.argtypes = [_vp, C.c_uint64, _vp]
        _LIB = h
    return _LIB


def stream_probe(read_ptrs: Sequence[int], write_ptrs: Sequence[int], update_ptrs: Sequence[int], elems: int,
                 stream: int = 0) -> None:
    """bench_aid_stream_probe: lists of device addresses of binary32 arrays of `elems` elements each."""
    def table(addrs):
        return (_vp * max(len(addrs), 1))(*[int(a) for a in addrs]) if addrs else None
    rc = lib().bench_aid_stream_probe(table(read_ptrs), len(read_ptrs), table(write_ptrs), len(write_ptrs),
                                      table(update_ptrs), len(update_ptrs), int(elems), _vp(stream))
    if rc != 0:
        raise BenchAidError(f"bench_aid_stream_probe failed: {rc}")


def paced_probe(read_ptrs: Sequence[int], write_ptrs: Sequence[int], update_ptrs: Sequence[int], elems: int,
                block_lanes: int, vectors_per_step: int, lds_bytes: int, stream: int = 0) -> None:
    """bench_aid_paced_probe: the same arrays, one array at a time, with an occupancy cap through unused LDS."""
    def table(addrs):
        return (_vp * max(len(addrs), 1))(*[int(a) for a in addrs]) if addrs else None
    rc = lib().bench_aid_paced_probe(table(read_ptrs), len(read_ptrs), table(write_ptrs), len(write_ptrs),
                                     table(update_ptrs), len(update_ptrs), int(elems), int(block_lanes),
                                     int(vectors_per_step), int(lds_bytes), _vp(stream))
    if rc != 0:
        raise BenchAidError(f"bench_aid_paced_probe failed: {rc}")


def cache_scrub(buf: int, nbytes: int, stream: int = 0) -> None:
    """bench_aid_cache_scrub on the device buffer at address `buf`."""
    rc = lib().bench_aid_cache_scrub(_vp(buf), int(nbytes), _vp(stream))
    if rc != 0:
        raise BenchAidError(f"bench_aid_cache_scrub failed: {rc}")

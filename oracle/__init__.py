"""TEST INFRASTRUCTURE -- not part of the product path.

CPU oracle for the non-uniform all-to-all: the MPI_Alltoallv definition
(recv[j][i] = send[i][j]) in plain C (alltoallv_oracle.c), loaded through ctypes,
plus `tuna_model`, a slow per-rank model of the paper's algorithms used to pin the
round structure.  Only tests, the smoke check and the benchmark's cpu_baseline leg
may import this package; the GPU library never does and shares no code with it.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "alltoallv_oracle.c")
_LIB = os.path.join(_HERE, "liboracle.so")

OK = 0
ERR_ARG = -1
ERR_COUNT_MISMATCH = -2
ERR_NEGATIVE_COUNT = -3


def build(force: bool = False) -> str:
    """Compile the C oracle with gcc (-O2, no vectorisation tricks asked for)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        tmp = _LIB + ".tmp.%d" % os.getpid()
        subprocess.check_call(["gcc", "-O2", "-std=c11", "-shared", "-fPIC", "-o", tmp, _SRC])
        os.replace(tmp, _LIB)
    return _LIB


_lib = None


def _load():
    global _lib
    if _lib is None:
        build()
        lib = ctypes.CDLL(_LIB)
        vp, ip, i32 = ctypes.c_void_p, ctypes.c_int, ctypes.c_int
        lib.oracle_check_counts.argtypes = [vp, vp, ip]
        lib.oracle_check_counts.restype = i32
        lib.oracle_alltoallv.argtypes = [vp, vp, vp, vp, vp, vp, ip]
        lib.oracle_alltoallv.restype = i32
        lib.oracle_alltoallv_receivers.argtypes = [vp, vp, vp, vp, vp, vp, ip, vp, ip]
        lib.oracle_alltoallv_receivers.restype = i32
        _lib = lib
    return _lib


def _p(a: np.ndarray) -> ctypes.c_void_p:
    return ctypes.c_void_p(a.ctypes.data)


def _mats(sendcounts, sdispls, recvcounts, rdispls):
    P = sendcounts.shape[0]
    sc = np.ascontiguousarray(sendcounts, dtype=np.int32)
    sd = np.ascontiguousarray(sdispls, dtype=np.int64)
    rc = np.ascontiguousarray(recvcounts, dtype=np.int32)
    rd = np.ascontiguousarray(rdispls, dtype=np.int64)
    assert sc.shape == sd.shape == rc.shape == rd.shape == (P, P)
    return P, sc, sd, rc, rd


def alltoallv(send: np.ndarray, sendcounts, sdispls, recv: np.ndarray, recvcounts, rdispls) -> int:
    """recv[rdispls[j,i] : +sendcounts[i,j]] = send[sdispls[i,j] : +sendcounts[i,j]] for all i, j.
    `send`/`recv` are uint8 arrays (whole allocations); `recv` is written in place.  Returns the C
    status code (0 = ok)."""
    P, sc, sd, rc, rd = _mats(sendcounts, sdispls, recvcounts, rdispls)
    assert send.dtype == np.uint8 and recv.dtype == np.uint8
    assert send.flags.c_contiguous and recv.flags.c_contiguous
    _bounds(send.size, sc, sd)
    _bounds(recv.size, rc, rd)
    return int(_load().oracle_alltoallv(_p(send), _p(sc), _p(sd), _p(recv), _p(rc), _p(rd), P))


def alltoallv_receivers(send, sendcounts, sdispls, recv, recvcounts, rdispls, receivers) -> int:
    """The same definition for a subset of receiving ranks only."""
    P, sc, sd, rc, rd = _mats(sendcounts, sdispls, recvcounts, rdispls)
    rv = np.ascontiguousarray(receivers, dtype=np.int32)
    _bounds(send.size, sc, sd)
    _bounds(recv.size, rc[rv], rd[rv])
    return int(_load().oracle_alltoallv_receivers(_p(send), _p(sc), _p(sd), _p(recv), _p(rc), _p(rd),
                                                  P, _p(rv), int(rv.size)))


def check_counts(sendcounts, recvcounts) -> int:
    sc = np.ascontiguousarray(sendcounts, dtype=np.int32)
    rc = np.ascontiguousarray(recvcounts, dtype=np.int32)
    return int(_load().oracle_check_counts(_p(sc), _p(rc), sc.shape[0]))


def _bounds(nbytes: int, counts: np.ndarray, displs: np.ndarray) -> None:
    """Host-side guard so a malformed test input raises instead of corrupting memory."""
    c = counts.astype(np.int64)
    live = c > 0
    if live.any():
        lo = displs[live].min()
        hi = (displs[live] + c[live]).max()
        if lo < 0 or hi > nbytes:
            raise ValueError("block outside the allocation: [%d, %d) vs %d bytes" % (lo, hi, nbytes))

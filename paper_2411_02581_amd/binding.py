"""ctypes binding of libtuna.so: argument marshalling only.

Every function has the name and the argument order of its C entry point in include/tuna.h.
Device arrays may be given as torch tensors (their data_ptr() is passed) or as integer device
addresses.  Nothing here computes: if the HIP library is missing and cannot be built the import
of the entry points fails loudly; there is no CPU fallback.
"""
from __future__ import annotations

import ctypes
import os
from typing import Any, Optional

from . import build as _build

TUNA_OK = 0
TUNA_ERR_ARG = -1
TUNA_ERR_COUNT_MISMATCH = -2
TUNA_ERR_NEGATIVE_COUNT = -3
TUNA_ERR_NOMEM = -4
TUNA_ERR_WORKSPACE_TOO_SMALL = -5
TUNA_ERR_HIP = -6
TUNA_ERR_TOO_LARGE = -7
TUNA_ERR_NOALLOC_LIMIT = -8
TUNA_NOALLOC_SCRATCH_BYTES = 64 << 20
TUNA_OPT_PROFILE = 1
TUNA_OPT_FUSED = 2
TUNA_OPT_STAGGERED = 3
TUNA_OPT_DENSE_T = 4
TUNA_OPT_BLOCK_COUNT = 5
TUNA_MAX_PHASES = 64
TUNA_RADIX_AUTO = 0
TUNA_MODE_AUTO, TUNA_MODE_STAGED, TUNA_MODE_FUSED = 0, 1, 2
TUNA_T_SLOTS, TUNA_T_EXACT, TUNA_T_AUTO = 0, 1, 2

EXPORTS = ("tuna_alltoallv", "tuna_alltoallv_hier", "tuna_alltoallv_noalloc", "tuna_alltoallv_ex", "tuna_alltoallv_init_ex",
           "tuna_opts_init", "tuna_ctx_create", "tuna_ctx_destroy", "tuna_ctx_get_stats", "tuna_build_id", "tuna_debug_phase_sizes", "tuna_workspace_bytes", "tuna_set_workspace",
           "tuna_release", "tuna_set_option", "tuna_get_stats", "tuna_plan_info", "tuna_plan_phase",
           "tuna_t_index", "tuna_plan_phase_device", "tuna_plan_phase_sources", "tuna_plain_copy", "tuna_select", "tuna_predict_ms", "tuna_calibrate", "tuna_model_constants", "tuna_alltoallv_init", "tuna_start", "tuna_plan_free",
           "tuna_strerror", "tuna_version")


class tuna_phase_stats_t(ctypes.Structure):
    _fields_ = [("dim", ctypes.c_int32), ("x", ctypes.c_int32), ("radix", ctypes.c_int32),
                ("rounds", ctypes.c_int32), ("blocks", ctypes.c_int64),
                ("payload_bytes", ctypes.c_int64), ("staged_bytes", ctypes.c_int64),
                ("ms_metadata", ctypes.c_float), ("ms_pack", ctypes.c_float),
                ("ms_exchange", ctypes.c_float), ("ms_unpack", ctypes.c_float)]


class tuna_stats_t(ctypes.Structure):
    _fields_ = [("P", ctypes.c_int32), ("Q", ctypes.c_int32), ("N", ctypes.c_int32),
                ("local_radix", ctypes.c_int32), ("global_radix", ctypes.c_int32),
                ("w_local", ctypes.c_int32), ("w_global", ctypes.c_int32),
                ("K_local", ctypes.c_int32), ("K_global", ctypes.c_int32),
                ("B_local", ctypes.c_int32), ("B_global", ctypes.c_int32),
                ("n_phases", ctypes.c_int32), ("granularity", ctypes.c_int32),
                ("fused", ctypes.c_int32), ("last_hip_error", ctypes.c_int32),
                ("dense_t", ctypes.c_int32),
                ("max_block_bytes", ctypes.c_int64), ("total_payload_bytes", ctypes.c_int64),
                ("temp_slots_per_rank", ctypes.c_int64), ("temp_bytes", ctypes.c_int64),
                ("staging_bytes", ctypes.c_int64), ("workspace_bytes", ctypes.c_int64),
                ("ms_prepare", ctypes.c_float), ("ms_self", ctypes.c_float),
                ("ms_total", ctypes.c_float), ("reserved_f", ctypes.c_float),
                ("phase", tuna_phase_stats_t * TUNA_MAX_PHASES)]


class tuna_opts_t(ctypes.Structure):
    _fields_ = [("struct_size", ctypes.c_int32), ("mode", ctypes.c_int32), ("staggered", ctypes.c_int32),
                ("t_layout", ctypes.c_int32), ("block_count", ctypes.c_int32), ("profile", ctypes.c_int32),
                ("reserved", ctypes.c_int32 * 2)]


class tuna_choice_t(ctypes.Structure):
    _fields_ = [("local_radix", ctypes.c_int32), ("global_radix", ctypes.c_int32), ("mode", ctypes.c_int32),
                ("t_layout", ctypes.c_int32), ("calibrated", ctypes.c_int32), ("reserved", ctypes.c_int32),
                ("predicted_ms", ctypes.c_double)]


class tuna_plan_info_t(ctypes.Structure):
    _fields_ = [("P", ctypes.c_int32), ("Q", ctypes.c_int32), ("N", ctypes.c_int32),
                ("local_radix", ctypes.c_int32), ("global_radix", ctypes.c_int32),
                ("w_local", ctypes.c_int32), ("w_global", ctypes.c_int32),
                ("K_local", ctypes.c_int32), ("K_global", ctypes.c_int32),
                ("B_local", ctypes.c_int32), ("B_global", ctypes.c_int32),
                ("n_phases", ctypes.c_int32),
                ("temp_slots_per_rank", ctypes.c_int64), ("blocks_sent_per_rank", ctypes.c_int64)]


_lib: Optional[ctypes.CDLL] = None


def library_path() -> str:
    return _build.LIB


def load() -> ctypes.CDLL:
    """Load libtuna.so.  The library carries a hash of the sources it was built from: when that differs
    from the sources next to it (or no library exists) it is rebuilt first, so that tests and benchmarks
    never report on code that is not the code in the tree."""
    global _lib
    if _lib is not None:
        return _lib
    path = os.environ.get("TUNA_LIBRARY", "")      # debugging aid: load another build of the library
    if not path:
        path = _build.LIB
        if not os.path.exists(path) or _built_from(path) != _build.source_hash():
            _build.build_library(force=True)
    lib = ctypes.CDLL(path)
    vp, i, i64p = ctypes.c_void_p, ctypes.c_int, ctypes.c_void_p
    lib.tuna_alltoallv.argtypes = [vp, vp, vp, vp, vp, vp, i, i, i, vp]
    lib.tuna_alltoallv_hier.argtypes = [vp, vp, vp, vp, vp, vp, i, i, i, i, vp]
    lib.tuna_alltoallv_noalloc.argtypes = [vp, vp, vp, vp, vp, vp, i, i, i, i, vp]
    lib.tuna_alltoallv_ex.argtypes = [vp, vp, vp, vp, vp, vp, vp, i, i, i, i, ctypes.POINTER(tuna_opts_t), vp]
    lib.tuna_alltoallv_init_ex.argtypes = [vp, vp, vp, vp, vp, vp, vp, i, i, i, i, ctypes.POINTER(tuna_opts_t), vp,
                                           ctypes.POINTER(ctypes.c_void_p)]
    lib.tuna_opts_init.argtypes = [ctypes.POINTER(tuna_opts_t)]
    lib.tuna_ctx_create.argtypes = [ctypes.POINTER(ctypes.c_void_p)]
    lib.tuna_ctx_destroy.argtypes = [vp]
    lib.tuna_ctx_get_stats.argtypes = [vp, ctypes.POINTER(tuna_stats_t)]
    lib.tuna_debug_phase_sizes.argtypes = [vp, vp, vp, vp, vp, vp, i, i, i, i, vp, vp, i]
    lib.tuna_build_id.argtypes = []
    lib.tuna_build_id.restype = ctypes.c_char_p
    lib.tuna_alltoallv_init.argtypes = [vp, vp, vp, vp, vp, vp, i, i, i, i, vp, ctypes.POINTER(ctypes.c_void_p)]
    lib.tuna_start.argtypes = [vp, vp]
    lib.tuna_plan_free.argtypes = [vp]
    lib.tuna_workspace_bytes.argtypes = [vp, i, i, i, i, ctypes.POINTER(ctypes.c_size_t)]
    lib.tuna_set_workspace.argtypes = [vp, ctypes.c_size_t]
    lib.tuna_release.argtypes = []
    lib.tuna_set_option.argtypes = [i, i]
    lib.tuna_get_stats.argtypes = [ctypes.POINTER(tuna_stats_t)]
    lib.tuna_plan_info.argtypes = [i, i, i, i, ctypes.POINTER(tuna_plan_info_t)]
    lib.tuna_plan_phase.argtypes = [i, i, i, i, i, vp, vp, i]
    lib.tuna_select.argtypes = [i, i, ctypes.c_int64, ctypes.c_int64, i, ctypes.POINTER(tuna_choice_t)]
    lib.tuna_predict_ms.argtypes = [i, i, i, i, i, i, ctypes.c_int64, ctypes.c_int64, i, ctypes.POINTER(ctypes.c_double)]
    lib.tuna_calibrate.argtypes = [vp]
    lib.tuna_model_constants.argtypes = [i, ctypes.POINTER(ctypes.c_double), i]
    lib.tuna_plan_phase_device.argtypes = [i, i, i, i, i, vp, i]
    lib.tuna_plan_phase_sources.argtypes = [i, i, i, i, i, i, vp, i]
    lib.tuna_t_index.argtypes = [i, i]
    lib.tuna_plain_copy.argtypes = [vp, vp, ctypes.c_size_t, vp]
    lib.tuna_strerror.argtypes = [i]
    lib.tuna_strerror.restype = ctypes.c_char_p
    lib.tuna_version.argtypes = []
    for name in EXPORTS:
        if name not in ("tuna_strerror", "tuna_build_id"):
            getattr(lib, name).restype = ctypes.c_int
    _lib = lib
    return lib


def _built_from(path: str) -> str:
    """tuna_build_id of the library file at `path`, read from the file (the library is not loaded: a
    stale one could not be unloaded again)."""
    marker = b"tuna-build-id:"
    try:
        with open(path, "rb") as f:
            data = f.read()
    except OSError:
        return ""
    k = data.find(marker)
    return data[k + len(marker):k + len(marker) + 16].decode("ascii", "replace") if k >= 0 else ""


def _ptr(a: Any, dtype=None) -> Optional[int]:
    """Device address of a torch tensor (checked) or a plain integer address."""
    if a is None:
        return None
    if isinstance(a, int):
        return a
    if not a.is_cuda:
        raise TypeError("device tensor expected")
    if not a.is_contiguous():
        raise TypeError("contiguous tensor expected")
    if dtype is not None and a.dtype != dtype:
        raise TypeError("tensor dtype %s, expected %s" % (a.dtype, dtype))
    return a.data_ptr()


def _stream(stream: Any) -> Optional[int]:
    if stream is None:
        import torch
        return torch.cuda.current_stream().cuda_stream
    if isinstance(stream, int):
        return stream
    return stream.cuda_stream


def tuna_alltoallv(sendbuf, sendcounts, sdispls, recvbuf, recvcounts, rdispls, P: int, radix: int,
                   ranks_per_node: int = 0, stream=None) -> int:
    import torch
    return load().tuna_alltoallv(_ptr(sendbuf), _ptr(sendcounts, torch.int32), _ptr(sdispls, torch.int64),
                                 _ptr(recvbuf), _ptr(recvcounts, torch.int32), _ptr(rdispls, torch.int64),
                                 P, radix, ranks_per_node, _stream(stream))


def tuna_alltoallv_hier(sendbuf, sendcounts, sdispls, recvbuf, recvcounts, rdispls, P: int,
                        ranks_per_node: int, local_radix: int, global_radix: int, stream=None) -> int:
    import torch
    return load().tuna_alltoallv_hier(_ptr(sendbuf), _ptr(sendcounts, torch.int32), _ptr(sdispls, torch.int64),
                                      _ptr(recvbuf), _ptr(recvcounts, torch.int32), _ptr(rdispls, torch.int64),
                                      P, ranks_per_node, local_radix, global_radix, _stream(stream))


def tuna_opts_init() -> tuna_opts_t:
    """A tuna_opts_t holding the process-wide defaults."""
    o = tuna_opts_t()
    rc = load().tuna_opts_init(ctypes.byref(o))
    if rc != TUNA_OK:
        raise RuntimeError("tuna_opts_init: " + tuna_strerror(rc))
    return o


def tuna_ctx_create():
    """Returns (code, context handle)."""
    ctx = ctypes.c_void_p(None)
    rc = load().tuna_ctx_create(ctypes.byref(ctx))
    return rc, ctx.value


def tuna_ctx_destroy(ctx) -> int:
    return load().tuna_ctx_destroy(ctx)


def tuna_ctx_get_stats(ctx) -> tuna_stats_t:
    st = tuna_stats_t()
    rc = load().tuna_ctx_get_stats(ctx, ctypes.byref(st))
    if rc != TUNA_OK:
        raise RuntimeError("tuna_ctx_get_stats: " + tuna_strerror(rc))
    return st


def tuna_alltoallv_ex(ctx, sendbuf, sendcounts, sdispls, recvbuf, recvcounts, rdispls, P: int, ranks_per_node: int,
                      local_radix: int, global_radix: int, opts: Optional[tuna_opts_t] = None, stream=None) -> int:
    import torch
    return load().tuna_alltoallv_ex(ctx, _ptr(sendbuf), _ptr(sendcounts, torch.int32), _ptr(sdispls, torch.int64),
                                    _ptr(recvbuf), _ptr(recvcounts, torch.int32), _ptr(rdispls, torch.int64),
                                    P, ranks_per_node, local_radix, global_radix,
                                    ctypes.byref(opts) if opts is not None else None, _stream(stream))


def tuna_alltoallv_init_ex(ctx, sendbuf, sendcounts, sdispls, recvbuf, recvcounts, rdispls, P: int,
                           ranks_per_node: int, local_radix: int, global_radix: int,
                           opts: Optional[tuna_opts_t] = None, stream=None):
    """Returns (code, plan handle)."""
    import torch
    plan = ctypes.c_void_p(None)
    rc = load().tuna_alltoallv_init_ex(ctx, _ptr(sendbuf), _ptr(sendcounts, torch.int32), _ptr(sdispls, torch.int64),
                                       _ptr(recvbuf), _ptr(recvcounts, torch.int32), _ptr(rdispls, torch.int64),
                                       P, ranks_per_node, local_radix, global_radix,
                                       ctypes.byref(opts) if opts is not None else None, _stream(stream),
                                       ctypes.byref(plan))
    return rc, plan.value


def tuna_debug_phase_sizes(sendbuf, sendcounts, sdispls, recvbuf, recvcounts, rdispls, P: int, ranks_per_node: int,
                           local_radix: int, global_radix: int, n_phases: int, stream=None):
    """Returns (code, sizes[n_phases + 1, P, P] int32): the device's block-size matrix before the first
    phase and after every phase."""
    import numpy as np
    import torch
    sizes = np.zeros((n_phases + 1, P, P), dtype=np.int32)
    rc = load().tuna_debug_phase_sizes(_ptr(sendbuf), _ptr(sendcounts, torch.int32), _ptr(sdispls, torch.int64),
                                       _ptr(recvbuf), _ptr(recvcounts, torch.int32), _ptr(rdispls, torch.int64),
                                       P, ranks_per_node, local_radix, global_radix, _stream(stream),
                                       sizes.ctypes.data, n_phases + 1)
    return rc, sizes


def tuna_build_id() -> str:
    return load().tuna_build_id().decode()


def tuna_alltoallv_noalloc(sendbuf, sendcounts, sdispls, recvbuf, recvcounts, rdispls, P: int,
                           ranks_per_node: int, local_radix: int, global_radix: int, stream=None) -> int:
    import torch
    return load().tuna_alltoallv_noalloc(_ptr(sendbuf), _ptr(sendcounts, torch.int32), _ptr(sdispls, torch.int64),
                                         _ptr(recvbuf), _ptr(recvcounts, torch.int32), _ptr(rdispls, torch.int64),
                                         P, ranks_per_node, local_radix, global_radix, _stream(stream))


def tuna_alltoallv_init(sendbuf, sendcounts, sdispls, recvbuf, recvcounts, rdispls, P: int,
                        ranks_per_node: int, local_radix: int, global_radix: int, stream=None):
    """Returns (code, plan handle).  The handle is an opaque integer for tuna_start / tuna_plan_free."""
    import torch
    plan = ctypes.c_void_p(None)
    rc = load().tuna_alltoallv_init(_ptr(sendbuf), _ptr(sendcounts, torch.int32), _ptr(sdispls, torch.int64),
                                    _ptr(recvbuf), _ptr(recvcounts, torch.int32), _ptr(rdispls, torch.int64),
                                    P, ranks_per_node, local_radix, global_radix, _stream(stream),
                                    ctypes.byref(plan))
    return rc, plan.value


def tuna_start(plan, stream=None) -> int:
    return load().tuna_start(plan, _stream(stream))


def tuna_plan_free(plan) -> int:
    return load().tuna_plan_free(plan)


def tuna_workspace_bytes(sendcounts, P: int, ranks_per_node: int, local_radix: int, global_radix: int):
    """Returns (code, bytes)."""
    import torch
    out = ctypes.c_size_t(0)
    rc = load().tuna_workspace_bytes(_ptr(sendcounts, torch.int32), P, ranks_per_node, local_radix,
                                     global_radix, ctypes.byref(out))
    return rc, int(out.value)


def tuna_set_workspace(workspace, nbytes: int) -> int:
    return load().tuna_set_workspace(_ptr(workspace), nbytes)


def tuna_release() -> int:
    return load().tuna_release()


def tuna_set_option(option: int, value: int) -> int:
    return load().tuna_set_option(option, value)


def tuna_get_stats() -> tuna_stats_t:
    st = tuna_stats_t()
    rc = load().tuna_get_stats(ctypes.byref(st))
    if rc != TUNA_OK:
        raise RuntimeError("tuna_get_stats: " + tuna_strerror(rc))
    return st


def tuna_plan_info(P: int, ranks_per_node: int, local_radix: int, global_radix: int):
    """Returns (code, tuna_plan_info_t).  Host only."""
    info = tuna_plan_info_t()
    rc = load().tuna_plan_info(P, ranks_per_node, local_radix, global_radix, ctypes.byref(info))
    return rc, info


def tuna_plan_phase(P: int, ranks_per_node: int, local_radix: int, global_radix: int, phase: int):
    """Returns (code, header[6], seg[nseg,6]) as numpy int32 arrays.  Host only."""
    import numpy as np
    header = np.zeros(6, dtype=np.int32)
    lib = load()
    rc = lib.tuna_plan_phase(P, ranks_per_node, local_radix, global_radix, phase, header.ctypes.data, None, 0)
    if rc != TUNA_OK:
        return rc, header, None
    seg = np.zeros((int(header[4]), 6), dtype=np.int32)
    rc = lib.tuna_plan_phase(P, ranks_per_node, local_radix, global_radix, phase, header.ctypes.data,
                             seg.ctypes.data, seg.shape[0])
    return rc, header, seg


def tuna_select(P: int, ranks_per_node: int, payload_bytes: int, max_block_bytes: int = 0, granularity: int = 0):
    """Returns (code, tuna_choice_t).  Host only."""
    ch = tuna_choice_t()
    rc = load().tuna_select(P, ranks_per_node, payload_bytes, max_block_bytes, granularity, ctypes.byref(ch))
    return rc, ch


def tuna_predict_ms(P: int, ranks_per_node: int, local_radix: int, global_radix: int, mode: int, t_layout: int,
                    payload_bytes: int, max_block_bytes: int = 0, granularity: int = 0):
    """Returns (code, predicted milliseconds of one immediate call).  Host only."""
    ms = ctypes.c_double(0.0)
    rc = load().tuna_predict_ms(P, ranks_per_node, local_radix, global_radix, mode, t_layout, payload_bytes,
                                max_block_bytes, granularity, ctypes.byref(ms))
    return rc, ms.value


def tuna_calibrate(stream=None) -> int:
    return load().tuna_calibrate(_stream(stream))


TUNA_MODEL_CONSTANTS = 10


def tuna_model_constants(mode: int):
    """Returns (code, [c0 .. c6, slot factor, byte-granular factor, line-granular factor]) of the cost model for `mode`.
    Host only."""
    c = (ctypes.c_double * TUNA_MODEL_CONSTANTS)()
    rc = load().tuna_model_constants(mode, c, TUNA_MODEL_CONSTANTS)
    return rc, list(c)


def tuna_plan_phase_device(P: int, ranks_per_node: int, local_radix: int, global_radix: int, phase: int, nseg: int):
    """Returns (code, seg[nseg,4]) as the device holds the table: {e, z, src_slot, dst_slot}."""
    import numpy as np
    seg = np.zeros((nseg, 4), dtype=np.int32)
    rc = load().tuna_plan_phase_device(P, ranks_per_node, local_radix, global_radix, phase, seg.ctypes.data, nseg)
    return rc, seg


def tuna_plan_phase_sources(P: int, ranks_per_node: int, local_radix: int, global_radix: int, phase: int, nseg: int,
                            on_device: bool = False):
    """Returns (code, src[nseg,2]): {phase of the block's previous move or -1, its position there}."""
    import numpy as np
    out = np.zeros((nseg, 2), dtype=np.int32)
    rc = load().tuna_plan_phase_sources(P, ranks_per_node, local_radix, global_radix, phase, 1 if on_device else 0,
                                        out.ctypes.data, nseg)
    return rc, out


def tuna_t_index(o: int, radix: int) -> int:
    return load().tuna_t_index(o, radix)


def tuna_plain_copy(src, dst, nbytes: int, stream=None) -> int:
    return load().tuna_plain_copy(_ptr(src), _ptr(dst), nbytes, _stream(stream))


def tuna_strerror(code: int) -> str:
    return load().tuna_strerror(code).decode()


def tuna_version() -> int:
    return load().tuna_version()

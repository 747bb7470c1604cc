"""ctypes binding of libflux_mi355.so: argument marshalling only.

Every function here has the name of the C entry point it calls (include/flux.h); tensors are
torch CUDA(HIP) tensors used purely as device buffers, streams are torch streams.  Nothing is
computed in Python.  Loading fails loudly when the library has not been built
(`python -m paper_2406_06858_amd.build`).
"""
from __future__ import annotations

import ctypes as C
import os
from dataclasses import dataclass

import torch

_LIB_PATH = os.path.join(os.path.dirname(os.path.abspath(__file__)), "libflux_mi355.so")
_lib = None

FLUX_OK, FLUX_ERR_INVALID_ARG, FLUX_ERR_SHAPE, FLUX_ERR_UNSUPPORTED = 0, 1, 2, 3
FLUX_ERR_WORKSPACE, FLUX_ERR_HIP, FLUX_ERR_TIMEOUT = 4, 5, 6
FLUX_BF16, FLUX_F32 = 0, 1
FLUX_OP_RS, FLUX_OP_AG = 0, 1
FLUX_FLAG_NO_SWIZZLE, FLUX_FLAG_NO_XCD_REMAP, FLUX_FLAG_COPY_MEMCPY = 0x1, 0x2, 0x4
FLUX_FLAG_NO_TAIL_SPLIT = 0x10
FLUX_FLAG_RS_WRITE_ONLY = 0x20
FLUX_FLAG_AG_ABSENT_OWNERS = 0x40
FLUX_FLAG_NO_RESIDENT_GRID = 0x100
FLUX_FLAG_AG_COPY_UPFRONT = 0x200
FLUX_FLAG_RS_ATOMIC = 0x80
FLUX_PHASE_GEMM, FLUX_PHASE_COMM = 0x1, 0x2
FLUX_MAX_RANKS = 16

EXPORTS = [
    "flux_gemm_rs", "flux_ag_gemm", "flux_gemm_ref_unfused", "flux_workspace_bytes",
    "flux_query_status", "flux_tile_coord", "flux_tile_shape", "flux_tile_config_count",
    "flux_tile_config_info", "flux_default_order", "flux_status_string", "flux_last_hip_error",
    "flux_version", "flux_profile_next_gemm", "flux_init_buffers", "flux_split_plan", "flux_gemm_ref_chunked",
    "flux_chunked_workspace_bytes", "flux_rs_reduce_slice",
    "flux_autotune_rs", "flux_autotune_ag", "flux_autotune_workspace_bytes", "flux_autotune_signal_count",
    "flux_trace_next_call", "flux_gemm_rs_static",
    "flux_gemm_rs_notify", "flux_rs_reduce_slice_ready", "flux_rs_ready_count", "flux_rs_resident_grid", "flux_ag_deferred_tiles",
]


class flux_problem_t(C.Structure):
    _fields_ = [
        ("M", C.c_int32), ("N", C.c_int32), ("K", C.c_int32),
        ("R", C.c_int32), ("rank", C.c_int32),
        ("partial_dtype", C.c_int32), ("out_dtype", C.c_int32),
        ("tile_config", C.c_int32), ("split_k", C.c_int32),
        ("flags", C.c_uint32),
        ("comm_tiles_per_chunk", C.c_int32), ("copy_workgroups", C.c_int32),
        ("link_gbps", C.c_int32), ("reserved", C.c_int32),
        ("spin_timeout_ticks", C.c_uint64),
        ("lda", C.c_int64), ("ldb", C.c_int64), ("ldc", C.c_int64),
        ("b_is_nk", C.c_int32), ("reserved2", C.c_int32),
    ]


class FluxError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        msg = lib().flux_status_string(status).decode()
        if status == FLUX_ERR_HIP:
            msg += f" (hipError_t {lib().flux_last_hip_error()})"
        super().__init__(f"{where}: {msg} [status {status}]")


def lib():
    """Loads the shared library on first use."""
    global _lib
    if _lib is None:
        if not os.path.exists(_LIB_PATH):
            raise RuntimeError(f"{_LIB_PATH} is missing: build it with `python -m paper_2406_06858_amd.build`")
        L = C.CDLL(_LIB_PATH)
        vp, pvp = C.c_void_p, C.POINTER(C.c_void_p)
        pp, pi32 = C.POINTER(flux_problem_t), C.POINTER(C.c_int32)
        L.flux_gemm_rs.argtypes = [pp, vp, vp, pvp, pvp, vp, C.c_size_t, vp]
        L.flux_gemm_rs_static.argtypes = [pp, vp, vp, pvp, pvp, vp]
        L.flux_gemm_rs_static.restype = C.c_int
        L.flux_gemm_rs_notify.argtypes = [pp, vp, vp, pvp, vp, vp, C.c_size_t, vp]
        L.flux_gemm_rs_notify.restype = C.c_int
        L.flux_rs_reduce_slice_ready.argtypes = [pp, pvp, vp, vp, C.c_int32, vp, C.c_size_t, vp]
        L.flux_rs_reduce_slice_ready.restype = C.c_int
        L.flux_rs_ready_count.argtypes = [pp]
        L.flux_rs_ready_count.restype = C.c_int32
        L.flux_ag_deferred_tiles.argtypes = [pp]
        L.flux_ag_deferred_tiles.restype = C.c_int32
        L.flux_rs_resident_grid.argtypes = [pp, C.POINTER(C.c_uint32)]
        L.flux_rs_resident_grid.restype = C.c_int32
        L.flux_ag_gemm.argtypes = [pp, pvp, vp, vp, vp, vp, pi32, vp, C.c_size_t, vp, vp]
        L.flux_gemm_ref_unfused.argtypes = [C.c_int, C.c_int, pp, vp, pvp, vp, vp, pvp, pvp, vp, vp, C.c_size_t, vp]
        L.flux_gemm_ref_chunked.argtypes = [C.c_int, pp, vp, pvp, vp, vp, pvp, pvp, vp, pi32, vp, C.c_size_t, vp, vp]
        L.flux_chunked_workspace_bytes.argtypes = [C.c_int, pp]
        L.flux_rs_reduce_slice.argtypes = [pp, pvp, vp, vp]
        L.flux_rs_reduce_slice.restype = C.c_int
        L.flux_chunked_workspace_bytes.restype = C.c_size_t
        pf = C.POINTER(C.c_float)
        L.flux_autotune_rs.argtypes = [pp, vp, vp, pvp, pvp, vp, C.c_size_t, vp, C.c_int32, pp, pf, pf]
        L.flux_autotune_ag.argtypes = [pp, pvp, vp, vp, vp, vp, C.c_int32, pi32, vp, C.c_size_t, vp, vp, C.c_int32, pp, pf, pf]
        L.flux_autotune_workspace_bytes.argtypes = [C.c_int, pp]
        L.flux_autotune_workspace_bytes.restype = C.c_size_t
        L.flux_autotune_signal_count.argtypes = [pp]
        L.flux_workspace_bytes.argtypes = [C.c_int, pp]
        L.flux_workspace_bytes.restype = C.c_size_t
        L.flux_init_buffers.argtypes = [C.c_int, pp, vp, C.c_size_t, vp, vp]
        L.flux_query_status.argtypes = [vp, pi32, pi32]
        L.flux_tile_coord.argtypes = [C.c_int, pp, pi32, C.c_int32, pi32, pi32]
        L.flux_tile_shape.argtypes = [C.c_int, pp, pi32, pi32, pi32, pi32, pi32]
        L.flux_split_plan.argtypes = [C.c_int, pp, pi32, pi32, pi32]
        L.flux_tile_config_info.argtypes = [C.c_int32, pi32, pi32, pi32]
        L.flux_default_order.argtypes = [C.c_int32, C.c_int32, pi32]
        L.flux_profile_next_gemm.argtypes = [vp, vp]
        L.flux_trace_next_call.argtypes = [vp, C.c_size_t]
        L.flux_trace_next_call.restype = C.c_int
        L.flux_status_string.argtypes = [C.c_int]
        L.flux_status_string.restype = C.c_char_p
        for name in ("flux_gemm_rs", "flux_ag_gemm", "flux_gemm_ref_unfused", "flux_query_status",
                     "flux_tile_coord", "flux_tile_shape", "flux_tile_config_count",
                     "flux_tile_config_info", "flux_default_order", "flux_last_hip_error", "flux_version",
                     "flux_profile_next_gemm", "flux_init_buffers", "flux_split_plan", "flux_gemm_ref_chunked"):
            getattr(L, name).restype = C.c_int
        _lib = L
    return _lib


_DT = {"bf16": FLUX_BF16, "f32": FLUX_F32, torch.bfloat16: FLUX_BF16, torch.float32: FLUX_F32}


def problem(M, N, K, R, rank, partial_dtype="bf16", out_dtype="bf16", tile_config=0, split_k=0,
            flags=0, comm_tiles_per_chunk=0, copy_workgroups=0, spin_timeout_ticks=0, link_gbps=0,
            lda=0, ldb=0, ldc=0, b_is_nk=0) -> flux_problem_t:
    return flux_problem_t(M, N, K, R, rank, _DT[partial_dtype], _DT[out_dtype], tile_config, split_k,
                          flags, comm_tiles_per_chunk, copy_workgroups, link_gbps, 0, spin_timeout_ticks,
                          lda, ldb, ldc, b_is_nk, 0)


def _ptr(t) -> int:
    return 0 if t is None else t.data_ptr()


def _ptr_list(ts):
    arr = (C.c_void_p * len(ts))()
    for i, t in enumerate(ts):
        arr[i] = _ptr(t)
    return arr


def _i32_list(xs):
    if xs is None:
        return None
    return (C.c_int32 * len(xs))(*[int(x) for x in xs])


def _stream(s) -> int:
    if s is None:
        s = torch.cuda.current_stream()
    return s.cuda_stream


def _check(status: int, where: str):
    if status != FLUX_OK:
        raise FluxError(status, where)


def flux_workspace_bytes(op: int, p: flux_problem_t) -> int:
    return int(lib().flux_workspace_bytes(op, C.byref(p)))


def flux_init_buffers(op, p, workspace=None, signals=None, stream=None):
    ws_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    _check(lib().flux_init_buffers(op, C.byref(p), _ptr(workspace), ws_bytes, _ptr(signals), _stream(stream)),
           "flux_init_buffers")


def flux_gemm_rs(p, A, B, peer_partials, out_slices, workspace=None, stream=None):
    ws_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    _check(lib().flux_gemm_rs(C.byref(p), _ptr(A), _ptr(B),
                              None if peer_partials is None else _ptr_list(peer_partials), _ptr_list(out_slices),
                              _ptr(workspace), ws_bytes, _stream(stream)), "flux_gemm_rs")


FLUX_STATIC_SCRATCH_BYTES = 32 << 20


def flux_gemm_rs_static(p, A, B, peer_partials, out_slices, stream=None):
    _check(lib().flux_gemm_rs_static(C.byref(p), _ptr(A), _ptr(B),
                                     None if peer_partials is None else _ptr_list(peer_partials), _ptr_list(out_slices),
                                     _stream(stream)), "flux_gemm_rs_static")


def flux_rs_ready_count(p) -> int:
    return int(lib().flux_rs_ready_count(C.byref(p)))


def flux_ag_deferred_tiles(p) -> int:
    return int(lib().flux_ag_deferred_tiles(C.byref(p)))


def flux_rs_resident_grid(p) -> tuple[int, int]:
    """(resident workgroups or 0, start delay of every second group of eight in 100 MHz ticks)."""
    d = C.c_uint32(0)
    n = int(lib().flux_rs_resident_grid(C.byref(p), C.byref(d)))
    return n, int(d.value)


def flux_gemm_rs_notify(p, A, B, out_slices, tile_ready, workspace=None, stream=None):
    ws_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    _check(lib().flux_gemm_rs_notify(C.byref(p), _ptr(A), _ptr(B), _ptr_list(out_slices), _ptr(tile_ready),
                                     _ptr(workspace), ws_bytes, _stream(stream)), "flux_gemm_rs_notify")


def flux_rs_reduce_slice_ready(p, staged, out, tile_ready, producers, workspace, stream=None):
    ws_bytes = workspace.numel() * workspace.element_size()
    _check(lib().flux_rs_reduce_slice_ready(C.byref(p), _ptr_list(staged), _ptr(out), _ptr(tile_ready), producers,
                                            _ptr(workspace), ws_bytes, _stream(stream)), "flux_rs_reduce_slice_ready")


def flux_ag_gemm(p, A_chunks, A_agg, B, Cout, signals, arrival_order, workspace, compute_stream, copy_stream):
    ws_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    _check(lib().flux_ag_gemm(C.byref(p), _ptr_list(A_chunks), _ptr(A_agg), _ptr(B), _ptr(Cout), _ptr(signals),
                              _i32_list(arrival_order), _ptr(workspace), ws_bytes,
                              _stream(compute_stream), _stream(copy_stream)), "flux_ag_gemm")


def flux_gemm_ref_unfused(op, phases, p, A=None, A_chunks=None, A_agg=None, B=None, peer_partials=None,
                          out_slices=None, Cout=None, workspace=None, stream=None):
    ws_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    _check(lib().flux_gemm_ref_unfused(
        op, phases, C.byref(p), _ptr(A), None if A_chunks is None else _ptr_list(A_chunks), _ptr(A_agg), _ptr(B),
        None if peer_partials is None else _ptr_list(peer_partials),
        None if out_slices is None else _ptr_list(out_slices), _ptr(Cout), _ptr(workspace), ws_bytes,
        _stream(stream)), "flux_gemm_ref_unfused")


def flux_gemm_ref_chunked(op, p, A=None, A_chunks=None, A_agg=None, B=None, peer_partials=None, out_slices=None,
                          Cout=None, arrival_order=None, workspace=None, compute_stream=None, comm_stream=None):
    ws_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    _check(lib().flux_gemm_ref_chunked(
        op, C.byref(p), _ptr(A), None if A_chunks is None else _ptr_list(A_chunks), _ptr(A_agg), _ptr(B),
        None if peer_partials is None else _ptr_list(peer_partials),
        None if out_slices is None else _ptr_list(out_slices), _ptr(Cout), _i32_list(arrival_order),
        _ptr(workspace), ws_bytes, _stream(compute_stream), _stream(comm_stream)), "flux_gemm_ref_chunked")


def flux_rs_reduce_slice(p, staged, out, stream=None):
    _check(lib().flux_rs_reduce_slice(C.byref(p), _ptr_list(staged), _ptr(out), _stream(stream)), "flux_rs_reduce_slice")


def flux_autotune_workspace_bytes(op, p) -> int:
    return int(lib().flux_autotune_workspace_bytes(op, C.byref(p)))


def flux_autotune_signal_count(p) -> int:
    return int(lib().flux_autotune_signal_count(C.byref(p)))


def flux_autotune_rs(p, A, B, peer_partials, out_slices, workspace=None, stream=None, reps=0):
    """Returns (tuned problem, ms of the winner, ms of the library's own pick)."""
    ws_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    tuned, best, default = flux_problem_t(), C.c_float(), C.c_float()
    _check(lib().flux_autotune_rs(C.byref(p), _ptr(A), _ptr(B), _ptr_list(peer_partials), _ptr_list(out_slices),
                                  _ptr(workspace), ws_bytes, _stream(stream), reps, C.byref(tuned), C.byref(best),
                                  C.byref(default)), "flux_autotune_rs")
    return tuned, best.value, default.value


def flux_autotune_ag(p, A_chunks, A_agg, B, Cout, signals, arrival_order, workspace, compute_stream, copy_stream, reps=0):
    """Returns (tuned problem, ms of the winner, ms of the library's own pick)."""
    ws_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    tuned, best, default = flux_problem_t(), C.c_float(), C.c_float()
    _check(lib().flux_autotune_ag(C.byref(p), _ptr_list(A_chunks), _ptr(A_agg), _ptr(B), _ptr(Cout), _ptr(signals),
                                  signals.numel(), _i32_list(arrival_order), _ptr(workspace), ws_bytes,
                                  _stream(compute_stream), _stream(copy_stream), reps, C.byref(tuned), C.byref(best),
                                  C.byref(default)), "flux_autotune_ag")
    return tuned, best.value, default.value


def flux_chunked_workspace_bytes(op, p) -> int:
    return int(lib().flux_chunked_workspace_bytes(op, C.byref(p)))


def flux_query_status(workspace):
    code, detail = C.c_int32(0), C.c_int32(0)
    _check(lib().flux_query_status(_ptr(workspace), C.byref(code), C.byref(detail)), "flux_query_status")
    return code.value, detail.value


def flux_tile_coord(op, p, arrival_order, block):
    mt, nt = C.c_int32(0), C.c_int32(0)
    _check(lib().flux_tile_coord(op, C.byref(p), _i32_list(arrival_order), block, C.byref(mt), C.byref(nt)),
           "flux_tile_coord")
    return mt.value, nt.value


@dataclass
class TileShape:
    tile_m: int
    tile_n: int
    tile_k: int
    split_k: int
    n_xcd: int


def flux_tile_shape(op, p) -> TileShape:
    v = [C.c_int32(0) for _ in range(5)]
    _check(lib().flux_tile_shape(op, C.byref(p), *[C.byref(x) for x in v]), "flux_tile_shape")
    return TileShape(*[x.value for x in v])


def flux_split_plan(op, p):
    """(full_tiles, split_tiles, split_k) a call would use."""
    v = [C.c_int32(0) for _ in range(3)]
    _check(lib().flux_split_plan(op, C.byref(p), *[C.byref(x) for x in v]), "flux_split_plan")
    return tuple(x.value for x in v)


def flux_tile_config_count() -> int:
    return lib().flux_tile_config_count()


def flux_tile_config_info(cfg_id: int):
    v = [C.c_int32(0) for _ in range(3)]
    _check(lib().flux_tile_config_info(cfg_id, *[C.byref(x) for x in v]), "flux_tile_config_info")
    return tuple(x.value for x in v)


def flux_default_order(rank: int, R: int):
    arr = (C.c_int32 * max(1, R - 1))()
    _check(lib().flux_default_order(rank, R, arr), "flux_default_order")
    return [arr[i] for i in range(R - 1)]


def flux_version() -> int:
    return lib().flux_version()


def tile_config_for(tile_m: int, tile_n: int) -> int:
    """Id of the compiled tile configuration with the given tile height and width."""
    for i in range(1, flux_tile_config_count() + 1):
        bm, bn, _ = flux_tile_config_info(i)
        if (bm, bn) == (tile_m, tile_n):
            return i
    raise ValueError(f"no tile configuration {tile_m}x{tile_n}")


# ---- HIP events created directly on the runtime, for timing a kernel on the library's stream ----
_hip = None


def _hiprt():
    global _hip
    if _hip is None:
        _hip = C.CDLL("libamdhip64.so")
        _hip.hipEventCreate.argtypes = [C.POINTER(C.c_void_p)]
        _hip.hipEventDestroy.argtypes = [C.c_void_p]
        _hip.hipEventSynchronize.argtypes = [C.c_void_p]
        _hip.hipEventRecord.argtypes = [C.c_void_p, C.c_void_p]
        _hip.hipEventElapsedTime.argtypes = [C.POINTER(C.c_float), C.c_void_p, C.c_void_p]
    return _hip


class HipEvent:
    """A timing-enabled hipEvent_t (plain handle; torch is not involved)."""

    def __init__(self):
        self.handle = C.c_void_p()
        if _hiprt().hipEventCreate(C.byref(self.handle)) != 0:
            raise RuntimeError("hipEventCreate failed")

    def record(self, stream=None):
        if _hiprt().hipEventRecord(self.handle, _stream(stream)) != 0:
            raise RuntimeError("hipEventRecord failed")

    def synchronize(self):
        if _hiprt().hipEventSynchronize(self.handle) != 0:
            raise RuntimeError("hipEventSynchronize failed")

    def elapsed_ms(self, later: "HipEvent") -> float:
        ms = C.c_float(0)
        if _hiprt().hipEventElapsedTime(C.byref(ms), self.handle, later.handle) != 0:
            raise RuntimeError("hipEventElapsedTime failed")
        return ms.value

    def __del__(self):
        try:
            _hiprt().hipEventDestroy(self.handle)
        except Exception:
            pass


def flux_profile_next_gemm(start: HipEvent | None, stop: HipEvent | None):
    _check(lib().flux_profile_next_gemm(None if start is None else start.handle,
                                        None if stop is None else stop.handle), "flux_profile_next_gemm")


TRACE_RECORD_BYTES = 64


def flux_trace_next_call(records):
    """`records`: a device tensor of at least 64 bytes per workgroup of the next call's grid (an int64
    tensor [grid, 8] reads as: word 0 = block | m_tile << 32, word 1 = n_tile | k_part << 32,
    word 2 = die | hw_id << 32, word 3 = tile, words 4..7 = the four clocks), or None to cancel."""
    n = 0 if records is None else records.numel() * records.element_size()
    _check(lib().flux_trace_next_call(_ptr(records), n), "flux_trace_next_call")

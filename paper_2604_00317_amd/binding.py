"""ctypes binding of libnimble_plan.so: argument marshalling only.

The functions carry the names of the C ABI (include/nimble_plan.h, and
include/nimble_plan_debug.h for the test and benchmark helpers).  Device buffers are torch
tensors (torch is used for device memory and streams, nothing else); every step of a plan runs
in the library's HIP kernels.  If the library is missing this module raises -- there is no
fallback path.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libnimble_plan.so")

NIMBLE_OK, NIMBLE_ERR_INVALID, NIMBLE_ERR_ALLOC, NIMBLE_ERR_HIP, NIMBLE_ERR_RANGE = range(5)
NIMBLE_COST_SUM, NIMBLE_COST_MAX, NIMBLE_LAYOUT_BATCH = 0, 1, 2
NIMBLE_REGIME_AUTO, NIMBLE_REGIME_RESIDENT, NIMBLE_REGIME_STREAM, NIMBLE_REGIME_PERSISTENT = \
    range(4)

EXPORTS = [
    "nimble_topo_create", "nimble_topo_destroy", "nimble_plan_solve", "nimble_plan_solve_batch",
    "nimble_last_error", "nimble_topo_num_links", "nimble_topo_num_comm",
    "nimble_topo_num_paths", "nimble_topo_nnz", "nimble_topo_bytes_per_iter",
    "nimble_topo_set_regime", "nimble_topo_regime", "nimble_debug_run_phase",
    "nimble_host_build_reverse", "nimble_debug_set_spin_limit", "nimble_topo_phase_bytes",
    "nimble_alg1_solve_batch", "nimble_plan_quantize", "nimble_plan_solve_warm",
    "nimble_plan_solve_adaptive",
    "nimble_host_records_roundtrip", "nimble_host_layout_stats",
    "nimble_host_build_reverse_streaming", "nimble_topo_resident_in_registers",
    "nimble_topo_adaptive_folds",
    "nimble_debug_stream_read", "nimble_topo_reserve", "nimble_host_resident_kernel",
    "nimble_plan_solve_static", "nimble_static_scratch_bytes", "nimble_debug_barrier_probe",
    "nimble_topo_reserve_batch", "nimble_debug_fail_allocation",
    "nimble_debug_fail_host_allocation", "nimble_debug_live_allocations",
]

_lib = None


class NimbleError(RuntimeError):
    def __init__(self, status: int, message: str):
        super().__init__(f"nimble status {status}: {message}")
        self.status = status


def load_library(build_if_missing: bool = True) -> ctypes.CDLL:
    """Loads the in-tree library; builds it first only when no built library exists."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        if not build_if_missing:
            raise FileNotFoundError(LIB_PATH)
        from . import build as _build
        _build.build()
    # Device pointers and streams cross the boundary, so the library and torch must share one
    # HIP runtime.  torch brings its own copy: it is imported first, and the library's dependency
    # on the runtime then resolves to the copy already in the process (loaded the other way
    # round, torch finds a runtime it was not built for and reports no GPU).
    import torch  # noqa: F401
    lib = ctypes.CDLL(LIB_PATH)
    vp, i32, i64, u32, dbl = (ctypes.c_void_p, ctypes.c_int32, ctypes.c_int64, ctypes.c_uint32,
                              ctypes.c_double)
    lib.nimble_topo_create.restype = ctypes.c_int
    lib.nimble_topo_create.argtypes = [i32, vp, i32, vp, i32, vp, vp, u32, ctypes.POINTER(vp)]
    lib.nimble_topo_destroy.restype = None
    lib.nimble_topo_destroy.argtypes = [vp]
    lib.nimble_plan_solve.restype = ctypes.c_int
    lib.nimble_plan_solve.argtypes = [vp, vp, dbl, i32, vp, vp, vp]
    lib.nimble_plan_solve_static.restype = ctypes.c_int
    lib.nimble_plan_solve_static.argtypes = [vp, vp, dbl, i32, vp, vp, vp]
    lib.nimble_static_scratch_bytes.restype = i64
    lib.nimble_static_scratch_bytes.argtypes = []
    lib.nimble_topo_reserve_batch.restype = ctypes.c_int
    lib.nimble_topo_reserve_batch.argtypes = [vp, i32, i32]
    lib.nimble_topo_reserve.restype = ctypes.c_int
    lib.nimble_topo_reserve.argtypes = [vp, i32]
    lib.nimble_host_resident_kernel.restype = ctypes.c_int
    lib.nimble_host_resident_kernel.argtypes = [i32, i32, vp, i32, vp, vp, vp]
    lib.nimble_plan_solve_batch.restype = ctypes.c_int
    lib.nimble_plan_solve_batch.argtypes = [vp, i32, vp, dbl, i32, vp, vp, vp]
    lib.nimble_last_error.restype = ctypes.c_char_p
    lib.nimble_last_error.argtypes = []
    for name in ("nimble_topo_num_links", "nimble_topo_num_comm", "nimble_topo_num_paths",
                 "nimble_topo_regime", "nimble_topo_resident_in_registers",
                 "nimble_topo_adaptive_folds"):
        getattr(lib, name).restype = i32
        getattr(lib, name).argtypes = [vp]
    for name in ("nimble_topo_nnz", "nimble_topo_bytes_per_iter"):
        getattr(lib, name).restype = i64
        getattr(lib, name).argtypes = [vp]
    lib.nimble_topo_phase_bytes.restype = i64
    lib.nimble_topo_phase_bytes.argtypes = [vp, i32]
    lib.nimble_topo_set_regime.restype = ctypes.c_int
    lib.nimble_topo_set_regime.argtypes = [vp, i32]
    lib.nimble_debug_run_phase.restype = ctypes.c_int
    lib.nimble_debug_run_phase.argtypes = [vp, i32, i32, vp, vp]
    lib.nimble_debug_barrier_probe.restype = ctypes.c_int
    lib.nimble_debug_barrier_probe.argtypes = [i32, i32, i32, i32, u32, vp, i64, vp, vp]
    lib.nimble_debug_fail_allocation.restype = ctypes.c_int
    lib.nimble_debug_fail_allocation.argtypes = [i32]
    lib.nimble_debug_fail_host_allocation.restype = None
    lib.nimble_debug_fail_host_allocation.argtypes = []
    lib.nimble_debug_live_allocations.restype = i64
    lib.nimble_debug_live_allocations.argtypes = []
    lib.nimble_debug_stream_read.restype = ctypes.c_int
    lib.nimble_debug_stream_read.argtypes = [vp, i64, i32, vp, vp]
    lib.nimble_debug_set_spin_limit.restype = ctypes.c_int
    lib.nimble_debug_set_spin_limit.argtypes = [vp, u32]
    lib.nimble_host_records_roundtrip.restype = ctypes.c_int
    lib.nimble_host_records_roundtrip.argtypes = [i32, i32, vp, i32, vp, vp, vp, vp, vp]
    lib.nimble_alg1_solve_batch.restype = ctypes.c_int
    lib.nimble_alg1_solve_batch.argtypes = [vp, i32, vp, ctypes.c_double, ctypes.c_double, i32,
                                            vp, vp, vp, vp]
    lib.nimble_plan_solve_warm.restype = ctypes.c_int
    lib.nimble_plan_solve_warm.argtypes = [vp, vp, ctypes.c_double, i32, vp, vp, vp, vp]
    lib.nimble_plan_solve_adaptive.restype = ctypes.c_int
    lib.nimble_plan_solve_adaptive.argtypes = [vp, vp, ctypes.c_double, i32, i32, vp, vp, vp, vp,
                                               vp]
    lib.nimble_plan_quantize.restype = ctypes.c_int
    lib.nimble_plan_quantize.argtypes = [vp, vp, vp, i32, ctypes.c_int64, ctypes.c_double, vp, vp]
    lib.nimble_host_layout_stats.restype = ctypes.c_int
    lib.nimble_host_layout_stats.argtypes = [i32, i32, vp, i32, vp, vp, vp]
    for name in ("nimble_host_build_reverse", "nimble_host_build_reverse_streaming"):
        getattr(lib, name).restype = ctypes.c_int
        getattr(lib, name).argtypes = [i32, i32, vp, i32, vp, vp, vp, vp, vp]
    _lib = lib
    return lib


def nimble_last_error() -> str:
    return load_library().nimble_last_error().decode()


def _check(status: int) -> None:
    if status != NIMBLE_OK:
        raise NimbleError(status, nimble_last_error())


def _host(a, dtype) -> np.ndarray:
    return np.ascontiguousarray(a, dtype=dtype)


def _hp(a: Optional[np.ndarray]):
    return None if a is None else a.ctypes.data_as(ctypes.c_void_p)


def _dev_ptr(t, dtype_name: str, numel: int, what: str):
    import torch
    if not isinstance(t, torch.Tensor) or not t.is_cuda:
        raise TypeError(f"{what} must be a device tensor")
    if t.dtype != getattr(torch, dtype_name) or not t.is_contiguous() or t.numel() != numel:
        raise ValueError(f"{what} must be contiguous {dtype_name} with {numel} elements")
    return ctypes.c_void_p(t.data_ptr())


def _stream_ptr(stream):
    import torch
    if stream is None:
        stream = torch.cuda.current_stream()
    return ctypes.c_void_p(stream.cuda_stream)


class Topo:
    """Owner of a nimble_topo_t handle."""

    def __init__(self, handle: int):
        self.handle = ctypes.c_void_p(handle)

    @property
    def n_links(self) -> int:
        return load_library().nimble_topo_num_links(self.handle)

    @property
    def n_comm(self) -> int:
        return load_library().nimble_topo_num_comm(self.handle)

    @property
    def n_paths(self) -> int:
        return load_library().nimble_topo_num_paths(self.handle)

    @property
    def nnz(self) -> int:
        return load_library().nimble_topo_nnz(self.handle)

    @property
    def bytes_per_iter(self) -> int:
        return load_library().nimble_topo_bytes_per_iter(self.handle)

    def phase_bytes(self, phase: int) -> int:
        return load_library().nimble_topo_phase_bytes(self.handle, int(phase))

    @property
    def regime(self) -> int:
        return load_library().nimble_topo_regime(self.handle)

    @property
    def adaptive_folds(self) -> bool:
        return load_library().nimble_topo_adaptive_folds(self.handle) == 1

    @property
    def resident_in_registers(self) -> bool:
        return load_library().nimble_topo_resident_in_registers(self.handle) == 1

    def close(self) -> None:
        if self.handle is not None and self.handle.value:
            load_library().nimble_topo_destroy(self.handle)
            self.handle = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


def nimble_topo_create(n_links, cap, n_comm, comm_path_ptr, n_paths, path_link_ptr, path_links,
                       flags: int = NIMBLE_COST_SUM) -> Topo:
    lib = load_library()
    cap = _host(cap, np.float64)
    cp = _host(comm_path_ptr, np.int32)
    lp = _host(path_link_ptr, np.int32)
    pl = _host(path_links, np.int32)
    if cap.shape != (n_links,) or cp.shape != (n_comm + 1,) or lp.shape != (n_paths + 1,):
        raise ValueError("array lengths do not match n_links / n_comm / n_paths")
    if n_paths >= 0 and lp.size and pl.shape != (max(int(lp[-1]), 0),):
        raise ValueError("path_links length must equal path_link_ptr[n_paths]")
    out = ctypes.c_void_p()
    _check(lib.nimble_topo_create(n_links, _hp(cap), n_comm, _hp(cp), n_paths, _hp(lp), _hp(pl),
                                  flags, ctypes.byref(out)))
    return Topo(out.value)


def nimble_topo_destroy(topo: Topo) -> None:
    topo.close()


def nimble_topo_set_regime(topo: Topo, regime: int) -> None:
    _check(load_library().nimble_topo_set_regime(topo.handle, regime))


def nimble_topo_reserve(topo: Topo, iters: int) -> None:
    _check(load_library().nimble_topo_reserve(topo.handle, int(iters)))


def nimble_topo_reserve_batch(topo: Topo, plans: int, iters: int) -> None:
    _check(load_library().nimble_topo_reserve_batch(topo.handle, int(plans), int(iters)))


def nimble_plan_solve(topo: Topo, d_traffic, eps: float, iters: int, d_splits, d_lambda,
                      stream=None) -> None:
    """Enqueues one plan on `stream` (torch stream; None = current)."""
    _check(load_library().nimble_plan_solve(
        topo.handle, _dev_ptr(d_traffic, "float64", topo.n_comm, "d_traffic"), float(eps),
        int(iters), _dev_ptr(d_splits, "float64", topo.n_paths, "d_splits"),
        _dev_ptr(d_lambda, "float64", 1, "d_lambda"), _stream_ptr(stream)))


def nimble_plan_solve_static(topo: Topo, d_traffic, eps: float, iters: int, d_splits, d_lambda,
                             stream=None) -> None:
    """nimble_plan_solve with its choice log in the library's static device scratch."""
    _check(load_library().nimble_plan_solve_static(
        topo.handle, _dev_ptr(d_traffic, "float64", topo.n_comm, "d_traffic"), float(eps),
        int(iters), _dev_ptr(d_splits, "float64", topo.n_paths, "d_splits"),
        _dev_ptr(d_lambda, "float64", 1, "d_lambda"), _stream_ptr(stream)))


def nimble_static_scratch_bytes() -> int:
    return int(load_library().nimble_static_scratch_bytes())


def nimble_plan_solve_batch(topo: Topo, batch: int, d_traffic, eps: float, iters: int, d_splits,
                            d_lambda, stream=None) -> None:
    _check(load_library().nimble_plan_solve_batch(
        topo.handle, int(batch),
        _dev_ptr(d_traffic, "float64", batch * topo.n_comm, "d_traffic"), float(eps), int(iters),
        _dev_ptr(d_splits, "float64", batch * topo.n_paths, "d_splits"),
        _dev_ptr(d_lambda, "float64", batch, "d_lambda"), _stream_ptr(stream)))


def nimble_alg1_solve_batch(topo: Topo, batch: int, d_traffic, phi: float, chi: float,
                            max_sweeps: int, d_flows, d_lambda, d_sweeps, stream=None) -> None:
    _check(load_library().nimble_alg1_solve_batch(
        topo.handle, int(batch),
        _dev_ptr(d_traffic, "float64", batch * topo.n_comm, "d_traffic"), float(phi), float(chi),
        int(max_sweeps), _dev_ptr(d_flows, "float64", batch * topo.n_paths, "d_flows"),
        _dev_ptr(d_lambda, "float64", batch, "d_lambda"),
        _dev_ptr(d_sweeps, "int32", batch, "d_sweeps"), _stream_ptr(stream)))


def nimble_plan_solve_warm(topo: Topo, d_traffic, eps: float, iters: int, d_len, d_splits,
                           d_lambda, stream=None) -> None:
    _check(load_library().nimble_plan_solve_warm(
        topo.handle, _dev_ptr(d_traffic, "float64", topo.n_comm, "d_traffic"), float(eps),
        int(iters), _dev_ptr(d_len, "float64", topo.n_links, "d_len"),
        _dev_ptr(d_splits, "float64", topo.n_paths, "d_splits"),
        _dev_ptr(d_lambda, "float64", 1, "d_lambda"), _stream_ptr(stream)))


def nimble_plan_solve_adaptive(topo: Topo, d_traffic, eps: float, max_iters: int,
                               check_every: int, d_splits, d_lambda, stream=None):
    """Returns (iterations made, best lower bound); splits and lambda land in the tensors."""
    iters = ctypes.c_int32(0)
    lb = ctypes.c_double(0.0)
    _check(load_library().nimble_plan_solve_adaptive(
        topo.handle, _dev_ptr(d_traffic, "float64", topo.n_comm, "d_traffic"), float(eps),
        int(max_iters), int(check_every),
        _dev_ptr(d_splits, "float64", topo.n_paths, "d_splits"),
        _dev_ptr(d_lambda, "float64", 1, "d_lambda"), ctypes.byref(iters), ctypes.byref(lb),
        _stream_ptr(stream)))
    return int(iters.value), float(lb.value)


def nimble_plan_quantize(topo: Topo, d_traffic, d_splits, iters: int, chi: int,
                         small_threshold: float, d_flows, stream=None) -> None:
    _check(load_library().nimble_plan_quantize(
        topo.handle, _dev_ptr(d_traffic, "float64", topo.n_comm, "d_traffic"),
        _dev_ptr(d_splits, "float64", topo.n_paths, "d_splits"), int(iters), int(chi),
        float(small_threshold), _dev_ptr(d_flows, "float64", topo.n_paths, "d_flows"),
        _stream_ptr(stream)))


def nimble_debug_run_phase(topo: Topo, phase: int, reps: int, d_traffic, stream=None) -> None:
    _check(load_library().nimble_debug_run_phase(
        topo.handle, int(phase), int(reps),
        _dev_ptr(d_traffic, "float64", topo.n_comm, "d_traffic"), _stream_ptr(stream)))


def nimble_debug_stream_read(d_buf, nbytes: int, reps: int, d_sink, stream=None) -> None:
    """Enqueue `reps` plain streaming reads of the first `nbytes` of the device tensor d_buf."""
    if not (d_buf.is_cuda and d_sink.is_cuda and d_buf.is_contiguous()):
        raise ValueError("d_buf and d_sink must be contiguous device tensors")
    if nbytes > d_buf.numel() * d_buf.element_size() or d_sink.numel() * d_sink.element_size() < 16:
        raise ValueError("nbytes exceeds d_buf, or d_sink is smaller than 16 bytes")
    _check(load_library().nimble_debug_stream_read(
        ctypes.c_void_p(d_buf.data_ptr()), int(nbytes), int(reps),
        ctypes.c_void_p(d_sink.data_ptr()), _stream_ptr(stream)))


def nimble_debug_barrier_probe(kind: int, blocks_per_cu: int, threads: int, rounds: int,
                               spin_limit: int, d_work, d_out, stream=None) -> None:
    """Enqueue the grid-barrier probe (see include/nimble_plan_debug.h); d_work is a uint8 device
    tensor, d_out an int32 device tensor of 32 elements."""
    _check(load_library().nimble_debug_barrier_probe(
        int(kind), int(blocks_per_cu), int(threads), int(rounds), int(spin_limit),
        ctypes.c_void_p(d_work.data_ptr()), int(d_work.numel() * d_work.element_size()),
        _dev_ptr(d_out, "int32", 32, "d_out"), _stream_ptr(stream)))


def nimble_debug_set_spin_limit(topo: Topo, polls: int) -> None:
    _check(load_library().nimble_debug_set_spin_limit(topo.handle, int(polls)))


def nimble_host_build_reverse(n_links, n_comm, comm_path_ptr, n_paths, path_link_ptr,
                              path_links, streaming: bool = False):
    """Host-only: the reverse link -> (commodity, path) CSR as the library builds it; with
    streaming=True decoded from the layout the link-load kernel walks."""
    cp = _host(comm_path_ptr, np.int32)
    lp = _host(path_link_ptr, np.int32)
    pl = _host(path_links, np.int32)
    nnz = int(lp[-1]) if lp.size else 0
    rev_ptr = np.zeros(n_links + 1, dtype=np.int32)
    rev_comm = np.zeros(max(nnz, 1), dtype=np.int32)
    rev_path = np.zeros(max(nnz, 1), dtype=np.int32)
    fn = (load_library().nimble_host_build_reverse_streaming if streaming
          else load_library().nimble_host_build_reverse)
    st = fn(n_links, n_comm, _hp(cp), n_paths, _hp(lp), _hp(pl), _hp(rev_ptr), _hp(rev_comm),
            _hp(rev_path))
    if st != NIMBLE_OK:
        raise NimbleError(st, "invalid CSR")
    return rev_ptr, rev_comm[:nnz], rev_path[:nnz]


def nimble_host_records_roundtrip(n_links, n_comm, comm_path_ptr, n_paths, path_link_ptr,
                                path_links):
    """Host-only: (links read back through the records, record of every path, number of records)."""
    cp = _host(comm_path_ptr, np.int32)
    lp = _host(path_link_ptr, np.int32)
    pl = _host(path_links, np.int32)
    links_out = np.full(max(int(lp[-1]), 1), -1, dtype=np.int32)
    path_rec = np.full(max(n_paths, 1), -1, dtype=np.int32)
    n_recs = ctypes.c_int32(0)
    st = load_library().nimble_host_records_roundtrip(n_links, n_comm, _hp(cp), n_paths, _hp(lp),
                                                    _hp(pl), _hp(links_out), _hp(path_rec),
                                                    ctypes.byref(n_recs))
    if st != NIMBLE_OK:
        raise NimbleError(st, "record round trip failed")
    return links_out[:int(lp[-1])], path_rec[:n_paths], int(n_recs.value)


def nimble_host_resident_kernel(n_links, n_comm, comm_path_ptr, n_paths, path_link_ptr,
                                path_links) -> int:
    """Host-only: 0 = the resident regime does not fit, 1 = its LDS kernel, 2 = its register
    kernel (see include/nimble_plan_debug.h)."""
    cp = _host(comm_path_ptr, np.int32)
    lp = _host(path_link_ptr, np.int32)
    pl = _host(path_links, np.int32)
    out = ctypes.c_int32(-1)
    st = load_library().nimble_host_resident_kernel(n_links, n_comm, _hp(cp), n_paths, _hp(lp),
                                                    _hp(pl), ctypes.byref(out))
    if st != NIMBLE_OK:
        raise NimbleError(st, "invalid CSR")
    return int(out.value)


def nimble_host_layout_stats(n_links, n_comm, comm_path_ptr, n_paths, path_link_ptr, path_links):
    """Host-only: dict of the sizes of the device layout (see include/nimble_plan_debug.h)."""
    cp = _host(comm_path_ptr, np.int32)
    lp = _host(path_link_ptr, np.int32)
    pl = _host(path_links, np.int32)
    out = np.zeros(22, dtype=np.int64)
    st = load_library().nimble_host_layout_stats(n_links, n_comm, _hp(cp), n_paths, _hp(lp),
                                                 _hp(pl), _hp(out))
    if st != NIMBLE_OK:
        raise NimbleError(st, "invalid CSR")
    keys = ["pairs", "octets", "singles", "octets_sigma", "single_chunks", "slots", "records",
            "record_stride", "link_blocks", "octets_padded", "pieces", "tile_items",
            "pieces_uniform", "strip_items", "strip_rows", "records_lane_major", "records_dict",
            "record_bodies", "group_blocks", "group_block_max_slots", "group_block_max_tasks",
            "record_bodies_product"]
    return dict(zip(keys, (int(v) for v in out)))


def plan(topo: Topo, traffic, eps: float, iters: int, device: str = "cuda:0"):
    """Convenience wrapper: host demand vector in, (splits, lambda) as numpy out."""
    import torch
    d = torch.as_tensor(np.ascontiguousarray(traffic, dtype=np.float64)).to(device)
    nan = float("nan")     # outputs start poisoned so that stale memory can never pass a check
    try:
        nimble_topo_reserve(topo, iters)  # the choice log, sized outside the solve
    except NimbleError as err:            # too long a log: the solve keeps per-path counters
        if err.status not in (NIMBLE_ERR_RANGE, NIMBLE_ERR_ALLOC):
            raise
    if d.dim() == 1:
        splits = torch.full((topo.n_paths,), nan, dtype=torch.float64, device=device)
        lam = torch.full((1,), nan, dtype=torch.float64, device=device)
        nimble_plan_solve(topo, d, eps, iters, splits, lam)
        torch.cuda.synchronize()
        return splits.cpu().numpy(), float(lam.item())
    b = d.shape[0]
    try:                                  # room for up to 64 plans per launch when streamed
        nimble_topo_reserve_batch(topo, min(b, 64), iters)
    except NimbleError as err:
        if err.status not in (NIMBLE_ERR_RANGE, NIMBLE_ERR_ALLOC):
            raise
    splits = torch.full((b * topo.n_paths,), nan, dtype=torch.float64, device=device)
    lam = torch.full((b,), nan, dtype=torch.float64, device=device)
    nimble_plan_solve_batch(topo, b, d.reshape(-1), eps, iters, splits, lam)
    torch.cuda.synchronize()
    return splits.cpu().numpy().reshape(b, topo.n_paths), lam.cpu().numpy()


def plan_alg1(topo: Topo, traffic, phi: float, chi: float, max_sweeps: int = 1 << 20,
              device: str = "cuda:0"):
    """Convenience wrapper of nimble_alg1_solve_batch: host demands [batch][n_comm] (or one
    vector) in, (flows, lambda, sweeps) as numpy out."""
    import torch
    d = torch.as_tensor(np.ascontiguousarray(traffic, dtype=np.float64)).to(device)
    single = d.dim() == 1
    b = 1 if single else d.shape[0]
    flows = torch.full((b * topo.n_paths,), float("nan"), dtype=torch.float64, device=device)
    lam = torch.full((b,), float("nan"), dtype=torch.float64, device=device)
    sweeps = torch.full((b,), -1, dtype=torch.int32, device=device)
    nimble_alg1_solve_batch(topo, b, d.reshape(-1), phi, chi, max_sweeps, flows, lam, sweeps)
    torch.cuda.synchronize()
    f = flows.cpu().numpy().reshape(b, topo.n_paths)
    if single:
        return f[0], float(lam.item()), int(sweeps.item())
    return f, lam.cpu().numpy(), sweeps.cpu().numpy()

"""ctypes loader for the C oracle (oracle/nimble_oracle.c) plus a numpy congestion evaluator.

Test infrastructure only: see the header of nimble_oracle.c.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from typing import Optional

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "nimble_oracle.c")
_SRC_ALG1 = os.path.join(_HERE, "alg1_oracle.c")
_SRC_ADAPT = os.path.join(_HERE, "adaptive_oracle.c")
_LIB = os.path.join(_HERE, "libnimble_oracle.so")
_lib = None


def build(force: bool = True) -> str:
    """Compile the oracle with gcc.  -ffp-contract=off keeps every statement one IEEE op."""
    newest = max(os.path.getmtime(_SRC), os.path.getmtime(_SRC_ALG1),
                 os.path.getmtime(_SRC_ADAPT))
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < newest:
        cmd = ["gcc", "-O2", "-std=c11", "-ffp-contract=off", "-fopenmp", "-fPIC", "-shared",
               "-Wall", "-Wextra", "-o", _LIB, _SRC, _SRC_ALG1, _SRC_ADAPT, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        # NIMBLE_ORACLE_LIB: a library built elsewhere from a deliberately altered copy of the
        # sources (the mutation test checks that the pins notice the alteration)
        variant = os.environ.get("NIMBLE_ORACLE_LIB")
        if not variant:
            build(force=False)
        lib = ctypes.CDLL(variant or _LIB)
        lib.nimble_oracle_solve.restype = ctypes.c_int
        lib.nimble_oracle_solve.argtypes = [
            ctypes.c_int32, ctypes.c_void_p, ctypes.c_int32, ctypes.c_void_p, ctypes.c_int32,
            ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_double, ctypes.c_int32,
            ctypes.c_uint32, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p,
            ctypes.c_void_p]
        lib.nimble_oracle_solve_warm.restype = ctypes.c_int
        lib.nimble_oracle_solve_warm.argtypes = [
            ctypes.c_int32, ctypes.c_void_p, ctypes.c_int32, ctypes.c_void_p, ctypes.c_int32,
            ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_double, ctypes.c_int32,
            ctypes.c_uint32, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p,
            ctypes.c_void_p, ctypes.c_void_p]
        lib.nimble_oracle_solve_adaptive.restype = ctypes.c_int
        lib.nimble_oracle_solve_adaptive.argtypes = [
            ctypes.c_int32, ctypes.c_void_p, ctypes.c_int32, ctypes.c_void_p, ctypes.c_int32,
            ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_double, ctypes.c_int32,
            ctypes.c_int32, ctypes.c_uint32, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p,
            ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p]
        lib.nimble_oracle_chunked_sum.restype = ctypes.c_double
        lib.nimble_oracle_chunked_sum.argtypes = [ctypes.c_void_p, ctypes.c_int64]
        lib.nimble_oracle_alg1.restype = ctypes.c_int
        lib.nimble_oracle_alg1.argtypes = [
            ctypes.c_int32, ctypes.c_void_p, ctypes.c_int32, ctypes.c_void_p, ctypes.c_int32,
            ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_double, ctypes.c_double,
            ctypes.c_int32, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p]
        lib.nimble_oracle_max_threads.restype = ctypes.c_int
        lib.nimble_oracle_set_threads.argtypes = [ctypes.c_int]
        _lib = lib
    return _lib


def max_threads() -> int:
    return int(_load().nimble_oracle_max_threads())


def set_threads(n: int) -> None:
    _load().nimble_oracle_set_threads(int(n))


def _p(a: Optional[np.ndarray]):
    return None if a is None else a.ctypes.data_as(ctypes.c_void_p)


def solve(n_links, cap, n_comm, comm_path_ptr, n_paths, path_link_ptr, path_links, demand,
          eps, iters, flags=0, want_lb=False, len0=None):
    """Run the oracle.  Returns dict(splits, lam, count, sumload[, lb][, len]).  len0: link
    lengths to start from (warm start); the lengths after the last iteration come back as
    "len"."""
    cap = np.ascontiguousarray(cap, dtype=np.float64)
    cp = np.ascontiguousarray(comm_path_ptr, dtype=np.int32)
    lp = np.ascontiguousarray(path_link_ptr, dtype=np.int32)
    pl = np.ascontiguousarray(path_links, dtype=np.int32)
    d = np.ascontiguousarray(demand, dtype=np.float64)
    assert cap.shape == (n_links,) and cp.shape == (n_comm + 1,) and lp.shape == (n_paths + 1,)
    assert d.shape == (n_comm,) and pl.shape == (int(lp[-1]),)
    splits = np.empty(n_paths, dtype=np.float64)
    lam = np.zeros(1, dtype=np.float64)
    count = np.empty(n_paths, dtype=np.uint32)
    sumload = np.empty(n_links, dtype=np.float64)
    lb = np.empty(iters, dtype=np.float64) if want_lb else None
    len_io = None
    if len0 is not None:
        len_io = np.array(len0, dtype=np.float64)
        assert len_io.shape == (n_links,)
    rc = _load().nimble_oracle_solve_warm(n_links, _p(cap), n_comm, _p(cp), n_paths, _p(lp),
                                          _p(pl), _p(d), float(eps), int(iters), int(flags),
                                          _p(len_io), _p(splits), _p(lam), _p(count),
                                          _p(sumload), _p(lb))
    if rc != 0:
        raise ValueError(f"nimble_oracle_solve failed with code {rc}")
    out = dict(splits=splits, lam=float(lam[0]), count=count, sumload=sumload)
    if len_io is not None:
        out["len"] = len_io
    if want_lb:
        out["lb"] = lb
    return out


def congestion(n_links, cap, comm_path_ptr, path_link_ptr, path_links, demand, splits):
    """max_e (1/cap_e) * sum_{p through e} d_k(p) * x_p  -- the objective of Eq. (1)-(3) in
    capacity-normalized path form, evaluated for given split fractions."""
    cp = np.asarray(comm_path_ptr, dtype=np.int64)
    lp = np.asarray(path_link_ptr, dtype=np.int64)
    path_comm = np.repeat(np.arange(len(cp) - 1), np.diff(cp))
    flow = np.asarray(demand, dtype=np.float64)[path_comm] * np.asarray(splits, dtype=np.float64)
    inc_path = np.repeat(np.arange(len(lp) - 1), np.diff(lp))
    load = np.bincount(np.asarray(path_links, dtype=np.int64), weights=flow[inc_path],
                       minlength=n_links)
    util = load / np.asarray(cap, dtype=np.float64)
    return float(util.max()), util


def alg1(n_links, cap, n_comm, comm_path_ptr, n_paths, path_link_ptr, path_links, demand,
         phi, chi, max_sweeps=1 << 20):
    """Algorithm 1 (sequential sweep, fraction phi of the remainder in chunks of chi).
    Returns dict(flows [n_paths] bytes, lam, sweeps, load [n_links])."""
    cap = np.ascontiguousarray(cap, dtype=np.float64)
    cp = np.ascontiguousarray(comm_path_ptr, dtype=np.int32)
    lp = np.ascontiguousarray(path_link_ptr, dtype=np.int32)
    pl = np.ascontiguousarray(path_links, dtype=np.int32)
    d = np.ascontiguousarray(demand, dtype=np.float64)
    assert cap.shape == (n_links,) and cp.shape == (n_comm + 1,) and lp.shape == (n_paths + 1,)
    assert d.shape == (n_comm,) and pl.shape == (int(lp[-1]),)
    flows = np.empty(max(n_paths, 1), dtype=np.float64)
    lam = np.zeros(1, dtype=np.float64)
    sweeps = np.zeros(1, dtype=np.int32)
    load = np.empty(n_links, dtype=np.float64)
    rc = _load().nimble_oracle_alg1(n_links, _p(cap), n_comm, _p(cp), n_paths, _p(lp), _p(pl),
                                    _p(d), float(phi), float(chi), int(max_sweeps), _p(flows),
                                    _p(lam), _p(sweeps), _p(load))
    if rc != 0:
        raise ValueError(f"nimble_oracle_alg1 failed with code {rc}")
    return dict(flows=flows[:n_paths], lam=float(lam[0]), sweeps=int(sweeps[0]), load=load)


def solve_adaptive(n_links, cap, n_comm, comm_path_ptr, n_paths, path_link_ptr, path_links,
                   demand, eps, max_iters, check_every, flags=0):
    """Adaptive-step variant with early stop.  Returns dict(splits, lam, iters, lb, weight,
    sigma [iters])."""
    cap = np.ascontiguousarray(cap, dtype=np.float64)
    cp = np.ascontiguousarray(comm_path_ptr, dtype=np.int32)
    lp = np.ascontiguousarray(path_link_ptr, dtype=np.int32)
    pl = np.ascontiguousarray(path_links, dtype=np.int32)
    d = np.ascontiguousarray(demand, dtype=np.float64)
    assert cap.shape == (n_links,) and cp.shape == (n_comm + 1,) and lp.shape == (n_paths + 1,)
    assert d.shape == (n_comm,) and pl.shape == (int(lp[-1]),)
    splits = np.empty(n_paths, dtype=np.float64)
    lam = np.zeros(1, dtype=np.float64)
    iters = np.zeros(1, dtype=np.int32)
    lb = np.zeros(1, dtype=np.float64)
    weight = np.empty(n_paths, dtype=np.float64)
    sigma = np.zeros(max_iters, dtype=np.float64)
    rc = _load().nimble_oracle_solve_adaptive(
        n_links, _p(cap), n_comm, _p(cp), n_paths, _p(lp), _p(pl), _p(d), float(eps),
        int(max_iters), int(check_every), int(flags), _p(splits), _p(lam), _p(iters), _p(lb),
        _p(weight), _p(sigma))
    if rc != 0:
        raise ValueError(f"nimble_oracle_solve_adaptive failed with code {rc}")
    n = int(iters[0])
    return dict(splits=splits, lam=float(lam[0]), iters=n, lb=float(lb[0]), weight=weight,
                sigma=sigma[:n])


def chunked_sum(x) -> float:
    """The fixed-association sum the adaptive variant uses for its lower bound."""
    x = np.ascontiguousarray(x, dtype=np.float64)
    return float(_load().nimble_oracle_chunked_sum(_p(x), x.size))

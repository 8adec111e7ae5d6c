"""Python binding of the C ABI declared in include/kvsched.h.

Argument marshalling only: torch tensors supply device memory and the HIP
stream; every step of the evaluation runs in the library's kernels.  There is
no fallback: if the shared library is missing and cannot be built, importing
a function from here fails.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Optional, Sequence

import numpy as np
import torch

from . import build as _build

SPS, SIMS = 0, 1
MODE_GBA, MODE_GSA, MODE_GBAD = 0, 1, 2
FEASIBLE_EJOB, FEASIBLE_EINVAL, FEASIBLE_ERANGE = 0xFC, 0xFE, 0xFF
OK, EINVAL, EJOB_INFEASIBLE, ERANGE, EHIP, ELIMIT = 0, 1, 2, 3, 4, 5
MAX_JOBS, MAX_POINTS, MAX_LEVELS = 16384, 64, 64


class KvsError(RuntimeError):
    def __init__(self, code: int, text: str):
        super().__init__(f"kvsched status {code}: {text}")
        self.code = code


class _Jobs(C.Structure):
    _fields_ = [("n_instances", C.c_int32), ("n_jobs", C.c_int32),
                ("o", C.c_void_p), ("s", C.c_void_p), ("o_est", C.c_void_p),
                ("s_scalar", C.c_int32), ("M", C.c_int64)]


class _Point(C.Structure):
    _fields_ = [("tau0", C.c_int32), ("sched", C.c_int32), ("k", C.c_int32), ("mode", C.c_int32)]


_lib = None


def library_path() -> str:
    return _build.LIB


def lib():
    """The loaded shared library; built first when there is none or a source is newer than it
    (a library older than its sources would run something else than the code in the tree)."""
    global _lib
    if _lib is None:
        if _build.is_stale():
            _build.build()
        L = C.CDLL(_build.LIB)
        vp, i32 = C.c_void_p, C.c_int32
        L.kvs_gba_simulate.restype = i32
        L.kvs_gba_simulate.argtypes = [C.POINTER(_Jobs), C.POINTER(_Point), i32, vp, vp, vp, vp, vp]
        L.kvs_schedule_eval.restype = i32
        L.kvs_schedule_eval.argtypes = [C.POINTER(_Jobs), C.POINTER(i32), C.POINTER(i32),
                                        C.POINTER(i32), i32, vp, vp, vp, vp, vp, vp]
        L.kvs_ladder_simulate.restype = i32
        L.kvs_ladder_simulate.argtypes = [C.POINTER(_Jobs)] + [C.POINTER(i32)] * 5 + [i32, vp, vp, vp, vp, vp]
        L.kvs_paper_ladder.restype = i32
        L.kvs_paper_ladder.argtypes = [C.c_int64, C.c_int64, i32, i32, C.POINTER(i32), C.POINTER(i32)]
        L.kvs_paper_ladder_quadratic.restype = i32
        L.kvs_paper_ladder_quadratic.argtypes = [C.c_int64, C.c_int64, i32, i32, i32, i32, C.POINTER(i32), C.POINTER(i32)]
        L.kvs_validate.restype = i32
        L.kvs_validate.argtypes = [C.POINTER(_Jobs), vp]
        L.kvs_validate_static.restype = i32
        L.kvs_validate_static.argtypes = [C.POINTER(_Jobs), vp]
        L.kvs_flow_bounds.restype = i32
        L.kvs_flow_bounds.argtypes = [C.POINTER(_Jobs), C.POINTER(i32), i32, vp, vp, vp]
        L.kvs_opt_perm.restype = i32
        L.kvs_opt_perm.argtypes = [C.POINTER(_Jobs), vp, vp]
        L.kvs_strerror.restype = C.c_char_p
        L.kvs_strerror.argtypes = [i32]
        L.kvs_version.restype = i32
        _lib = L
    return _lib


def strerror(code: int) -> str:
    return lib().kvs_strerror(code).decode()


def _check(code: int) -> None:
    if code != OK:
        raise KvsError(code, strerror(code))


def _dev_i32(t: Optional[torch.Tensor], shape, name: str) -> Optional[int]:
    if t is None:
        return None
    if not (t.is_cuda and t.dtype == torch.int32 and t.is_contiguous() and tuple(t.shape) == tuple(shape)):
        raise ValueError(f"{name}: need a contiguous int32 device tensor of shape {tuple(shape)}")
    return t.data_ptr()


def _dev_out(out: dict, name: str, shape, dtype, device) -> int:
    t = out.get(name)
    if not (isinstance(t, torch.Tensor) and t.is_cuda and t.device == device and t.dtype == dtype
            and t.is_contiguous() and tuple(t.shape) == tuple(shape)):
        raise ValueError(f"out[{name!r}]: need a contiguous {dtype} tensor of shape {tuple(shape)} on {device}")
    return t.data_ptr()


def _jobs(o: torch.Tensor, s, M: int, o_est: Optional[torch.Tensor]) -> _Jobs:
    if o.dim() != 2:
        raise ValueError("o: need [n_instances][n_jobs]")
    shape = tuple(o.shape)
    s_t = s if isinstance(s, torch.Tensor) else None
    return _Jobs(shape[0], shape[1], _dev_i32(o, shape, "o"), _dev_i32(s_t, shape, "s"),
                 _dev_i32(o_est, shape, "o_est"), 0 if s_t is not None else int(s), int(M))


def _stream(stream) -> Optional[int]:
    st = torch.cuda.current_stream() if stream is None else stream
    return st.cuda_stream or None


def gba_simulate(o: torch.Tensor, s, M: int, points, o_est: Optional[torch.Tensor] = None,
                 out: Optional[dict] = None, stream=None) -> dict:
    """kvs_gba_simulate.  `points`: rows (tau0, sched, k, mode).  `s`: int or
    device tensor.  Returns device tensors peak, feasible, flow, job_steps of
    shape [n_pts][n_instances]; valid after the stream is synchronised."""
    pts = np.asarray(points, dtype=np.int32).reshape(-1, 4)
    P, I = len(pts), o.shape[0]
    if out is None:
        out = dict(peak=torch.empty((P, I), dtype=torch.int64, device=o.device),
                   feasible=torch.empty((P, I), dtype=torch.uint8, device=o.device),
                   flow=torch.empty((P, I), dtype=torch.int64, device=o.device),
                   job_steps=torch.empty((P, I), dtype=torch.int64, device=o.device))
    arr = (_Point * max(P, 1))(*[_Point(*map(int, r)) for r in pts])
    jobs = _jobs(o, s, M, o_est)
    _check(lib().kvs_gba_simulate(C.byref(jobs), arr, P, _dev_out(out, "peak", (P, I), torch.int64, o.device),
                                  _dev_out(out, "feasible", (P, I), torch.uint8, o.device),
                                  _dev_out(out, "flow", (P, I), torch.int64, o.device),
                                  _dev_out(out, "job_steps", (P, I), torch.int64, o.device), _stream(stream)))
    return out


def schedule_eval(o: torch.Tensor, s, M: int, tau: Sequence[int], k: Sequence[int],
                  sched: Sequence[int], stream=None) -> dict:
    """kvs_schedule_eval: one SPS / SimS invocation per point on every instance."""
    tau = np.ascontiguousarray(tau, dtype=np.int32)
    k = np.ascontiguousarray(k, dtype=np.int32)
    sched = np.ascontiguousarray(sched, dtype=np.int32)
    P, I = len(tau), o.shape[0]
    if not (len(k) == P and len(sched) == P):
        raise ValueError("tau, k, sched: need the same length")
    out = dict(peak=torch.empty((P, I), dtype=torch.int64, device=o.device),
               feasible=torch.empty((P, I), dtype=torch.uint8, device=o.device),
               flow=torch.empty((P, I), dtype=torch.int64, device=o.device),
               n_completed=torch.empty((P, I), dtype=torch.int32, device=o.device),
               job_steps=torch.empty((P, I), dtype=torch.int64, device=o.device))
    p32 = C.POINTER(C.c_int32)
    jobs = _jobs(o, s, M, None)
    _check(lib().kvs_schedule_eval(C.byref(jobs), tau.ctypes.data_as(p32), k.ctypes.data_as(p32),
                                   sched.ctypes.data_as(p32), P, out["peak"].data_ptr(),
                                   out["feasible"].data_ptr(), out["flow"].data_ptr(),
                                   out["n_completed"].data_ptr(), out["job_steps"].data_ptr(),
                                   _stream(stream)))
    return out


def paper_ladder(M: int, s: int, alpha_num: int, alpha_den: int = 1) -> np.ndarray:
    """kvs_paper_ladder: the slices floor(beta alpha^p) of Algorithms 1 and 2 (host only)."""
    lad = np.zeros(MAX_LEVELS, np.int32)
    n = C.c_int32(0)
    _check(lib().kvs_paper_ladder(int(M), int(s), int(alpha_num), int(alpha_den),
                                  lad.ctypes.data_as(C.POINTER(C.c_int32)), C.byref(n)))
    return lad[:n.value].copy()


def paper_ladder_quadratic(M: int, s: int, a: int, b: int, c: int, d: int) -> np.ndarray:
    """kvs_paper_ladder_quadratic: the slices for alpha = (a + b sqrt(c)) / d (host only)."""
    lad = np.zeros(MAX_LEVELS, np.int32)
    n = C.c_int32(0)
    _check(lib().kvs_paper_ladder_quadratic(int(M), int(s), int(a), int(b), int(c), int(d),
                                            lad.ctypes.data_as(C.POINTER(C.c_int32)), C.byref(n)))
    return lad[:n.value].copy()


def ladder_simulate(o: torch.Tensor, s, M: int, ladders, points, o_est: Optional[torch.Tensor] = None,
                    stream=None) -> dict:
    """kvs_ladder_simulate.  `ladders`: one 1-d sequence of slices per point;
    `points`: rows (sched, k, mode)."""
    pts = np.asarray(points, dtype=np.int32).reshape(-1, 3)
    P, I = len(pts), o.shape[0]
    if len(ladders) != P:
        raise ValueError("one ladder per point")
    lad = np.zeros((max(P, 1), MAX_LEVELS), np.int32)
    nlv = np.zeros(max(P, 1), np.int32)
    for q, l in enumerate(ladders):
        if len(l) > MAX_LEVELS:
            raise KvsError(ELIMIT, strerror(ELIMIT))
        lad[q, :len(l)] = l
        nlv[q] = len(l)
    sched, k, mode = (np.ascontiguousarray(pts[:, j]) for j in range(3))
    out = dict(peak=torch.empty((P, I), dtype=torch.int64, device=o.device),
               feasible=torch.empty((P, I), dtype=torch.uint8, device=o.device),
               flow=torch.empty((P, I), dtype=torch.int64, device=o.device),
               job_steps=torch.empty((P, I), dtype=torch.int64, device=o.device))
    p32 = C.POINTER(C.c_int32)
    jobs = _jobs(o, s, M, o_est)
    _check(lib().kvs_ladder_simulate(C.byref(jobs), lad.ctypes.data_as(p32), nlv.ctypes.data_as(p32),
                                     sched.ctypes.data_as(p32), k.ctypes.data_as(p32),
                                     mode.ctypes.data_as(p32), P, out["peak"].data_ptr(),
                                     out["feasible"].data_ptr(), out["flow"].data_ptr(),
                                     out["job_steps"].data_ptr(), _stream(stream)))
    return out


def flow_bounds(o: torch.Tensor, s, M: int, tau0: Sequence[int], area: bool = True,
                out: Optional[dict] = None, stream=None) -> dict:
    """kvs_flow_bounds.  Returns device tensors upper_gba [len(tau0)][n_instances] and (if
    `area`) area_lb_num [n_instances]; valid after the stream is synchronised."""
    P, I = len(tau0), o.shape[0]
    if out is None:
        out = dict(upper_gba=torch.empty((P, I), dtype=torch.int64, device=o.device))
        if area:
            out["area_lb_num"] = torch.empty((I,), dtype=torch.int64, device=o.device)
    arr = (C.c_int32 * max(P, 1))(*map(int, tau0))
    jobs = _jobs(o, s, M, None)
    a = out.get("area_lb_num")
    _check(lib().kvs_flow_bounds(C.byref(jobs), arr, P, _dev_out(out, "upper_gba", (P, I), torch.int64, o.device),
                                 _dev_out(out, "area_lb_num", (I,), torch.int64, o.device) if a is not None else None,
                                 _stream(stream)))
    return out


def opt_perm(o: torch.Tensor, s: int, M: int, out: Optional[torch.Tensor] = None,
             stream=None) -> torch.Tensor:
    """kvs_opt_perm.  Returns the device tensor best_flow [n_instances]."""
    if out is None:
        out = torch.empty((o.shape[0],), dtype=torch.int64, device=o.device)
    jobs = _jobs(o, int(s), M, None)
    _check(lib().kvs_opt_perm(C.byref(jobs), _dev_out({"best_flow": out}, "best_flow", (o.shape[0],), torch.int64,
                                                      o.device), _stream(stream)))
    return out


def validate(o: torch.Tensor, s, M: int, o_est: Optional[torch.Tensor] = None, stream=None) -> int:
    """kvs_validate: returns the status code (OK, EINVAL, ERANGE, EJOB_INFEASIBLE)."""
    jobs = _jobs(o, s, M, o_est)
    return int(lib().kvs_validate(C.byref(jobs), _stream(stream)))


def validate_static(o: torch.Tensor, s, M: int, o_est: Optional[torch.Tensor] = None, stream=None) -> int:
    """kvs_validate_static: kvs_validate without any device allocation."""
    jobs = _jobs(o, s, M, o_est)
    return int(lib().kvs_validate_static(C.byref(jobs), _stream(stream)))


def version() -> int:
    return int(lib().kvs_version())

"""CPU oracle for KV-cache schedule evaluation -- TEST INFRASTRUCTURE ONLY.

Thin ctypes access to ``kvs_oracle.c`` (plain C, single-threaded, literal
round-by-round stepping of the model of Section 2.1 of "Competitive
Non-Clairvoyant KV-Cache Scheduling for LLM Inference").  Only the tests, the
smoke check and the CPU-baseline leg of the benchmark may import this package;
the GPU library and its Python binding never do, and this package imports
nothing of theirs.

Two C files: ``kvs_oracle.c`` is the oracle proper (literal stepping, the
bounds, exhaustive search); ``kvs_events.c`` is a second, independently written
evaluator of the same schedules from start / end events, fast enough to cover
every instance of the largest workload, and trusted only where the tests show
it equal to the stepper.  Both are compiled with gcc into one library on first
use (and again when a source is newer than the library).
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRCS = [os.path.join(_HERE, "kvs_oracle.c"), os.path.join(_HERE, "kvs_events.c")]
_LIB = os.path.join(_HERE, "libkvs_oracle.so")

SPS, SIMS = 0, 1
MODE_GBA, MODE_GSA = 0, 1
OK, EINVAL, EJOB_INFEASIBLE, ENOMEM = 0, 1, 2, 3


class OracleError(RuntimeError):
    def __init__(self, code: int):
        super().__init__(f"oracle status {code}")
        self.code = code


def build(force: bool = False) -> str:
    """Compile the C oracle into a shared library next to its source."""
    stale = (not os.path.exists(_LIB)) or any(os.path.getmtime(_LIB) < os.path.getmtime(p) for p in _SRCS)
    if force or stale:
        tmp = _LIB + f".tmp{os.getpid()}"
        subprocess.check_call(
            ["gcc", "-O2", "-std=c11", "-Wall", "-Wextra", "-shared", "-fPIC", "-o", tmp, *_SRCS]
        )
        os.replace(tmp, _LIB)
    return _LIB


_lib = None


def lib():
    global _lib
    if _lib is None:
        _lib = C.CDLL(build())
        i64, i32 = C.c_int64, C.c_int32
        p32, p64, pu8 = C.POINTER(C.c_int32), C.POINTER(C.c_int64), C.POINTER(C.c_uint8)
        _lib.kvo_peak_formula.restype = i64
        _lib.kvo_peak_formula.argtypes = [i64, i64, i64]
        _lib.kvo_kstar.restype = i64
        _lib.kvo_kstar.argtypes = [i64, i64, i64]
        _lib.kvo_area.restype = i64
        _lib.kvo_area.argtypes = [i64, i64]
        _lib.kvo_step_runs.restype = C.c_int
        _lib.kvo_step_runs.argtypes = [i64, p64, p64, p64, p64, p64]
        _lib.kvo_schedule_eval.restype = C.c_int
        _lib.kvo_schedule_eval.argtypes = [i64, p32, p32, i64, i64, i64, i64, C.c_int,
                                           p64, p32, p64, p64, p64]
        _lib.kvo_gba_simulate.restype = C.c_int
        _lib.kvo_gba_simulate.argtypes = [i64, p32, p32, p32, i64, i64, i64, C.c_int, i64,
                                          C.c_int, p64, p32, p64, p64, p64]
        _lib.kvo_gba_simulate_batch.restype = C.c_int
        _lib.kvo_gba_simulate_batch.argtypes = [i64, i64, i64, p32, p32, p32, i64, i64, i64,
                                                p32, p32, p32, p32, p64, pu8, p64, p64]
        _lib.kvo_ladder_simulate.restype = C.c_int
        _lib.kvo_ladder_simulate.argtypes = [i64, p32, p32, p32, i64, i64, p32, i64, C.c_int, i64,
                                             C.c_int, p64, p32, p64, p64, p64]
        _lib.kvo_ladder_simulate_batch.restype = C.c_int
        _lib.kvo_ladder_simulate_batch.argtypes = [i64, i64, i64, p32, p32, p32, i64, i64, i64,
                                                   p32, i64, p32, p32, p32, p32, p64, pu8, p64, p64]
        _lib.kvo_paper_ladder.restype = i64
        _lib.kvo_paper_ladder.argtypes = [i64, i64, i64, i64, p32, i64]
        _lib.kvo_schedule_eval_batch.restype = C.c_int
        _lib.kvo_schedule_eval_batch.argtypes = [i64, i64, i64, p32, p32, i64, i64, i64,
                                                 p32, p32, p32, p64, pu8, p64, p32, p64]
        _lib.kvo_opt_perm.restype = C.c_int
        _lib.kvo_opt_perm.argtypes = [i64, p32, i64, i64, p64]
        _lib.kvo_opt_exact.restype = C.c_int
        _lib.kvo_opt_exact.argtypes = [i64, p32, i64, i64, p64]
        _lib.kvo_area_lb.restype = C.c_int
        _lib.kvo_area_lb.argtypes = [i64, p32, p32, i64, p64]
        _lib.kvo_upper_gba.restype = C.c_int
        _lib.kvo_upper_gba.argtypes = [i64, p32, p32, i64, i64, i64, p64]
        _lib.kvo_gbad_simulate.restype = C.c_int
        _lib.kvo_gbad_simulate.argtypes = [i64, p32, p32, i64, i64, i64, C.c_int, i64, p64, p32, p64, p64, p64, p64]
        _lib.kvo_gbad_simulate_batch.restype = C.c_int
        _lib.kvo_gbad_simulate_batch.argtypes = [i64, i64, i64, p32, p32, i64, i64, i64, p32, p32, p32,
                                                 p64, pu8, p64, p64]
        _lib.kve_gba_simulate_batch.restype = C.c_int
        _lib.kve_gba_simulate_batch.argtypes = _lib.kvo_gba_simulate_batch.argtypes
        _lib.kve_ladder_simulate.restype = C.c_int
        _lib.kve_ladder_simulate.argtypes = [i64, p32, p32, p32, i64, i64, p32, i64, C.c_int, i64,
                                             C.c_int, p64, p32, p64, p64]
    return _lib


def _p32(a):
    return None if a is None else a.ctypes.data_as(C.POINTER(C.c_int32))


def _p64(a):
    return a.ctypes.data_as(C.POINTER(C.c_int64))


def _i32(a):
    return None if a is None else np.ascontiguousarray(a, dtype=np.int32)


def _check(rc):
    if rc != OK:
        raise OracleError(rc)


def peak_formula(k: int, tau: int, s: int) -> int:
    return int(lib().kvo_peak_formula(k, tau, s))


def kstar(tau: int, s: int, M: int) -> int:
    return int(lib().kvo_kstar(tau, s, M))


def area(o: int, s: int) -> int:
    return int(lib().kvo_area(o, s))


def step_runs(start, dur, s):
    """Occupancy peak and job-steps of explicit runs (sorted by start)."""
    start = np.ascontiguousarray(start, dtype=np.int64)
    dur = np.ascontiguousarray(dur, dtype=np.int64)
    s = np.ascontiguousarray(s, dtype=np.int64)
    peak, steps = C.c_int64(), C.c_int64()
    _check(lib().kvo_step_runs(len(start), _p64(start), _p64(dur), _p64(s),
                               C.byref(peak), C.byref(steps)))
    return peak.value, steps.value


def schedule_eval(o, s, M, tau, k=0, sched=SPS):
    """One SPS / SimS invocation on the whole sequence.  `s`: int or array."""
    o = _i32(o)
    s_arr = None if np.isscalar(s) else _i32(s)
    s_scalar = int(s) if np.isscalar(s) else 0
    peak, flow, nc, steps = C.c_int64(), C.c_int64(), C.c_int64(), C.c_int64()
    feas = C.c_int32()
    _check(lib().kvo_schedule_eval(len(o), _p32(o), _p32(s_arr), s_scalar, M, tau, k, sched,
                                   C.byref(peak), C.byref(feas), C.byref(flow), C.byref(nc),
                                   C.byref(steps)))
    return dict(peak=peak.value, feasible=feas.value, flow=flow.value,
                n_completed=nc.value, job_steps=steps.value)


def gba_simulate(o, s, M, tau0=1, sched=SPS, k=0, mode=MODE_GBA, o_est=None):
    """One instance at one sweep point.  `s`: int or array."""
    o = _i32(o)
    s_arr = None if np.isscalar(s) else _i32(s)
    s_scalar = int(s) if np.isscalar(s) else 0
    e = _i32(o_est)
    peak, flow, steps, phases = C.c_int64(), C.c_int64(), C.c_int64(), C.c_int64()
    feas = C.c_int32()
    _check(lib().kvo_gba_simulate(len(o), _p32(o), _p32(s_arr), _p32(e), s_scalar, M, tau0,
                                  sched, k, mode, C.byref(peak), C.byref(feas), C.byref(flow),
                                  C.byref(steps), C.byref(phases)))
    return dict(peak=peak.value, feasible=feas.value, flow=flow.value,
                job_steps=steps.value, n_phases=phases.value)


def paper_ladder(M: int, s: int, num: int, den: int = 1, max_levels: int = 128):
    """Slices floor(beta alpha^p), p = 0..l, of Algorithms 1 and 2 for alpha = num/den."""
    lad = np.zeros(max_levels, np.int32)
    L = lib().kvo_paper_ladder(M, s, num, den, _p32(lad), max_levels)
    if L < 0:
        raise OracleError(EINVAL)
    return lad[:L].copy()


def paper_ladder_quadratic(M: int, s: int, a: int, b: int, c: int, d: int):
    """Slices floor(beta alpha^p), p = 0..l, of Algorithms 1 and 2 for the scaling factor
    alpha = (a + b sqrt(c)) / d > 1 with integers a, b, c >= 0, d >= 1, in exact integer arithmetic.

    alpha^q = (A + B sqrt(c)) / d^q with integers A, B >= 0, so for integers X, y >= 0
        y alpha^q <= X  <=>  y B sqrt(c) <= X d^q - y A  <=>  X d^q - y A >= 0 and (y B)^2 c <= (X d^q - y A)^2.
    l is the largest q with alpha^q <= M - s, and tau_p is the largest y with y alpha^(l-p) <= M - s,
    found by bisection over y (Python integers do not overflow)."""
    X = M - s
    if X < 1 or s < 0 or min(a, b, c) < 0 or d < 1:
        raise OracleError(EINVAL)

    def times_alpha(A, B):          # (A + B sqrt c)(a + b sqrt c) = (A a + B b c) + (A b + B a) sqrt c
        return A * a + B * b * c, A * b + B * a

    def le(y, A, B, q):             # y * alpha^q <= X ?
        rhs = X * d ** q - y * A
        return rhs >= 0 and (y * B) ** 2 * c <= rhs * rhs

    # alpha > 1  <=>  a + b sqrt(c) > d
    if not (a > d or (b > 0 and (d - a) ** 2 < b * b * c)):
        raise OracleError(EINVAL)
    powers = [(1, 0)]               # alpha^q as (A, B), over d^q
    while True:
        A, B = times_alpha(*powers[-1])
        if not le(1, A, B, len(powers)):
            break
        powers.append((A, B))
    l = len(powers) - 1
    lad = []
    for p in range(l + 1):
        q = l - p
        A, B = powers[q]
        lo, hi = 0, X               # largest y in [0, X] with y alpha^q <= X
        while lo < hi:
            mid = (lo + hi + 1) // 2
            if le(mid, A, B, q):
                lo = mid
            else:
                hi = mid - 1
        lad.append(lo)
    return np.asarray(lad, np.int32)


def ladder_simulate(o, s, M, ladder, sched=SPS, k=0, mode=MODE_GBA, o_est=None):
    """One instance on an explicit ladder of slices.  `s`: int or array."""
    o = _i32(o)
    s_arr = None if np.isscalar(s) else _i32(s)
    s_scalar = int(s) if np.isscalar(s) else 0
    e = _i32(o_est)
    lad = _i32(ladder)
    peak, flow, steps, phases = C.c_int64(), C.c_int64(), C.c_int64(), C.c_int64()
    feas = C.c_int32()
    _check(lib().kvo_ladder_simulate(len(o), _p32(o), _p32(s_arr), _p32(e), s_scalar, M,
                                     _p32(lad), len(lad), sched, k, mode, C.byref(peak),
                                     C.byref(feas), C.byref(flow), C.byref(steps),
                                     C.byref(phases)))
    return dict(peak=peak.value, feasible=feas.value, flow=flow.value,
                job_steps=steps.value, n_phases=phases.value)


def ladder_simulate_batch(o, s, M, ladders, points, o_est=None, i0=0, i1=None):
    """Instances [i0, i1) at every point q = (sched, k, mode) on the slices ladders[q]
    (a list of 1-d arrays).  Returns dict of arrays shaped [n_pts][i1 - i0]."""
    o = _i32(o)
    I, n = o.shape
    i1 = I if i1 is None else i1
    s_arr = None if np.isscalar(s) else _i32(s)
    s_scalar = int(s) if np.isscalar(s) else 0
    e = _i32(o_est)
    pts = np.asarray(points, dtype=np.int32).reshape(-1, 3)
    sched, k, mode = (np.ascontiguousarray(pts[:, j]) for j in range(3))
    P, cnt = len(pts), i1 - i0
    stride = max(len(l) for l in ladders)
    lad = np.zeros((P, stride), np.int32)
    nlv = np.zeros(P, np.int32)
    for q, l in enumerate(ladders):
        lad[q, :len(l)] = l
        nlv[q] = len(l)
    peak = np.zeros((P, cnt), np.int64)
    flow = np.zeros((P, cnt), np.int64)
    steps = np.zeros((P, cnt), np.int64)
    feas = np.zeros((P, cnt), np.uint8)
    _check(lib().kvo_ladder_simulate_batch(i0, i1, n, _p32(o), _p32(s_arr), _p32(e), s_scalar,
                                           M, P, _p32(lad), stride, _p32(nlv), _p32(sched),
                                           _p32(k), _p32(mode), _p64(peak),
                                           feas.ctypes.data_as(C.POINTER(C.c_uint8)), _p64(flow),
                                           _p64(steps)))
    return dict(peak=peak, feasible=feas, flow=flow, job_steps=steps)


def gba_simulate_batch(o, s, M, points, o_est=None, i0=0, i1=None, threads=1, evaluator="stepper"):
    """Instances [i0, i1) of [I][n] arrays at every point (tau0, sched, k, mode).

    `threads` > 1 runs disjoint instance ranges on that many threads (instances are independent; each
    call into C is single-threaded and releases the interpreter lock).  `evaluator`: "stepper" is the
    oracle proper (round by round), "events" the second evaluator of kvs_events.c.

    Returns dict of arrays shaped [n_pts][i1 - i0]."""
    o = _i32(o)
    I, n = o.shape
    i1 = I if i1 is None else i1
    s_arr = None if np.isscalar(s) else _i32(s)
    s_scalar = int(s) if np.isscalar(s) else 0
    e = _i32(o_est)
    pts = np.asarray(points, dtype=np.int32).reshape(-1, 4)
    tau0, sched, k, mode = (np.ascontiguousarray(pts[:, j]) for j in range(4))
    P, cnt = len(pts), i1 - i0
    fn = {"stepper": lib().kvo_gba_simulate_batch, "events": lib().kve_gba_simulate_batch}[evaluator]
    pu8 = C.POINTER(C.c_uint8)

    def run(a, b):
        part = dict(peak=np.zeros((P, b - a), np.int64), feasible=np.zeros((P, b - a), np.uint8),
                    flow=np.zeros((P, b - a), np.int64), job_steps=np.zeros((P, b - a), np.int64))
        rc = fn(a, b, n, _p32(o), _p32(s_arr), _p32(e), s_scalar, M, P, _p32(tau0), _p32(sched), _p32(k),
                _p32(mode), _p64(part["peak"]), part["feasible"].ctypes.data_as(pu8), _p64(part["flow"]),
                _p64(part["job_steps"]))
        return rc, part

    threads = max(1, min(int(threads), cnt))
    if threads == 1:
        rc, out = run(i0, i1)
        _check(rc)
        return out
    from concurrent.futures import ThreadPoolExecutor
    cuts = np.linspace(i0, i1, 4 * threads + 1).astype(np.int64)   # a few ranges per thread evens out the load
    spans = [(int(a), int(b)) for a, b in zip(cuts[:-1], cuts[1:]) if b > a]
    with ThreadPoolExecutor(threads) as ex:
        parts = list(ex.map(lambda ab: run(*ab), spans))
    for rc, _ in parts:
        _check(rc)
    return {key: np.concatenate([part[key] for _, part in parts], axis=1)
            for key in ("peak", "feasible", "flow", "job_steps")}


def events_ladder_simulate(o, s, M, ladder, sched=SPS, k=0, mode=MODE_GBA, o_est=None):
    """The second evaluator (kvs_events.c) on one instance and an explicit ladder of slices."""
    o = _i32(o)
    s_arr = None if np.isscalar(s) else _i32(s)
    s_scalar = int(s) if np.isscalar(s) else 0
    e = _i32(o_est)
    lad = _i32(ladder)
    peak, flow, steps = C.c_int64(), C.c_int64(), C.c_int64()
    feas = C.c_int32()
    _check(lib().kve_ladder_simulate(len(o), _p32(o), _p32(s_arr), _p32(e), s_scalar, M, _p32(lad),
                                     len(lad), sched, k, mode, C.byref(peak), C.byref(feas),
                                     C.byref(flow), C.byref(steps)))
    return dict(peak=peak.value, feasible=feas.value, flow=flow.value, job_steps=steps.value)


def schedule_eval_batch(o, s, M, points, i0=0, i1=None):
    """Instances [i0, i1) at every point (tau, k, sched)."""
    o = _i32(o)
    I, n = o.shape
    i1 = I if i1 is None else i1
    s_arr = None if np.isscalar(s) else _i32(s)
    s_scalar = int(s) if np.isscalar(s) else 0
    pts = np.asarray(points, dtype=np.int32).reshape(-1, 3)
    tau, k, sched = (np.ascontiguousarray(pts[:, j]) for j in range(3))
    P, cnt = len(pts), i1 - i0
    peak = np.zeros((P, cnt), np.int64)
    flow = np.zeros((P, cnt), np.int64)
    steps = np.zeros((P, cnt), np.int64)
    nc = np.zeros((P, cnt), np.int32)
    feas = np.zeros((P, cnt), np.uint8)
    _check(lib().kvo_schedule_eval_batch(i0, i1, n, _p32(o), _p32(s_arr), s_scalar, M, P,
                                         _p32(tau), _p32(k), _p32(sched), _p64(peak),
                                         feas.ctypes.data_as(C.POINTER(C.c_uint8)), _p64(flow),
                                         _p32(nc), _p64(steps)))
    return dict(peak=peak, feasible=feas, flow=flow, n_completed=nc, job_steps=steps)


def gbad_simulate(o, s, M, tau0=1, sched=SPS, k=0, starts=False):
    """Algorithm 2 with dynamic refill (GBA-D) on one instance.  `starts`: also return the start
    round of every job in the refilled and in the baseline schedule."""
    o = _i32(o)
    s_arr = None if np.isscalar(s) else _i32(s)
    s_scalar = int(s) if np.isscalar(s) else 0
    peak, flow, steps = C.c_int64(), C.c_int64(), C.c_int64()
    feas = C.c_int32()
    st = np.zeros(len(o), np.int64)
    bs = np.zeros(len(o), np.int64)
    _check(lib().kvo_gbad_simulate(len(o), _p32(o), _p32(s_arr), s_scalar, M, tau0, sched, k,
                                   C.byref(peak), C.byref(feas), C.byref(flow), C.byref(steps),
                                   _p64(st), _p64(bs)))
    r = dict(peak=peak.value, feasible=feas.value, flow=flow.value, job_steps=steps.value)
    if starts:
        r["start"], r["base_start"] = st, bs
    return r


def gbad_simulate_batch(o, s, M, points, i0=0, i1=None, threads=1):
    """GBA-D on instances [i0, i1) at every point (tau0, sched, k); arrays [n_pts][i1 - i0]."""
    o = _i32(o)
    I, n = o.shape
    i1 = I if i1 is None else i1
    s_arr = None if np.isscalar(s) else _i32(s)
    s_scalar = int(s) if np.isscalar(s) else 0
    pts = np.asarray(points, dtype=np.int32).reshape(-1, 3)
    tau0, sched, k = (np.ascontiguousarray(pts[:, j]) for j in range(3))
    P = len(pts)
    pu8 = C.POINTER(C.c_uint8)

    def run(a, b):
        part = dict(peak=np.zeros((P, b - a), np.int64), feasible=np.zeros((P, b - a), np.uint8),
                    flow=np.zeros((P, b - a), np.int64), job_steps=np.zeros((P, b - a), np.int64))
        rc = lib().kvo_gbad_simulate_batch(a, b, n, _p32(o), _p32(s_arr), s_scalar, M, P, _p32(tau0),
                                           _p32(sched), _p32(k), _p64(part["peak"]),
                                           part["feasible"].ctypes.data_as(pu8), _p64(part["flow"]),
                                           _p64(part["job_steps"]))
        return rc, part

    threads = max(1, min(int(threads), i1 - i0))
    if threads == 1:
        rc, out = run(i0, i1)
        _check(rc)
        return out
    from concurrent.futures import ThreadPoolExecutor
    cuts = np.linspace(i0, i1, 4 * threads + 1).astype(np.int64)
    spans = [(int(a), int(b)) for a, b in zip(cuts[:-1], cuts[1:]) if b > a]
    with ThreadPoolExecutor(threads) as ex:
        parts = list(ex.map(lambda ab: run(*ab), spans))
    for rc, _ in parts:
        _check(rc)
    return {key: np.concatenate([part[key] for _, part in parts], axis=1)
            for key in ("peak", "feasible", "flow", "job_steps")}


def opt_perm(o, s: int, M: int) -> int:
    o = _i32(o)
    best = C.c_int64()
    _check(lib().kvo_opt_perm(len(o), _p32(o), s, M, C.byref(best)))
    return best.value


def opt_exact(o, s: int, M: int) -> int:
    o = _i32(o)
    best = C.c_int64()
    _check(lib().kvo_opt_exact(len(o), _p32(o), s, M, C.byref(best)))
    return best.value


def area_lb(o, s) -> int:
    """Numerator of the area lower bound on OPT: sum_j (n - j + 1) * Area_j, areas ascending
    (proof of the area-based lower bound for OPT).  OPT >= area_lb / M."""
    o = _i32(o)
    s_arr = None if np.isscalar(s) else _i32(s)
    num = C.c_int64()
    _check(lib().kvo_area_lb(len(o), _p32(o), _p32(s_arr), int(s) if np.isscalar(s) else 0,
                             C.byref(num)))
    return num.value


def upper_gba(o, s, M: int, tau0: int) -> int:
    """UpperGBA = sum_p (n_p * S_p + Q_p) on the ladder tau0 * 2^p (analysis of GBA, Step 3)."""
    o = _i32(o)
    s_arr = None if np.isscalar(s) else _i32(s)
    up = C.c_int64()
    _check(lib().kvo_upper_gba(len(o), _p32(o), _p32(s_arr), int(s) if np.isscalar(s) else 0,
                               M, tau0, C.byref(up)))
    return up.value

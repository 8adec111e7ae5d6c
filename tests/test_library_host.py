"""Host-side checks of the GPU library that need no GPU: it loads, exports
every symbol the header declares, rejects bad arguments before touching the
device, and its integer helpers agree with plain Python arithmetic."""
import ctypes as C
import os
import random
import re

import pytest

from paper_2601_22996_amd import build as B

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def L():
    if not os.path.exists(B.LIB):
        B.build()
    lib = C.CDLL(B.LIB)
    lib.kvs_host_class_index.restype = C.c_uint32
    lib.kvs_host_class_index.argtypes = [C.c_uint32, C.c_uint32]
    lib.kvs_host_div.restype = C.c_uint32
    lib.kvs_host_div.argtypes = [C.c_uint32, C.c_uint32]
    lib.kvs_host_kstar.restype = C.c_uint64
    lib.kvs_host_kstar.argtypes = [C.c_uint64, C.c_uint64, C.c_uint64]
    lib.kvs_strerror.restype = C.c_char_p
    return lib


def test_exports_every_declared_symbol(L):
    header = open(os.path.join(ROOT, "include", "kvsched.h")).read()
    names = set(re.findall(r"\b(kvs_[a-z_]+)\s*\(", header))
    assert {"kvs_gba_simulate", "kvs_schedule_eval", "kvs_validate", "kvs_strerror",
            "kvs_version"} <= names
    for name in names:
        assert hasattr(L, name), name
    assert L.kvs_version() >= 100
    assert L.kvs_strerror(0) == b"ok"


def test_argument_checks_return_before_any_device_work(L):
    class Jobs(C.Structure):
        _fields_ = [("n_instances", C.c_int32), ("n_jobs", C.c_int32), ("o", C.c_void_p),
                    ("s", C.c_void_p), ("o_est", C.c_void_p), ("s_scalar", C.c_int32),
                    ("M", C.c_int64)]

    class Point(C.Structure):
        _fields_ = [("tau0", C.c_int32), ("sched", C.c_int32), ("k", C.c_int32), ("mode", C.c_int32)]

    L.kvs_gba_simulate.restype = C.c_int32
    L.kvs_gba_simulate.argtypes = [C.POINTER(Jobs), C.POINTER(Point), C.c_int32] + [C.c_void_p] * 5
    pt = Point(1, 0, 0, 0)
    EINVAL, ELIMIT = 1, 5
    call = lambda j, p, n: L.kvs_gba_simulate(C.byref(j), C.byref(p), n, None, None, None, None, None)
    assert L.kvs_gba_simulate(None, C.byref(pt), 1, None, None, None, None, None) == EINVAL
    assert call(Jobs(4, 8, None, None, None, 0, 100), pt, 1) == EINVAL          # o is null
    assert call(Jobs(-1, 8, 1, None, None, 0, 100), pt, 1) == EINVAL
    assert call(Jobs(4, 0, 1, None, None, 0, 100), pt, 1) == EINVAL
    assert call(Jobs(4, 8, 1, None, None, 0, 0), pt, 1) == EINVAL               # M < 1
    assert call(Jobs(4, 8, 1, None, None, -1, 100), pt, 1) == EINVAL            # s_scalar < 0
    assert call(Jobs(4, 16385, 1, None, None, 0, 100), pt, 1) == ELIMIT
    assert call(Jobs(4, 8, 1, None, None, 0, 100), pt, 65) == ELIMIT
    assert call(Jobs(4, 8, 1, None, None, 0, 100), Point(0, 0, 0, 0), 1) == EINVAL   # tau0 < 1
    assert call(Jobs(4, 8, 1, None, None, 0, 100), Point(1, 2, 0, 0), 1) == EINVAL   # sched
    assert call(Jobs(4, 8, 1, None, None, 0, 100), Point(1, 0, -1, 0), 1) == EINVAL  # k < 0
    assert call(Jobs(4, 8, 1, None, None, 0, 100), Point(1, 0, 0, 7), 1) == EINVAL   # mode
    assert call(Jobs(4, 8, 1, None, None, 0, 100), pt, 1) == EINVAL             # null outputs
    assert call(Jobs(0, 8, None, None, None, 0, 100), pt, 1) == 0               # nothing to do
    assert call(Jobs(4, 8, 1, None, None, 0, 100), pt, 0) == 0


def test_class_index_matches_definition(L):
    def cls(x, t):
        p = 0
        while t * 2 ** p < x:
            p += 1
        return p
    for t in list(range(1, 40)) + [100, 1000, 2 ** 20, 2 ** 30 - 1, 2 ** 30]:
        for x in list(range(1, 200)) + [2 ** 30, 2 ** 30 - 1, 2 ** 29 + 1, 2 ** 20 + 3]:
            assert L.kvs_host_class_index(x, t) == cls(x, t), (x, t)


def test_constant_division_is_exact_below_2_31(L):
    rnd = random.Random(7)
    top = 2 ** 31 - 1
    for _ in range(100000):
        d = rnd.choice([rnd.randint(1, 70), rnd.randint(1, top), 2 ** rnd.randint(0, 30),
                        rnd.randint(1, 70000)])
        m = rnd.randint(0, top // d)
        for x in (rnd.randint(0, top), top, m * d, max(0, m * d - 1), min(top, m * d + d - 1)):
            assert L.kvs_host_div(x, d) == x // d, (x, d)


def test_kstar_matches_scan_of_the_peak_formula(L):
    import math

    def peak(k, tau, s):
        return s * k + (tau * k + tau + k - math.gcd(tau, k)) // 2

    rnd = random.Random(3)
    for _ in range(3000):
        tau, s, M = rnd.randint(1, 300), rnd.randint(0, 300), rnd.randint(1, 6000)
        k = 0
        while peak(k + 1, tau, s) <= M:
            k += 1
        assert L.kvs_host_kstar(tau, s, M) == k, (tau, s, M)
    assert L.kvs_host_kstar(1, 0, 2 ** 39) == 2 ** 39


def test_paper_ladder_matches_the_oracle_and_the_definition(L):
    import numpy as np
    import oracle as O
    L.kvs_paper_ladder.restype = C.c_int32
    L.kvs_paper_ladder.argtypes = [C.c_int64, C.c_int64, C.c_int32, C.c_int32,
                                   C.POINTER(C.c_int32), C.POINTER(C.c_int32)]

    def lib_ladder(M, s, num, den):
        lad = (C.c_int32 * 64)()
        n = C.c_int32(0)
        rc = L.kvs_paper_ladder(M, s, num, den, lad, C.byref(n))
        return rc, list(lad[:n.value])

    from fractions import Fraction
    rnd = random.Random(11)
    for _ in range(300):
        num, den = rnd.choice([(2, 1), (3, 2), (4, 3), (3, 1), (7, 4), (5, 3)])
        s = rnd.randint(0, 5000)
        M = s + rnd.randint(1, 2 ** rnd.randint(1, 20))
        rc, got = lib_ladder(M, s, num, den)
        assert rc == 0
        a = Fraction(num, den)
        ell = 0
        while a ** (ell + 1) <= M - s:
            ell += 1
        beta = Fraction(M - s) / a ** ell
        assert 1 <= beta < a
        want = [int(beta * a ** p) for p in range(ell + 1)]       # floor of an exact rational
        assert got == want == O.paper_ladder(M, s, num, den).tolist()
        assert got[-1] == M - s
    assert lib_ladder(10, 10, 2, 1)[0] == 1 and lib_ladder(10, 0, 1, 1)[0] == 1
    assert lib_ladder(2 ** 30, 0, 4, 3)[0] == 5                    # needs more than 64 levels

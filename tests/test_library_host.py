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
    lib.kvs_host_ladder_level.restype = C.c_uint32
    lib.kvs_host_ladder_level.argtypes = [C.c_uint32, C.POINTER(C.c_uint32), C.c_uint32]
    lib.kvs_strerror.restype = C.c_char_p
    return lib


def test_built_library_is_not_older_than_its_sources():
    # the GPU tests and the benchmark load the built library as it is; a library older than the
    # sources would test and time something else than what is committed
    if not os.path.exists(B.LIB):
        B.build()
    assert not B.is_stale(), "run `python paper_2601_22996_amd/build.py`: a source is newer than the library"


def test_exports_every_declared_symbol(L):
    header = open(os.path.join(ROOT, "include", "kvsched.h")).read()
    names = set(re.findall(r"\b(kvs_[a-z_]+)\s*\(", header))
    assert {"kvs_gba_simulate", "kvs_schedule_eval", "kvs_validate", "kvs_validate_static", "kvs_strerror",
            "kvs_version"} <= names
    assert not any(n.startswith("kvs_host_") for n in names), "test hooks belong in kvsched_test.h"
    hooks = set(re.findall(r"\b(kvs_[a-z_]+)\s*\(", open(os.path.join(ROOT, "include", "kvsched_test.h")).read()))
    assert hooks and all(n.startswith("kvs_host_") for n in hooks)
    for name in names | hooks:
        assert hasattr(L, name), name
    # the product binding marshals the product interface only
    binding = open(os.path.join(ROOT, "paper_2601_22996_amd", "kvsched.py")).read()
    assert "kvs_host_" not in binding
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


def test_ladder_level_counts_the_slices_below_a_length(L):
    # explicit ladders of every length up to the limit, lengths at, between, below and above the
    # slices; a length above the last slice has no level (answer n_lv), also on a full 64-slice ladder
    rng = random.Random(11)
    for n_lv in list(range(1, 9)) + [31, 32, 33, 62, 63, 64]:
        for _ in range(20):
            lad = sorted(rng.randrange(1, 5000) for _ in range(n_lv))
            arr = (C.c_uint32 * n_lv)(*lad)
            xs = {1, lad[0], lad[-1], lad[-1] + 1, 2 ** 30} | {v + d for v in lad for d in (-1, 0, 1) if v + d >= 1}
            for x in xs:
                want = sum(1 for v in lad if v < x)
                assert L.kvs_host_ladder_level(x, arr, n_lv) == want, (n_lv, x, lad)
    full = (C.c_uint32 * 64)(*range(1, 65))
    assert L.kvs_host_ladder_level(64, full, 64) == 63 and L.kvs_host_ladder_level(65, full, 64) == 64


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


def test_quadratic_ladder_matches_the_exact_oracle_or_refuses(L):
    # the library works with intervals of 64-bit-mantissa numbers and falls back on 128-bit integers:
    # where it answers, the answer is the exact ladder (the oracle's, in unbounded integer
    # arithmetic); where neither can decide a floor it says KVS_ELIMIT
    import numpy as np
    import oracle as O
    L.kvs_paper_ladder_quadratic.restype = C.c_int32
    L.kvs_paper_ladder_quadratic.argtypes = [C.c_int64, C.c_int64] + [C.c_int32] * 4 + [C.POINTER(C.c_int32)] * 2

    def lib(M, s, a, b, c, d):
        lad, n = (C.c_int32 * 64)(), C.c_int32()
        rc = L.kvs_paper_ladder_quadratic(M, s, a, b, c, d, lad, C.byref(n))
        return rc, list(lad[:n.value])

    rng = random.Random(5)
    answered = 0
    for a, b, c, d in [(7, 1, 13, 6), (1, 1, 5, 2), (0, 1, 2, 1), (3, 2, 3, 4), (0, 1, 3, 1), (5, 3, 7, 9)]:
        for _ in range(200):
            s = rng.randrange(0, 3000)
            M = s + rng.choice([1, 2, 3, 10, 160, 1000, 4096, 65536, 10 ** 6, 2 ** 30, rng.randrange(1, 2 ** 30)])
            rc, lad = lib(M, s, a, b, c, d)
            assert rc in (0, 5), rc
            if rc == 0:
                answered += 1
                assert lad == O.paper_ladder_quadratic(M, s, a, b, c, d).tolist(), (M, s, a, b, c, d)
    assert answered >= 1190            # undecidable floors are rare
    assert lib(256, 96, 7, 1, 13, 6) == (0, [1, 2, 5, 9, 16, 28, 51, 90, 160])
    # floors that are hit exactly (a rational factor, powers of sqrt 2) are decided in integers
    assert lib(256, 96, 2, 0, 0, 1) == (0, [1, 2, 5, 10, 20, 40, 80, 160])
    assert lib(1024, 0, 0, 1, 2, 1)[1] == O.paper_ladder_quadratic(1024, 0, 0, 1, 2, 1).tolist()
    assert lib(100, 0, 1, 0, 0, 1)[0] == 1                                           # alpha = 1
    assert lib(100, 100, 7, 1, 13, 6)[0] == 1 and lib(2 ** 31, 0, 7, 1, 13, 6)[0] == 1
    assert lib(2 ** 30, 0, 0, 1, 0, 1000)[0] == 1                                    # alpha = 0
    # a factor so close to 1 that 64 levels do not reach M - s
    assert lib(2 ** 20, 0, 100, 1, 2, 101)[0] == 5


def test_floor_sum_matches_the_plain_sum(L):
    L.kvs_host_floor_sum.restype = C.c_uint64
    L.kvs_host_floor_sum.argtypes = [C.c_uint64] * 3
    rnd = random.Random(11)
    for _ in range(4000):
        n = rnd.randint(1, 400)
        k = rnd.choice([1, 2, 3, rnd.randint(1, 60), rnd.randint(1, 10 ** 6), rnd.randint(1, 2 ** 40)])
        tau = rnd.choice([1, 2, rnd.randint(1, 50), rnd.randint(1, 10 ** 6), rnd.randint(1, 2 ** 31 - 1)])
        assert L.kvs_host_floor_sum(n, k, tau) == sum(i * tau // k for i in range(n)), (n, k, tau)
    # the largest phase the kernels accept: n * tau just below 2^31
    n, tau = 16384, 2 ** 17 - 1
    assert L.kvs_host_floor_sum(n, 1, tau) == tau * n * (n - 1) // 2
    assert L.kvs_host_floor_sum(n, 7, tau) == sum(i * tau // 7 for i in range(n))


def test_list_schedules_of_every_order_against_the_oracle(L):
    """The kernel's enumeration (a work unit = a prefix of the order, all orders of the last
    four jobs below it depth first; event rounds only, jumps in the search for a start) run on
    the host for every work unit: the minimum over the units is the oracle's."""
    import math
    import numpy as np
    import oracle as O
    L.kvs_host_best_of_unit.restype = C.c_int64
    L.kvs_host_best_of_unit.argtypes = [C.c_uint32, C.c_int32, C.POINTER(C.c_int32), C.c_int64, C.c_int64]
    L.kvs_host_perm_units.restype = C.c_uint32
    L.kvs_host_perm_units.argtypes = [C.c_int32]
    for n in range(1, 11):
        assert L.kvs_host_perm_units(n) == math.factorial(n) // math.factorial(min(n, 4))
    rng = np.random.default_rng(8)
    for case in range(48):
        n = int(rng.integers(1, 8))
        o = rng.integers(1, 12, n).astype(np.int32)
        s = int(rng.integers(0, 5))
        M = int(rng.integers(s + 12, 45)) if case % 4 else s + int(o.max())   # no two jobs overlap
        ptr = o.ctypes.data_as(C.POINTER(C.c_int32))
        units = L.kvs_host_perm_units(n)
        best = min(L.kvs_host_best_of_unit(u, n, ptr, s, M) for u in range(units))
        assert best == O.opt_perm(o, s, M), (o, s, M)
        assert L.kvs_host_best_of_unit(units, n, ptr, s, M) == -1                # no such unit
    # by hand: two jobs that cannot overlap: shortest first, 2 + 5
    o = np.array([3, 2], np.int32)
    assert L.kvs_host_best_of_unit(0, 2, o.ctypes.data_as(C.POINTER(C.c_int32)), 2, 5) == 7
    # o = 2, 2, s = 0, M = 3: the second job starts one round later
    o = np.array([2, 2], np.int32)
    assert L.kvs_host_best_of_unit(0, 2, o.ctypes.data_as(C.POINTER(C.c_int32)), 0, 3) == 5
    # five jobs: unit u fixes the first job (the u-th of the input) and enumerates the rest below
    # it.  No two jobs can overlap (s + 1 = 5 each, M = 8), so the best order is shortest first:
    # 1 + 2 + 3 + 4 + 7 when a unit job leads, 3 + 4 + 5 + 6 + 7 when the long one does
    o = np.array([3, 1, 1, 1, 1], np.int32)
    ptr = o.ctypes.data_as(C.POINTER(C.c_int32))
    per_first = [L.kvs_host_best_of_unit(u, 5, ptr, 4, 8) for u in range(5)]
    assert per_first == [25, 17, 17, 17, 17] and O.opt_perm(o, 4, 8) == 17


def test_bounds_argument_checks(L):
    class Jobs(C.Structure):
        _fields_ = [("n_instances", C.c_int32), ("n_jobs", C.c_int32), ("o", C.c_void_p),
                    ("s", C.c_void_p), ("o_est", C.c_void_p), ("s_scalar", C.c_int32),
                    ("M", C.c_int64)]
    i32 = C.c_int32
    L.kvs_flow_bounds.restype = i32
    L.kvs_flow_bounds.argtypes = [C.POINTER(Jobs), C.POINTER(i32), i32, C.c_void_p, C.c_void_p, C.c_void_p]
    L.kvs_opt_perm.restype = i32
    L.kvs_opt_perm.argtypes = [C.POINTER(Jobs), C.c_void_p, C.c_void_p]
    EINVAL, ELIMIT = 1, 5
    one = (i32 * 1)(1)
    fb = lambda j, t, n, up, ar: L.kvs_flow_bounds(C.byref(j), t, n, up, ar, None)
    assert L.kvs_flow_bounds(None, one, 1, 8, 8, None) == EINVAL
    assert fb(Jobs(4, 8, None, None, None, 0, 100), one, 1, 8, 8) == EINVAL      # o is null
    assert fb(Jobs(4, 8, 1, None, None, 0, 100), one, 1, None, 8) == EINVAL      # no room for the bound
    assert fb(Jobs(4, 8, 1, None, None, 0, 100), (i32 * 1)(0), 1, 8, 8) == EINVAL  # tau0 < 1
    assert fb(Jobs(4, 8, 1, None, None, 0, 0), one, 1, 8, 8) == EINVAL           # M < 1
    assert fb(Jobs(4, 16385, 1, None, None, 0, 100), one, 1, 8, 8) == ELIMIT
    assert fb(Jobs(4, 8, 1, None, None, 0, 100), one, 65, 8, 8) == ELIMIT
    assert fb(Jobs(0, 8, None, None, None, 0, 100), one, 1, 8, 8) == 0           # nothing to do
    assert fb(Jobs(4, 8, 1, None, None, 0, 100), one, 0, None, None) == 0
    op = lambda j, out: L.kvs_opt_perm(C.byref(j), out, None)
    assert op(Jobs(4, 8, 1, 1, None, 0, 100), 8) == EINVAL                       # per-job prompts
    assert op(Jobs(4, 11, 1, None, None, 0, 100), 8) == ELIMIT
    assert op(Jobs(4, 8, 1, None, None, 0, 100), None) == EINVAL
    assert op(Jobs(0, 8, None, None, None, 0, 100), None) == 0

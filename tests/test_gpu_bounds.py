"""Parity of the bound evaluators (kvs_flow_bounds, kvs_opt_perm) against the CPU oracle,
through the C ABI.  Bit-exact: every quantity is an integer."""
import json
import os

import numpy as np
import pytest

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")

import oracle as O
from paper_2601_22996_amd import workloads as W

GOLD = json.load(open(os.path.join(os.path.dirname(__file__), "golden", "paper_values.json")))


@pytest.fixture(scope="module")
def K():
    assert torch.cuda.is_available(), "these tests need the GPU"
    from paper_2601_22996_amd import kvsched
    kvsched.lib()
    return kvsched


def dev(a):
    return None if a is None else torch.from_numpy(np.ascontiguousarray(a, dtype=np.int32)).cuda()


def gpu_bounds(K, o, s, M, tau0):
    r = K.flow_bounds(dev(o), s if np.isscalar(s) else dev(s), M, tau0)
    torch.cuda.synchronize()
    return r["upper_gba"].cpu().numpy(), r["area_lb_num"].cpu().numpy()


def oracle_bounds(o, s, M, tau0, rows=None):
    rows = range(o.shape[0]) if rows is None else rows
    up = np.array([[O.upper_gba(o[i], s if np.isscalar(s) else s[i], M, t) for i in rows] for t in tau0],
                  np.int64).reshape(len(tau0), -1)
    ar = np.array([O.area_lb(o[i], s if np.isscalar(s) else s[i]) for i in rows], np.int64)
    return up, ar


def test_printed_values_and_hand_examples(K):
    g, u = GOLD["example1_sps"], GOLD["uniform_gba"]
    up, ar = gpu_bounds(K, np.full((1, g["n"]), g["o"]), g["s"], g["M"], [g["tau"]])
    assert up[0, 0] == g["flow"] and ar[0] == 120 * 15          # n(n+1)/2 * Area(5, 0)
    up, _ = gpu_bounds(K, np.full((2, u["n"]), u["o"]), u["s"], u["M"], [16, 1])
    assert up[:, 1].tolist() == [u["flow"], u["flow"] + 200 * 15]
    up, ar = gpu_bounds(K, np.array([[1, 1, 3, 4]]), 0, 4, [1])
    assert up[0, 0] == 20 and ar[0] == 4 * 1 + 3 * 1 + 2 * 6 + 1 * 10
    up, _ = gpu_bounds(K, np.array([[1, 1, 1, 1, 2]]), 0, 2, [1])
    assert up[0, 0] == 11
    _, ar = gpu_bounds(K, np.array([[2, 4]]), np.array([[10, 0]]), 64, [1])
    assert ar[0] == 2 * 10 + 23                                   # ordered by area, not by length


@pytest.mark.parametrize("n", [1, 2, 15, 16, 17, 63, 64, 65, 257, 1000, 1024, 1025, 2048, 2049, 4096, 4097, 8193])
def test_random_instances(K, n):
    rng = np.random.default_rng(1000 + n)
    I = 24 if n <= 1000 else (6 if n <= 4100 else 2)
    o = np.minimum(rng.geometric(1 / 40, (I, n)), 3000).astype(np.int32)
    o[0] = 1                                                      # a single class
    hetero = n % 2 == 1
    s = rng.integers(0, 300, (I, n)).astype(np.int32) if hetero else int(rng.integers(0, 300))
    M = int(rng.integers(4000, 60000))
    tau0 = [1, 2, 3, 4, 5, 6, 7, 12, 16, 100, 1024, 4096]
    up, ar = gpu_bounds(K, o, s, M, tau0)
    wup, war = oracle_bounds(o, s, M, tau0)
    assert np.array_equal(up, wup), np.argwhere(up != wup)[:4]
    assert np.array_equal(ar, war), np.argwhere(ar != war)[:4]


@pytest.mark.parametrize("n", [600, 5000])
def test_area_bound_with_crowded_buckets(K, n):
    """The area bound ranks keys inside buckets of leading bits and falls back on a full sort when
    a bucket is crowded (more than 128 keys): instances just below and just above that, with ties
    inside a bucket and neighbouring values that share one, against the oracle."""
    rng = np.random.default_rng(77 + n)
    rows = []
    for crowd in (127, 128, 129, 400):
        o = rng.integers(1, 2000, n).astype(np.int32)
        s = rng.integers(0, 300, n).astype(np.int32)
        at = rng.choice(n, crowd, replace=False)
        o[at] = 1                              # areas s + 1 = 5001 and 5002: one bucket at either
        s[at] = rng.integers(5000, 5002, crowd)  # resolution (16 or 32 values wide there), many ties
        rows.append((o, s))
    o = np.stack([r[0] for r in rows])
    s = np.stack([r[1] for r in rows])
    _, ar = gpu_bounds(K, o, s, 1 << 20, [1])
    _, war = oracle_bounds(o, s, 1 << 20, [1])
    assert np.array_equal(ar, war), (ar, war)


def test_64_points_and_outputs_optional(K):
    rng = np.random.default_rng(4)
    o = np.minimum(rng.geometric(1 / 100, (5, 700)), 5000).astype(np.int32)
    s = rng.integers(0, 64, (5, 700)).astype(np.int32)
    tau0 = list(range(1, 65))                                     # 32 distinct odd bases
    up, ar = gpu_bounds(K, o, s, 20000, tau0)
    wup, war = oracle_bounds(o, s, 20000, tau0)
    assert np.array_equal(up, wup) and np.array_equal(ar, war)
    r = K.flow_bounds(dev(o), dev(s), 20000, tau0, area=False)    # no area output
    torch.cuda.synchronize()
    assert np.array_equal(r["upper_gba"].cpu().numpy(), wup)
    r = K.flow_bounds(dev(o), dev(s), 20000, [])                  # no points
    torch.cuda.synchronize()
    assert np.array_equal(r["area_lb_num"].cpu().numpy(), war)


def test_largest_instance_and_long_jobs(K):
    rng = np.random.default_rng(6)
    n = 16384
    o = np.minimum((16 * rng.random((2, n)) ** (-1 / 1.2)).astype(np.int64), 100000).astype(np.int32)
    s = rng.integers(0, 5000, (2, n)).astype(np.int32)
    M = 1 << 22
    tau0 = [1, 3, 64]
    up, ar = gpu_bounds(K, o, s, M, tau0)
    wup, war = oracle_bounds(o, s, M, tau0)
    assert np.array_equal(up, wup) and np.array_equal(ar, war)


def test_in_band_errors(K):
    o = np.full((4, 50), 7, np.int32)
    o[1, 3] = 0                                                   # o < 1
    o[2, 9] = 95                                                  # s + o > M
    up, ar = gpu_bounds(K, o, 10, 100, [1, 8])
    assert up[:, 1].tolist() == [-1, -1] and up[:, 2].tolist() == [-1, -1] and ar[1] == ar[2] == -1
    wup, war = oracle_bounds(o, 10, 100, [1, 8], rows=[0, 3])
    assert np.array_equal(up[:, [0, 3]], wup) and np.array_equal(ar[[0, 3]], war)
    # a class with n_p * tau_p >= 2^31: 4 jobs of length 2^30 on the slice 2^30
    big = np.full((1, 4), 1 << 30, np.int32)
    up, ar = gpu_bounds(K, big, 0, 1 << 32, [1, 1 << 30])
    assert up[:, 0].tolist() == [-1, -1]
    assert ar[0] == O.area_lb(big[0], 0)                          # 10 * Area(2^30, 0) < 2^63
    # the area sum leaves 64 bits: 16384 jobs of area 2^59
    big = np.full((1, 16384), 1 << 30, np.int32)
    _, ar = gpu_bounds(K, big, 0, 1 << 32, [])
    assert ar[0] == -1


def test_upper_bound_holds_against_the_simulated_flow(K):
    """Lemma "GBA Upper Bound via Packing Efficiency" on the device's own schedules: the bound of
    kvs_flow_bounds is never below the flow time of kvs_gba_simulate at the same initial slice."""
    w = W.WORKLOADS[3]
    d = W.generate(w, 0, 512)
    tau0 = [1, 2, 4, 8, 16, 32, 64, 128]
    r = K.flow_bounds(dev(d["o"]), dev(d["s"]), w.M, tau0)
    g = K.gba_simulate(dev(d["o"]), dev(d["s"]), w.M, [(t, 0, 0, 0) for t in tau0])
    torch.cuda.synchronize()
    assert bool((r["upper_gba"] >= g["flow"]).all()) and bool((g["flow"] > 0).all())
    # and the optimum lies above the area bound: area_lb / M <= OPT <= GBA
    assert bool((r["area_lb_num"][None, :] <= g["flow"] * w.M).all())


@pytest.mark.parametrize("cfg,count,sample", [(2, 4096, 64), (3, 4096, 48), (5, 256, 12)])
def test_workloads_at_full_size_sampled(K, cfg, count, sample):
    w = W.WORKLOADS[cfg]
    d = W.generate(w, 0, count)
    s = d["s"] if d["s"] is not None else d["s_scalar"]
    tau0 = [1, 2, 4, 8, 16, 32, 64, 128]
    up, ar = gpu_bounds(K, d["o"], s, w.M, tau0)
    assert up.min() > 0 and ar.min() > 0
    rows = np.random.default_rng(cfg).choice(count, sample, replace=False)
    wup, war = oracle_bounds(d["o"], s, w.M, tau0, rows=rows)
    assert np.array_equal(up[:, rows], wup) and np.array_equal(ar[rows], war)


# ---------------------------------------------------------------------------
# best list schedule over all orders
# ---------------------------------------------------------------------------
def gpu_opt(K, o, s, M):
    r = K.opt_perm(dev(o), s, M)
    torch.cuda.synchronize()
    return r.cpu().numpy()


def test_opt_perm_config1_and_hand_cases(K):
    w = W.WORKLOADS[1]
    d = W.generate(w, 0, 1)
    got = gpu_opt(K, d["o"], d["s_scalar"], w.M)
    assert got[0] == O.opt_perm(d["o"][0], d["s_scalar"], w.M)
    assert gpu_opt(K, np.array([[3, 2]]), 2, 5)[0] == 7
    assert gpu_opt(K, np.array([[2, 2]]), 0, 3)[0] == 5
    assert gpu_opt(K, np.array([[3, 2]]), 0, 3)[0] == 6
    assert gpu_opt(K, np.array([[9]]), 4, 13)[0] == 9


@pytest.mark.parametrize("n", [1, 2, 3, 5, 7, 8, 9])
def test_opt_perm_random(K, n):
    rng = np.random.default_rng(50 + n)
    I = 40 if n <= 7 else (12 if n == 8 else 2)
    o = rng.integers(1, 33, (I, n)).astype(np.int32)
    s = int(rng.integers(0, 20))
    M = int(rng.integers(s + 33, 300))
    o[0] = M - s                                                  # nothing overlaps
    got = gpu_opt(K, o, s, M)
    want = [O.opt_perm(o[i], s, M) for i in range(I)]
    assert got.tolist() == want


def test_opt_perm_ten_jobs_and_errors(K):
    rng = np.random.default_rng(77)
    o = rng.integers(1, 9, (3, 10)).astype(np.int32)
    o[1, 4] = 0                                                   # invalid job
    o[2, 0] = 40                                                  # s + o > M
    got = gpu_opt(K, o, 2, 30)
    assert got[1] == -1 and got[2] == -1
    assert got[0] == O.opt_perm(o[0], 2, 30)
    long = np.full((1, 4), 1 << 19, np.int32)                     # lengths sum to 2^21 > the limit
    assert gpu_opt(K, long, 0, 1 << 30)[0] == -1

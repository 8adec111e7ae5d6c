"""The seeded input generator: the same numbers for an instance whatever range, chunking or
thread count produced it; values inside the ranges the workloads are specified with."""
import numpy as np
import pytest

from paper_2601_22996_amd import workloads as W


@pytest.mark.parametrize("cfg", [2, 3, 4, 5])
def test_ranges_are_reproducible_and_independent_of_chunking(cfg):
    w = W.WORKLOADS[cfg]
    hi = min(w.n_instances, 700)
    whole = W.generate(w, 0, hi, threads=1)
    parts = [W.generate(w, a, b, threads=3) for a, b in ((0, 256), (256, 300), (300, hi))]
    for key in ("o", "s", "o_est"):
        if whole[key] is None:
            assert all(p[key] is None for p in parts)
            continue
        assert whole[key].dtype == np.int32 and whole[key].shape == (hi, w.n_jobs)
        assert np.array_equal(whole[key], np.concatenate([p[key] for p in parts]))
    again = W.generate(w, 0, hi, threads=4)
    assert np.array_equal(again["o"], whole["o"])
    assert whole["M"] == w.M


@pytest.mark.parametrize("cfg", [1, 2, 3, 4, 5])
def test_values_respect_the_specified_ranges(cfg):
    w = W.WORKLOADS[cfg]
    d = W.generate(w, 0, min(w.n_instances, 300))
    o = d["o"].astype(np.int64)
    s = d["s"].astype(np.int64) if d["s"] is not None else np.int64(d["s_scalar"])
    assert o.min() >= 1 and (np.asarray(s) >= 0).all()
    assert (s + o).max() <= w.M                                   # every job fits the budget alone
    caps = {1: 32, 2: 4096, 3: 8192, 4: 8192, 5: 16384}
    assert o.max() <= caps[cfg]
    if w.s_range is not None:
        assert d["s"].min() >= w.s_range[0] and d["s"].max() <= w.s_range[1]
    if w.estimates:
        e = d["o_est"].astype(np.int64)
        assert e.min() >= 1 and (e + s).max() <= w.M
        assert 0.2 < float(np.mean(e == o)) < 0.99 or float(np.mean(np.abs(np.log(e / o)))) > 0.1
    if cfg == 5:                                                  # Pareto(1.5) from 16: median 16 * 2^(2/3)
        assert o.min() == 16 and 24 <= float(np.median(o)) <= 27
    if cfg == 2:                                                  # geometric with mean 256, capped
        assert 230 <= float(o.mean()) <= 280


def test_sweeps_have_the_specified_points():
    assert len(W.WORKLOADS[1].sweep()) == 1
    assert len(W.WORKLOADS[2].sweep()) == 14
    assert len(W.WORKLOADS[3].sweep()) == 8
    assert len(W.WORKLOADS[4].sweep()) == 8
    pts = W.WORKLOADS[5].sweep()
    assert len(pts) == 16 and sorted(set(pts[:, 0].tolist())) == [1, 2, 4, 8, 16, 32, 64, 128]
    assert set(pts[:, 1].tolist()) == {W.SPS, W.SIMS} and (pts[:, 2] == 0).all()

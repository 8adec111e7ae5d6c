"""Seeded synthetic instances for the five evaluation workloads.

Input generation only: this module holds none of the scheduling arithmetic and
is the one piece of code that both the GPU path and its CPU checker are fed
from.  The instances stand in for the right-skewed response-length traces of
the paper's numerical experiments (appendix "Numerical Experiments"), which
are not redistributable: lengths are drawn from geometric, log-normal and
Pareto laws with the sizes listed in `WORKLOADS`.

Instances are generated in blocks of `BLOCK` consecutive instances, each block
from its own `numpy` PCG64 stream seeded by (workload seed, block index), so
any instance range can be produced without producing the ones before it and a
range always holds the same numbers whatever else is generated.
"""
from __future__ import annotations

import threading
from dataclasses import dataclass, field
from typing import Optional

import numpy as np

BLOCK = 256
SPS, SIMS = 0, 1
MODE_GBA, MODE_GSA, MODE_GBAD = 0, 1, 2


@dataclass(frozen=True)
class Workload:
    name: str
    n_instances: int
    n_jobs: int
    M: int
    seed: int
    s_scalar: Optional[int]          # None: per-job prompt lengths
    s_range: Optional[tuple]         # (lo, hi) inclusive when per-job
    o_law: str
    estimates: bool
    tau0: tuple
    scheds: tuple
    mode: int = MODE_GBA
    points: tuple = field(default=(), compare=False)

    def sweep(self) -> np.ndarray:
        """Sweep points as int32 rows (tau0, sched, k, mode); k = 0 is automatic."""
        rows = [(t, sc, 0, self.mode) for t in self.tau0 for sc in self.scheds]
        return np.asarray(rows, dtype=np.int32)


_POW2_64 = (1, 2, 4, 8, 16, 32, 64)
_POW2_128 = (1, 2, 4, 8, 16, 32, 64, 128)

WORKLOADS = {
    1: Workload("cfg1_tiny_uniform", 1, 8, 256, 0, 16, None, "uniform_1_32", False,
                (1,), (SPS,)),
    2: Workload("cfg2_geometric_s128", 4096, 1000, 65536, 1, 128, None, "geometric_256_cap4096",
                False, _POW2_64, (SPS, SIMS)),
    3: Workload("cfg3_lognormal_hetero_s", 4096, 2000, 262144, 2, None, (32, 2048),
                "lognormal_5_1_cap8192", False, _POW2_128, (SPS,)),
    4: Workload("cfg4_geometric_estimates", 1024, 2000, 131072, 3, 256, None,
                "geometric_512_cap8192", True, _POW2_128, (SPS,)),
    5: Workload("cfg5_pareto_hetero_s", 65536, 10000, 1048576, 4, None, (64, 4096),
                "pareto_1p5_min16_cap16384", False, _POW2_128, (SPS, SIMS)),
}


_scratch = threading.local()


def _buf(shape) -> np.ndarray:
    """Per-thread float64 scratch, reused between blocks (fresh pages are slow)."""
    b = getattr(_scratch, "buf", None)
    if b is None or b.shape != shape:
        b = np.empty(shape, np.float64)
        _scratch.buf = b
    return b


def _draw_o(law: str, rng: np.random.Generator, shape, out: np.ndarray) -> None:
    """Response lengths of one block into `out` (int32), clamped to >= 1."""
    if law == "uniform_1_32":
        out[...] = rng.integers(1, 33, size=shape)
    elif law == "geometric_256_cap4096":
        out[...] = np.minimum(rng.geometric(1.0 / 256.0, size=shape), 4096)
    elif law == "geometric_512_cap8192":
        out[...] = np.minimum(rng.geometric(1.0 / 512.0, size=shape), 8192)
    elif law == "lognormal_5_1_cap8192":
        b = _buf(shape)
        rng.standard_normal(out=b)
        np.add(b, 5.0, out=b)                       # N(5, 1)
        np.exp(b, out=b)
        np.rint(b, out=b)
        np.clip(b, 1, 8192, out=b)
        out[...] = b
    elif law == "pareto_1p5_min16_cap16384":
        b = _buf(shape)
        rng.random(out=b)
        np.subtract(1.0, b, out=b)                  # in (0, 1]
        np.power(b, -1.0 / 1.5, out=b)
        np.multiply(b, 16.0, out=b)
        np.floor(b, out=b)
        np.minimum(b, 16384, out=b)
        out[...] = b
    else:
        raise ValueError(law)
    np.maximum(out, 1, out=out)


def _block(w: Workload, b: int, o: np.ndarray, s, e) -> None:
    """Block `b` (BLOCK instances) into the given int32 arrays of shape [BLOCK][n]."""
    rng = np.random.Generator(np.random.PCG64(np.random.SeedSequence([w.seed, b])))
    shape = (BLOCK, w.n_jobs)
    _draw_o(w.o_law, rng, shape, o)
    if s is not None:
        lo, hi = w.s_range
        s[...] = rng.integers(lo, hi + 1, size=shape, dtype=np.int32)
    if e is not None:
        f = _buf(shape)
        rng.standard_normal(out=f)
        np.multiply(f, 0.5, out=f)                  # N(0, sigma = 0.5)
        np.exp(f, out=f)
        np.multiply(f, o, out=f)
        np.rint(f, out=f)
        np.clip(f, 1, w.M - w.s_scalar, out=f)
        e[...] = f


def generate(w: Workload, i0: int = 0, i1: Optional[int] = None, threads: int = 1,
             out: Optional[dict] = None) -> dict:
    """Instances [i0, i1) of workload `w` as row-major int32 arrays.

    Returns dict(o=[cnt][n], s=[cnt][n] or None, o_est=[cnt][n] or None,
    s_scalar=int, M=int).  `threads` > 1 draws blocks concurrently; the
    result does not depend on it.  `out` may hand in arrays of a previous call
    with the same shapes, to be overwritten."""
    i1 = w.n_instances if i1 is None else i1
    if not (0 <= i0 <= i1 <= w.n_instances):
        raise ValueError("instance range out of bounds")
    cnt = i1 - i0
    if out is not None and out["o"].shape == (cnt, w.n_jobs):
        o, s, e = out["o"], out["s"], out["o_est"]
    else:
        o = np.empty((cnt, w.n_jobs), np.int32)
        s = np.empty((cnt, w.n_jobs), np.int32) if w.s_scalar is None else None
        e = np.empty((cnt, w.n_jobs), np.int32) if w.estimates else None

    def fill(b: int) -> None:
        lo, hi = max(i0, b * BLOCK), min(i1, (b + 1) * BLOCK)
        dst = slice(lo - i0, hi - i0)
        if hi - lo == BLOCK:
            _block(w, b, o[dst], None if s is None else s[dst], None if e is None else e[dst])
            return
        bo = np.empty((BLOCK, w.n_jobs), np.int32)
        bs = np.empty_like(bo) if s is not None else None
        be = np.empty_like(bo) if e is not None else None
        _block(w, b, bo, bs, be)
        src = slice(lo - b * BLOCK, hi - b * BLOCK)
        o[dst] = bo[src]
        if s is not None:
            s[dst] = bs[src]
        if e is not None:
            e[dst] = be[src]

    blocks = range(i0 // BLOCK, (i1 + BLOCK - 1) // BLOCK) if cnt else range(0)
    if threads > 1 and len(blocks) > 1:
        from concurrent.futures import ThreadPoolExecutor
        with ThreadPoolExecutor(max_workers=threads) as ex:
            list(ex.map(fill, blocks))
    else:
        for b in blocks:
            fill(b)
    return dict(o=o, s=s, o_est=e, s_scalar=(w.s_scalar or 0), M=w.M)

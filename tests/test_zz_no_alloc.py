"""The entry point that allocates nothing (kvs_validate_static) against kvs_validate,
through the C ABI: two calls in a row, the second on a smaller input, then the
other findings, which must not leak from one call into the next."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")


@pytest.fixture(scope="module")
def K():
    assert torch.cuda.is_available(), "these tests need the GPU"
    from paper_2601_22996_amd import kvsched
    kvsched.lib()
    return kvsched


def dev(a):
    return torch.from_numpy(np.ascontiguousarray(a, dtype=np.int32)).cuda()


def test_static_validate_matches_validate_on_consecutive_calls(K):
    rng = np.random.default_rng(12)
    M = 5000
    big_o = rng.integers(1, 3000, (300, 2500)).astype(np.int32)
    big_s = rng.integers(0, 2000, (300, 2500)).astype(np.int32)
    big_o[211, 1999] = 4000                                   # s + o > M for one job of the large input
    big_s[211, 1999] = 1500
    small_o = rng.integers(1, 3000, (7, 130)).astype(np.int32)   # clean and smaller
    small_s = rng.integers(0, 2000, (7, 130)).astype(np.int32)
    cases = [(big_o, big_s, None), (small_o, small_s, None)]
    # further calls: each kind of finding, then a clean input again
    bad = small_o.copy(); bad[3, 7] = 0
    cases.append((bad, small_s, None))
    cases.append((small_o, small_s, None))
    est = small_o.copy(); est[6, 129] = -4
    cases.append((small_o, small_s, est))
    lng = small_o.copy(); lng[0, 0] = 2 ** 30 + 1
    cases.append((lng, small_s, None))
    cases.append((small_o, 17, None))                         # common prompt length
    want_codes = [K.EJOB_INFEASIBLE, K.OK, K.EINVAL, K.OK, K.EINVAL, K.ERANGE, K.OK]
    for (o, s, e), want in zip(cases, want_codes):
        do = dev(o)
        ds = s if np.isscalar(s) else dev(s)
        de = None if e is None else dev(e)
        Mx = 2 ** 31 if want == K.ERANGE else M
        ref = K.validate(do, ds, Mx, de)
        got = K.validate_static(do, ds, Mx, de)
        assert ref == want and got == ref, (ref, got, want)
    # on a side stream, and an empty batch
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    assert K.validate_static(dev(big_o), dev(big_s), M, stream=side) == K.EJOB_INFEASIBLE
    assert K.validate_static(dev(small_o), dev(small_s), M, stream=side) == K.OK
    assert K.validate_static(dev(small_o)[:0], 3, M) == K.OK

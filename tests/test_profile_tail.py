"""Latency tables from measured latency distributions (Section 8 of the paper, second limitation: a model whose
latency depends on its input is given the tail of its measured latencies as processing time).

The reference (oracle/profile_oracle.py) is pinned to values known by hand and to numpy's inverted-CDF percentile;
the library's estimator_profile_tail (host code, no device work) must agree with it on every entry."""
import ctypes

import numpy as np
import pytest

from oracle import profile_oracle as po
from paper_1812_01776_amd import estimator as binding


# ---- the reference against what is known without it
def test_percentile_of_the_first_hundred_integers():
    xs = list(range(1, 101))
    assert po.percentile_tail(xs, 9900) == 99
    assert po.percentile_tail(xs, 10000) == 100
    assert po.percentile_tail(xs, 100) == 1
    assert po.percentile_tail(xs, 5000) == 50
    assert po.percentile_tail(xs, 5001) == 51      # just above half: the next sample
    assert po.percentile_tail(list(range(1, 1001)), 9990) == 999
    assert po.percentile_tail([5], 1) == 5 and po.percentile_tail([5], 10000) == 5
    assert po.percentile_tail([9, 1, 5, 5, 3], 6000) == 5   # order of the samples does not matter; ties count once each


@pytest.mark.parametrize("seed", range(6))
def test_percentile_is_numpys_inverted_cdf(seed):
    rng = np.random.default_rng(seed)
    n = int(rng.integers(1, 700))
    xs = rng.integers(1, 50, size=n) if seed % 2 else rng.integers(1, 2**32, size=n, dtype=np.uint64)
    for pct in (100, 2500, 5000, 9000, 9900, 9990, 10000):
        if (pct * n) % 10000 == 0 and pct != 10000:
            continue  # (numpy multiplies in floating point: leave out the ranks that land exactly on an integer)
        assert po.percentile_tail(xs, pct) == int(np.percentile(xs, pct / 100.0, method="inverted_cdf"))


def test_sigma_tail_by_hand():
    assert po.sigma_tail([7] * 5, 3000) == 7                  # no spread
    assert po.sigma_tail([0, 0, 20, 20], 3000) == 40          # mean 10, sigma 10
    assert po.sigma_tail([0, 0, 20, 20], 0) == 10
    assert po.sigma_tail([0, 0, 20, 20], 1500) == 25
    assert po.sigma_tail([1, 2, 3, 4], 1000) == 4             # 2.5 + sqrt(1.25) = 3.618...
    assert po.sigma_tail([1, 2, 3, 4], 2000) == 5             # 2.5 + 2.236... = 4.736...
    assert po.sigma_tail([1, 2], 1000) == 2                   # 1.5 + 0.5 exactly 2: no rounding up past it
    assert po.sigma_tail([1, 2], 1001) == 3
    assert po.sigma_tail([1, 1, 2], 0) == 2                   # mean 4/3 rounded up
    assert po.sigma_tail([0, 3], 1000) == 3                   # 1.5 + 1.5


@pytest.mark.parametrize("seed", range(4))
def test_sigma_tail_close_to_floating_point(seed):
    rng = np.random.default_rng(100 + seed)
    xs = rng.gamma(4.0, 2500.0, size=2000).astype(np.uint32) + 1
    for k in (0, 1000, 2000, 3000):
        want = float(np.mean(xs)) + k / 1000.0 * float(np.std(xs))
        got = po.sigma_tail(xs, k)
        assert want - 1e-6 <= got < want + 1.0 + 1e-6


def test_tails_order():
    rng = np.random.default_rng(7)
    xs = rng.gamma(2.0, 4000.0, size=999).astype(np.uint32) + 1
    p = [po.percentile_tail(xs, q) for q in (5000, 9000, 9900, 10000)]
    assert p == sorted(p) and p[-1] == int(xs.max())
    s = [po.sigma_tail(xs, k) for k in (0, 1000, 2000, 3000)]
    assert s == sorted(s) and s[0] >= int(np.floor(xs.mean()))


# ---- the library against the reference
@pytest.fixture(scope="module")
def lib():
    return binding.load_library()


def _cases():
    rng = np.random.default_rng(2024)
    yield rng.gamma(3.0, 3000.0, size=(2, 3, 8, 500)).astype(np.uint32) + 1          # a [S][H][Bmax] table of 500 samples
    yield rng.integers(1, 2**32, size=(5, 64), dtype=np.uint64).astype(np.uint32)   # the whole 32-bit range
    yield rng.integers(1, 4, size=(40, 33)).astype(np.uint32)                        # many ties, perfect-square variances
    yield np.full((3, 17), 0xFFFFFFFF, np.uint32)                                    # the largest latency, no spread
    yield rng.integers(1, 1000, size=(7, 1)).astype(np.uint32)                       # one sample per entry
    yield np.array([[1, 2], [1, 4], [1, 1]], np.uint32)                              # sums that land on integers


@pytest.mark.parametrize("case", range(6))
def test_library_matches_reference(lib, case):
    x = list(_cases())[case]
    flat = x.reshape(-1, x.shape[-1])
    for pct in (1, 5000, 9900, 9990, 10000):
        got = binding.profile_tail(x, binding.EST_TAIL_PERCENTILE, pct, lib)
        assert got.shape == x.shape[:-1]
        assert got.reshape(-1).tolist() == [po.percentile_tail(r, pct) for r in flat]
    for k in (0, 1000, 1001, 2500, 3000):
        want = [po.sigma_tail(r, k) for r in flat]
        if max(want) > 0xFFFFFFFF:
            with pytest.raises(binding.EstimatorError):
                binding.profile_tail(x, binding.EST_TAIL_SIGMA, k, lib)
            continue
        assert binding.profile_tail(x, binding.EST_TAIL_SIGMA, k, lib).reshape(-1).tolist() == want


def test_library_largest_sample_count(lib):
    rng = np.random.default_rng(5)
    x = rng.integers(1, 2**32, size=(1, 65536), dtype=np.uint64).astype(np.uint32)
    assert int(binding.profile_tail(x, binding.EST_TAIL_PERCENTILE, 9900, lib)[0]) == int(np.sort(x[0])[64881 - 1])  # ceil(0.99 x 65536) = 64881
    got = int(binding.profile_tail(x, binding.EST_TAIL_SIGMA, 1000, lib)[0])
    want = float(np.mean(x[0].astype(np.float64))) + float(np.std(x[0].astype(np.float64)))
    assert abs(got - want) < 16.0  # (float64 at 2^32 scale; the exact comparison is in test_library_matches_reference)


def test_library_errors_leave_output_untouched(lib):
    x = np.array([[3, 4, 5]], np.uint32)
    out = np.full(1, 77, np.uint32)

    def call(samples, n_entries, n_samples, mode, param, o=out):
        return lib.estimator_profile_tail(samples, ctypes.c_uint64(n_entries), ctypes.c_uint32(n_samples), ctypes.c_uint32(mode),
                                          ctypes.c_uint32(param), o.ctypes.data_as(ctypes.c_void_p) if o is not None else None)

    p = x.ctypes.data_as(ctypes.c_void_p)
    assert call(p, 0, 3, 0, 9900) == binding.EST_OK                      # nothing to do
    assert call(None, 1, 3, 0, 9900) == binding.EST_EINVAL
    assert call(p, 1, 3, 0, 9900, None) == binding.EST_EINVAL
    assert call(p, 1, 0, 0, 9900) == binding.EST_EINVAL                  # no samples
    assert call(p, 1, 65537, 0, 9900) == binding.EST_EINVAL
    assert call(p, 1, 3, 2, 9900) == binding.EST_EINVAL                  # unknown mode
    assert call(p, 1, 3, 0, 0) == binding.EST_EINVAL and call(p, 1, 3, 0, 10001) == binding.EST_EINVAL
    assert call(p, 1, 3, 1, 10001) == binding.EST_EINVAL
    z = np.zeros((1, 3), np.uint32)
    assert call(z.ctypes.data_as(ctypes.c_void_p), 1, 3, 0, 9900) == binding.EST_EINVAL   # a zero latency
    assert out[0] == 77
    assert call(p, 1, 3, 0, 9900) == binding.EST_OK and out[0] == 5

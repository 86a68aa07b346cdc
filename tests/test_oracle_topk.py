"""Pins for the oracle's Top_K operator (CPU only).

Pins: brute-force subset enumeration (tie rule, special values), the three
invariants (nnz == K, residual + sent == input, min|sent| >= max|residual|),
the contraction bound of the paper's Eq. "topk_bound", the special cases K = 0
and K = d, and agreement with numpy's lexsort on mid-sized inputs.
"""
import numpy as np
import pytest

from _brute import brute_topk_set, mag_key


def f32(*vals):
    return np.array(vals, dtype=np.float32)


def special_vectors():
    nan = np.float32(np.nan)
    inf = np.float32(np.inf)
    den = np.float32(1e-42)  # denormal
    yield f32(1, 1, 1, 1, 1, 1, 1)                       # all equal
    yield f32(0.0, -0.0, 0.0, -0.0, 0.0)                  # mixed signed zeros
    yield f32(1, 2, 3, 4, 5, 6, 7, 8)                     # increasing
    yield f32(8, 7, 6, 5, 4, 3, 2, 1)                     # decreasing
    yield f32(2, -2, 2, -2, 1, -1, 3, -3, 3)              # equal magnitudes, opposite signs
    yield f32(1, nan, 3, -inf, 2, inf, 0)                 # NaN > Inf > finite
    yield np.array([1.0, -np.nan, np.inf], np.float32)    # negative NaN still largest
    yield f32(den, 0, -den, 2 * den, 0, 1e-38, -0.0)      # denormals kept, not flushed
    yield f32(5)                                          # d = 1
    yield f32(-1, 1)                                      # d = 2 tie


@pytest.mark.parametrize("x", list(special_vectors()))
def test_brute_force_special(oracle, x):
    d = x.shape[0]
    for K in range(d + 1):
        idx, val, res = oracle.topk(x.copy(), K)
        assert list(idx) == brute_topk_set(x, K)
        assert np.array_equal(val.view(np.uint32), x[idx].view(np.uint32))


def test_brute_force_random_with_ties(oracle):
    rng = np.random.default_rng(7)
    for trial in range(150):
        d = int(rng.integers(1, 13))
        # few distinct magnitudes -> many ties, random signs
        x = (rng.integers(0, 4, size=d) * rng.choice([-1.0, 1.0], size=d)).astype(np.float32)
        if trial % 3 == 0:
            x = rng.standard_normal(d).astype(np.float32)
        K = int(rng.integers(0, d + 1))
        idx, val, res = oracle.topk(x.copy(), K)
        assert list(idx) == brute_topk_set(x, K), (x, K)


def check_invariants(x, K, idx, val, res):
    d = x.shape[0]
    # nnz == K, indices strictly ascending and in range
    assert idx.shape[0] == K
    if K:
        assert np.all(np.diff(idx.astype(np.int64)) > 0)
        assert int(idx[-1]) < d
    # sent values are the input bits at those positions
    assert np.array_equal(val.view(np.uint32), x[idx].view(np.uint32))
    # residual + sent == input exactly: residual is +0 at sent positions, input elsewhere
    sent = np.zeros(d, np.float32)
    sent[idx] = val
    assert np.all(res.view(np.uint32)[idx] == 0)
    mask = np.ones(d, bool)
    mask[idx] = False
    assert np.array_equal(res.view(np.uint32)[mask], x.view(np.uint32)[mask])
    finite = np.isfinite(x)
    assert np.array_equal((res + sent)[finite], x[finite])
    # min |sent| >= max |residual|
    if 0 < K < d:
        assert mag_key(val).min() >= mag_key(res).max()


@pytest.mark.parametrize("d,K", [(1000, 1), (1000, 10), (4097, 33), (65536, 66), (100003, 1001),
                                 (5000, 0), (5000, 5000), (5000, 4999)])
def test_invariants_and_lexsort(oracle, d, K):
    rng = np.random.default_rng(d * 31 + K)
    x = rng.standard_normal(d).astype(np.float32)
    # inject duplicated magnitudes with both signs so that ties are exercised
    dup = rng.integers(0, d, size=d // 10)
    src = rng.integers(0, d, size=d // 10)
    x[dup] = np.abs(x[src]) * rng.choice([-1.0, 1.0], size=dup.shape[0]).astype(np.float32)
    idx, val, res = oracle.topk(x.copy(), K)
    check_invariants(x, K, idx, val, res)
    # library routine: lexsort by (magnitude descending, index ascending)
    key = mag_key(x).astype(np.int64)
    order = np.lexsort((np.arange(d), -key))
    expect = np.sort(order[:K]).astype(np.uint32)
    assert np.array_equal(idx, expect)


def test_tie_rule_lower_index_wins(oracle):
    # three distinct magnitudes, the K-th falls inside a long run of equal values
    d = 3000
    x = np.empty(d, np.float32)
    x[0::3] = 1.0
    x[1::3] = -2.0
    x[2::3] = 3.0
    K = 1000 + 1000 + 137        # all 3's, all 2's, and the first 137 of the 1's
    idx, val, res = oracle.topk(x.copy(), K)
    ones = idx[np.abs(val) == 1.0]
    assert ones.shape[0] == 137
    assert np.array_equal(ones, np.arange(0, 3 * 137, 3).astype(np.uint32))
    check_invariants(x, K, idx, val, res)


def test_contraction_bound(oracle):
    """|Top_K(w) - w|^2 <= (d - K)/d |w|^2  (the paper's Eq. "topk_bound")."""
    rng = np.random.default_rng(3)
    for d, K in [(10, 3), (1000, 1), (1000, 500), (50890, 51), (29034, 30)]:
        for dist in ("normal", "laplace", "const"):
            if dist == "normal":
                x = rng.standard_normal(d)
            elif dist == "laplace":
                x = rng.laplace(size=d)
            else:
                x = np.ones(d)
            x = x.astype(np.float32)
            idx, val, res = oracle.topk(x, K)
            lhs = np.sum(res.astype(np.float64) ** 2)
            rhs = (d - K) / d * np.sum(x.astype(np.float64) ** 2)
            assert lhs <= rhs * (1 + 1e-12)


def test_k_rule_matches_paper_sizes():
    """K = d - floor((1 - 0.001) d) for the model sizes the paper's experiments list."""
    from workloads import k_from_fraction
    sizes = {50890: 51, 1199882: 1200, 242762: 243, 29034: 30, 20040522: 20041}
    for d, K in sizes.items():
        assert k_from_fraction(d, 1, 1000) == K
        assert d - int(np.floor((1 - 0.001) * d)) == K
    assert k_from_fraction(1 << 20, 1, 1000) == 1049


def test_bad_arguments(oracle):
    with pytest.raises(ValueError):
        oracle.topk(np.zeros(4, np.float32), 5)

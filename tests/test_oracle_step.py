"""Pins for the oracle's whole step (Algorithm 2), CPU only.

Pins: single-rounding multiply-adds checked against exact rational arithmetic;
K_up = K_dn = d reduces to the dense SGD iteration (Eq. 2); K_dn = d reduces to
Algorithm 1 (server residual identically zero, downlink = whole aggregate); the
conservation identity of Lemma 1 (bit-exact on dyadic inputs, to rounding on
random ones); the bound "at most K_uplink * N non-zero indices" of the
communication section; identical workers aggregate back to one worker's message.
"""
from fractions import Fraction

import numpy as np
import pytest


def round_f32(x: Fraction) -> np.float32:
    """Round an exact rational to the nearest fp32 (ties to even), normal range only."""
    if x == 0:
        return np.float32(0.0)
    s = -1 if x < 0 else 1
    x = abs(x)
    e = 0
    while x >= 2:
        x /= 2
        e += 1
    while x < 1:
        x *= 2
        e -= 1
    assert -126 <= e <= 127
    m = x * (1 << 23)                      # in [2^23, 2^24)
    fl = m.numerator // m.denominator
    rem = m - fl
    if rem > Fraction(1, 2) or (rem == Fraction(1, 2) and (fl & 1)):
        fl += 1
    return np.float32(s * float(fl) * 2.0 ** (e - 23))


def fma_exact(a, b, c) -> np.float32:
    return round_f32(Fraction(float(a)) * Fraction(float(b)) + Fraction(float(c)))


def bits(a):
    return np.ascontiguousarray(a).view(np.uint32)


def test_round_helper_is_sane():
    rng = np.random.default_rng(0)
    for v in rng.standard_normal(200).astype(np.float32):
        assert round_f32(Fraction(float(v))) == v
    # a case where fused and unfused differ
    a, b, c = np.float32(0.01), np.float32(3.0000002), np.float32(1e-9)
    assert fma_exact(a, b, c) == np.float32(np.float64(a) * np.float64(b) + np.float64(c))


def test_every_multiply_add_is_one_rounding(oracle):
    """Non-dyadic alpha and p: the three multiply-adds of the step must each equal the
    exactly rounded a*b + c, which an unfused multiply followed by an add does not."""
    rng = np.random.default_rng(11)
    N, d = 3, 64
    g = rng.standard_normal((N, d)).astype(np.float32)
    eps = (rng.standard_normal((N, d)) * 0.01).astype(np.float32)
    delta = (rng.standard_normal(d) * 0.001).astype(np.float32)
    w = rng.standard_normal(d).astype(np.float32)
    p = np.array([0.2, 0.5, 0.3], np.float32)
    alpha_in, alpha_out = np.float32(0.01), np.float32(0.7)
    g0, eps0, delta0, w0 = g.copy(), eps.copy(), delta.copy(), w.copy()
    out = oracle.bidir_step(g, eps, delta, w, p, d, d, float(alpha_in), float(alpha_out))
    # with K = d every coordinate is sent both ways, so each output is a pure fma chain
    differs = 0
    for i in range(d):
        acc = delta0[i]
        for q in range(N):
            a = fma_exact(alpha_in, g0[q, i], eps0[q, i])
            unf = np.float32(np.float32(alpha_in * g0[q, i]) + eps0[q, i])
            differs += int(unf != a)
            assert bits(out["up_val"][q, i:i + 1])[0] == bits(np.array([a]))[0]
            acc = fma_exact(p[q], a, acc)
        assert bits(out["dn_val"][i:i + 1])[0] == bits(np.array([acc]))[0]
        wi = fma_exact(-alpha_out, acc, w0[i])
        assert bits(w[i:i + 1])[0] == bits(np.array([wi]))[0]
    assert differs > 0, "inputs must discriminate fused from unfused"


def test_full_k_is_dense_sgd(oracle):
    """K_up = K_dn = d: w_t = w_{t-1} - alpha * sum_q p_q g^q (Eq. 2), residuals stay zero."""
    rng = np.random.default_rng(5)
    N, d = 4, 500
    p = np.full(N, 0.25, np.float32)
    alpha = 0.125
    w = rng.integers(-64, 64, d).astype(np.float32)
    w_ref = w.astype(np.float64).copy()
    eps = np.zeros((N, d), np.float32)
    delta = np.zeros(d, np.float32)
    for t in range(5):
        g = rng.integers(-16, 17, (N, d)).astype(np.float32)      # dyadic: all ops exact
        out = oracle.bidir_step(g, eps, delta, w, p, d, d, alpha, 1.0)
        w_ref -= alpha * (p.astype(np.float64)[:, None] * g.astype(np.float64)).sum(0)
        assert np.array_equal(w.astype(np.float64), w_ref)
        assert not eps.view(np.uint32).any() and not delta.view(np.uint32).any()
        assert np.array_equal(out["dn_idx"], np.arange(d, dtype=np.uint32))
    # generic (rounded) inputs: agreement to fp32 rounding
    w = rng.standard_normal(d).astype(np.float32)
    w_ref = w.astype(np.float64).copy()
    g = rng.standard_normal((N, d)).astype(np.float32)
    oracle.bidir_step(g, eps, delta, w, p, d, d, 0.01, 1.0)
    w_ref -= 0.01 * (0.25 * g.astype(np.float64)).sum(0)
    assert np.allclose(w, w_ref, rtol=0, atol=1e-6)


def test_full_downlink_is_algorithm_1(oracle):
    """K_dn = d: delta stays zero and the model moves by the whole aggregate
    sum_q p_q Top_K(a^q), i.e. unidirectional Top_K SGD."""
    rng = np.random.default_rng(6)
    N, d, K = 5, 2000, 20
    p = rng.dirichlet(np.ones(N)).astype(np.float32)
    w = rng.standard_normal(d).astype(np.float32)
    eps = np.zeros((N, d), np.float32)
    delta = np.zeros(d, np.float32)
    for t in range(4):
        g = rng.standard_normal((N, d)).astype(np.float32)
        a = eps.astype(np.float64) + 0.05 * g.astype(np.float64)
        w_prev = w.astype(np.float64).copy()
        out = oracle.bidir_step(g, eps, delta, w, p, K, d, 0.05, 1.0)
        assert not delta.view(np.uint32).any()
        agg = np.zeros(d)
        for q in range(N):
            # each worker's message is its K largest |a| (random data: no ties)
            top = np.sort(np.argsort(-np.abs(a[q]), kind="stable")[:K])
            assert np.array_equal(out["up_idx"][q], top.astype(np.uint32))
            np.add.at(agg, top, float(p[q]) * out["up_val"][q].astype(np.float64))
        assert np.allclose(w_prev - w, agg, rtol=0, atol=1e-6)
        assert out["union_nnz"] <= N * K
        assert out["union_nnz"] == np.count_nonzero(agg)


def lemma1_sides(w, eps, delta, p):
    lhs = (w.astype(np.float64) - (p.astype(np.float64)[:, None] * eps.astype(np.float64)).sum(0)
           - delta.astype(np.float64))
    return lhs


def test_lemma1_conservation_exact_on_dyadic_inputs(oracle):
    """w~_t = w_t - sum_q p_q eps_t^q - delta_t satisfies w~_t = w~_{t-1} - alpha sum_q p_q g^q
    (Lemma 1).  With small-integer g, p_q = 1/4 and alpha = 1/8 no operation rounds, so the
    identity must hold exactly whatever Top_K selects."""
    rng = np.random.default_rng(8)
    N, d, K_up, K_dn = 4, 1000, 7, 5
    p = np.full(N, 0.25, np.float32)
    alpha = 0.125
    w = rng.integers(-32, 32, d).astype(np.float32)
    eps = np.zeros((N, d), np.float32)
    delta = np.zeros(d, np.float32)
    wt = lemma1_sides(w, eps, delta, p)
    for t in range(12):
        g = rng.integers(-8, 9, (N, d)).astype(np.float32)
        oracle.bidir_step(g, eps, delta, w, p, K_up, K_dn, alpha, 1.0)
        wt = wt - alpha * (0.25 * g.astype(np.float64)).sum(0)
        assert np.array_equal(lemma1_sides(w, eps, delta, p), wt)


def test_lemma1_conservation_random_inputs(oracle):
    rng = np.random.default_rng(9)
    N, d, K_up, K_dn = 6, 5000, 50, 25
    p = rng.dirichlet(np.ones(N)).astype(np.float32)
    w = rng.standard_normal(d).astype(np.float32)
    eps = np.zeros((N, d), np.float32)
    delta = np.zeros(d, np.float32)
    wt = lemma1_sides(w, eps, delta, p)
    for t in range(10):
        alpha = 0.1 / (t + 1) ** 0.6            # a decaying step-size sequence
        g = rng.standard_normal((N, d)).astype(np.float32)
        oracle.bidir_step(g, eps, delta, w, p, K_up, K_dn, alpha, 1.0)
        wt = wt - np.float64(np.float32(alpha)) * (p.astype(np.float64)[:, None]
                                                   * g.astype(np.float64)).sum(0)
        assert np.allclose(lemma1_sides(w, eps, delta, p), wt, rtol=0, atol=2e-5)


def test_identical_workers_aggregate_to_one_message(oracle):
    rng = np.random.default_rng(10)
    d, K = 3000, 40
    row = rng.standard_normal(d).astype(np.float32)
    for N in (2, 4):
        g = np.tile(row if N == 2 else np.round(row * 64) / 64, (N, 1)).astype(np.float32)
        eps = np.zeros((N, d), np.float32)
        delta = np.zeros(d, np.float32)
        w = np.zeros(d, np.float32)
        p = np.full(N, 1.0 / N, np.float32)
        out = oracle.bidir_step(g, eps, delta, w, p, K, K, 1.0, 1.0)
        for q in range(1, N):
            assert np.array_equal(out["up_idx"][q], out["up_idx"][0])
        assert out["union_nnz"] == K
        assert np.array_equal(out["dn_idx"], out["up_idx"][0])
        assert np.array_equal(bits(out["dn_val"]), bits(out["up_val"][0]))


def test_step_equals_its_stages(oracle):
    rng = np.random.default_rng(12)
    N, d, K_up, K_dn = 3, 4000, 17, 9
    g = rng.standard_normal((N, d)).astype(np.float32)
    p = rng.dirichlet(np.ones(N)).astype(np.float32)
    eps = (rng.standard_normal((N, d)) * 0.1).astype(np.float32)
    delta = (rng.standard_normal(d) * 0.01).astype(np.float32)
    w = rng.standard_normal(d).astype(np.float32)
    e2, d2, w2 = eps.copy(), delta.copy(), w.copy()
    out = oracle.bidir_step(g, eps, delta, w, p, K_up, K_dn, 0.3, 0.9)
    ui, uv = oracle.worker_stage(g, e2, 0.3, K_up, nthreads=1)
    nnz = oracle.aggregate(ui, uv, p, d2)
    di, dv = oracle.downlink(d2, K_dn)
    oracle.update(di, dv, 0.9, w2)
    for a, b in ((out["up_idx"], ui), (out["dn_idx"], di)):
        assert np.array_equal(a, b)
    for a, b in ((out["up_val"], uv), (out["dn_val"], dv), (eps, e2), (delta, d2), (w, w2)):
        assert np.array_equal(bits(a), bits(b))
    assert out["union_nnz"] == nnz


def test_untouched_coordinates_keep_delta_bits(oracle):
    """Coordinates no uplink names keep the server residual bit for bit (including -0)."""
    d = 64
    delta = np.full(d, -0.0, np.float32)
    up_idx = np.array([[3, 5]], np.uint32)
    up_val = np.array([[1.0, -2.0]], np.float32)
    oracle.aggregate(up_idx, up_val, np.array([0.5], np.float32), delta)
    expect = np.full(d, -0.0, np.float32)
    expect[3], expect[5] = 0.5, -1.0
    assert np.array_equal(bits(delta), bits(expect))


def test_algorithm_1_step_equals_bidirectional_with_full_downlink(oracle):
    """Pin for the unidirectional step: same w and eps as Algorithm 2 with K_dn = d (whose
    server residual stays zero), message = the named coordinates with the aggregate."""
    rng = np.random.default_rng(21)
    N, d, K = 7, 3001, 25
    p = rng.dirichlet(np.ones(N)).astype(np.float32)
    w = rng.standard_normal(d).astype(np.float32)
    w[5], w[6] = 0.0, -0.0
    eps = np.zeros((N, d), np.float32)
    w2, eps2, delta2 = w.copy(), eps.copy(), np.zeros(d, np.float32)
    for t in range(5):
        g = rng.standard_normal((N, d)).astype(np.float32)
        uni = oracle.unidir_step(g, eps, w, p, K, 0.07, 0.9)
        bi = oracle.bidir_step(g, eps2, delta2, w2, p, K, d, 0.07, 0.9)
        assert np.array_equal(bits(w), bits(w2)) and np.array_equal(bits(eps), bits(eps2))
        assert not delta2.view(np.uint32).any()
        assert np.array_equal(uni["up_idx"], bi["up_idx"])
        assert uni["dn_count"] == bi["union_nnz"] <= N * K
        named = np.unique(uni["up_idx"])
        assert np.array_equal(uni["dn_idx"], named.astype(np.uint32))
        assert np.array_equal(bits(uni["dn_val"]), bits(bi["dn_val"][named]))
        # the message is the weighted sum of the uplinks (to rounding)
        ref = np.zeros(d)
        for q in range(N):
            np.add.at(ref, uni["up_idx"][q], float(p[q]) * uni["up_val"][q].astype(np.float64))
        assert np.allclose(uni["dn_val"], ref[named], rtol=0, atol=1e-6)

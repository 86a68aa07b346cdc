"""Pins for the oracle's per-step estimates of rho, rho_hat and 1-gamma (CPU only): the
definitions of Assumptions 2, 5 and 6 written out in numpy fp64 on dyadic inputs (where the
oracle's fp32 chains are exact, so both must agree to fp64 rounding), the degenerate cases
the definitions fix (one worker: rho_hat = 0; K = d: all three are 0), the contraction bound
of Eq. "topk_bound", and that the step itself is unchanged."""
import numpy as np
import pytest


def topk_dense(x, K):
    """Top_K as a dense vector, plain numpy (stable: lower index wins ties)."""
    order = np.argsort(-np.abs(x), kind="stable")[:K]
    out = np.zeros_like(x)
    out[order] = x[order]
    return out


def reference(g, eps, delta, p, alpha, K_up, K_dn):
    g, eps, delta, p = (a.astype(np.float64) for a in (g, eps, delta, p))
    a = eps + alpha * g
    s = (p[:, None] * g).sum(0)
    tops = np.stack([topk_dense(a[q], K_up) for q in range(a.shape[0])])
    m = (p[:, None] * tops).sum(0)
    den = np.linalg.norm(alpha * s)
    rho = np.linalg.norm(topk_dense(delta + (p[:, None] * a).sum(0), K_dn)
                         - topk_dense(delta + m, K_dn)) / den
    rho_hat = np.linalg.norm(topk_dense((p[:, None] * a).sum(0), K_up) - m) / den
    gam_w = [np.sum((a[q] - tops[q]) ** 2) / np.sum(a[q] ** 2) for q in range(a.shape[0])]
    gt = delta + m
    gam_s = np.sum((gt - topk_dense(gt, K_dn)) ** 2) / np.sum(gt ** 2)
    nnz = np.count_nonzero(np.abs(tops).sum(0)) / g.shape[1]
    return rho, rho_hat, gam_w, gam_s, den, nnz


@pytest.mark.parametrize("K_up,K_dn", [(9, 6), (5, 11)])     # either may be the larger one
def test_matches_the_written_out_definitions_on_dyadic_inputs(oracle, K_up, K_dn):
    rng = np.random.default_rng(31)
    N, d = 4, 600
    p = np.full(N, 0.25, np.float32)
    alpha = 0.125
    eps = np.zeros((N, d), np.float32)
    delta = np.zeros(d, np.float32)
    w = np.zeros(d, np.float32)
    for t in range(6):
        # distinct magnitudes (no ties), small dyadic values: every fp32 operation is exact
        g = (rng.permutation(N * d).reshape(N, d) - N * d // 2).astype(np.float32) / 64.0
        want = reference(g, eps, delta, p, alpha, K_up, K_dn)
        e0, d0, w0 = eps.copy(), delta.copy(), w.copy()
        got = oracle.bidir_step_diag(g, eps, delta, w, p, K_up, K_dn, alpha, 1.0)
        plain = oracle.bidir_step(g, e0, d0, w0, p, K_up, K_dn, alpha, 1.0)
        for a, b in ((eps, e0), (delta, d0), (w, w0)):
            assert np.array_equal(a.view(np.uint32), b.view(np.uint32))
        assert np.array_equal(got["dn_idx"], plain["dn_idx"])
        assert np.isclose(got["rho"], want[0], rtol=1e-12, atol=1e-15)
        assert np.isclose(got["rho_hat"], want[1], rtol=1e-12, atol=1e-15)
        assert np.allclose(got["one_minus_gamma_workers"], want[2], rtol=1e-12)
        assert np.isclose(got["one_minus_gamma_server"], want[3], rtol=1e-12)
        assert np.isclose(got["one_minus_gamma_max"], max(max(want[2]), want[3]), rtol=1e-12)
        assert np.isclose(got["denominator"], want[4], rtol=1e-12)
        assert np.isclose(got["nnz_fraction"], want[5], rtol=0, atol=0)
        assert got["rho_hat"] > 0 and got["rho"] >= 0


def test_degenerate_cases(oracle):
    rng = np.random.default_rng(32)
    d = 500
    # one worker with weight 1 and no server residual: Top_K(sum) is the worker's own message
    g = rng.standard_normal((1, d)).astype(np.float32)
    out = oracle.bidir_step_diag(g, np.zeros((1, d), np.float32), np.zeros(d, np.float32),
                                 np.zeros(d, np.float32), np.ones(1, np.float32), 20, 20, 0.5, 1.0)
    assert out["rho_hat"] == 0.0 and out["rho"] == 0.0
    assert 0.0 < out["one_minus_gamma_max"] <= (d - 20) / d
    # K = d: nothing is dropped anywhere
    N = 3
    g = rng.standard_normal((N, d)).astype(np.float32)
    p = rng.dirichlet(np.ones(N)).astype(np.float32)
    out = oracle.bidir_step_diag(g, np.zeros((N, d), np.float32), np.zeros(d, np.float32),
                                 np.zeros(d, np.float32), p, d, d, 0.1, 1.0)
    assert out["rho"] == 0.0 and out["rho_hat"] == 0.0 and out["one_minus_gamma_max"] == 0.0
    assert out["nnz_fraction"] == 1.0


def test_contraction_bound_on_random_steps(oracle):
    """1 - gamma <= (d - K)/d for every compression (Eq. "topk_bound")."""
    rng = np.random.default_rng(33)
    N, d, K_up, K_dn = 5, 4000, 40, 20
    p = rng.dirichlet(np.ones(N)).astype(np.float32)
    eps = np.zeros((N, d), np.float32)
    delta = np.zeros(d, np.float32)
    w = np.zeros(d, np.float32)
    for t in range(4):
        g = rng.standard_normal((N, d)).astype(np.float32)
        want = reference(g, eps, delta, p, np.float32(0.05), K_up, K_dn)
        out = oracle.bidir_step_diag(g, eps, delta, w, p, K_up, K_dn, 0.05, 1.0)
        assert np.all(out["one_minus_gamma_workers"] <= (d - K_up) / d)
        assert out["one_minus_gamma_server"] <= (d - K_dn) / d
        # random fp32 data: the fp64 definitions agree to fp32 rounding of the chains
        assert np.isclose(out["rho"], want[0], rtol=1e-3)
        assert np.isclose(out["rho_hat"], want[1], rtol=1e-3)
        assert np.isclose(out["denominator"], want[4], rtol=1e-5)

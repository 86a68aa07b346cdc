"""The paper's worked example (Appendix, "Toy Example") run through the oracle.

Three workers minimise F(w) = 1/3 sum_q 1/2 |w - c_q|^2, c = (1, 5, 10), d = 100,
K = 1, alpha = 0.01, w_0 ~ N(20, 1) drawn with "random seed 10".  The gradients are
closed form (g^q = w - c_q).  The paper prints two norms observed in the
unidirectional run "at t = 210" and the optimum F* = 6100/9 at w = 16/3.

Reading used here: the seeded draw is numpy's legacy global generator
(``np.random.seed(10); np.random.normal(20, 1, 100)``), the state is fp32, and
"t = 210" counts iterations from zero (the 211th pass through the loop).  With
that reading both printed norms come out to the two decimals the paper gives.
"""
import os

import numpy as np

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "toy_example.txt")
CENTRES = np.array([1.0, 5.0, 10.0], np.float32)


def golden():
    vals = {}
    with open(GOLDEN) as fh:
        for line in fh:
            if line.startswith("#") or not line.strip():
                continue
            k, v = line.split()
            vals[k] = float(v)
    return vals


def loss(w):
    w = w.astype(np.float64)
    return sum(0.5 * np.sum((w - c) ** 2) for c in CENTRES.astype(np.float64)) / 3.0


def run(oracle, steps, K_dn, observe_at=None):
    N, d, alpha = 3, 100, 0.01
    np.random.seed(10)
    w = np.random.normal(20, 1, d).astype(np.float32)
    eps = np.zeros((N, d), np.float32)
    delta = np.zeros(d, np.float32)
    p = np.full(N, 1.0 / 3.0, np.float32)
    seen, losses = None, []
    for t in range(steps):
        g = (w[None, :] - CENTRES[:, None]).astype(np.float32)
        a = eps.astype(np.float64) + alpha * g.astype(np.float64)
        out = oracle.bidir_step(g, eps, delta, w, p, 1, K_dn, alpha, 1.0)
        if t == observe_at:
            sum_a = a.sum(0)
            sum_top = np.zeros(d)
            for q in range(N):
                sum_top[out["up_idx"][q]] += out["up_val"][q]
            top_of_sum = np.zeros(d)
            j = np.argmax(np.abs(sum_top))
            top_of_sum[j] = sum_top[j]
            seen = (np.linalg.norm(sum_a - sum_top), np.linalg.norm(sum_a - top_of_sum))
        losses.append(loss(w))
    return seen, np.array(losses)


def test_printed_norms_of_the_unidirectional_run(oracle):
    gold = golden()
    (n_up, n_bi), _ = run(oracle, 211, K_dn=100, observe_at=210)
    assert round(n_up, 2) == gold["norm_uplink"]
    assert round(n_bi, 2) == gold["norm_bidirectional"]
    assert n_bi < n_up       # the appendix's point: the downlink Top_K lands closer


def test_closed_form_optimum_bounds_both_runs(oracle):
    gold = golden()
    f_star = gold["optimum_value_num"] / gold["optimum_value_den"]
    w_star = np.full(100, gold["optimum_w_num"] / gold["optimum_w_den"])
    assert abs(loss(w_star) - f_star) < 1e-9
    _, uni = run(oracle, 400, K_dn=100)
    _, bi = run(oracle, 400, K_dn=1)
    assert uni.min() >= f_star and bi.min() >= f_star
    # both runs descend from F(w_0) ~ 1e4 to a neighbourhood of F* and stay there
    assert uni[-100:].max() < 1.1 * f_star and bi[-100:].max() < 1.1 * f_star

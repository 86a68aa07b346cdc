"""Randomised GPU parity sweep: shapes, K, value distributions and select paths drawn from a
seeded generator; two steps of bidir_step per case, every output bit for bit against the
oracle.  Covers what the hand-picked cases may miss: odd N, K_up != K_dn up to d, rows of
zeros, constant rows, mostly-zero rows, few-valued rows, infinities and denormals."""
import numpy as np
import pytest
import torch

pytestmark = pytest.mark.gpu


def draw_rows(rng, kind, N, d):
    if kind == "normal":
        return rng.standard_normal((N, d)).astype(np.float32)
    if kind == "heavy":
        return (rng.standard_t(2, size=(N, d)) * 1e-3).astype(np.float32)
    if kind == "levels":
        lv = rng.integers(1, 5)
        return (rng.integers(0, lv + 1, size=(N, d)) * rng.choice([-1.0, 1.0], size=(N, d))
                ).astype(np.float32)
    if kind == "quantized":
        return (np.round(rng.standard_normal((N, d)) * 16) / 16).astype(np.float32)
    if kind == "sparse":
        g = rng.standard_normal((N, d)).astype(np.float32)
        g[rng.random((N, d)) < 0.9] = 0.0
        return g
    if kind == "constant":
        return np.full((N, d), np.float32(rng.choice([-2.5, 0.0, 1e-3])), np.float32)
    if kind == "extremes":
        g = rng.standard_normal((N, d)).astype(np.float32)
        m = rng.random((N, d))
        g[m < 0.01] = np.inf
        g[(m >= 0.01) & (m < 0.02)] = -np.inf
        g[(m >= 0.02) & (m < 0.10)] = 1e-42
        g[(m >= 0.10) & (m < 0.12)] = 3e38
        return g
    raise ValueError(kind)


KINDS = ["normal", "heavy", "levels", "quantized", "sparse", "constant", "extremes"]


@pytest.mark.parametrize("seed", range(48))
def test_random_case(oracle, seed):
    import _gpu_util as G
    rng = np.random.default_rng(1000 + seed)
    N = int(rng.integers(1, 13))
    d = int(np.exp(rng.uniform(np.log(1), np.log(400_000))))
    if seed % 4 == 0:
        d = max(d, 70_000)                       # make the single-pass path reachable
    def draw_k():
        u = rng.random()
        if u < 0.15:
            return d
        if u < 0.6:
            return int(rng.integers(1, max(2, d // 64 + 1)))
        return int(rng.integers(1, d + 1))
    K_up, K_dn = draw_k(), draw_k()
    kind = KINDS[seed % len(KINDS)]
    path = int(rng.integers(0, 3))
    if seed % 5 == 4:
        path = 3                                 # the three-launch select where the shape allows
    alpha = float(rng.choice([1.0, 0.5, 0.01, 0.37]))
    a_out = float(rng.choice([1.0, 0.3]))
    p = rng.dirichlet(np.ones(N)).astype(np.float32)
    w0 = rng.standard_normal(d).astype(np.float32)
    st = G.GpuState(N, d, K_up, K_dn, w0, p)
    st.ctx.set_path(path)
    tag = f"seed {seed}: N={N} d={d} K_up={K_up} K_dn={K_dn} {kind} path={path}"
    for t in range(2):
        g = draw_rows(rng, kind if t == 0 else KINDS[(seed + 3) % len(KINDS)], N, d)
        if kind == "extremes" or (t == 1 and KINDS[(seed + 3) % len(KINDS)] == "extremes"):
            # inf - inf would make NaN, whose payload after a multiply-add is not compared
            g = np.where(np.isinf(g), np.float32(3e38), g).astype(np.float32) if t == 1 else g
        st.step_and_compare(oracle, torch.from_numpy(g).to(G.dev()), alpha, a_out,
                            f"{tag} step {t}")


@pytest.mark.parametrize("seed", range(24))
def test_random_case_over_several_steps(oracle, seed):
    """Five steps on one context with the kind of gradient changing from step to step, on
    shapes the single-pass select serves: from its third call on that select starts from the
    bounds of the call before, which here belong to another distribution every time (lists
    that overflow or fall short, early zeros to take back, rows redone by the dense path and
    picked up again).  Every output of every step bit for bit against the oracle."""
    import _gpu_util as G
    rng = np.random.default_rng(5000 + seed)
    N = int(rng.integers(1, 9))
    d = int(np.exp(rng.uniform(np.log(66_000), np.log(500_000))))
    K_up = int(rng.integers(1, d // 64 + 1))
    K_dn = int(rng.integers(1, d // 64 + 1)) if seed % 3 else int(rng.integers(1, d + 1))
    path = 2 if seed % 4 else 0
    alpha = float(rng.choice([1.0, 0.5, 0.01, 0.37]))
    a_out = float(rng.choice([1.0, 0.3]))
    p = rng.dirichlet(np.ones(N)).astype(np.float32)
    w0 = rng.standard_normal(d).astype(np.float32)
    st = G.GpuState(N, d, K_up, K_dn, w0, p)
    st.ctx.set_path(path)
    tag = f"seed {seed}: N={N} d={d} K_up={K_up} K_dn={K_dn} path={path}"
    same_kind = seed % 2 == 0                    # half the cases keep one distribution
    for t in range(5):
        kind = KINDS[seed % len(KINDS)] if same_kind else KINDS[(seed + 3 * t) % len(KINDS)]
        g = draw_rows(rng, kind, N, d)
        if t > 0:                                # inf - inf would make NaN (payload not compared)
            g = np.where(np.isinf(g), np.float32(3e38), g).astype(np.float32)
        if same_kind and kind == "normal":
            g *= np.float32(1.0 + 0.2 * t)       # a drifting scale
        st.step_and_compare(oracle, torch.from_numpy(g).to(G.dev()), alpha, a_out,
                            f"{tag} step {t} ({kind})")

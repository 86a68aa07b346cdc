"""Host checks of the seeded input generators and the config table (CPU only)."""
import numpy as np
import torch

import workloads as wl


def splitmix_reference(key, i):
    """SplitMix64's output mix on Python integers, for one counter."""
    m = (1 << 64) - 1
    z = (key + i * 0x9E3779B97F4A7C15) & m
    z = ((z ^ (z >> 30)) * 0xBF58476D1CE4E5B9) & m
    z = ((z ^ (z >> 27)) * 0x94D049BB133111EB) & m
    return z ^ (z >> 31)


def test_hash_bits_match_python_integers():
    key = wl.stream_key(123, 4, 5)
    z = wl.hash_bits(key, 1000, 16, "cpu").numpy().view(np.uint64)
    for j in range(16):
        assert int(z[j]) == splitmix_reference(key, 1000 + j)


def test_config_table():
    c = wl.CONFIGS
    assert (c["C1"].N, c["C1"].d, c["C1"].K_up, c["C1"].K_dn) == (4, 1 << 20, 1049, 1049)
    assert (c["C2"].N, c["C2"].d, c["C2"].K_up) == (16, 11_173_962, 111_740)
    assert (c["C3"].N, c["C3"].K_up, c["C3"].K_dn) == (32, 25_558, 25_558)
    assert (c["C4"].N, c["C4"].K_up, c["C4"].K_dn) == (64, 25_558, 12_779)
    assert (c["C5"].N, c["C5"].d, c["C5"].K_up, c["C5"].K_dn) == (64, 110_000_000, 11_000, 11_000)


def test_draws_are_reproducible_and_distinct():
    cfg = wl.CONFIGS["C1"].scaled(50_000)
    src = wl.GradientSource(cfg, "cpu")
    a, b = src.step(1), src.step(1)
    assert torch.equal(a, b)
    assert not torch.equal(a, src.step(2))
    assert not torch.equal(a[0], a[1])
    assert wl.checksum(a) == wl.checksum(b)


def test_distributions_have_the_stated_scale():
    d = 200_000
    g = wl.GradientSource(wl.CONFIGS["C1"].scaled(d), "cpu").row(1, 0)
    assert abs(g.mean().item()) < 0.02 and abs(g.std().item() - 1.0) < 0.02
    g = wl.GradientSource(wl.CONFIGS["C2"].scaled(d), "cpu").step(1)
    assert abs(g.var().item() - 2e-3) < 2e-4            # shared + own component
    c = np.corrcoef(g[0].numpy(), g[1].numpy())[0, 1]
    assert 0.4 < c < 0.6                                 # the shared half
    g = wl.GradientSource(wl.CONFIGS["C3"].scaled(d), "cpu").row(1, 0)
    assert abs(g.abs().mean().item() - 1e-3) < 5e-5      # Laplace: E|x| = b
    cfg4 = wl.CONFIGS["C4"].scaled(d)
    g = wl.GradientSource(cfg4, "cpu").row(1, 0)
    key = g.abs().numpy().view(np.uint32)
    dup_frac = 1.0 - np.unique(key).shape[0] / d
    assert 0.03 < dup_frac < 0.08                        # about 5 % duplicated magnitudes
    p = wl.p_weights(cfg4)
    assert p.shape == (64,) and abs(p.sum() - 1.0) < 1e-5 and p.min() > 0
    cfg5 = wl.CONFIGS["C5"].scaled(d)
    g = wl.GradientSource(cfg5, "cpu").row(1, 0)
    lg = np.log10(g.abs().numpy() + 1e-30)
    assert lg.max() > -2.5 and np.median(lg) < -2.0      # several decades of scale
    w = wl.weights0(cfg5, "cpu")
    assert abs(w.std().item() - 0.1) < 0.005


def test_transforms_are_finite_at_the_extreme_counters():
    ext = torch.tensor([0, -1, 1 << 62, -(1 << 63), (1 << 63) - 1, 1 << 40, (1 << 40) - 1],
                       dtype=torch.int64)
    for f in (wl.normal_from_bits, wl.laplace_from_bits, wl.student_t2_from_bits):
        v = f(ext)
        assert bool(torch.isfinite(v).all()), f.__name__
    # and over a large sweep of the top bits
    hi = (torch.arange(0, 1 << 24, 7, dtype=torch.int64) << 40)
    for f in (wl.normal_from_bits, wl.laplace_from_bits, wl.student_t2_from_bits):
        assert bool(torch.isfinite(f(hi)).all()), f.__name__
        assert bool(torch.isfinite(f(hi | ((1 << 40) - 1))).all()), f.__name__

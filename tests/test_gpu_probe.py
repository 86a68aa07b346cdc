"""The HBM probe kernels (libbts_probe.so, a measurement instrument of its own): they do what
their kinds say, at every occupancy setting."""
import numpy as np
import pytest
import torch

pytestmark = pytest.mark.gpu


def test_hbm_probe_kinds():
    import paper_2209_15203_amd as bts
    assert torch.cuda.is_available(), "these tests need the MI355X"
    dev = torch.device("cuda:0")
    n = 512 * 1000 + 300                      # whole 512-float chunks only: a tail stays untouched
    whole = n // 512 * 512
    rng = np.random.default_rng(5)
    src = torch.from_numpy(rng.standard_normal(n).astype(np.float32)).to(dev)
    dst0 = torch.from_numpy(rng.standard_normal(n).astype(np.float32)).to(dev)
    from paper_2209_15203_amd import binding
    for waves, by_regs in ((0, False), (12, False), (12, True), (20, True), (24, False)):
        # read: nothing is written
        dst = dst0.clone()
        ms = binding.hbm_probe(0, src, dst, waves, by_regs, repeats=2)
        assert ms > 0.0
        assert torch.equal(dst, dst0)
        # copy
        ms = binding.hbm_probe(1, src, dst, waves, by_regs, repeats=2)
        assert ms > 0.0
        assert torch.equal(dst[:whole], src[:whole]) and torch.equal(dst[whole:], dst0[whole:])
        # fma-stream: one untimed launch and one timed launch = two applications of
        # dst = fma(0.5, src, dst); 0.5 * src is exact, so each is one rounded addition
        dst = dst0.clone()
        binding.hbm_probe(2, src, dst, waves, by_regs, repeats=1)
        want = dst0.clone()
        for _ in range(2):
            want[:whole] = want[:whole] + 0.5 * src[:whole]
        assert torch.equal(dst, want)
    with pytest.raises(bts.BtsError):
        binding.hbm_probe(3, src, dst)
    with pytest.raises(bts.BtsError):
        binding.hbm_probe(2, src, dst, waves_per_cu=13)

"""GPU parity on the paper's own workload shapes (experiments section): model sizes
d in {29,034; 50,890; 242,762; 1,199,882; 20,040,522}, N in {20, 50, 100} workers,
K = d - floor(0.999 d) both ways, p_q = 1/N (not a power of two, so a fused and an
unfused multiply-add differ).  Synthetic gradients stand in for the training runs; four
steps with carried residuals (from the third on the single-pass select starts from the
bounds of the step before), every output bit for bit against the oracle.

Also the appendix toy example (N = 3, d = 100, K = 1, closed-form gradients that depend
on w) stepped through the GPU library for 300 iterations in both the bidirectional and the
unidirectional (K_dn = d) form.
"""
import numpy as np
import pytest
import torch

import workloads as wl

pytestmark = pytest.mark.gpu

PAPER_D = [29_034, 50_890, 242_762, 1_199_882, 20_040_522]


def shapes():
    for d in PAPER_D:
        for N in (20, 50, 100):
            if d > 2_000_000 and N > 20:        # the paper trains its largest model on 20 workers only
                continue
            yield N, d


@pytest.mark.timeout(600)
@pytest.mark.parametrize("N,d", list(shapes()))
def test_paper_shape(oracle, N, d):
    import _gpu_util as G
    K = wl.k_from_fraction(d, 1, 1000)
    cfg = wl.Config(f"paper-d{d}-N{N}", 100 + N, N, d, K, K, 4, "normal")
    src = wl.GradientSource(cfg, G.dev())
    p = np.full(N, 1.0 / N, np.float32)
    st = G.GpuState(N, d, K, K, wl.weights0(cfg, "cpu").numpy(), p)
    for t in (1, 2, 3, 4):
        st.step_and_compare(oracle, src.step(t), 0.05, 1.0, f"{cfg.name} step {t}")


CENTRES = np.array([1.0, 5.0, 10.0], np.float32)


@pytest.mark.parametrize("K_dn", [1, 100])
def test_toy_example_on_the_gpu(oracle, K_dn):
    """w feeds back into the gradients here, so any one-bit difference would grow; the GPU
    trajectory must equal the oracle's for all 300 iterations.  K_dn = 100 = d is the
    unidirectional algorithm."""
    import _gpu_util as G
    import paper_2209_15203_amd as bts
    N, d, alpha = 3, 100, 0.01
    np.random.seed(10)
    w0 = np.random.normal(20, 1, d).astype(np.float32)
    D = G.dev()
    c = torch.from_numpy(CENTRES).to(D)
    ctx = bts.BtsContext(N, d, 1, K_dn)
    eps = torch.zeros((N, d), device=D)
    delta = torch.zeros(d, device=D)
    w = torch.from_numpy(w0.copy()).to(D)
    p = torch.full((N,), 1.0 / 3.0, device=D)
    ui = torch.zeros((N, 1), dtype=torch.int32, device=D)
    uv = torch.zeros((N, 1), device=D)
    di = torch.zeros(K_dn, dtype=torch.int32, device=D)
    dv = torch.zeros(K_dn, device=D)
    h_eps = np.zeros((N, d), np.float32)
    h_delta = np.zeros(d, np.float32)
    h_w = w0.copy()
    h_p = np.full(N, 1.0 / 3.0, np.float32)
    for t in range(300):
        g = w[None, :] - c[:, None]                         # exact in fp32 on both sides
        h_g = (h_w[None, :] - CENTRES[:, None]).astype(np.float32)
        if t == 210 and K_dn == d:
            a = eps.double().cpu().numpy() + alpha * g.double().cpu().numpy()
        bts.bidir_step(ctx, g.contiguous(), eps, delta, w, p, alpha, 1.0, ui, uv, di, dv, None)
        want = oracle.bidir_step(h_g, h_eps, h_delta, h_w, h_p, 1, K_dn, alpha, 1.0)
        if t == 210 and K_dn == d:
            # the two norms the paper prints for the unidirectional run, from the GPU's
            # own uplink messages
            torch.cuda.synchronize()
            sum_top = np.zeros(d)
            gi, gv = ui.cpu().numpy(), uv.cpu().numpy()
            for q in range(N):
                sum_top[gi[q]] += gv[q]
            top = np.zeros(d)
            j = np.argmax(np.abs(sum_top))
            top[j] = sum_top[j]
            assert round(float(np.linalg.norm(a.sum(0) - sum_top)), 2) == 21.80
            assert round(float(np.linalg.norm(a.sum(0) - top)), 2) == 21.54
        if t % 50 == 49 or t < 3:
            torch.cuda.synchronize()
            G.assert_same_bits(w, h_w, f"w at iteration {t}")
            G.assert_same_bits(eps, h_eps, f"eps at iteration {t}")
            G.assert_same_bits(delta, h_delta, f"delta at iteration {t}")
            G.assert_same_bits(ui, want["up_idx"], f"up_idx at iteration {t}")
            G.assert_same_bits(di, want["dn_idx"], f"dn_idx at iteration {t}")
    f_star = 6100.0 / 9.0
    loss = sum(0.5 * float(((w.double() - float(ci)) ** 2).sum()) for ci in CENTRES) / 3.0
    assert f_star <= loss < 1.1 * f_star

"""GPU parity at the benchmark's full sizes, in the launch configuration bench.py times.

Every step of every configuration (C1 3 steps, C2/C3/C4 10, C5 5, residuals carried) goes
through the CPU oracle in full -- the full stable sort of every worker row, the aggregation
onto the carried delta, the server's sort, the update -- and every output of the step
(uplink messages, eps, downlink message, delta, w, union nnz) is compared as uint32 words.
"""
import time

import numpy as np
import pytest
import torch

import workloads as wl

pytestmark = pytest.mark.gpu


@pytest.fixture
def say(capsys):
    """Progress lines that reach the terminal while output is captured: a step of the
    largest configuration takes the oracle most of a minute, and a run that stays silent
    for minutes is taken to be hung."""
    def _say(msg):
        with capsys.disabled():
            print(msg, flush=True)
    return _say


def assert_rows_same_bits(got: torch.Tensor, want: np.ndarray, what: str):
    """got (device, 2-D) against want (host, 2-D) as uint32 words, one row at a time on the
    device (a row of the largest configuration is 440 MB; the whole matrix 28 GB)."""
    assert tuple(got.shape) == tuple(want.shape), f"{what}: shape"
    for q in range(got.shape[0]):
        ref = torch.from_numpy(want[q].view(np.int32)).to(got.device)
        if not torch.equal(got[q].view(torch.int32), ref):
            bad = torch.nonzero(got[q].view(torch.int32) != ref).ravel()
            i = int(bad[0])
            raise AssertionError(
                f"{what}: row {q}: {bad.numel()} words differ, first at {i}: got "
                f"0x{int(got[q].view(torch.int32)[i]) & 0xFFFFFFFF:08x} want "
                f"0x{int(ref[i]) & 0xFFFFFFFF:08x}")


def run_full_size(oracle, name, alpha_in, alpha_out, say):
    import _gpu_util as G
    import paper_2209_15203_amd as bts
    cfg = wl.CONFIGS[name]
    N, d = cfg.N, cfg.d
    D = G.dev()
    src = wl.GradientSource(cfg, D)
    p_host = wl.p_weights(cfg)
    w0 = wl.weights0(cfg, D)
    ctx = bts.BtsContext(N, d, cfg.K_up, cfg.K_dn)
    eps = torch.zeros((N, d), dtype=torch.float32, device=D)
    delta = torch.zeros(d, dtype=torch.float32, device=D)
    w = w0.clone()
    p = torch.from_numpy(p_host).to(D)
    ui = torch.zeros((N, cfg.K_up), dtype=torch.int32, device=D)
    uv = torch.zeros((N, cfg.K_up), dtype=torch.float32, device=D)
    di = torch.zeros(cfg.K_dn, dtype=torch.int32, device=D)
    dv = torch.zeros(cfg.K_dn, dtype=torch.float32, device=D)
    nnz = torch.zeros(1, dtype=torch.int32, device=D)
    g = torch.empty((N, d), dtype=torch.float32, device=D)

    h_g = np.empty((N, d), np.float32)
    h_eps = np.zeros((N, d), np.float32)
    h_delta = np.zeros(d, np.float32)
    h_w = w0.cpu().numpy().copy()
    t_start = time.perf_counter()
    for t in range(1, cfg.steps + 1):
        src.fill(t, g)
        tag = f"{name} step {t}"
        say(f"[{name}] step {t}/{cfg.steps} at {time.perf_counter() - t_start:.0f} s")
        bts.bidir_step(ctx, g, eps, delta, w, p, alpha_in, alpha_out, ui, uv, di, dv, nnz)
        torch.cuda.synchronize()
        torch.from_numpy(h_g).copy_(g)           # straight into the oracle's input buffer
        want = oracle.bidir_step(h_g, h_eps, h_delta, h_w, p_host, cfg.K_up, cfg.K_dn,
                                 alpha_in, alpha_out)
        G.assert_same_bits(ui, want["up_idx"], f"{tag} up_idx")
        G.assert_same_bits(uv, want["up_val"], f"{tag} up_val")
        assert_rows_same_bits(eps, h_eps, f"{tag} eps")
        G.assert_same_bits(di, want["dn_idx"], f"{tag} dn_idx")
        G.assert_same_bits(dv, want["dn_val"], f"{tag} dn_val")
        G.assert_same_bits(delta, h_delta, f"{tag} delta")
        G.assert_same_bits(w, h_w, f"{tag} w")
        assert int(nnz.item()) == want["union_nnz"], f"{tag} union nnz"
    say(f"[{name}] {cfg.steps} steps compared in {time.perf_counter() - t_start:.0f} s")


@pytest.mark.timeout(900)
@pytest.mark.parametrize("name", ["C1", "C2", "C3", "C4", "C5"])
def test_full_size_config(oracle, name, say):
    """Paper form: the step size inside a (alpha_in = alpha, alpha_out = 1)."""
    run_full_size(oracle, name, wl.CONFIGS[name].alpha, 1.0, say)


@pytest.mark.timeout(600)
def test_full_size_other_alpha_form_c2(oracle, say):
    """The other placement of the step size (alpha_in = 1, alpha_out = alpha: residual added
    to the raw gradient, w -= alpha * message) at a benchmark size: C2, every step."""
    run_full_size(oracle, "C2", 1.0, wl.CONFIGS["C2"].alpha, say)


@pytest.mark.timeout(600)
def test_full_size_dense_path_c3(oracle):
    """The dense select path (the fallback of the single-pass path) forced at a benchmark
    size: C3, one step, every output bit for bit against the oracle."""
    import _gpu_util as G
    cfg = wl.CONFIGS["C3"]
    src = wl.GradientSource(cfg, G.dev())
    w0 = wl.weights0(cfg, G.dev()).cpu().numpy()
    st = G.GpuState(cfg.N, cfg.d, cfg.K_up, cfg.K_dn, w0, wl.p_weights(cfg))
    st.ctx.set_path(1)
    st.step_and_compare(oracle, src.step(1), cfg.alpha, 1.0, "C3 dense step 1")
    assert st.ctx.last_path(0) == (0, cfg.N)


@pytest.mark.timeout(600)
def test_full_size_unidirectional_c3(oracle):
    """Algorithm 1 at a benchmark size (C3: 32 workers, d = 25,557,032): two steps, every
    output bit for bit against the oracle."""
    import _gpu_util as G
    import paper_2209_15203_amd as bts
    cfg = wl.CONFIGS["C3"]
    N, d, K = cfg.N, cfg.d, cfg.K_up
    D = G.dev()
    src = wl.GradientSource(cfg, D)
    p_host = wl.p_weights(cfg)
    w0 = wl.weights0(cfg, D)
    ctx = bts.BtsContext(N, d, K, cfg.K_dn)
    eps = torch.zeros((N, d), dtype=torch.float32, device=D)
    w = w0.clone()
    p = torch.from_numpy(p_host).to(D)
    ui = torch.zeros((N, K), dtype=torch.int32, device=D)
    uv = torch.zeros((N, K), dtype=torch.float32, device=D)
    di = torch.zeros(N * K, dtype=torch.int32, device=D)
    dv = torch.zeros(N * K, dtype=torch.float32, device=D)
    dc = torch.zeros(1, dtype=torch.int32, device=D)
    g = torch.empty((N, d), dtype=torch.float32, device=D)
    h_eps = np.zeros((N, d), np.float32)
    h_w = w0.cpu().numpy().copy()
    for t in (1, 2):
        src.fill(t, g)
        print(f"[C3 unidirectional] step {t}/2", flush=True)
        bts.unidir_step(ctx, g, eps, w, p, cfg.alpha, 1.0, ui, uv, di, dv, dc)
        torch.cuda.synchronize()
        want = oracle.unidir_step(g.cpu().numpy(), h_eps, h_w, p_host, K, cfg.alpha, 1.0)
        n = int(dc.item())
        assert n == want["dn_count"]
        G.assert_same_bits(ui, want["up_idx"], f"step {t} up_idx")
        G.assert_same_bits(uv, want["up_val"], f"step {t} up_val")
        G.assert_same_bits(eps, h_eps, f"step {t} eps")
        G.assert_same_bits(di[:n], want["dn_idx"], f"step {t} message indices")
        G.assert_same_bits(dv[:n], want["dn_val"], f"step {t} message values")
        G.assert_same_bits(w, h_w, f"step {t} w")


@pytest.mark.timeout(600)
@pytest.mark.parametrize("path", [1, 2])
def test_indices_beyond_2_to_31(path):
    """One row longer than 2^31 coordinates (d = 2^31 + 2^20 + 3, ragged tail): indices use
    the full unsigned 32-bit range.  The oracle would need many minutes to sort such a row,
    so the expected result is built in: bounded noise (|x| <= 1) with 3K planted values of
    distinct larger magnitudes, some of them past 2^31 and in the last partial chunk.  Top_K
    must return exactly the K largest planted coordinates, ascending, and zero them."""
    import _gpu_util as G
    import paper_2209_15203_amd as bts
    D = G.dev()
    d = (1 << 31) + (1 << 20) + 3
    K, P = 4096, 3 * 4096
    g = torch.empty(d, dtype=torch.float32, device=D)
    step = 1 << 26
    gen = torch.Generator(device=D)
    gen.manual_seed(77)
    for s in range(0, d, step):
        n = min(step, d - s)
        g[s:s + n] = torch.rand(n, generator=gen, device=D) * 2.0 - 1.0
    rng = np.random.default_rng(5)
    planted = np.unique(np.concatenate([
        rng.integers(0, d, size=2 * P, dtype=np.int64),
        np.arange(d - 40, d, dtype=np.int64),                   # the ragged tail
        (1 << 31) + np.arange(-12, 12, dtype=np.int64)]))       # around the sign bit of int32
    must = np.concatenate([np.arange(d - 40, d), (1 << 31) + np.arange(-12, 12)])
    rest = np.setdiff1d(planted, must)
    planted = np.concatenate([must, rng.permutation(rest)[:P - must.size]])
    # distinct magnitudes 2 + j/P; the special positions get the largest ones
    mags = (2.0 + (P - 1 - np.arange(P, dtype=np.float32)) / P).astype(np.float32)
    vals = mags * rng.choice(np.array([-1.0, 1.0], np.float32), size=P)
    g[torch.from_numpy(planted).to(D)] = torch.from_numpy(vals).to(D)
    order = np.argsort(planted[:K])
    want_idx, want_val = planted[:K][order], vals[:K][order]    # the K largest magnitudes
    assert want_idx[-1] == d - 1 and (want_idx > (1 << 31)).sum() >= 12
    eps = torch.zeros(d, dtype=torch.float32, device=D)
    ctx = bts.BtsContext(1, d, K, K)
    ctx.set_path(path)
    ui = torch.zeros((1, K), dtype=torch.int32, device=D)
    uv = torch.zeros((1, K), dtype=torch.float32, device=D)
    bts.topk_compress(ctx, g.view(1, d), eps.view(1, d), 1.0, ui, uv)
    torch.cuda.synchronize()
    got_idx = ui.cpu().numpy().view(np.uint32).ravel().astype(np.int64)
    assert np.array_equal(got_idx, want_idx)
    G.assert_same_bits(uv.ravel(), want_val, "values")
    t_sel = torch.from_numpy(want_idx).to(D)
    assert not bool(eps[t_sel].view(torch.int32).any())
    # everything else is a = 0 + 1*g = g, untouched
    probe = torch.cat([torch.from_numpy(rng.integers(0, d, size=1 << 20, dtype=np.int64)),
                       torch.from_numpy(planted[K:])]).to(D)
    keep = ~torch.isin(probe, t_sel)
    assert torch.equal(eps[probe][keep].view(torch.int32), g[probe][keep].view(torch.int32))
    fast, dense = ctx.last_path(0)
    assert (fast, dense) == ((1, 0) if path == 2 else (0, 1))

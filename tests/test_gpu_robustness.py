"""GPU tests of the edges of the contract: NaN passing through the multiply-adds (the one
stated relaxation of the parity bar), the recovery paths taken after a failed launch (forced
from the host, no fault involved), and argument checks that must happen before anything is
queued."""
import ctypes as C

import numpy as np
import pytest
import torch

pytestmark = pytest.mark.gpu


def assert_same_bits_nan_payload_masked(got, want, what):
    """The relaxation: where the oracle's word is a NaN the GPU's must be a NaN too (sign and
    payload, 2^24 - 2 patterns, not compared); every other word bit for bit."""
    import _gpu_util as G
    g, w = G.bits(got).ravel(), G.bits(want).ravel()
    assert g.shape == w.shape, what
    g_nan, w_nan = (g & 0x7FFFFFFF) > 0x7F800000, (w & 0x7FFFFFFF) > 0x7F800000
    assert np.array_equal(g_nan, w_nan), f"{what}: NaNs at different places"
    assert np.array_equal(g[~w_nan], w[~w_nan]), f"{what}: a non-NaN word differs"
    return int(w_nan.sum())


@pytest.mark.parametrize("path", [0, 1, 2, 3])
def test_nan_through_the_multiply_adds(oracle, path):
    """NaN enters through g (quiet, negative, signalling payloads) and is made by
    inf - inf in the error compensation.  Guaranteed: a NaN of a ranks above every other
    value, so with fewer NaNs than K all of them are sent (indices bit-exact), the residual
    holds +0 there, and the NaN travels on through the aggregation, the downlink message
    and the model update.  Not compared: the sign and payload bits of a NaN that came out of
    a multiply-add (hardware and libm differ there)."""
    import _gpu_util as G
    import paper_2209_15203_amd as bts
    rng = np.random.default_rng(99)
    N, d, K_up, K_dn = 3, 70_001, 64, 40
    g = rng.standard_normal((N, d)).astype(np.float32)
    eps0 = (0.5 * rng.standard_normal((N, d))).astype(np.float32)
    gb = g.view(np.uint32)
    gb[0, 5] = 0x7FC00000            # quiet NaN
    gb[0, 60_000] = 0xFFC12345       # negative quiet NaN with a payload
    gb[1, 12_345] = 0x7F800001       # signalling NaN
    g[2, 777] = np.inf               # inf - inf in a = eps + alpha g
    eps0[2, 777] = -np.inf
    g[2, 4096] = -np.inf             # a plain infinity: ranks below the NaNs, above the rest
    D = G.dev()
    p = np.array([0.5, 0.3, 0.2], np.float32)
    w0 = rng.standard_normal(d).astype(np.float32)
    st = G.GpuState(N, d, K_up, K_dn, w0, p)
    st.ctx.set_path(path)
    st.eps.copy_(torch.from_numpy(eps0))
    st.h_eps[:] = eps0
    bts.bidir_step(st.ctx, torch.from_numpy(g).to(D), st.eps, st.delta, st.w, st.p, 0.37, 1.0,
                   st.up_idx, st.up_val, st.dn_idx, st.dn_val, st.nnz)
    torch.cuda.synchronize()
    want = oracle.bidir_step(g, st.h_eps, st.h_delta, st.h_w, p, K_up, K_dn, 0.37, 1.0)
    G.assert_same_bits(st.up_idx, want["up_idx"], "up_idx")
    assert assert_same_bits_nan_payload_masked(st.up_val, want["up_val"], "up_val") == 4
    G.assert_same_bits(st.eps, st.h_eps, "eps")           # every NaN was sent: no NaN left
    G.assert_same_bits(st.dn_idx, want["dn_idx"], "dn_idx")
    assert assert_same_bits_nan_payload_masked(st.dn_val, want["dn_val"], "dn_val") == 4
    G.assert_same_bits(st.delta, st.h_delta, "delta")
    assert assert_same_bits_nan_payload_masked(st.w, st.h_w, "w") == 4
    for q, i in ((0, 5), (0, 60_000), (1, 12_345), (2, 777)):
        assert i in want["up_idx"][q] and i in want["dn_idx"]
    assert int(st.nnz.item()) == want["union_nnz"]


@pytest.mark.parametrize("path", [1, 2, 3])
def test_step_after_a_failed_call_recovers(oracle, path):
    """The library keeps its scratch clean between calls; after a call that failed half way
    it must clear what that call may have left and stop trusting the aggregation's range
    tables.  The condition is forced from the host (bts_testing_mark_dirty) after a normal
    step has left real contents behind; the next steps must still match the oracle bit for
    bit, on both select paths and with the aggregation finding its ranges by binary search."""
    import _gpu_util as G
    import workloads as wl
    cfg = wl.CONFIGS["C2"].scaled(150_001, N=5, steps=4)
    src = wl.GradientSource(cfg, G.dev())
    w0 = wl.weights0(cfg, "cpu").numpy()
    st = G.GpuState(cfg.N, cfg.d, cfg.K_up, cfg.K_dn, w0, wl.p_weights(cfg))
    st.ctx.set_path(path)
    for t in range(1, cfg.steps + 1):
        if t in (2, 3):
            st.ctx.testing_mark_dirty()
        st.step_and_compare(oracle, src.step(t), cfg.alpha, 1.0, f"path {path} step {t}")
    fast, dense = st.ctx.last_path(0)
    assert (fast, dense) == ((cfg.N, 0) if path == 2 else (0, cfg.N))
    # the three-launch select fills the aggregation's range tables itself; after the forced
    # failure those tables are no longer trusted and the aggregation searches instead


def test_binding_refuses_undersized_tensors():
    """A tensor smaller than the shape of the context would make a kernel run past its end;
    the binding refuses it on the host."""
    import _gpu_util as G
    import paper_2209_15203_amd as bts
    D = G.dev()
    N, d, K = 3, 5000, 50
    ctx = bts.BtsContext(N, d, K, K)
    f = lambda *s: torch.zeros(s, dtype=torch.float32, device=D)
    i = lambda *s: torch.zeros(s, dtype=torch.int32, device=D)
    good = dict(g=f(N, d), eps=f(N, d), delta=f(d), w=f(d), p=f(N), up_idx=i(N, K),
                up_val=f(N, K), dn_idx=i(K), dn_val=f(K))
    small = dict(g=f(N, d - 1), eps=f(N - 1, d), delta=f(d - 1), w=f(d - 1), p=f(N - 1),
                 up_idx=i(N, K - 1), up_val=f(N, K - 1), dn_idx=i(K - 1), dn_val=f(K - 1))
    for name, t in small.items():
        a = dict(good)
        a[name] = t
        with pytest.raises(TypeError):
            bts.bidir_step(ctx, a["g"], a["eps"], a["delta"], a["w"], a["p"], 0.01, 1.0,
                           a["up_idx"], a["up_val"], a["dn_idx"], a["dn_val"])
    ctx.enable_diagnostics()
    with pytest.raises(TypeError):
        bts.bidir_step_diag(ctx, good["g"], good["eps"], good["delta"], good["w"], good["p"],
                            0.01, 1.0, good["up_idx"], good["up_val"], good["dn_idx"],
                            good["dn_val"], torch.zeros(8 + N - 1, dtype=torch.float64, device=D))
    with pytest.raises(TypeError):
        bts.unidir_step(ctx, good["g"], good["eps"], good["w"], good["p"], 0.01, 1.0,
                        good["up_idx"], good["up_val"], i(N * K - 1), f(N * K - 1), i(1))
    with pytest.raises(TypeError):
        bts.topk_compress_noalloc(good["g"], f(N, d - 1), 0.01, good["up_idx"], good["up_val"])
    bts.bidir_step(ctx, *(good[k] for k in ("g", "eps", "delta", "w", "p")), 0.01, 1.0,
                   *(good[k] for k in ("up_idx", "up_val", "dn_idx", "dn_val")))
    torch.cuda.synchronize()


def test_diag_step_checks_every_argument_before_it_queues_anything():
    """bidir_step_diag with a bad argument (null w, null message buffer, misaligned eps)
    returns BTS_EINVAL and leaves eps, delta and its scratch untouched."""
    import _gpu_util as G
    import paper_2209_15203_amd as bts
    D = G.dev()
    N, d, K = 2, 4096, 16
    ctx = bts.BtsContext(N, d, K, K)
    ctx.enable_diagnostics()
    g = torch.randn(N, d, device=D)
    eps = torch.randn(N * d + 4, device=D)
    delta = torch.randn(d, device=D)
    w = torch.randn(d, device=D)
    p = torch.full((N,), 0.5, device=D)
    ui = torch.zeros((N, K), dtype=torch.int32, device=D)
    uv = torch.zeros((N, K), device=D)
    di = torch.zeros(K, dtype=torch.int32, device=D)
    dv = torch.zeros(K, device=D)
    diag = torch.full((8 + N,), -1.0, dtype=torch.float64, device=D)
    eps0, delta0 = eps.clone(), delta.clone()
    ptr = lambda t: C.c_void_p(t.data_ptr())
    lib = bts.load_library()
    def call(pw, pui, peps):
        return lib.bidir_step_diag(ctx._h, ptr(g), peps, ptr(delta), pw, ptr(p), 0.01, 1.0, pui,
                                   ptr(uv), ptr(di), ptr(dv), ptr(diag))
    assert call(None, ptr(ui), ptr(eps)) == -1
    assert call(ptr(w), None, ptr(eps)) == -1
    assert call(ptr(w), ptr(ui), C.c_void_p(eps.data_ptr() + 4)) == -1
    torch.cuda.synchronize()
    assert torch.equal(eps, eps0) and torch.equal(delta, delta0)
    assert bool((diag == -1.0).all())
    assert call(ptr(w), ptr(ui), ptr(eps)) == 0
    torch.cuda.synchronize()
    assert float(diag[3]) >= 0.0


def test_bounds_handed_from_call_to_call_never_decide_the_result(oracle):
    """From its third call on a context's single-pass select starts from bounds the call
    before left behind instead of sampling.  The gradients' scale jumps by factors of 50
    between calls here, so those bounds are far off in both directions (lists that overflow,
    lists that fall short, coordinates zeroed early that are not sent after all): every call
    must still match the oracle bit for bit, and once the scale holds still the rows must
    finish in the single pass again (the redo sets a row's bounds from its exact threshold)."""
    import _gpu_util as G
    import paper_2209_15203_amd as bts
    rng = np.random.default_rng(4242)
    N, d, K = 3, 300_007, 600
    D = G.dev()
    ctx = bts.BtsContext(N, d, K, K)
    ctx.set_path(2)
    eps = np.zeros((N, d), np.float32)
    te = torch.from_numpy(eps).to(D)
    ui = torch.zeros((N, K), dtype=torch.int32, device=D)
    uv = torch.zeros((N, K), dtype=torch.float32, device=D)
    scales = [1.0, 1.0, 1.0, 50.0, 1.0, 0.02, 0.02, 0.02, 0.02, 30.0, 30.0, 30.0]
    paths = []
    for step, sc in enumerate(scales):
        g = (rng.standard_normal((N, d)) * sc).astype(np.float32)
        if step == 5:
            eps[:] = 0.0                # forget the large residuals, so that the scale can drop
            te.zero_()
        bts.topk_compress(ctx, torch.from_numpy(g).to(D), te, 0.5, ui, uv)
        torch.cuda.synchronize()
        wi, wv = oracle.worker_stage(g, eps, 0.5, K)
        G.assert_same_bits(ui, wi, f"step {step} up_idx")
        G.assert_same_bits(uv, wv, f"step {step} up_val")
        G.assert_same_bits(te, eps, f"step {step} eps")
        paths.append(ctx.last_path(0))
    assert paths[0] == (N, 0) and paths[1] == (N, 0) and paths[2] == (N, 0), paths
    assert any(p[1] > 0 for p in paths[3:7]), f"the jumps should have sent rows to the redo: {paths}"
    assert paths[8] == (N, 0) and paths[11] == (N, 0), f"bounds did not recover: {paths}"


@pytest.mark.parametrize("K_dn", [500, 6000])
def test_whole_step_with_rows_that_the_dense_path_redoes(oracle, K_dn):
    """A whole step on the single-pass path in which some worker rows are handed to the dense
    path (three magnitudes only: a third of the row ties at the top and the candidate lists
    overflow) and the others finish in the single pass.  The select's last launch then fills
    the aggregation's range tables both ways (from the finished messages; pair by pair for
    the redone rows) and applies the downlink message to the model (K_dn = 6000: after the
    emission; 500: by the emitting lanes); every output must be the oracle's, over several
    steps with carried residuals."""
    import _gpu_util as G
    rng = np.random.default_rng(777 + K_dn)
    N, d, K_up = 6, 400_003, 700
    D = G.dev()
    p = rng.dirichlet(np.ones(N)).astype(np.float32)
    w0 = rng.standard_normal(d).astype(np.float32)
    st = G.GpuState(N, d, K_up, K_dn, w0, p)
    st.ctx.set_path(2)
    saw_both = False
    for step in range(5):
        g = rng.standard_normal((N, d)).astype(np.float32)
        tied = rng.integers(1, 4, size=(N // 2, d)).astype(np.float32)
        g[::2] = tied * rng.choice(np.array([-1.0, 1.0], np.float32), size=tied.shape)
        if step >= 3:
            g[::2] *= 1e-3            # now the tied rows are small next to their residuals
        st.step_and_compare(oracle, torch.from_numpy(g).to(D), 0.25, 1.0, f"step {step}")
        fast, dense = st.ctx.last_path(0)
        assert fast + dense == N
        saw_both = saw_both or (fast > 0 and dense > 0)
    assert saw_both, "no step mixed rows of both kinds"


def test_the_same_gradient_fed_again_and_again(oracle):
    """A caller that times the step in a loop over ONE gradient tensor: the residuals then grow
    coherently and the thresholds by a half, a third, a quarter ... per step, faster than the
    bounds handed from call to call follow at first.  The rows that are redone report it to the
    host, which samples again for a few calls; after that the trend is slow enough to follow.
    Every call exact; only a call or two may have rows redone."""
    import _gpu_util as G
    import paper_2209_15203_amd as bts
    rng = np.random.default_rng(2024)
    N, d, K = 4, 300_007, 600
    D = G.dev()
    ctx = bts.BtsContext(N, d, K, K)
    ctx.set_path(2)
    g = rng.standard_normal((N, d)).astype(np.float32)
    tg = torch.from_numpy(g).to(D)
    eps = np.zeros((N, d), np.float32)
    te = torch.from_numpy(eps).to(D)
    ui = torch.zeros((N, K), dtype=torch.int32, device=D)
    uv = torch.zeros((N, K), dtype=torch.float32, device=D)
    redone = []
    for step in range(14):
        bts.topk_compress(ctx, tg, te, 0.5, ui, uv)
        torch.cuda.synchronize()
        wi, wv = oracle.worker_stage(g, eps, 0.5, K)
        G.assert_same_bits(ui, wi, f"step {step} up_idx")
        G.assert_same_bits(uv, wv, f"step {step} up_val")
        G.assert_same_bits(te, eps, f"step {step} eps")
        redone.append(ctx.last_path(0)[1])
    assert sum(1 for r in redone if r) <= 3, f"rows kept being redone: {redone}"
    assert redone[-4:] == [0, 0, 0, 0], f"the select did not settle: {redone}"

"""GPU parity tests: every entry point of the C ABI against the CPU oracle, bit for bit
(0 ulp on every fp32 output, exact on every index), on the same seeded inputs."""
import numpy as np
import pytest
import torch

import workloads as wl

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def G():
    import _gpu_util
    assert torch.cuda.is_available(), "these tests need the MI355X"
    return _gpu_util


def tied_rows(rng, N, d, levels=3):
    """Rows whose magnitudes take only a few values, random signs: boundary ties everywhere."""
    mag = rng.integers(1, levels + 1, size=(N, d)).astype(np.float32)
    return mag * rng.choice(np.array([-1.0, 1.0], np.float32), size=(N, d))


SHAPES = [
    # N, d, K   (ragged rows: d % 4 != 0 puts rows off 16-byte alignment; d below one chunk;
    #            several chunks and a tail; K = 1, K = d; from d = 65536 on and K <= d/64 the
    #            single-pass path is possible and path mode 2 takes it)
    (1, 1, 1), (3, 5, 2), (2, 63, 7), (4, 1000, 10), (3, 2049, 33), (5, 4099, 4099),
    (2, 10007, 1), (7, 30011, 301), (4, 65536, 66), (3, 100003, 1001), (2, 262147, 5000),
    (1, 70001, 1), (5, 65537, 1024), (2, 262147, 3000), (3, 1048579, 1049), (9, 300001, 37),
    # the one-workgroup-per-row path ends at d = 8192
    (64, 8192, 82), (3, 8191, 8191), (2, 7000, 1), (2, 8193, 9),
]
# AUTO: by shape (one workgroup per row up to d = 8192; the three-launch select for small K on
# rows up to 2^22 where the call is bound by launches); THREE_LAUNCH: that select wherever
# the shape allows it (K <= 8192, K <= d / 64, 8192 < d <= 2^22), else the dense path
AUTO, DENSE, SINGLE_PASS, THREE_LAUNCH = 0, 1, 2, 3


def make_rows(rng, kind, N, d):
    """(g, eps0, alpha) for one compress call."""
    if kind == "normal":
        return (rng.standard_normal((N, d)).astype(np.float32),
                (rng.standard_normal((N, d)) * 0.5).astype(np.float32), 0.37)
    if kind == "ties":                      # three magnitudes: the candidate list overflows
        return tied_rows(rng, N, d), np.zeros((N, d), np.float32), 1.0
    if kind == "quantized":                 # a grid of values: small tie groups at the threshold
        g = (np.round(rng.standard_normal((N, d)) * 256) / 256).astype(np.float32)
        return g, np.zeros((N, d), np.float32), 1.0
    if kind == "mixed":                     # some rows finish in one pass, some fall back
        g = rng.standard_normal((N, d)).astype(np.float32)
        g[::2] = tied_rows(rng, len(g[::2]), d)
        return g, np.zeros((N, d), np.float32), 1.0
    raise ValueError(kind)


@pytest.mark.parametrize("N,d,K", SHAPES)
@pytest.mark.parametrize("kind", ["normal", "ties", "quantized", "mixed"])
@pytest.mark.parametrize("path", [AUTO, DENSE, SINGLE_PASS, THREE_LAUNCH])
def test_topk_compress(G, oracle, N, d, K, kind, path):
    import paper_2209_15203_amd as bts
    three_launch_ok = K <= 8192 and K * 64 <= d and 8192 < d <= (1 << 22)
    if path == AUTO and d > 8192 and not three_launch_ok:
        pytest.skip("by shape this is the dense path, covered")
    if path == THREE_LAUNCH and not three_launch_ok:
        pytest.skip("the shape does not allow the three-launch select (it is the dense path)")
    rng = np.random.default_rng(N * 1000003 + d * 7 + K)
    g, eps0, alpha = make_rows(rng, kind, N, d)
    D = G.dev()
    ctx = bts.BtsContext(N, d, K, K)
    ctx.set_path(path)
    tg, te = torch.from_numpy(g).to(D), torch.from_numpy(eps0).to(D)
    ui = torch.full((N, K), -1, dtype=torch.int32, device=D)
    uv = torch.zeros((N, K), dtype=torch.float32, device=D)
    bts.topk_compress(ctx, tg, te, alpha, ui, uv)
    torch.cuda.synchronize()
    h_eps = eps0.copy()
    want_i, want_v = oracle.worker_stage(g, h_eps, alpha, K)
    G.assert_same_bits(ui, want_i, "up_idx")
    G.assert_same_bits(uv, want_v, "up_val")
    G.assert_same_bits(te, h_eps, "eps")
    G.assert_same_bits(tg, g, "g must not be modified")
    fast, dense = ctx.last_path(0)
    assert fast + dense == N
    if path == SINGLE_PASS and d >= 65536 and K * 64 <= d:
        if kind in ("normal", "quantized"):
            assert fast == N, "iid rows must finish in the single pass"
        # three-valued rows: a third of the row ties at the top; at the larger d that
        # overflows the candidate list (dense fallback), at the smaller it fits and the
        # single pass splits the ties by index itself
        if kind == "ties" and d >= 262147:
            assert dense == N, "three-valued rows overflow the candidate list"
        if kind == "mixed" and N > 1 and d >= 262147:
            assert 0 < fast < N
    else:
        assert fast == 0


def test_k_zero_is_plain_error_accumulation(G, oracle):
    import paper_2209_15203_amd as bts
    rng = np.random.default_rng(1)
    N, d = 3, 5001
    g = rng.standard_normal((N, d)).astype(np.float32)
    e = rng.standard_normal((N, d)).astype(np.float32)
    D = G.dev()
    ctx = bts.BtsContext(N, d, 0, 0)
    tg, te = torch.from_numpy(g).to(D), torch.from_numpy(e).to(D)
    bts.topk_compress(ctx, tg, te, 0.01, None, None)
    torch.cuda.synchronize()
    h = e.copy()
    oracle.worker_stage(g, h, 0.01, 0)
    G.assert_same_bits(te, h, "eps")


def test_threshold_run_spanning_many_workgroups(G, oracle):
    """Three distinct magnitudes at a realistic d; the K-th largest falls inside a run of
    equal keys that spans hundreds of workgroups, so the lowest-index rule decides."""
    import paper_2209_15203_amd as bts
    d = 3_000_001
    x = np.empty(d, np.float32)
    x[0::3], x[1::3], x[2::3] = 1.0, -2.0, 3.0
    n3, n2 = len(x[2::3]), len(x[1::3])
    D = G.dev()
    for K, path in ((n3 + n2 + 123_457, DENSE), (n3 - 5, DENSE), (n3 + 1, 0), (17, DENSE),
                    (17, SINGLE_PASS), (40_000, SINGLE_PASS)):
        ctx = bts.BtsContext(1, d, K, K)
        ctx.set_path(path)
        t = torch.from_numpy(x.copy()).to(D)
        oi = torch.zeros(K, dtype=torch.int32, device=D)
        ov = torch.zeros(K, dtype=torch.float32, device=D)
        bts.downlink_topk(ctx, t, oi, ov)
        torch.cuda.synchronize()
        h = x.copy()
        wi, wv = oracle.downlink(h, K)
        G.assert_same_bits(oi, wi, f"K={K} idx")
        G.assert_same_bits(ov, wv, f"K={K} val")
        G.assert_same_bits(t, h, f"K={K} residual")


@pytest.mark.parametrize("start", [300_000, 655_360 - 17])
def test_all_kept_coordinates_in_one_contiguous_block(G, oracle, start):
    """Every large value sits in one block of 60,000 consecutive coordinates (runs of 512
    candidates per wave chunk, directory tiles with tens of thousands of entries, a strided
    sample that may miss the block or land inside it): whichever way the rows finish, the
    result is the oracle's."""
    import paper_2209_15203_amd as bts
    rng = np.random.default_rng(start)
    N, d, K = 3, 1 << 20, 40_000
    g = (rng.standard_normal((N, d)) * 1e-3).astype(np.float32)
    for q in range(N):
        block = rng.permutation(60_000).astype(np.float32) + 1000.0      # distinct magnitudes
        g[q, start + 7 * q:start + 7 * q + 60_000] = block * rng.choice([-1.0, 1.0], size=60_000)
    e = np.zeros_like(g)
    D = G.dev()
    for path in (SINGLE_PASS, DENSE):
        ctx = bts.BtsContext(N, d, K, K)
        ctx.set_path(path)
        tg, te = torch.from_numpy(g).to(D), torch.from_numpy(e).to(D)
        ui = torch.zeros((N, K), dtype=torch.int32, device=D)
        uv = torch.zeros((N, K), dtype=torch.float32, device=D)
        bts.topk_compress(ctx, tg, te, 1.0, ui, uv)
        torch.cuda.synchronize()
        h = e.copy()
        wi, wv = oracle.worker_stage(g, h, 1.0, K)
        G.assert_same_bits(ui, wi, f"path {path} up_idx")
        G.assert_same_bits(uv, wv, f"path {path} up_val")
        G.assert_same_bits(te, h, f"path {path} eps")


def test_threshold_far_above_the_sampled_bound_goes_to_the_dense_path(G, oracle):
    """The single-pass select works in a window of four octaves above its sampled lower
    bound.  Here 1.5 K spikes of magnitude 1e3..2e3 sit on N(0,1) noise: the sample puts
    the bound into the noise tail, the K-th largest is a spike, far beyond the window, so
    the rows must be handed to the dense path -- and the result is still the oracle's."""
    import paper_2209_15203_amd as bts
    rng = np.random.default_rng(31)
    N, d, K = 3, 1 << 20, 1024
    g = rng.standard_normal((N, d)).astype(np.float32)
    for q in range(N):
        at = rng.choice(d, size=3 * K // 2, replace=False)
        g[q, at] = (rng.uniform(1e3, 2e3, size=at.size) * rng.choice([-1.0, 1.0], size=at.size)
                    ).astype(np.float32)
    e = np.zeros_like(g)
    D = G.dev()
    ctx = bts.BtsContext(N, d, K, K)
    ctx.set_path(SINGLE_PASS)
    tg, te = torch.from_numpy(g).to(D), torch.from_numpy(e).to(D)
    ui = torch.zeros((N, K), dtype=torch.int32, device=D)
    uv = torch.zeros((N, K), dtype=torch.float32, device=D)
    bts.topk_compress(ctx, tg, te, 1.0, ui, uv)
    torch.cuda.synchronize()
    assert ctx.last_path(0) == (0, N), "every row should have left the window"
    h = e.copy()
    wi, wv = oracle.worker_stage(g, h, 1.0, K)
    G.assert_same_bits(ui, wi, "up_idx")
    G.assert_same_bits(uv, wv, "up_val")
    G.assert_same_bits(te, h, "eps")
    # the same context then serves an ordinary batch in one pass again
    g2 = rng.standard_normal((N, d)).astype(np.float32)
    tg2 = torch.from_numpy(g2).to(D)
    bts.topk_compress(ctx, tg2, te, 1.0, ui, uv)
    torch.cuda.synchronize()
    assert ctx.last_path(0) == (N, 0)
    wi, wv = oracle.worker_stage(g2, h, 1.0, K)
    G.assert_same_bits(ui, wi, "up_idx, second batch")
    G.assert_same_bits(te, h, "eps, second batch")


@pytest.mark.parametrize("d,path", [(9001, DENSE), (200_001, DENSE), (200_001, SINGLE_PASS),
                                    (200_001, THREE_LAUNCH)])
def test_special_values_are_ordered_by_magnitude_bits(G, oracle, d, path):
    """NaN > Inf > finite > denormal > zero, +0 ties with -0, values copied bit for bit."""
    import paper_2209_15203_amd as bts
    rng = np.random.default_rng(2)
    x = rng.standard_normal(d).astype(np.float32)
    xb = x.view(np.uint32)
    xb[10] = 0x7FC00001          # NaN with payload
    xb[20] = 0xFFC00000          # negative NaN
    xb[30] = 0x7F800000          # +Inf
    xb[40] = 0xFF800000          # -Inf
    xb[50:60] = 0x00000003       # denormals
    xb[60:70] = 0x80000003
    xb[100:200] = 0x80000000     # -0
    xb[200:300] = 0x00000000     # +0
    x[300:4000] = 0.0
    D = G.dev()
    ks = (1, 2, 3, 4, 5, 4000, 5285, 5290, 5300, 5320, 8990, d) if d < 10_000 else \
        (1, 2, 3, 4, 5, 100, 3000)
    for K in ks:
        ctx = bts.BtsContext(1, d, K, K)
        ctx.set_path(path)
        t = torch.from_numpy(x.copy()).to(D)
        oi = torch.zeros(K, dtype=torch.int32, device=D)
        ov = torch.zeros(K, dtype=torch.float32, device=D)
        bts.downlink_topk(ctx, t, oi, ov)
        torch.cuda.synchronize()
        h = x.copy()
        wi, wv = oracle.downlink(h, K)
        G.assert_same_bits(oi, wi, f"K={K} idx")
        G.assert_same_bits(ov, wv, f"K={K} val")
        G.assert_same_bits(t, h, f"K={K} residual")


def test_denormals_survive_error_compensation(G, oracle):
    import paper_2209_15203_amd as bts
    rng = np.random.default_rng(3)
    N, d, K = 2, 4100, 40
    g = (rng.standard_normal((N, d)) * 1e-38).astype(np.float32)      # products are denormal
    e = (rng.standard_normal((N, d)) * 1e-40).astype(np.float32)
    D = G.dev()
    ctx = bts.BtsContext(N, d, K, K)
    tg, te = torch.from_numpy(g).to(D), torch.from_numpy(e).to(D)
    ui = torch.zeros((N, K), dtype=torch.int32, device=D)
    uv = torch.zeros((N, K), dtype=torch.float32, device=D)
    bts.topk_compress(ctx, tg, te, 0.01, ui, uv)
    torch.cuda.synchronize()
    h = e.copy()
    wi, wv = oracle.worker_stage(g, h, 0.01, K)
    assert np.count_nonzero(h) > d, "the expected residuals must contain denormals"
    G.assert_same_bits(ui, wi, "up_idx")
    G.assert_same_bits(uv, wv, "up_val")
    G.assert_same_bits(te, h, "eps")


@pytest.mark.parametrize("N,d,K", [(1, 100, 10), (4, 5000, 50), (16, 200_003, 2001),
                                   (64, 50_001, 500), (300, 4096, 64)])
def test_sparse_aggregate(G, oracle, N, d, K):
    """Fixed worker order, one fused multiply-add per term, non-dyadic weights, heavy
    collisions between workers; untouched coordinates (including -0) keep their bits."""
    import paper_2209_15203_amd as bts
    rng = np.random.default_rng(N + d + K)
    # concentrate the indices so that many workers hit the same coordinates
    hot = max(K, d // 8)
    up_idx = np.stack([np.sort(rng.choice(hot, size=K, replace=False)) for _ in range(N)]
                      ).astype(np.uint32)
    up_idx[N // 2:] += np.uint32(d - hot)          # second half of the workers at the far end
    up_val = rng.standard_normal((N, K)).astype(np.float32)
    p = rng.dirichlet(np.ones(N)).astype(np.float32)
    delta = (rng.standard_normal(d) * 0.1).astype(np.float32)
    delta[::7] = -0.0
    D = G.dev()
    ctx = bts.BtsContext(N, d, K, K)
    ti = torch.from_numpy(up_idx.view(np.int32)).to(D)
    tv, tp, td = (torch.from_numpy(a).to(D) for a in (up_val, p, delta))
    nnz = torch.zeros(1, dtype=torch.int32, device=D)
    bts.sparse_aggregate(ctx, ti, tv, tp, td, nnz)
    torch.cuda.synchronize()
    h = delta.copy()
    want_nnz = oracle.aggregate(up_idx, up_val, p, h)
    G.assert_same_bits(td, h, "g_t")
    assert int(nnz.item()) == want_nnz
    # union_nnz is optional
    td2 = torch.from_numpy(delta).to(D)
    bts.sparse_aggregate(ctx, ti, tv, tp, td2, None)
    torch.cuda.synchronize()
    G.assert_same_bits(td2, h, "g_t without union_nnz")


@pytest.mark.parametrize("N,d,K", [(64, 1500, 4), (130, 5000, 3), (200, 3000, 40)])
def test_sparse_aggregate_every_worker_names_the_same_coordinates(G, oracle, N, d, K):
    """The longest possible chain per coordinate: all N workers send the same indices, so
    every named coordinate takes N dependent fused multiply-adds in ascending q."""
    import paper_2209_15203_amd as bts
    rng = np.random.default_rng(7 * N + K)
    one = np.sort(rng.choice(d, size=K, replace=False)).astype(np.uint32)
    up_idx = np.tile(one, (N, 1))
    up_val = rng.standard_normal((N, K)).astype(np.float32)
    p = rng.dirichlet(np.ones(N)).astype(np.float32)
    delta = rng.standard_normal(d).astype(np.float32)
    D = G.dev()
    ctx = bts.BtsContext(N, d, K, K)
    ti = torch.from_numpy(up_idx.view(np.int32)).to(D)
    tv, tp, td = (torch.from_numpy(a).to(D) for a in (up_val, p, delta))
    nnz = torch.zeros(1, dtype=torch.int32, device=D)
    for _ in range(2):                      # the second call finds the tables and flags clean
        td.copy_(torch.from_numpy(delta))
        bts.sparse_aggregate(ctx, ti, tv, tp, td, nnz)
        torch.cuda.synchronize()
        h = delta.copy()
        want_nnz = oracle.aggregate(up_idx, up_val, p, h)
        G.assert_same_bits(td, h, "g_t")
        assert int(nnz.item()) == want_nnz == K


def test_sparse_sgd_update(G, oracle):
    import paper_2209_15203_amd as bts
    rng = np.random.default_rng(4)
    d, K = 100_000, 777
    idx = np.sort(rng.choice(d, K, replace=False)).astype(np.uint32)
    val = rng.standard_normal(K).astype(np.float32)
    w = rng.standard_normal(d).astype(np.float32)
    D = G.dev()
    ctx = bts.BtsContext(1, d, K, K)
    tw = torch.from_numpy(w).to(D)
    bts.sparse_sgd_update(ctx, torch.from_numpy(idx.view(np.int32)).to(D),
                          torch.from_numpy(val).to(D), K, 0.013, tw)
    torch.cuda.synchronize()
    h = w.copy()
    oracle.update(idx, val, 0.013, h)
    G.assert_same_bits(tw, h, "w")


SMALL = {"C1": 70_001, "C2": 120_002, "C3": 90_008, "C4": 70_003, "C5": 150_000}


@pytest.mark.parametrize("name", ["C1", "C2", "C3", "C4", "C5"])
@pytest.mark.parametrize("mode", ["paper", "literal"])
@pytest.mark.parametrize("path", [DENSE, SINGLE_PASS, THREE_LAUNCH])
def test_bidir_step_scaled_configs(G, oracle, name, mode, path):
    """Each benchmark recipe at a d the oracle finishes in seconds (several chunks and a
    ragged tail), a few steps with carried residuals, in the paper's form
    (alpha inside a^q, update without alpha) and in the form with the step size applied at
    the update."""
    cfg = wl.CONFIGS[name].scaled(SMALL[name], steps=3)
    if cfg.N > 16:
        cfg = wl.CONFIGS[name].scaled(SMALL[name], N=16, steps=3)
    a_in, a_out = (cfg.alpha, 1.0) if mode == "paper" else (1.0, cfg.alpha)
    src = wl.GradientSource(cfg, G.dev())
    p = wl.p_weights(cfg) if cfg.N == wl.CONFIGS[name].N else \
        wl.p_weights(wl.CONFIGS[name])[:cfg.N].copy()
    st = G.GpuState(cfg.N, cfg.d, cfg.K_up, cfg.K_dn, wl.weights0(cfg, "cpu").numpy(), p)
    st.ctx.set_path(path)
    for t in range(1, cfg.steps + 1):
        st.step_and_compare(oracle, src.step(t), a_in, a_out, f"{cfg.name} step {t}")
        if path == SINGLE_PASS:
            assert st.ctx.last_path(0)[0] > 0, "no uplink row took the single-pass path"


@pytest.mark.parametrize("name", ["C1", "C2", "C3", "C4", "C5"])
@pytest.mark.parametrize("path", [DENSE, SINGLE_PASS, THREE_LAUNCH])
def test_unidir_step_scaled_configs(G, oracle, name, path):
    """Algorithm 1 (the paper's unidirectional baseline) as its own entry point: worker
    compression, then w -= alpha_out * sum_q p_q Top_K(a^q) with the sum returned as a
    sparse message; every output bit for bit against the oracle over three steps."""
    import paper_2209_15203_amd as bts
    cfg = wl.CONFIGS[name].scaled(SMALL[name], N=min(wl.CONFIGS[name].N, 16), steps=3)
    D = G.dev()
    src = wl.GradientSource(cfg, D)
    p = wl.p_weights(wl.CONFIGS[name])[:cfg.N].copy()
    N, d, K = cfg.N, cfg.d, cfg.K_up
    ctx = bts.BtsContext(N, d, K, K)
    ctx.set_path(path)
    eps = torch.zeros((N, d), device=D)
    w0 = wl.weights0(cfg, "cpu").numpy()
    w = torch.from_numpy(w0.copy()).to(D)
    tp = torch.from_numpy(p).to(D)
    ui = torch.zeros((N, K), dtype=torch.int32, device=D)
    uv = torch.zeros((N, K), device=D)
    di = torch.full((N * K,), -1, dtype=torch.int32, device=D)
    dv = torch.zeros(N * K, device=D)
    dc = torch.zeros(1, dtype=torch.int32, device=D)
    h_eps, h_w = np.zeros((N, d), np.float32), w0.copy()
    for t in range(1, 4):
        g = src.step(t)
        a_out = 1.0 if t < 3 else 0.5
        bts.unidir_step(ctx, g, eps, w, tp, cfg.alpha, a_out, ui, uv, di, dv, dc)
        torch.cuda.synchronize()
        want = oracle.unidir_step(g.cpu().numpy(), h_eps, h_w, p, K, cfg.alpha, a_out)
        n = int(dc.item())
        assert n == want["dn_count"]
        G.assert_same_bits(ui, want["up_idx"], f"step {t} up_idx")
        G.assert_same_bits(uv, want["up_val"], f"step {t} up_val")
        G.assert_same_bits(eps, h_eps, f"step {t} eps")
        G.assert_same_bits(di[:n], want["dn_idx"], f"step {t} message indices")
        G.assert_same_bits(dv[:n], want["dn_val"], f"step {t} message values")
        G.assert_same_bits(w, h_w, f"step {t} w")
    # the message is optional
    w2 = w.clone()
    g = src.step(4)
    e2 = eps.clone()
    bts.unidir_step(ctx, g, eps, w, tp, cfg.alpha, 1.0, ui, uv, di, dv, dc)
    bts.unidir_step(ctx, g, e2, w2, tp, cfg.alpha, 1.0, ui, uv, None, None, None)
    torch.cuda.synchronize()
    assert torch.equal(w.view(torch.int32), w2.view(torch.int32))


def test_bidir_step_equals_the_four_calls_and_is_deterministic(G):
    import paper_2209_15203_amd as bts
    cfg = wl.CONFIGS["C4"].scaled(80_005, N=8, steps=2)
    D = G.dev()
    src = wl.GradientSource(cfg, D)
    p = torch.from_numpy(wl.p_weights(wl.CONFIGS["C4"])[:8].copy()).to(D)
    runs = []
    for variant in ("step", "calls", "step", "dense"):
        ctx = bts.BtsContext(cfg.N, cfg.d, cfg.K_up, cfg.K_dn)
        ctx.set_path(DENSE if variant == "dense" else SINGLE_PASS)
        eps = torch.zeros((cfg.N, cfg.d), device=D)
        delta = torch.zeros(cfg.d, device=D)
        w = wl.weights0(cfg, D)
        ui = torch.zeros((cfg.N, cfg.K_up), dtype=torch.int32, device=D)
        uv = torch.zeros((cfg.N, cfg.K_up), device=D)
        di = torch.zeros(cfg.K_dn, dtype=torch.int32, device=D)
        dv = torch.zeros(cfg.K_dn, device=D)
        for t in (1, 2):
            g = src.step(t)
            if variant in ("step", "dense"):
                bts.bidir_step(ctx, g, eps, delta, w, p, cfg.alpha, 1.0, ui, uv, di, dv, None)
            else:
                bts.topk_compress(ctx, g, eps, cfg.alpha, ui, uv)
                bts.sparse_aggregate(ctx, ui, uv, p, delta, None)
                bts.downlink_topk(ctx, delta, di, dv)
                bts.sparse_sgd_update(ctx, di, dv, cfg.K_dn, 1.0, w)
        torch.cuda.synchronize()
        runs.append([t.clone() for t in (eps, delta, w, ui, uv, di, dv)])
    for other in runs[1:]:
        for a, b in zip(runs[0], other):
            assert torch.equal(a.view(torch.int32), b.view(torch.int32))


def test_misaligned_buffers_are_rejected(G):
    import paper_2209_15203_amd as bts
    D = G.dev()
    ctx = bts.BtsContext(1, 64, 4, 4)
    buf = torch.zeros(65 + 4, device=D)
    off = buf[1:65]                      # 4-byte aligned only
    ui = torch.zeros(4, dtype=torch.int32, device=D)
    uv = torch.zeros(4, device=D)
    with pytest.raises(bts.BtsError):
        bts.downlink_topk(ctx, off, ui, uv)
    with pytest.raises(bts.BtsError):
        bts.topk_compress(ctx, off, torch.zeros(64, device=D), 1.0, ui, uv)


def _fresh_state(cfg, D):
    return dict(eps=torch.zeros((cfg.N, cfg.d), device=D), delta=torch.zeros(cfg.d, device=D),
                w=wl.weights0(cfg, D), ui=torch.zeros((cfg.N, cfg.K_up), dtype=torch.int32, device=D),
                uv=torch.zeros((cfg.N, cfg.K_up), device=D),
                di=torch.zeros(cfg.K_dn, dtype=torch.int32, device=D),
                dv=torch.zeros(cfg.K_dn, device=D))


def _step(bts, ctx, st, g, p, alpha):
    bts.bidir_step(ctx, g, st["eps"], st["delta"], st["w"], p, alpha, 1.0, st["ui"], st["uv"],
                   st["di"], st["dv"], None)


def test_resume_from_copied_state_and_path_switching(G, oracle):
    """The state of the algorithm lives in the caller's buffers only: four steps in one go
    equal two steps, a copy of (eps, delta, w) into new buffers and a NEW context, and two
    more steps.  The first run also switches the select path every step, which checks that
    each path leaves the shared scratch (directory, counters, histograms) clean."""
    import paper_2209_15203_amd as bts
    cfg = wl.CONFIGS["C3"].scaled(300_007, N=6, steps=4)
    D = G.dev()
    src = wl.GradientSource(cfg, D)
    p = torch.full((cfg.N,), 1.0 / cfg.N, device=D)
    gs = [src.step(t) for t in range(1, 5)]
    a = _fresh_state(cfg, D)
    ctx = bts.BtsContext(cfg.N, cfg.d, cfg.K_up, cfg.K_dn)
    for t, mode in enumerate((SINGLE_PASS, THREE_LAUNCH, DENSE, 0)):
        ctx.set_path(mode)
        _step(bts, ctx, a, gs[t], p, cfg.alpha)
    b = _fresh_state(cfg, D)
    ctx1 = bts.BtsContext(cfg.N, cfg.d, cfg.K_up, cfg.K_dn)
    ctx1.set_path(DENSE)
    for t in range(2):
        _step(bts, ctx1, b, gs[t], p, cfg.alpha)
    torch.cuda.synchronize()
    c = _fresh_state(cfg, D)
    for k in ("eps", "delta", "w"):
        c[k].copy_(b[k])
    ctx1.close()
    ctx2 = bts.BtsContext(cfg.N, cfg.d, cfg.K_up, cfg.K_dn)
    ctx2.set_path(SINGLE_PASS)
    for t in range(2, 4):
        _step(bts, ctx2, c, gs[t], p, cfg.alpha)
    torch.cuda.synchronize()
    for k in a:
        assert torch.equal(a[k].view(torch.int32), c[k].view(torch.int32)), k
    # and against the oracle
    h_eps = np.zeros((cfg.N, cfg.d), np.float32)
    h_delta = np.zeros(cfg.d, np.float32)
    h_w = wl.weights0(cfg, D).cpu().numpy().copy()      # the very buffer the GPU started from
    for t in range(4):
        oracle.bidir_step(gs[t].cpu().numpy(), h_eps, h_delta, h_w, p.cpu().numpy(), cfg.K_up,
                          cfg.K_dn, cfg.alpha, 1.0)
    G.assert_same_bits(a["eps"], h_eps, "eps")
    G.assert_same_bits(a["delta"], h_delta, "delta")
    G.assert_same_bits(a["w"], h_w, "w")


def test_two_contexts_on_two_streams(G):
    """Two independent problems queued on two HIP streams (default priority) at the same
    time give the same bits as running them one after the other."""
    import paper_2209_15203_amd as bts
    D = G.dev()
    cfgs = [wl.CONFIGS["C1"].scaled(400_003, N=5, steps=3), wl.CONFIGS["C4"].scaled(250_001, N=7, steps=3)]
    streams = [torch.cuda.Stream(device=D), torch.cuda.Stream(device=D)]
    serial, overlapped = [], []
    for run in ("serial", "overlapped"):
        states, ctxs, gsets, ps = [], [], [], []
        for cfg in cfgs:
            src = wl.GradientSource(cfg, D)
            gsets.append([src.step(t) for t in (1, 2, 3)])
            ps.append(torch.full((cfg.N,), 1.0 / cfg.N, device=D))
            states.append(_fresh_state(cfg, D))
        torch.cuda.synchronize()
        for cfg, s in zip(cfgs, streams):
            ctx = bts.BtsContext(cfg.N, cfg.d, cfg.K_up, cfg.K_dn, stream=s)
            ctx.set_path(SINGLE_PASS)
            ctxs.append(ctx)
        if run == "serial":
            for i in range(2):
                for t in range(3):
                    _step(bts, ctxs[i], states[i], gsets[i][t], ps[i], 0.01)
                streams[i].synchronize()
        else:
            for t in range(3):
                for i in range(2):
                    _step(bts, ctxs[i], states[i], gsets[i][t], ps[i], 0.01)
            for s in streams:
                s.synchronize()
        (serial if run == "serial" else overlapped).extend(states)
    for sa, sb in zip(serial, overlapped):
        for k in sa:
            assert torch.equal(sa[k].view(torch.int32), sb[k].view(torch.int32)), k


def test_bidir_step_replays_from_a_hip_graph(G, oracle):
    """The step queues kernels only (no host synchronisation, no memset nodes), so it can be
    captured once into a HIP graph and replayed.  Every replay, with fresh gradients copied
    into the captured input buffer and ordinary eager work in between, must give the same
    bits as the oracle."""
    import paper_2209_15203_amd as bts
    cfg = wl.CONFIGS["C2"].scaled(400_002, N=6, steps=5)
    D = G.dev()
    src = wl.GradientSource(cfg, D)
    p_host = np.full(cfg.N, 1.0 / cfg.N, np.float32)
    p = torch.from_numpy(p_host).to(D)
    side = torch.cuda.Stream(device=D)
    st = _fresh_state(cfg, D)
    w0 = st["w"].cpu().numpy().copy()
    g_static = torch.zeros((cfg.N, cfg.d), device=D)
    ctx = bts.BtsContext(cfg.N, cfg.d, cfg.K_up, cfg.K_dn, stream=side)
    ctx.set_path(SINGLE_PASS)
    h_eps = np.zeros((cfg.N, cfg.d), np.float32)
    h_delta = np.zeros(cfg.d, np.float32)
    h_w = w0
    # one eager step first (warm-up outside the capture), checked like the replays
    steps = [src.step(t) for t in range(1, 6)]
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    for t, g in enumerate(steps):
        g_static.copy_(g)
        torch.cuda.synchronize()
        if t == 0:
            with torch.cuda.stream(side):
                _step(bts, ctx, st, g_static, p, cfg.alpha)
            side.synchronize()
        elif t == 1:
            with torch.cuda.graph(graph, stream=side):
                _step(bts, ctx, st, g_static, p, cfg.alpha)
            graph.replay()          # capture records, replay runs
        else:
            _ = (g_static * 2.0).sum().item()      # unrelated eager work between replays
            graph.replay()
        torch.cuda.synchronize()
        want = oracle.bidir_step(g.cpu().numpy(), h_eps, h_delta, h_w, p_host, cfg.K_up,
                                 cfg.K_dn, cfg.alpha, 1.0)
        G.assert_same_bits(st["ui"], want["up_idx"], f"replay {t} up_idx")
        G.assert_same_bits(st["eps"], h_eps, f"replay {t} eps")
        G.assert_same_bits(st["di"], want["dn_idx"], f"replay {t} dn_idx")
        G.assert_same_bits(st["dv"], want["dn_val"], f"replay {t} dn_val")
        G.assert_same_bits(st["delta"], h_delta, f"replay {t} delta")
        G.assert_same_bits(st["w"], h_w, f"replay {t} w")

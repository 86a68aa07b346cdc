"""topk_compress_noalloc (the entry point that allocates nothing) against topk_compress.

Called through the C ABI with ctypes, on two calls in a row, the second with a smaller
input: the fixed scratch array keeps the first call's contents, and the second call must
not be disturbed by them.  Every output must equal topk_compress's bit for bit (and, as a
cross-check, the CPU oracle's).
"""
import ctypes as C

import numpy as np
import pytest
import torch

pytestmark = pytest.mark.gpu

# (N, d, K_up, alpha): the second is smaller in every dimension; the third goes back up
# with ragged rows (d % 4 != 0) and ties at the threshold
CALLS = [(8, 300_007, 300, 0.37), (3, 70_001, 70, 0.01), (5, 262_147, 5000, 1.0)]


def _rows(rng, N, d, ties):
    if ties:
        mag = rng.integers(1, 4, size=(N, d)).astype(np.float32)
        return mag * rng.choice(np.array([-1.0, 1.0], np.float32), size=(N, d)), \
            np.zeros((N, d), np.float32)
    return (rng.standard_normal((N, d)).astype(np.float32),
            (0.5 * rng.standard_normal((N, d))).astype(np.float32))


def test_noalloc_matches_topk_compress_on_consecutive_calls(oracle):
    import _gpu_util as G
    import paper_2209_15203_amd as bts
    lib = bts.load_library()
    D = G.dev()
    stream = torch.cuda.current_stream()
    rng = np.random.default_rng(20221001)
    for n_call, (N, d, K, alpha) in enumerate(CALLS):
        g, eps0 = _rows(rng, N, d, ties=(n_call == 2))
        tg = torch.from_numpy(g).to(D)
        # the existing entry point, on a context
        e_ref = torch.from_numpy(eps0).to(D)
        i_ref = torch.full((N, K), -1, dtype=torch.int32, device=D)
        v_ref = torch.zeros((N, K), dtype=torch.float32, device=D)
        with bts.BtsContext(N, d, K, K) as ctx:
            bts.topk_compress(ctx, tg, e_ref, alpha, i_ref, v_ref)
            torch.cuda.synchronize()
        # the entry point that allocates nothing, straight through the C ABI
        e_new = torch.from_numpy(eps0).to(D)
        i_new = torch.full((N, K), -1, dtype=torch.int32, device=D)
        v_new = torch.zeros((N, K), dtype=torch.float32, device=D)
        print(f"[noalloc] call {n_call}: N={N} d={d} K={K}", flush=True)
        rc = lib.topk_compress_noalloc(C.c_void_p(tg.data_ptr()), C.c_void_p(e_new.data_ptr()),
                                       N, d, K, alpha, C.c_void_p(i_new.data_ptr()),
                                       C.c_void_p(v_new.data_ptr()),
                                       C.c_void_p(stream.cuda_stream))
        assert rc == 0, rc
        torch.cuda.synchronize()
        tag = f"call {n_call}"
        G.assert_same_bits(i_new, i_ref, f"{tag} up_idx")
        G.assert_same_bits(v_new, v_ref, f"{tag} up_val")
        G.assert_same_bits(e_new, e_ref, f"{tag} eps")
        G.assert_same_bits(tg, g, f"{tag} g must not be modified")
        h_eps = eps0.copy()
        want_i, want_v = oracle.worker_stage(g, h_eps, alpha, K)
        G.assert_same_bits(i_new, want_i, f"{tag} up_idx vs oracle")
        G.assert_same_bits(v_new, want_v, f"{tag} up_val vs oracle")
        G.assert_same_bits(e_new, h_eps, f"{tag} eps vs oracle")


def test_noalloc_rejects_shapes_beyond_its_scratch_and_k_zero_works(oracle):
    import _gpu_util as G
    import paper_2209_15203_amd as bts
    lib = bts.load_library()
    D = G.dev()
    x = torch.zeros(1024, dtype=torch.float32, device=D)
    i = torch.zeros(16, dtype=torch.int32, device=D)
    p = lambda t: C.c_void_p(t.data_ptr())
    # more rows than the scratch serves; more wave chunks than it serves (nothing is read:
    # the call returns before it queues anything)
    assert lib.topk_compress_noalloc(p(x), p(x), 257, 4, 1, 1.0, p(i), p(x), None) == -4
    assert lib.topk_compress_noalloc(p(x), p(x), 2, 400_000_000, 1, 1.0, p(i), p(x), None) == -4
    assert lib.topk_compress_noalloc(p(x), p(x), 0, 4, 1, 1.0, p(i), p(x), None) == -1
    assert lib.topk_compress_noalloc(None, p(x), 1, 4, 1, 1.0, p(i), p(x), None) == -1
    assert lib.topk_compress_noalloc(p(x), p(x), 1, 4, 5, 1.0, p(i), p(x), None) == -1
    # K = 0: plain error accumulation
    rng = np.random.default_rng(3)
    g = rng.standard_normal((3, 5001)).astype(np.float32)
    e = rng.standard_normal((3, 5001)).astype(np.float32)
    tg, te = torch.from_numpy(g).to(D), torch.from_numpy(e).to(D)
    bts.topk_compress_noalloc(tg, te, 0.01, None, None)
    torch.cuda.synchronize()
    h = e.copy()
    oracle.worker_stage(g, h, 0.01, 0)
    G.assert_same_bits(te, h, "eps")

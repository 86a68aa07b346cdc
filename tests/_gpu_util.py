"""Shared helpers of the GPU parity tests: run the HIP library through its Python binding
and compare every output with the CPU oracle bit for bit (as uint32 words)."""
from __future__ import annotations

import numpy as np
import torch

import paper_2209_15203_amd as bts


def dev():
    return torch.device("cuda:0")


def bits(a) -> np.ndarray:
    if isinstance(a, torch.Tensor):
        a = a.detach().cpu().numpy()
    a = np.ascontiguousarray(a)
    return a.view(np.uint32) if a.dtype != np.uint32 else a


def assert_same_bits(got, want, what: str):
    g, w = bits(got), bits(want)
    assert g.shape == w.shape, f"{what}: shape {g.shape} vs {w.shape}"
    if not np.array_equal(g, w):
        bad = np.flatnonzero(g.ravel() != w.ravel())
        raise AssertionError(f"{what}: {bad.size} of {g.size} words differ, first at flat index "
                             f"{bad[0]}: got 0x{int(g.ravel()[bad[0]]):08x} "
                             f"want 0x{int(w.ravel()[bad[0]]):08x}")


class GpuState:
    """Device buffers of one problem (state + messages) next to a host copy for the oracle."""

    def __init__(self, N, d, K_up, K_dn, w0: np.ndarray, p: np.ndarray):
        self.N, self.d, self.K_up, self.K_dn = N, d, K_up, K_dn
        D = dev()
        self.ctx = bts.BtsContext(N, d, K_up, K_dn)
        self.eps = torch.zeros((N, d), dtype=torch.float32, device=D)
        self.delta = torch.zeros(d, dtype=torch.float32, device=D)
        self.w = torch.from_numpy(w0.copy()).to(D)
        self.p = torch.from_numpy(p.copy()).to(D)
        self.up_idx = torch.full((N, max(K_up, 1)), -1, dtype=torch.int32, device=D)[:, :K_up].contiguous() \
            if K_up else torch.empty((N, 0), dtype=torch.int32, device=D)
        self.up_val = torch.zeros((N, K_up), dtype=torch.float32, device=D)
        self.dn_idx = torch.full((max(K_dn, 1),), -1, dtype=torch.int32, device=D)[:K_dn].contiguous()
        self.dn_val = torch.zeros(K_dn, dtype=torch.float32, device=D)
        self.nnz = torch.zeros(1, dtype=torch.int32, device=D)
        # oracle side
        self.h_eps = np.zeros((N, d), np.float32)
        self.h_delta = np.zeros(d, np.float32)
        self.h_w = w0.copy()
        self.h_p = p.copy()

    def step_and_compare(self, oracle, g: torch.Tensor, alpha_in: float, alpha_out: float,
                         tag: str = ""):
        bts.bidir_step(self.ctx, g, self.eps, self.delta, self.w, self.p, alpha_in, alpha_out,
                       self.up_idx, self.up_val, self.dn_idx, self.dn_val, self.nnz)
        torch.cuda.synchronize()
        want = oracle.bidir_step(g.cpu().numpy(), self.h_eps, self.h_delta, self.h_w, self.h_p,
                                 self.K_up, self.K_dn, alpha_in, alpha_out)
        assert_same_bits(self.up_idx, want["up_idx"], f"{tag} up_idx")
        assert_same_bits(self.up_val, want["up_val"], f"{tag} up_val")
        assert_same_bits(self.eps, self.h_eps, f"{tag} eps")
        assert_same_bits(self.dn_idx, want["dn_idx"], f"{tag} dn_idx")
        assert_same_bits(self.dn_val, want["dn_val"], f"{tag} dn_val")
        assert_same_bits(self.delta, self.h_delta, f"{tag} delta")
        assert_same_bits(self.w, self.h_w, f"{tag} w")
        assert int(self.nnz.item()) == want["union_nnz"], f"{tag} union_nnz"
        return want

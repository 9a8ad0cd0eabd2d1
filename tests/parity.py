"""Shared helpers of the GPU parity tests: run one layer through the C ABI and compare it
with the CPU oracle on the same seeded inputs."""
from __future__ import annotations

import numpy as np
import torch

from oracle import hgf_oracle as orc
from paper_2602_05269_amd import binding as hb

ATOL, RTOL = 2e-3, 1e-2      # fp16 outputs: |y_gpu - y_ref| <= ATOL + RTOL * |y_ref|


def dev(a: np.ndarray) -> torch.Tensor:
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def assert_close_fp16(y_gpu: np.ndarray, y_ref: np.ndarray, what: str = "y", scale=None) -> None:
    """Elementwise |y_gpu - y_ref| <= ATOL + RTOL * scale, scale = |y_ref| unless given (a sum of
    the magnitudes of the two paths, where the output is a small difference of large terms)."""
    y_gpu = y_gpu.astype(np.float64)
    err = np.abs(y_gpu - y_ref)
    bound = ATOL + RTOL * (np.abs(y_ref) if scale is None else scale)
    bad = err > bound
    if bad.any():
        idx = np.argwhere(bad)
        where = ", ".join(f"axis {a}: {len(np.unique(idx[:, a]))} distinct in [{idx[:, a].min()}, {idx[:, a].max()}]"
                          for a in range(idx.shape[1]))
        worst = np.unravel_index(err.argmax(), err.shape)
        raise AssertionError(f"{what}: {int(bad.sum())} of {bad.size} outside tolerance ({where}); worst err "
                             f"{err.max():.3e} at {worst}: got {y_gpu[worst]!r}, reference {y_ref[worst]!r}")


class GpuLayer:
    """One synthetic case resident on the GPU, with the oracle's view of the same case."""

    def __init__(self, case: dict, ws: hb.Workspace | None = None, rank0: bool = False):
        self.case = case
        self.K, self.N = case["d_in"], case["d_out"]
        self.rank = 0 if rank0 else case["rank"]
        self.ws = ws or hb.Workspace(64, max(self.K, 64), max(self.N, 64), 128)
        self.W = dev(case["W"])
        A = B = alpha = None
        if self.rank:
            A, B, alpha = dev(case["A"]), dev(case["B"]), dev(case["alpha"])
        self.layer = hb.Layer.from_latent(self.W, A, B, alpha, self.ws)
        self.T_ref, self.s_w_ref = orc.ternarize(case["W"])

    def check_weights(self):
        T = hb.hgf_unpack_weights(self.layer.packed, self.N, self.K).cpu().numpy()
        s_w = self.layer.s_w.cpu().numpy()[0]
        assert s_w.view(np.uint32) == np.float32(self.s_w_ref).view(np.uint32), (s_w, self.s_w_ref)
        assert np.array_equal(T, self.T_ref)

    def forward(self, x: np.ndarray, ws: hb.Workspace | None = None):
        ws = ws or self.ws
        xd = dev(x)
        M = x.shape[0]
        acc = torch.full((M, self.N), -12345, dtype=torch.int32, device="cuda")
        y = hb.hgf_linear_forward(xd, self.layer, ws, acc_debug=acc)
        torch.cuda.synchronize()
        return y.cpu().numpy(), acc.cpu().numpy()

    def oracle(self, x: np.ndarray, rows=None, dense: bool = False):
        """The oracle's view of this layer on input x (on the sampled output rows `rows`).
        dense: the integer contraction by the BLAS product that the CPU tests prove equal
        to the oracle's triple loop (full-size cases, every element)."""
        c = self.case
        T, A, B, alpha = self.T_ref, c.get("A"), c.get("B"), c.get("alpha")
        if self.rank == 0:
            A = B = alpha = None
        if rows is not None:
            T = T[rows]
            if self.rank:
                B, alpha = B[rows], alpha[rows]
        return orc.linear_forward(x, T, self.s_w_ref, A, B, alpha, dense_gemm=dense)

    def check_forward(self, x: np.ndarray, rows=None, tokens=None, ws=None):
        y, acc = self.forward(x, ws)
        xo = x if tokens is None else x[tokens]
        ref = self.oracle(xo, rows)
        if tokens is not None:
            y, acc = y[tokens], acc[tokens]
        if rows is not None:
            y, acc = y[:, rows], acc[:, rows]
        assert np.array_equal(acc, ref["acc"]), "int32 accumulators differ from the oracle"
        assert_close_fp16(y, ref["y"])
        return y, ref

"""Helpers shared by the GPU parity tests (not collected by pytest)."""
from __future__ import annotations

import numpy as np

REL_FRO_TOL = 2e-3          # relative Frobenius error bound of the workload statement
ELEM_TOL = 1e-2             # per-element bound: |err| <= 1e-2 * max|C_ref|


def dev(x: np.ndarray):
    import torch
    return torch.from_numpy(np.ascontiguousarray(x)).cuda()


class DeviceProblem:
    """Inputs of one problem on the GPU plus an output buffer pre-filled with NaN, so a
    kernel that leaves an element unwritten is caught."""

    def __init__(self, A, qweight, scales, qzeros, group_size):
        import torch
        self.m, self.k = A.shape
        self.n = qweight.shape[1]
        self.g = group_size
        self.A, self.qweight, self.scales, self.qzeros = dev(A), dev(qweight), dev(scales), dev(qzeros)
        self.C = torch.full((self.m, self.n), float("nan"), dtype=torch.float16, device="cuda")

    def args(self):
        return (self.A, self.qweight, self.scales, self.qzeros, self.C, self.m, self.n, self.k, self.g)

    def result(self) -> np.ndarray:
        import torch
        torch.cuda.synchronize()
        return self.C.cpu().numpy()


def assert_parity(C_gpu: np.ndarray, Cref: np.ndarray, what: str = ""):
    """GPU fp16 output against the oracle's fp64 result, element by element."""
    got = C_gpu.astype(np.float64)
    assert np.isfinite(got).all(), f"{what}: non-finite output"
    err = got - Cref
    ref_norm = np.linalg.norm(Cref)
    rel = np.linalg.norm(err) / ref_norm if ref_norm > 0 else np.linalg.norm(err)
    amax = np.abs(Cref).max()
    emax = np.abs(err).max()
    assert rel <= REL_FRO_TOL, f"{what}: relative Frobenius error {rel:.3e} > {REL_FRO_TOL}"
    assert emax <= ELEM_TOL * amax + 1e-30, f"{what}: max |err| {emax:.3e} > {ELEM_TOL} * {amax:.3e}"
    return rel, emax

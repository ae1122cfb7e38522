"""Two independently written CPU implementations on the five workload configurations (no GPU):
the C oracle (the definition, one element at a time) against a numpy restatement (byte-view
unpackers written with array operations, dense float64 weight, numpy's matmul), to 1e-6 relative.
Configuration 5 is checked on a 512-column slice, which has the full k = 16384.
Also: the stored tiny fixture is what its committed generator writes.
"""
import importlib.util
import pathlib

import numpy as np
import pytest

import oracle_pins
from paper_2402_00025_amd.inputs import make_inputs

GOLDEN = pathlib.Path(__file__).resolve().parent / "golden"


def _restatement(A, qweight, scales, qzeros, g, col_block=1024):
    """numpy float64 product, in column blocks so that the dense weight stays small."""
    m, n = A.shape[0], qweight.shape[1]
    out = np.empty((m, n), np.float64)
    A64 = A.astype(np.float64)
    for j0 in range(0, n, col_block):
        j1 = min(j0 + col_block, n)
        W = oracle_pins.np_dense_weight(qweight[:, j0:j1], scales[:, j0:j1], qzeros[:, j0 // 8:j1 // 8], g)
        out[:, j0:j1] = A64 @ W
    return out


CONFIGS = [
    ("cfg1", 1, 1024, 1024, None),
    ("cfg2", 16, 4096, 4096, None),
    ("cfg3_4096_rows", 16, 4096, 4096, (1, 2, 4, 8)),
    ("cfg4_and_cfg3_8192", 16, 8192, 8192, (1, 2, 4, 8)),
    ("cfg5_slice", 8, 16384, 16384, None),
]


@pytest.mark.parametrize("name,m,n,k,row_subsets", CONFIGS, ids=[c[0] for c in CONFIGS])
def test_c_oracle_agrees_with_numpy_restatement(oracle, name, m, n, k, row_subsets):
    g = 128
    x = make_inputs(m, n, k, g, seed=0)
    qw, s, qz = x.qweight, x.scales, x.qzeros
    if name == "cfg5_slice":
        qw, s, qz = (np.ascontiguousarray(t) for t in (qw[:, :512], s[:, :512], qz[:, :64]))
    ref = _restatement(x.A, qw, s, qz, g)
    scale = np.abs(ref).max()
    Cref, C16 = oracle.gemm(x.A, qw, s, qz, g)
    assert np.abs(Cref - ref).max() <= 1e-6 * scale
    assert np.linalg.norm(Cref - ref) <= 1e-6 * np.linalg.norm(ref)
    # the fp16 output is the single rounding of the fp64 result
    assert np.array_equal(C16.view(np.uint16), Cref.astype(np.float16).view(np.uint16))
    # Algorithm 1's fp32 accumulator stays inside its forward error bound at full size
    if name in ("cfg1", "cfg2"):
        C32, _ = oracle.gemm(x.A, qw, s, qz, g, acc="f32")
        assert np.abs(C32 - ref).max() <= 1e-4 * scale
    # fewer activation rows (the m sweep of configuration 3): the same rows of the result
    for rows in row_subsets or ():
        Cm, _ = oracle.gemm(np.ascontiguousarray(x.A[:rows]), qw, s, qz, g)
        assert np.array_equal(Cm.view(np.uint64), Cref[:rows].view(np.uint64))


def test_tiny_fixture_is_what_its_generator_writes():
    spec = importlib.util.spec_from_file_location("make_tiny_fixture", GOLDEN / "make_tiny_fixture.py")
    mod = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(mod)
    assert mod.fixture_text() == (GOLDEN / "tiny_m2_n16_k16_g8.txt").read_text()

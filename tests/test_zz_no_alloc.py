"""w4a16_gemm_static, the entry point that allocates nothing (its split-k state lives in a static
device array), through the C ABI against w4a16_gemm, the entry point it is a variant of: two calls
in a row, the second with a smaller input, for the fixed-point reduction (up to four rows:
order-independent, so bit for bit) and for the packed-fp16 adds with in-kernel zeroing (to the
parity tolerance, and both against the oracle)."""
import ctypes

import numpy as np
import pytest

from gpu_util import DeviceProblem, assert_parity
from paper_2402_00025_amd import binding as b
from paper_2402_00025_amd.inputs import make_inputs

pytestmark = pytest.mark.gpu


def _raw_static(p, split_k):
    """The raw C ABI call: plain pointers and sizes, return code checked here."""
    import torch
    L = b.lib()
    vp = ctypes.c_void_p
    rc = L.w4a16_gemm_static(vp(p.A.data_ptr()), vp(p.qweight.data_ptr()), vp(p.scales.data_ptr()),
                             vp(p.qzeros.data_ptr()), vp(p.C.data_ptr()), p.m, p.n, p.k, p.g, split_k,
                             vp(torch.cuda.current_stream().cuda_stream))
    assert rc == b.OK, b.strerror(rc)


def _pair(oracle, m, n, k, split_k, seed, exact):
    x = make_inputs(m, n, k, 128, seed=seed)
    Cref, _ = oracle.gemm(x.A, x.qweight, x.scales, x.qzeros, 128)
    p = DeviceProblem(x.A, x.qweight, x.scales, x.qzeros, 128)
    b.w4a16_gemm(*p.args(), split_k)
    want = p.result().copy()
    p.C.fill_(float("nan"))
    _raw_static(p, split_k)
    got = p.result().copy()
    what = f"static m={m} n={n} k={k} S={split_k}"
    assert_parity(got, Cref, what)
    assert_parity(want, Cref, what + " (w4a16_gemm)")
    if exact:
        assert np.array_equal(got.view(np.uint16), want.view(np.uint16)), what
    else:
        # two runs of packed-fp16 atomics differ by their rounding order only
        assert_parity(got, want.astype(np.float64), what + " against w4a16_gemm")
    return p


def test_static_entry_two_calls_second_smaller(oracle):
    import torch
    assert torch.cuda.is_available()
    # sixteen rows: packed-fp16 adds, zeroing protocol in the static array (library's split, then a given one)
    _pair(oracle, 16, 4096, 4096, 0, 0, exact=False)
    _pair(oracle, 16, 1032, 2048, 4, 1, exact=False)
    # up to four rows: fixed-point words in the static array
    _pair(oracle, 1, 4096, 4096, 4, 2, exact=True)     # a given split: 64-column tiles, fixed-point words
    _pair(oracle, 1, 4096, 4096, 0, 6, exact=False)    # the library's split: two strips per wave at one row as well
    _pair(oracle, 3, 1024, 1024, 4, 3, exact=True)
    # the streaming kernel's protocol (a larger matrix), then a small one again
    _pair(oracle, 8, 8192, 8192, 0, 4, exact=False)
    _pair(oracle, 5, 520, 1024, 2, 5, exact=False)
    assert b.w4a16_phase_timeouts() == 0


def test_static_entry_repeats_and_allocates_nothing(oracle):
    """The same buffers again and again (the array keeps the last call's state), with the free
    device memory unchanged over the calls."""
    import torch
    x = make_inputs(16, 2048, 4096, 128, seed=7)
    Cref, _ = oracle.gemm(x.A, x.qweight, x.scales, x.qzeros, 128)
    p = DeviceProblem(x.A, x.qweight, x.scales, x.qzeros, 128)
    x2 = make_inputs(3, 1024, 2048, 128, seed=8)
    Cref2, _ = oracle.gemm(x2.A, x2.qweight, x2.scales, x2.qzeros, 128)
    p2 = DeviceProblem(x2.A, x2.qweight, x2.scales, x2.qzeros, 128)
    for p_, s_ in ((p, 0), (p2, 4)):   # warm: code objects loaded, static address resolved
        _raw_static(p_, s_)
    torch.cuda.synchronize()
    free_before, _ = torch.cuda.mem_get_info()
    for it in range(6):
        p.C.fill_(float("nan"))
        p2.C.fill_(float("nan"))
        _raw_static(p, 0)
        _raw_static(p2, 4)
        assert_parity(p.result(), Cref, f"repeat {it}")
        assert_parity(p2.result(), Cref2, f"repeat {it} small")
    free_after, _ = torch.cuda.mem_get_info()
    assert free_after == free_before
    assert b.w4a16_phase_timeouts() == 0


def test_static_entry_limits():
    import torch
    x = make_inputs(16, 1024, 8192, 128, seed=9)
    p = DeviceProblem(x.A, x.qweight, x.scales, x.qzeros, 128)
    L = b.lib()
    vp = ctypes.c_void_p
    args = [vp(t.data_ptr()) for t in (p.A, p.qweight, p.scales, p.qzeros, p.C)]
    st = vp(torch.cuda.current_stream().cuda_stream)
    # sixteen rows with 64 slices: the zeroing protocol's words for that split are not in the array
    assert L.w4a16_gemm_static(*args, 16, 1024, 8192, 128, 64, st) == b.ERR_LIMIT
    # four rows with 64 slices use the fixed-point words: inside the array
    assert L.w4a16_gemm_static(*args, 4, 1024, 8192, 128, 64, st) == b.OK
    torch.cuda.synchronize()

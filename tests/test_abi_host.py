"""The C-ABI library without a GPU: it loads, exports what include/w4a16.h declares, and its
argument checks and launch planning behave as the header says.  No compute call is made."""
import ctypes
import pathlib
import re

import pytest

from paper_2402_00025_amd import binding as b
from paper_2402_00025_amd import inputs

ROOT = pathlib.Path(__file__).resolve().parent.parent
HEADER = (ROOT / "include" / "w4a16.h").read_text()


def declared_functions():
    body = re.sub(r"/\*.*?\*/", "", HEADER, flags=re.S)
    return sorted(set(re.findall(r"\b(w[2348]a16_[a-z_0-9]+)\s*\(", body)))


def test_library_exports_every_declared_symbol():
    names = declared_functions()
    assert set(names) == set(b.EXPORTS)
    L = b.lib()
    for name in names:
        assert hasattr(L, name), name


def test_error_codes_match_header():
    for name, val in (("W4A16_OK", b.OK), ("W4A16_ERR_NULL", b.ERR_NULL), ("W4A16_ERR_SHAPE", b.ERR_SHAPE),
                      ("W4A16_ERR_SPLIT", b.ERR_SPLIT), ("W4A16_ERR_UNSUPPORTED", b.ERR_UNSUPPORTED),
                      ("W4A16_ERR_HIP", b.ERR_HIP), ("W4A16_ERR_STATE", b.ERR_STATE), ("W4A16_ERR_LIMIT", b.ERR_LIMIT),
                      ("W4A16_REDUCE_ATOMIC_F32", b.REDUCE_ATOMIC_F32),
                      ("W4A16_REDUCE_ATOMIC_PK_F16", b.REDUCE_ATOMIC_PK_F16), ("W4A16_REDUCE_WORKSPACE", b.REDUCE_WORKSPACE),
                      ("W4A16_REDUCE_ATOMIC_FIXED", b.REDUCE_ATOMIC_FIXED),
                      ("W4A16_REDUCE_ATOMIC_PK_F16_PHASE", b.REDUCE_ATOMIC_PK_F16_PHASE)):
        mt = re.search(rf"#define\s+{name}\s+\(?(-?\d+)\)?", HEADER)
        assert mt and int(mt.group(1)) == val, name
    for code in range(-8, 1):
        assert isinstance(b.strerror(code), str) and b.strerror(code)
    texts = [b.strerror(code) for code in range(-7, 1)]
    assert len(set(texts)) == len(texts) and b.strerror(-8) not in texts   # every code has a text of its own


@pytest.mark.parametrize("args,code", [
    ((16, 4096, 4096, 128, 4), b.OK),
    ((1, 1024, 1024, 128, 4), b.OK),
    ((8, 16384, 16384, 128, 32), b.OK),
    ((16, 4096, 4096, 128, 0), b.OK),            # 0 = let the library choose
    ((0, 4096, 4096, 128, 1), b.ERR_SHAPE),
    ((1, 4100, 4096, 128, 1), b.ERR_SHAPE),      # n % 8
    ((1, 4, 4096, 128, 1), b.ERR_SHAPE),
    ((1, 4096, 4100, 128, 1), b.ERR_SHAPE),      # k % group_size
    ((1, 4096, 4096, 100, 1), b.ERR_SHAPE),      # group_size % 8
    ((1, 4096, 64, 128, 1), b.ERR_SHAPE),        # k < group_size
    ((1, 4096, 4096, 128, -1), b.ERR_SPLIT),
    ((1, 4096, 4096, 128, 3), b.ERR_SPLIT),      # k % split_k
    ((1, 4096, 4096, 128, 64), b.ERR_SPLIT),     # (k / split_k) % group_size
    ((17, 4096, 4096, 128, 1), b.OK),            # rows beyond 16 run as further launches
    ((1, 4096, 4096, 96, 1), b.ERR_SHAPE),       # 4096 % 96
    ((1, 4096, 3840, 96, 1), b.ERR_UNSUPPORTED), # a legal GPTQ shape this build does not implement
])
def test_check(args, code):
    assert b.w4a16_check(*args) == code


def test_gemm_rejects_before_touching_hip():
    L = b.lib()
    p = ctypes.c_void_p(4096)       # never dereferenced: every call below fails validation first
    odd = ctypes.c_void_p(4100)
    assert L.w4a16_gemm(None, p, p, p, p, 1, 1024, 1024, 128, 4, None) == b.ERR_NULL
    assert L.w4a16_gemm(p, p, p, p, None, 1, 1024, 1024, 128, 4, None) == b.ERR_NULL
    assert L.w4a16_gemm(p, p, p, p, p, 1, 1020, 1024, 128, 4, None) == b.ERR_SHAPE
    assert L.w4a16_gemm(p, p, p, p, p, 1, 1024, 1024, 128, 3, None) == b.ERR_SPLIT
    assert L.w4a16_gemm(p, p, p, p, p, 32, 1024, 1024, 100, 4, None) == b.ERR_SHAPE
    assert L.w4a16_gemm(p, odd, p, p, p, 1, 1024, 1024, 128, 4, None) == b.ERR_UNSUPPORTED
    assert L.w4a16_gemm_dp(p, p, p, None, p, 1, 1024, 1024, 128, None) == b.ERR_NULL
    assert L.w4a16_gemm_dp(p, p, p, p, p, 1, 1024, 1000, 128, None) == b.ERR_SHAPE
    assert L.w4a16_gemm_ex(p, p, p, p, p, 1, 1024, 1024, 128, 4, 48, 0, 0, None) == b.ERR_UNSUPPORTED   # tile_cols
    assert L.w4a16_gemm_ex(p, p, p, p, p, 1, 1024, 1024, 128, 4, 64, 3, 0, None) == b.ERR_UNSUPPORTED   # waves
    assert L.w4a16_gemm_ex(p, p, p, p, p, 1, 1024, 1024, 128, 4, 64, 2, 9, None) == b.ERR_UNSUPPORTED   # reduce
    assert L.w4a16_gemm_streamk(p, None, p, p, p, 1, 1024, 1024, 128, 0, None) == b.ERR_NULL
    assert L.w4a16_gemm_streamk(p, p, p, p, p, 1, 1024, 1000, 128, 0, None) == b.ERR_SHAPE
    assert L.w4a16_gemm_streamk(p, p, p, p, p, 1, 1024, 1024, 64, 0, None) == b.ERR_UNSUPPORTED   # group_size
    assert L.w4a16_gemm_streamk(p, p, p, p, p, 1, 1024, 1024, 128, -2, None) == b.ERR_UNSUPPORTED  # workgroups
    assert L.w4a16_gemm_streamk_bits(5, p, p, p, p, p, 1, 1024, 1024, 128, 0, None) == b.ERR_UNSUPPORTED   # width
    assert L.w4a16_gemm_streamk_bits(3, p, p, p, p, p, 1, 1040, 1024, 128, 0, None) == b.ERR_SHAPE         # n % 32
    assert L.w4a16_gemm_streamk_bits(2, p, None, p, p, p, 1, 1024, 1024, 128, 0, None) == b.ERR_NULL
    assert L.w8a16_gemm(p, p, None, p, p, 1, 1024, 1024, 128, 4, None) == b.ERR_NULL
    assert L.w8a16_gemm(p, p, p, p, p, 1, 1020, 1024, 128, 4, None) == b.ERR_SHAPE
    assert L.w8a16_gemm(p, p, p, p, p, 1, 1024, 1024, 128, 3, None) == b.ERR_SPLIT
    assert L.w8a16_gemm_dp(p, p, p, p, odd, 1, 1024, 1024, 128, None) == b.ERR_UNSUPPORTED
    assert L.w2a16_gemm(p, p, p, p, p, 1, 1032, 1024, 128, 4, None) == b.ERR_SHAPE     # n % 16
    assert L.w2a16_gemm_dp(None, p, p, p, p, 1, 1024, 1024, 128, None) == b.ERR_NULL
    assert L.w3a16_gemm(p, p, p, p, p, 1, 1040, 1024, 128, 4, None) == b.ERR_SHAPE     # n % 32
    assert L.w3a16_gemm(p, p, p, p, p, 1, 1024, 1024, 128, 3, None) == b.ERR_SPLIT
    assert L.w3a16_gemm(p, p, p, None, p, 1, 1024, 1024, 128, 4, None) == b.ERR_NULL
    assert L.w3a16_gemm_dp(p, p, odd, p, p, 1, 1024, 1024, 128, None) == b.ERR_UNSUPPORTED
    q = ctypes.c_void_p(8192)
    assert L.w4a16_actorder_prepare(p, p, q, p, None, 1024, 1024, 128, None) == b.ERR_NULL
    assert L.w4a16_actorder_prepare(p, p, q, p, p, 1020, 1024, 128, None) == b.ERR_SHAPE
    assert L.w4a16_actorder_prepare(p, p, p, p, p, 1024, 1024, 128, None) == b.ERR_UNSUPPORTED   # in place
    assert L.w4a16_gemm_actorder(p, p, p, p, p, None, p, 1, 1024, 1024, 128, 0, None) == b.ERR_NULL
    assert L.w4a16_gemm_actorder(p, p, p, p, p, q, p, 1, 1024, 1024, 128, 3, None) == b.ERR_SPLIT
    assert L.w4a16_gemm_actorder(p, p, p, p, p, p, p, 1, 1024, 1024, 128, 0, None) == b.ERR_UNSUPPORTED  # A_work is A
    assert L.w4a16_read_probe(None, 4096, 0, None) == b.ERR_NULL
    assert L.w4a16_read_probe(p, 4100, 0, None) == b.ERR_SHAPE
    assert L.w4a16_read_probe(odd, 4096, 0, None) == b.ERR_SHAPE
    assert L.w4a16_read_probe(p, 4096, 10, None) == b.ERR_UNSUPPORTED
    assert L.w4a16_unpack(None, p, p, p, 1024, 1024, 128, None) == b.ERR_NULL
    assert L.w4a16_unpack(p, p, p, p, 1020, 1024, 128, None) == b.ERR_SHAPE
    assert L.w4a16_dequant(p, p, p, None, 1024, 1024, 128, None) == b.ERR_NULL
    # the entry point that allocates nothing: its own limits on top of w4a16_gemm's checks
    assert L.w4a16_gemm_static(None, p, p, p, p, 1, 1024, 1024, 128, 4, None) == b.ERR_NULL
    assert L.w4a16_gemm_static(p, p, p, p, p, 1, 1020, 1024, 128, 4, None) == b.ERR_SHAPE
    assert L.w4a16_gemm_static(p, p, p, p, p, 1, 1024, 1024, 128, 3, None) == b.ERR_SPLIT
    assert L.w4a16_gemm_static(p, p, p, p, p, 17, 1024, 1024, 128, 4, None) == b.ERR_LIMIT    # m > 16
    assert L.w4a16_gemm_static(p, p, p, p, p, 16, 16392, 1024, 128, 4, None) == b.ERR_LIMIT   # n > 16384
    assert L.w4a16_gemm_static(p, p, p, p, p, 17, 1020, 1024, 128, 4, None) == b.ERR_SHAPE    # a bad shape stays one
    assert L.w4a16_set_phase_spin_limit(-1) == b.ERR_UNSUPPORTED
    assert L.w4a16_set_phase_spin_limit(0) == b.OK


def test_reported_plans_can_be_passed_back():
    """Whatever launch w4a16_plan reports for a shape is accepted, unchanged, when it is given
    explicitly (a data-parallel shaped launch names a reduction it does not use)."""
    import numpy as np
    rng = np.random.default_rng(0)
    for _ in range(1500):
        m = int(rng.integers(1, 17))
        n = int(rng.integers(1, 3600)) * 8
        k = int(rng.integers(1, 120)) * 128
        pl = b.w4a16_plan(m, n, k, 128)
        assert b.w4a16_plan(m, n, k, 128, **pl) == pl, (m, n, k, pl)


def test_workspace_size():
    """w4a16_workspace_bytes: 0 for a bad n_max, otherwise the documented layout (head, tickets,
    phase levels of split_k 2..64, fp32 sums and fixed-point words for sixteen rows)."""
    assert b.w4a16_workspace_bytes(0) == 0 and b.w4a16_workspace_bytes(4100) == 0
    assert b.w4a16_workspace_bytes(65544) == 0
    levels = sum(4096 * (1 + s) for s in range(2, 65))
    for n in (8, 4096, 16384, 65536):
        words = 64 + n // 16 + levels
        words = (words + 63) // 64 * 64
        words += 16 * n + 32 * n
        assert b.w4a16_workspace_bytes(n) == 4 * words, n
    assert b.w4a16_workspace_bytes(16384) < 40 << 20


def test_plan_is_consistent():
    for m in (1, 16):
        for nk in (1024, 4096, 8192, 16384):
            for dp in (False, True):
                pl = b.w4a16_plan(m, nk, nk, 128, dp=dp)
                groups = nk // 128
                assert groups % pl["split_k"] == 0
                assert pl["tile_cols"] in (16, 32, 64, 128, 256) and 1 <= pl["waves"] <= 16
                # k parts of a workgroup: all its waves, or (256-column tiles) sets of four
                kparts = pl["waves"] // 4 if pl["tile_cols"] == 256 else pl["waves"]
                assert (groups // pl["split_k"]) % kparts == 0
                if pl["tile_cols"] == 256:
                    assert not dp and nk >= 8192
                if dp:
                    assert pl["split_k"] == 1
    # a requested split is kept
    assert b.w4a16_plan(16, 4096, 4096, 128, split_k=8)["split_k"] == 8
    with pytest.raises(b.W4A16Error):
        b.w4a16_plan(16, 4096, 4096, 128, split_k=8, waves=8)   # 4 groups per workgroup cannot feed 8 waves


def test_uneven_k_shares_host_rules():
    """w4a16_gemm keeps Algorithm 1's equal shares for a requested split_k; the library's own
    plan and the _ex entry point deal whole compute groups, counts differing by at most one."""
    L = b.lib()
    p = ctypes.c_void_p(4096)
    assert b.w4a16_check(1, 1024, 1408, 128, 0) == b.OK                                     # 11 groups, library's choice
    assert b.w4a16_check(1, 1024, 1408, 128, 2) == b.ERR_SPLIT
    assert L.w4a16_gemm(p, p, p, p, p, 1, 1024, 1408, 128, 2, None) == b.ERR_SPLIT          # 11 groups cannot be halved
    assert L.w4a16_gemm_ex(p, p, p, p, p, 1, 1024, 1408, 128, 16, 64, 1, 0, None) == b.ERR_SPLIT   # 16 slices, 11 groups
    assert L.w4a16_gemm_ex(p, p, p, p, p, 1, 1024, 1408, 128, 4, 64, 4, 0, None) == b.ERR_UNSUPPORTED  # 16 parts
    assert L.w4a16_gemm_ex(p, p, p, p, p, 16, 1024, 1408, 128, 2, 256, 8, 0, None) == b.ERR_SPLIT  # 8-wave streaming needs equal parts
    # llama-style projections, k = 11008 and 13824 included: the plan always has work for every part
    for m in (1, 16):
        for (n, k) in ((4096, 11008), (11008, 4096), (12288, 4096), (13824, 5120), (5120, 13824), (28672, 8192),
                       (8192, 28672), (22016, 4096), (10240, 8192)):
            for dp in (False, True):
                pl = b.w4a16_plan(m, n, k, 128, dp=dp)
                kparts = pl["waves"] // 4 if pl["tile_cols"] == 256 else pl["waves"]
                assert 1 <= pl["split_k"] * kparts <= k // 128
                tiles = -(-n // pl["tile_cols"])
                assert tiles * pl["split_k"] >= 160, (m, n, k, dp, pl)


def test_plan_invariants_over_a_grid_of_shapes():
    """Whatever the library picks must be a launch the kernels accept: enough compute groups for
    every k part, the exact-fit condition of the two-strip launch, equal parts for eight-wave
    streaming workgroups, a reduction flavour that takes the split, and a split small enough
    for the accuracy of the packed-fp16 adds."""
    ns = (8, 72, 1024, 2304, 4096, 4360, 5120, 6144, 9216, 11008, 12288, 14336, 22016, 28672, 66048)
    ks = (128, 512, 1024, 1408, 2048, 4096, 5120, 7168, 8192, 11008, 13824, 28672)
    count = 0
    for g in (32, 64, 128, 256):
        for m in (1, 3, 4, 5, 8, 16, 17, 40, 64):
            for n in ns:
                for k in ks:
                    if k % g or n * k >= 1 << 31:
                        continue
                    for dp in (False, True):
                        pl = b.w4a16_plan(m, n, k, g, dp=dp)
                        S, tc, wv, red = pl["split_k"], pl["tile_cols"], pl["waves"], pl["reduce"]
                        cg = k // min(g, 128)
                        assert tc in (16, 32, 64, 128, 256) and 1 <= wv <= 16 and S >= 1, (m, n, k, g, dp, pl)
                        kparts = wv // 4 if tc == 256 else wv
                        assert S * kparts <= cg, (m, n, k, g, dp, pl)
                        if dp:
                            assert S == 1 and tc in (16, 32, 64)
                            continue
                        if tc == 128:
                            assert S * wv == cg and g >= 128 and 2 <= S <= 64 and n <= 65536 and m <= 16
                        if tc == 256:
                            assert g >= 128 and wv in (4, 8)
                            if wv == 8:
                                assert cg % (2 * S) == 0 and m <= 16
                        else:
                            assert m <= 16 or g < 128        # more rows go to the streaming kernel where it applies
                        if S > 1:
                            assert red in (1, 2, 3, 4, 5)
                            if red == 5:
                                assert S <= 64 and n <= 65536
                            if red == 4:
                                assert S <= 64
                            if red in (2, 5):
                                assert S <= 32, (m, n, k, g, pl)     # the library's own choice keeps the fp16 adds accurate
                        count += 1
    assert count > 3000


def test_algorithmic_bytes():
    """The library, the input module and the figures derived from the paper's profile agree."""
    for (m, nk, expect) in ((1, 1024, 548864), (1, 4096, 8732672), (16, 4096, 8978432), (1, 8192, 34897920),
                            (16, 8192, 35389440), (8, 16384, 139984896)):
        assert b.w4a16_algorithmic_bytes(m, nk, nk, 128) == expect
        assert inputs.algorithmic_bytes(m, nk, nk, 128) == expect
    # Paper, Nsight Compute table (m=16, n=k=4096): throughput x latency is the traffic the
    # profiler saw; the formula must land within 5 % of it for both kernels.
    gold = dict(line.split() for line in (ROOT / "tests/golden/paper_nsight_m16_n4096_k4096.txt").read_text().splitlines()
                if line and not line.startswith("#"))
    ours = b.w4a16_algorithmic_bytes(int(gold["m"]), int(gold["n"]), int(gold["k"]), 128)
    for kind in ("splitk", "dp"):
        seen = float(gold[f"{kind}_throughput_GBps"]) * 1e9 * float(gold[f"{kind}_latency_us"]) * 1e-6
        assert abs(ours / seen - 1) < 0.06
    # and the paper's grid sizes: 4x more workgroups for SplitK at split_k = 4
    assert int(gold["splitk_grid"]) == 4 * int(gold["dp_grid"])


def test_plan_invariants_of_the_other_field_widths():
    """The same for the 8-, 3- and 2-bit entry points: 64-column tiles, two strips or the streaming
    kernel with one row tile, and launches the kernels accept."""
    ns = (32, 96, 1024, 2304, 4096, 5152, 6144, 9216, 11008, 14336, 22016, 28672)
    ks = (256, 1024, 1408, 2048, 4096, 5120, 7168, 8192, 11008, 13824, 28672)
    count = 0
    for bits in (8, 3, 2):
        for g in (32, 128, 256):
            for m in (1, 2, 4, 5, 9, 16, 40):
                for n in ns:
                    for k in ks:
                        if k % g or n * k * bits // 8 >= 1 << 31:
                            continue
                        for dp in (False, True):
                            pl = b.w4a16_plan_bits(bits, m, n, k, g, dp=dp)
                            S, tc, wv, red = pl["split_k"], pl["tile_cols"], pl["waves"], pl["reduce"]
                            cg = k // min(g, 128)
                            assert tc in (16, 32, 64, 128, 256) and 1 <= wv <= 8 and S >= 1, (bits, m, n, k, g, dp, pl)
                            kparts = wv // 4 if tc == 256 else wv
                            assert S * kparts <= cg, (bits, m, n, k, g, dp, pl)
                            if dp:
                                assert S == 1 and tc in (16, 32, 64) and wv <= 8
                                continue
                            if tc == 128:
                                assert S * wv == cg and g >= 128 and 4 <= S <= 16 and m >= 2
                            if tc == 256:
                                assert g >= 128 and wv in (4, 8) and (wv == 4 or cg % (2 * S) == 0)
                            if S > 1 and red in (2, 5):
                                assert S <= 32
                            count += 1
    assert count > 4000


def test_plan_of_the_other_field_widths():
    # two strips per wave where the 4-bit rule has them, by the number of weights
    for bits in (8, 3, 2):
        assert b.w4a16_plan_bits(bits, 16, 4096, 4096, 128) == dict(split_k=8, tile_cols=128, waves=4, reduce=5)
        assert b.w4a16_plan_bits(bits, 16, 8192, 8192, 128)["tile_cols"] == 256      # streaming kernel
        assert b.w4a16_plan_bits(bits, 1, 4096, 4096, 128)["tile_cols"] == 64        # one row: no two strips
        assert b.w4a16_plan_bits(bits, 16, 4096, 4096, 128, split_k=4)["tile_cols"] == 64   # a requested split
        assert b.w4a16_plan_bits(bits, 16, 4096, 4096, 128, dp=True)["split_k"] == 1
    assert b.w4a16_plan_bits(2, 16, 11008, 4096, 128)["tile_cols"] == 128
    assert b.w4a16_plan_bits(3, 16, 11008, 4096, 128)["tile_cols"] == 256
    assert b.w4a16_plan_bits(8, 16, 11008, 4096, 128)["tile_cols"] == 256
    for bits in (8, 3, 2):
        # the streaming kernel under the 4-bit rules at every width
        assert b.w4a16_plan_bits(bits, 8, 8192, 8192, 128) == b.w4a16_plan(8, 8192, 8192, 128)
        # few rows on a large matrix (3-bit fields: not where 256 tiles of 64 columns fill the machine once)
        assert b.w4a16_plan_bits(bits, 3, 16384, 16384, 128)["tile_cols"] == (64 if bits == 3 else 256)
        assert b.w4a16_plan_bits(bits, 16, 16384, 16384, 128)["tile_cols"] == 256
        assert b.w4a16_plan_bits(bits, 6, 28672, 4096, 128)["tile_cols"] == 256
        # short k: unsplit narrow tiles up to fifteen groups, a split from sixteen on
        assert b.w4a16_plan_bits(bits, 6, 8192, 1536, 128) == dict(split_k=1, tile_cols=32, waves=8, reduce=5)
        assert b.w4a16_plan_bits(bits, 16, 8192, 2048, 128)["split_k"] > 1
    assert b.w4a16_plan_bits(4, 16, 4096, 4096, 128) == b.w4a16_plan(16, 4096, 4096, 128)
    L = b.lib()
    assert L.w4a16_plan_bits(5, 16, 4096, 4096, 128, 0, None, None, None, None) == b.ERR_UNSUPPORTED
    assert L.w4a16_plan_bits(3, 16, 4104, 4096, 128, 0, None, None, None, None) == b.ERR_SHAPE


def test_8bit_algorithmic_bytes():
    for (m, n, k) in ((1, 1024, 1024), (16, 4096, 4096), (8, 4096, 11008)):
        expect = k * n + (k // 128) * n * 2 + (k // 128) * n + m * k * 2 + m * n * 2
        assert b.w8a16_algorithmic_bytes(m, n, k, 128) == expect
        assert inputs.algorithmic_bytes(m, n, k, 128, bits=8) == expect
    for (m, n, k) in ((1, 1024, 1024), (16, 4096, 4096)):
        expect = k * n // 4 + (k // 128) * n * 2 + (k // 128) * (n // 16) * 4 + m * k * 2 + m * n * 2
        assert b.w2a16_algorithmic_bytes(m, n, k, 128) == expect
        assert inputs.algorithmic_bytes(m, n, k, 128, bits=2) == expect
    for (m, n, k) in ((1, 1024, 1024), (16, 4096, 4096), (8, 4096, 11008)):
        expect = k * n * 3 // 8 + (k // 128) * n * 2 + (k // 128) * (n * 3 // 8) + m * k * 2 + m * n * 2
        assert b.w3a16_algorithmic_bytes(m, n, k, 128) == expect
        assert inputs.algorithmic_bytes(m, n, k, 128, bits=3) == expect
    x = inputs.make_inputs(2, 64, 256, 128, seed=5, bits=3)
    assert x.qweight.shape == (24, 64) and x.qzeros.shape == (2, 6) and x.scales.shape == (2, 64)
    x = inputs.make_inputs(2, 64, 256, 128, seed=5, bits=8)
    assert x.qweight.shape == (64, 64) and x.qzeros.shape == (2, 16) and x.scales.shape == (2, 64)


def test_input_generator_shapes_and_determinism():
    x = inputs.make_inputs(3, 64, 256, 128, seed=5)
    y = inputs.make_inputs(3, 64, 256, 128, seed=5)
    assert x.A.shape == (3, 256) and x.qweight.shape == (32, 64) and x.scales.shape == (2, 64) and x.qzeros.shape == (2, 8)
    for a, c in ((x.A, y.A), (x.qweight, y.qweight), (x.scales, y.scales), (x.qzeros, y.qzeros)):
        assert a.tobytes() == c.tobytes()
    assert (x.qweight < 0).any()
    assert 0.001 <= float(x.scales.min()) and float(x.scales.max()) <= 0.01
    z = inputs.make_inputs(3, 64, 256, 128, seed=6)
    assert z.qweight.tobytes() != x.qweight.tobytes()


def test_large_shape_parity_cases_cover_every_launch_kind():
    """The full-size parity cases (seeded random shapes plus the shapes that moved a plan rule)
    reach every kind of launch the plan can choose."""
    import numpy as np
    rng = np.random.Generator(np.random.Philox(77))
    shapes = []
    while len(shapes) < 20:
        n = int(rng.integers(128, 3600)) * 8
        k = int(rng.integers(8, 120)) * 128
        m = int(rng.choice([1, 2, 4, 6, 8, 12, 16]))
        if n * k <= (1 << 27):
            shapes.append((m, n, k))
    shapes += [(2, 25112, 4096), (8, 22232, 7808), (1, 2304, 3072), (6, 7216, 2304), (16, 8216, 1920),
               (4, 1864, 1408), (12, 4248, 2688), (1, 23064, 8192)]
    kinds = set()
    for (m, n, k) in shapes:
        pl = b.w4a16_plan(m, n, k, 128)
        kinds.add((pl["tile_cols"], pl["waves"], pl["split_k"] > 1, pl["reduce"] if pl["split_k"] > 1 else 0))
    assert {kd[0] for kd in kinds} >= {16, 32, 64, 128, 256}, kinds
    assert (256, 8, True, b.REDUCE_ATOMIC_PK_F16_PHASE) in kinds, kinds
    assert (64, 4, True, b.REDUCE_ATOMIC_FIXED) in kinds, kinds
    assert any(kd[0] == 64 and not kd[2] for kd in kinds), kinds


def test_plan_invariants_on_random_shapes():
    """Properties every launch the library chooses has, over 6000 random shapes and all field
    widths: the split fits k and the reduction's limits, two strips come with one group per wave,
    fixed-point adds only up to four rows, and the streaming kernel's workgroup count stays where
    the measurements put it (at most 256, or close to two per compute unit), never just above 256."""
    import numpy as np
    rng = np.random.default_rng(5)
    for _ in range(6000):
        bits = int(rng.choice([4, 4, 8, 3, 2]))
        m = int(rng.integers(1, 65))
        n = int(rng.integers(1, 3600)) * 32
        k = int(rng.integers(1, 120)) * 128
        pl = b.w4a16_plan(m, n, k, 128) if bits == 4 else b.w4a16_plan_bits(bits, m, n, k, 128)
        what = (bits, m, n, k, pl)
        groups = k // 128
        S, tc, w, r = pl["split_k"], pl["tile_cols"], pl["waves"], pl["reduce"]
        assert 1 <= S <= min(groups, 64) and tc in (16, 32, 64, 128, 256) and 1 <= w <= 16, what
        kparts = w // 4 if tc == 256 else w
        assert S * kparts <= groups, what
        workgroups = -(-n // tc) * S
        if tc == 256 and S > 1:
            assert workgroups <= 256 or 416 <= workgroups <= 512, what
        if tc == 128:
            assert w == 4 and S * 4 == groups, what
        if S > 1:
            assert r in (b.REDUCE_ATOMIC_PK_F16, b.REDUCE_ATOMIC_FIXED, b.REDUCE_ATOMIC_PK_F16_PHASE), what
            assert r != b.REDUCE_ATOMIC_FIXED or m <= 4, what

"""HIP path against the CPU oracle on a real MI355X, through the C ABI (binding = marshalling).

Tolerance (stated with the workload): relative Frobenius error <= 2e-3 and per-element
|err| <= 1e-2 * max|C_ref| against the oracle's fp64-accumulated result; unpacking and
single-term results bit-exact.
"""
import numpy as np
import pytest

from gpu_util import DeviceProblem, assert_parity, dev
from oracle_pins import (np_dense_weight, np_dense_weight_3bit, np_dense_weight_bits, random_act_order, random_case,
                         random_case_3bit, random_case_bits)
from paper_2402_00025_amd import binding as b
from paper_2402_00025_amd.inputs import make_inputs

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module", autouse=True)
def _gpu():
    import torch
    assert torch.cuda.is_available(), "these tests need the MI355X"
    b.lib()          # fail loudly if the HIP library is missing
    yield
    torch.cuda.synchronize()


# ------------------------------------------------------------------ probes: the plain read
@pytest.mark.parametrize("nbytes", [16, 4096 + 16, 8 << 20])
def test_read_probe_runs_every_launch_shape_and_writes_nothing(nbytes):
    """The measurement probe (ten launch shapes, five of them with the non-temporal hint) reads a
    buffer of any multiple of 16 bytes and leaves it and its surroundings as they were."""
    import torch

    guard = 256
    buf = torch.randint(0, 255, (nbytes + 2 * guard,), dtype=torch.uint8, device="cuda")
    before = buf.clone()
    view = buf[guard:guard + nbytes]
    for shape in range(10):
        b.w4a16_read_probe(view, nbytes, shape)
    torch.cuda.synchronize()
    assert torch.equal(buf, before)
    with pytest.raises(b.W4A16Error):
        b.w4a16_read_probe(view, nbytes, 10)


# ------------------------------------------------------------------ probes: bit-exact unpack
@pytest.mark.parametrize("n,k,g", [(1024, 1024, 128), (200, 384, 128), (8, 32, 32), (72, 512, 64)])
def test_unpack_bit_exact(oracle, n, k, g):
    import torch
    _, qw, _, qz = random_case(1, n, k, g, seed=21)
    q = torch.empty((k, n), dtype=torch.uint8, device="cuda")
    z = torch.empty((k // g, n), dtype=torch.uint8, device="cuda")
    b.w4a16_unpack(dev(qw), dev(qz), q, z, n, k, g)
    torch.cuda.synchronize()
    assert np.array_equal(q.cpu().numpy(), oracle.unpack_qweight(qw))
    assert np.array_equal(z.cpu().numpy(), oracle.unpack_qzeros(qz))


def test_unpack_known_words(oracle):
    import torch
    words = np.array([[0x76543210, 0x89ABCDEF - (1 << 32), 0, -1, 0x0F0F0F0F, -0x0F0F0F10, 0x12345678, -2]],
                     dtype=np.int64).astype(np.int32)
    zw = np.array([[0x76543210]], dtype=np.int32)
    q = torch.empty((8, 8), dtype=torch.uint8, device="cuda")
    z = torch.empty((1, 8), dtype=torch.uint8, device="cuda")
    b.w4a16_unpack(dev(words), dev(zw), q, z, 8, 8, 8)
    torch.cuda.synchronize()
    qh = q.cpu().numpy()
    assert qh[:, 0].tolist() == [0, 1, 2, 3, 4, 5, 6, 7]
    assert qh[:, 1].tolist() == [15, 14, 13, 12, 11, 10, 9, 8]
    assert np.array_equal(qh, oracle.unpack_qweight(words))
    assert z.cpu().numpy()[0].tolist() == [0, 1, 2, 3, 4, 5, 6, 7]


@pytest.mark.parametrize("n,k,g", [(256, 512, 128), (200, 384, 128), (64, 256, 32), (64, 512, 256)])
def test_dequant_bit_exact(oracle, n, k, g):
    """fp16((q - z) * s): one rounding of an exact product, so equal to the oracle's W rounded once."""
    import torch
    _, qw, s, qz = random_case(1, n, k, g, seed=22)
    W = torch.empty((k, n), dtype=torch.float16, device="cuda")
    b.w4a16_dequant(dev(qw), dev(s), dev(qz), W, n, k, g)
    torch.cuda.synchronize()
    ref = oracle.dequant(qw, s, qz, g).astype(np.float16)
    assert np.array_equal(W.cpu().numpy().view(np.uint16), ref.view(np.uint16))


# ------------------------------------------------------------------ configuration 1
def test_cfg1(oracle):
    x = make_inputs(1, 1024, 1024, 128, seed=0)
    Cref, _ = oracle.gemm(x.A, x.qweight, x.scales, x.qzeros, 128)
    p = DeviceProblem(x.A, x.qweight, x.scales, x.qzeros, 128)
    b.w4a16_gemm(*p.args(), 4)
    assert_parity(p.result(), Cref, "cfg1 splitk=4")
    p.C.fill_(float("nan"))
    b.w4a16_gemm_dp(*p.args())
    assert_parity(p.result(), Cref, "cfg1 dp")
    assert b.w4a16_phase_timeouts() == 0


# ------------------------------------------------------------------ small shapes: tiles, ragged tail, every knob
SMALL = [
    # m, n, k, g, split_k, tile_cols, waves, reduce
    (1, 200, 512, 128, 1, 64, 1, 0),
    (2, 200, 512, 128, 2, 64, 2, 1),
    (3, 200, 512, 128, 4, 64, 1, 1),
    (5, 200, 1024, 128, 2, 64, 4, 3),
    (16, 200, 1024, 128, 4, 64, 2, 2),
    (16, 328, 1024, 128, 8, 64, 1, 1),
    (7, 136, 512, 128, 2, 32, 2, 1),
    (16, 136, 512, 128, 1, 32, 4, 0),
    (4, 72, 512, 128, 4, 16, 1, 3),
    (16, 72, 1024, 128, 2, 16, 4, 2),
    (16, 264, 2048, 128, 1, 64, 16, 0),
    (9, 264, 2048, 128, 2, 64, 8, 1),
    (16, 192, 512, 32, 2, 64, 4, 1),
    (11, 192, 512, 64, 4, 64, 2, 3),
    (16, 192, 1024, 256, 2, 64, 2, 1),
    (13, 192, 1024, 256, 1, 32, 4, 0),
    (1, 8, 128, 128, 1, 16, 1, 0),
    (16, 8, 256, 128, 2, 64, 1, 1),
    (16, 200, 1024, 128, 4, 64, 2, 4),
    (3, 328, 1024, 128, 8, 64, 1, 4),
    (16, 136, 512, 128, 2, 32, 2, 4),
    (5, 72, 1024, 128, 2, 16, 4, 4),
    (16, 200, 1024, 128, 4, 64, 2, 5),
    (3, 328, 1024, 128, 8, 64, 1, 5),
    (16, 136, 512, 128, 2, 32, 2, 5),
    (5, 72, 1024, 128, 2, 16, 4, 5),
    (16, 264, 2048, 128, 2, 64, 8, 5),
    (9, 192, 512, 32, 16, 64, 1, 5),
]


@pytest.mark.parametrize("m,n,k,g,split_k,tile_cols,waves,reduce", SMALL)
def test_small_shapes(oracle, m, n, k, g, split_k, tile_cols, waves, reduce):
    A, qw, s, qz = random_case(m, n, k, g, seed=100 + m + n)
    Cref, _ = oracle.gemm(A, qw, s, qz, g)
    p = DeviceProblem(A, qw, s, qz, g)
    b.w4a16_gemm_ex(*p.args(), split_k, tile_cols, waves, reduce)
    assert_parity(p.result(), Cref, f"splitk m={m} n={n} k={k} S={split_k}")
    # second call into the same C: overwritten, not accumulated; scratch left clean by the first
    b.w4a16_gemm_ex(*p.args(), split_k, tile_cols, waves, reduce)
    assert_parity(p.result(), Cref, "second call")
    # data-parallel kernel on the same tile shape
    if (k // g) % waves == 0:
        p.C.fill_(float("nan"))
        b.w4a16_gemm_dp_ex(*p.args(), tile_cols, waves)
        assert_parity(p.result(), Cref, f"dp m={m} n={n} k={k}")


# ------------------------------------------------------------------ exact cases
@pytest.mark.parametrize("split_k,reduce", [(1, 0), (4, 1), (4, 2), (4, 3), (4, 4), (4, 5), (2, 5)])
def test_one_hot_rows_bit_exact(split_k, reduce):
    """A row equal to e_r selects row r of W: one non-zero term, every other partial sum is an
    exact zero, so every reduction flavour must return fp16(w[r, :]) exactly.  Sweeps all k."""
    m, n, k, g = 16, 200, 1024, 128
    _, qw, s, qz = random_case(m, n, k, g, seed=31)
    W = np_dense_weight(qw, s, qz, g)
    p = DeviceProblem(np.zeros((m, k), np.float16), qw, s, qz, g)
    import torch
    for base in range(0, k, m):
        rows = [(base + 7 * i) % k for i in range(m)]
        A = np.zeros((m, k), np.float16)
        for i, r in enumerate(rows):
            A[i, r] = 1.0
        p.A.copy_(torch.from_numpy(A))
        b.w4a16_gemm_ex(*p.args(), split_k, 64, 2, reduce)
        got = p.result()
        assert np.array_equal(got.view(np.uint16), W[rows, :].astype(np.float16).view(np.uint16)), base


@pytest.mark.parametrize("split_k", [1, 4])
def test_zero_cases_exact(split_k):
    m, n, k, g = 5, 200, 512, 128
    A, qw, s, qz = random_case(m, n, k, g, seed=33)
    p = DeviceProblem(np.zeros_like(A), qw, s, qz, g)
    b.w4a16_gemm(*p.args(), split_k)
    assert not p.result().view(np.uint16).any()            # A == 0 -> +0 everywhere
    # q == z everywhere
    zwords = np.random.Generator(np.random.Philox(2)).integers(0, 16, size=(k // g, n), dtype=np.uint8)
    zcol = zwords.astype(np.uint32)
    # a word whose eight fields all equal z[gi][j]: z * 0x11111111
    qw_eq = np.repeat((zcol * np.uint32(0x11111111)).astype(np.uint32), g // 8, axis=0).view(np.int32)
    qz_eq = np.zeros((k // g, n // 8), np.uint32)
    for i in range(8):
        qz_eq |= zcol[:, i::8] << np.uint32(4 * i)
    p2 = DeviceProblem(A, qw_eq, s, qz_eq.view(np.int32), g)
    b.w4a16_gemm(*p2.args(), split_k)
    assert not p2.result().astype(np.float32).any()


def test_constant_fields_closed_form():
    """q = q0, z = z0 everywhere: C[i, j] = (q0 - z0) * s_j * sum_k A[i, k]."""
    m, n, k, g = 4, 128, 1024, 128
    rng = np.random.Generator(np.random.Philox(35))
    A = rng.standard_normal((m, k), dtype=np.float32).astype(np.float16)
    s_col = rng.uniform(0.001, 0.01, size=n).astype(np.float16)
    scales = np.tile(s_col, (k // g, 1))
    q0, z0 = 13, 6
    qw = np.full((k // 8, n), q0 * 0x11111111, dtype=np.uint32).view(np.int32)
    qz = np.full((k // g, n // 8), z0 * 0x11111111, dtype=np.uint32).view(np.int32)
    expect = (q0 - z0) * s_col.astype(np.float64)[None, :] * A.astype(np.float64).sum(axis=1)[:, None]
    for split_k in (1, 2, 8):
        p = DeviceProblem(A, qw, scales, qz, g)
        b.w4a16_gemm(*p.args(), split_k)
        got = p.result().astype(np.float64)
        assert np.abs(got - expect).max() <= 2e-3 * np.abs(expect).max() + 1e-6


def test_deterministic_variants():
    """The data-parallel kernel, split_k = 1 and the workspace reduction give the same bits on
    every run; the atomic variants may differ in the last bits between runs."""
    m, n, k, g = 16, 256, 2048, 128
    A, qw, s, qz = random_case(m, n, k, g, seed=37)
    p = DeviceProblem(A, qw, s, qz, g)
    for call in (lambda: b.w4a16_gemm_dp(*p.args()),
                 lambda: b.w4a16_gemm(*p.args(), 1),
                 lambda: b.w4a16_gemm_ex(*p.args(), 4, 64, 2, b.REDUCE_WORKSPACE),
                 lambda: b.w4a16_gemm_ex(*p.args(), 8, 64, 2, b.REDUCE_ATOMIC_FIXED)):
        call()
        first = p.result().copy()
        for _ in range(3):
            p.C.fill_(float("nan"))
            call()
            assert np.array_equal(p.result().view(np.uint16), first.view(np.uint16))


def test_auto_split(oracle):
    A, qw, s, qz = random_case(8, 512, 2048, 128, seed=39)
    Cref, _ = oracle.gemm(A, qw, s, qz, 128)
    p = DeviceProblem(A, qw, s, qz, 128)
    b.w4a16_gemm(*p.args(), 0)
    assert_parity(p.result(), Cref, "auto split")


def test_on_side_stream(oracle):
    import torch
    A, qw, s, qz = random_case(4, 256, 1024, 128, seed=41)
    Cref, _ = oracle.gemm(A, qw, s, qz, 128)
    p = DeviceProblem(A, qw, s, qz, 128)
    st = torch.cuda.Stream()
    st.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(st):
        b.w4a16_gemm(*p.args(), 4, stream=st)
    st.synchronize()
    assert_parity(p.result(), Cref, "side stream")


def test_more_than_16_rows(oracle):
    """m = 40: three MFMA row tiles (16 + 16 + 8), SplitK and DP."""
    A, qw, s, qz = random_case(40, 264, 1024, 128, seed=43)
    Cref, _ = oracle.gemm(A, qw, s, qz, 128)
    p = DeviceProblem(A, qw, s, qz, 128)
    b.w4a16_gemm(*p.args(), 4)
    assert_parity(p.result(), Cref, "m=40 splitk")
    p.C.fill_(float("nan"))
    b.w4a16_gemm_dp(*p.args())
    assert_parity(p.result(), Cref, "m=40 dp")


ROW_TILES = [
    # m, n, k, g, split_k, tile_cols, waves, reduce: more than 16 rows are row tiles of one launch
    # of the streaming kernel (up to 64 rows), further rows further launches
    (17, 264, 1024, 128, 2, 0, 0, 0),      # two row tiles, the second with one row
    (32, 256, 1024, 128, 4, 256, 4, 5),    # two full tiles, phase protocol
    (33, 328, 1408, 128, 2, 256, 4, 2),    # three tiles, 6 and 5 groups per part, fill kernel
    (48, 200, 2048, 128, 1, 0, 0, 0),      # three tiles, direct store
    (50, 264, 1664, 128, 4, 0, 0, 0),      # four tiles, 4,3,3,3 groups
    (64, 512, 2048, 128, 8, 256, 4, 5),    # four full tiles, 2 groups per part
    (64, 136, 1024, 128, 8, 0, 0, 0),      # one group per part: ring depth 1
    (64, 264, 1280, 256, 2, 0, 0, 0),      # group_size 256
    (65, 264, 1024, 128, 2, 0, 0, 0),      # 64 rows in one launch, one more in a second
    (150, 200, 1024, 128, 0, 0, 0, 0),     # 64 + 64 + 22, the library's split
    (40, 264, 1024, 64, 2, 0, 0, 0),       # group_size 64: one launch per 16 rows
    (40, 264, 1024, 128, 2, 64, 2, 1),     # 64-column tiles asked for: one launch per 16 rows
]


@pytest.mark.parametrize("m,n,k,g,split_k,tile_cols,waves,reduce", ROW_TILES)
def test_row_tiles(oracle, m, n, k, g, split_k, tile_cols, waves, reduce):
    A, qw, s, qz = random_case(m, n, k, g, seed=700 + m + n)
    Cref, _ = oracle.gemm(A, qw, s, qz, g)
    p = DeviceProblem(A, qw, s, qz, g)
    for call in range(2):
        p.C.fill_(float("nan"))
        b.w4a16_gemm_ex(*p.args(), split_k, tile_cols, waves, reduce)
        assert_parity(p.result(), Cref, f"m={m} n={n} k={k} g={g} S={split_k} tile={tile_cols} call {call}")
    assert b.w4a16_phase_timeouts() == 0


@pytest.mark.parametrize("split_k", [1, 4])
def test_row_tiles_one_hot_bit_exact(split_k):
    """64 one-hot rows per call: every row tile must pick its own rows of A and write its own
    rows of C; swept over all k."""
    m, n, k, g = 64, 264, 1024, 128
    _, qw, s, qz = random_case(m, n, k, g, seed=49)
    W = np_dense_weight(qw, s, qz, g)
    p = DeviceProblem(np.zeros((m, k), np.float16), qw, s, qz, g)
    import torch
    for base in range(0, k, m):
        rows = [(base + 5 * i) % k for i in range(m)]
        A = np.zeros((m, k), np.float16)
        for i, r in enumerate(rows):
            A[i, r] = 1.0
        p.A.copy_(torch.from_numpy(A))
        b.w4a16_gemm_ex(*p.args(), split_k, 0, 0, 0)
        got = p.result()
        assert np.array_equal(got.view(np.uint16), W[rows, :].astype(np.float16).view(np.uint16)), base


def test_phase_mode_call_sequences(oracle):
    """The in-kernel zeroing protocol keeps per-tile state between calls: run calls of different
    shapes, split factors and tile widths back to back into NaN-filled outputs, twice each,
    and require parity every time and no wait that ran out."""
    cases = [(16, 328, 1024, 4, 64, 2), (5, 200, 2048, 8, 64, 2), (16, 328, 1024, 2, 32, 4),
             (1, 72, 1024, 8, 16, 1), (16, 328, 1024, 8, 64, 1), (16, 136, 1024, 2, 64, 4)]
    probs = []
    for (m, n, k, S, tc, wv) in cases:
        A, qw, s, qz = random_case(m, n, k, 128, seed=500 + m + n + S)
        Cref, _ = oracle.gemm(A, qw, s, qz, 128)
        probs.append((DeviceProblem(A, qw, s, qz, 128), Cref, S, tc, wv))
    for rnd in range(3):
        for (p, Cref, S, tc, wv) in probs:
            for _ in range(2):
                p.C.fill_(float("nan"))
                b.w4a16_gemm_ex(*p.args(), S, tc, wv, b.REDUCE_ATOMIC_PK_F16_PHASE)
                assert_parity(p.result(), Cref, f"phase S={S} tile={tc} waves={wv} round={rnd}")
    assert b.w4a16_phase_timeouts() == 0


def test_hip_graph_replays(oracle):
    """Calls captured in a HIP graph and replayed: the split-k state the library keeps between
    calls (per-tile flags and counts, fixed-point words, tickets) must come out right on every
    replay, also with eager calls of other shapes on the same tiles between the replays."""
    import torch
    cases = [
        # m, n, k, split_k, tile_cols, waves, reduce
        (16, 512, 1024, 8, 64, 1, b.REDUCE_ATOMIC_PK_F16_PHASE),   # one group per wave: service wavefront
        (16, 512, 2048, 4, 64, 2, b.REDUCE_ATOMIC_PK_F16_PHASE),   # in-wave protocol
        (9, 520, 2048, 4, 256, 4, b.REDUCE_ATOMIC_PK_F16_PHASE),   # streaming kernel
        (3, 512, 1024, 4, 64, 2, b.REDUCE_ATOMIC_FIXED),
        (16, 512, 1024, 4, 64, 2, b.REDUCE_ATOMIC_PK_F16),         # fill kernel + atomics
        (16, 512, 1024, 2, 64, 2, b.REDUCE_ATOMIC_F32),
        (16, 520, 1024, 2, 128, 4, b.REDUCE_ATOMIC_PK_F16_PHASE),  # two strips per wave
        (40, 520, 2048, 4, 256, 4, b.REDUCE_ATOMIC_PK_F16_PHASE),  # three row tiles, more than 64 KiB of LDS
        (16, 520, 1408, 4, 256, 4, b.REDUCE_ATOMIC_PK_F16_PHASE),  # uneven shares, phantom group
    ]
    probs = []
    for (m, n, k, S, tc, wv, red) in cases:
        A, qw, s, qz = random_case(m, n, k, 128, seed=700 + m + k + S)
        Cref, _ = oracle.gemm(A, qw, s, qz, 128)
        probs.append((DeviceProblem(A, qw, s, qz, 128), Cref, S, tc, wv, red))
    other = DeviceProblem(*random_case(16, 512, 2048, 128, seed=777), 128)
    for (p, _, S, tc, wv, red) in probs:   # eager warm-up: scratch allocation happens outside the capture
        b.w4a16_gemm_ex(*p.args(), S, tc, wv, red)
    torch.cuda.synchronize()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g, stream=side):
        for (p, _, S, tc, wv, red) in probs:
            b.w4a16_gemm_ex(*p.args(), S, tc, wv, red, stream=torch.cuda.current_stream())
    for rep in range(4):
        for (p, *_rest) in probs:
            p.C.fill_(float("nan"))
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        for (p, Cref, S, tc, wv, red) in probs:
            assert_parity(p.C.cpu().numpy(), Cref, f"replay {rep}: S={S} tile={tc} waves={wv} reduce={red}")
        # eager work between replays, on the same tiles with other split factors
        b.w4a16_gemm_ex(*other.args(), 8, 64, 2, b.REDUCE_ATOMIC_PK_F16_PHASE)
        b.w4a16_gemm_ex(*other.args(), 4, 256, 4, b.REDUCE_ATOMIC_PK_F16_PHASE)
        torch.cuda.synchronize()
    assert b.w4a16_phase_timeouts() == 0


# ------------------------------------------------------------------ streaming SplitK kernel (activations shared through LDS)
STREAM_SMALL = [
    # m, n, k, g, split_k, waves (4 per k part), reduce
    (16, 256, 512, 128, 1, 4, 0),      # four groups per wave, ring depth 4, direct store
    (16, 256, 512, 128, 4, 4, 0),      # one group per wave
    (16, 512, 1024, 128, 2, 8, 0),     # two k parts added in LDS, two groups per wave
    (1, 256, 1024, 128, 2, 4, 0),
    (3, 328, 1024, 128, 4, 4, 0),      # ragged: second tile has one live strip and an eighth
    (5, 200, 1024, 128, 2, 8, 2),      # fill kernel + atomics, overhanging strip
    (16, 72, 2048, 128, 2, 4, 0),      # eight groups per wave: steady loop
    (7, 136, 4096, 128, 2, 4, 5),      # 16 groups per wave: several steady iterations
    (16, 264, 1536, 128, 2, 4, 0),     # six groups per wave: ring depth 2
    (13, 264, 1536, 128, 4, 4, 0),     # three groups per wave: ring depth 1
    (9, 192, 1024, 256, 2, 8, 0),      # group_size 256
    (16, 192, 2048, 128, 1, 8, 0),     # direct store with k parts, dead strip
    (4, 512, 8192, 128, 1, 4, 0),      # 64 groups per wave
    (16, 512, 4096, 128, 8, 4, 5),
    (16, 1024, 2048, 128, 16, 4, 5),   # one group per wave, 16 slices
]


@pytest.mark.parametrize("m,n,k,g,split_k,waves,reduce", STREAM_SMALL)
def test_stream_kernel_small_shapes(oracle, m, n, k, g, split_k, waves, reduce):
    A, qw, s, qz = random_case(m, n, k, g, seed=300 + m + n)
    Cref, _ = oracle.gemm(A, qw, s, qz, g)
    p = DeviceProblem(A, qw, s, qz, g)
    b.w4a16_gemm_ex(*p.args(), split_k, 256, waves, reduce)
    assert_parity(p.result(), Cref, f"stream m={m} n={n} k={k} S={split_k} waves={waves} reduce={reduce}")
    p.C.fill_(float("nan"))
    b.w4a16_gemm_ex(*p.args(), split_k, 256, waves, reduce)
    assert_parity(p.result(), Cref, "second call")
    assert b.w4a16_phase_timeouts() == 0


@pytest.mark.parametrize("split_k,waves", [(1, 4), (4, 4), (2, 8), (8, 4)])
def test_stream_kernel_one_hot_rows_bit_exact(split_k, waves):
    """Same single-term argument as test_one_hot_rows_bit_exact, through the LDS-staged
    activation operand: pins its slot order, the chunk ring, the k parts and the slice boundaries."""
    m, n, k, g = 16, 328, 1024, 128
    _, qw, s, qz = random_case(m, n, k, g, seed=45)
    W = np_dense_weight(qw, s, qz, g)
    p = DeviceProblem(np.zeros((m, k), np.float16), qw, s, qz, g)
    import torch
    for base in range(0, k, m):
        rows = [(base + 7 * i) % k for i in range(m)]
        A = np.zeros((m, k), np.float16)
        for i, r in enumerate(rows):
            A[i, r] = 1.0
        p.A.copy_(torch.from_numpy(A))
        b.w4a16_gemm_ex(*p.args(), split_k, 256, waves, 0)
        got = p.result()
        assert np.array_equal(got.view(np.uint16), W[rows, :].astype(np.float16).view(np.uint16)), base


# ------------------------------------------------------------------ k that does not divide evenly
# The compute groups are dealt to the split_k * (k parts per workgroup) parts in order, the
# first (groups % parts) parts getting one more: shapes whose group count has few factors
# (llama's k = 11008 has 86 groups of 128) still get a balanced launch.
UNEVEN = [
    # m, n, k, g, split_k, tile_cols, waves, reduce
    (16, 200, 1408, 128, 2, 64, 4, 1),     # 11 groups over 8 parts: 2,2,2,1,1,1,1,1
    (16, 200, 1408, 128, 1, 64, 4, 0),     # 3,3,3,2: direct store
    (5, 328, 1408, 128, 4, 64, 2, 5),      # phase protocol, parts of one and two groups
    (16, 264, 1664, 128, 2, 64, 4, 4),     # 13 groups over 8 parts, fixed-point adds
    (7, 136, 1408, 128, 3, 32, 1, 3),      # split_k = 3: 4,4,3, workspace
    (16, 192, 2752, 32, 4, 64, 4, 2),      # 86 compute groups of 32 over 16 parts: 6 x 6, 10 x 5
    (9, 192, 1408, 64, 3, 64, 2, 2),       # 22 compute groups over 6 parts
    (16, 192, 1280, 256, 4, 64, 1, 1),     # 10 compute groups of 128 over 4: a part boundary inside a quantisation group
    (3, 72, 2432, 128, 1, 16, 16, 0),      # 19 groups over 16 waves
    (16, 200, 1408, 128, 8, 64, 1, 5),     # 8 slices of one or two groups
    (16, 256, 1408, 128, 2, 256, 4, 0),    # streaming kernel: 6 and 5 groups (odd tail of the ring)
    (16, 328, 1408, 128, 4, 256, 4, 0),    # 3,3,3,2
    (11, 328, 1408, 128, 8, 256, 4, 5),    # 2,2,2,1,...: ring depth 1
    (16, 264, 1408, 128, 3, 256, 4, 2),    # split_k = 3: 4,4,3, fill kernel
    (16, 512, 1408, 128, 1, 256, 4, 0),    # 11 groups in one part
    (8, 264, 1280, 256, 4, 256, 4, 0),     # group_size 256, 3,3,2,2
    (16, 264, 1664, 128, 4, 256, 4, 5),    # 4,3,3,3
]


@pytest.mark.parametrize("m,n,k,g,split_k,tile_cols,waves,reduce", UNEVEN)
def test_uneven_k_shares(oracle, m, n, k, g, split_k, tile_cols, waves, reduce):
    A, qw, s, qz = random_case(m, n, k, g, seed=500 + m + n)
    Cref, _ = oracle.gemm(A, qw, s, qz, g)
    p = DeviceProblem(A, qw, s, qz, g)
    for call in range(2):
        p.C.fill_(float("nan"))
        b.w4a16_gemm_ex(*p.args(), split_k, tile_cols, waves, reduce)
        assert_parity(p.result(), Cref, f"m={m} n={n} k={k} g={g} S={split_k} tile={tile_cols} waves={waves} call {call}")
    assert b.w4a16_phase_timeouts() == 0
    if tile_cols != 256:
        p.C.fill_(float("nan"))
        b.w4a16_gemm_dp_ex(*p.args(), tile_cols, waves)
        assert_parity(p.result(), Cref, f"dp m={m} n={n} k={k} waves={waves}")


@pytest.mark.parametrize("split_k,tile_cols,waves", [(2, 64, 4), (3, 64, 2), (1, 32, 8), (2, 256, 4), (4, 256, 4),
                                                     (8, 256, 4), (3, 256, 4)])
def test_uneven_k_shares_one_hot_bit_exact(split_k, tile_cols, waves):
    """One non-zero term per output row, swept over every k: a group that two parts both take,
    or that none takes, changes a result that must be fp16(w[r, :]) exactly."""
    m, n, k, g = 16, 264, 1408, 128
    _, qw, s, qz = random_case(m, n, k, g, seed=47)
    W = np_dense_weight(qw, s, qz, g)
    p = DeviceProblem(np.zeros((m, k), np.float16), qw, s, qz, g)
    import torch
    for base in range(0, k, m):
        rows = [(base + 7 * i) % k for i in range(m)]
        A = np.zeros((m, k), np.float16)
        for i, r in enumerate(rows):
            A[i, r] = 1.0
        p.A.copy_(torch.from_numpy(A))
        b.w4a16_gemm_ex(*p.args(), split_k, tile_cols, waves, 0)
        got = p.result()
        assert np.array_equal(got.view(np.uint16), W[rows, :].astype(np.float16).view(np.uint16)), base


def test_auto_plan_awkward_k(oracle):
    """k = 86 groups (the shape of llama's 11008) with the library's own launch, both kernels."""
    for m, n in ((16, 512), (1, 264)):
        A, qw, s, qz = random_case(m, n, 11008, 128, seed=61 + m)
        Cref, _ = oracle.gemm(A, qw, s, qz, 128)
        p = DeviceProblem(A, qw, s, qz, 128)
        b.w4a16_gemm(*p.args(), 0)
        assert_parity(p.result(), Cref, f"auto m={m} n={n}")
        p.C.fill_(float("nan"))
        b.w4a16_gemm_dp(*p.args())
        assert_parity(p.result(), Cref, f"dp m={m} n={n}")


# ------------------------------------------------------------------ two strips per wave
TWO_STRIPS = [
    # m, n, k, g, split_k, waves: 128-column tiles, one compute group per wave (split_k * waves = k / 128)
    (16, 256, 1024, 128, 2, 4),
    (16, 200, 1024, 128, 2, 4),     # second tile: one full strip and 8 columns of the other
    (7, 264, 512, 128, 4, 1),       # third tile has only its first 8 columns
    (16, 136, 2048, 256, 4, 4),     # group_size 256
    (3, 72, 1024, 128, 8, 1),       # first strip 64 columns, second 8
    (16, 1024, 4096, 128, 8, 4),
]


@pytest.mark.parametrize("m,n,k,g,split_k,waves", TWO_STRIPS)
def test_two_strips_per_wave(oracle, m, n, k, g, split_k, waves):
    A, qw, s, qz = random_case(m, n, k, g, seed=600 + m + n)
    Cref, _ = oracle.gemm(A, qw, s, qz, g)
    p = DeviceProblem(A, qw, s, qz, g)
    for call in range(3):
        p.C.fill_(float("nan"))
        b.w4a16_gemm_ex(*p.args(), split_k, 128, waves, 0)
        assert_parity(p.result(), Cref, f"two strips m={m} n={n} k={k} S={split_k} call {call}")
    assert b.w4a16_phase_timeouts() == 0


def test_two_strips_one_hot_bit_exact():
    m, n, k, g = 16, 200, 1024, 128
    _, qw, s, qz = random_case(m, n, k, g, seed=57)
    W = np_dense_weight(qw, s, qz, g)
    p = DeviceProblem(np.zeros((m, k), np.float16), qw, s, qz, g)
    import torch
    for base in range(0, k, m):
        rows = [(base + 7 * i) % k for i in range(m)]
        A = np.zeros((m, k), np.float16)
        for i, r in enumerate(rows):
            A[i, r] = 1.0
        p.A.copy_(torch.from_numpy(A))
        b.w4a16_gemm_ex(*p.args(), 2, 128, 4, 0)
        got = p.result()
        assert np.array_equal(got.view(np.uint16), W[rows, :].astype(np.float16).view(np.uint16)), base


# ------------------------------------------------------------------ StreamK variant
STREAMK = [
    # m, n, k, g, workgroups
    (16, 512, 1024, 128, 1),      # one workgroup walks both tiles: whole tiles, stored
    (16, 512, 1024, 128, 2),      # one tile each: no fill kernel
    (16, 512, 1024, 128, 3),      # 16 iterations over 3: segments of 5, 3 + 2, 6
    (16, 512, 1024, 128, 16),     # one group per workgroup
    (16, 512, 1024, 128, 5),      # 3, 3, 2 + 1, 3, 4
    (7, 328, 1408, 128, 4),       # 22 iterations, ragged second tile
    (1, 264, 2048, 128, 7),
    (16, 1032, 1536, 128, 13),    # 5 tiles x 12 groups over 13
    (9, 520, 1280, 256, 6),       # group_size 256
    (16, 256, 4096, 128, 0),      # library default: more workgroups than iterations
    (16, 2048, 2048, 128, 0),
    (40, 520, 1024, 128, 5),      # three launches of 16, 16, 8 rows
]


@pytest.mark.parametrize("m,n,k,g,workgroups", STREAMK)
def test_streamk(oracle, m, n, k, g, workgroups):
    A, qw, s, qz = random_case(m, n, k, g, seed=800 + m + n)
    Cref, _ = oracle.gemm(A, qw, s, qz, g)
    p = DeviceProblem(A, qw, s, qz, g)
    for call in range(2):
        p.C.fill_(float("nan"))
        b.w4a16_gemm_streamk(*p.args(), workgroups)
        assert_parity(p.result(), Cref, f"streamk m={m} n={n} k={k} g={g} W={workgroups} call {call}")


@pytest.mark.parametrize("workgroups", [1, 3, 5, 7, 16, 24])
def test_streamk_one_hot_bit_exact(workgroups):
    """One non-zero term per row, swept over all k: every iteration belongs to exactly one
    segment of exactly one workgroup."""
    m, n, k, g = 16, 520, 1024, 128
    _, qw, s, qz = random_case(m, n, k, g, seed=51)
    W = np_dense_weight(qw, s, qz, g)
    p = DeviceProblem(np.zeros((m, k), np.float16), qw, s, qz, g)
    import torch
    for base in range(0, k, m):
        rows = [(base + 7 * i) % k for i in range(m)]
        A = np.zeros((m, k), np.float16)
        for i, r in enumerate(rows):
            A[i, r] = 1.0
        p.A.copy_(torch.from_numpy(A))
        b.w4a16_gemm_streamk(*p.args(), workgroups)
        got = p.result()
        assert np.array_equal(got.view(np.uint16), W[rows, :].astype(np.float16).view(np.uint16)), base


def test_streamk_full_size(oracle):
    """The headline shape and a non-square one at full size, library default."""
    for (m, n, k) in ((16, 4096, 4096), (16, 5120, 13824)):
        x = make_inputs(m, n, k, 128, seed=3)
        Cref, _ = oracle.gemm(x.A, x.qweight, x.scales, x.qzeros, 128)
        p = DeviceProblem(x.A, x.qweight, x.scales, x.qzeros, 128)
        b.w4a16_gemm_streamk(*p.args(), 0)
        assert_parity(p.result(), Cref, f"streamk m={m} n={n} k={k}")


# ------------------------------------------------------------------ 8-bit fields
EIGHT_BIT = [
    # m, n, k, g, split_k
    (1, 200, 512, 128, 1),
    (16, 200, 1024, 128, 4),      # two groups per part
    (16, 328, 1024, 128, 8),      # one group per part, ragged last tile
    (5, 72, 1408, 128, 0),        # 11 groups, the library's split
    (16, 264, 2048, 128, 2),      # eight groups per workgroup: steady loop
    (3, 136, 1024, 256, 2),       # group_size 256
    (16, 192, 512, 64, 2),        # group_size 64
    (9, 192, 256, 32, 4),         # group_size 32
    (4, 64, 4096, 128, 0),        # few rows: fixed-point reduction
    (40, 264, 1024, 128, 4),      # three launches of 16, 16, 8 rows
    (16, 8, 256, 128, 2),         # a single 8-column strip
]


@pytest.mark.parametrize("m,n,k,g,split_k", EIGHT_BIT)
def test_8bit_fields(oracle, m, n, k, g, split_k):
    A, qw, s, qz = random_case_bits(m, n, k, g, 8, seed=900 + m + n)
    Cref, _ = oracle.gemm_bits(A, qw, s, qz, g, 8)
    p = DeviceProblem(A, qw, s, qz, g)
    for call in range(2):
        p.C.fill_(float("nan"))
        b.w8a16_gemm(*p.args(), split_k)
        assert_parity(p.result(), Cref, f"8-bit splitk m={m} n={n} k={k} g={g} S={split_k} call {call}")
    p.C.fill_(float("nan"))
    b.w8a16_gemm_dp(*p.args())
    assert_parity(p.result(), Cref, f"8-bit dp m={m} n={n} k={k} g={g}")
    assert b.w4a16_phase_timeouts() == 0


@pytest.mark.parametrize("split_k", [1, 4])
def test_8bit_one_hot_rows_bit_exact(split_k):
    """One non-zero term per row, swept over all k: pins the byte order inside a word, the two
    word rows of a lane, the zero-point bytes and the scale columns."""
    m, n, k, g = 16, 200, 1024, 128
    _, qw, s, qz = random_case_bits(m, n, k, g, 8, seed=53)
    W = np_dense_weight_bits(qw, s, qz, g, 8)
    p = DeviceProblem(np.zeros((m, k), np.float16), qw, s, qz, g)
    import torch
    for base in range(0, k, m):
        rows = [(base + 7 * i) % k for i in range(m)]
        A = np.zeros((m, k), np.float16)
        for i, r in enumerate(rows):
            A[i, r] = 1.0
        p.A.copy_(torch.from_numpy(A))
        b.w8a16_gemm(*p.args(), split_k)
        got = p.result()
        assert np.array_equal(got.view(np.uint16), W[rows, :].astype(np.float16).view(np.uint16)), base


def test_8bit_full_size(oracle):
    """The headline shape with 8-bit fields, SplitK (library's split) and data-parallel."""
    x = make_inputs(16, 4096, 4096, 128, seed=0, bits=8)
    Cref, _ = oracle.gemm_bits(x.A, x.qweight, x.scales, x.qzeros, 128, 8)
    p = DeviceProblem(x.A, x.qweight, x.scales, x.qzeros, 128)
    b.w8a16_gemm(*p.args(), 0)
    assert_parity(p.result(), Cref, "8-bit splitk 4096^2")
    p.C.fill_(float("nan"))
    b.w8a16_gemm_dp(*p.args())
    assert_parity(p.result(), Cref, "8-bit dp 4096^2")


# ------------------------------------------------------------------ more than 16 rows at the other field widths
def _case_and_ref(oracle, bits, m, n, k, g, seed):
    if bits == 3:
        A, qw, s, qz = random_case_3bit(m, n, k, g, seed=seed)
        return A, qw, s, qz, oracle.gemm_3bit(A, qw, s, qz, g)[0]
    A, qw, s, qz = random_case_bits(m, n, k, g, bits, seed=seed)
    return A, qw, s, qz, oracle.gemm_bits(A, qw, s, qz, g, bits)[0]


@pytest.mark.parametrize("bits", [8, 3, 2])
@pytest.mark.parametrize("m,n,k,g,split_k", [
    (17, 288, 1024, 128, 0),      # two row tiles, the second with one row; ragged last column tile
    (40, 544, 2048, 128, 4),      # three row tiles
    (64, 288, 1408, 128, 0),      # four row tiles, 11 groups (uneven shares)
    (33, 320, 1024, 256, 2),      # group_size 256
    (150, 288, 1024, 128, 2),     # three launches of 64, 64 and 22 rows
    (48, 288, 512, 64, 2),        # group_size 64: one launch per 16 rows
])
def test_row_tiles_other_field_widths(oracle, bits, m, n, k, g, split_k):
    """Up to 64 rows share one pass over the weights (row tiles of the streaming kernel) at 8-, 3-
    and 2-bit fields as well; each width against its own oracle function."""
    A, qw, s, qz, Cref = _case_and_ref(oracle, bits, m, n, k, g, seed=1300 + bits + m)
    p = DeviceProblem(A, qw, s, qz, g)
    gemm = {8: b.w8a16_gemm, 3: b.w3a16_gemm, 2: b.w2a16_gemm}[bits]
    for call in range(2):
        p.C.fill_(float("nan"))
        gemm(*p.args(), split_k)
        assert_parity(p.result(), Cref, f"{bits}-bit m={m} n={n} k={k} g={g} S={split_k} call {call}")
    pl = b.w4a16_plan_bits(bits, m, n, k, g, split_k=split_k)
    assert pl["tile_cols"] == (256 if g >= 128 else 64)     # the plan of one launch: row tiles where the streaming kernel takes them
    assert b.w4a16_phase_timeouts() == 0


@pytest.mark.parametrize("bits", [8, 3, 2])
def test_row_tiles_other_field_widths_one_hot_bit_exact(bits):
    """One non-zero term per row, 64 rows at a time, swept over all k: the row tiles' operands, the
    field order and the parameters of every width, bit for bit."""
    import torch
    m, n, k, g = 64, 288, 1024, 128
    if bits == 3:
        _, qw, s, qz = random_case_3bit(m, n, k, g, seed=77)
        W = np_dense_weight_3bit(qw, s, qz, g)
    else:
        _, qw, s, qz = random_case_bits(m, n, k, g, bits, seed=77)
        W = np_dense_weight_bits(qw, s, qz, g, bits)
    p = DeviceProblem(np.zeros((m, k), np.float16), qw, s, qz, g)
    gemm = {8: b.w8a16_gemm, 3: b.w3a16_gemm, 2: b.w2a16_gemm}[bits]
    for base in range(0, k, m):
        rows = [(base + 5 * i) % k for i in range(m)]
        A = np.zeros((m, k), np.float16)
        for i, r in enumerate(rows):
            A[i, r] = 1.0
        p.A.copy_(torch.from_numpy(A))
        gemm(*p.args(), 4)
        got = p.result()
        assert np.array_equal(got.view(np.uint16), W[rows, :].astype(np.float16).view(np.uint16)), (bits, base)


# ------------------------------------------------------------------ StreamK at the other field widths
@pytest.mark.parametrize("bits", [8, 3, 2])
@pytest.mark.parametrize("m,n,k,g,workgroups", [
    (16, 544, 1024, 128, 0),      # library default (capped by the iterations)
    (5, 544, 1408, 128, 7),       # segments across tiles, odd group counts
    (16, 288, 2048, 256, 3),      # group_size 256
    (20, 800, 1024, 128, 24),     # two launches of 16 and 4 rows; ragged last tile
    (1, 288, 512, 128, 2),        # whole tiles per workgroup: no fill launch
])
def test_streamk_other_field_widths(oracle, bits, m, n, k, g, workgroups):
    A, qw, s, qz, Cref = _case_and_ref(oracle, bits, m, n, k, g, seed=1400 + bits + m)
    p = DeviceProblem(A, qw, s, qz, g)
    for call in range(2):
        p.C.fill_(float("nan"))
        b.w4a16_gemm_streamk_bits(bits, *p.args(), workgroups)
        assert_parity(p.result(), Cref, f"streamk {bits}-bit m={m} n={n} k={k} g={g} W={workgroups} call {call}")


@pytest.mark.parametrize("bits", [8, 3, 2])
def test_streamk_other_field_widths_one_hot_bit_exact(bits):
    import torch
    m, n, k, g = 16, 544, 1024, 128
    if bits == 3:
        _, qw, s, qz = random_case_3bit(m, n, k, g, seed=78)
        W = np_dense_weight_3bit(qw, s, qz, g)
    else:
        _, qw, s, qz = random_case_bits(m, n, k, g, bits, seed=78)
        W = np_dense_weight_bits(qw, s, qz, g, bits)
    p = DeviceProblem(np.zeros((m, k), np.float16), qw, s, qz, g)
    for workgroups in (5, 16):
        for base in range(0, k, m):
            rows = [(base + 7 * i) % k for i in range(m)]
            A = np.zeros((m, k), np.float16)
            for i, r in enumerate(rows):
                A[i, r] = 1.0
            p.A.copy_(torch.from_numpy(A))
            b.w4a16_gemm_streamk_bits(bits, *p.args(), workgroups)
            got = p.result()
            assert np.array_equal(got.view(np.uint16), W[rows, :].astype(np.float16).view(np.uint16)), (bits, workgroups, base)


# ------------------------------------------------------------------ 2-bit fields
TWO_BIT = [
    # m, n, k, g, split_k   (n a multiple of 16)
    (1, 208, 512, 128, 1),
    (16, 208, 1024, 128, 4),
    (16, 336, 1024, 128, 8),      # ragged last tile
    (5, 80, 1408, 128, 0),        # 11 groups, the library's split
    (16, 272, 2048, 128, 2),
    (3, 144, 1024, 256, 2),
    (16, 192, 512, 64, 2),
    (9, 192, 256, 32, 4),
    (40, 272, 1024, 128, 4),
    (16, 16, 256, 128, 2),
]


@pytest.mark.parametrize("m,n,k,g,split_k", TWO_BIT)
def test_2bit_fields(oracle, m, n, k, g, split_k):
    A, qw, s, qz = random_case_bits(m, n, k, g, 2, seed=950 + m + n)
    Cref, _ = oracle.gemm_bits(A, qw, s, qz, g, 2)
    p = DeviceProblem(A, qw, s, qz, g)
    for call in range(2):
        p.C.fill_(float("nan"))
        b.w2a16_gemm(*p.args(), split_k)
        assert_parity(p.result(), Cref, f"2-bit splitk m={m} n={n} k={k} g={g} S={split_k} call {call}")
    p.C.fill_(float("nan"))
    b.w2a16_gemm_dp(*p.args())
    assert_parity(p.result(), Cref, f"2-bit dp m={m} n={n} k={k} g={g}")
    assert b.w4a16_phase_timeouts() == 0


@pytest.mark.parametrize("split_k", [1, 4])
def test_2bit_one_hot_rows_bit_exact(split_k):
    """One non-zero term per row, swept over all k: pins the field order inside a word, the word
    halves of the lane groups, the zero-point fields and the scale columns."""
    m, n, k, g = 16, 208, 1024, 128
    _, qw, s, qz = random_case_bits(m, n, k, g, 2, seed=59)
    W = np_dense_weight_bits(qw, s, qz, g, 2)
    p = DeviceProblem(np.zeros((m, k), np.float16), qw, s, qz, g)
    import torch
    for base in range(0, k, m):
        rows = [(base + 7 * i) % k for i in range(m)]
        A = np.zeros((m, k), np.float16)
        for i, r in enumerate(rows):
            A[i, r] = 1.0
        p.A.copy_(torch.from_numpy(A))
        b.w2a16_gemm(*p.args(), split_k)
        got = p.result()
        assert np.array_equal(got.view(np.uint16), W[rows, :].astype(np.float16).view(np.uint16)), base


# ------------------------------------------------------------------ 3-bit fields
THREE_BIT = [
    # m, n, k, g, split_k   (n a multiple of 32)
    (1, 224, 512, 128, 1),
    (16, 224, 1024, 128, 4),
    (16, 352, 1024, 128, 8),      # one group per part, ragged last tile (352 = 5 * 64 + 32)
    (5, 96, 1408, 128, 0),        # 11 groups, the library's split
    (16, 288, 2048, 128, 2),      # eight groups per workgroup: steady loop
    (3, 160, 1024, 256, 2),       # group_size 256
    (16, 192, 512, 64, 2),        # group_size 64
    (9, 192, 256, 32, 4),         # group_size 32: a group is one stream
    (4, 64, 4096, 128, 0),        # few rows: fixed-point reduction
    (40, 288, 1024, 128, 4),      # three launches of 16, 16, 8 rows
    (16, 32, 256, 128, 2),        # half a tile
]


@pytest.mark.parametrize("m,n,k,g,split_k", THREE_BIT)
def test_3bit_fields(oracle, m, n, k, g, split_k):
    A, qw, s, qz = random_case_3bit(m, n, k, g, seed=970 + m + n)
    Cref, _ = oracle.gemm_3bit(A, qw, s, qz, g)
    p = DeviceProblem(A, qw, s, qz, g)
    for call in range(2):
        p.C.fill_(float("nan"))
        b.w3a16_gemm(*p.args(), split_k)
        assert_parity(p.result(), Cref, f"3-bit splitk m={m} n={n} k={k} g={g} S={split_k} call {call}")
    p.C.fill_(float("nan"))
    b.w3a16_gemm_dp(*p.args())
    assert_parity(p.result(), Cref, f"3-bit dp m={m} n={n} k={k} g={g}")
    assert b.w4a16_phase_timeouts() == 0


@pytest.mark.parametrize("split_k", [1, 4])
def test_3bit_one_hot_rows_bit_exact(split_k):
    """One non-zero term per row, swept over all k: pins the position of every value in its stream
    (the two that lie across words among them), the word rows and funnel shifts of the lane
    groups, the zero-point streams along n and the scale columns."""
    m, n, k, g = 16, 224, 1024, 128
    _, qw, s, qz = random_case_3bit(m, n, k, g, seed=61)
    W = np_dense_weight_3bit(qw, s, qz, g)
    p = DeviceProblem(np.zeros((m, k), np.float16), qw, s, qz, g)
    import torch
    for base in range(0, k, m):
        rows = [(base + 7 * i) % k for i in range(m)]
        A = np.zeros((m, k), np.float16)
        for i, r in enumerate(rows):
            A[i, r] = 1.0
        p.A.copy_(torch.from_numpy(A))
        b.w3a16_gemm(*p.args(), split_k)
        got = p.result()
        assert np.array_equal(got.view(np.uint16), W[rows, :].astype(np.float16).view(np.uint16)), base


def _random_shapes_3bit(count, seed):
    rng = np.random.Generator(np.random.Philox(seed))
    out = []
    for _ in range(count):
        g = int(rng.choice([32, 64, 128, 128, 128, 256]))
        k = g * int(rng.integers(1, 41))
        n = 32 * int(rng.integers(1, 60))
        m = int(rng.choice([1, 2, 4, 5, 8, 13, 16, 17, 33]))
        out.append((m, n, k, g))
    return out


@pytest.mark.parametrize("m,n,k,g", _random_shapes_3bit(16, seed=2025))
def test_3bit_random_shapes(oracle, m, n, k, g):
    """The library's own split (uneven k shares among them) and the data-parallel kernel."""
    A, qw, s, qz = random_case_3bit(m, n, k, g, seed=3000 + m + n + k)
    Cref, _ = oracle.gemm_3bit(A, qw, s, qz, g)
    p = DeviceProblem(A, qw, s, qz, g)
    for call in range(2):
        p.C.fill_(float("nan"))
        b.w3a16_gemm(*p.args(), 0)
        assert_parity(p.result(), Cref, f"3-bit auto m={m} n={n} k={k} g={g} call {call}")
    p.C.fill_(float("nan"))
    b.w3a16_gemm_dp(*p.args())
    assert_parity(p.result(), Cref, f"3-bit dp m={m} n={n} k={k} g={g}")
    assert b.w4a16_phase_timeouts() == 0


def test_3bit_full_size(oracle):
    """The headline shape with 3-bit fields, SplitK (library's split) and data-parallel."""
    x = make_inputs(16, 4096, 4096, 128, seed=0, bits=3)
    Cref, _ = oracle.gemm_3bit(x.A, x.qweight, x.scales, x.qzeros, 128)
    p = DeviceProblem(x.A, x.qweight, x.scales, x.qzeros, 128)
    b.w3a16_gemm(*p.args(), 0)
    assert_parity(p.result(), Cref, "3-bit splitk 4096^2")
    p.C.fill_(float("nan"))
    b.w3a16_gemm_dp(*p.args())
    assert_parity(p.result(), Cref, "3-bit dp 4096^2")


def test_hip_graph_replays_other_field_widths_and_activation_ordering(oracle):
    """The 8-, 3- and 2-bit entry points (per-wave, two-strip and streaming launches) and the
    activation-ordering pair (prepare + product) captured in one HIP graph and replayed, with
    eager calls between the replays."""
    import torch
    cases = [
        # bits, m, n, k
        (8, 16, 512, 1024), (3, 5, 512, 1024), (2, 3, 512, 2048),      # per-wave
        (8, 16, 5152, 2048), (3, 9, 5152, 2048), (2, 2, 5152, 2048),   # two strips per wave
        (8, 7, 5152, 5248), (2, 12, 5152, 5248),                       # streaming kernel, uneven shares
    ]
    probs = []
    for (bits, m, n, k) in cases:
        if bits == 3:
            A, qw, s, qz = random_case_3bit(m, n, k, 128, seed=6000 + m + k)
            Cref, _ = oracle.gemm_3bit(A, qw, s, qz, 128)
            gemm = b.w3a16_gemm
        else:
            A, qw, s, qz = random_case_bits(m, n, k, 128, bits, seed=6000 + m + k)
            Cref, _ = oracle.gemm_bits(A, qw, s, qz, 128, bits)
            gemm = b.w8a16_gemm if bits == 8 else b.w2a16_gemm
        probs.append((DeviceProblem(A, qw, s, qz, 128), Cref, gemm, f"{bits}-bit m={m} n={n} k={k}"))
    # activation ordering: the group map is sorted and the rows repacked inside the graph as well
    m, n, k, g = 16, 520, 1024, 128
    A, qw, s, qz = random_case(m, n, k, g, seed=6100)
    g_idx = random_act_order(k, g, seed=6101)
    Cref_ao, _ = oracle.gemm_gidx(A, qw, s, qz, g_idx)
    pa = DeviceProblem(A, qw, s, qz, g)
    d_gidx = dev(g_idx)
    qw_sorted = torch.empty_like(pa.qweight)
    perm = torch.full((k,), -1, dtype=torch.int32, device="cuda")
    status = torch.full((1,), 7, dtype=torch.int32, device="cuda")
    A_work = torch.empty_like(pa.A)

    def run_all(stream=None):
        for (p, _, gemm, _) in probs:
            gemm(*p.args(), 0, stream=stream)
        b.w4a16_actorder_prepare(pa.qweight, d_gidx, qw_sorted, perm, status, n, k, g, stream=stream)
        b.w4a16_gemm_actorder(pa.A, qw_sorted, pa.scales, pa.qzeros, perm, A_work, pa.C, m, n, k, g, 0, stream=stream)

    run_all()                                  # eager warm-up: scratch allocation happens outside the capture
    torch.cuda.synchronize()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        run_all(stream=torch.cuda.current_stream())
    for rep in range(3):
        for (p, *_rest) in probs:
            p.C.fill_(float("nan"))
        pa.C.fill_(float("nan"))
        status.fill_(7)
        perm.fill_(-1)
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for (p, Cref, _, what) in probs:
            assert_parity(p.C.cpu().numpy(), Cref, f"replay {rep}: {what}")
        assert int(status.item()) == 0
        assert_parity(pa.C.cpu().numpy(), Cref_ao, f"replay {rep}: activation ordering")
        # eager work between the replays on the same tiles
        probs[3][2](*probs[3][0].args(), 4)
        probs[6][2](*probs[6][0].args(), 0)
        torch.cuda.synchronize()
    assert b.w4a16_phase_timeouts() == 0


# ------------------------------------------------------------------ two strips per wave, other field widths
@pytest.mark.parametrize("bits", [8, 3, 2])
@pytest.mark.parametrize("m,n,k,g", [
    (16, 5152, 2048, 128),     # 41 tiles of 128 columns (the last one a quarter full), split_k 4
    (3, 2592, 4096, 128),      # few rows, split_k 8, last tile a quarter full
    (9, 5120, 2048, 256),      # group_size 256: two compute groups per parameter row
])
def test_two_strips_other_field_widths(oracle, bits, m, n, k, g):
    """The library's own launch for these shapes is the two-strip kernel (128-column tiles, one
    compute group per wave, zeroing by the service wavefront) at every field width."""
    plan = b.w4a16_plan_bits(bits, m, n, k, g)
    assert plan["tile_cols"] == 128 and plan["split_k"] * 4 == k // 128, plan
    if bits == 3:
        A, qw, s, qz = random_case_3bit(m, n, k, g, seed=4000 + m)
        Cref, _ = oracle.gemm_3bit(A, qw, s, qz, g)
        gemm = b.w3a16_gemm
    else:
        A, qw, s, qz = random_case_bits(m, n, k, g, bits, seed=4000 + m)
        Cref, _ = oracle.gemm_bits(A, qw, s, qz, g, bits)
        gemm = b.w8a16_gemm if bits == 8 else b.w2a16_gemm
    p = DeviceProblem(A, qw, s, qz, g)
    for call in range(3):
        p.C.fill_(float("nan"))
        gemm(*p.args(), 0)
        assert_parity(p.result(), Cref, f"{bits}-bit two strips m={m} n={n} k={k} g={g} call {call}")
    assert b.w4a16_phase_timeouts() == 0


@pytest.mark.parametrize("bits", [8, 3, 2])
def test_two_strips_other_field_widths_one_hot_bit_exact(bits):
    """One non-zero term per row over all k on a two-strip launch: both strips of every wave pick
    the right fields, zero points and scales."""
    m, n, k, g = 16, 5152, 2048, 128
    assert b.w4a16_plan_bits(bits, m, n, k, g)["tile_cols"] == 128
    if bits == 3:
        _, qw, s, qz = random_case_3bit(m, n, k, g, seed=67)
        W = np_dense_weight_3bit(qw, s, qz, g)
        gemm = b.w3a16_gemm
    else:
        _, qw, s, qz = random_case_bits(m, n, k, g, bits, seed=67)
        W = np_dense_weight_bits(qw, s, qz, g, bits)
        gemm = b.w8a16_gemm if bits == 8 else b.w2a16_gemm
    p = DeviceProblem(np.zeros((m, k), np.float16), qw, s, qz, g)
    import torch
    for base in range(0, k, m):
        rows = [(base + 7 * i) % k for i in range(m)]
        A = np.zeros((m, k), np.float16)
        for i, r in enumerate(rows):
            A[i, r] = 1.0
        p.A.copy_(torch.from_numpy(A))
        gemm(*p.args(), 0)
        got = p.result()
        assert np.array_equal(got.view(np.uint16), W[rows, :].astype(np.float16).view(np.uint16)), base


# ------------------------------------------------------------------ streaming kernel, other field widths
@pytest.mark.parametrize("bits,m,n,k,g", [
    (8, 7, 5152, 5248, 128),      # 41 groups over 8 slices: uneven shares, odd counts (phantom group)
    (2, 7, 5152, 5248, 128),
    (8, 16, 5152, 5376, 256),     # group_size 256
    (2, 12, 2592, 16384, 128),    # 23 slices (a split that fills the machine), last tile an eighth full
    (8, 12, 2592, 16384, 128),
    (3, 9, 8224, 8320, 128),      # 65 groups over 7 slices
    (3, 16, 8192, 8192, 128),
    (8, 16, 8192, 8192, 128),
    (2, 16, 8192, 8192, 128),
    (2, 6, 13312, 8192, 128),     # eight waves: two k parts of eight groups in each of four slices
    (3, 16, 16896, 9216, 128),    # eight waves, three slices
])
def test_streaming_kernel_other_field_widths(oracle, bits, m, n, k, g):
    """The library's own launch for these shapes is the streaming kernel (256-column tiles,
    activations shared through LDS) at the other field widths."""
    plan = b.w4a16_plan_bits(bits, m, n, k, g)
    assert plan["tile_cols"] == 256, plan
    assert plan["waves"] == (8 if n > 13000 else 4), plan
    if bits == 3:
        A, qw, s, qz = random_case_3bit(m, n, k, g, seed=5000 + m)
        Cref, _ = oracle.gemm_3bit(A, qw, s, qz, g)
        gemm = b.w3a16_gemm
    else:
        A, qw, s, qz = random_case_bits(m, n, k, g, bits, seed=5000 + m)
        Cref, _ = oracle.gemm_bits(A, qw, s, qz, g, bits)
        gemm = b.w8a16_gemm if bits == 8 else b.w2a16_gemm
    p = DeviceProblem(A, qw, s, qz, g)
    for call in range(3):
        p.C.fill_(float("nan"))
        gemm(*p.args(), 0)
        assert_parity(p.result(), Cref, f"{bits}-bit streaming m={m} n={n} k={k} g={g} call {call} plan {plan}")
    assert b.w4a16_phase_timeouts() == 0


@pytest.mark.parametrize("bits,m,n,k", [(8, 7, 5152, 5248), (2, 7, 5152, 5248), (3, 9, 8224, 8320)])
def test_streaming_kernel_other_field_widths_one_hot_bit_exact(bits, m, n, k):
    """One non-zero term per row on a streaming launch with uneven shares: sampled k (every
    position of a 32-value stream and of a group, first and last groups of the slices)."""
    g = 128
    assert b.w4a16_plan_bits(bits, m, n, k, g)["tile_cols"] == 256
    if bits == 3:
        _, qw, s, qz = random_case_3bit(m, n, k, g, seed=71)
        W = np_dense_weight_3bit(qw, s, qz, g)
        gemm = b.w3a16_gemm
    else:
        _, qw, s, qz = random_case_bits(m, n, k, g, bits, seed=71)
        W = np_dense_weight_bits(qw, s, qz, g, bits)
        gemm = b.w8a16_gemm if bits == 8 else b.w2a16_gemm
    p = DeviceProblem(np.zeros((m, k), np.float16), qw, s, qz, g)
    import torch
    for base in range(0, k, 97):
        rows = [(base + 131 * i) % k for i in range(m)]
        A = np.zeros((m, k), np.float16)
        for i, r in enumerate(rows):
            A[i, r] = 1.0
        p.A.copy_(torch.from_numpy(A))
        gemm(*p.args(), 0)
        got = p.result()
        assert np.array_equal(got.view(np.uint16), W[rows, :].astype(np.float16).view(np.uint16)), base


# ------------------------------------------------------------------ seeded random shapes
def _random_shapes(count, seed):
    rng = np.random.Generator(np.random.Philox(seed))
    out = []
    for _ in range(count):
        g = int(rng.choice([32, 64, 128, 128, 128, 256]))
        groups = int(rng.integers(1, 25))
        k = g * groups
        n = 8 * int(rng.integers(1, 90))
        m = int(rng.choice([1, 2, 3, 4, 5, 7, 8, 11, 15, 16, 17, 31, 33, 64, 70]))
        out.append((m, n, k, g))
    return out


@pytest.mark.parametrize("m,n,k,g", _random_shapes(48, seed=2024))
def test_random_shapes_library_plan(oracle, m, n, k, g):
    """Whatever launch the library picks for a shape (per-wave, two strips, streaming with one
    or several row tiles, uneven shares), SplitK, data-parallel and StreamK agree with the oracle."""
    A, qw, s, qz = random_case(m, n, k, g, seed=1000 + m + n + k)
    Cref, _ = oracle.gemm(A, qw, s, qz, g)
    p = DeviceProblem(A, qw, s, qz, g)
    for call in range(2):
        p.C.fill_(float("nan"))
        b.w4a16_gemm(*p.args(), 0)
        assert_parity(p.result(), Cref, f"auto m={m} n={n} k={k} g={g} call {call} plan {b.w4a16_plan(m, n, k, g)}")
    p.C.fill_(float("nan"))
    b.w4a16_gemm_dp(*p.args())
    assert_parity(p.result(), Cref, f"dp m={m} n={n} k={k} g={g}")
    if g >= 128:
        p.C.fill_(float("nan"))
        b.w4a16_gemm_streamk(*p.args(), 0)
        assert_parity(p.result(), Cref, f"streamk m={m} n={n} k={k} g={g}")
    assert b.w4a16_phase_timeouts() == 0


def _random_large_shapes(count, seed):
    """Shapes of the size the plan's rules are about (n up to 28800, k up to 15232, up to 64 MiB
    of packed weights so that the oracle stays at about a second per shape)."""
    rng = np.random.Generator(np.random.Philox(seed))
    out = []
    while len(out) < count:
        n = int(rng.integers(128, 3600)) * 8
        k = int(rng.integers(8, 120)) * 128
        m = int(rng.choice([1, 2, 4, 6, 8, 12, 16]))
        if n * k <= (1 << 27):
            out.append((m, n, k))
    return out


# shapes on which an audit of the plan moved a rule: eight-wave streaming workgroups at two rows,
# close to two workgroups per compute unit, six slices of one group per wave, unsplit 32- and
# 64-column tiles with a long k, 129 tiles
_PLAN_RULE_SHAPES = [(2, 25112, 4096), (8, 22232, 7808), (1, 2304, 3072), (6, 7216, 2304), (16, 8216, 1920),
                     (4, 1864, 1408), (12, 4248, 2688), (1, 23064, 8192),
                     # two strips on 144 workgroups, one group per wave kept over a two-wave split, a nearly even
                     # split (97 and 49 groups), two strips ahead of unsplit tiles
                     (6, 6144, 1536), (16, 1024, 4096), (12, 1856, 12416), (6, 1536, 6272), (2, 8192, 2048), (16, 11264, 2560)]


@pytest.mark.parametrize("m,n,k", _random_large_shapes(20, seed=77) + _PLAN_RULE_SHAPES)
def test_random_large_shapes_library_plan(oracle, m, n, k):
    """The launch the library picks at full-size shapes (every branch of the plan: narrow unsplit
    tiles, 64-column tiles with fixed-point adds, two strips, the streaming kernel with four and
    eight waves) against the oracle, twice in a row (the in-kernel zeroing counts calls)."""
    A, qw, s, qz = random_case(m, n, k, 128, seed=m + n + k)
    Cref, _ = oracle.gemm(A, qw, s, qz, 128)
    p = DeviceProblem(A, qw, s, qz, 128)
    plan = b.w4a16_plan(m, n, k, 128)
    for call in range(2):
        p.C.fill_(float("nan"))
        b.w4a16_gemm(*p.args(), 0)
        assert_parity(p.result(), Cref, f"m={m} n={n} k={k} call {call} plan {plan}")
    assert b.w4a16_phase_timeouts() == 0


@pytest.mark.parametrize("bits", [8, 3, 2])
@pytest.mark.parametrize("m,n,k", [(m, n // 32 * 32, k) for (m, n, k) in _random_large_shapes(8, seed=78)] +   # a zero-point word holds 32 / bits columns
                         [(16, 15392, 2048), (9, 8192, 8192), (20, 13312, 4096),
                          # runs of several groups per wave with the service wavefront (even and ragged), the streaming
                          # kernel at six rows, two slices of it on a wide matrix, a split of short k
                          (6, 1536, 12288), (16, 928, 11776), (6, 16896, 4096), (12, 27712, 5632), (16, 8192, 2048)])
def test_random_large_shapes_other_field_widths(oracle, bits, m, n, k):
    """The same at 8-, 3- and 2-bit fields, whose plans have their own bounds; each width against its
    own oracle function."""
    A, qw, s, qz, Cref = _case_and_ref(oracle, bits, m, n, k, 128, seed=bits + m + n + k)
    p = DeviceProblem(A, qw, s, qz, 128)
    gemm = {8: b.w8a16_gemm, 3: b.w3a16_gemm, 2: b.w2a16_gemm}[bits]
    plan = b.w4a16_plan_bits(bits, m, n, k, 128)
    for call in range(2):
        p.C.fill_(float("nan"))
        gemm(*p.args(), 0)
        assert_parity(p.result(), Cref, f"{bits}-bit m={m} n={n} k={k} call {call} plan {plan}")
    assert b.w4a16_phase_timeouts() == 0


@pytest.mark.parametrize("m,n,k,split_k,tile_cols,waves", [
    (16, 8192, 2048, 0, 0, 0),       # two strips per wave by the plan, split_k 4
    (8, 16400, 1024, 0, 0, 0),       # two strips, split_k 2, ragged last tile
    (3, 8192, 2048, 0, 0, 0),        # two strips at few rows (in-kernel zeroing instead of fixed-point adds)
    (16, 5632, 8192, 4, 256, 8),     # eight-wave streaming workgroups, two k parts of eight groups
    (9, 5632, 16384, 0, 0, 0),       # a split that is no power of two (11 slices)
    (16, 16896, 9216, 0, 0, 0),      # the plan's own eight-wave choice: three slices, two k parts of twelve groups
    (16, 2304, 4096, 0, 0, 0),       # under-filled launch
])
def test_medium_shapes_plan_variants(oracle, m, n, k, split_k, tile_cols, waves):
    x = make_inputs(m, n, k, 128, seed=5)
    Cref, _ = oracle.gemm(x.A, x.qweight, x.scales, x.qzeros, 128)
    p = DeviceProblem(x.A, x.qweight, x.scales, x.qzeros, 128)
    for call in range(2):
        p.C.fill_(float("nan"))
        b.w4a16_gemm_ex(*p.args(), split_k, tile_cols, waves, 0)
        assert_parity(p.result(), Cref, f"m={m} n={n} k={k} call {call} plan {b.w4a16_plan(m, n, k, 128)}")
    assert b.w4a16_phase_timeouts() == 0


def test_phase_protocol_64_slices_one_hot_bit_exact():
    """The in-kernel zeroing with its largest split (64 slices): one non-zero term per row, so
    the 63 other packed-fp16 adds of every element are exact zeros and the result is exact."""
    m, n, k, g = 16, 72, 8192, 128
    _, qw, s, qz = random_case(m, n, k, g, seed=61)
    W = np_dense_weight(qw, s, qz, g)
    p = DeviceProblem(np.zeros((m, k), np.float16), qw, s, qz, g)
    import torch
    for base in range(0, k, 16 * m):
        rows = [(base + 131 * i) % k for i in range(m)]
        A = np.zeros((m, k), np.float16)
        for i, r in enumerate(rows):
            A[i, r] = 1.0
        p.A.copy_(torch.from_numpy(A))
        b.w4a16_gemm_ex(*p.args(), 64, 64, 1, b.REDUCE_ATOMIC_PK_F16_PHASE)
        got = p.result()
        assert np.array_equal(got.view(np.uint16), W[rows, :].astype(np.float16).view(np.uint16)), base
    assert b.w4a16_phase_timeouts() == 0


# ------------------------------------------------------------------ reduction flavours at their limits
@pytest.mark.parametrize("m,n,k,g,split_k,tile_cols,waves,reduce", [
    (5, 72, 16384, 128, 128, 64, 1, 1),      # 128 slices, fp32 atomics + ticket
    (5, 72, 16384, 128, 128, 64, 1, 3),      # 128 slices, workspace summed in slice order
    (16, 72, 8192, 128, 64, 64, 1, 4),       # 64 slices, fixed-point adds at 16 rows
    (16, 136, 8192, 128, 63, 64, 1, 4),      # 63 slices: 64 groups dealt unevenly
    (3, 65536, 256, 128, 2, 64, 1, 5),       # the last tile origin the in-kernel zeroing covers
    (16, 65536, 512, 128, 4, 256, 4, 5),     # the same for the streaming kernel
    (16, 65536, 512, 128, 4, 128, 1, 5),     # and for two strips per wave
    (2, 72, 8192, 32, 64, 64, 4, 4),         # group_size 32: 256 compute groups, one per wave
])
def test_reduction_limits(oracle, m, n, k, g, split_k, tile_cols, waves, reduce):
    A, qw, s, qz = random_case(m, n, k, g, seed=1400 + m + k % 71)
    Cref, _ = oracle.gemm(A, qw, s, qz, g)
    p = DeviceProblem(A, qw, s, qz, g)
    for call in range(3):
        p.C.fill_(float("nan"))
        b.w4a16_gemm_ex(*p.args(), split_k, tile_cols, waves, reduce)
        assert_parity(p.result(), Cref, f"m={m} n={n} k={k} g={g} S={split_k} tile={tile_cols} reduce={reduce} call {call}")
    assert b.w4a16_phase_timeouts() == 0


def test_random_call_sequence(oracle):
    """120 calls in random order over a pool of problems and launch variants that share the
    library's per-device scratch (flags and counts of several split factors, fixed-point words,
    tickets, workspace): every call must leave that state right for whichever call comes next."""
    rng = np.random.Generator(np.random.Philox(77))
    pool = []
    for (m, n, k, g) in ((16, 520, 2048, 128), (3, 520, 2048, 128), (9, 1032, 1024, 128), (16, 264, 4096, 256),
                         (5, 200, 1408, 128), (40, 520, 2048, 128)):
        A, qw, s, qz = random_case(m, n, k, g, seed=1500 + m + n)
        Cref, _ = oracle.gemm(A, qw, s, qz, g)
        cg = k // 128
        variants = [(0, 0, 0, 0), (1, 64, 4, 0)]
        if m <= 16:
            for S in (2, 4, 8):
                if S * 4 <= cg:
                    variants += [(S, 64, 4, r) for r in (1, 2, 3, 4, 5)]
                    variants += [(S, 256, 4, 5), (S, 256, 4, 2), (S, 32, 2, 5)]
            if cg % 4 == 0 and cg // 4 in (2, 4, 8):
                variants.append((cg // 4, 128, 4, 0))
            variants += [("dp",), ("streamk", 0), ("streamk", 5)]
        else:
            variants += [(2, 256, 4, 5), (4, 0, 0, 0), ("dp",)]
        pool.append((DeviceProblem(A, qw, s, qz, g), Cref, variants))
    for step in range(120):
        p, Cref, variants = pool[int(rng.integers(len(pool)))]
        v = variants[int(rng.integers(len(variants)))]
        p.C.fill_(float("nan"))
        if v[0] == "dp":
            b.w4a16_gemm_dp(*p.args())
        elif v[0] == "streamk":
            b.w4a16_gemm_streamk(*p.args(), v[1])
        else:
            b.w4a16_gemm_ex(*p.args(), *v)
        assert_parity(p.result(), Cref, f"step {step}: m={p.m} n={p.n} k={p.k} g={p.g} variant {v}")
    assert b.w4a16_phase_timeouts() == 0


@pytest.mark.parametrize("m,n,k,g,split_k,tile_cols,waves", [
    (16, 200, 1536, 128, 3, 64, 4),       # three slices of four groups, per-wave kernel
    (9, 328, 1920, 128, 5, 64, 1),        # five slices of three groups
    (16, 520, 3072, 128, 6, 256, 4),      # streaming kernel, six slices
    (16, 520, 1664, 128, 13, 256, 4),     # thirteen slices of one group: ring depth 1
    (7, 264, 5120, 128, 10, 128, 4),      # two strips per wave, ten slices
    (16, 264, 3584, 128, 7, 64, 4),       # seven slices, service wavefront (one group per wave)
])
def test_phase_protocol_any_split(oracle, m, n, k, g, split_k, tile_cols, waves):
    """The in-kernel zeroing keeps its flags and counts per split_k, for any split_k up to 64."""
    A, qw, s, qz = random_case(m, n, k, g, seed=1600 + m + k % 53)
    Cref, _ = oracle.gemm(A, qw, s, qz, g)
    p = DeviceProblem(A, qw, s, qz, g)
    for call in range(3):
        p.C.fill_(float("nan"))
        b.w4a16_gemm_ex(*p.args(), split_k, tile_cols, waves, b.REDUCE_ATOMIC_PK_F16_PHASE)
        assert_parity(p.result(), Cref, f"m={m} n={n} k={k} S={split_k} tile={tile_cols} call {call}")
    assert b.w4a16_phase_timeouts() == 0


# ------------------------------------------------------------------ extremes of the shape range
@pytest.mark.parametrize("m,n,k,g,split_k", [
    (4, 66048, 256, 128, 2),      # n beyond the 65536 columns the in-kernel zeroing covers: fill kernel instead
    (16, 66048, 512, 128, 0),     # the library's own choice there
    (9, 66048, 2048, 128, 4),     # streaming kernel beyond 65536 columns: fill kernel + atomics
    (9, 8, 65536, 128, 0),        # one 8-column strip, 512 groups
    (4, 8, 65536, 128, 64),       # 64 slices of 8 groups, fixed-point adds
    (16, 8, 65536, 128, 32),      # 32 slices with packed-fp16 adds (more would leave too little of the tolerance)
    (1, 16, 32768, 32, 16),       # group_size 32: 1024 compute groups
    (64, 72, 16384, 128, 0),      # four row tiles on a narrow matrix
])
def test_extreme_shapes(oracle, m, n, k, g, split_k):
    A, qw, s, qz = random_case(m, n, k, g, seed=1100 + m + n % 97)
    Cref, _ = oracle.gemm(A, qw, s, qz, g)
    p = DeviceProblem(A, qw, s, qz, g)
    for call in range(2):
        p.C.fill_(float("nan"))
        b.w4a16_gemm_ex(*p.args(), split_k, 0, 0, 0)
        assert_parity(p.result(), Cref, f"m={m} n={n} k={k} g={g} S={split_k} call {call} plan {b.w4a16_plan(min(m, 64), n, k, g, split_k=split_k)}")
    p.C.fill_(float("nan"))
    b.w4a16_gemm_dp(*p.args())
    assert_parity(p.result(), Cref, f"dp m={m} n={n} k={k} g={g}")
    assert b.w4a16_phase_timeouts() == 0


# ------------------------------------------------------------------ activation ordering (group index per row)
@pytest.mark.parametrize("m,n,k,g,split_k", [
    (1, 200, 512, 128, 0),
    (16, 264, 1024, 128, 4),
    (7, 136, 1408, 128, 0),       # 11 groups
    (16, 192, 512, 32, 2),
    (9, 72, 1024, 256, 2),
    (40, 264, 1024, 128, 0),      # more than 16 rows
    (16, 4096, 4096, 128, 0),     # the headline shape
])
def test_activation_ordering(oracle, m, n, k, g, split_k):
    import torch
    A, qw, s, qz = random_case(m, n, k, g, seed=1200 + m + n % 89)
    g_idx = random_act_order(k, g, seed=1300 + k)
    Cref, _ = oracle.gemm_gidx(A, qw, s, qz, g_idx)
    p = DeviceProblem(A, qw, s, qz, g)
    d_gidx = dev(g_idx)
    qw_sorted = torch.empty_like(p.qweight)
    perm = torch.full((k,), -1, dtype=torch.int32, device="cuda")
    status = torch.full((1,), 7, dtype=torch.int32, device="cuda")
    A_work = torch.empty_like(p.A)
    b.w4a16_actorder_prepare(p.qweight, d_gidx, qw_sorted, perm, status, n, k, g)
    torch.cuda.synchronize()
    assert int(status.item()) == 0
    order = np.argsort(g_idx, kind="stable")
    assert np.array_equal(perm.cpu().numpy(), order)
    assert np.array_equal(oracle.unpack_qweight(qw_sorted.cpu().numpy()), oracle.unpack_qweight(qw)[order])
    for call in range(2):
        p.C.fill_(float("nan"))
        b.w4a16_gemm_actorder(p.A, qw_sorted, p.scales, p.qzeros, perm, A_work, p.C, m, n, k, g, split_k)
        assert_parity(p.result(), Cref, f"act-order m={m} n={n} k={k} g={g} S={split_k} call {call}")
    # the plain product of the same buffers is something else: the group map matters
    if k // g > 1:
        b.w4a16_gemm(*p.args(), 0)
        assert np.abs(p.result().astype(np.float64) - Cref).max() > 1e-2 * np.abs(Cref).max()


def test_activation_ordering_rejects_bad_group_map():
    import torch
    n, k, g = 64, 512, 128
    _, qw, s, qz = random_case(1, n, k, g, seed=5)
    for bad in (np.zeros(k, np.int32),                                  # every row in group 0
                np.concatenate([np.arange(k - 1) // g, [99]]).astype(np.int32),   # an index outside the groups
                np.full(k, -5, np.int32)):
        qws = torch.empty((k // 8, n), dtype=torch.int32, device="cuda")
        perm = torch.full((k,), 1 << 30, dtype=torch.int32, device="cuda")   # garbage the kernel must not follow
        status = torch.zeros((1,), dtype=torch.int32, device="cuda")
        b.w4a16_actorder_prepare(dev(qw), dev(bad), qws, perm, status, n, k, g)
        torch.cuda.synchronize()
        assert int(status.item()) == 1


# ------------------------------------------------------------------ full-size configurations
def _full(oracle, m, nk, seed=0):
    x = make_inputs(m, nk, nk, 128, seed=seed)
    Cref, _ = oracle.gemm(x.A, x.qweight, x.scales, x.qzeros, 128)
    return x, Cref, DeviceProblem(x.A, x.qweight, x.scales, x.qzeros, 128)


def test_cfg2_split_sweep(oracle):
    """m = 16, n = k = 4096, split_k in {1, 2, 4, 8, 16}, every reduction flavour, and DP."""
    x, Cref, p = _full(oracle, 16, 4096)
    for split_k in (1, 2, 4, 8, 16):
        for reduce in (b.REDUCE_ATOMIC_F32, b.REDUCE_ATOMIC_PK_F16, b.REDUCE_WORKSPACE, b.REDUCE_ATOMIC_FIXED,
                       b.REDUCE_ATOMIC_PK_F16_PHASE):
            if split_k == 1 and reduce == b.REDUCE_ATOMIC_PK_F16_PHASE:
                continue
            p.C.fill_(float("nan"))
            b.w4a16_gemm_ex(*p.args(), split_k, 0, 0, reduce)
            assert_parity(p.result(), Cref, f"cfg2 S={split_k} reduce={reduce}")
    p.C.fill_(float("nan"))
    b.w4a16_gemm_dp(*p.args())
    assert_parity(p.result(), Cref, "cfg2 dp")
    assert b.w4a16_phase_timeouts() == 0


@pytest.mark.parametrize("nk", [4096, 8192])
def test_cfg3_m_sweep(oracle, nk):
    """m in {1, 2, 4, 8, 16} x n = k in {4096, 8192}: SplitK (library default) and DP."""
    x16 = make_inputs(16, nk, nk, 128, seed=0)
    for m in (1, 2, 4, 8, 16):
        A = np.ascontiguousarray(x16.A[:m])
        Cref, _ = oracle.gemm(A, x16.qweight, x16.scales, x16.qzeros, 128)
        p = DeviceProblem(A, x16.qweight, x16.scales, x16.qzeros, 128)
        b.w4a16_gemm(*p.args(), 0)
        assert_parity(p.result(), Cref, f"cfg3 splitk m={m} nk={nk}")
        p.C.fill_(float("nan"))
        b.w4a16_gemm_dp(*p.args())
        assert_parity(p.result(), Cref, f"cfg3 dp m={m} nk={nk}")
    assert b.w4a16_phase_timeouts() == 0


def test_cfg4_split_sweep(oracle):
    x, Cref, p = _full(oracle, 16, 8192)
    for split_k in (1, 2, 4, 8, 16, 32):
        p.C.fill_(float("nan"))
        b.w4a16_gemm(*p.args(), split_k)
        assert_parity(p.result(), Cref, f"cfg4 S={split_k}")
    assert b.w4a16_phase_timeouts() == 0


def test_cfg5_split_sweep(oracle):
    x, Cref, p = _full(oracle, 8, 16384)
    for split_k in (1, 4, 16, 32):
        p.C.fill_(float("nan"))
        b.w4a16_gemm(*p.args(), split_k)
        assert_parity(p.result(), Cref, f"cfg5 S={split_k}")
    p.C.fill_(float("nan"))
    b.w4a16_gemm_dp(*p.args())
    assert_parity(p.result(), Cref, "cfg5 dp")
    assert b.w4a16_phase_timeouts() == 0

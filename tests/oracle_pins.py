"""Pins of the CPU oracle: every check compares the oracle with something that is not the
oracle (numpy's float16 and matmul, exact rational arithmetic, closed forms, hand-written
digits).  Each pin is a function of an `Oracle` binding so the mutation tests can run the
same pins against deliberately broken builds of the C source.
"""
from __future__ import annotations

import pathlib
from fractions import Fraction

import numpy as np

GOLDEN = pathlib.Path(__file__).resolve().parent / "golden"


# --------------------------------------------------------------------------- helpers
def np_unpack_qweight(qweight: np.ndarray) -> np.ndarray:
    """numpy restatement used as a second, independently written unpacker:
    view each word as 4 little-endian bytes, low nibble first."""
    r, n = qweight.shape
    by = np.ascontiguousarray(qweight).view(np.uint8).reshape(r, n, 4)      # byte b = bits 8b..8b+7
    nib = np.stack([by & 0xF, by >> 4], axis=-1).reshape(r, n, 8)           # field 2b, 2b+1
    return np.ascontiguousarray(nib.transpose(0, 2, 1)).reshape(r * 8, n)


def np_unpack_qzeros(qzeros: np.ndarray) -> np.ndarray:
    g, c = qzeros.shape
    by = np.ascontiguousarray(qzeros).view(np.uint8).reshape(g, c, 4)
    nib = np.stack([by & 0xF, by >> 4], axis=-1).reshape(g, c * 8)
    return nib


def np_dense_weight(qweight, scales, qzeros, group_size) -> np.ndarray:
    """float64 W [k, n] from the numpy unpackers."""
    q = np_unpack_qweight(qweight).astype(np.int64)
    z = np.repeat(np_unpack_qzeros(qzeros).astype(np.int64), group_size, axis=0)
    s = np.repeat(scales.astype(np.float64), group_size, axis=0)
    return (q - z) * s


def random_case(m, n, k, g, seed):
    rng = np.random.Generator(np.random.Philox(seed))
    A = rng.standard_normal((m, k), dtype=np.float32).astype(np.float16)
    qw = rng.integers(0, 1 << 32, size=(k // 8, n), dtype=np.uint32).view(np.int32)
    s = rng.uniform(0.001, 0.01, size=(k // g, n)).astype(np.float16)
    qz = rng.integers(0, 1 << 32, size=(k // g, n // 8), dtype=np.uint32).view(np.int32)
    return A, qw, s, qz


# --------------------------------------------------------------------------- fp16 conversions
def pin_half_to_float_exhaustive(o):
    """All 65536 fp16 bit patterns against numpy's float16 -> float32."""
    bits = np.arange(65536, dtype=np.uint16)
    ref = bits.view(np.float16).astype(np.float32)
    got = np.array([o.half_to_float(int(b)) for b in bits], dtype=np.float32)
    nan = np.isnan(ref)
    assert np.array_equal(np.isnan(got), nan)
    assert np.array_equal(got[~nan].view(np.uint32), ref[~nan].view(np.uint32))


def pin_double_to_half_rounding(o):
    """Round-to-nearest-even from fp64 in one rounding, against numpy's float64 -> float16:
    every representable half, every midpoint between neighbours, the neighbours of the
    midpoints, overflow, subnormals and random doubles."""
    halves = np.arange(0, 0x7C00, dtype=np.uint16).view(np.float16).astype(np.float64)
    mids = (halves[:-1] + halves[1:]) / 2
    pts = np.concatenate([halves, mids, np.nextafter(mids, np.inf), np.nextafter(mids, -np.inf),
                          [65504.0, 65519.9, 65520.0, 65520.1, 1e9, 2.0 ** -25, 2.0 ** -24 * 0.5000001,
                           2.0 ** -26, 1e-300, 0.0]])
    rng = np.random.Generator(np.random.Philox(7))
    pts = np.concatenate([pts, rng.standard_normal(4000) * 10.0 ** rng.integers(-8, 5, 4000)])
    pts = np.concatenate([pts, -pts])
    with np.errstate(over="ignore"):
        ref = pts.astype(np.float16).view(np.uint16)
    got = np.array([o.double_to_half(float(x)) for x in pts], dtype=np.uint16)
    bad = np.nonzero(got != ref)[0]
    assert bad.size == 0, (pts[bad[:5]], got[bad[:5]], ref[bad[:5]])
    # float32 entry point
    f = pts.astype(np.float32)
    with np.errstate(over="ignore"):
        ref32 = f.astype(np.float16).view(np.uint16)
    got32 = np.array([o.float_to_half(x) for x in f[:3000]], dtype=np.uint16)
    assert np.array_equal(got32, ref32[:3000])


# --------------------------------------------------------------------------- pack / unpack
def pin_unpack_known_words(o):
    """Hand-written words whose fields are read off their hex digits."""
    words = np.array([[0x76543210, 0x89ABCDEF - (1 << 32), 0, -1]], dtype=np.int64).astype(np.int32)
    q = o.unpack_qweight(words)             # [8, 4]
    assert q[:, 0].tolist() == [0, 1, 2, 3, 4, 5, 6, 7]
    assert q[:, 1].tolist() == [15, 14, 13, 12, 11, 10, 9, 8]
    assert q[:, 2].tolist() == [0] * 8 and q[:, 3].tolist() == [15] * 8
    z = o.unpack_qzeros(words)              # [1, 32]
    assert z[0, :8].tolist() == [0, 1, 2, 3, 4, 5, 6, 7]
    assert z[0, 8:16].tolist() == [15, 14, 13, 12, 11, 10, 9, 8]
    assert z[0, 24:].tolist() == [15] * 8


def pin_pack_unpack_bijection(o):
    rng = np.random.Generator(np.random.Philox(11))
    q = rng.integers(0, 16, size=(64, 40), dtype=np.uint8)
    assert np.array_equal(o.unpack_qweight(o.pack_qweight(q)), q)
    words = rng.integers(0, 1 << 32, size=(8, 40), dtype=np.uint32).view(np.int32)
    assert (words < 0).any()
    assert np.array_equal(o.pack_qweight(o.unpack_qweight(words)), words)
    z = rng.integers(0, 16, size=(5, 48), dtype=np.uint8)
    assert np.array_equal(o.unpack_qzeros(o.pack_qzeros(z)), z)
    zw = rng.integers(0, 1 << 32, size=(5, 6), dtype=np.uint32).view(np.int32)
    assert np.array_equal(o.pack_qzeros(o.unpack_qzeros(zw)), zw)
    # against the byte-view numpy unpackers (written differently: bytes and nibbles, no shifts by 4*i)
    assert np.array_equal(o.unpack_qweight(words), np_unpack_qweight(words))
    assert np.array_equal(o.unpack_qzeros(zw), np_unpack_qzeros(zw))


# --------------------------------------------------------------------------- tiny brute force
def load_tiny_fixture():
    sections, cur = {}, None
    for line in (GOLDEN / "tiny_m2_n16_k16_g8.txt").read_text().splitlines():
        if not line or line.startswith("#"):
            continue
        if line.startswith("["):
            cur = line[1:line.index("]")]
            sections[cur] = []
        else:
            sections[cur].append(line)
    q = [[int(c, 16) for c in row] for row in sections["q"]]
    z = [[int(c, 16) for c in row] for row in sections["z"]]
    se = [[int(t) for t in row.split()] for row in sections["scale_exponent"]]
    A = [[int(t) for t in row.split()] for row in sections["A"]]
    qweight = [[int(t, 16) for t in row.split()] for row in sections["qweight"]]
    qzeros = [[int(t, 16) for t in row.split()] for row in sections["qzeros"]]
    return q, z, se, A, qweight, qzeros


def pin_tiny_exact_rationals(o):
    """m=2, n=k=16, g=8: packed words go to the oracle, the unpacked digits go to an exact
    rational expansion of every dot product.  All values are dyadic and small, so the fp32
    and fp64 oracles must both be exactly equal to the rational result."""
    q, z, se, A, qweight, qzeros = load_tiny_fixture()
    m, k, n, g = 2, 16, 16, 8
    expect = [[sum(Fraction(A[i][kk]) * (q[kk][j] - z[kk // g][j]) * Fraction(2) ** se[kk // g][j]
                   for kk in range(k)) for j in range(n)] for i in range(m)]
    A_np = np.array(A, dtype=np.float16)
    s_np = np.array([[2.0 ** e for e in row] for row in se], dtype=np.float16)
    qw_np = np.array(qweight, dtype=np.uint32).view(np.int32)
    qz_np = np.array(qzeros, dtype=np.uint32).view(np.int32)
    assert np.array_equal(o.unpack_qweight(qw_np), np.array(q, dtype=np.uint8))
    assert np.array_equal(o.unpack_qzeros(qz_np), np.array(z, dtype=np.uint8))
    for acc in ("f64", "f32"):
        for split_k, block_k in ((1, 0), (2, 0), (2, 4)):
            Cref, C16 = o.gemm(A_np, qw_np, s_np, qz_np, g, split_k=split_k, block_k=block_k, acc=acc)
            for i in range(m):
                for j in range(n):
                    assert Fraction(float(Cref[i, j])) == expect[i][j], (acc, split_k, i, j)
                    assert Fraction(float(C16[i, j])) == expect[i][j]   # exactly representable in fp16 too
    W = o.dequant(qw_np, s_np, qz_np, g)
    for kk in range(k):
        for j in range(n):
            assert Fraction(float(W[kk, j])) == (q[kk][j] - z[kk // g][j]) * Fraction(2) ** se[kk // g][j]


def pin_random_tiny_vs_fractions(o):
    """Random tiny case against exact rationals built from the numpy byte-view unpackers."""
    m, n, k, g = 2, 16, 16, 8
    A, qw, s, qz = random_case(m, n, k, g, seed=3)
    q = np_unpack_qweight(qw)
    z = np_unpack_qzeros(qz)
    Cref, _ = o.gemm(A, qw, s, qz, g)
    for i in range(m):
        for j in range(n):
            ex = sum(Fraction(float(A[i, kk])) * (int(q[kk, j]) - int(z[kk // g, j])) * Fraction(float(s[kk // g, j]))
                     for kk in range(k))
            assert abs(Fraction(float(Cref[i, j])) - ex) <= abs(ex) * Fraction(1, 2 ** 48) + Fraction(1, 2 ** 60)


# --------------------------------------------------------------------------- closed forms
def pin_closed_forms(o):
    m, n, k, g = 3, 64, 256, 128
    rng = np.random.Generator(np.random.Philox(5))
    A = rng.standard_normal((m, k), dtype=np.float32).astype(np.float16)
    s_col = rng.uniform(0.001, 0.01, size=n).astype(np.float16)
    scales = np.tile(s_col, (k // g, 1))
    rowsum = A.astype(np.float64).sum(axis=1)
    for q0, z0 in ((11, 4), (2, 9), (15, 0)):
        qw = np.full((k // 8, n), (q0 * 0x11111111) & 0xFFFFFFFF, dtype=np.uint32).view(np.int32)
        qz = np.full((k // g, n // 8), (z0 * 0x11111111) & 0xFFFFFFFF, dtype=np.uint32).view(np.int32)
        Cref, _ = o.gemm(A, qw, scales, qz, g)
        expect = (q0 - z0) * s_col.astype(np.float64)[None, :] * rowsum[:, None]
        bound = 1e-12 * np.abs(A.astype(np.float64)).sum(axis=1)[:, None] * 15 * 0.01 + 1e-300
        assert np.all(np.abs(Cref - expect) <= bound)
    # q == z everywhere  =>  exactly zero, also in fp32 mode
    words = rng.integers(0, 1 << 32, size=(k // g, n // 8), dtype=np.uint32)
    zfields = np_unpack_qzeros(words.view(np.int32))                      # [k/g, n]
    qfields = np.repeat(zfields, g, axis=0).astype(np.uint8)              # q[kk][j] = z[kk/g][j]
    qw = o.pack_qweight(qfields)
    for acc in ("f64", "f32"):
        Cref, C16 = o.gemm(A, qw, scales, words.view(np.int32), g, acc=acc)
        assert not Cref.any() and not C16.view(np.uint16).any()
    # A == 0  =>  exactly zero
    A0 = np.zeros_like(A)
    _, qw_r, s_r, qz_r = random_case(m, n, k, g, seed=6)
    Cref, C16 = o.gemm(A0, qw_r, s_r, qz_r, g)
    assert not Cref.any()


def pin_matmul_library(o):
    """Reduction to numpy's float64 matmul over the numpy-unpacked dense weight, with the
    classical forward error bound; fp32 mode within k * 2^-24 * sum|a||w|."""
    for (m, n, k, g, seed) in ((5, 96, 512, 128, 1), (16, 64, 1024, 64, 2), (1, 200, 384, 128, 3)):
        A, qw, s, qz = random_case(m, n, k, g, seed)
        W = np_dense_weight(qw, s, qz, g)
        ref = A.astype(np.float64) @ W
        absdot = np.abs(A.astype(np.float64)) @ np.abs(W)
        Wo = o.dequant(qw, s, qz, g)
        assert np.array_equal(Wo.astype(np.float64), W)
        C64, C16 = o.gemm(A, qw, s, qz, g)
        assert np.all(np.abs(C64 - ref) <= 2 * k * 2.0 ** -53 * absdot + 1e-300)
        C32, _ = o.gemm(A, qw, s, qz, g, acc="f32")
        assert np.all(np.abs(C32 - ref) <= k * 2.0 ** -24 * absdot + 1e-300)
        assert np.array_equal(C16.view(np.uint16), C64.astype(np.float16).view(np.uint16))
        for split_k, block_k in ((2, 0), (4, 0), (4, 32), (3, 64)):
            if block_k == 0 and k % split_k:
                continue
            Cs, _ = o.gemm(A, qw, s, qz, g, split_k=split_k, block_k=block_k)
            assert np.all(np.abs(Cs - ref) <= 2 * k * 2.0 ** -53 * absdot + 1e-300)
            Cs32, _ = o.gemm(A, qw, s, qz, g, split_k=split_k, block_k=block_k, acc="f32")
            assert np.all(np.abs(Cs32 - ref) <= k * 2.0 ** -24 * absdot + 1e-300)


def pin_one_hot_rows(o):
    """A row equal to a unit vector e_r selects row r of W: a single term, so the result is
    exact in every mode and the fp16 output is the single rounding of w[r, :]."""
    m, n, k, g = 16, 72, 512, 128
    _, qw, s, qz = random_case(m, n, k, g, seed=9)
    W = np_dense_weight(qw, s, qz, g)
    rows = [0, 1, 7, 8, 9, 127, 128, 129, 255, 256, 300, 383, 384, 500, 510, 511]
    A = np.zeros((m, k), np.float16)
    for i, r in enumerate(rows):
        A[i, r] = 1.0
    for kw in (dict(), dict(acc="f32"), dict(split_k=4), dict(split_k=4, block_k=32, acc="f32")):
        Cref, C16 = o.gemm(A, qw, s, qz, g, **kw)
        assert np.array_equal(Cref, W[rows, :])
        assert np.array_equal(C16.view(np.uint16), W[rows, :].astype(np.float16).view(np.uint16))


def pin_group_boundary(o):
    """Scale 1 in one group and 0 elsewhere leaves exactly that group's partial sum."""
    m, n, k, g = 2, 32, 512, 128
    A, qw, _, qz = random_case(m, n, k, g, seed=4)
    q = np_unpack_qweight(qw).astype(np.int64)
    z = np_unpack_qzeros(qz).astype(np.int64)
    for gstar in range(k // g):
        s = np.zeros((k // g, n), np.float16)
        s[gstar] = 1.0
        sl = slice(g * gstar, g * (gstar + 1))
        expect = A[:, sl].astype(np.float64) @ (q[sl] - z[gstar][None, :]).astype(np.float64)
        Cref, _ = o.gemm(A, qw, s, qz, g)
        assert np.all(np.abs(Cref - expect) <= 1e-12 * np.abs(expect) + 1e-9)


def pin_linearity_and_permutation(o):
    m, n, k, g = 4, 64, 256, 128
    A, qw, s, qz = random_case(m, n, k, g, seed=8)
    C1, _ = o.gemm(A, qw, s, qz, g, acc="f32")
    C2, _ = o.gemm(A, qw, (s.astype(np.float32) * 2).astype(np.float16), qz, g, acc="f32")
    assert np.array_equal(C2, 2 * C1)                    # doubling scales is exact in binary
    perm = np.random.Generator(np.random.Philox(1)).permutation(n // 8)
    cols = (perm[:, None] * 8 + np.arange(8)[None, :]).reshape(-1)
    Cp, _ = o.gemm(A, qw[:, cols], s[:, cols], qz[:, perm], g, acc="f32")
    assert np.array_equal(Cp, C1[:, cols])
    # row permutation of A permutes rows of C
    Cr, _ = o.gemm(A[::-1], qw, s, qz, g, acc="f32")
    assert np.array_equal(Cr, C1[::-1])


def pin_splitk_invariance(o):
    """All partitions of k give the same sum up to reassociation."""
    m, n, k, g = 16, 128, 2048, 128
    A, qw, s, qz = random_case(m, n, k, g, seed=12)
    C1, _ = o.gemm(A, qw, s, qz, g)
    scale = np.abs(C1).max()
    for split_k, block_k in ((2, 0), (8, 0), (16, 0), (4, 32), (8, 64)):
        Cs, _ = o.gemm(A, qw, s, qz, g, split_k=split_k, block_k=block_k)
        assert np.abs(Cs - C1).max() <= 1e-13 * scale
        Cs32, _ = o.gemm(A, qw, s, qz, g, split_k=split_k, block_k=block_k, acc="f32")
        assert np.abs(Cs32 - C1).max() <= 1e-5 * scale


def pin_partition_order_by_cancellation(o):
    """Which k index goes into which partial sum, made visible through fp32 rounding, with the
    expected values worked out by hand.  All weights are 256 (q = 1, z = 0, s = 256); k = 32;
    the terms are +2^23 at k = 0, 1/4 at k = 8..15, -2^23 at k = 16.  An fp32 sum that holds 2^23
    loses every 1/4 added to it (the unit in the last place there is 1).
      Algorithm 1's walk with split_k = 2 over k-blocks of 8: program 0 takes blocks 0 and 2
      (2^23 - 2^23 = 0), program 1 takes blocks 1 and 3 (8 * 1/4 = 2): total 2.
      Two contiguous halves: 2^23 + 8 lost quarters = 2^23, then -2^23: total 0.
      No split: the quarters are lost as well: 0.  fp64 accumulators: always exactly 2."""
    n, k, g = 8, 32, 32
    A = np.zeros((1, k), np.float16)
    A[0, 0] = 32768.0
    A[0, 8:16] = 2.0 ** -10
    A[0, 16] = -32768.0
    qw = np.full((k // 8, n), 0x11111111, dtype=np.uint32).view(np.int32)
    qz = np.zeros((k // g, n // 8), np.int32)
    s = np.full((k // g, n), 256.0, np.float16)
    for blocked in (False, True):
        for kw, expect in ((dict(split_k=2, block_k=8, acc="f32"), 2.0), (dict(split_k=2, acc="f32"), 0.0),
                           (dict(acc="f32"), 0.0), (dict(split_k=2, block_k=8), 2.0), (dict(split_k=2), 2.0),
                           (dict(), 2.0), (dict(split_k=4, block_k=8, acc="f32"), 2.0),
                           (dict(split_k=4, acc="f32"), 2.0)):
            Cref, _ = o.gemm(A, qw, s, qz, g, blocked=blocked, **kw)
            assert np.array_equal(Cref, np.full((1, n), expect)), (blocked, kw, Cref)


def pin_blocked_arrangement_is_the_definition(o):
    """The arrangement kept for the timed CPU baseline (column blocks of 128, a cached weight
    row) against the definition, bit for bit: three and more blocks, a ragged last block, one
    block, both accumulators, both kinds of partition; and on its own against numpy's matmul."""
    for (m, n, k, g, seed) in ((5, 392, 512, 128, 31), (16, 520, 256, 64, 32), (3, 384, 384, 128, 33), (2, 72, 256, 32, 34)):
        A, qw, s, qz = random_case(m, n, k, g, seed)
        for kw in (dict(), dict(acc="f32"), dict(split_k=2), dict(split_k=4, block_k=32, acc="f32"), dict(split_k=2, block_k=64)):
            Cp, Cp16 = o.gemm(A, qw, s, qz, g, **kw)
            Cb, Cb16 = o.gemm(A, qw, s, qz, g, blocked=True, **kw)
            assert np.array_equal(Cb.view(np.uint64), Cp.view(np.uint64)), (n, kw)
            assert np.array_equal(Cb16.view(np.uint16), Cp16.view(np.uint16)), (n, kw)
        W = np_dense_weight(qw, s, qz, g)
        ref = A.astype(np.float64) @ W
        absdot = np.abs(A.astype(np.float64)) @ np.abs(W)
        Cb, _ = o.gemm(A, qw, s, qz, g, blocked=True)
        assert np.all(np.abs(Cb - ref) <= 2 * k * 2.0 ** -53 * absdot + 1e-300)


def pin_distribution(o):
    """Output statistics of the synthetic workload: Var(C) = k * Var(q - z) * E[s^2] * E[a^2]
    with Var(q - z) = 2 * (16^2 - 1) / 12 = 42.5 and E[s^2] = (a^2 + ab + b^2) / 3."""
    from paper_2402_00025_amd.inputs import make_inputs
    x = make_inputs(16, 1024, 1024, 128, seed=0)
    Cref, _ = o.gemm(x.A, x.qweight, x.scales, x.qzeros, 128)
    es2 = (0.001 ** 2 + 0.001 * 0.01 + 0.01 ** 2) / 3
    sigma = (1024 * 42.5 * es2) ** 0.5
    assert abs(Cref.std() / sigma - 1) < 0.05
    assert abs(Cref.mean()) < 0.05 * sigma


# --------------------------------------------------------------------------- other field widths
def np_unpack_rows_bits(words: np.ndarray, bits: int) -> np.ndarray:
    """numpy restatement for fields along the rows (qweight): bytes first (a little-endian view),
    then the fields inside each byte by integer division, no shifts by bits * i."""
    r, n = words.shape
    by = np.ascontiguousarray(words).view(np.uint8).reshape(r, n, 4).astype(np.int64)
    per = 8 // bits
    fields = np.stack([(by // (1 << (bits * t))) % (1 << bits) for t in range(per)], axis=-1)   # [r, n, 4, per]
    fields = fields.reshape(r, n, 4 * per)
    return np.ascontiguousarray(fields.transpose(0, 2, 1)).reshape(r * 4 * per, n).astype(np.uint8)


def np_unpack_cols_bits(words: np.ndarray, bits: int) -> np.ndarray:
    """The same for fields along the columns (qzeros)."""
    g, c = words.shape
    by = np.ascontiguousarray(words).view(np.uint8).reshape(g, c, 4).astype(np.int64)
    per = 8 // bits
    fields = np.stack([(by // (1 << (bits * t))) % (1 << bits) for t in range(per)], axis=-1)
    return fields.reshape(g, c * 4 * per).astype(np.uint8)


def random_case_bits(m, n, k, g, bits, seed):
    rng = np.random.Generator(np.random.Philox(seed))
    f = 32 // bits
    A = rng.standard_normal((m, k), dtype=np.float32).astype(np.float16)
    qw = rng.integers(0, 1 << 32, size=(k // f, n), dtype=np.uint32).view(np.int32)
    s = rng.uniform(0.001, 0.01, size=(k // g, n)).astype(np.float16)
    qz = rng.integers(0, 1 << 32, size=(k // g, n // f), dtype=np.uint32).view(np.int32)
    return A, qw, s, qz


def np_dense_weight_bits(qweight, scales, qzeros, group_size, bits) -> np.ndarray:
    q = np_unpack_rows_bits(qweight, bits).astype(np.int64)
    z = np.repeat(np_unpack_cols_bits(qzeros, bits).astype(np.int64), group_size, axis=0)
    s = np.repeat(scales.astype(np.float64), group_size, axis=0)
    return (q - z) * s


def pin_bits_known_words(o):
    """Hand-written words: bytes for 8 bits, hex digits for 4, binary digits for 2."""
    w = np.array([[0x04030201, 0x80FF7F00 - (1 << 32), -1, 0]], dtype=np.int64).astype(np.int32)
    q8 = o.unpack_qweight_bits(w, 8)
    assert q8[:, 0].tolist() == [1, 2, 3, 4] and q8[:, 1].tolist() == [0, 127, 255, 128]
    assert q8[:, 2].tolist() == [255] * 4 and q8[:, 3].tolist() == [0] * 4
    z8 = o.unpack_qzeros_bits(w, 8)
    assert z8[0].tolist() == [1, 2, 3, 4, 0, 127, 255, 128, 255, 255, 255, 255, 0, 0, 0, 0]
    w4 = np.array([[0x76543210]], dtype=np.int32)
    assert o.unpack_qweight_bits(w4, 4)[:, 0].tolist() == [0, 1, 2, 3, 4, 5, 6, 7]
    assert o.unpack_qzeros_bits(w4, 4)[0].tolist() == [0, 1, 2, 3, 4, 5, 6, 7]
    w2 = np.array([[0b11_10_01_00_00_01_10_11_11_11_00_00_01_01_10_10 - (1 << 32)]], dtype=np.int64).astype(np.int32)
    expect = [2, 2, 1, 1, 0, 0, 3, 3, 3, 2, 1, 0, 0, 1, 2, 3]          # lowest field first
    assert o.unpack_qweight_bits(w2, 2)[:, 0].tolist() == expect
    assert o.unpack_qzeros_bits(w2, 2)[0].tolist() == expect


def pin_bits_unpack_library_and_bijection(o):
    rng = np.random.Generator(np.random.Philox(13))
    for bits in (2, 4, 8):
        f = 32 // bits
        words = rng.integers(0, 1 << 32, size=(6, 40), dtype=np.uint32).view(np.int32)
        assert (words < 0).any()
        q = o.unpack_qweight_bits(words, bits)
        assert q.shape == (6 * f, 40) and int(q.max()) == (1 << bits) - 1
        assert np.array_equal(q, np_unpack_rows_bits(words, bits))
        assert np.array_equal(o.pack_qweight_bits(q, bits), words)
        zw = rng.integers(0, 1 << 32, size=(3, 5), dtype=np.uint32).view(np.int32)
        z = o.unpack_qzeros_bits(zw, bits)
        assert z.shape == (3, 5 * f)
        assert np.array_equal(z, np_unpack_cols_bits(zw, bits))
        assert np.array_equal(o.pack_qzeros_bits(z, bits), zw)
        fields = rng.integers(0, 1 << bits, size=(2 * f, 24), dtype=np.uint8)
        assert np.array_equal(o.unpack_qweight_bits(o.pack_qweight_bits(fields, bits), bits), fields)
    # 8-bit fields are the bytes of the word
    words = rng.integers(0, 1 << 32, size=(4, 8), dtype=np.uint32).view(np.int32)
    by = words.view(np.uint8).reshape(4, 8, 4)
    assert np.array_equal(o.unpack_qweight_bits(words, 8), by.transpose(0, 2, 1).reshape(16, 8))


def pin_bits4_is_the_4bit_path(o):
    """bits = 4 of the general functions against the 4-bit functions (pinned on their own)."""
    A, qw, s, qz = random_case(5, 72, 512, 128, seed=17)
    assert np.array_equal(o.unpack_qweight_bits(qw, 4), o.unpack_qweight(qw))
    assert np.array_equal(o.unpack_qzeros_bits(qz, 4), o.unpack_qzeros(qz))
    Cb, Cb16 = o.gemm_bits(A, qw, s, qz, 128, 4)
    C4, C416 = o.gemm(A, qw, s, qz, 128)
    assert np.array_equal(Cb.view(np.uint64), C4.view(np.uint64))
    assert np.array_equal(Cb16.view(np.uint16), C416.view(np.uint16))


def pin_bits_matmul_library(o):
    """numpy float64 matmul over the numpy-unpacked dense weight, classical error bound."""
    for (m, n, k, g, bits, seed) in ((5, 96, 512, 128, 8, 1), (16, 64, 256, 64, 8, 2), (3, 64, 512, 128, 2, 3),
                                     (1, 200, 384, 128, 8, 4)):
        A, qw, s, qz = random_case_bits(m, n, k, g, bits, seed)
        W = np_dense_weight_bits(qw, s, qz, g, bits)
        ref = A.astype(np.float64) @ W
        absdot = np.abs(A.astype(np.float64)) @ np.abs(W)
        C64, C16 = o.gemm_bits(A, qw, s, qz, g, bits)
        assert np.all(np.abs(C64 - ref) <= 2 * k * 2.0 ** -53 * absdot + 1e-300)
        assert np.array_equal(C16.view(np.uint16), C64.astype(np.float16).view(np.uint16))


def pin_bits_tiny_vs_fractions(o):
    """Exact rationals on a tiny 8-bit case; two groups, so the group index matters."""
    m, n, k, g, bits = 2, 8, 16, 8, 8
    A, qw, s, qz = random_case_bits(m, n, k, g, bits, seed=23)
    q = np_unpack_rows_bits(qw, bits)
    z = np_unpack_cols_bits(qz, bits)
    Cref, _ = o.gemm_bits(A, qw, s, qz, g, bits)
    for i in range(m):
        for j in range(n):
            ex = sum(Fraction(float(A[i, kk])) * (int(q[kk, j]) - int(z[kk // g, j])) * Fraction(float(s[kk // g, j]))
                     for kk in range(k))
            assert abs(Fraction(float(Cref[i, j])) - ex) <= abs(ex) * Fraction(1, 2 ** 48) + Fraction(1, 2 ** 60)


def pin_bits_closed_forms_and_one_hot(o):
    m, n, k, g = 3, 64, 256, 128
    rng = np.random.Generator(np.random.Philox(29))
    A = rng.standard_normal((m, k), dtype=np.float32).astype(np.float16)
    s_col = rng.uniform(0.001, 0.01, size=n).astype(np.float16)
    scales = np.tile(s_col, (k // g, 1))
    rowsum = A.astype(np.float64).sum(axis=1)
    for bits, q0, z0 in ((8, 200, 77), (8, 3, 255), (2, 3, 1)):
        f = 32 // bits
        rep = sum(1 << (bits * i) for i in range(f))
        qw = np.full((k // f, n), (q0 * rep) & 0xFFFFFFFF, dtype=np.uint32).view(np.int32)
        qz = np.full((k // g, n // f), (z0 * rep) & 0xFFFFFFFF, dtype=np.uint32).view(np.int32)
        Cref, _ = o.gemm_bits(A, qw, scales, qz, g, bits)
        expect = (q0 - z0) * s_col.astype(np.float64)[None, :] * rowsum[:, None]
        bound = 1e-12 * np.abs(A.astype(np.float64)).sum(axis=1)[:, None] * 255 * 0.01 + 1e-300
        assert np.all(np.abs(Cref - expect) <= bound)
    # one-hot rows pick rows of W exactly (8 bits)
    _, qw, s, qz = random_case_bits(8, 72, 256, 128, 8, seed=31)
    W = np_dense_weight_bits(qw, s, qz, 128, 8)
    rows = [0, 3, 4, 127, 128, 131, 200, 255]
    A1 = np.zeros((8, 256), np.float16)
    for i, r in enumerate(rows):
        A1[i, r] = 1.0
    Cref, C16 = o.gemm_bits(A1, qw, s, qz, 128, 8)
    assert np.array_equal(Cref, W[rows, :])
    assert np.array_equal(C16.view(np.uint16), W[rows, :].astype(np.float16).view(np.uint16))


# --------------------------------------------------------------------------- 3-bit fields
def np_unpack_stream3(words3: np.ndarray) -> np.ndarray:
    """numpy restatement: [..., 3] words of a 96-bit stream -> [..., 32] values, through a
    little-endian byte view and unpackbits (bit b of the stream is bit b % 8 of byte b // 8)."""
    w = np.ascontiguousarray(words3).astype("<u4")
    by = w.view(np.uint8).reshape(*w.shape[:-1], 12)
    bit = np.unpackbits(by, axis=-1, bitorder="little").reshape(*w.shape[:-1], 32, 3)
    return (bit[..., 0] + 2 * bit[..., 1] + 4 * bit[..., 2]).astype(np.uint8)


def np_unpack_rows_3bit(qweight: np.ndarray) -> np.ndarray:
    r, n = qweight.shape
    w3 = qweight.view(np.uint32).reshape(r // 3, 3, n).transpose(0, 2, 1)        # [k/32, n, 3]
    return np.ascontiguousarray(np_unpack_stream3(w3).transpose(0, 2, 1)).reshape(r // 3 * 32, n)


def np_unpack_cols_3bit(qzeros: np.ndarray) -> np.ndarray:
    g, c = qzeros.shape
    return np_unpack_stream3(qzeros.view(np.uint32).reshape(g, c // 3, 3)).reshape(g, c // 3 * 32)


def random_case_3bit(m, n, k, g, seed):
    rng = np.random.Generator(np.random.Philox(seed))
    A = rng.standard_normal((m, k), dtype=np.float32).astype(np.float16)
    qw = rng.integers(0, 1 << 32, size=(k // 32 * 3, n), dtype=np.uint32).view(np.int32)
    s = rng.uniform(0.001, 0.01, size=(k // g, n)).astype(np.float16)
    qz = rng.integers(0, 1 << 32, size=(k // g, n // 32 * 3), dtype=np.uint32).view(np.int32)
    return A, qw, s, qz


def np_dense_weight_3bit(qweight, scales, qzeros, group_size) -> np.ndarray:
    q = np_unpack_rows_3bit(qweight).astype(np.int64)
    z = np.repeat(np_unpack_cols_3bit(qzeros).astype(np.int64), group_size, axis=0)
    s = np.repeat(scales.astype(np.float64), group_size, axis=0)
    return (q - z) * s


def pin_3bit_known_words(o):
    """Hand-written streams.  Octal digits are 3-bit values: the 96-bit number whose octal
    digits, from the least significant, are the 32 values, cut into three 32-bit words."""
    vals = [(5 * u + 3) % 8 for u in range(32)]
    big = sum(v << (3 * u) for u, v in enumerate(vals))
    words = np.array([(big >> (32 * t)) & 0xFFFFFFFF for t in range(3)], dtype=np.uint32).view(np.int32)
    col = np.zeros((3, 32), np.int32)
    col[:, 7] = words
    q = o.unpack_qweight_3bit(col)
    assert q[:, 7].tolist() == vals and not q[:, :7].any() and not q[:, 8:].any()
    z = o.unpack_qzeros_3bit(words.reshape(1, 3))
    assert z[0].tolist() == vals
    # the two values that lie across words, alone: value 10 = bits 30, 31 of word 0 and bit 0 of
    # word 1; value 21 = bit 31 of word 1 and bits 0, 1 of word 2
    one = np.zeros((32, 32), np.uint8)
    one[10, 0] = 7
    one[21, 1] = 5
    one[31, 2] = 6
    w = o.pack_qweight_3bit(one).view(np.uint32)
    assert w[:, 0].tolist() == [0xC0000000, 0x00000001, 0]
    assert w[:, 1].tolist() == [0, 0x80000000, 0x00000002]
    assert w[:, 2].tolist() == [0, 0, 0xC0000000]
    zrow = np.zeros((1, 64), np.uint8)
    zrow[0, 32 + 10] = 3
    zrow[0, 32 + 21] = 6
    wz = o.pack_qzeros_3bit(zrow).view(np.uint32)
    assert wz[0].tolist() == [0, 0, 0, 0xC0000000, 0x00000000, 0x00000003]


def pin_3bit_unpack_library_and_bijection(o):
    rng = np.random.Generator(np.random.Philox(41))
    words = rng.integers(0, 1 << 32, size=(9, 64), dtype=np.uint32).view(np.int32)
    q = o.unpack_qweight_3bit(words)
    assert q.shape == (96, 64) and int(q.max()) == 7
    assert np.array_equal(q, np_unpack_rows_3bit(words))
    assert np.array_equal(o.pack_qweight_3bit(q), words)
    zw = rng.integers(0, 1 << 32, size=(5, 6), dtype=np.uint32).view(np.int32)
    z = o.unpack_qzeros_3bit(zw)
    assert z.shape == (5, 64)
    assert np.array_equal(z, np_unpack_cols_3bit(zw))
    assert np.array_equal(o.pack_qzeros_3bit(z), zw)
    fields = rng.integers(0, 8, size=(64, 32), dtype=np.uint8)
    assert np.array_equal(o.unpack_qweight_3bit(o.pack_qweight_3bit(fields)), fields)
    assert np.array_equal(o.unpack_qzeros_3bit(o.pack_qzeros_3bit(fields)), fields)


def pin_3bit_is_the_4bit_product_on_the_same_fields(o):
    """Fields 0..7 packed at 3 bits and at 4 bits give the same product, bit for bit (same sum order)."""
    m, n, k, g = 4, 64, 256, 64
    rng = np.random.Generator(np.random.Philox(43))
    A = rng.standard_normal((m, k), dtype=np.float32).astype(np.float16)
    q = rng.integers(0, 8, size=(k, n), dtype=np.uint8)
    z = rng.integers(0, 8, size=(k // g, n), dtype=np.uint8)
    s = rng.uniform(0.001, 0.01, size=(k // g, n)).astype(np.float16)
    C3, C316 = o.gemm_3bit(A, o.pack_qweight_3bit(q), s, o.pack_qzeros_3bit(z), g)
    C4, C416 = o.gemm(A, o.pack_qweight(q), s, o.pack_qzeros(z), g)
    assert np.array_equal(C3, C4)
    assert np.array_equal(C316.view(np.uint16), C416.view(np.uint16))


def pin_3bit_matmul_library(o):
    for (m, n, k, g, seed) in ((5, 96, 512, 128, 1), (16, 64, 256, 64, 2), (1, 160, 384, 128, 4), (3, 32, 96, 32, 5)):
        A, qw, s, qz = random_case_3bit(m, n, k, g, seed)
        W = np_dense_weight_3bit(qw, s, qz, g)
        ref = A.astype(np.float64) @ W
        absdot = np.abs(A.astype(np.float64)) @ np.abs(W)
        C64, C16 = o.gemm_3bit(A, qw, s, qz, g)
        assert np.all(np.abs(C64 - ref) <= 2 * k * 2.0 ** -53 * absdot + 1e-300)
        assert np.array_equal(C16.view(np.uint16), C64.astype(np.float16).view(np.uint16))


def pin_3bit_tiny_vs_fractions_and_one_hot(o):
    """Exact rationals on a tiny case with two groups; one-hot rows pick rows of W exactly,
    among them k = 10, 21 (across words) and the rows next to a stream boundary."""
    m, n, k, g = 2, 32, 64, 32
    A, qw, s, qz = random_case_3bit(m, n, k, g, seed=47)
    q = np_unpack_rows_3bit(qw)
    z = np_unpack_cols_3bit(qz)
    Cref, _ = o.gemm_3bit(A, qw, s, qz, g)
    for i in range(m):
        for j in range(0, n, 3):
            ex = sum(Fraction(float(A[i, kk])) * (int(q[kk, j]) - int(z[kk // g, j])) * Fraction(float(s[kk // g, j]))
                     for kk in range(k))
            assert abs(Fraction(float(Cref[i, j])) - ex) <= abs(ex) * Fraction(1, 2 ** 48) + Fraction(1, 2 ** 60)
    _, qw, s, qz = random_case_3bit(8, 96, 256, 128, seed=53)
    W = np_dense_weight_3bit(qw, s, qz, 128)
    rows = [0, 10, 21, 31, 32, 127, 128, 255]
    A1 = np.zeros((8, 256), np.float16)
    for i, r in enumerate(rows):
        A1[i, r] = 1.0
    Cref, C16 = o.gemm_3bit(A1, qw, s, qz, 128)
    assert np.array_equal(Cref, W[rows, :])
    assert np.array_equal(C16.view(np.uint16), W[rows, :].astype(np.float16).view(np.uint16))


# --------------------------------------------------------------------------- group index per row
def random_act_order(k, g, seed):
    """A group map as GPTQ's activation ordering makes it: a random order of the rows, cut into
    runs of g; row perm[i] belongs to group i // g."""
    rng = np.random.Generator(np.random.Philox(seed))
    perm = rng.permutation(k).astype(np.int32)
    g_idx = np.empty(k, np.int32)
    g_idx[perm] = np.arange(k, dtype=np.int32) // g
    return g_idx


def pin_gidx_contiguous_is_plain(o):
    A, qw, s, qz = random_case(5, 72, 512, 128, seed=41)
    g_idx = (np.arange(512) // 128).astype(np.int32)
    Cg, Cg16 = o.gemm_gidx(A, qw, s, qz, g_idx)
    C4, C416 = o.gemm(A, qw, s, qz, 128)
    assert np.array_equal(Cg.view(np.uint64), C4.view(np.uint64))
    assert np.array_equal(Cg16.view(np.uint16), C416.view(np.uint16))


def pin_gidx_matmul_library(o):
    """numpy float64 matmul over a dense weight gathered with g_idx by numpy indexing."""
    for (m, n, k, g, seed) in ((5, 96, 512, 128, 1), (16, 64, 256, 32, 2), (1, 200, 384, 64, 3)):
        A, qw, s, qz = random_case(m, n, k, g, seed)
        g_idx = random_act_order(k, g, seed + 100)
        q = np_unpack_qweight(qw).astype(np.int64)
        z = np_unpack_qzeros(qz).astype(np.int64)[g_idx]            # [k, n]
        sc = s.astype(np.float64)[g_idx]
        W = (q - z) * sc
        ref = A.astype(np.float64) @ W
        absdot = np.abs(A.astype(np.float64)) @ np.abs(W)
        C64, C16 = o.gemm_gidx(A, qw, s, qz, g_idx)
        assert np.all(np.abs(C64 - ref) <= 2 * k * 2.0 ** -53 * absdot + 1e-300)
        assert np.array_equal(C16.view(np.uint16), C64.astype(np.float16).view(np.uint16))
        # the group map matters: the contiguous one gives another result
        Cplain, _ = o.gemm(A, qw, s, qz, g)
        assert np.abs(Cplain - C64).max() > 1e-3 * np.abs(C64).max()


def pin_gidx_row_permutation_invariance(o):
    """Reordering the rows of W, with their group indices, and the columns of A alike leaves every
    term of every sum unchanged; only the order of an fp64 summation moves."""
    m, n, k, g = 4, 64, 256, 64
    A, qw, s, qz = random_case(m, n, k, g, seed=43)
    g_idx = random_act_order(k, g, seed=44)
    C0, _ = o.gemm_gidx(A, qw, s, qz, g_idx)
    P = np.random.Generator(np.random.Philox(45)).permutation(k)
    qw_p = o.pack_qweight(o.unpack_qweight(qw)[P])
    Cp, _ = o.gemm_gidx(A[:, P], qw_p, s, qz, g_idx[P])
    assert np.all(np.abs(Cp - C0) <= 1e-12 * (np.abs(C0) + 1))
    # sorting the rows by group makes the groups contiguous: the plain product applies
    order = np.argsort(g_idx, kind="stable")
    Cs, _ = o.gemm(A[:, order], o.pack_qweight(o.unpack_qweight(qw)[order]), s, qz, g)
    assert np.all(np.abs(Cs - C0) <= 1e-12 * (np.abs(C0) + 1))


def pin_gidx_tiny_vs_fractions(o):
    m, n, k, g = 2, 8, 16, 8
    A, qw, s, qz = random_case(m, n, k, g, seed=47)
    g_idx = np.array([1, 0, 0, 1, 1, 1, 0, 0, 0, 1, 0, 1, 1, 0, 1, 0], np.int32)
    q = np_unpack_qweight(qw)
    z = np_unpack_qzeros(qz)
    Cref, _ = o.gemm_gidx(A, qw, s, qz, g_idx)
    for i in range(m):
        for j in range(n):
            ex = sum(Fraction(float(A[i, kk])) * (int(q[kk, j]) - int(z[g_idx[kk], j])) * Fraction(float(s[g_idx[kk], j]))
                     for kk in range(k))
            assert abs(Fraction(float(Cref[i, j])) - ex) <= abs(ex) * Fraction(1, 2 ** 48) + Fraction(1, 2 ** 60)


ALL_PINS = [
    pin_half_to_float_exhaustive,
    pin_double_to_half_rounding,
    pin_unpack_known_words,
    pin_pack_unpack_bijection,
    pin_tiny_exact_rationals,
    pin_random_tiny_vs_fractions,
    pin_closed_forms,
    pin_matmul_library,
    pin_one_hot_rows,
    pin_group_boundary,
    pin_linearity_and_permutation,
    pin_splitk_invariance,
    pin_partition_order_by_cancellation,
    pin_blocked_arrangement_is_the_definition,
    pin_distribution,
    pin_bits_known_words,
    pin_bits_unpack_library_and_bijection,
    pin_bits4_is_the_4bit_path,
    pin_bits_matmul_library,
    pin_bits_tiny_vs_fractions,
    pin_bits_closed_forms_and_one_hot,
    pin_3bit_known_words,
    pin_3bit_unpack_library_and_bijection,
    pin_3bit_is_the_4bit_product_on_the_same_fields,
    pin_3bit_matmul_library,
    pin_3bit_tiny_vs_fractions_and_one_hot,
    pin_gidx_contiguous_is_plain,
    pin_gidx_matmul_library,
    pin_gidx_row_permutation_invariance,
    pin_gidx_tiny_vs_fractions,
]

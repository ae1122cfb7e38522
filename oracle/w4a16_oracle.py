"""ctypes binding of the C oracle (oracle/w4a16_oracle.c).  Test infrastructure only.

Every function takes and returns numpy host arrays.  The shared library is built by
oracle/build.py (also run by __graft_entry__.build()); if it is missing or older than
its source it is compiled on first use, which needs only gcc.

`Oracle(path)` binds any build of the C file (the mutation tests bind deliberately
broken copies); the module-level functions use the committed source.
"""
from __future__ import annotations

import ctypes
import pathlib

import numpy as np

_HERE = pathlib.Path(__file__).resolve().parent
_LIB_PATH = _HERE / "libw4a16_oracle.so"

_i32p = ctypes.POINTER(ctypes.c_int32)
_u16p = ctypes.POINTER(ctypes.c_uint16)
_u8p = ctypes.POINTER(ctypes.c_uint8)
_f32p = ctypes.POINTER(ctypes.c_float)
_f64p = ctypes.POINTER(ctypes.c_double)


class OracleError(ValueError):
    pass


def _c(a: np.ndarray, dtype) -> np.ndarray:
    a = np.ascontiguousarray(a)
    if a.dtype != dtype:
        raise TypeError(f"expected {dtype}, got {a.dtype}")
    return a


def _ptr(a: np.ndarray, ctype):
    return a.ctypes.data_as(ctypes.POINTER(ctype))


class Oracle:
    def __init__(self, lib_path):
        lib = ctypes.CDLL(str(lib_path))
        lib.w4a16_oracle_half_to_float.argtypes = [ctypes.c_uint16]
        lib.w4a16_oracle_half_to_float.restype = ctypes.c_float
        lib.w4a16_oracle_float_to_half.argtypes = [ctypes.c_float]
        lib.w4a16_oracle_float_to_half.restype = ctypes.c_uint16
        lib.w4a16_oracle_double_to_half.argtypes = [ctypes.c_double]
        lib.w4a16_oracle_double_to_half.restype = ctypes.c_uint16
        lib.w4a16_oracle_unpack_qweight.argtypes = [_i32p, _u8p, ctypes.c_int, ctypes.c_int]
        lib.w4a16_oracle_unpack_qweight.restype = None
        lib.w4a16_oracle_unpack_qzeros.argtypes = [_i32p, _u8p, ctypes.c_int, ctypes.c_int]
        lib.w4a16_oracle_unpack_qzeros.restype = None
        lib.w4a16_oracle_pack_qweight.argtypes = [_u8p, _i32p, ctypes.c_int, ctypes.c_int]
        lib.w4a16_oracle_pack_qweight.restype = None
        lib.w4a16_oracle_pack_qzeros.argtypes = [_u8p, _i32p, ctypes.c_int, ctypes.c_int]
        lib.w4a16_oracle_pack_qzeros.restype = None
        lib.w4a16_oracle_dequant.argtypes = [_i32p, _u16p, _i32p, _f32p, ctypes.c_int, ctypes.c_int, ctypes.c_int]
        lib.w4a16_oracle_dequant.restype = None
        lib.w4a16_oracle_gemm.argtypes = [_u16p, _i32p, _u16p, _i32p, _f64p, _u16p] + [ctypes.c_int] * 8
        lib.w4a16_oracle_gemm.restype = ctypes.c_int
        lib.w4a16_oracle_gemm_blocked.argtypes = lib.w4a16_oracle_gemm.argtypes
        lib.w4a16_oracle_gemm_blocked.restype = ctypes.c_int
        for name in ("unpack_qweight_bits", "unpack_qzeros_bits"):
            fn = getattr(lib, "w4a16_oracle_" + name)
            fn.argtypes = [_i32p, _u8p, ctypes.c_int, ctypes.c_int, ctypes.c_int]
            fn.restype = ctypes.c_int
        for name in ("pack_qweight_bits", "pack_qzeros_bits"):
            fn = getattr(lib, "w4a16_oracle_" + name)
            fn.argtypes = [_u8p, _i32p, ctypes.c_int, ctypes.c_int, ctypes.c_int]
            fn.restype = ctypes.c_int
        lib.w4a16_oracle_gemm_bits.argtypes = [_u16p, _i32p, _u16p, _i32p, _f64p, _u16p] + [ctypes.c_int] * 6
        lib.w4a16_oracle_gemm_bits.restype = ctypes.c_int
        for name in ("unpack_qweight_3bit", "unpack_qzeros_3bit"):
            fn = getattr(lib, "w4a16_oracle_" + name)
            fn.argtypes = [_i32p, _u8p, ctypes.c_int, ctypes.c_int]
            fn.restype = None
        for name in ("pack_qweight_3bit", "pack_qzeros_3bit"):
            fn = getattr(lib, "w4a16_oracle_" + name)
            fn.argtypes = [_u8p, _i32p, ctypes.c_int, ctypes.c_int]
            fn.restype = None
        lib.w4a16_oracle_gemm_3bit.argtypes = [_u16p, _i32p, _u16p, _i32p, _f64p, _u16p] + [ctypes.c_int] * 5
        lib.w4a16_oracle_gemm_3bit.restype = ctypes.c_int
        lib.w4a16_oracle_gemm_gidx.argtypes = [_u16p, _i32p, _u16p, _i32p, _i32p, _f64p, _u16p] + [ctypes.c_int] * 5
        lib.w4a16_oracle_gemm_gidx.restype = ctypes.c_int
        self.lib = lib

    # ---- fp16 conversions (round to nearest even; the paper does not name a mode)
    def half_to_float(self, bits: int) -> float:
        return float(self.lib.w4a16_oracle_half_to_float(int(bits)))

    def float_to_half(self, x) -> int:
        return int(self.lib.w4a16_oracle_float_to_half(float(np.float32(x))))

    def double_to_half(self, x) -> int:
        return int(self.lib.w4a16_oracle_double_to_half(float(x)))

    # ---- pack / unpack (paper Section 2: packed int32 weights, bitwise unpacking)
    def unpack_qweight(self, qweight: np.ndarray) -> np.ndarray:
        """int32 [k/8, n] -> uint8 [k, n]."""
        qweight = _c(qweight, np.int32)
        r, n = qweight.shape
        q = np.empty((r * 8, n), np.uint8)
        self.lib.w4a16_oracle_unpack_qweight(_ptr(qweight, ctypes.c_int32), _ptr(q, ctypes.c_uint8), n, r * 8)
        return q

    def unpack_qzeros(self, qzeros: np.ndarray) -> np.ndarray:
        """int32 [groups, n/8] -> uint8 [groups, n]."""
        qzeros = _c(qzeros, np.int32)
        g, c = qzeros.shape
        z = np.empty((g, c * 8), np.uint8)
        self.lib.w4a16_oracle_unpack_qzeros(_ptr(qzeros, ctypes.c_int32), _ptr(z, ctypes.c_uint8), c * 8, g)
        return z

    def pack_qweight(self, q: np.ndarray) -> np.ndarray:
        q = _c(q, np.uint8)
        k, n = q.shape
        assert k % 8 == 0
        out = np.empty((k // 8, n), np.int32)
        self.lib.w4a16_oracle_pack_qweight(_ptr(q, ctypes.c_uint8), _ptr(out, ctypes.c_int32), n, k)
        return out

    def pack_qzeros(self, z: np.ndarray) -> np.ndarray:
        z = _c(z, np.uint8)
        g, n = z.shape
        assert n % 8 == 0
        out = np.empty((g, n // 8), np.int32)
        self.lib.w4a16_oracle_pack_qzeros(_ptr(z, ctypes.c_uint8), _ptr(out, ctypes.c_int32), n, g)
        return out

    # ---- dequantisation (paper Section 2: scale and shift)
    def dequant(self, qweight, scales, qzeros, group_size: int) -> np.ndarray:
        """fp32 W [k, n] with W = (q - z) * s, exact."""
        qweight = _c(qweight, np.int32)
        scales = _c(scales, np.float16)
        qzeros = _c(qzeros, np.int32)
        r, n = qweight.shape
        k = r * 8
        if scales.shape != (k // group_size, n) or qzeros.shape != (k // group_size, n // 8):
            raise OracleError("scales / qzeros shapes do not match k, n, group_size")
        W = np.empty((k, n), np.float32)
        self.lib.w4a16_oracle_dequant(_ptr(qweight, ctypes.c_int32), _ptr(scales.view(np.uint16), ctypes.c_uint16),
                                      _ptr(qzeros, ctypes.c_int32), _ptr(W, ctypes.c_float), n, k, group_size)
        return W

    # ---- the product (paper Algorithm 1; Section 3 first paragraph for the DP variant)
    def gemm(self, A, qweight, scales, qzeros, group_size: int, split_k: int = 1, block_k: int = 0,
             acc: str = "f64", threads: int = 0, return_threads: bool = False, blocked: bool = False):
        """Cref (float64 [m, n]) and its fp16 rounding C16 (float16 [m, n]): the definition, one
        output element at a time.  blocked=True calls the arrangement kept for the timed CPU
        baseline instead (same operations per element, bit-identical results; no parity test
        uses it).

        acc = "f64": fp64 accumulators (the definition); "f32": Algorithm 1's fp32 accumulator.
        split_k partial sums: contiguous chunks of k (block_k = 0) or Algorithm 1's strided
        walk over k-blocks of block_k.
        """
        A = _c(A, np.float16)
        qweight = _c(qweight, np.int32)
        scales = _c(scales, np.float16)
        qzeros = _c(qzeros, np.int32)
        m, k = A.shape
        r, n = qweight.shape
        if r * 8 != k:
            raise OracleError("qweight rows must be k / 8")
        if group_size <= 0 or k % group_size or scales.shape != (k // group_size, n) \
                or qzeros.shape != (k // group_size, n // 8):
            raise OracleError("scales / qzeros shapes do not match k, n, group_size")
        Cref = np.empty((m, n), np.float64)
        C16 = np.empty((m, n), np.float16)
        fn = self.lib.w4a16_oracle_gemm_blocked if blocked else self.lib.w4a16_oracle_gemm
        rc = fn(
            _ptr(A.view(np.uint16), ctypes.c_uint16), _ptr(qweight, ctypes.c_int32),
            _ptr(scales.view(np.uint16), ctypes.c_uint16), _ptr(qzeros, ctypes.c_int32),
            _ptr(Cref, ctypes.c_double), _ptr(C16.view(np.uint16), ctypes.c_uint16),
            m, n, k, group_size, split_k, block_k, {"f64": 0, "f32": 1}[acc], threads)
        if rc < 0:
            raise OracleError(f"w4a16_oracle_gemm rejected its arguments (code {rc})")
        if return_threads:
            return Cref, C16, rc
        return Cref, C16


    # ---- other field widths (paper Section 2: the method carries over to other n-bit schemes)
    def unpack_qweight_bits(self, qweight: np.ndarray, bits: int) -> np.ndarray:
        """int32 [k/f, n] -> uint8 [k, n], f = 32 / bits fields per word along k."""
        qweight = _c(qweight, np.int32)
        r, n = qweight.shape
        f = 32 // bits
        q = np.empty((r * f, n), np.uint8)
        if self.lib.w4a16_oracle_unpack_qweight_bits(_ptr(qweight, ctypes.c_int32), _ptr(q, ctypes.c_uint8), n, r * f, bits):
            raise OracleError("bits must be 2, 4 or 8")
        return q

    def unpack_qzeros_bits(self, qzeros: np.ndarray, bits: int) -> np.ndarray:
        """int32 [groups, n/f] -> uint8 [groups, n]."""
        qzeros = _c(qzeros, np.int32)
        g, c = qzeros.shape
        f = 32 // bits
        z = np.empty((g, c * f), np.uint8)
        if self.lib.w4a16_oracle_unpack_qzeros_bits(_ptr(qzeros, ctypes.c_int32), _ptr(z, ctypes.c_uint8), c * f, g, bits):
            raise OracleError("bits must be 2, 4 or 8")
        return z

    def pack_qweight_bits(self, q: np.ndarray, bits: int) -> np.ndarray:
        q = _c(q, np.uint8)
        k, n = q.shape
        f = 32 // bits
        assert k % f == 0
        out = np.empty((k // f, n), np.int32)
        if self.lib.w4a16_oracle_pack_qweight_bits(_ptr(q, ctypes.c_uint8), _ptr(out, ctypes.c_int32), n, k, bits):
            raise OracleError("bits must be 2, 4 or 8")
        return out

    def pack_qzeros_bits(self, z: np.ndarray, bits: int) -> np.ndarray:
        z = _c(z, np.uint8)
        g, n = z.shape
        f = 32 // bits
        assert n % f == 0
        out = np.empty((g, n // f), np.int32)
        if self.lib.w4a16_oracle_pack_qzeros_bits(_ptr(z, ctypes.c_uint8), _ptr(out, ctypes.c_int32), n, g, bits):
            raise OracleError("bits must be 2, 4 or 8")
        return out

    def gemm_bits(self, A, qweight, scales, qzeros, group_size: int, bits: int, threads: int = 0):
        """Cref (float64 [m, n]) and its fp16 rounding for fields of `bits` bits: the definition,
        fp64 accumulation in ascending k."""
        A = _c(A, np.float16)
        qweight = _c(qweight, np.int32)
        scales = _c(scales, np.float16)
        qzeros = _c(qzeros, np.int32)
        f = 32 // bits
        m, k = A.shape
        r, n = qweight.shape
        if r * f != k:
            raise OracleError("qweight rows must be k / (32 / bits)")
        if group_size <= 0 or k % group_size or scales.shape != (k // group_size, n) \
                or qzeros.shape != (k // group_size, n // f):
            raise OracleError("scales / qzeros shapes do not match k, n, group_size, bits")
        Cref = np.empty((m, n), np.float64)
        C16 = np.empty((m, n), np.float16)
        rc = self.lib.w4a16_oracle_gemm_bits(
            _ptr(A.view(np.uint16), ctypes.c_uint16), _ptr(qweight, ctypes.c_int32),
            _ptr(scales.view(np.uint16), ctypes.c_uint16), _ptr(qzeros, ctypes.c_int32),
            _ptr(Cref, ctypes.c_double), _ptr(C16.view(np.uint16), ctypes.c_uint16),
            m, n, k, group_size, bits, threads)
        if rc < 0:
            raise OracleError(f"w4a16_oracle_gemm_bits rejected its arguments (code {rc})")
        return Cref, C16


    # ---- 3-bit fields: 32 values in a 96-bit stream of three consecutive words
    def unpack_qweight_3bit(self, qweight: np.ndarray) -> np.ndarray:
        """int32 [3 k / 32, n] -> uint8 [k, n]."""
        qweight = _c(qweight, np.int32)
        r, n = qweight.shape
        if r % 3:
            raise OracleError("3-bit qweight has a multiple of three word rows")
        k = r // 3 * 32
        q = np.empty((k, n), np.uint8)
        self.lib.w4a16_oracle_unpack_qweight_3bit(_ptr(qweight, ctypes.c_int32), _ptr(q, ctypes.c_uint8), n, k)
        return q

    def unpack_qzeros_3bit(self, qzeros: np.ndarray) -> np.ndarray:
        """int32 [groups, 3 n / 32] -> uint8 [groups, n]."""
        qzeros = _c(qzeros, np.int32)
        g, c = qzeros.shape
        if c % 3:
            raise OracleError("a 3-bit qzeros row has a multiple of three words")
        n = c // 3 * 32
        z = np.empty((g, n), np.uint8)
        self.lib.w4a16_oracle_unpack_qzeros_3bit(_ptr(qzeros, ctypes.c_int32), _ptr(z, ctypes.c_uint8), n, g)
        return z

    def pack_qweight_3bit(self, q: np.ndarray) -> np.ndarray:
        q = _c(q, np.uint8)
        k, n = q.shape
        assert k % 32 == 0
        out = np.empty((k // 32 * 3, n), np.int32)
        self.lib.w4a16_oracle_pack_qweight_3bit(_ptr(q, ctypes.c_uint8), _ptr(out, ctypes.c_int32), n, k)
        return out

    def pack_qzeros_3bit(self, z: np.ndarray) -> np.ndarray:
        z = _c(z, np.uint8)
        g, n = z.shape
        assert n % 32 == 0
        out = np.empty((g, n // 32 * 3), np.int32)
        self.lib.w4a16_oracle_pack_qzeros_3bit(_ptr(z, ctypes.c_uint8), _ptr(out, ctypes.c_int32), n, g)
        return out

    def gemm_3bit(self, A, qweight, scales, qzeros, group_size: int, threads: int = 0):
        """Cref (float64 [m, n]) and its fp16 rounding for 3-bit fields: the definition, fp64
        accumulation in ascending k."""
        A = _c(A, np.float16)
        qweight = _c(qweight, np.int32)
        scales = _c(scales, np.float16)
        qzeros = _c(qzeros, np.int32)
        m, k = A.shape
        r, n = qweight.shape
        if k % 32 or r != k // 32 * 3:
            raise OracleError("qweight rows must be 3 k / 32")
        if group_size <= 0 or k % group_size or n % 32 or scales.shape != (k // group_size, n) \
                or qzeros.shape != (k // group_size, n // 32 * 3):
            raise OracleError("scales / qzeros shapes do not match k, n, group_size")
        Cref = np.empty((m, n), np.float64)
        C16 = np.empty((m, n), np.float16)
        rc = self.lib.w4a16_oracle_gemm_3bit(
            _ptr(A.view(np.uint16), ctypes.c_uint16), _ptr(qweight, ctypes.c_int32),
            _ptr(scales.view(np.uint16), ctypes.c_uint16), _ptr(qzeros, ctypes.c_int32),
            _ptr(Cref, ctypes.c_double), _ptr(C16.view(np.uint16), ctypes.c_uint16),
            m, n, k, group_size, threads)
        if rc < 0:
            raise OracleError(f"w4a16_oracle_gemm_3bit rejected its arguments (code {rc})")
        return Cref, C16

    # ---- group index per row (GPTQ's activation ordering; outside the paper)
    def gemm_gidx(self, A, qweight, scales, qzeros, g_idx, threads: int = 0):
        """Cref (float64 [m, n]) and its fp16 rounding with W[kk] = (q[kk] - z[g_idx[kk]]) * s[g_idx[kk]]."""
        A = _c(A, np.float16)
        qweight = _c(qweight, np.int32)
        scales = _c(scales, np.float16)
        qzeros = _c(qzeros, np.int32)
        g_idx = _c(g_idx, np.int32)
        m, k = A.shape
        r, n = qweight.shape
        groups = scales.shape[0]
        if r * 8 != k or g_idx.shape != (k,) or scales.shape != (groups, n) or qzeros.shape != (groups, n // 8):
            raise OracleError("shapes do not match")
        Cref = np.empty((m, n), np.float64)
        C16 = np.empty((m, n), np.float16)
        rc = self.lib.w4a16_oracle_gemm_gidx(
            _ptr(A.view(np.uint16), ctypes.c_uint16), _ptr(qweight, ctypes.c_int32),
            _ptr(scales.view(np.uint16), ctypes.c_uint16), _ptr(qzeros, ctypes.c_int32),
            _ptr(g_idx, ctypes.c_int32), _ptr(Cref, ctypes.c_double), _ptr(C16.view(np.uint16), ctypes.c_uint16),
            m, n, k, groups, threads)
        if rc < 0:
            raise OracleError(f"w4a16_oracle_gemm_gidx rejected its arguments (code {rc})")
        return Cref, C16


_default = None


def default() -> Oracle:
    """The oracle built from the committed source, compiled on demand."""
    global _default
    if _default is None:
        src = _HERE / "w4a16_oracle.c"
        if not _LIB_PATH.exists() or _LIB_PATH.stat().st_mtime < src.stat().st_mtime:
            from . import build as _build
            _build.build()
        _default = Oracle(_LIB_PATH)
    return _default


def half_to_float(bits):
    return default().half_to_float(bits)


def float_to_half(x):
    return default().float_to_half(x)


def double_to_half(x):
    return default().double_to_half(x)


def unpack_qweight(qweight):
    return default().unpack_qweight(qweight)


def unpack_qzeros(qzeros):
    return default().unpack_qzeros(qzeros)


def pack_qweight(q):
    return default().pack_qweight(q)


def pack_qzeros(z):
    return default().pack_qzeros(z)


def dequant(qweight, scales, qzeros, group_size):
    return default().dequant(qweight, scales, qzeros, group_size)


def gemm_bits(A, qweight, scales, qzeros, group_size, bits, **kw):
    return default().gemm_bits(A, qweight, scales, qzeros, group_size, bits, **kw)


def gemm_3bit(A, qweight, scales, qzeros, group_size, **kw):
    return default().gemm_3bit(A, qweight, scales, qzeros, group_size, **kw)


def gemm(A, qweight, scales, qzeros, group_size, **kw):
    return default().gemm(A, qweight, scales, qzeros, group_size, **kw)


def gemm_blocked(A, qweight, scales, qzeros, group_size, **kw):
    return default().gemm(A, qweight, scales, qzeros, group_size, blocked=True, **kw)

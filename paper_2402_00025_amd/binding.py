"""Thin ctypes binding of libw4a16.so (see include/w4a16.h): argument marshalling only.

Every function has the name of the C entry point it calls.  Tensor arguments are torch
tensors on the GPU (PyTorch is used for device memory and streams only); their data
pointers are passed through unchanged.  A negative return code raises W4A16Error.

There is no fallback: if the library has not been built, loading raises.
"""
from __future__ import annotations

import ctypes
import pathlib

_HERE = pathlib.Path(__file__).resolve().parent
LIB_PATH = _HERE / "libw4a16.so"

OK = 0
ERR_NULL, ERR_SHAPE, ERR_SPLIT, ERR_UNSUPPORTED, ERR_HIP, ERR_STATE, ERR_LIMIT = -1, -2, -3, -4, -5, -6, -7
REDUCE_AUTO, REDUCE_ATOMIC_F32, REDUCE_ATOMIC_PK_F16, REDUCE_WORKSPACE, REDUCE_ATOMIC_FIXED = 0, 1, 2, 3, 4
REDUCE_ATOMIC_PK_F16_PHASE = 5

#: every symbol include/w4a16.h declares
EXPORTS = (
    "w4a16_gemm", "w4a16_gemm_dp", "w4a16_gemm_streamk", "w4a16_gemm_ex", "w4a16_gemm_dp_ex", "w4a16_plan", "w4a16_plan_bits",
    "w4a16_check",
    "w4a16_unpack", "w4a16_dequant", "w4a16_algorithmic_bytes", "w4a16_strerror", "w4a16_last_hip_error",
    "w4a16_release_scratch", "w4a16_phase_timeouts", "w8a16_gemm", "w8a16_gemm_dp", "w8a16_algorithmic_bytes",
    "w2a16_gemm", "w2a16_gemm_dp", "w2a16_algorithmic_bytes", "w3a16_gemm", "w3a16_gemm_dp", "w3a16_algorithmic_bytes", "w4a16_actorder_prepare", "w4a16_gemm_actorder",
    "w4a16_read_probe", "w4a16_gemm_static", "w4a16_set_phase_spin_limit", "w4a16_workspace_bytes",
    "w4a16_set_workspace", "w4a16_reserve_scratch", "w4a16_gemm_streamk_bits",
)

_lib = None


class W4A16Error(RuntimeError):
    def __init__(self, code: int, where: str):
        self.code = code
        detail = ""
        if code in (ERR_HIP, ERR_STATE):
            detail = " [" + lib().w4a16_last_hip_error().decode() + "]"
        super().__init__(f"{where} failed with code {code}: {strerror(code)}{detail}")


def lib() -> ctypes.CDLL:
    """The loaded library; raises if it was never built (run __graft_entry__.build())."""
    global _lib
    if _lib is not None:
        return _lib
    if not LIB_PATH.exists():
        raise FileNotFoundError(
            f"{LIB_PATH} is missing: build it with `python -m paper_2402_00025_amd.build` "
            "(there is no CPU fallback for the HIP path)")
    # PyTorch ships its own copy of the HIP runtime (same soname as ROCm's).  Stream handles are
    # only valid inside the runtime instance that made them, so torch's copy must be the one
    # this library binds to: load torch first, then the dynamic loader reuses its runtime.
    import torch  # noqa: F401

    L = ctypes.CDLL(str(LIB_PATH))
    vp, ci = ctypes.c_void_p, ctypes.c_int
    ip = ctypes.POINTER(ctypes.c_int)
    L.w4a16_gemm.argtypes = [vp] * 5 + [ci] * 5 + [vp]
    L.w4a16_gemm_dp.argtypes = [vp] * 5 + [ci] * 4 + [vp]
    L.w4a16_gemm_static.argtypes = [vp] * 5 + [ci] * 5 + [vp]
    L.w4a16_set_phase_spin_limit.argtypes = [ci]
    L.w4a16_workspace_bytes.argtypes = [ci]
    L.w4a16_workspace_bytes.restype = ctypes.c_longlong
    L.w4a16_set_workspace.argtypes = [vp, ctypes.c_longlong, ci, vp]
    L.w4a16_reserve_scratch.argtypes = [ci]
    L.w4a16_gemm_streamk.argtypes = [vp] * 5 + [ci] * 5 + [vp]
    L.w4a16_gemm_streamk_bits.argtypes = [ci] + [vp] * 5 + [ci] * 5 + [vp]
    L.w8a16_gemm.argtypes = [vp] * 5 + [ci] * 5 + [vp]
    L.w8a16_gemm_dp.argtypes = [vp] * 5 + [ci] * 4 + [vp]
    L.w8a16_algorithmic_bytes.argtypes = [ci] * 4
    L.w8a16_algorithmic_bytes.restype = ctypes.c_longlong
    L.w4a16_actorder_prepare.argtypes = [vp] * 5 + [ci] * 3 + [vp]
    L.w4a16_gemm_actorder.argtypes = [vp] * 7 + [ci] * 5 + [vp]
    L.w4a16_read_probe.argtypes = [vp, ctypes.c_longlong, ci, vp]
    L.w2a16_gemm.argtypes = [vp] * 5 + [ci] * 5 + [vp]
    L.w2a16_gemm_dp.argtypes = [vp] * 5 + [ci] * 4 + [vp]
    L.w2a16_algorithmic_bytes.argtypes = [ci] * 4
    L.w2a16_algorithmic_bytes.restype = ctypes.c_longlong
    L.w3a16_gemm.argtypes = [vp] * 5 + [ci] * 5 + [vp]
    L.w3a16_gemm_dp.argtypes = [vp] * 5 + [ci] * 4 + [vp]
    L.w3a16_algorithmic_bytes.argtypes = [ci] * 4
    L.w3a16_algorithmic_bytes.restype = ctypes.c_longlong
    L.w4a16_gemm_ex.argtypes = [vp] * 5 + [ci] * 8 + [vp]
    L.w4a16_gemm_dp_ex.argtypes = [vp] * 5 + [ci] * 6 + [vp]
    L.w4a16_plan.argtypes = [ci] * 5 + [ip] * 4
    L.w4a16_plan_bits.argtypes = [ci] * 6 + [ip] * 4
    L.w4a16_check.argtypes = [ci] * 5
    L.w4a16_unpack.argtypes = [vp] * 4 + [ci] * 3 + [vp]
    L.w4a16_dequant.argtypes = [vp] * 4 + [ci] * 3 + [vp]
    L.w4a16_algorithmic_bytes.argtypes = [ci] * 4
    L.w4a16_algorithmic_bytes.restype = ctypes.c_longlong
    L.w4a16_strerror.argtypes = [ci]
    L.w4a16_strerror.restype = ctypes.c_char_p
    L.w4a16_last_hip_error.argtypes = []
    L.w4a16_last_hip_error.restype = ctypes.c_char_p
    L.w4a16_release_scratch.argtypes = []
    L.w4a16_phase_timeouts.argtypes = []
    L.w4a16_phase_timeouts.restype = ctypes.c_longlong
    for name in EXPORTS:
        if name not in ("w4a16_algorithmic_bytes", "w8a16_algorithmic_bytes", "w2a16_algorithmic_bytes",
                        "w3a16_algorithmic_bytes", "w4a16_strerror", "w4a16_last_hip_error",
                        "w4a16_phase_timeouts", "w4a16_workspace_bytes"):
            getattr(L, name).restype = ci
    _lib = L
    return L


def _p(t):
    """Device pointer of a torch tensor (or a raw int / None)."""
    if t is None:
        return None
    if isinstance(t, int):
        return ctypes.c_void_p(t)
    return ctypes.c_void_p(t.data_ptr())


def _stream(stream):
    if stream is None:
        import torch
        return ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)
    if isinstance(stream, int):
        return ctypes.c_void_p(stream)
    return ctypes.c_void_p(stream.cuda_stream)


def _check(rc: int, where: str) -> None:
    if rc != OK:
        raise W4A16Error(rc, where)


def strerror(code: int) -> str:
    return lib().w4a16_strerror(int(code)).decode()


def w4a16_gemm(A, qweight, scales, qzeros, C, m, n, k, group_size, split_k, stream=None) -> None:
    _check(lib().w4a16_gemm(_p(A), _p(qweight), _p(scales), _p(qzeros), _p(C), m, n, k, group_size, split_k,
                            _stream(stream)), "w4a16_gemm")


def w4a16_gemm_static(A, qweight, scales, qzeros, C, m, n, k, group_size, split_k, stream=None) -> None:
    _check(lib().w4a16_gemm_static(_p(A), _p(qweight), _p(scales), _p(qzeros), _p(C), m, n, k, group_size, split_k,
                                   _stream(stream)), "w4a16_gemm_static")


def w4a16_gemm_dp(A, qweight, scales, qzeros, C, m, n, k, group_size, stream=None) -> None:
    _check(lib().w4a16_gemm_dp(_p(A), _p(qweight), _p(scales), _p(qzeros), _p(C), m, n, k, group_size,
                               _stream(stream)), "w4a16_gemm_dp")


def w8a16_gemm(A, qweight, scales, qzeros, C, m, n, k, group_size, split_k=0, stream=None) -> None:
    _check(lib().w8a16_gemm(_p(A), _p(qweight), _p(scales), _p(qzeros), _p(C), m, n, k, group_size, split_k,
                            _stream(stream)), "w8a16_gemm")


def w8a16_gemm_dp(A, qweight, scales, qzeros, C, m, n, k, group_size, stream=None) -> None:
    _check(lib().w8a16_gemm_dp(_p(A), _p(qweight), _p(scales), _p(qzeros), _p(C), m, n, k, group_size,
                               _stream(stream)), "w8a16_gemm_dp")


def w8a16_algorithmic_bytes(m, n, k, group_size) -> int:
    return int(lib().w8a16_algorithmic_bytes(m, n, k, group_size))


def w2a16_gemm(A, qweight, scales, qzeros, C, m, n, k, group_size, split_k=0, stream=None) -> None:
    _check(lib().w2a16_gemm(_p(A), _p(qweight), _p(scales), _p(qzeros), _p(C), m, n, k, group_size, split_k,
                            _stream(stream)), "w2a16_gemm")


def w2a16_gemm_dp(A, qweight, scales, qzeros, C, m, n, k, group_size, stream=None) -> None:
    _check(lib().w2a16_gemm_dp(_p(A), _p(qweight), _p(scales), _p(qzeros), _p(C), m, n, k, group_size,
                               _stream(stream)), "w2a16_gemm_dp")


def w2a16_algorithmic_bytes(m, n, k, group_size) -> int:
    return int(lib().w2a16_algorithmic_bytes(m, n, k, group_size))


def w3a16_gemm(A, qweight, scales, qzeros, C, m, n, k, group_size, split_k=0, stream=None) -> None:
    _check(lib().w3a16_gemm(_p(A), _p(qweight), _p(scales), _p(qzeros), _p(C), m, n, k, group_size, split_k,
                            _stream(stream)), "w3a16_gemm")


def w3a16_gemm_dp(A, qweight, scales, qzeros, C, m, n, k, group_size, stream=None) -> None:
    _check(lib().w3a16_gemm_dp(_p(A), _p(qweight), _p(scales), _p(qzeros), _p(C), m, n, k, group_size,
                               _stream(stream)), "w3a16_gemm_dp")


def w3a16_algorithmic_bytes(m, n, k, group_size) -> int:
    return int(lib().w3a16_algorithmic_bytes(m, n, k, group_size))


def w4a16_actorder_prepare(qweight, g_idx, qweight_sorted, perm, status, n, k, group_size, stream=None) -> None:
    _check(lib().w4a16_actorder_prepare(_p(qweight), _p(g_idx), _p(qweight_sorted), _p(perm), _p(status), n, k,
                                        group_size, _stream(stream)), "w4a16_actorder_prepare")


def w4a16_gemm_actorder(A, qweight_sorted, scales, qzeros, perm, A_work, C, m, n, k, group_size, split_k=0,
                        stream=None) -> None:
    _check(lib().w4a16_gemm_actorder(_p(A), _p(qweight_sorted), _p(scales), _p(qzeros), _p(perm), _p(A_work), _p(C),
                                     m, n, k, group_size, split_k, _stream(stream)), "w4a16_gemm_actorder")


def w4a16_read_probe(buffer, nbytes, shape=0, stream=None) -> None:
    _check(lib().w4a16_read_probe(_p(buffer), nbytes, shape, _stream(stream)), "w4a16_read_probe")


def w4a16_gemm_streamk(A, qweight, scales, qzeros, C, m, n, k, group_size, workgroups=0, stream=None) -> None:
    _check(lib().w4a16_gemm_streamk(_p(A), _p(qweight), _p(scales), _p(qzeros), _p(C), m, n, k, group_size,
                                    workgroups, _stream(stream)), "w4a16_gemm_streamk")


def w4a16_gemm_streamk_bits(bits, A, qweight, scales, qzeros, C, m, n, k, group_size, workgroups=0, stream=None) -> None:
    _check(lib().w4a16_gemm_streamk_bits(bits, _p(A), _p(qweight), _p(scales), _p(qzeros), _p(C), m, n, k, group_size,
                                         workgroups, _stream(stream)), "w4a16_gemm_streamk_bits")


def w4a16_gemm_ex(A, qweight, scales, qzeros, C, m, n, k, group_size, split_k, tile_cols=0, waves=0, reduce=0,
                  stream=None) -> None:
    _check(lib().w4a16_gemm_ex(_p(A), _p(qweight), _p(scales), _p(qzeros), _p(C), m, n, k, group_size, split_k,
                               tile_cols, waves, reduce, _stream(stream)), "w4a16_gemm_ex")


def w4a16_gemm_dp_ex(A, qweight, scales, qzeros, C, m, n, k, group_size, tile_cols=0, waves=0, stream=None) -> None:
    _check(lib().w4a16_gemm_dp_ex(_p(A), _p(qweight), _p(scales), _p(qzeros), _p(C), m, n, k, group_size,
                                  tile_cols, waves, _stream(stream)), "w4a16_gemm_dp_ex")


def w4a16_plan(m, n, k, group_size, dp=False, split_k=0, tile_cols=0, waves=0, reduce=0) -> dict:
    s, t, w, r = (ctypes.c_int(v) for v in (split_k, tile_cols, waves, reduce))
    _check(lib().w4a16_plan(m, n, k, group_size, int(bool(dp)), ctypes.byref(s), ctypes.byref(t), ctypes.byref(w),
                            ctypes.byref(r)), "w4a16_plan")
    return dict(split_k=s.value, tile_cols=t.value, waves=w.value, reduce=r.value)


def w4a16_plan_bits(bits, m, n, k, group_size, dp=False, split_k=0) -> dict:
    s, t, w, r = (ctypes.c_int(v) for v in (split_k, 0, 0, 0))
    _check(lib().w4a16_plan_bits(bits, m, n, k, group_size, int(bool(dp)), ctypes.byref(s), ctypes.byref(t),
                                 ctypes.byref(w), ctypes.byref(r)), "w4a16_plan_bits")
    return dict(split_k=s.value, tile_cols=t.value, waves=w.value, reduce=r.value)


def w4a16_check(m, n, k, group_size, split_k) -> int:
    """The raw return code (no exception): 0 or a negative W4A16_ERR_* value."""
    return int(lib().w4a16_check(m, n, k, group_size, split_k))


def w4a16_unpack(qweight, qzeros, q_u8, z_u8, n, k, group_size, stream=None) -> None:
    _check(lib().w4a16_unpack(_p(qweight), _p(qzeros), _p(q_u8), _p(z_u8), n, k, group_size, _stream(stream)),
           "w4a16_unpack")


def w4a16_dequant(qweight, scales, qzeros, W, n, k, group_size, stream=None) -> None:
    _check(lib().w4a16_dequant(_p(qweight), _p(scales), _p(qzeros), _p(W), n, k, group_size, _stream(stream)),
           "w4a16_dequant")


def w4a16_algorithmic_bytes(m, n, k, group_size) -> int:
    return int(lib().w4a16_algorithmic_bytes(m, n, k, group_size))


def w4a16_phase_timeouts() -> int:
    v = int(lib().w4a16_phase_timeouts())
    if v < 0:
        _check(v, "w4a16_phase_timeouts")
    return v


def w4a16_release_scratch() -> None:
    _check(lib().w4a16_release_scratch(), "w4a16_release_scratch")


def w4a16_set_phase_spin_limit(polls: int) -> None:
    _check(lib().w4a16_set_phase_spin_limit(polls), "w4a16_set_phase_spin_limit")


def w4a16_workspace_bytes(n_max: int) -> int:
    return int(lib().w4a16_workspace_bytes(n_max))


def w4a16_set_workspace(workspace, nbytes: int, n_max: int, stream=None) -> None:
    _check(lib().w4a16_set_workspace(_p(workspace), nbytes, n_max, _stream(stream)), "w4a16_set_workspace")


def w4a16_reserve_scratch(n_max: int) -> None:
    _check(lib().w4a16_reserve_scratch(n_max), "w4a16_reserve_scratch")

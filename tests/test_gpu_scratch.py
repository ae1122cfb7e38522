"""Split-k scratch of the library under HIP graphs, several streams and failure (GPU):
a captured call survives a later growth of the library's buffers; a call that would have to
allocate during a capture is refused; streams with workspaces of their own are independent;
a wait of the in-kernel zeroing that runs out ends the kernel, is counted, poisons the tile,
and makes the next call fail until the scratch is released; NaN goes through the fixed-point adds."""
import ctypes

import numpy as np
import pytest

from gpu_util import DeviceProblem, assert_parity
from oracle_pins import random_case
from paper_2402_00025_amd import binding as b

pytestmark = pytest.mark.gpu


@pytest.fixture(autouse=True)
def _fresh_scratch():
    import torch
    assert torch.cuda.is_available()
    torch.cuda.synchronize()
    b.w4a16_release_scratch()
    yield
    b.w4a16_set_phase_spin_limit(0)
    torch.cuda.synchronize()
    b.w4a16_release_scratch()


def _problem(oracle, m, n, k, seed):
    A, qw, s, qz = random_case(m, n, k, 128, seed=seed)
    Cref, _ = oracle.gemm(A, qw, s, qz, 128)
    return DeviceProblem(A, qw, s, qz, 128), Cref


def test_captured_call_survives_growth_of_the_scratch(oracle):
    """Capture a fixed-point call and a workspace-flavour call at small sizes, then run eager calls
    that need larger buffers (the library allocates new ones and keeps the old ones alive), then
    replay: the graph still points at the old buffers and must find them intact."""
    import torch
    small, Cs = _problem(oracle, 3, 512, 1024, seed=41)
    small_ws, Cw = _problem(oracle, 16, 512, 1024, seed=42)
    # larger than the buffers' first sizes: more than 16384 columns for the fixed-point words,
    # more partial tiles for the workspace flavour
    big, Cb = _problem(oracle, 2, 32768, 256, seed=43)
    big_ws, Cbw = _problem(oracle, 16, 4096, 1024, seed=44)
    b.w4a16_gemm_ex(*small.args(), 4, 64, 2, b.REDUCE_ATOMIC_FIXED)       # eager: allocates
    b.w4a16_gemm_ex(*small_ws.args(), 2, 64, 2, b.REDUCE_WORKSPACE)
    torch.cuda.synchronize()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g, stream=side):
        b.w4a16_gemm_ex(*small.args(), 4, 64, 2, b.REDUCE_ATOMIC_FIXED, stream=torch.cuda.current_stream())
        b.w4a16_gemm_ex(*small_ws.args(), 2, 64, 2, b.REDUCE_WORKSPACE, stream=torch.cuda.current_stream())
    for rep in range(3):
        b.w4a16_gemm_ex(*big.args(), 2, 64, 1, b.REDUCE_ATOMIC_FIXED)      # grows on the first round
        assert_parity(big.result(), Cb, f"eager big fixed, round {rep}")
        b.w4a16_gemm_ex(*big_ws.args(), 8, 64, 1, b.REDUCE_WORKSPACE)
        assert_parity(big_ws.result(), Cbw, f"eager big workspace, round {rep}")
        small.C.fill_(float("nan"))
        small_ws.C.fill_(float("nan"))
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        assert_parity(small.C.cpu().numpy(), Cs, f"replay {rep} fixed")
        assert_parity(small_ws.C.cpu().numpy(), Cw, f"replay {rep} workspace")
        # and eager again at the small size, now in the new buffers
        small.C.fill_(float("nan"))
        b.w4a16_gemm_ex(*small.args(), 4, 64, 2, b.REDUCE_ATOMIC_FIXED)
        assert_parity(small.result(), Cs, f"eager small after growth {rep}")


def test_allocation_during_capture_is_refused(oracle):
    """The first call with a split_k whose words do not exist yet, issued under capture: error,
    nothing captured for it; after w4a16_reserve_scratch the same capture works."""
    import torch
    p, Cref = _problem(oracle, 16, 512, 1024, seed=45)
    L = b.lib()
    vp = ctypes.c_void_p
    ptrs = [vp(t.data_ptr()) for t in (p.A, p.qweight, p.scales, p.qzeros, p.C)]
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g, stream=side):
        st = vp(torch.cuda.current_stream().cuda_stream)
        rc = L.w4a16_gemm_ex(*ptrs, 16, 512, 1024, 128, 4, 64, 2, b.REDUCE_ATOMIC_PK_F16_PHASE, st)
        rc_dp = L.w4a16_gemm_dp(*ptrs, 16, 512, 1024, 128, st)     # needs no scratch: fine under capture
    assert rc == b.ERR_STATE and rc_dp == b.OK
    assert "capture" in L.w4a16_last_hip_error().decode()
    b.w4a16_reserve_scratch(512)
    torch.cuda.synchronize()
    g2 = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g2, stream=side):
        b.w4a16_gemm_ex(*p.args(), 4, 64, 2, b.REDUCE_ATOMIC_PK_F16_PHASE, stream=torch.cuda.current_stream())
    for rep in range(2):
        p.C.fill_(float("nan"))
        torch.cuda.synchronize()
        g2.replay()
        torch.cuda.synchronize()
        assert_parity(p.C.cpu().numpy(), Cref, f"replay {rep} after reserve")
    assert b.w4a16_phase_timeouts() == 0


def test_streams_with_their_own_workspaces(oracle):
    """Two streams, each bound to a workspace of its own, issue split-k calls on the same tile
    origins at the same time; every result is right and nothing times out."""
    import torch
    n_max = 2048
    nbytes = b.w4a16_workspace_bytes(n_max)
    streams = [torch.cuda.Stream(), torch.cuda.Stream()]
    spaces = [torch.empty(nbytes, dtype=torch.uint8, device="cuda").fill_(0xFF) for _ in streams]  # bind must clear it
    torch.cuda.synchronize()
    for st, ws in zip(streams, spaces):
        b.w4a16_set_workspace(ws, nbytes, n_max, stream=st)
    cases = [(16, 1024, 2048, 4, 64, 2, b.REDUCE_ATOMIC_PK_F16_PHASE), (3, 1024, 2048, 8, 64, 2, b.REDUCE_ATOMIC_FIXED),
             (9, 1032, 2048, 4, 256, 4, b.REDUCE_ATOMIC_PK_F16_PHASE), (16, 1024, 1024, 2, 128, 4, b.REDUCE_ATOMIC_PK_F16_PHASE),
             (16, 520, 1024, 2, 64, 2, b.REDUCE_ATOMIC_F32)]
    probs = []
    for si in range(2):
        for ci, (m, n, k, S, tc, wv, red) in enumerate(cases):
            p, Cref = _problem(oracle, m, n, k, seed=60 + 10 * si + ci)
            probs.append((si, p, Cref, S, tc, wv, red))
    torch.cuda.synchronize()
    for rnd in range(4):
        for (si, p, _, S, tc, wv, red) in probs:
            p.C.fill_(float("nan"))
        torch.cuda.synchronize()
        # interleave the two streams' calls
        for ci in range(len(cases)):
            for si in range(2):
                _, p, _, S, tc, wv, red = probs[si * len(cases) + ci]
                b.w4a16_gemm_ex(*p.args(), S, tc, wv, red, stream=streams[si])
        torch.cuda.synchronize()
        for (si, p, Cref, S, tc, wv, red) in probs:
            assert_parity(p.C.cpu().numpy(), Cref, f"round {rnd} stream {si} S={S} tile={tc} reduce={red}")
    assert b.w4a16_phase_timeouts() == 0
    # beyond the workspace's n_max: refused
    wide, _ = _problem(oracle, 16, 4096, 512, seed=90)
    L = b.lib()
    vp = ctypes.c_void_p
    rc = L.w4a16_gemm_ex(*[vp(t.data_ptr()) for t in (wide.A, wide.qweight, wide.scales, wide.qzeros, wide.C)],
                         16, 4096, 512, 128, 2, 64, 2, b.REDUCE_ATOMIC_PK_F16_PHASE, vp(streams[0].cuda_stream))
    assert rc == b.ERR_LIMIT
    for st in streams:
        b.w4a16_set_workspace(None, 0, 0, stream=st)
    torch.cuda.synchronize()


@pytest.mark.parametrize("tile_cols,waves,split_k,k", [(64, 1, 8, 1024), (64, 2, 4, 2048), (256, 4, 4, 2048)])
def test_wait_that_runs_out_is_loud(oracle, tile_cols, waves, split_k, k):
    """Failure path of the in-kernel zeroing, forced from the host: the per-tile call counts of a
    bound workspace are corrupted for the slices other than the first, so those workgroups wait
    for a value the flag never takes; with a poll limit of 4 every kernel still ends.  The waits
    are counted, the tiles are poisoned with NaN, the next call returns W4A16_ERR_STATE without
    launching, and releasing the scratch makes the library usable again."""
    import torch
    n_max = 1024
    nbytes = b.w4a16_workspace_bytes(n_max)
    ws = torch.empty(nbytes, dtype=torch.uint8, device="cuda")
    st = torch.cuda.current_stream()
    b.w4a16_set_workspace(ws, nbytes, n_max, stream=st)
    p, Cref = _problem(oracle, 16, 512, k, seed=95)
    red = b.REDUCE_ATOMIC_PK_F16_PHASE
    b.w4a16_gemm_ex(*p.args(), split_k, tile_cols, waves, red)            # a good call first
    assert_parity(p.result(), Cref, "before the corruption")
    assert b.w4a16_phase_timeouts() == 0
    # workspace layout (32-bit words): 64 head, n_max / 16 tickets, then the levels of split_k = 2, 3, ...:
    # flags [4096], counts [4096][split_k]
    words = ws.view(torch.int32)
    level = 64 + n_max // 16 + 4096 * ((split_k - 2) + ((split_k - 1) * split_k // 2 - 1))
    counts = words[level + 4096: level + 4096 * (1 + split_k)].view(4096, split_k)
    counts[:, 1:] += 5
    torch.cuda.synchronize()
    b.w4a16_set_phase_spin_limit(4)
    p.C.fill_(0.0)
    b.w4a16_gemm_ex(*p.args(), split_k, tile_cols, waves, red)            # ends normally, wrong and loud
    torch.cuda.synchronize()
    got = p.C.cpu().numpy()
    assert b.w4a16_phase_timeouts() > 0
    step = 256 if tile_cols == 256 else tile_cols
    assert np.isnan(got[0, 0::step].astype(np.float32)).all()             # first pair of every tile poisoned
    L = b.lib()
    vp = ctypes.c_void_p
    ptrs = [vp(t.data_ptr()) for t in (p.A, p.qweight, p.scales, p.qzeros, p.C)]
    rc = L.w4a16_gemm_ex(*ptrs, 16, 512, k, 128, split_k, tile_cols, waves, red, vp(st.cuda_stream))
    assert rc == b.ERR_STATE                                               # sticky, no synchronisation needed
    rc = L.w4a16_gemm(*ptrs, 16, 512, k, 128, 0, vp(st.cuda_stream))
    assert rc in (b.ERR_STATE, b.OK)   # OK only if the library's plan needs no scratch for this shape
    b.w4a16_set_phase_spin_limit(0)
    b.w4a16_release_scratch()                                              # also forgets the binding
    p.C.fill_(float("nan"))
    b.w4a16_gemm_ex(*p.args(), split_k, tile_cols, waves, red)
    assert_parity(p.result(), Cref, "after the release")
    assert b.w4a16_phase_timeouts() == 0


def test_nan_and_infinity_through_the_fixed_point_adds(oracle):
    """Up to four rows with a split: a NaN activation makes its whole output row NaN (as the
    definition and every other reduction do), an infinite one gives NaN or infinities, and the
    rows beside them are untouched."""
    import torch
    A, qw, s, qz = random_case(4, 520, 2048, 128, seed=97)
    A[1, 700] = np.float16(np.nan)
    A[3, 5] = np.float16(np.inf)
    p = DeviceProblem(A, qw, s, qz, 128)
    Cref, _ = oracle.gemm(A, qw, s, qz, 128)
    assert np.isnan(Cref[1]).all() and np.isfinite(Cref[[0, 2]]).all()
    for split_k, waves in ((4, 2), (16, 1), (1, 4)):
        p.C.fill_(0.0)
        b.w4a16_gemm_ex(*p.args(), split_k, 64, waves, b.REDUCE_ATOMIC_FIXED)
        got = p.result().astype(np.float64)
        assert np.isnan(got[1]).all(), split_k
        assert not np.isfinite(got[3]).any(), split_k
        assert_parity(got[[0, 2]].astype(np.float16), Cref[[0, 2]], f"finite rows, S={split_k}")
        # a second call into the same words: nothing of the NaN is left behind
        A2 = A.copy()
        A2[1, 700] = np.float16(0.5)
        A2[3, 5] = np.float16(-0.25)
        p2 = DeviceProblem(A2, qw, s, qz, 128)
        C2, _ = oracle.gemm(A2, qw, s, qz, 128)
        b.w4a16_gemm_ex(*p2.args(), split_k, 64, waves, b.REDUCE_ATOMIC_FIXED)
        assert_parity(p2.result(), C2, f"after the NaN call, S={split_k}")

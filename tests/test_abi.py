"""The C-ABI library loads, exports every symbol include/flashfps.h declares,
and its host-side logic (sizes, validation, error strings) behaves as the
header says.  No compute call is made: this file runs without a GPU."""
import ctypes
import os
import re

import pytest

import paper_2604_17720_amd.binding as fb

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared_symbols():
    text = open(os.path.join(ROOT, "include", "flashfps.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(ffps_[a-z_]+)\s*\(", text)))


def test_every_declared_symbol_is_exported():
    L = fb.lib()
    names = _declared_symbols()
    assert sorted(names) == sorted(fb.EXPORTS)
    for n in names:
        assert getattr(L, n) is not None


def test_version_and_error_strings():
    assert fb.ffps_version() >= 100
    seen = set()
    for code in (0, -1, -2, -3, -4, -5, -6, -7):
        s = fb.ffps_strerror(code)
        assert s and s not in seen
        seen.add(s)
    assert "unknown" in fb.ffps_strerror(-99)


def test_prune_sizes_match_golden_table():
    with open(os.path.join(ROOT, "tests", "golden", "prune_sizes.txt")) as f:
        rows = [list(map(int, l.split())) for l in f if l.strip() and not l.startswith("#")]
    for n, m, kn, kd, fl, nc, k, r in rows:
        assert fb.ffps_prune_sizes(n, m, kn, kd, fl) == (nc, k, r)


@pytest.mark.parametrize("args", [
    (0, 1, 1, 1, 3), (10, 0, 1, 1, 3), (10, 11, 1, 1, 3), (10, 5, 0, 4, 3), (10, 5, 5, 4, 3),
    (10, 5, 1, 0, 3), (10, 5, 1, 4, 8), (100, 50, 1, 4, 1),   # k = 50 > N' = 25
])
def test_prune_sizes_rejects(args):
    with pytest.raises(fb.FlashFPSError) as e:
        fb.ffps_prune_sizes(*args)
    assert e.value.code == fb.FFPS_ERR_INVALID_ARG


def test_workspace_bytes_monotone_and_validated():
    a = fb.ffps_workspace_bytes(1, 1024, 512)
    b = fb.ffps_workspace_bytes(1, 200000, 50000)
    c = fb.ffps_workspace_bytes(8, 200000, 50000)
    assert 0 < a < b < c and a % 256 == 0
    assert b >= 200000 * 12 + 50000 * 4
    for bad in [(0, 10, 5), (1, 0, 1), (1, 10, 0), (1, 10, 11), (1 << 16, 1 << 16, 1)]:
        with pytest.raises(fb.FlashFPSError):
            fb.ffps_workspace_bytes(*bad)


def test_entry_points_validate_before_touching_the_device():
    """Invalid calls return FFPS_ERR_INVALID_ARG / WORKSPACE_TOO_SMALL from host
    checks alone (the pointers below are never dereferenced)."""
    L = fb.lib()
    fake = ctypes.c_void_p(0x1000)
    big = ctypes.c_size_t(1 << 40)
    null = ctypes.c_void_p(0)

    def exact(xyz=fake, B=1, N=100, M=10, start=0, variant=0, idx=fake, ws=fake, wsb=big):
        return L.ffps_exact(xyz, B, N, M, start, variant, idx, null, ws, wsb, null)

    assert exact(xyz=null) == fb.FFPS_ERR_INVALID_ARG
    assert exact(idx=null) == fb.FFPS_ERR_INVALID_ARG
    assert exact(ws=null) == fb.FFPS_ERR_INVALID_ARG
    assert exact(B=0) == fb.FFPS_ERR_INVALID_ARG
    assert exact(N=0) == fb.FFPS_ERR_INVALID_ARG
    assert exact(M=0) == fb.FFPS_ERR_INVALID_ARG
    assert exact(M=101) == fb.FFPS_ERR_INVALID_ARG
    assert exact(start=-1) == fb.FFPS_ERR_INVALID_ARG
    assert exact(start=100) == fb.FFPS_ERR_INVALID_ARG
    assert exact(variant=9) == fb.FFPS_ERR_INVALID_ARG
    assert exact(variant=1 << 17) == fb.FFPS_ERR_INVALID_ARG      # above the picks cap and the test knob
    assert exact(variant=-1) == fb.FFPS_ERR_INVALID_ARG
    assert fb.FFPS_VARIANT_TEST_NO_WAIT == 1 << 16 and fb.variant_with_picks(2, 7) == 2 | (7 << 8)
    assert exact(wsb=ctypes.c_size_t(16)) == fb.FFPS_ERR_WORKSPACE_TOO_SMALL

    k = ctypes.c_int(-7)
    def prune(kn=1, kd=4, flags=3, M=10, wsb=big):
        return L.ffps_prune(fake, 1, 100, M, 0, kn, kd, flags, 0, 0, fake, ctypes.byref(k), fake, wsb, null)
    assert prune(kn=0) == fb.FFPS_ERR_INVALID_ARG
    assert prune(kn=5) == fb.FFPS_ERR_INVALID_ARG
    assert prune(flags=8) == fb.FFPS_ERR_INVALID_ARG
    assert prune(flags=1, M=50) == fb.FFPS_ERR_INVALID_ARG      # k = 50 > N' = 25
    assert prune(wsb=ctypes.c_size_t(16)) == fb.FFPS_ERR_WORKSPACE_TOO_SMALL
    assert k.value == -7                                         # untouched on failure

    def stages(ms, mode=0, L_=None):
        arr = (ctypes.c_int * len(ms))(*ms)
        return L.ffps_cached_stages(fake, 1, 100, len(ms) if L_ is None else L_, arr, 0, 1, 1, 0, 0,
                                    mode, 0, fake, fake, big, null)
    assert stages([50, 60]) == fb.FFPS_ERR_INVALID_ARG           # increasing
    assert stages([101]) == fb.FFPS_ERR_INVALID_ARG              # M1 > N
    assert stages([50, 0]) == fb.FFPS_ERR_INVALID_ARG
    assert stages([50], mode=2) == fb.FFPS_ERR_INVALID_ARG
    assert stages([50], L_=0) == fb.FFPS_ERR_INVALID_ARG

    # The helper kernels of FPS-Prune and the stage chain carry the cloud number in
    # gridDim.y: more than 65535 clouds are refused before anything is enqueued.
    arr = (ctypes.c_int * 1)(2)
    assert L.ffps_prune(fake, 65536, 4, 2, 0, 1, 1, 3, 0, 0, fake, ctypes.byref(k), fake, big,
                        null) == fb.FFPS_ERR_INVALID_ARG
    assert L.ffps_cached_stages(fake, 65536, 4, 1, arr, 0, 1, 1, 0, 0, 0, 0, fake, fake, big,
                                null) == fb.FFPS_ERR_INVALID_ARG
    assert L.ffps_gather_rows(fake, 65536, 4, 3, fake, 2, 2, fake, null) == fb.FFPS_ERR_INVALID_ARG


def test_plan_of_the_five_configurations_and_its_limits():
    """Host logic behind FFPS_VARIANT_AUTO on a 256-CU device: which kernel runs,
    on how many workgroups, with how many reporting units per round."""
    import paper_2604_17720_amd.binding as fb
    WG, GRID, STREAM = fb.FFPS_VARIANT_WG, fb.FFPS_VARIANT_GRID, fb.FFPS_VARIANT_STREAM
    plan = fb.ffps_describe_plan
    assert plan(1, 1024) == (WG, 1, 448, 1)            # config 1: one unit per worker lane
    assert plan(32, 1024) == (WG, 1, 448, 32)          # config 2
    assert plan(8, 16384) == (GRID, 32, 224, 8)        # config 3: 32 workgroups x 7 reporting waves
    assert plan(1, 200000) == (GRID, 256, 256, 1)      # config 4: one unit per workgroup
    assert plan(1, 300000) == (GRID, 256, 256, 1)      # config 5
    # the boundaries of the kernels
    assert plan(1, 256)[0] == WG and plan(1, 256)[2] == 0          # one-pick kernel, no rounds
    assert plan(1, 257)[2] == 448 and plan(1, 4608)[2] == 448
    assert plan(1, 4608)[0] == WG and plan(1, 4609)[0] == GRID
    assert plan(1, 256 * 12288)[0] == GRID and plan(1, 256 * 12288 + 1)[0] == STREAM
    assert plan(1, 1 << 25) == (STREAM, 256, 256, 1)
    # the streaming kernel counts points in 32-bit integers and steps by 8192
    assert plan(1, 2 ** 31 - 1 - 8192 - 1024)[0] == STREAM
    with pytest.raises(fb.FlashFPSError) as e:
        plan(1, 2 ** 31 - 1 - 8192 - 1023)
    assert e.value.code == fb.FFPS_ERR_UNSUPPORTED_SIZE
    # explicit variants and their size limits
    assert plan(4, 20000, WG) == (WG, 1, 0, 4)
    with pytest.raises(fb.FlashFPSError) as e:
        plan(1, 24577, WG)
    assert e.value.code == fb.FFPS_ERR_UNSUPPORTED_SIZE
    with pytest.raises(fb.FlashFPSError):
        plan(1, 256 * 12288 + 1, GRID)
    for bad in ((0, 10, 0, 256), (1, 0, 0, 256), (1, 10, 7, 256), (1, 10, 0, 0)):
        with pytest.raises(fb.FlashFPSError) as e:
            plan(*bad)
        assert e.value.code == fb.FFPS_ERR_INVALID_ARG
    # invariants of the cluster plan over a sweep of shapes
    for B in (1, 2, 3, 8, 17, 40, 300):
        for N in (4609, 9000, 12500, 16384, 50000, 100000, 786433, 3000000):
            k, g, u, c = plan(B, N, GRID)
            assert k == GRID and 1 <= g <= 256 and 1 <= c <= B and g * c <= 256
            assert g <= u <= 256 and u % g == 0 and u // g in (1, 7)
            assert N <= g * 12288                      # every workgroup's slice fits its registers
    # a smaller device gets fewer workgroups, never more units than the exchange area holds
    k, g, u, c = plan(1, 200000, GRID, 64)
    assert g <= 64 and u <= 256


def test_torch_operators_register_and_infer_shapes():
    """torch.ops.flashfps.* exist and their shape functions work on fake tensors
    (no kernel runs, so no GPU is needed)."""
    import torch
    from torch._subclasses.fake_tensor import FakeTensorMode

    import paper_2604_17720_amd.torch_ops  # noqa: F401
    with FakeTensorMode():
        x = torch.empty(2, 100, 3, device="cuda")
        assert torch.ops.flashfps.fps_exact(x, 10, 0).shape == (2, 10)
        assert torch.ops.flashfps.fps_prune(x, 12, 1, 4, 3, 0, 0).shape == (2, 12)
        st = torch.ops.flashfps.fps_stages(x, [10, 5], 0, 1, 1, 0, 0, 0)
        assert st.shape == (2, 15) and st.dtype == torch.int32
        idx = torch.empty(2, 7, dtype=torch.int32, device="cuda")
        assert torch.ops.flashfps.gather_rows(x, idx).shape == (2, 7, 3)

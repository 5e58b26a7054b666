"""Host-side checks of the C ABI: the library loads, exports every symbol the header declares,
and rejects bad arguments before touching any device (so these run without a GPU)."""
import ctypes
import os
import re

import pytest

from paper_2512_09010_amd import binding as lv
from paper_2512_09010_amd import build as lvbuild

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def L():
    lvbuild.build(force=False)
    return lv.lib()


def declared_symbols():
    text = open(os.path.join(ROOT, "include", "luvc.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(luvc_[a-z0-9_]+)\s*\(", text)))


def test_exports_match_header(L):
    names = declared_symbols()
    assert set(names) == set(lv.EXPORTS)
    for n in names:
        assert hasattr(L, n), n
    assert b"gfx950" in L.luvc_version()


def test_keep_count(L):
    assert lv.luvc_keep_count(1024, 0.20) == 205
    assert lv.luvc_keep_count(196, 0.05) == 10
    assert lv.luvc_keep_count(144, 0.25) == 36
    assert lv.luvc_keep_count(720, 0.15) == 108
    assert lv.luvc_keep_count(2048, 0.10) == 205
    assert lv.luvc_keep_count(10, 0.0) == 1 and lv.luvc_keep_count(10, 3.0) == 10
    assert lv.luvc_keep_count(0, 0.5) == 0


def test_plan(L):
    assert lv.luvc_oim_plan(24, 24, 144) == [(1, 12), (0, 12)]
    assert lv.luvc_oim_plan(64, 64, 1024) == [(1, 32), (0, 32)]
    assert lv.luvc_oim_plan(112, 112, 196) == [(1, 56), (0, 56), (1, 28), (0, 28), (1, 14), (0, 14)]
    assert lv.luvc_oim_plan(16, 16, 16 * 14) == [(1, 2)]            # the paper's merge number 2 on one axis
    assert lv.luvc_oim_plan(8, 8, 64) == []
    assert lv.luvc_oim_plan(9, 7, 4 * 3) == [(1, 4), (0, 5)]          # odd lines: every source merges (ceil)
    with pytest.raises(lv.LuvcError):
        lv.luvc_oim_plan(16, 16, 255)                                # 255 is no multiple of 16
    with pytest.raises(lv.LuvcError):
        lv.luvc_oim_plan(16, 16, 0)
    with pytest.raises(lv.LuvcError):
        lv.luvc_oim_plan(16, 16, 257)
    # every plan lands exactly on its target
    for H, W, t in [(24, 24, 144), (10, 6, 15), (7, 5, 6), (33, 17, 128), (33, 17, 20 * 8)]:
        h, w = H, W
        for axis, m in lv.luvc_oim_plan(H, W, t):
            assert 0 < m <= ((w if axis else h) + 1) // 2
            if axis:
                w -= m
            else:
                h -= m
        assert h * w == t


def P(passes):
    return lv._passes(passes), len(passes)


def test_workspace_queries(L):
    p, n = P([(1, 32), (0, 32)])
    a = L.luvc_oim_workspace_bytes(8, 64, 64, 1280, lv.LUVC_BF16, p, n)
    assert a > 8 * 64 * 32 * 1280 * 2 and a % 256 == 0
    assert L.luvc_oim_workspace_bytes(8, 64, 64, 1280, 7, p, n) == 0
    assert L.luvc_oim_workspace_bytes(0, 64, 64, 1280, lv.LUVC_BF16, p, n) == 0
    bad, nb = P([(1, 33)])
    assert L.luvc_oim_workspace_bytes(8, 64, 64, 1280, lv.LUVC_BF16, bad, nb) == 0
    assert L.luvc_spu_workspace_bytes(8, 1024, 3584, lv.LUVC_BF16, 102) > 0
    assert L.luvc_spu_workspace_bytes(8, 1024, 3584, lv.LUVC_BF16, 513) == 0
    assert L.luvc_spu_workspace_bytes(8, 0, 3584, lv.LUVC_BF16, 0) == 0


FAKE = ctypes.c_void_p(0x1000)          # never dereferenced: every call below must fail validation first


def test_oim_merge_rejects_bad_arguments(L):
    p, n = P([(1, 2), (0, 2)])
    args = lambda **kw: [kw.get("x", FAKE), None, kw.get("B", 1), kw.get("H", 8), kw.get("W", 8), kw.get("D", 64),
                         kw.get("dt", lv.LUVC_F32), kw.get("p", p), kw.get("n", n), kw.get("target", 0),
                         kw.get("xo", FAKE), kw.get("so", FAKE), None, None, kw.get("ws", None), kw.get("wsb", 0), None]
    assert L.luvc_oim_merge(*args(x=None)) == lv.LUVC_ERR_INVALID_ARG
    assert L.luvc_oim_merge(*args(xo=None)) == lv.LUVC_ERR_INVALID_ARG
    assert L.luvc_oim_merge(*args(so=None)) == lv.LUVC_ERR_INVALID_ARG
    assert L.luvc_oim_merge(*args(B=0)) == lv.LUVC_ERR_INVALID_ARG
    assert L.luvc_oim_merge(*args(D=-1)) == lv.LUVC_ERR_INVALID_ARG
    assert L.luvc_oim_merge(*args(dt=5)) == lv.LUVC_ERR_INVALID_ARG
    assert L.luvc_oim_merge(*args(n=0)) == lv.LUVC_ERR_INVALID_ARG
    assert L.luvc_oim_merge(*args(n=99)) == lv.LUVC_ERR_INVALID_ARG
    assert L.luvc_oim_merge(*args(target=35)) == lv.LUVC_ERR_INVALID_ARG       # schedule ends at 6x6 = 36
    assert "36" in lv.last_error()
    for bad in ([(1, 5)], [(2, 1)], [(1, -1)], [(1, 4), (1, 2), (1, 1), (1, 1)]):
        bp, bn = P(bad)
        assert L.luvc_oim_merge(*args(p=bp, n=bn)) == lv.LUVC_ERR_INVALID_ARG, bad
    # valid arguments but no / short / misaligned workspace
    assert L.luvc_oim_merge(*args()) == lv.LUVC_ERR_WORKSPACE
    assert L.luvc_oim_merge(*args(ws=ctypes.c_void_p(0x10000), wsb=16)) == lv.LUVC_ERR_WORKSPACE
    assert L.luvc_oim_merge(*args(ws=ctypes.c_void_p(0x10008), wsb=1 << 30)) == lv.LUVC_ERR_WORKSPACE
    assert lv.last_error() != ""


def test_spu_rejects_bad_arguments(L):
    sc = lambda **kw: [kw.get("x", FAKE), kw.get("B", 2), kw.get("N", 64), kw.get("D", 128), kw.get("rs", 128),
                       kw.get("dt", lv.LUVC_BF16), kw.get("sigma", 6), 1, kw.get("out", FAKE), kw.get("ws", None),
                       kw.get("wsb", 0), None]
    assert L.luvc_spu_score(*sc(x=None)) == lv.LUVC_ERR_INVALID_ARG
    assert L.luvc_spu_score(*sc(out=None)) == lv.LUVC_ERR_INVALID_ARG
    assert L.luvc_spu_score(*sc(N=0)) == lv.LUVC_ERR_INVALID_ARG
    assert L.luvc_spu_score(*sc(rs=127)) == lv.LUVC_ERR_INVALID_ARG
    assert L.luvc_spu_score(*sc(sigma=33)) == lv.LUVC_ERR_INVALID_ARG
    assert L.luvc_spu_score(*sc(sigma=-1)) == lv.LUVC_ERR_INVALID_ARG
    assert L.luvc_spu_score(*sc(dt=2)) == lv.LUVC_ERR_INVALID_ARG
    assert L.luvc_spu_score(*sc(N=1 << 20, sigma=5)) == lv.LUVC_ERR_UNSUPPORTED
    assert L.luvc_spu_score(*sc()) == lv.LUVC_ERR_WORKSPACE
    pr = lambda **kw: [kw.get("x", FAKE), kw.get("s", FAKE), kw.get("B", 2), kw.get("N", 64), kw.get("D", 128),
                       kw.get("rs", 128), kw.get("dt", lv.LUVC_BF16), kw.get("k", 8), kw.get("idx", FAKE),
                       kw.get("xo", FAKE), None, 0, None]
    assert L.luvc_spu_prune(*pr(s=None)) == lv.LUVC_ERR_INVALID_ARG
    assert L.luvc_spu_prune(*pr(idx=None)) == lv.LUVC_ERR_INVALID_ARG
    assert L.luvc_spu_prune(*pr(x=None)) == lv.LUVC_ERR_INVALID_ARG            # x_out without x
    assert L.luvc_spu_prune(*pr(k=0)) == lv.LUVC_ERR_INVALID_ARG
    assert L.luvc_spu_prune(*pr(k=65)) == lv.LUVC_ERR_INVALID_ARG
    assert L.luvc_spu_prune(*pr(rs=4)) == lv.LUVC_ERR_INVALID_ARG
    assert L.luvc_spu_prune(*pr(B=-3)) == lv.LUVC_ERR_INVALID_ARG


def test_wide_matching_arguments(L):
    """luvc_oim_merge_wide / luvc_oim_wide_workspace_bytes validate on the host: nothing is enqueued for a bad call."""
    passes = [(1, 2), (0, 2)]
    need1 = lv.luvc_oim_wide_workspace_bytes(2, 16, 16, 64, lv.LUVC_BF16, passes, 1)
    need0 = lv.luvc_oim_wide_workspace_bytes(2, 16, 16, 64, lv.LUVC_BF16, passes, 0)
    assert need1 == lv.luvc_oim_workspace_bytes(2, 16, 16, 64, lv.LUVC_BF16, passes)     # radius 1 is the adjacent matching
    assert need0 >= need1 + 2 * 16 * 8 * 8 * 8 and need0 % 256 == 0                      # + the source x destination matrices
    assert lv.luvc_oim_wide_workspace_bytes(2, 16, 16, 64, lv.LUVC_BF16, passes, -1) == 0
    parr = lv._passes(passes)
    rc = L.luvc_oim_merge_wide(None, None, 2, 16, 16, 64, lv.LUVC_BF16, parr, 2, 0, 0, None, None, None, None, None, 0, None)
    assert rc == lv.LUVC_ERR_INVALID_ARG
    rc = L.luvc_oim_merge_wide(ctypes.c_void_p(256), None, 2, 16, 16, 64, lv.LUVC_BF16, parr, 2, -3, 0,
                               ctypes.c_void_p(256), ctypes.c_void_p(256), None, None, ctypes.c_void_p(256), 1 << 30, None)
    assert rc == lv.LUVC_ERR_INVALID_ARG and b"radius" in L.luvc_last_error()
    rc = L.luvc_oim_merge_wide(ctypes.c_void_p(256), None, 1, 1, 4096, 64, lv.LUVC_BF16, lv._passes([(1, 2)]), 1, 0, 0,
                               ctypes.c_void_p(256), ctypes.c_void_p(256), None, None, ctypes.c_void_p(256), 1 << 40, None)
    assert rc == lv.LUVC_ERR_UNSUPPORTED                                                  # line longer than the wide path takes


def test_wide_and_keyed_workspaces_cover_the_one_launch_passes(L):
    """The workspace of a wide-matching call holds what the one-launch passes need on top of the three-launch ones: two
    grids of row ids and a row per merged destination (at most m per line and pass); the keyed call adds the same rows
    for the keys.  Sizes grow with the schedule and shrink to the plain call's for radius 1."""
    B, H, W, D, Dm = 2, 24, 20, 64, 16
    one = [(1, 2)]
    three = [(1, 2), (0, 2), (1, 2)]
    w1 = lv.luvc_oim_wide_workspace_bytes(B, H, W, D, lv.LUVC_BF16, one, 0)
    w3 = lv.luvc_oim_wide_workspace_bytes(B, H, W, D, lv.LUVC_BF16, three, 0)
    ids = 2 * B * H * W * 4
    rows1 = B * H * 2 * D * 2                                   # one pass along W: 2 merged destinations per row of the grid
    rows3 = rows1 + B * (W - 2) * 2 * D * 2 + B * (H - 2) * 2 * D * 2
    assert w1 >= ids + rows1 and w3 >= ids + rows3 and w3 > w1
    k3 = lv.luvc_oim_keyed_workspace_bytes(B, H, W, D, Dm, lv.LUVC_BF16, three, 0)
    assert k3 >= w3 + rows3 // D * Dm
    k1 = lv.luvc_oim_keyed_workspace_bytes(B, H, W, D, Dm, lv.LUVC_BF16, three, 1)
    assert k1 < k3 and k1 >= lv.luvc_oim_workspace_bytes(B, H, W, D, lv.LUVC_BF16, three)
    assert lv.luvc_oim_keyed_workspace_bytes(B, H, W, D, 0, lv.LUVC_BF16, three, 0) == 0


def test_selftest_entry_points_reject_bad_arguments(L):
    rc = L.luvc_selftest_screen_tile(None, None, 64, lv.LUVC_BF16, None, None)
    assert rc == lv.LUVC_ERR_INVALID_ARG
    rc = L.luvc_selftest_screen_tile(ctypes.c_void_p(256), ctypes.c_void_p(256), 12, lv.LUVC_BF16, ctypes.c_void_p(256), None)   # 24-byte rows
    assert rc == lv.LUVC_ERR_INVALID_ARG
    rc = L.luvc_selftest_screen_tile(ctypes.c_void_p(264), ctypes.c_void_p(256), 64, lv.LUVC_BF16, ctypes.c_void_p(256), None)   # misaligned rows
    assert rc == lv.LUVC_ERR_INVALID_ARG
    rc = L.luvc_selftest_screen_tile(ctypes.c_void_p(256), ctypes.c_void_p(256), 64, 9, ctypes.c_void_p(256), None)
    assert rc == lv.LUVC_ERR_INVALID_ARG
    rc = L.luvc_selftest_fdot2(None, None, 4, 4, None, None)
    assert rc == lv.LUVC_ERR_INVALID_ARG


def test_anyres_plan_and_cascade_keeps_against_the_oracle(L, oracle):
    """Host arithmetic of the library against the oracle's separately written routines, over many shapes."""
    for H in (1, 2, 7, 16, 24, 37, 64, 112, 200):
        for W in (1, 3, 8, 24, 31, 64, 128, 224):
            for cap in (1, 10, 64, 144, 1024, 10 ** 6):
                assert lv.luvc_oim_plan_anyres(H, W, cap) == oracle.plan_anyres(H, W, cap), (H, W, cap)
    with pytest.raises(lv.LuvcError):
        lv.luvc_oim_plan_anyres(4, 4, 0)
    with pytest.raises(lv.LuvcError):
        lv.luvc_oim_plan_anyres(4096, 4096, 1, max_passes=3)          # needs more passes than the caller has room for
    for N0 in (1, 8, 196, 1024, 2048):
        for ratio in (0.05, 0.2, 0.5, 1.0):
            for stages in (1, 2, 5):
                for elim in (False, True):
                    assert lv.luvc_spu_cascade_keeps(N0, ratio, stages, elim) == oracle.cascade_keeps(N0, ratio, stages, elim)


def test_ragged_queries_and_arguments(L):
    """Workspace of a ragged call = the largest need of its runs; bad items are rejected on the host."""
    i32 = lambda v: (ctypes.c_int32 * len(v))(*v)
    passes = [(1, 12), (0, 12), (1, 8), (1, 4), (1, 12), (0, 12)]
    H, W, npz = [24, 16, 24], [24, 16, 24], [2, 2, 2]
    need = L.luvc_oim_ragged_workspace_bytes(3, i32(H), i32(W), 64, lv.LUVC_BF16, lv._passes(passes), i32(npz))
    a = lv.luvc_oim_workspace_bytes(1, 24, 24, 64, lv.LUVC_BF16, passes[0:2])
    b = lv.luvc_oim_workspace_bytes(1, 16, 16, 64, lv.LUVC_BF16, passes[2:4])
    assert need == max(a, b) > 0
    # equal neighbours form one run: the need is that of a batch of two
    need2 = L.luvc_oim_ragged_workspace_bytes(2, i32([24, 24]), i32([24, 24]), 64, lv.LUVC_BF16, lv._passes(passes[0:2] * 2), i32([2, 2]))
    assert need2 == lv.luvc_oim_workspace_bytes(2, 24, 24, 64, lv.LUVC_BF16, passes[0:2])
    assert L.luvc_oim_ragged_workspace_bytes(2, i32([24, 0]), i32([24, 24]), 64, lv.LUVC_BF16, lv._passes(passes[0:2] * 2), i32([2, 2])) == 0
    assert L.luvc_oim_ragged_workspace_bytes(1, i32([4]), i32([4]), 64, lv.LUVC_BF16, lv._passes([(1, 3)]), i32([1])) == 0      # m too large
    ns, sg = [1024, 1024, 196], [102, 102, 4]
    need = L.luvc_spu_ragged_workspace_bytes(3, i32(ns), 256, lv.LUVC_BF16, i32(sg))
    assert need == max(lv.luvc_spu_workspace_bytes(2, 1024, 256, lv.LUVC_BF16, 102), lv.luvc_spu_workspace_bytes(1, 196, 256, lv.LUVC_BF16, 4))
    assert L.luvc_spu_ragged_workspace_bytes(2, i32([8, 8]), 16, lv.LUVC_BF16, i32([4, 5])) == 0                                # sigma > N/2
    # a stage call with a bad item is refused before anything is enqueued (no device is touched: pointers are dummies)
    one = ctypes.c_void_p(256)
    rc = L.luvc_spu_stage_ragged(one, 2, i32([8, 8]), 16, 16, lv.LUVC_BF16, i32([2, 2]), 1, i32([3, 9]), None, one, one, one, None, None, 0, None)
    assert rc == lv.LUVC_ERR_INVALID_ARG and b"n_keep" in L.luvc_last_error()
    rc = L.luvc_oim_merge_ragged(one, None, 1, i32([4]), i32([4]), 16, lv.LUVC_BF16, lv._passes([(2, 1)]), i32([1]), one, one, None, None, None, 0, None)
    assert rc == lv.LUVC_ERR_INVALID_ARG and b"axis" in L.luvc_last_error()


def test_header_is_plain_c(tmp_path):
    """include/luvc.h must be usable from C (and C++) without any HIP or torch header."""
    import shutil
    import subprocess
    src = tmp_path / "use_luvc.c"
    src.write_text('#include "luvc.h"\nint main(void) { luvc_oim_pass p = {1, 2}; luvc_status (*f)(int, int, int64_t, luvc_oim_pass*, int, int*) = luvc_oim_plan; return (int)sizeof(p) - 8 + (f ? 0 : 1); }\n')
    inc = os.path.join(ROOT, "include")
    for cc, std in (("gcc", "-std=c99"), ("g++", "-std=c++11")):
        if shutil.which(cc) is None:
            pytest.skip(f"{cc} not installed")
        args = [cc, std, "-Wall", "-Werror", "-pedantic", "-fsyntax-only", "-I", inc]
        args += ["-x", "c++", str(src)] if cc == "g++" else [str(src)]
        r = subprocess.run(args, capture_output=True, text=True)
        assert r.returncode == 0, r.stderr

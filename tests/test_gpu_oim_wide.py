"""GPU parity: luvc_oim_merge_wide (candidates beyond the adjacent destinations, up to the whole line; the
bipartite matching of the paper's Section 3.1 cost and its merge number 2) against the CPU oracle."""
import numpy as np
import pytest
import torch

from paper_2512_09010_amd import binding as lv
from paper_2512_09010_amd import workloads as wl
from gpu_util import OIM_MARGIN, RTOL, assert_close, oim_reference, round_mode, to_dev, to_host_f64

pytestmark = pytest.mark.gpu
W_AX, H_AX = 1, 0


def run_wide(oracle, x_io, dtype, passes, radius, sizes=None, tag=""):
    print(f"[oim wide] {tag} shape={x_io.shape} dtype={dtype} passes={passes} radius={radius}", flush=True)
    s_dev = None if sizes is None else torch.from_numpy(np.ascontiguousarray(sizes, dtype=np.int32)).cuda()
    out = lv.luvc_oim_merge_wide(to_dev(x_io, dtype), passes, radius, sizes=s_dev)
    torch.cuda.synchronize()
    ref = oim_reference(oracle, wl.widen(x_io, dtype), passes, out["merged_map"].cpu().numpy(), dtype, sizes=sizes, R=radius)
    assert out["x"].shape == ref["x"].shape
    np.testing.assert_array_equal(out["sizes"].cpu().numpy().astype(np.int64), ref["sizes"])
    np.testing.assert_array_equal(out["merged_map"].cpu().numpy(), ref["merged_map"])
    np.testing.assert_array_equal(out["kept_map"].cpu().numpy(), ref["kept_map"])
    got = to_host_f64(out["x"])
    assert_close(got, ref["x"], RTOL[dtype], f"{tag} features")
    if dtype == "bf16":
        np.testing.assert_array_equal(got, ref["x"])         # fp64 merge in the oracle's term order, one rounding
    return out, ref


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("radius", [0, 2, 3])
@pytest.mark.parametrize("B,H,W,D,passes", [
    (1, 1, 2, 8, [(W_AX, 1)]),
    (1, 3, 1, 8, [(H_AX, 1)]),
    (2, 5, 7, 24, [(W_AX, 4)]),
    (2, 6, 9, 40, [(W_AX, 2), (H_AX, 2)]),                 # the paper's merge number 2
    (1, 9, 6, 40, [(H_AX, 2), (W_AX, 2)]),                 # Algorithm 1 order: height first
    (1, 16, 16, 72, [(W_AX, 2), (H_AX, 2), (W_AX, 2), (H_AX, 2), (W_AX, 2), (H_AX, 2)]),   # three OIM operations
    (2, 4, 4, 33, [(W_AX, 1), (H_AX, 0)]),                 # rows that are not 16-byte multiples, m = 0 pass
    (1, 3, 70, 48, [(W_AX, 35)]),                          # 35 sources x 35 destinations: several 16 x 16 tiles with ragged edges
    (1, 71, 2, 16, [(H_AX, 10)]),
    (2, 7, 11, 520, [(W_AX, 6), (H_AX, 4)]),               # channels not a multiple of the 32-channel block
])
def test_wide_small_random(oracle, dtype, radius, B, H, W, D, passes):
    rng = np.random.default_rng(B * 1000 + H * 100 + W * 10 + D + radius)
    x = wl.cast_io(rng.standard_normal((B, H, W, D)).astype(np.float32), dtype)
    run_wide(oracle, x, dtype, passes, radius, tag="random")
    sizes = rng.integers(1, 6, (B, H, W))
    run_wide(oracle, x, dtype, passes, radius, sizes=sizes, tag="random+sizes")


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_wide_many_sources_into_one_destination(oracle, dtype):
    # every source of a line is a noisy copy of the line's last destination: they all fold into it
    rng = np.random.default_rng(5)
    B, H, W, D = 1, 4, 18, 64
    x = rng.standard_normal((B, H, W, D)).astype(np.float32)
    for h in range(H):
        for w in range(0, W, 2):
            x[0, h, w] = x[0, h, W - 1] + 0.01 * rng.standard_normal(D)
    x = wl.cast_io(x, dtype)
    out, ref = run_wide(oracle, x, dtype, [(W_AX, 9)], 0, tag="funnel")
    assert (ref["sizes"][0, :, -1] == 10).all()              # nine sources and the destination itself
    sizes = rng.integers(1, 4, (B, H, W))
    run_wide(oracle, x, dtype, [(W_AX, 9)], 0, sizes=sizes, tag="funnel+sizes")


def test_wide_radius_one_is_the_adjacent_matching(oracle):
    rng = np.random.default_rng(9)
    x = wl.cast_io(wl.smooth_field(rng, 2, 8, 10, 64, 2.0) + 0.1 * rng.standard_normal((2, 8, 10, 64)).astype(np.float32), "bf16")
    passes = [(W_AX, 2), (H_AX, 2)]
    a = lv.luvc_oim_merge_wide(to_dev(x, "bf16"), passes, 1)
    b = lv.luvc_oim_merge(to_dev(x, "bf16"), passes)
    torch.cuda.synchronize()
    for k in ("x", "sizes", "merged_map", "kept_map"):
        assert torch.equal(a[k], b[k]), k


@pytest.mark.parametrize("i", [1, 3])
def test_wide_workload_shapes(oracle, i):
    """Encoder-sized grids of the benchmark workloads with the paper's setting: whole-line matching, merge number 2,
    three OIM operations (W then H, three times)."""
    w = wl.workload(i)
    x = wl.oim_input(w)[:2]
    passes = [(W_AX, 2), (H_AX, 2)] * 3
    run_wide(oracle, x, w.dtype, passes, 0, tag=w.name)


@pytest.mark.parametrize("seed", range(16))
def test_wide_random_schedules(oracle, seed):
    """Seeded random grids, radii (whole line, 2..4) and schedules of up to four passes with any m."""
    rng = np.random.default_rng(2000 + seed)
    dtype = "bf16" if seed % 2 else "f32"
    radius = int(rng.choice([0, 0, 2, 3, 4]))
    B, H, W = int(rng.integers(1, 3)), int(rng.integers(1, 30)), int(rng.integers(1, 30))
    D = int(rng.choice([8, 24, 33, 64, 72, 136]))
    passes, h, w = [], H, W
    for _ in range(int(rng.integers(1, 5))):
        axis = int(rng.integers(0, 2))
        length = w if axis else h
        m = 0 if length == 1 else min(int(rng.integers(0, (length + 1) // 2 + 1)), length - 1)
        passes.append((axis, m))
        if axis:
            w -= m
        else:
            h -= m
    x = wl.cast_io(wl.smooth_field(rng, B, H, W, D, 2.0) + 0.3 * rng.standard_normal((B, H, W, D)).astype(np.float32), dtype)
    sizes = rng.integers(1, 4, (B, H, W)) if seed % 3 == 0 else None
    run_wide(oracle, x, dtype, passes, radius, sizes=sizes, tag=f"fuzz{seed}")


def test_wide_merge_near_a_rounding_tie(oracle):
    """Means that sit on a bf16 rounding boundary except for a term 2^-24 times smaller, through the wide merge."""
    D = 64
    rng = np.random.default_rng(12)
    x = (0.05 * rng.standard_normal((1, 3, 2, D))).astype(np.float32)
    sizes = np.ones((1, 3, 2), np.int64)
    sizes[0, 1, :] = 2
    a, b = -0.197265625, -0.380859375                    # (a + 2 b) / 4 = -245.5 * 2^-10
    for ch in range(32):
        scale = 2.0 ** (ch % 7 - 3)
        sign = -1.0 if ch & 8 else 1.0
        nudge = (1.0 if ch & 16 else -1.0) * 2.0 ** -26
        x[0, 0, 0, ch], x[0, 1, 0, ch], x[0, 2, 0, ch] = sign * a * scale, sign * b * scale, nudge * scale
    x_io = wl.cast_io(x, "bf16")
    run_wide(oracle, x_io, "bf16", [(H_AX, 2)], 0, sizes=sizes, tag="tie+tiny")
    run_wide(oracle, np.ascontiguousarray(x_io.transpose(0, 2, 1, 3)), "bf16", [(W_AX, 2)], 2, sizes=np.ascontiguousarray(sizes.transpose(0, 2, 1)), tag="tie+tiny W")


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("B,H,W,D,passes,radius", [
    (1, 2, 128, 16, [(W_AX, 3), (W_AX, 2)], 0),            # longest line of the one-launch passes
    (1, 127, 2, 24, [(H_AX, 64)], 0),                      # every source merged, odd length
    (1, 2, 140, 16, [(W_AX, 5), (H_AX, 1)], 0),            # longer lines: the three-launch passes
    (1, 300, 1, 8, [(H_AX, 7)], 3),
    (2, 20, 20, 64, [(W_AX, 0), (H_AX, 3), (W_AX, 10), (H_AX, 0)], 0),   # passes that merge nothing between passes that do
])
def test_wide_line_lengths_around_the_one_launch_limit(oracle, dtype, B, H, W, D, passes, radius):
    rng = np.random.default_rng(H * 1000 + W + D)
    x = wl.cast_io(wl.smooth_field(rng, B, H, W, D, 2.0) + 0.3 * rng.standard_normal((B, H, W, D)).astype(np.float32), dtype)
    sizes = rng.integers(1, 4, (B, H, W))
    run_wide(oracle, x, dtype, passes, radius, tag="lengths")
    run_wide(oracle, x, dtype, passes, radius, sizes=sizes, tag="lengths+sizes")


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_wide_one_launch_passes_and_three_launch_passes_agree(dtype):
    """The same call on a 16-byte aligned input (row ids between the passes, one launch per pass, tokens moved once) and
    on a copy that starts 8 bytes off (every pass materialised by three launches): identical outputs."""
    rng = np.random.default_rng(31)
    B, H, W, D = 2, 24, 20, 136
    tdt = torch.float32 if dtype == "f32" else torch.bfloat16
    x = torch.from_numpy(wl.smooth_field(rng, B, H, W, D, 2.0) + 0.3 * rng.standard_normal((B, H, W, D)).astype(np.float32)).to(tdt).cuda()
    off = 8 // x.element_size()
    flat = torch.empty(x.numel() + off, dtype=tdt, device="cuda")
    flat[off:] = x.reshape(-1)
    x_off = flat[off:].view(B, H, W, D)
    assert x.data_ptr() % 16 == 0 and x_off.data_ptr() % 16 == 8
    sizes = torch.from_numpy(rng.integers(1, 5, (B, H, W)).astype(np.int32)).cuda()
    for passes, radius in (([(W_AX, 2), (H_AX, 2)] * 3, 0), ([(H_AX, 5), (W_AX, 10), (H_AX, 1)], 2)):
        a = lv.luvc_oim_merge_wide(x, passes, radius, sizes=sizes)
        b = lv.luvc_oim_merge_wide(x_off, passes, radius, sizes=sizes)
        torch.cuda.synchronize()
        for k in ("x", "sizes", "merged_map", "kept_map"):
            assert torch.equal(a[k], b[k]), (passes, radius, k)


def test_wide_without_maps(oracle):
    rng = np.random.default_rng(37)
    x = wl.cast_io(rng.standard_normal((2, 10, 12, 64)).astype(np.float32), "bf16")
    passes = [(W_AX, 2), (H_AX, 2), (W_AX, 3)]
    ref = oracle.oim_merge(wl.widen(x, "bf16"), passes, R=0, round_mode=oracle.ROUND_BF16)
    assert ref["margin"] > OIM_MARGIN
    out = lv.luvc_oim_merge_wide(to_dev(x, "bf16"), passes, 0, want_maps=False)
    torch.cuda.synchronize()
    np.testing.assert_array_equal(to_host_f64(out["x"]), ref["x"])
    np.testing.assert_array_equal(out["sizes"].cpu().numpy().astype(np.int64), ref["sizes"])


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("D", [8, 16, 24, 72, 520, 1280, 2048])
def test_screening_tile_error_stays_inside_the_bound_the_decisions_assume(dtype, D):
    """The 32 x 32 tile of dot products formed on the matrix cores in the storage precision against exact sums, on rows
    chosen to provoke accumulation error: the screening of the wide matching assumes an error of at most D 2^-23 times
    the sum of the magnitudes of the products (it budgets twice that, relative to the product of the norms)."""
    rng = np.random.default_rng(D)
    tdt = torch.float32 if dtype == "f32" else torch.bfloat16
    cases = {
        "normal": (rng.standard_normal((32, D)), rng.standard_normal((32, D))),
        "positive, equal magnitudes": (1.0 + rng.random((32, D)) / 128, 1.0 + rng.random((32, D)) / 128),
        "wide range": (rng.standard_normal((32, D)) * 2.0 ** rng.integers(-20, 20, (32, D)), rng.standard_normal((32, D)) * 2.0 ** rng.integers(-20, 20, (32, D))),
        "cancelling": (np.tile([1.0, -1.0], (32, D // 2)) * (1.0 + rng.random((32, D)) / 64), np.ones((32, D)) + rng.random((32, D)) / 64),
        "one large term first": (np.concatenate([np.full((32, 1), 4096.0), rng.random((32, D - 1))], 1), np.concatenate([np.full((32, 1), 4096.0), rng.random((32, D - 1))], 1)),
    }
    for name, (a, c) in cases.items():
        ta, tc = torch.from_numpy(a).to(tdt).cuda(), torch.from_numpy(c).to(tdt).cuda()
        got = lv.luvc_selftest_screen_tile(ta, tc).cpu().numpy().astype(np.float64)
        a64, c64 = ta.cpu().to(torch.float64).numpy(), tc.cpu().to(torch.float64).numpy()
        exact = a64 @ c64.T
        mags = np.abs(a64) @ np.abs(c64).T
        worst = (np.abs(got - exact) / mags).max()
        print(f"[screen tile] {dtype} D={D} {name}: worst error {worst:.3e} of the magnitudes, allowed {D * 2.0 ** -23:.3e}", flush=True)
        assert worst <= D * 2.0 ** -23, (name, worst)


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_wide_decisions_the_screening_cannot_tell(oracle, dtype):
    """Lines of near-duplicate tokens (all cosines of a line within the screening's error of each other: every pair is
    repeated in fp64), lines of identical tokens (exact ties: the lower position wins twice over), and a zero token."""
    rng = np.random.default_rng(41)
    base = rng.standard_normal((1, 1, 1, 64)).astype(np.float32)
    for (H, W, passes, radius) in ((6, 24, [(W_AX, 2), (H_AX, 2)], 0), (3, 128, [(W_AX, 64)], 0), (4, 128, [(W_AX, 2)], 0),
                                   (128, 2, [(H_AX, 5)], 3), (10, 12, [(W_AX, 6), (H_AX, 5)], 2)):
        x = base + 1e-3 * rng.standard_normal((2, H, W, 64)).astype(np.float32)
        x[0, 1] = x[0, 1, 0]                  # a row of identical tokens
        x[1, :, 1] = x[1, 0, 1]               # a column of identical tokens
        x[1, 2, W // 2] = 0.0
        sizes = rng.integers(1, 4, (2, H, W))
        run_wide(oracle, wl.cast_io(x, dtype), dtype, passes, radius, tag="close calls")
        run_wide(oracle, wl.cast_io(x, dtype), dtype, passes, radius, sizes=sizes, tag="close calls+sizes")


def test_wide_determinism():
    rng = np.random.default_rng(43)
    x = to_dev(wl.cast_io(wl.smooth_field(rng, 2, 40, 36, 136, 2.0) + 0.05 * rng.standard_normal((2, 40, 36, 136)).astype(np.float32), "bf16"), "bf16")
    passes = [(W_AX, 2), (H_AX, 2)] * 2
    a = lv.luvc_oim_merge_wide(x, passes, 0)
    for _ in range(3):
        b = lv.luvc_oim_merge_wide(x, passes, 0)
        torch.cuda.synchronize()
        for k in ("x", "sizes", "merged_map", "kept_map"):
            assert torch.equal(a[k], b[k]), k

"""GPU parity: luvc_oim_merge (through the C ABI) against the CPU oracle, element by element."""
import numpy as np
import pytest
import torch

from paper_2512_09010_amd import binding as lv
from paper_2512_09010_amd import workloads as wl
from gpu_util import OIM_MARGIN, RTOL, assert_close, oim_reference, round_mode, to_dev, to_host_f64

pytestmark = pytest.mark.gpu
W_AX, H_AX = 1, 0


def run_case(oracle, x_io, dtype, passes, sizes=None, tag=""):
    print(f"[oim] {tag} shape={x_io.shape} dtype={dtype} passes={passes}", flush=True)
    s_dev = None if sizes is None else torch.from_numpy(np.ascontiguousarray(sizes, dtype=np.int32)).cuda()
    out = lv.luvc_oim_merge(to_dev(x_io, dtype), passes, sizes=s_dev)
    torch.cuda.synchronize()
    # the oracle; where one of its decisions is closer than fp64 can resolve, the alternative the GPU took is
    # accepted there if it is within OIM_MARGIN of the best one (gpu_util.oim_reference)
    ref = oim_reference(oracle, wl.widen(x_io, dtype), passes, out["merged_map"].cpu().numpy(), dtype, sizes=sizes)
    assert out["x"].shape == ref["x"].shape
    np.testing.assert_array_equal(out["sizes"].cpu().numpy().astype(np.int64), ref["sizes"])
    np.testing.assert_array_equal(out["merged_map"].cpu().numpy(), ref["merged_map"])
    np.testing.assert_array_equal(out["kept_map"].cpu().numpy(), ref["kept_map"])
    got = to_host_f64(out["x"])
    assert_close(got, ref["x"], RTOL[dtype], f"{tag} features")
    if dtype == "bf16":
        # the merge is evaluated in fp64 and rounded once, so bf16 outputs agree to the bit
        np.testing.assert_array_equal(got, ref["x"])
    return out, ref


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("B,H,W,D,passes", [
    (1, 1, 2, 8, [(W_AX, 1)]),
    (1, 2, 1, 8, [(H_AX, 1)]),
    (2, 5, 7, 24, [(W_AX, 4)]),
    (2, 5, 7, 24, [(H_AX, 3)]),
    (2, 6, 9, 40, [(W_AX, 2), (H_AX, 2)]),               # the paper's merge number 2
    (1, 9, 6, 40, [(H_AX, 2), (W_AX, 2)]),
    (3, 8, 8, 64, [(W_AX, 4), (H_AX, 4)]),
    (1, 16, 16, 72, [(W_AX, 2), (H_AX, 2), (W_AX, 2), (H_AX, 2), (W_AX, 2), (H_AX, 2)]),   # three OIM operations
    (2, 4, 4, 33, [(W_AX, 1), (H_AX, 0)]),               # D that defeats 16-byte rows, m = 0 pass
    (1, 3, 300, 16, [(W_AX, 37)]),                        # a line longer than the workgroup
    (1, 300, 2, 16, [(H_AX, 150)]),
    (2, 7, 11, 520, [(W_AX, 6), (H_AX, 4)]),             # several 16-byte chunks per lane + ragged tail
])
def test_small_random(oracle, dtype, B, H, W, D, passes):
    rng = np.random.default_rng(B * 1000 + H * 100 + W * 10 + D)
    x = wl.cast_io(rng.standard_normal((B, H, W, D)).astype(np.float32), dtype)
    run_case(oracle, x, dtype, passes, tag="random")
    sizes = rng.integers(1, 6, (B, H, W))
    run_case(oracle, x, dtype, passes, sizes=sizes, tag="random+sizes")


def _halving(H, W, order):
    """Schedule of halving passes: order is a string of 'W' / 'H'."""
    passes = []
    for ax in order:
        if ax == "W":
            passes.append((W_AX, (W + 1) // 2)); W -= (W + 1) // 2
        else:
            passes.append((H_AX, (H + 1) // 2)); H -= (H + 1) // 2
    return passes


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("B,H,W,D,order", [
    (2, 2, 2, 16, "WH"),          # smallest pair
    (2, 8, 8, 64, "WH"),
    (2, 8, 8, 64, "HW"),          # Algorithm 1 order: height first
    (1, 9, 7, 40, "WH"),          # odd lengths on both axes: the last source of a line has one neighbour
    (1, 7, 9, 40, "HW"),
    (1, 3, 2, 24, "WH"),
    (2, 12, 10, 520, "WH"),       # several 16-byte chunks per lane, ragged last chunk
    (1, 70, 6, 48, "WH"),         # second-pass lines longer than one workgroup: runs with recomputed rows around them
    (1, 6, 70, 48, "HW"),
    (1, 131, 4, 32, "WH"),        # three runs, odd length
    (1, 16, 16, 72, "WHWH"),      # two pairs in one call: maps compose
    (1, 16, 12, 72, "HWHW"),
    (1, 16, 16, 72, "WHW"),       # a pair followed by a single pass
    (1, 12, 12, 1024, "WH"),      # four chunks per lane (fp32 at D=1024 is the single-image configuration)
    (2, 32, 48, 72, "WWHW"),      # a single pass, then a fused pair, then a single pass: intermediates alternate per launch
    (2, 48, 32, 72, "HHWH"),
    (1, 32, 32, 64, "WWHHW"),
])
def test_halving_pairs(oracle, dtype, B, H, W, D, order):
    rng = np.random.default_rng(B * 1000 + H * 100 + W * 10 + D + len(order))
    x = wl.cast_io(wl.smooth_field(rng, B, H, W, D, 2.0) + 0.1 * rng.standard_normal((B, H, W, D)).astype(np.float32), dtype)
    passes = _halving(H, W, order)
    run_case(oracle, x, dtype, passes, tag="pair smooth")
    sizes = rng.integers(1, 6, (B, H, W))
    run_case(oracle, x, dtype, passes, sizes=sizes, tag="pair smooth+sizes")
    xr = wl.cast_io(rng.standard_normal((B, H, W, D)).astype(np.float32), dtype)
    run_case(oracle, xr, dtype, passes, sizes=sizes, tag="pair random+sizes")


def test_pair_without_maps(oracle):
    # the maps are optional outputs: a call that asks for neither still produces the same tokens
    rng = np.random.default_rng(11)
    x = wl.cast_io(wl.smooth_field(rng, 2, 8, 8, 64, 2.0), "bf16")
    passes = _halving(8, 8, "WH")
    ref = oracle.oim_merge(wl.widen(x, "bf16"), passes, round_mode=round_mode(oracle, "bf16"))
    out = lv.luvc_oim_merge(to_dev(x, "bf16"), passes, want_maps=False)
    torch.cuda.synchronize()
    np.testing.assert_array_equal(to_host_f64(out["x"]), ref["x"])
    np.testing.assert_array_equal(out["sizes"].cpu().numpy().astype(np.int64), ref["sizes"])


def test_pair_tiny_values(oracle):
    # a sprinkle of values around and below the smallest normal bf16 / fp32-exact magnitudes: merged
    # results in the subnormal range must still be the correctly rounded ones
    rng = np.random.default_rng(17)
    x = wl.smooth_field(rng, 1, 8, 8, 256, 2.0)
    tiny = rng.random(x.shape) < 0.05
    x[tiny] *= np.float32(1e-38)
    x[rng.random(x.shape) < 0.01] = 0.0
    sizes = rng.integers(1, 4, (1, 8, 8))
    for dtype in ("bf16", "f32"):
        run_case(oracle, wl.cast_io(x, dtype), dtype, _halving(8, 8, "WH"), tag="tiny values")
        run_case(oracle, wl.cast_io(x, dtype), dtype, _halving(8, 8, "WH"), sizes=sizes, tag="tiny values+sizes")


def test_pair_close_calls(oracle):
    # rows of near-duplicate tokens: most cosines differ by less than the fp32 screening bound, so the
    # fp64 repeat of both passes decides; exact duplicates tie and go to the lower position
    rng = np.random.default_rng(13)
    base = rng.standard_normal((1, 1, 1, 256)).astype(np.float32)
    x = base + 1e-3 * rng.standard_normal((2, 12, 12, 256)).astype(np.float32)
    x[0, 3] = x[0, 3, 0]          # a row of identical tokens
    x[1, :, 5] = x[1, 0, 5]       # a column of identical tokens
    for dtype in ("bf16", "f32"):
        for order in ("WH", "HW"):
            run_case(oracle, wl.cast_io(x, dtype), dtype, _halving(12, 12, order), tag="close calls " + order)


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_smooth_field_general_m(oracle, dtype):
    rng = np.random.default_rng(77)
    x = wl.cast_io(wl.smooth_field(rng, 2, 12, 14, 96, 2.0), dtype)
    for passes in ([(W_AX, 3), (H_AX, 3)], [(W_AX, 7), (H_AX, 6)], [(H_AX, 1), (W_AX, 5)]):
        run_case(oracle, x, dtype, passes, tag="smooth")


def test_degenerate_inputs(oracle):
    # identical tokens: every cosine ties at 1 -> lower position wins everywhere; zero tokens: clamped norms
    v = np.random.default_rng(5).standard_normal(32).astype(np.float32)
    x = np.broadcast_to(v, (1, 6, 6, 32)).copy()
    out, ref = run_case(oracle, wl.cast_io(x, "bf16"), "bf16", [(W_AX, 3), (H_AX, 3)], tag="constant")
    assert out["sizes"].sum().item() == 36
    z = np.zeros((1, 4, 6, 16), np.float32)
    run_case(oracle, z, "f32", [(W_AX, 2)], tag="zeros")


@pytest.mark.parametrize("i", [0, 1, 2, 3, 4])
def test_mini_workloads(oracle, i):
    w = wl.mini(i)
    x = wl.oim_input(w)
    cur, sizes = x, None
    for call in w.oim_calls:
        out, ref = run_case(oracle, cur, w.dtype, call, sizes=sizes, tag=w.name)
        # chain the next call on the oracle's output so both sides keep reading identical bits
        cur = wl.cast_io(ref["x"].astype(np.float32), w.dtype)
        sizes = ref["sizes"]


def test_determinism(oracle):
    w = wl.mini(1)
    x = to_dev(wl.oim_input(w), w.dtype)
    a = lv.luvc_oim_merge(x, w.oim_calls[0])
    b = lv.luvc_oim_merge(x, w.oim_calls[0])
    torch.cuda.synchronize()
    for k in ("x", "sizes", "merged_map", "kept_map"):
        assert torch.equal(a[k].view(torch.uint8) if a[k].dtype == torch.bfloat16 else a[k],
                           b[k].view(torch.uint8) if b[k].dtype == torch.bfloat16 else b[k]), k


@pytest.mark.parametrize("seed", range(24))
def test_random_schedules(oracle, seed):
    """Seeded random grids and schedules (any axis order, m from 0 to a full halving, up to six passes), so that every
    mix of the single-pass, fused-pair and general launches and every hand-over between them is met."""
    rng = np.random.default_rng(1000 + seed)
    dtype = "bf16" if seed % 2 else "f32"
    B, H, W = int(rng.integers(1, 4)), int(rng.integers(1, 40)), int(rng.integers(1, 40))
    D = int(rng.choice([8, 24, 33, 64, 72, 136]))
    passes, h, w = [], H, W
    for _ in range(int(rng.integers(1, 7))):
        axis = int(rng.integers(0, 2))
        length = w if axis else h
        if length == 1:
            m = 0
        else:
            kind = rng.integers(0, 3)
            m = (length + 1) // 2 if kind == 0 else int(rng.integers(0, (length + 1) // 2 + 1))
            m = min(m, length - 1)
        passes.append((axis, m))
        if axis:
            w -= m
        else:
            h -= m
    x = wl.cast_io(wl.smooth_field(rng, B, H, W, D, 2.0) + 0.2 * rng.standard_normal((B, H, W, D)).astype(np.float32), dtype)
    sizes = rng.integers(1, 4, (B, H, W)) if seed % 3 == 0 else None
    run_case(oracle, x, dtype, passes, sizes=sizes, tag=f"fuzz{seed}")


def test_pair_merge_near_a_rounding_tie(oracle):
    """A three-token merge whose mean sits on a bf16 rounding boundary except for a term 2^-24 times smaller: the
    intermediate token of the fused pair must be rounded from the exact fp64 mean, once (an fp32 stop on the way
    would swallow the small term and resolve the tie the other way)."""
    D = 64
    rng = np.random.default_rng(12)
    x = (0.05 * rng.standard_normal((1, 3, 2, D))).astype(np.float32)
    sizes = np.ones((1, 3, 2), np.int64)
    sizes[0, 1, :] = 2                                   # the destination row counts double: S = 4 per column
    a, b = -0.197265625, -0.380859375                    # (a + 2 b) / 4 = -245.5 * 2^-10: a tie at bf16 resolution
    for ch in range(32):
        scale = 2.0 ** (ch % 7 - 3)
        sign = -1.0 if ch & 8 else 1.0
        nudge = (1.0 if ch & 16 else -1.0) * 2.0 ** -26   # pushes the mean off the tie, towards or away from "even"
        x[0, 0, 0, ch], x[0, 1, 0, ch], x[0, 2, 0, ch] = sign * a * scale, sign * b * scale, nudge * scale
        x[0, :, 1, ch] = 0.01 * scale                     # the neighbour the W pass merges it with: small, so one unit shows
    x_io = wl.cast_io(x, "bf16")
    np.testing.assert_array_equal(wl.widen(x_io, "bf16")[0, :, 0, :32], x[0, :, 0, :32])      # all chosen values are bf16 values
    run_case(oracle, x_io, "bf16", [(H_AX, 2)], sizes=sizes, tag="tie+tiny H (single halving pass)")
    run_case(oracle, np.concatenate([x_io, x_io], axis=1), "bf16", [(H_AX, 2)], sizes=np.concatenate([sizes, sizes], axis=1),
             tag="tie+tiny H (general pass: two of three sources)")
    run_case(oracle, x_io, "bf16", [(H_AX, 2), (W_AX, 1)], sizes=sizes, tag="tie+tiny HW")
    xt = np.ascontiguousarray(x_io.transpose(0, 2, 1, 3))
    run_case(oracle, xt, "bf16", [(W_AX, 2), (H_AX, 1)], sizes=np.ascontiguousarray(sizes.transpose(0, 2, 1)), tag="tie+tiny WH")


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_large_sizes(oracle, dtype):
    """Sizes far beyond anything a merge schedule produces (up to 10^6 per token; sums stay below 2^31): the fp64
    weighted mean stays exact in its products and must still match bit for bit (bf16) / to 1e-5 (fp32)."""
    rng = np.random.default_rng(21)
    B, H, W, D = 2, 10, 12, 72
    x = wl.cast_io(wl.smooth_field(rng, B, H, W, D, 2.0) + 0.1 * rng.standard_normal((B, H, W, D)).astype(np.float32), dtype)
    sizes = rng.integers(1, 10 ** 6, (B, H, W))
    run_case(oracle, x, dtype, [(W_AX, 6), (H_AX, 5)], sizes=sizes, tag="large sizes pair")
    run_case(oracle, x, dtype, [(W_AX, 2), (H_AX, 2), (W_AX, 2)], sizes=sizes, tag="large sizes m=2")
    run_case(oracle, x, dtype, [(H_AX, 5)], sizes=sizes, tag="large sizes single")


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_decisions_closer_than_the_arithmetic_resolves(oracle, dtype):
    """Destinations that are scaled copies of each other: a source between them sees two cosines that are equal in exact
    arithmetic and differ, if at all, in the last bit of an fp64 evaluation.  The oracle's margin is then tiny without
    being zero, the GPU's operation order may resolve such a decision the other way, and the comparison has to accept
    that alternative (and nothing else)."""
    rng = np.random.default_rng(31)
    B, H, W, D = 2, 8, 10, 64
    x = rng.standard_normal((B, H, W, D)).astype(np.float32)
    x = (x.view(np.uint32) & np.uint32(0xFFF00000)).view(np.float32).copy()   # 4 significant bits: times 15 is still a bf16 value
    x[:, :, 3] = 3 * x[:, :, 1]                                              # destination 3 of every row is a multiple of destination 1
    x[:, :, 7] = 3 * x[:, :, 5]
    x[:, 5] = 5 * x[:, 3]                                                    # and row 5 a multiple of row 3
    x_io = wl.cast_io(x, dtype)
    np.testing.assert_array_equal(wl.widen(x_io, dtype), x)
    margins = []
    for passes in ([(W_AX, 5)], [(W_AX, 5), (H_AX, 4)], [(H_AX, 4), (W_AX, 5)], [(W_AX, 2), (H_AX, 2)], [(H_AX, 3)]):
        run_case(oracle, x_io, dtype, passes, tag="scaled copies")
        margins.append(oracle.oim_merge(wl.widen(x_io, dtype), passes, round_mode=round_mode(oracle, dtype))["margin"])
    assert min(margins) <= OIM_MARGIN                                       # the case does visit the situation it is written for


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("exp2", [-63, -40, 55, 63])
def test_extreme_magnitudes(oracle, dtype, exp2):
    """Features scaled by 2^-63 (~1e-19), 2^-40, 2^55 and 2^63 (~1e19): fp32 squared norms underflow, lose terms or
    overflow there, so the fp32 screening must abstain and the fp64 values decide - through the fused pair kernel,
    the single halving pass and the general path (m = 2)."""
    rng = np.random.default_rng(1000 + exp2)
    x = (rng.standard_normal((2, 8, 10, 96)) * 2.0 ** exp2).astype(np.float32)
    x_io = wl.cast_io(x, dtype)
    for passes in (_halving(8, 10, "WH"), _halving(8, 10, "HW"), [(W_AX, 5)], [(H_AX, 4)], [(W_AX, 2), (H_AX, 2)]):
        run_case(oracle, x_io, dtype, passes, tag=f"scaled 2^{exp2}")
    # one image of ordinary magnitude beside a tiny and a huge one, and zero tokens in between
    y = rng.standard_normal((3, 8, 10, 96)).astype(np.float32)
    y[1] *= 2.0 ** exp2
    y[2, :, 3:5] = 0.0
    run_case(oracle, wl.cast_io(y, dtype), dtype, _halving(8, 10, "WH"), tag=f"mixed 2^{exp2}")


def test_packed_bf16_dot_rounds_like_the_screening_bound_assumes():
    """The error bound of the fp32 screening takes every step acc <- acc + x0 y0 + x1 y1 of the packed bf16 dot product
    as at most two roundings to nearest (relative 2^-24 each) of partial sums bounded by the sum of the magnitudes of
    the terms.  Held here against exact sums (fp64 is exact for products of bf16 values and sums of 40 of them over
    this range) on random rows, rows with cancellation and rows of one sign."""
    rng = np.random.default_rng(5)
    rows, words = 4096, 20
    xs = [rng.standard_normal((rows, 2 * words)), np.abs(rng.standard_normal((rows, 2 * words))),
          rng.standard_normal((rows, 2 * words)) * np.exp2(rng.integers(-8, 8, (rows, 2 * words)))]
    ys = [rng.standard_normal((rows, 2 * words)), np.abs(rng.standard_normal((rows, 2 * words))),
          rng.standard_normal((rows, 2 * words))]
    for x, y in zip(xs, ys):
        xb, yb = wl.cast_io(x.astype(np.float32), "bf16"), wl.cast_io(y.astype(np.float32), "bf16")
        got = lv.luvc_selftest_fdot2(to_dev(xb, "bf16"), to_dev(yb, "bf16")).cpu().numpy().astype(np.float64)
        xe, ye = wl.widen(xb, "bf16"), wl.widen(yb, "bf16")
        exact = (xe * ye).sum(axis=1)
        mag = np.abs(xe * ye).sum(axis=1)
        bound = 2 * words * 2.0 ** -24 * mag
        assert (np.abs(got - exact) <= bound).all(), float((np.abs(got - exact) / bound).max())
        print(f"[fdot2] worst error / bound = {float((np.abs(got - exact) / bound).max()):.3f}", flush=True)

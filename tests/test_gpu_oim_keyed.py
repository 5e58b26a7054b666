"""GPU parity: luvc_oim_merge_keyed (decisions on the keys, merge applied to the tokens; Section 3.1 counts the
similarity in "the dimension of keys") and luvc_value_enhance (Eq. 3, V + log s) against the CPU oracle."""
import numpy as np
import pytest
import torch

from paper_2512_09010_amd import binding as lv
from paper_2512_09010_amd import workloads as wl
from gpu_util import OIM_MARGIN, RTOL, assert_close, oim_reference, round_mode, to_dev, to_host_f64

pytestmark = pytest.mark.gpu
W_AX, H_AX = 1, 0


def run_keyed(oracle, x_io, k_io, dtype, passes, radius, sizes=None, tag=""):
    print(f"[oim keyed] {tag} x={x_io.shape} keys={k_io.shape} dtype={dtype} passes={passes} radius={radius}", flush=True)
    s_dev = None if sizes is None else torch.from_numpy(np.ascontiguousarray(sizes, dtype=np.int32)).cuda()
    out = lv.luvc_oim_merge_keyed(to_dev(x_io, dtype), to_dev(k_io, dtype), passes, radius, sizes=s_dev)
    torch.cuda.synchronize()
    ref = oim_reference(oracle, wl.widen(x_io, dtype), passes, out["merged_map"].cpu().numpy(), dtype, sizes=sizes, R=radius,
                        metric=wl.widen(k_io, dtype))
    np.testing.assert_array_equal(out["sizes"].cpu().numpy().astype(np.int64), ref["sizes"])
    np.testing.assert_array_equal(out["merged_map"].cpu().numpy(), ref["merged_map"])
    np.testing.assert_array_equal(out["kept_map"].cpu().numpy(), ref["kept_map"])
    for name in ("x", "metric"):
        got = to_host_f64(out[name])
        assert_close(got, ref[name], RTOL[dtype], f"{tag} {name}")
        if dtype == "bf16":
            np.testing.assert_array_equal(got, ref[name])
    return out, ref


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("radius", [1, 0, 2])
@pytest.mark.parametrize("B,H,W,D,Dm,passes", [
    (1, 1, 3, 8, 8, [(W_AX, 1)]),
    (2, 6, 9, 40, 16, [(W_AX, 2), (H_AX, 2)]),                  # merge number 2, keys narrower than the tokens
    (1, 9, 6, 24, 64, [(H_AX, 2), (W_AX, 2), (H_AX, 1)]),       # keys wider than the tokens, three passes
    (2, 4, 5, 33, 7, [(W_AX, 3), (H_AX, 0)]),                   # rows that are not 16-byte multiples, m = 0 pass
    (1, 12, 12, 520, 72, [(W_AX, 6), (H_AX, 6)]),               # halving passes on the general kernels
])
def test_keyed_small_random(oracle, dtype, radius, B, H, W, D, Dm, passes):
    rng = np.random.default_rng(B * 1000 + H * 100 + W * 10 + D + Dm + radius)
    x = wl.cast_io(rng.standard_normal((B, H, W, D)).astype(np.float32), dtype)
    keys = wl.cast_io(rng.standard_normal((B, H, W, Dm)).astype(np.float32), dtype)
    run_keyed(oracle, x, keys, dtype, passes, radius, tag="random")
    sizes = rng.integers(1, 6, (B, H, W))
    run_keyed(oracle, x, keys, dtype, passes, radius, sizes=sizes, tag="random+sizes")


def test_keyed_with_the_tokens_as_keys_is_the_plain_call():
    rng = np.random.default_rng(17)
    x = to_dev(wl.cast_io(wl.smooth_field(rng, 2, 8, 10, 64, 2.0) + 0.1 * rng.standard_normal((2, 8, 10, 64)).astype(np.float32), "bf16"), "bf16")
    passes = [(W_AX, 2), (H_AX, 2)]
    for radius in (1, 0):
        a = lv.luvc_oim_merge_keyed(x, x, passes, radius)
        b = lv.luvc_oim_merge_wide(x, passes, radius)
        torch.cuda.synchronize()
        for k in ("x", "sizes", "merged_map", "kept_map"):
            assert torch.equal(a[k], b[k]), (radius, k)
        assert torch.equal(a["metric"], a["x"])


def test_keyed_without_metric_output(oracle):
    rng = np.random.default_rng(18)
    x = wl.cast_io(rng.standard_normal((1, 6, 6, 32)).astype(np.float32), "bf16")
    keys = wl.cast_io(rng.standard_normal((1, 6, 6, 16)).astype(np.float32), "bf16")
    passes = [(W_AX, 2), (H_AX, 2)]
    ref = oracle.oim_merge_keyed(wl.widen(x, "bf16"), wl.widen(keys, "bf16"), passes, R=0, round_mode=oracle.ROUND_BF16)
    out = lv.luvc_oim_merge_keyed(to_dev(x, "bf16"), to_dev(keys, "bf16"), passes, 0, want_metric=False, want_maps=False)
    torch.cuda.synchronize()
    assert out["metric"] is None
    np.testing.assert_array_equal(to_host_f64(out["x"]), ref["x"])


def _halving(H, W, order):
    passes = []
    for ax in order:
        if ax == "W":
            passes.append((W_AX, (W + 1) // 2)); W -= (W + 1) // 2
        else:
            passes.append((H_AX, (H + 1) // 2)); H -= (H + 1) // 2
    return passes


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("B,H,W,D,Dm,order", [
    (2, 2, 2, 16, 8, "WH"),            # smallest pair
    (2, 8, 8, 64, 32, "WH"),
    (2, 8, 8, 64, 128, "HW"),          # Algorithm 1 order: height first; keys wider than the tokens
    (1, 9, 7, 40, 24, "WH"),           # odd lengths on both axes
    (1, 7, 9, 40, 24, "HW"),
    (1, 3, 2, 24, 16, "WH"),
    (2, 12, 10, 520, 72, "WH"),        # ragged last piece of a token and of a key
    (1, 70, 6, 48, 16, "WH"),          # second-pass lines cut into runs: rows outside a run are looked at for decisions only
    (1, 6, 70, 48, 136, "HW"),
    (1, 131, 4, 32, 64, "WH"),         # three runs, odd length
    (1, 24, 24, 1280, 128, "WH"),      # the token width of the batch workloads, keys of one attention head
    (1, 12, 12, 2048, 256, "HW"),      # largest token, eight wavefronts per workgroup
    (1, 12, 12, 640, 512, "WH"),       # largest key in bf16 (1 KB); in fp32 it is beyond the fused kernel: general kernels
    (1, 16, 16, 72, 40, "WHWH"),       # two pairs in one call: maps compose, the second pair decides on the merged keys
    (1, 16, 16, 72, 40, "WHW"),        # a pair followed by a single pass on the general kernels
    (2, 32, 24, 72, 40, "WWHW"),       # single, pair, single: intermediates alternate per launch
])
def test_keyed_halving_pairs(oracle, dtype, B, H, W, D, Dm, order):
    rng = np.random.default_rng(B * 1000 + H * 100 + W * 10 + D + Dm + len(order))
    x = wl.cast_io(rng.standard_normal((B, H, W, D)).astype(np.float32), dtype)
    keys = wl.cast_io(wl.smooth_field(rng, B, H, W, Dm, 2.0) + 0.1 * rng.standard_normal((B, H, W, Dm)).astype(np.float32), dtype)
    passes = _halving(H, W, order)
    run_keyed(oracle, x, keys, dtype, passes, 1, tag="pair smooth keys")
    sizes = rng.integers(1, 6, (B, H, W))
    run_keyed(oracle, x, keys, dtype, passes, 1, sizes=sizes, tag="pair smooth keys+sizes")
    kr = wl.cast_io(rng.standard_normal((B, H, W, Dm)).astype(np.float32), dtype)
    run_keyed(oracle, x, kr, dtype, passes, 1, sizes=sizes, tag="pair random keys+sizes")


def test_keyed_pair_with_the_tokens_as_keys_is_the_plain_call():
    # both kernels decide on fp64 cosines (the plain one wherever its fp32 screening is unsure); their sums run in
    # different orders, which only a decision closer than 1e-15 could notice - these inputs have none
    rng = np.random.default_rng(19)
    for (B, H, W, D, order) in ((2, 16, 16, 128, "WH"), (1, 70, 10, 256, "HW"), (1, 13, 11, 512, "WHWH")):
        x = to_dev(wl.cast_io(wl.smooth_field(rng, B, H, W, D, 2.0) + 0.1 * rng.standard_normal((B, H, W, D)).astype(np.float32), "bf16"), "bf16")
        passes = _halving(H, W, order)
        a = lv.luvc_oim_merge_keyed(x, x, passes, 1)
        b = lv.luvc_oim_merge(x, passes)
        torch.cuda.synchronize()
        for k in ("x", "sizes", "merged_map", "kept_map"):
            assert torch.equal(a[k], b[k]), (H, W, D, order, k)
        assert torch.equal(a["metric"], a["x"])


def test_keyed_pair_close_calls_and_degenerate_keys(oracle):
    # near-duplicate keys (cosines closer than fp32 resolves), rows and columns of identical keys (ties go to the
    # lower position), zero keys (cosine through the norm clamp)
    rng = np.random.default_rng(23)
    base = rng.standard_normal((1, 1, 1, 64)).astype(np.float32)
    keys = base + 1e-3 * rng.standard_normal((2, 12, 12, 64)).astype(np.float32)
    keys[0, 3] = keys[0, 3, 0]
    keys[1, :, 5] = keys[1, 0, 5]
    keys[1, 7, 2:6] = 0.0
    x = rng.standard_normal((2, 12, 12, 96)).astype(np.float32)
    for dtype in ("bf16", "f32"):
        for order in ("WH", "HW"):
            run_keyed(oracle, wl.cast_io(x, dtype), wl.cast_io(keys, dtype), dtype, _halving(12, 12, order), 1, tag="close calls " + order)


def test_keyed_pair_without_metric_and_maps(oracle):
    rng = np.random.default_rng(29)
    x = wl.cast_io(rng.standard_normal((2, 10, 12, 64)).astype(np.float32), "bf16")
    keys = wl.cast_io(rng.standard_normal((2, 10, 12, 32)).astype(np.float32), "bf16")
    passes = _halving(10, 12, "HW")
    ref = oracle.oim_merge_keyed(wl.widen(x, "bf16"), wl.widen(keys, "bf16"), passes, R=1, round_mode=oracle.ROUND_BF16)
    assert ref["margin"] > OIM_MARGIN
    out = lv.luvc_oim_merge_keyed(to_dev(x, "bf16"), to_dev(keys, "bf16"), passes, 1, want_metric=False, want_maps=False)
    torch.cuda.synchronize()
    assert out["metric"] is None
    np.testing.assert_array_equal(to_host_f64(out["x"]), ref["x"])
    np.testing.assert_array_equal(out["sizes"].cpu().numpy().astype(np.int64), ref["sizes"])


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("B,H,W,D,Dm,passes,radius", [
    (2, 24, 20, 136, 64, [(W_AX, 2), (H_AX, 2)] * 3, 0),        # the appendix setting on the keys: whole line, merge number 2, three operations
    (1, 40, 36, 72, 128, [(H_AX, 5), (W_AX, 18), (H_AX, 1)], 2),
    (1, 3, 128, 32, 16, [(W_AX, 64)], 0),                        # longest line of the one-launch passes, every source merged
    (1, 2, 140, 32, 16, [(W_AX, 3)], 0),                         # beyond it: three launches per pass and tensor
])
def test_keyed_wide_matching(oracle, dtype, B, H, W, D, Dm, passes, radius):
    rng = np.random.default_rng(B * 1000 + H * 100 + W * 10 + D + Dm + radius)
    x = wl.cast_io(rng.standard_normal((B, H, W, D)).astype(np.float32), dtype)
    keys = wl.cast_io(wl.smooth_field(rng, B, H, W, Dm, 2.0) + 0.2 * rng.standard_normal((B, H, W, Dm)).astype(np.float32), dtype)
    run_keyed(oracle, x, keys, dtype, passes, radius, tag="wide keys")
    sizes = rng.integers(1, 5, (B, H, W))
    run_keyed(oracle, x, keys, dtype, passes, radius, sizes=sizes, tag="wide keys+sizes")


def test_keyed_wide_one_launch_passes_and_three_launch_passes_agree():
    """The same keyed call on 16-byte aligned keys (row ids between the passes, one launch per pass) and on a copy of the
    keys that starts 8 bytes off (every pass materialised, four launches per pass): identical outputs."""
    rng = np.random.default_rng(47)
    B, H, W, D, Dm = 2, 20, 24, 72, 40
    x = torch.from_numpy(rng.standard_normal((B, H, W, D)).astype(np.float32)).to(torch.bfloat16).cuda()
    k = torch.from_numpy(wl.smooth_field(rng, B, H, W, Dm, 2.0) + 0.2 * rng.standard_normal((B, H, W, Dm)).astype(np.float32)).to(torch.bfloat16).cuda()
    flat = torch.empty(k.numel() + 4, dtype=torch.bfloat16, device="cuda")
    flat[4:] = k.reshape(-1)
    k_off = flat[4:].view(B, H, W, Dm)
    assert k.data_ptr() % 16 == 0 and k_off.data_ptr() % 16 == 8
    passes = [(W_AX, 2), (H_AX, 2)] * 2
    a = lv.luvc_oim_merge_keyed(x, k, passes, 0)
    b = lv.luvc_oim_merge_keyed(x, k_off, passes, 0)
    c = lv.luvc_oim_merge_keyed(x, k, passes, 0, want_metric=False, want_maps=False)
    torch.cuda.synchronize()
    for key in ("x", "metric", "sizes", "merged_map", "kept_map"):
        assert torch.equal(a[key], b[key]), key
    assert torch.equal(a["x"], c["x"]) and torch.equal(a["sizes"], c["sizes"]) and c["metric"] is None


@pytest.mark.parametrize("dtype,shape", [("f32", (3, 7, 33)), ("bf16", (2, 64, 1280)), ("bf16", (5, 3, 10)), ("f32", (1, 19, 256))])
def test_value_enhance(oracle, dtype, shape):
    rng = np.random.default_rng(sum(shape))
    v = wl.cast_io(rng.standard_normal(shape).astype(np.float32), dtype)
    sizes = rng.integers(1, 40, shape[:-1])
    sizes.flat[0] = 1
    ref = oracle.value_enhance(wl.widen(v, dtype), sizes, round_mode=round_mode(oracle, dtype))
    out = lv.luvc_value_enhance(to_dev(v, dtype), torch.from_numpy(sizes.astype(np.int32)).cuda())
    torch.cuda.synchronize()
    got = to_host_f64(out)
    # the sum is formed in fp64 and rounded once on both sides; the two logarithms may differ in their last fp64 bit,
    # which can only move a result that sits on a rounding boundary: one unit of the storage type at most
    ulp = 2.0 ** -7 if dtype == "bf16" else 2.0 ** -23
    assert (np.abs(got - ref) <= ulp * np.abs(ref)).all()
    assert (got == ref).mean() > 0.999
    np.testing.assert_array_equal(got.reshape(-1, shape[-1])[0], wl.widen(v, dtype).reshape(-1, shape[-1])[0])     # s = 1: untouched


@pytest.mark.parametrize("block", range(6))
def test_keyed_and_wide_calls_on_seeded_random_cases(oracle, block):
    """Seeded random grids, schedules (halving or any m), radii and key widths through luvc_oim_merge_keyed: every code path
    behind it (fused pair kernel, one-launch wide passes, separate stages), with noisy, near-duplicate and constant keys."""
    for seed in range(10 * block, 10 * block + 10):
        rng = np.random.default_rng(70000 + seed)
        dtype = "bf16" if seed % 2 else "f32"
        radius = int(rng.choice([0, 0, 1, 1, 2, 3]))
        B, H, W = int(rng.integers(1, 3)), int(rng.integers(1, 36)), int(rng.integers(1, 36))
        D, Dm = int(rng.choice([8, 16, 24, 64, 136, 520])), int(rng.choice([8, 16, 40, 64, 128]))
        halving = bool(rng.integers(0, 2))
        passes, h, w = [], H, W
        for _ in range(int(rng.integers(1, 5))):
            axis = int(rng.integers(0, 2))
            length = w if axis else h
            if halving:
                m = (length + 1) // 2 if length > 1 else 0
            else:
                m = 0 if length == 1 else min(int(rng.integers(0, (length + 1) // 2 + 1)), length - 1)
            passes.append((axis, m))
            if axis:
                w -= m
            else:
                h -= m
        kind = int(rng.integers(0, 3))                      # noisy keys, near-duplicate keys, constant keys (every decision a tie)
        x = wl.cast_io(wl.smooth_field(rng, B, H, W, D, 2.0) + 0.3 * rng.standard_normal((B, H, W, D)).astype(np.float32), dtype)
        keys = wl.smooth_field(rng, B, H, W, Dm, 2.0) * (0.0 if kind == 2 else 1.0) + 1.0 + [0.3, 1e-3, 0.0][kind] * rng.standard_normal((B, H, W, Dm)).astype(np.float32)
        sizes = rng.integers(1, 4, (B, H, W)) if seed % 3 == 0 else None
        run_keyed(oracle, x, wl.cast_io(keys.astype(np.float32), dtype), dtype, passes, radius, sizes=sizes, tag=f"fuzz{seed} kind{kind}")

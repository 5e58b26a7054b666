"""GPU parity: ragged batches (luvc_oim_merge_ragged, luvc_oim_plan_anyres, luvc_spu_stage_ragged through the C ABI)
against the CPU oracle, item by item: every image / sample of a packed batch must come out exactly as the oracle
computes it on its own."""
import numpy as np
import pytest
import torch

from paper_2512_09010_amd import binding as lv
from paper_2512_09010_amd import workloads as wl
from gpu_util import OIM_MARGIN, RTOL, SPU_MARGIN, assert_close, round_mode, to_dev, to_host_f64

pytestmark = pytest.mark.gpu


def oim_ragged_case(oracle, shapes, D, dtype, max_tokens, seed, with_sizes):
    rng = np.random.default_rng(seed)
    schedules = [lv.luvc_oim_plan_anyres(h, w, max_tokens) for h, w in shapes]
    for (h, w), sch in zip(shapes, schedules):
        assert sch == oracle.plan_anyres(h, w, max_tokens), (h, w)
    imgs = [wl.cast_io(wl.smooth_field(rng, 1, h, w, D, 2.0) + 0.1 * rng.standard_normal((1, h, w, D)).astype(np.float32), dtype)
            for h, w in shapes]
    sizes = [rng.integers(1, 5, (1, h, w)) for h, w in shapes] if with_sizes else None
    print(f"[ragged oim] shapes={shapes} D={D} dtype={dtype} cap={max_tokens} sizes={with_sizes}", flush=True)
    packed = np.concatenate([a.reshape(-1, D) for a in imgs])
    s_dev = None
    if with_sizes:
        s_dev = torch.from_numpy(np.concatenate([s.reshape(-1) for s in sizes]).astype(np.int32)).cuda()
    out = lv.luvc_oim_merge_ragged(to_dev(packed, dtype), shapes, schedules, sizes=s_dev)
    torch.cuda.synchronize()
    gx, gs = to_host_f64(out["x"]), out["sizes"].cpu().numpy().astype(np.int64)
    gm, gk = out["merged_map"].cpu().numpy(), out["kept_map"].cpu().numpy()
    ti = to = 0
    for i, ((h, w), sch) in enumerate(zip(shapes, schedules)):
        ref = oracle.oim_merge(wl.widen(imgs[i], dtype), sch, sizes=None if sizes is None else sizes[i], round_mode=round_mode(oracle, dtype))
        ho, wo = out["out_shapes"][i]
        assert ref["x"].shape == (1, ho, wo, D)
        assert ref["margin"] > OIM_MARGIN or ref["margin"] == 0.0, (i, ref["margin"])
        n_in, n_out = h * w, ho * wo
        np.testing.assert_array_equal(gs[to:to + n_out], ref["sizes"].reshape(-1))
        np.testing.assert_array_equal(gm[ti:ti + n_in], ref["merged_map"].reshape(-1))
        np.testing.assert_array_equal(gk[to:to + n_out], ref["kept_map"].reshape(-1))
        assert_close(gx[to:to + n_out], ref["x"].reshape(n_out, D), RTOL[dtype], f"image {i}")
        if dtype == "bf16":
            np.testing.assert_array_equal(gx[to:to + n_out], ref["x"].reshape(n_out, D))
        ti += n_in
        to += n_out
    assert ti == packed.shape[0] and to == gx.shape[0]


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_oim_anyres_batch(oracle, dtype):
    # wide, tall and square images; equal neighbours form runs of 2 and 3; one image is within the budget already
    shapes = [(16, 48), (16, 48), (40, 12), (24, 24), (24, 24), (24, 24), (8, 8), (9, 31), (1, 70)]
    oim_ragged_case(oracle, shapes, 64, dtype, 144, 1, with_sizes=False)
    oim_ragged_case(oracle, shapes, 72, dtype, 64, 2, with_sizes=True)


def test_oim_ragged_explicit_schedules(oracle):
    """Schedules that differ on equal shapes split a run; the paper's merge number 2 on both axes."""
    rng = np.random.default_rng(3)
    shapes = [(10, 12), (10, 12), (10, 12), (6, 6)]
    schedules = [[(1, 2), (0, 2)], [(1, 2), (0, 2)], [(0, 2), (1, 2), (0, 2)], [(1, 3)]]
    D, dtype = 40, "bf16"
    imgs = [wl.cast_io(rng.standard_normal((1, h, w, D)).astype(np.float32), dtype) for h, w in shapes]
    packed = np.concatenate([a.reshape(-1, D) for a in imgs])
    out = lv.luvc_oim_merge_ragged(to_dev(packed, dtype), shapes, schedules)
    torch.cuda.synchronize()
    gx = to_host_f64(out["x"])
    to = 0
    for i, sch in enumerate(schedules):
        ref = oracle.oim_merge(wl.widen(imgs[i], dtype), sch, round_mode=round_mode(oracle, dtype))
        n_out = ref["x"].shape[1] * ref["x"].shape[2]
        assert ref["margin"] > OIM_MARGIN
        np.testing.assert_array_equal(gx[to:to + n_out], ref["x"].reshape(n_out, D))
        to += n_out
    assert to == gx.shape[0]


def spu_ragged_case(oracle, lengths, D, dtype, ratio, seed, origin_shift=None):
    rng = np.random.default_rng(seed)
    sigmas = [max(1, int(ratio * n / 2)) if n > 1 else 0 for n in lengths]
    keeps = [lv.luvc_keep_count(n, ratio) for n in lengths]
    xs = [wl.cast_io((rng.standard_normal((1, n, D)) + np.sin(np.arange(n) / 5.0)[None, :, None] * rng.standard_normal((1, 1, D))).astype(np.float32), dtype)
          for n in lengths]
    print(f"[ragged spu] lengths={lengths} D={D} dtype={dtype} keeps={keeps}", flush=True)
    packed = np.concatenate([a.reshape(-1, D) for a in xs])
    org = None
    if origin_shift is not None:
        org = torch.from_numpy(np.concatenate([np.arange(n, dtype=np.int32) * 2 + origin_shift for n in lengths])).cuda()
    out = lv.luvc_spu_stage_ragged(to_dev(packed, dtype), lengths, sigmas, keeps, origin=org)
    torch.cuda.synchronize()
    gsc = out["scores"].cpu().numpy().astype(np.float64)
    gk, go, gx = out["kept_idx"].cpu().numpy(), out["origin"].cpu().numpy(), to_host_f64(out["x"])
    ti = to = 0
    for i, n in enumerate(lengths):
        o_in = None if origin_shift is None else (np.arange(n, dtype=np.int32) * 2 + origin_shift)[None, :]
        ref = oracle.spu_stage(wl.widen(xs[i], dtype), sigmas[i], keeps[i], True, o_in)
        floor = 1e-6 * np.abs(ref["scores"]).max()
        assert (np.abs(gsc[ti:ti + n] - ref["scores"][0]) <= 1e-5 * np.abs(ref["scores"][0]) + floor).all(), i
        assert ref["margin"] > SPU_MARGIN, (i, ref["margin"])
        k = keeps[i]
        np.testing.assert_array_equal(gk[to:to + k], ref["kept_idx"][0])
        np.testing.assert_array_equal(go[to:to + k], ref["origin"][0])
        np.testing.assert_array_equal(gx[to:to + k], ref["x"][0])
        ti += n
        to += k
    assert ti == packed.shape[0] and to == gk.shape[0]
    # scores only
    sc_only = lv.luvc_spu_stage_ragged(to_dev(packed, dtype), lengths, sigmas, None)
    torch.cuda.synchronize()
    np.testing.assert_array_equal(sc_only["scores"].cpu().numpy(), out["scores"].cpu().numpy())


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_spu_ragged_batch(oracle, dtype):
    # lengths on the fft path (1024, 720, 256), the fused direct path (196, 64) and the general path (300, 97, 1); runs of 2
    lengths = [1024, 1024, 720, 196, 196, 300, 64, 97, 256, 1]
    spu_ragged_case(oracle, lengths, 96, dtype, 0.25, 4)
    spu_ragged_case(oracle, lengths[2:], 70, dtype, 0.1, 5, origin_shift=7)


def test_ragged_errors():
    x = torch.zeros((20, 8), device="cuda")
    with pytest.raises(lv.LuvcError):
        lv.luvc_spu_stage_ragged(x, [12, 8], [7, 1], [3, 3])                   # sigma > N/2 in the first sample
    with pytest.raises(lv.LuvcError):
        lv.luvc_spu_stage_ragged(x, [12, 8], [2, 1], [3, 9])                   # keep > N in the second sample
    with pytest.raises(lv.LuvcError):
        lv.luvc_oim_merge_ragged(x, [(2, 5), (2, 5)], [[(1, 2)], [(1, 4)]])    # m too large for the second image
    with pytest.raises(lv.LuvcError):
        lv.luvc_oim_plan_anyres(0, 4, 10)

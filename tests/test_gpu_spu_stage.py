"""GPU parity: luvc_spu_stage / luvc_spu_cascade_keeps (through the C ABI) against the CPU oracle.

A cascade is run stage by stage.  Between two stages stands a synthetic "LLM layer" (channel mixing and a
tanh, computed on the host in fp64 and rounded to the I/O dtype) whose output is handed to BOTH sides, so every
stage is compared on identical inputs and the origins are compared after composition over all stages."""
import numpy as np
import pytest
import torch

from paper_2512_09010_amd import binding as lv
from paper_2512_09010_amd import workloads as wl
from gpu_util import SPU_MARGIN, to_dev, to_host_f64

pytestmark = pytest.mark.gpu
SCORE_RTOL = 1e-5


def run_cascade(oracle, x0, dtype, keeps, sigmas, ham, tag):
    rng = np.random.default_rng(11)
    B, N, D = x0.shape
    mix = rng.standard_normal((D, D)) / np.sqrt(D)
    x_io, org_ref, org_dev = x0, None, None
    for stage, (k, sg) in enumerate(zip(keeps, sigmas)):
        print(f"[stage] {tag} stage={stage} x={x_io.shape} dtype={dtype} sigma={sg} keep={k}", flush=True)
        ref = oracle.spu_stage(wl.widen(x_io, dtype), sg, k, ham, org_ref)
        xd = to_dev(x_io, dtype)
        got = lv.luvc_spu_stage(xd, sg, k, ham, origin=org_dev)
        torch.cuda.synchronize()
        if k == 0:
            assert got["kept_idx"].shape == (B, 0) and got["origin"].shape == (B, 0) and got["x"].shape == (B, 0, D)
            return
        g = got["scores"].cpu().numpy().astype(np.float64)
        floor = 1e-6 * np.abs(ref["scores"]).max()
        assert (np.abs(g - ref["scores"]) <= SCORE_RTOL * np.abs(ref["scores"]) + floor).all(), (tag, stage)
        assert ref["margin"] > SPU_MARGIN, (tag, stage, ref["margin"])   # the keep set is unique at fp32 accuracy
        np.testing.assert_array_equal(got["kept_idx"].cpu().numpy(), ref["kept_idx"])
        np.testing.assert_array_equal(got["origin"].cpu().numpy(), ref["origin"])
        np.testing.assert_array_equal(to_host_f64(got["x"]), ref["x"])   # the original rows, bit for bit
        # the "layer": same values for both sides
        x_io = wl.cast_io(np.tanh(ref["x"] @ mix).astype(np.float32), dtype)
        org_ref, org_dev = ref["origin"], got["origin"]
    assert (np.diff(org_ref, axis=1) > 0).all() and org_ref.min() >= 0 and org_ref.max() < N


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
@pytest.mark.parametrize("B,N,D,ratio,stages", [
    (2, 1024, 96, 0.5, 4),        # 1024 -> 512 -> 256 (fft path) -> 128 -> 0
    (3, 720, 70, 0.3, 3),         # 720 (Q = 15) -> 216 -> 65 (direct path) -> 0
    (1, 5000, 40, 0.25, 3),       # above the single-launch prune limit: select + gather launches
    (2, 37, 9, 0.6, 3),
])
def test_cascade_random(oracle, dtype, B, N, D, ratio, stages):
    rng = np.random.default_rng(N + D)
    x0 = wl.cast_io((rng.standard_normal((B, N, D)) + 2.0 * np.sin(np.arange(N) / 9.0)[None, :, None] * rng.standard_normal((B, 1, D))).astype(np.float32), dtype)
    keeps = lv.luvc_spu_cascade_keeps(N, ratio, stages)
    assert keeps == oracle.cascade_keeps(N, ratio, stages) and keeps[-1] == 0
    alive = [N] + keeps[:-1]
    sigmas = [max(1, n // 10) for n in alive]
    run_cascade(oracle, x0, dtype, keeps, sigmas, True, f"random-{N}")


def test_cascade_workload_shape(oracle):
    """Three stages that start from the SPU input of the small benchmark workload (same recipe, same sigma rule)."""
    w = wl.mini(1)
    x0 = wl.spu_input(w)
    keeps = lv.luvc_spu_cascade_keeps(w.spu_N, 0.4, 3, eliminate=False)
    sigmas = [max(1, n // 10) for n in [w.spu_N] + keeps[:-1]]
    run_cascade(oracle, x0, "bf16", keeps, sigmas, True, "mini1")


def test_keeps_schedule_and_errors():
    assert lv.luvc_spu_cascade_keeps(1024, 0.2, 3) == [205, 41, 0]
    assert lv.luvc_spu_cascade_keeps(1024, 0.2, 3, eliminate=False) == [205, 41, 8]
    with pytest.raises(lv.LuvcError):
        lv.luvc_spu_cascade_keeps(0, 0.2, 3)
    with pytest.raises(lv.LuvcError):
        lv.luvc_spu_cascade_keeps(16, 1.5, 3)
    x = torch.zeros((1, 8, 4), device="cuda")
    with pytest.raises(lv.LuvcError):
        lv.luvc_spu_stage(x, 2, 9)                       # n_keep > N
    with pytest.raises(lv.LuvcError):
        lv.luvc_spu_stage(x, 5, 3)                       # sigma > N/2

"""GPU: luvc_spu_score_static (scratch in a static device array, no allocation) against luvc_spu_score, through the
C ABI: two calls in a row on the one array, the second smaller than the first, then a third on another kernel path."""
import numpy as np
import pytest
import torch

from paper_2512_09010_amd import binding as lv
from paper_2512_09010_amd import workloads as wl
from gpu_util import to_dev

pytestmark = pytest.mark.gpu


def _x(seed, B, N, D, dtype):
    rng = np.random.default_rng(seed)
    return to_dev(wl.cast_io(rng.standard_normal((B, N, D)).astype(np.float32), dtype), dtype)


def test_static_scratch_matches_the_workspace_call():
    cases = [(4, 1024, 512, "bf16", 102),      # fft path: 16 channel tiles per sample, two tile groups
             (2, 720, 200, "f32", 54),         # smaller, right after it, on the same array: 16 x 15 transform, ragged last tile
             (3, 196, 256, "bf16", 4),         # direct pass-band transform in one launch
             (2, 50, 96, "f32", 25),           # three-launch path (tables and spectra in the scratch as well)
             (4, 1024, 512, "bf16", 102)]      # the first shape again, after the others have left their traces
    for i, (B, N, D, dtype, sigma) in enumerate(cases):
        print(f"[static] call {i}: B={B} N={N} D={D} {dtype} sigma={sigma}", flush=True)
        x = _x(40 + i, B, N, D, dtype)
        need = lv.luvc_spu_workspace_bytes(B, N, D, lv.LUVC_BF16 if dtype == "bf16" else lv.LUVC_F32, sigma)
        assert 0 < need <= lv.SPU_STATIC_SCRATCH_BYTES
        out = torch.full((B, N), -1.0, dtype=torch.float32, device="cuda")
        got = lv.luvc_spu_score_static(x, sigma, True, out=out)
        want = lv.luvc_spu_score(x, sigma, True)
        torch.cuda.synchronize()
        assert torch.equal(got, want), f"call {i}: scores differ from luvc_spu_score"
        assert bool((got >= 0).all())


def test_static_scratch_rejects_what_does_not_fit():
    B, N, D, sigma = 40, 2048, 4096, 102
    assert lv.luvc_spu_workspace_bytes(B, N, D, lv.LUVC_BF16, sigma) > lv.SPU_STATIC_SCRATCH_BYTES
    x = torch.empty((B, N, D), dtype=torch.bfloat16, device="cuda")       # never read: both calls fail their checks
    with pytest.raises(lv.LuvcError) as e:
        lv.luvc_spu_score_static(x, sigma, True)
    assert e.value.status == lv.LUVC_ERR_WORKSPACE and "static buffer holds" in str(e.value)
    with pytest.raises(lv.LuvcError) as e:
        lv.luvc_spu_score_static(x, N, True)                # sigma beyond N/2: rejected by the argument checks
    assert e.value.status == lv.LUVC_ERR_INVALID_ARG

"""Helpers for the GPU parity tests: numpy <-> device marshalling and the comparison rules."""
import numpy as np
import torch

from paper_2512_09010_amd import workloads as wl

# Tolerances of the parity bar: relative, per element, on values stored in the I/O dtype.
RTOL = {"f32": 1e-5, "bf16": 2e-2}
OIM_MARGIN = 1e-10      # fp64-accumulated cosines: below this gap a decision may legitimately differ
SPU_MARGIN = 2e-6       # relative gap of fp32 scores at the keep boundary (measured score error <= 1.3e-7, bound ~1e-6)


def to_dev(a: np.ndarray, dtype: str) -> torch.Tensor:
    if dtype == "bf16":
        return torch.from_numpy(np.ascontiguousarray(a).view(np.int16)).view(torch.bfloat16).cuda()
    return torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).cuda()


def to_host_f64(t: torch.Tensor) -> np.ndarray:
    if t.dtype == torch.bfloat16:
        bits = t.contiguous().view(torch.int16).cpu().numpy().view(np.uint16)
        return wl.bf16_bits_to_f32(bits).astype(np.float64)
    return t.cpu().numpy().astype(np.float64)


def round_mode(orc, dtype):
    return orc.ROUND_BF16 if dtype == "bf16" else orc.ROUND_F32


def assert_close(got, want, rtol, what=""):
    got, want = np.asarray(got, np.float64), np.asarray(want, np.float64)
    assert got.shape == want.shape, (what, got.shape, want.shape)
    err = np.abs(got - want)
    bound = rtol * np.abs(want) + 1e-30
    bad = err > bound
    if bad.any():
        i = np.unravel_index(np.argmax(err - bound), err.shape)
        raise AssertionError(f"{what}: {bad.sum()} of {bad.size} elements off; worst at {i}: got {got[i]!r} want {want[i]!r}")


def oim_reference(orc, x64, passes, gpu_merged_map, dtype, sizes=None, R=1, metric=None):
    """What the GPU's OIM outputs are compared with: the oracle's result - unless the GPU's map differs from it AND some
    decision of the oracle is closer than OIM_MARGIN, i.e. closer than fp64 arithmetic in another operation order can
    resolve.  Then the reference is the oracle's method with, at those decisions only, the alternative the GPU's map
    shows, provided it is within OIM_MARGIN of the best one (tests/oim_replay.py; alternatives with identical bits stay
    bound to the lower-position rule).  Any other difference still fails the comparison that follows."""
    rm = round_mode(orc, dtype)
    if metric is None:
        ref = orc.oim_merge(x64, passes, sizes=sizes, R=R, round_mode=rm)
    else:
        ref = orc.oim_merge_keyed(x64, metric, passes, sizes=sizes, R=R, round_mode=rm)
    gpu_map = np.asarray(gpu_merged_map).reshape(ref["merged_map"].shape)
    if ref["margin"] > OIM_MARGIN or np.array_equal(gpu_map, ref["merged_map"]):
        return ref
    from oim_replay import replay
    alt = replay(orc, x64, passes, gpu_map, sizes=sizes, R=R, round_mode=rm, eps=OIM_MARGIN, metric=metric)
    print(f"[oim] decision margin {ref['margin']:.3e} <= {OIM_MARGIN} and the maps differ in "
          f"{int((gpu_map != ref['merged_map']).sum())} entries: {alt['close']} close decisions follow the GPU's map "
          f"where it is within the tolerance", flush=True)
    return alt

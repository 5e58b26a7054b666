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

"""ctypes binding over ``libluvc.so`` - same names as the C ABI in ``include/luvc.h``.

Argument marshalling only: every step of OIM and SPU runs in the HIP kernels.  PyTorch is used
for device memory (tensors own the buffers) and for the current stream handle.  There is no
CPU fallback: if the library is missing or cannot be loaded, importing callers get an error.
"""
from __future__ import annotations

import ctypes
import os
from typing import List, Optional, Sequence, Tuple

_HERE = os.path.dirname(os.path.abspath(__file__))
# LUVC_HOST_SANITIZE=1 loads the build whose host code carries the sanitizers (see build.py)
LIB_PATH = os.path.join(_HERE, "libluvc_san.so" if os.environ.get("LUVC_HOST_SANITIZE", "") not in ("", "0") else "libluvc.so")

LUVC_OK, LUVC_ERR_INVALID_ARG, LUVC_ERR_UNSUPPORTED, LUVC_ERR_WORKSPACE, LUVC_ERR_HIP = range(5)
LUVC_F32, LUVC_BF16 = 0, 1

EXPORTS = ("luvc_version", "luvc_last_error", "luvc_oim_plan", "luvc_oim_workspace_bytes", "luvc_oim_merge",
           "luvc_oim_wide_workspace_bytes", "luvc_oim_merge_wide",
           "luvc_oim_keyed_workspace_bytes", "luvc_oim_merge_keyed", "luvc_value_enhance", "luvc_spu_workspace_bytes", "luvc_spu_score", "luvc_spu_score_static", "luvc_keep_count", "luvc_spu_prune",
           "luvc_spu_cascade_keeps", "luvc_spu_stage",
           "luvc_oim_plan_anyres", "luvc_oim_ragged_workspace_bytes", "luvc_oim_merge_ragged",
           "luvc_spu_ragged_workspace_bytes", "luvc_spu_stage_ragged",
           "luvc_profile_start", "luvc_profile_stop", "luvc_profile_kernel", "luvc_selftest_fdot2", "luvc_selftest_screen_tile")


class LuvcPass(ctypes.Structure):
    _fields_ = [("axis", ctypes.c_int32), ("m", ctypes.c_int32)]


class LuvcError(RuntimeError):
    def __init__(self, status: int, text: str):
        super().__init__(f"libluvc status {status}: {text}")
        self.status = status


_lib = None


def lib() -> ctypes.CDLL:
    """Load libluvc.so (built beforehand by ``paper_2512_09010_amd.build``); raises if it is absent."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise FileNotFoundError(f"{LIB_PATH} is not built; run `python -m paper_2512_09010_amd.build` "
                                "(there is no fallback implementation)")
    L = ctypes.CDLL(LIB_PATH)
    i, i64, vp, sz = ctypes.c_int, ctypes.c_int64, ctypes.c_void_p, ctypes.c_size_t
    pp = ctypes.POINTER(LuvcPass)
    L.luvc_version.restype = ctypes.c_char_p
    L.luvc_last_error.restype = ctypes.c_char_p
    L.luvc_oim_plan.argtypes = [i, i, i64, pp, i, ctypes.POINTER(i)]
    L.luvc_oim_plan.restype = i
    L.luvc_oim_workspace_bytes.argtypes = [i, i, i, i, i, pp, i]
    L.luvc_oim_workspace_bytes.restype = sz
    L.luvc_oim_merge.argtypes = [vp, vp, i, i, i, i, i, pp, i, i64, vp, vp, vp, vp, vp, sz, vp]
    L.luvc_oim_merge.restype = i
    L.luvc_oim_wide_workspace_bytes.argtypes = [i, i, i, i, i, pp, i, i]
    L.luvc_oim_wide_workspace_bytes.restype = sz
    L.luvc_oim_merge_wide.argtypes = [vp, vp, i, i, i, i, i, pp, i, i, i64, vp, vp, vp, vp, vp, sz, vp]
    L.luvc_oim_merge_wide.restype = i
    L.luvc_oim_keyed_workspace_bytes.argtypes = [i, i, i, i, i, i, pp, i, i]
    L.luvc_oim_keyed_workspace_bytes.restype = sz
    L.luvc_oim_merge_keyed.argtypes = [vp, vp, vp, i, i, i, i, i, i, pp, i, i, i64, vp, vp, vp, vp, vp, vp, sz, vp]
    L.luvc_oim_merge_keyed.restype = i
    L.luvc_value_enhance.argtypes = [vp, vp, i64, i, i64, i, vp, i64, vp]
    L.luvc_value_enhance.restype = i
    L.luvc_spu_workspace_bytes.argtypes = [i, i, i, i, i]
    L.luvc_spu_workspace_bytes.restype = sz
    L.luvc_spu_score.argtypes = [vp, i, i, i, i64, i, i, i, vp, vp, sz, vp]
    L.luvc_spu_score.restype = i
    L.luvc_spu_score_static.argtypes = [vp, i, i, i, i64, i, i, i, vp, vp]
    L.luvc_spu_score_static.restype = i
    L.luvc_keep_count.argtypes = [i, ctypes.c_double]
    L.luvc_keep_count.restype = i
    L.luvc_spu_prune.argtypes = [vp, vp, i, i, i, i64, i, i, vp, vp, vp, sz, vp]
    L.luvc_spu_prune.restype = i
    L.luvc_spu_cascade_keeps.argtypes = [i, ctypes.c_double, i, i, ctypes.POINTER(ctypes.c_int)]
    L.luvc_spu_cascade_keeps.restype = i
    L.luvc_spu_stage.argtypes = [vp, i, i, i, i64, i, i, i, i, vp, vp, vp, vp, vp, vp, sz, vp]
    L.luvc_spu_stage.restype = i
    ip = ctypes.POINTER(ctypes.c_int32)
    L.luvc_oim_plan_anyres.argtypes = [i, i, i64, pp, i, ctypes.POINTER(ctypes.c_int)]
    L.luvc_oim_plan_anyres.restype = i
    L.luvc_oim_ragged_workspace_bytes.argtypes = [i, ip, ip, i, i, pp, ip]
    L.luvc_oim_ragged_workspace_bytes.restype = sz
    L.luvc_oim_merge_ragged.argtypes = [vp, vp, i, ip, ip, i, i, pp, ip, vp, vp, vp, vp, vp, sz, vp]
    L.luvc_oim_merge_ragged.restype = i
    L.luvc_spu_ragged_workspace_bytes.argtypes = [i, ip, i, i, ip]
    L.luvc_spu_ragged_workspace_bytes.restype = sz
    L.luvc_spu_stage_ragged.argtypes = [vp, i, ip, i, i64, i, ip, i, ip, vp, vp, vp, vp, vp, vp, sz, vp]
    L.luvc_spu_stage_ragged.restype = i
    L.luvc_profile_start.argtypes = [ctypes.POINTER(vp), i]
    L.luvc_profile_start.restype = i
    L.luvc_profile_stop.argtypes = []
    L.luvc_profile_stop.restype = i
    L.luvc_profile_kernel.argtypes = [i]
    L.luvc_profile_kernel.restype = ctypes.c_char_p
    L.luvc_selftest_fdot2.argtypes = [vp, vp, i, i, vp, vp]
    L.luvc_selftest_fdot2.restype = i
    L.luvc_selftest_screen_tile.argtypes = [vp, vp, i, i, vp, vp]
    L.luvc_selftest_screen_tile.restype = i
    _lib = L
    return L


def last_error() -> str:
    return lib().luvc_last_error().decode()


def _check(status: int):
    if status != LUVC_OK:
        raise LuvcError(status, last_error())


def _passes(passes: Sequence[Tuple[int, int]]):
    arr = (LuvcPass * max(1, len(passes)))()
    for k, (axis, m) in enumerate(passes):
        arr[k].axis, arr[k].m = int(axis), int(m)
    return arr


def _dtype_code(t) -> int:
    import torch
    if t.dtype == torch.float32:
        return LUVC_F32
    if t.dtype == torch.bfloat16:
        return LUVC_BF16
    raise TypeError(f"unsupported dtype {t.dtype}")


def _stream(stream) -> int:
    import torch
    s = stream if stream is not None else torch.cuda.current_stream()
    return int(s.cuda_stream)


def _ptr(t) -> Optional[int]:
    return None if t is None else int(t.data_ptr())


def luvc_version() -> str:
    return lib().luvc_version().decode()


def luvc_keep_count(N: int, keep_ratio: float) -> int:
    return lib().luvc_keep_count(int(N), float(keep_ratio))


def luvc_oim_plan(H: int, W: int, target_tokens: int, max_passes: int = 16) -> List[Tuple[int, int]]:
    arr = (LuvcPass * max_passes)()
    n = ctypes.c_int(0)
    _check(lib().luvc_oim_plan(H, W, int(target_tokens), arr, max_passes, ctypes.byref(n)))
    return [(arr[k].axis, arr[k].m) for k in range(n.value)]


def luvc_oim_workspace_bytes(B, H, W, D, dtype_code, passes) -> int:
    return lib().luvc_oim_workspace_bytes(B, H, W, D, dtype_code, _passes(passes), len(passes))


def out_grid(H: int, W: int, passes) -> Tuple[int, int]:
    for axis, m in passes:
        if axis == 1:
            W -= m
        else:
            H -= m
    return H, W


def luvc_oim_merge(x, passes, sizes=None, target_tokens: int = 0, want_maps: bool = True, workspace=None, stream=None,
                   out=None):
    """x: CUDA tensor [B,H,W,D] (fp32 or bf16, contiguous).  Returns dict(x, sizes, merged_map, kept_map)."""
    import torch
    assert x.is_cuda and x.is_contiguous() and x.dim() == 4
    B, H, W, D = x.shape
    code = _dtype_code(x)
    parr = _passes(passes)
    Ho, Wo = out_grid(H, W, passes)
    need = lib().luvc_oim_workspace_bytes(B, H, W, D, code, parr, len(passes))
    if workspace is None:
        workspace = torch.empty(max(need, 256), dtype=torch.uint8, device=x.device)
    if out is None:
        out = dict(
            x=torch.empty((B, max(Ho, 0), max(Wo, 0), D), dtype=x.dtype, device=x.device),
            sizes=torch.empty((B, max(Ho, 0), max(Wo, 0)), dtype=torch.int32, device=x.device),
            merged_map=torch.empty((B, H * W), dtype=torch.int32, device=x.device) if want_maps else None,
            kept_map=torch.empty((B, max(Ho, 0) * max(Wo, 0)), dtype=torch.int32, device=x.device) if want_maps else None,
        )
    if sizes is not None:
        assert sizes.is_cuda and sizes.dtype == torch.int32 and sizes.is_contiguous() and sizes.numel() == B * H * W
    _check(lib().luvc_oim_merge(_ptr(x), _ptr(sizes), B, H, W, D, code, parr, len(passes), int(target_tokens),
                                _ptr(out["x"]), _ptr(out["sizes"]), _ptr(out.get("merged_map")), _ptr(out.get("kept_map")),
                                _ptr(workspace), workspace.numel(), _stream(stream)))
    return out


def luvc_oim_wide_workspace_bytes(B, H, W, D, dtype_code, passes, radius) -> int:
    return lib().luvc_oim_wide_workspace_bytes(B, H, W, D, dtype_code, _passes(passes), len(passes), int(radius))


def luvc_oim_merge_wide(x, passes, radius: int, sizes=None, target_tokens: int = 0, want_maps: bool = True, workspace=None,
                        stream=None, out=None):
    """As luvc_oim_merge with candidates within `radius` (0 = the whole line).  Returns dict(x, sizes, merged_map, kept_map)."""
    import torch
    assert x.is_cuda and x.is_contiguous() and x.dim() == 4
    B, H, W, D = x.shape
    code = _dtype_code(x)
    parr = _passes(passes)
    Ho, Wo = out_grid(H, W, passes)
    need = lib().luvc_oim_wide_workspace_bytes(B, H, W, D, code, parr, len(passes), int(radius))
    if workspace is None:
        workspace = torch.empty(max(need, 256), dtype=torch.uint8, device=x.device)
    if out is None:
        out = dict(
            x=torch.empty((B, max(Ho, 0), max(Wo, 0), D), dtype=x.dtype, device=x.device),
            sizes=torch.empty((B, max(Ho, 0), max(Wo, 0)), dtype=torch.int32, device=x.device),
            merged_map=torch.empty((B, H * W), dtype=torch.int32, device=x.device) if want_maps else None,
            kept_map=torch.empty((B, max(Ho, 0) * max(Wo, 0)), dtype=torch.int32, device=x.device) if want_maps else None,
        )
    if sizes is not None:
        assert sizes.is_cuda and sizes.dtype == torch.int32 and sizes.is_contiguous() and sizes.numel() == B * H * W
    _check(lib().luvc_oim_merge_wide(_ptr(x), _ptr(sizes), B, H, W, D, code, parr, len(passes), int(radius), int(target_tokens),
                                     _ptr(out["x"]), _ptr(out["sizes"]), _ptr(out.get("merged_map")), _ptr(out.get("kept_map")),
                                     _ptr(workspace), workspace.numel(), _stream(stream)))
    return out


def luvc_oim_keyed_workspace_bytes(B, H, W, D, Dm, dtype_code, passes, radius) -> int:
    return lib().luvc_oim_keyed_workspace_bytes(B, H, W, D, Dm, dtype_code, _passes(passes), len(passes), int(radius))


def luvc_oim_merge_keyed(x, metric, passes, radius: int = 1, sizes=None, target_tokens: int = 0, want_maps: bool = True,
                         want_metric: bool = True, workspace=None, stream=None, out=None):
    """Decisions on metric [B,H,W,Dm], merge applied to x [B,H,W,D].  Returns dict(x, metric, sizes, merged_map, kept_map)."""
    import torch
    assert x.is_cuda and x.is_contiguous() and x.dim() == 4 and metric.is_cuda and metric.is_contiguous() and metric.dim() == 4
    assert metric.shape[:3] == x.shape[:3] and metric.dtype == x.dtype
    B, H, W, D = x.shape
    Dm = metric.shape[3]
    code = _dtype_code(x)
    parr = _passes(passes)
    Ho, Wo = out_grid(H, W, passes)
    need = lib().luvc_oim_keyed_workspace_bytes(B, H, W, D, Dm, code, parr, len(passes), int(radius))
    if workspace is None:
        workspace = torch.empty(max(need, 256), dtype=torch.uint8, device=x.device)
    if out is None:
        out = dict(
            x=torch.empty((B, max(Ho, 0), max(Wo, 0), D), dtype=x.dtype, device=x.device),
            metric=torch.empty((B, max(Ho, 0), max(Wo, 0), Dm), dtype=x.dtype, device=x.device) if want_metric else None,
            sizes=torch.empty((B, max(Ho, 0), max(Wo, 0)), dtype=torch.int32, device=x.device),
            merged_map=torch.empty((B, H * W), dtype=torch.int32, device=x.device) if want_maps else None,
            kept_map=torch.empty((B, max(Ho, 0) * max(Wo, 0)), dtype=torch.int32, device=x.device) if want_maps else None,
        )
    if sizes is not None:
        assert sizes.is_cuda and sizes.dtype == torch.int32 and sizes.is_contiguous() and sizes.numel() == B * H * W
    _check(lib().luvc_oim_merge_keyed(_ptr(x), _ptr(metric), _ptr(sizes), B, H, W, D, Dm, code, parr, len(passes), int(radius),
                                      int(target_tokens), _ptr(out["x"]), _ptr(out.get("metric")), _ptr(out["sizes"]),
                                      _ptr(out.get("merged_map")), _ptr(out.get("kept_map")),
                                      _ptr(workspace), workspace.numel(), _stream(stream)))
    return out


def luvc_value_enhance(v, sizes, stream=None, out=None):
    """v: CUDA tensor [..., D] (last dim contiguous, rows evenly strided), sizes int32 [...]: returns v + log(sizes)."""
    import torch
    assert v.is_cuda and v.stride(-1) == 1 and sizes.is_cuda and sizes.dtype == torch.int32 and sizes.is_contiguous()
    D = v.shape[-1]
    rows = sizes.numel()
    assert v.numel() == rows * D and v.is_contiguous()
    if out is None:
        out = torch.empty_like(v)
    _check(lib().luvc_value_enhance(_ptr(v), _ptr(sizes), rows, D, D, _dtype_code(v), _ptr(out), D, _stream(stream)))
    return out


def luvc_spu_workspace_bytes(B, N, D, dtype_code, sigma) -> int:
    return lib().luvc_spu_workspace_bytes(B, N, D, dtype_code, sigma)


def luvc_spu_score(x, sigma: int, use_hamming: bool = True, workspace=None, stream=None, out=None):
    """x: CUDA tensor [B,N,D] (last dim contiguous; token stride may exceed D).  Returns scores [B,N] fp32."""
    import torch
    assert x.is_cuda and x.dim() == 3 and x.stride(2) == 1 and x.stride(0) == x.shape[1] * x.stride(1)
    B, N, D = x.shape
    code = _dtype_code(x)
    need = lib().luvc_spu_workspace_bytes(B, N, D, code, int(sigma))
    if workspace is None:
        workspace = torch.empty(max(need, 256), dtype=torch.uint8, device=x.device)
    if out is None:
        out = torch.empty((B, N), dtype=torch.float32, device=x.device)
    _check(lib().luvc_spu_score(_ptr(x), B, N, D, x.stride(1), code, int(sigma), int(bool(use_hamming)), _ptr(out),
                                _ptr(workspace), workspace.numel(), _stream(stream)))
    return out


SPU_STATIC_SCRATCH_BYTES = 8 << 20


def luvc_spu_score_static(x, sigma: int, use_hamming: bool = True, stream=None, out=None):
    """luvc_spu_score on the library's static scratch (no workspace; pass `out` to keep the call free of allocations)."""
    import torch
    assert x.is_cuda and x.dim() == 3 and x.stride(2) == 1 and x.stride(0) == x.shape[1] * x.stride(1)
    B, N, D = x.shape
    if out is None:
        out = torch.empty((B, N), dtype=torch.float32, device=x.device)
    _check(lib().luvc_spu_score_static(_ptr(x), B, N, D, x.stride(1), _dtype_code(x), int(sigma), int(bool(use_hamming)),
                                       _ptr(out), _stream(stream)))
    return out


def luvc_spu_prune(x, scores, n_keep: int, gather: bool = True, stream=None, out=None):
    """Returns dict(kept_idx [B,n_keep] int32 ascending, x [B,n_keep,D] or None)."""
    import torch
    assert scores.is_cuda and scores.dtype == torch.float32 and scores.is_contiguous() and scores.dim() == 2
    B, N = scores.shape
    D, stride, code, xp = 1, 1, LUVC_F32, None
    if x is not None:
        assert x.is_cuda and x.dim() == 3 and x.stride(2) == 1 and x.shape[:2] == scores.shape
        D, stride, code, xp = x.shape[2], x.stride(1), _dtype_code(x), _ptr(x)
    if out is None:
        out = dict(kept_idx=torch.empty((B, max(n_keep, 0)), dtype=torch.int32, device=scores.device),
                   x=torch.empty((B, max(n_keep, 0), D), dtype=x.dtype, device=x.device) if (gather and x is not None) else None)
    _check(lib().luvc_spu_prune(xp, _ptr(scores), B, N, D, stride, code, int(n_keep), _ptr(out["kept_idx"]),
                                _ptr(out.get("x")), None, 0, _stream(stream)))
    return out


def luvc_spu_cascade_keeps(N0: int, keep_ratio: float, n_stages: int, eliminate: bool = True):
    """Keep counts of the stages of a cascade: one keep ratio stage after stage, 0 at the end when eliminate."""
    keeps = (ctypes.c_int * max(int(n_stages), 1))()
    n = lib().luvc_spu_cascade_keeps(int(N0), float(keep_ratio), int(n_stages), int(bool(eliminate)), keeps)
    if n != n_stages or n_stages < 1:
        raise LuvcError(LUVC_ERR_INVALID_ARG, "luvc_spu_cascade_keeps rejected its arguments")
    return [int(k) for k in keeps[:n]]


def luvc_spu_stage(x, sigma: int, n_keep: int, use_hamming: bool = True, origin=None, gather: bool = True,
                   workspace=None, stream=None, out=None):
    """One cascade stage on x [B,N,D].  Returns dict(scores [B,N] fp32, kept_idx, origin [B,n_keep] int32,
    x [B,n_keep,D] or None); with n_keep = 0 nothing is launched and the tensors are empty."""
    import torch
    assert x.is_cuda and x.dim() == 3 and x.stride(2) == 1 and x.stride(0) == x.shape[1] * x.stride(1)
    B, N, D = x.shape
    code = _dtype_code(x)
    if origin is not None:
        assert origin.is_cuda and origin.dtype == torch.int32 and origin.is_contiguous() and tuple(origin.shape) == (B, N)
    k = max(int(n_keep), 0)
    if workspace is None:
        need = lib().luvc_spu_workspace_bytes(B, N, D, code, int(sigma)) if k else 0
        workspace = torch.empty(max(need, 256), dtype=torch.uint8, device=x.device)
    if out is None:
        out = dict(scores=torch.empty((B, N), dtype=torch.float32, device=x.device),
                   kept_idx=torch.empty((B, k), dtype=torch.int32, device=x.device),
                   origin=torch.empty((B, k), dtype=torch.int32, device=x.device),
                   x=torch.empty((B, k, D), dtype=x.dtype, device=x.device) if gather else None)
    _check(lib().luvc_spu_stage(_ptr(x), B, N, D, x.stride(1), code, int(sigma), int(bool(use_hamming)), int(n_keep),
                                _ptr(origin), _ptr(out["scores"]), _ptr(out["kept_idx"]), _ptr(out["origin"]),
                                _ptr(out.get("x")), _ptr(workspace), workspace.numel(), _stream(stream)))
    return out


def _i32(values):
    return (ctypes.c_int32 * max(1, len(values)))(*[int(v) for v in values])


def luvc_oim_plan_anyres(H: int, W: int, max_tokens: int, max_passes: int = 16) -> List[Tuple[int, int]]:
    arr = (LuvcPass * max_passes)()
    n = ctypes.c_int(0)
    _check(lib().luvc_oim_plan_anyres(H, W, int(max_tokens), arr, max_passes, ctypes.byref(n)))
    return [(arr[k].axis, arr[k].m) for k in range(n.value)]


def luvc_oim_merge_ragged(x, shapes, schedules, sizes=None, want_maps: bool = True, workspace=None, stream=None):
    """x: CUDA tensor [sum H_i*W_i, D], image after image; shapes [(H_i, W_i)]; schedules: one pass list per image.
    Returns dict(x [sum H'_i*W'_i, D], sizes, merged_map, kept_map, out_shapes)."""
    import torch
    assert x.is_cuda and x.is_contiguous() and x.dim() == 2 and len(shapes) == len(schedules)
    T, D = x.shape
    assert T == sum(h * w for h, w in shapes)
    code = _dtype_code(x)
    Hs, Ws = _i32([h for h, _ in shapes]), _i32([w for _, w in shapes])
    flat = [p for sch in schedules for p in sch]
    parr, nps = _passes(flat), _i32([len(sch) for sch in schedules])
    out_shapes = [out_grid(h, w, sch) for (h, w), sch in zip(shapes, schedules)]
    To = sum(max(h, 0) * max(w, 0) for h, w in out_shapes)
    if workspace is None:
        need = lib().luvc_oim_ragged_workspace_bytes(len(shapes), Hs, Ws, D, code, parr, nps)
        workspace = torch.empty(max(need, 256), dtype=torch.uint8, device=x.device)
    if sizes is not None:
        assert sizes.is_cuda and sizes.dtype == torch.int32 and sizes.is_contiguous() and sizes.numel() == T
    out = dict(x=torch.empty((To, D), dtype=x.dtype, device=x.device),
               sizes=torch.empty((To,), dtype=torch.int32, device=x.device),
               merged_map=torch.empty((T,), dtype=torch.int32, device=x.device) if want_maps else None,
               kept_map=torch.empty((To,), dtype=torch.int32, device=x.device) if want_maps else None,
               out_shapes=out_shapes)
    _check(lib().luvc_oim_merge_ragged(_ptr(x), _ptr(sizes), len(shapes), Hs, Ws, D, code, parr, nps, _ptr(out["x"]),
                                       _ptr(out["sizes"]), _ptr(out["merged_map"]), _ptr(out["kept_map"]),
                                       _ptr(workspace), workspace.numel(), _stream(stream)))
    return out


def luvc_spu_stage_ragged(x, lengths, sigmas, keeps=None, use_hamming: bool = True, origin=None, gather: bool = True,
                          workspace=None, stream=None):
    """x: CUDA tensor [sum N_i, D] (rows evenly strided), sample after sample; lengths, sigmas, keeps: per sample.
    Returns dict(scores [sum N_i] fp32, kept_idx, origin [sum keep_i] int32, x [sum keep_i, D] or None)."""
    import torch
    assert x.is_cuda and x.dim() == 2 and x.stride(1) == 1 and len(lengths) == len(sigmas)
    T, D = x.shape
    assert T == sum(lengths)
    code = _dtype_code(x)
    Ns, Sg = _i32(lengths), _i32(sigmas)
    Kp = _i32(keeps) if keeps is not None else None
    K = sum(max(int(k), 0) for k in keeps) if keeps is not None else 0
    if origin is not None:
        assert origin.is_cuda and origin.dtype == torch.int32 and origin.is_contiguous() and origin.numel() == T
    if workspace is None:
        need = lib().luvc_spu_ragged_workspace_bytes(len(lengths), Ns, D, code, Sg)
        workspace = torch.empty(max(need, 256), dtype=torch.uint8, device=x.device)
    out = dict(scores=torch.empty((T,), dtype=torch.float32, device=x.device),
               kept_idx=torch.empty((K,), dtype=torch.int32, device=x.device),
               origin=torch.empty((K,), dtype=torch.int32, device=x.device),
               x=torch.empty((K, D), dtype=x.dtype, device=x.device) if (gather and keeps is not None) else None)
    # a tensor without elements has no address: hand the library a one-element stand-in it will not touch
    pad = torch.empty((1,), dtype=torch.int32, device=x.device)
    ki = out["kept_idx"] if K else pad
    og = out["origin"] if K else pad
    _check(lib().luvc_spu_stage_ragged(_ptr(x), len(lengths), Ns, D, x.stride(0), code, Sg, int(bool(use_hamming)), Kp,
                                       _ptr(origin), _ptr(out["scores"]), _ptr(ki), _ptr(og), _ptr(out["x"]) if K else None,
                                       _ptr(workspace), workspace.numel(), _stream(stream)))
    return out


class LaunchProfile:
    """Durations of the kernels libluvc launches between start() and stop(), from HIP events recorded on
    the launch stream (luvc_profile_start / luvc_profile_stop).  Only marshals: the events come from the
    HIP runtime, the recording is done by the library."""

    def __init__(self, max_launches: int):
        self._hip = ctypes.CDLL("libamdhip64.so")
        self._hip.hipEventCreate.argtypes = [ctypes.POINTER(ctypes.c_void_p)]
        self._hip.hipEventElapsedTime.argtypes = [ctypes.POINTER(ctypes.c_float), ctypes.c_void_p, ctypes.c_void_p]
        self._hip.hipEventSynchronize.argtypes = [ctypes.c_void_p]
        self._hip.hipEventDestroy.argtypes = [ctypes.c_void_p]
        self.n = 2 * int(max_launches)
        self.events = (ctypes.c_void_p * self.n)()
        for k in range(self.n):
            e = ctypes.c_void_p()
            if self._hip.hipEventCreate(ctypes.byref(e)) != 0:
                raise RuntimeError("hipEventCreate failed")
            self.events[k] = e
        self.count = 0

    def start(self):
        _check(lib().luvc_profile_start(self.events, self.n))

    def stop(self) -> int:
        self.count = lib().luvc_profile_stop()
        return self.count

    def results(self):
        """[(kernel name, milliseconds)] in launch order; call after the stream has been synchronised."""
        out = []
        for k in range(self.count):
            ms = ctypes.c_float(0)
            self._hip.hipEventSynchronize(self.events[2 * k + 1])
            if self._hip.hipEventElapsedTime(ctypes.byref(ms), self.events[2 * k], self.events[2 * k + 1]) != 0:
                raise RuntimeError("hipEventElapsedTime failed")
            out.append((lib().luvc_profile_kernel(k).decode(), float(ms.value)))
        return out

    def close(self):
        for k in range(self.n):
            if self.events[k]:
                self._hip.hipEventDestroy(self.events[k])
                self.events[k] = None


def luvc_selftest_fdot2(x, y, stream=None):
    """x, y [rows, 2 * words] bf16 -> [rows] fp32: the packed bf16 dot product instruction chained over a row."""
    import torch
    assert x.is_cuda and x.dtype == torch.bfloat16 and x.shape == y.shape and x.dim() == 2 and x.shape[1] % 2 == 0
    assert x.is_contiguous() and y.is_contiguous()
    out = torch.empty((x.shape[0],), dtype=torch.float32, device=x.device)
    _check(lib().luvc_selftest_fdot2(_ptr(x), _ptr(y), x.shape[0], x.shape[1] // 2, _ptr(out), _stream(stream)))
    return out


def luvc_selftest_screen_tile(a, c, stream=None):
    """a, c [32, D] (fp32 or bf16) -> [32, 32] fp32: the screening tile of the wide matching, <a_i, c_j> on the matrix cores."""
    import torch
    assert a.is_cuda and a.shape == c.shape and a.dim() == 2 and a.shape[0] == 32 and a.dtype == c.dtype
    assert a.is_contiguous() and c.is_contiguous()
    out = torch.empty((32, 32), dtype=torch.float32, device=a.device)
    _check(lib().luvc_selftest_screen_tile(_ptr(a), _ptr(c), a.shape[1], _dtype_code(a), _ptr(out), _stream(stream)))
    return out

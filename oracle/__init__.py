"""Loader for the CPU oracle (plain C, fp64) of the OIM + SPU path.

TEST INFRASTRUCTURE ONLY: imported by ``tests/``, by ``__graft_entry__.smoke``
and by the ``cpu_baseline`` leg of ``bench.py``.  The product package never
imports this module and this module never imports the product package.

Most functions below only marshal numpy arrays into ``luvc_oracle.c``, where the
arithmetic of the method lives (similarity, matching, merge, transform, mask,
energy, selection).  Three small pieces of the later rows are written here in
python instead, each a few lines of integer bookkeeping around those C routines:
``cascade_keeps`` (keep counts of an SPU cascade), ``spu_stage`` (one cascade
stage = the C score and prune routines plus the composition of origins) and
``plan_anyres`` (the aspect-ratio schedule).  They are pinned like the rest
(``tests/test_oracle_spu.py``, ``tests/test_oracle_oim.py``).
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "luvc_oracle.c")
# LUVC_ORACLE_SANITIZE=1 selects a build with AddressSanitizer and UndefinedBehaviorSanitizer (its own file, so the
# ordinary build is left alone); the process then needs gcc's libasan.so preloaded, see README.
_SANITIZE = os.environ.get("LUVC_ORACLE_SANITIZE", "") not in ("", "0")
_LIB = os.path.join(_HERE, "libluvc_oracle_san.so" if _SANITIZE else "libluvc_oracle.so")

ROUND_NONE, ROUND_F32, ROUND_BF16 = 0, 1, 2


def build(force: bool = True) -> str:
    """Compile the oracle with gcc (``-O2``, OpenMP over independent images/samples)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        opt = ["-O1", "-g", "-fsanitize=address,undefined", "-fno-sanitize-recover=undefined", "-fno-omit-frame-pointer"] if _SANITIZE else ["-O2"]
        subprocess.check_call(
            ["gcc", *opt, "-fopenmp", "-std=c99", "-D_GNU_SOURCE", "-shared", "-fPIC", "-Wall",
             "-o", _LIB, _SRC, "-lm"])
    return _LIB


_lib = None


def lib() -> ctypes.CDLL:
    global _lib
    if _lib is None:
        build(force=False)
        L = ctypes.CDLL(_LIB)
        c_dp = ctypes.POINTER(ctypes.c_double)
        c_lp = ctypes.POINTER(ctypes.c_int64)
        c_ip = ctypes.POINTER(ctypes.c_int32)
        i = ctypes.c_int
        L.oracle_oim_pass.argtypes = [c_dp, c_lp, i, i, i, i, i, i, i, i, c_dp, c_lp, c_ip, c_ip, c_dp]
        L.oracle_oim_pass.restype = i
        L.oracle_oim_merge.argtypes = [c_dp, c_lp, i, i, i, i, c_ip, c_ip, i, i, i, c_dp, c_lp, c_ip, c_ip, c_dp]
        L.oracle_oim_merge.restype = i
        L.oracle_oim_apply.argtypes = [c_dp, c_lp, i, i, i, i, i, c_ip, c_ip, i, c_dp]
        L.oracle_oim_apply.restype = i
        L.oracle_oim_merge_keyed.argtypes = [c_dp, c_dp, c_lp, i, i, i, i, i, c_ip, c_ip, i, i, i, c_dp, c_dp, c_lp, c_ip, c_ip, c_dp]
        L.oracle_oim_merge_keyed.restype = i
        L.oracle_value_enhance.argtypes = [c_dp, c_lp, ctypes.c_int64, i, i, c_dp]
        L.oracle_value_enhance.restype = i
        L.oracle_spu_mask.argtypes = [i, i, i, i]
        L.oracle_spu_mask.restype = ctypes.c_double
        L.oracle_spu_score.argtypes = [c_dp, i, i, i, i, i, c_dp, c_dp, c_dp]
        L.oracle_spu_score.restype = i
        L.oracle_spu_prune.argtypes = [c_dp, c_dp, i, i, i, i, c_ip, c_dp, c_dp]
        L.oracle_spu_prune.restype = i
        L.oracle_keep_count.argtypes = [i, ctypes.c_double]
        L.oracle_keep_count.restype = i
        _lib = L
    return _lib


def _dp(a):
    return None if a is None else a.ctypes.data_as(ctypes.POINTER(ctypes.c_double))


def _lp(a):
    return None if a is None else a.ctypes.data_as(ctypes.POINTER(ctypes.c_int64))


def _ip(a):
    return None if a is None else a.ctypes.data_as(ctypes.POINTER(ctypes.c_int32))


def _f64(a):
    return np.ascontiguousarray(a, dtype=np.float64)


def out_shape(H, W, passes):
    for axis, m in passes:
        if axis == 1:
            W -= m
        else:
            H -= m
    return H, W


def oim_merge(x, passes, sizes=None, R=1, round_mode=ROUND_NONE):
    """x [B,H,W,D] (any float dtype, widened to fp64); passes = [(axis, m), ...].

    Returns dict(x, sizes, merged_map, kept_map, margin).
    """
    x = _f64(x)
    B, H, W, D = x.shape
    Ho, Wo = out_shape(H, W, passes)
    if Ho < 1 or Wo < 1:
        raise ValueError("schedule removes every token of an axis")
    s_in = None if sizes is None else np.ascontiguousarray(sizes, dtype=np.int64).reshape(B, H, W)
    x_out = np.empty((B, Ho, Wo, D), np.float64)
    s_out = np.empty((B, Ho, Wo), np.int64)
    merged = np.empty((B, H * W), np.int32)
    kept = np.empty((B, Ho * Wo), np.int32)
    axes = np.array([p[0] for p in passes], np.int32)
    ms = np.array([p[1] for p in passes], np.int32)
    margin = ctypes.c_double(float("inf"))
    rc = lib().oracle_oim_merge(_dp(x), _lp(s_in), B, H, W, D, _ip(axes), _ip(ms), len(passes), R, round_mode,
                                _dp(x_out), _lp(s_out), _ip(merged), _ip(kept), ctypes.byref(margin))
    if rc != 0:
        raise ValueError("oracle_oim_merge rejected its arguments")
    return dict(x=x_out, sizes=s_out, merged_map=merged, kept_map=kept, margin=margin.value)


def oim_merge_keyed(x, metric, passes, sizes=None, R=1, round_mode=ROUND_NONE):
    """Decisions on metric [B,H,W,Dm], merge applied to x [B,H,W,D] (and to the metric).

    Returns dict(x, metric, sizes, merged_map, kept_map, margin).
    """
    x, metric = _f64(x), _f64(metric)
    B, H, W, D = x.shape
    Dm = metric.shape[3]
    assert metric.shape[:3] == (B, H, W)
    Ho, Wo = out_shape(H, W, passes)
    if Ho < 1 or Wo < 1:
        raise ValueError("schedule removes every token of an axis")
    s_in = None if sizes is None else np.ascontiguousarray(sizes, dtype=np.int64).reshape(B, H, W)
    x_out = np.empty((B, Ho, Wo, D), np.float64)
    k_out = np.empty((B, Ho, Wo, Dm), np.float64)
    s_out = np.empty((B, Ho, Wo), np.int64)
    merged = np.empty((B, H * W), np.int32)
    kept = np.empty((B, Ho * Wo), np.int32)
    axes = np.array([p[0] for p in passes], np.int32)
    ms = np.array([p[1] for p in passes], np.int32)
    margin = ctypes.c_double(float("inf"))
    rc = lib().oracle_oim_merge_keyed(_dp(x), _dp(metric), _lp(s_in), B, H, W, D, Dm, _ip(axes), _ip(ms), len(passes), R, round_mode,
                                      _dp(x_out), _dp(k_out), _lp(s_out), _ip(merged), _ip(kept), ctypes.byref(margin))
    if rc != 0:
        raise ValueError("oracle_oim_merge_keyed rejected its arguments")
    return dict(x=x_out, metric=k_out, sizes=s_out, merged_map=merged, kept_map=kept, margin=margin.value)


def value_enhance(v, sizes, round_mode=ROUND_NONE):
    """v [..., D] + log(sizes [...]) on every channel (Eq. 3)."""
    v = _f64(v)
    s = np.ascontiguousarray(sizes, dtype=np.int64)
    assert s.shape == v.shape[:-1]
    out = np.empty_like(v)
    rc = lib().oracle_value_enhance(_dp(v), _lp(s), int(s.size), v.shape[-1], round_mode, _dp(out))
    if rc != 0:
        raise ValueError("oracle_value_enhance rejected its arguments")
    return out


def spu_mask(N, sigma, use_hamming=True):
    return np.array([lib().oracle_spu_mask(k, N, sigma, int(bool(use_hamming))) for k in range(N)])


def spu_score(x, sigma, use_hamming=True, want_filtered=False):
    """x [B,N,D] -> scores [B,N] fp64 (and the filtered signal when asked)."""
    x = _f64(x)
    B, N, D = x.shape
    scores = np.empty((B, N), np.float64)
    filt = np.empty((B, N, D), np.float64) if want_filtered else None
    mi = ctypes.c_double(0.0)
    rc = lib().oracle_spu_score(_dp(x), B, N, D, sigma, int(bool(use_hamming)), _dp(scores), _dp(filt),
                                ctypes.byref(mi))
    if rc != 0:
        raise ValueError("oracle_spu_score rejected its arguments")
    if want_filtered:
        return scores, filt, mi.value
    return scores


def spu_prune(scores, n_keep, x=None):
    """scores [B,N] -> kept_idx [B,n_keep] ascending (+ gathered rows of x, + margin)."""
    scores = _f64(scores)
    B, N = scores.shape
    kept = np.empty((B, n_keep), np.int32)
    xo = None
    D = 1
    if x is not None:
        x = _f64(x)
        D = x.shape[2]
        xo = np.empty((B, n_keep, D), np.float64)
    margin = ctypes.c_double(float("inf"))
    rc = lib().oracle_spu_prune(_dp(scores), _dp(x), B, N, D, n_keep, _ip(kept), _dp(xo), ctypes.byref(margin))
    if rc != 0:
        raise ValueError("oracle_spu_prune rejected its arguments")
    return dict(kept_idx=kept, x=xo, margin=margin.value)


def keep_count(N, ratio):
    return lib().oracle_keep_count(N, float(ratio))


def cascade_keeps(N0, ratio, n_stages, eliminate=True):
    """Keep counts of an SPU cascade (Section 3.3, last paragraph): the paper removes the visual tokens
    progressively and entirely at the end but prints no per-stage counts; the reading taken here applies
    one keep ratio stage after stage, with 0 in the last stage when `eliminate`."""
    keeps, n = [], int(N0)
    for i in range(int(n_stages)):
        n = 0 if (eliminate and i == n_stages - 1) else keep_count(n, ratio)
        keeps.append(n)
    return keeps


def spu_stage(x, sigma, n_keep, use_hamming=True, origin=None):
    """One cascade stage: Algorithm 2 on the tokens still alive (x [B,N,D]), and the position each kept
    token had before the first stage (origin [B,N], identity when None)."""
    x = _f64(x)
    B, N, D = x.shape
    if origin is None:
        origin = np.tile(np.arange(N, dtype=np.int32), (B, 1))
    origin = np.asarray(origin)
    if n_keep == 0:
        return dict(scores=None, kept_idx=np.empty((B, 0), np.int32), origin=np.empty((B, 0), np.int32),
                    x=np.empty((B, 0, D), np.float64), margin=float("inf"))
    scores = spu_score(x, sigma, use_hamming)
    pr = spu_prune(scores, n_keep, x)
    org = np.empty((B, n_keep), np.int32)
    for b in range(B):
        for q in range(n_keep):
            org[b, q] = origin[b, pr["kept_idx"][b, q]]
    return dict(scores=scores, kept_idx=pr["kept_idx"], origin=org, x=pr["x"], margin=pr["margin"])


def plan_anyres(H, W, max_tokens):
    """Aspect-ratio-adaptive schedule (appendix on the iterative strategy of OIM: the merges per axis follow
    the aspect ratio of the image; no rule is printed).  Reading: while the grid holds more than max_tokens
    tokens, halve its longer side (the row merge when the sides are equal); a grid that is small enough
    gets the single pass that merges nothing."""
    passes = []
    while H * W > max_tokens:
        if W >= H:
            passes.append((1, (W + 1) // 2))
            W //= 2
        else:
            passes.append((0, (H + 1) // 2))
            H //= 2
    return passes or [(1, 0)]

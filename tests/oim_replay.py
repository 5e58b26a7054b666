"""The acceptance rule for OIM maps when a decision of the oracle is closer than the arithmetic can resolve.

An OIM pass (paper Section 3.2, Algorithm 1) takes two kinds of decisions on cosines: which candidate destination a
source prefers, and which m sources of a line are merged.  Where the winning and the losing alternative are further
apart than `eps` the decision is unique and the GPU must take it; where they are closer, either alternative is a
correct result of the method carried out in finite precision.  `replay` walks the schedule pass by pass on the CPU and
takes, at every decision that is closer than eps, the alternative the GPU's maps show (if that alternative is within
eps of the best one under the cosines computed here in fp64), and the oracle's choice everywhere else.  Alternatives
whose tokens are bit for bit the same tie exactly on any arithmetic: there the lower position is the only answer.
The merge itself is the oracle's (oracle_oim_apply on the maps of the pass), so the features that come out are what
the oracle computes for those decisions.  The caller then compares maps, sizes and features with the GPU's as usual: a GPU
decision that is not eps-optimal cannot be reproduced here and fails that comparison.

Test infrastructure only (it calls the oracle); nothing in the product imports it.
"""
import ctypes

import numpy as np


def _cosine(u, v):
    nu, nv = max(np.sqrt(float(u @ u)), 1e-12), max(np.sqrt(float(v @ v)), 1e-12)
    return float(u @ v) / (nu * nv)


def _flat(axis, W, line, p):
    return line * W + p if axis else p * W + line


def _one_pass(orc, y, x_list, sizes, axis, m, R, round_mode, slot_of, eps):
    """y [B,H,W,Dy]: tensor the decisions are taken on; x_list: tensors merged along (y itself may be among them).
    slot_of [B,H*W]: final GPU slot of every token of the current grid.  Returns the merged tensors, sizes, the
    maps of this pass and the number of decisions that were closer than eps."""
    B, H, W, _ = y.shape
    length, nlines = (W, H) if axis else (H, W)
    Ho, Wo = (H, W - m) if axis else (H - m, W)
    merged_map = np.empty((B, H * W), np.int32)
    kept_map = np.empty((B, Ho * Wo), np.int32)
    close = 0
    for b in range(B):
        tok = y[b].reshape(H * W, -1)
        for line in range(nlines):
            pos = [_flat(axis, W, line, p) for p in range(length)]
            pick, score = {}, {}
            for a in range(0, length, 2):
                cands = [c for c in range(1, length, 2) if R <= 0 or abs(c - a) <= 2 * R - 1]
                if not cands:
                    continue
                sims = [_cosine(tok[pos[a]], tok[pos[c]]) for c in cands]
                j = int(np.argmax(sims))                                # first maximum: the lower position
                # alternatives: candidates within eps of the best - but a candidate whose token has the very bits of the
                # best one is an exact tie on any arithmetic, and those go to the lower position
                near = [i for i in range(len(cands)) if sims[j] - sims[i] <= eps
                        and (i == j or not np.array_equal(tok[pos[cands[i]]], tok[pos[cands[j]]]))]
                if len(near) > 1:
                    close += 1
                    same = [i for i in near if slot_of[b, pos[cands[i]]] == slot_of[b, pos[a]]]
                    if same and j not in same:
                        j = same[0]
                pick[a], score[a] = cands[j], sims[j]
            order = sorted(pick, key=lambda a: (-score[a], a))
            chosen = set(order[:m])
            if 0 < m < len(order) and score[order[m - 1]] - score[order[m]] <= eps:
                close += 1
                gpu_set = {a for a in pick if slot_of[b, pos[a]] == slot_of[b, pos[pick[a]]]}
                if len(gpu_set) == m:
                    worst_in = min(score[a] for a in gpu_set)
                    best_out = max(score[a] for a in pick if a not in gpu_set)
                    # two sources with the same bits (their own and their destination's) tie exactly: lower position first
                    same_bits = lambda a, c: (np.array_equal(tok[pos[a]], tok[pos[c]])
                                              and np.array_equal(tok[pos[pick[a]]], tok[pos[pick[c]]]))
                    tie_rule = all(a < c for a in gpu_set for c in pick if c not in gpu_set and same_bits(a, c))
                    if worst_in >= best_out - eps and tie_rule:
                        chosen = gpu_set
            q = 0
            for p in range(length):
                if p in chosen:
                    continue
                out = _flat(axis, Wo, line, q)
                kept_map[b, out] = pos[p]
                merged_map[b, pos[p]] = out
                q += 1
            for a in chosen:
                merged_map[b, pos[a]] = merged_map[b, pos[pick[a]]]
    L = orc.lib()
    dp, lp, ip = (ctypes.POINTER(t) for t in (ctypes.c_double, ctypes.c_int64, ctypes.c_int32))
    s64 = np.ascontiguousarray(sizes, np.int64)
    outs = []
    for t in x_list:
        t = np.ascontiguousarray(t, np.float64)
        o = np.empty((B, Ho, Wo, t.shape[3]), np.float64)
        rc = L.oracle_oim_apply(t.ctypes.data_as(dp), s64.ctypes.data_as(lp), B, H, W, t.shape[3], Ho * Wo,
                                merged_map.ctypes.data_as(ip), kept_map.ctypes.data_as(ip), round_mode, o.ctypes.data_as(dp))
        assert rc == 0
        outs.append(o)
    s_out = np.stack([np.bincount(merged_map[b], weights=s64[b].ravel(), minlength=Ho * Wo) for b in range(B)])
    return outs, s_out.astype(np.int64).reshape(B, Ho, Wo), merged_map, kept_map, close


def replay(orc, x, passes, gpu_merged_map, sizes=None, R=1, round_mode=0, eps=1e-10, metric=None):
    """x [B,H,W,D] fp64 (values of the I/O dtype), gpu_merged_map [B,H*W] as the GPU returned it.
    Returns dict(x, sizes, merged_map, kept_map, close[, metric])."""
    x = np.ascontiguousarray(x, np.float64)
    B, H, W, _ = x.shape
    s = np.ones((B, H, W), np.int64) if sizes is None else np.asarray(sizes, np.int64).reshape(B, H, W)
    tot_merged = np.tile(np.arange(H * W, dtype=np.int32), (B, 1))
    tot_kept = tot_merged.copy()
    gpu = np.asarray(gpu_merged_map).reshape(B, H * W)
    y = None if metric is None else np.ascontiguousarray(metric, np.float64)
    close = 0
    for axis, m in passes:
        slot_of = np.take_along_axis(gpu, tot_kept.astype(np.int64), axis=1)     # GPU slot of the anchor of every current token
        if y is None:
            (x,), s, mm, km, c = _one_pass(orc, x, [x], s, axis, m, R, round_mode, slot_of, eps)
        else:
            (x, y), s, mm, km, c = _one_pass(orc, y, [x, y], s, axis, m, R, round_mode, slot_of, eps)
        close += c
        tot_merged = np.take_along_axis(mm, tot_merged.astype(np.int64), axis=1)
        tot_kept = np.take_along_axis(tot_kept, km.astype(np.int64), axis=1)
    out = dict(x=x, sizes=s, merged_map=tot_merged, kept_map=tot_kept, close=close)
    if y is not None:
        out["metric"] = y
    return out

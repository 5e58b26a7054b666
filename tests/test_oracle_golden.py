"""Pins of the CPU oracle against the values the paper prints (tests/golden/paper_values.txt, each with its citation)."""
import os

import numpy as np

W_AX, H_AX = 1, 0


def paper_values():
    vals = {}
    with open(os.path.join(os.path.dirname(__file__), "golden", "paper_values.txt")) as f:
        for line in f:
            line = line.split("#")[0].strip()
            if "=" in line:
                k, v = line.split("=")
                vals[k.strip()] = float(v)
    return vals


def test_window_constants_of_eq5(oracle):
    pv = paper_values()
    a0, a1 = pv["hamming_a0"], pv["hamming_a1"]
    for N in (9, 144, 1025):
        half = (N - 1) // 2
        m = oracle.spu_mask(N, N // 2, True)
        assert m[0] == a0 + a1 == 1.0                                   # DC passes unchanged
        np.testing.assert_allclose(m[half], a0 + a1 * np.cos(2 * np.pi * half / (N - 1)), rtol=1e-15)
        if N % 2 == 1:
            np.testing.assert_allclose(m[half], a0 - a1, rtol=1e-12)    # the far end of the window: 0.08
        # the two constants can be read back from any two bins
        f1, f2 = 1, max(2, half // 2)
        c1, c2 = np.cos(2 * np.pi * f1 / (N - 1)), np.cos(2 * np.pi * f2 / (N - 1))
        got_a1 = (m[f1] - m[f2]) / (c1 - c2)
        np.testing.assert_allclose([m[f1] - got_a1 * c1, got_a1], [a0, a1], rtol=1e-9)


def test_token_counts_of_the_appendix_setting(oracle):
    pv = paper_values()
    m, ops = int(pv["oim_merge_number"]), int(pv["oim_operations_video"])
    side = int(round(pv["tokens_per_patch"] ** 0.5))
    assert side * side == pv["tokens_per_patch"]
    x = np.random.default_rng(0).standard_normal((1, side, side, 4))
    h = w = side
    sizes = None
    for op in range(ops):
        r1 = oracle.oim_merge(x, [(W_AX, m)], sizes=sizes, R=0)
        assert r1["x"].shape[1:3] == (h, w - m)                          # H x W -> H x (W - m)
        r2 = oracle.oim_merge(r1["x"], [(H_AX, m)], sizes=r1["sizes"], R=0)
        assert r2["x"].shape[1:3] == (h - m, w - m)                      # -> (H - m) x (W - m)
        assert r2["sizes"].sum() == side * side                          # the size vector still counts every original token
        x, sizes, h, w = r2["x"], r2["sizes"], h - m, w - m
    assert h * w == (side - ops * m) ** 2 == 100

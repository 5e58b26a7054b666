"""GPU parity: luvc_spu_score / luvc_spu_prune (through the C ABI) against the CPU oracle."""
import numpy as np
import pytest
import torch

from paper_2512_09010_amd import binding as lv
from paper_2512_09010_amd import workloads as wl
from gpu_util import SPU_MARGIN, to_dev, to_host_f64

pytestmark = pytest.mark.gpu

# fp32 arithmetic on both storage types: the scores themselves are held to the fp32 bar
SCORE_RTOL = 1e-5


def score_case(oracle, x_io, dtype, sigma, ham=True, tag="", stride_pad=0):
    print(f"[spu] {tag} shape={x_io.shape} dtype={dtype} sigma={sigma} ham={ham}", flush=True)
    ref = oracle.spu_score(wl.widen(x_io, dtype), sigma, ham)
    xd = to_dev(x_io, dtype)
    if stride_pad:
        B, N, D = xd.shape
        wide = torch.full((B, N, D + stride_pad), float("nan"), dtype=xd.dtype, device="cuda")
        wide[:, :, :D] = xd
        xd = wide[:, :, :D]
    got = lv.luvc_spu_score(xd, sigma, ham)
    torch.cuda.synchronize()
    floor = 1e-6 * np.abs(ref).max()                # tokens whose filtered energy vanishes carry no relative meaning
    g = got.cpu().numpy().astype(np.float64)
    err = np.abs(g - ref)
    assert (err <= SCORE_RTOL * np.abs(ref) + floor).all(), (tag, float((err / (np.abs(ref) + floor)).max()))
    return xd, got, ref


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("B,N,D,sigma", [
    (1, 1, 8, 0), (1, 2, 8, 1), (2, 5, 3, 2), (2, 16, 64, 3), (1, 97, 70, 10), (2, 144, 200, 18),
    (1, 196, 130, 4), (1, 256, 64, 128), (2, 130, 65, 0), (1, 300, 96, 31),
    # shapes served by the transform-decomposition FFT path (N = 16 Q N2 with Q = 16, 15 or 9, 2 sigma + 1 <= 16 Q)
    (2, 256, 64, 20), (1, 256, 32, 127), (1, 512, 70, 127), (1, 768, 33, 50), (2, 1024, 96, 102), (1, 2048, 40, 0),
    (1, 1280, 31, 64),
    (2, 240, 64, 119), (1, 240, 33, 0), (2, 720, 70, 54), (1, 480, 40, 60), (1, 1200, 34, 100),      # Q = 15
    (2, 144, 64, 71), (1, 144, 200, 18), (1, 288, 37, 30), (1, 432, 64, 72), (1, 1008, 32, 7),       # Q = 9
    # one-launch direct path beyond a single batch of token pairs per wavefront, odd and even lengths, up to its LDS limit
    (2, 600, 70, 3), (1, 601, 33, 5), (1, 1500, 33, 2), (1, 3000, 64, 1), (1, 4000, 40, 1), (1, 513, 64, 11),
])
def test_score_small_random(oracle, dtype, B, N, D, sigma):
    rng = np.random.default_rng(N * 31 + D)
    x = wl.cast_io(rng.standard_normal((B, N, D)).astype(np.float32), dtype)
    score_case(oracle, x, dtype, sigma, True, "random")
    score_case(oracle, x, dtype, sigma, False, "random-rect")


def test_score_strided_rows(oracle):
    rng = np.random.default_rng(3)
    x = wl.cast_io(rng.standard_normal((2, 40, 72)).astype(np.float32), "bf16")
    score_case(oracle, x, "bf16", 5, True, "strided", stride_pad=24)
    x = wl.cast_io(rng.standard_normal((2, 512, 72)).astype(np.float32), "bf16")
    score_case(oracle, x, "bf16", 30, True, "strided-fft", stride_pad=24)
    score_case(oracle, x, "bf16", 30, True, "strided-fft-odd", stride_pad=7)       # odd token stride: unaligned pairs
    xf = rng.standard_normal((1, 256, 50)).astype(np.float32)
    score_case(oracle, xf, "f32", 9, False, "strided-fft-f32", stride_pad=3)


def test_score_repeated_calls_with_poisoned_workspace(oracle):
    """The per-sample completion counters and the cross-workgroup hand-over of the tile energies: many calls
    in a row on one workspace that is overwritten with NaN patterns before each call must reproduce the
    first result bit for bit (a stale or early read would return NaN or another call's values)."""
    rng = np.random.default_rng(77)
    shapes = [(3, 1024, 200, 102), (5, 720, 130, 54), (2, 2048, 96, 40)]
    for B, N, D, sigma in shapes:
        xa = wl.cast_io(rng.standard_normal((B, N, D)).astype(np.float32), "bf16")
        xb = wl.cast_io(rng.standard_normal((B, N, D)).astype(np.float32), "bf16")
        _, want_a, _ = score_case(oracle, xa, "bf16", sigma, True, "repeat-a")
        _, want_b, _ = score_case(oracle, xb, "bf16", sigma, True, "repeat-b")
        da, db = to_dev(xa, "bf16"), to_dev(xb, "bf16")
        ws = torch.empty(lv.luvc_spu_workspace_bytes(B, N, D, lv.LUVC_BF16, sigma), dtype=torch.uint8, device="cuda")
        out = torch.empty((B, N), dtype=torch.float32, device="cuda")
        bad = torch.zeros((), dtype=torch.int64, device="cuda")
        for it in range(40):
            for d, want in ((da, want_a), (db, want_b)):
                ws.fill_(0xFF)
                out.fill_(float("nan"))
                lv.luvc_spu_score(d, sigma, True, workspace=ws, out=out)
                bad += (out.view(torch.int32) != want.view(torch.int32)).sum()
        torch.cuda.synchronize()
        assert bad.item() == 0, (B, N, D, sigma, bad.item())


def test_score_calls_overlapping_on_two_streams():
    """Score calls in flight at the same time on two streams (own workspaces) share nothing but the library's
    static completion counters, which are handed out per call: every result must equal the serial one bit for bit."""
    rng = np.random.default_rng(123)
    cases = [(4, 1024, 3584 // 4, 102), (3, 720, 512, 54), (2, 196, 300, 4)]          # fft (Q = 16, 15) and the one-launch dense path
    data = []
    for B, N, D, sigma in cases:
        x = to_dev(wl.cast_io(rng.standard_normal((B, N, D)).astype(np.float32), "bf16"), "bf16")
        want = lv.luvc_spu_score(x, sigma, True)
        ws = [torch.empty(lv.luvc_spu_workspace_bytes(B, N, D, lv.LUVC_BF16, sigma), dtype=torch.uint8, device="cuda") for _ in range(2)]
        outs = [torch.empty((B, N), dtype=torch.float32, device="cuda") for _ in range(2)]
        data.append((x, sigma, want, ws, outs))
    torch.cuda.synchronize()
    streams = [torch.cuda.Stream(), torch.cuda.Stream()]
    bad = [torch.zeros((), dtype=torch.int64, device="cuda") for _ in range(2)]
    for it in range(30):
        for k, st in enumerate(streams):
            x, sigma, want, ws, outs = data[(it + k) % len(data)]
            with torch.cuda.stream(st):
                outs[k].fill_(float("nan"))
                lv.luvc_spu_score(x, sigma, True, workspace=ws[k], stream=st, out=outs[k])
                bad[k] += (outs[k].view(torch.int32) != want.view(torch.int32)).sum()
    torch.cuda.synchronize()
    assert bad[0].item() == 0 and bad[1].item() == 0, (bad[0].item(), bad[1].item())


def test_score_special_signals(oracle):
    N, D = 64, 64
    n = np.arange(N)
    const = np.broadcast_to(np.linspace(-1, 1, D, dtype=np.float32), (1, N, D)).copy()
    _, got, ref = score_case(oracle, const, "f32", 6, True, "constant")
    np.testing.assert_allclose(got.cpu().numpy(), np.linalg.norm(const[0, 0]), rtol=1e-5)
    high = np.broadcast_to(np.cos(np.pi * n)[None, :, None].astype(np.float32), (1, N, D)).copy()
    got = lv.luvc_spu_score(to_dev(high, "f32"), 6, False)
    assert got.abs().max().item() < 1e-4 * np.sqrt(D)          # the Nyquist ripple is outside the pass-band


@pytest.mark.parametrize("i", [0, 1, 2, 3, 4])
def test_mini_workloads(oracle, i):
    w = wl.mini(i)
    x = wl.spu_input(w)
    xd, got, ref = score_case(oracle, x, w.dtype, w.sigma, True, w.name)
    n_keep = w.n_keep
    assert n_keep == lv.luvc_keep_count(w.spu_N, w.keep_ratio) == oracle.keep_count(w.spu_N, w.keep_ratio)
    pr = lv.luvc_spu_prune(xd, got, n_keep)
    torch.cuda.synchronize()
    kept = pr["kept_idx"].cpu().numpy()
    # (i) the selection itself is exact: same answer as the oracle's selection on the GPU's own scores
    own = oracle.spu_prune(got.cpu().numpy().astype(np.float64), n_keep)
    np.testing.assert_array_equal(kept, own["kept_idx"])
    # (ii) and equal to the oracle's keep set whenever its boundary gap exceeds the fp32 error of the scores
    full = oracle.spu_prune(ref, n_keep, wl.widen(x, w.dtype))
    if full["margin"] > SPU_MARGIN:
        np.testing.assert_array_equal(kept, full["kept_idx"])
        np.testing.assert_array_equal(to_host_f64(pr["x"]), full["x"])     # original tokens, bit copies
    else:
        print(f"keep boundary gap {full['margin']:.2e} below {SPU_MARGIN}: set compared on own scores only")


def adversarial_scores(N, rng):
    cases = [np.ones(N, np.float32), np.zeros(N, np.float32), np.arange(N, dtype=np.float32), np.arange(N, dtype=np.float32)[::-1].copy(),
             np.round(rng.random(N).astype(np.float32) * 4) / 4,
             rng.random(N).astype(np.float32),
             np.where(rng.random(N) < 0.5, np.float32(0.0), np.float32(-0.0)).astype(np.float32),
             (rng.random(N).astype(np.float32) * np.float32(1e-41)),                 # denormals
             np.where(rng.random(N) < 0.1, np.float32(np.inf), rng.random(N).astype(np.float32)).astype(np.float32),
             rng.standard_normal(N).astype(np.float32)]                              # negative values order correctly too
    return np.stack(cases)


@pytest.mark.parametrize("N,k", [(1, 1), (7, 3), (64, 64), (257, 1), (1024, 205), (2048, 205), (3000, 1500), (720, 108),
                                 (4096, 4095), (4097, 33), (9000, 1000)])     # above 4096 tokens: selection and gather as two launches
def test_select_against_stable_sort(oracle, N, k):
    rng = np.random.default_rng(N + k)
    sc = adversarial_scores(N, rng)
    print(f"[select] N={N} k={k}", flush=True)
    pr = lv.luvc_spu_prune(None, torch.from_numpy(sc).cuda(), k, gather=False)
    torch.cuda.synchronize()
    kept = pr["kept_idx"].cpu().numpy()
    want = oracle.spu_prune(sc.astype(np.float64), k)["kept_idx"]
    np.testing.assert_array_equal(kept, want)
    assert (np.diff(kept, axis=1) > 0).all() if k > 1 else True


def test_select_nonfinite_stays_well_formed():
    N, k = 500, 100
    sc = np.random.default_rng(0).standard_normal(N).astype(np.float32)
    sc[::7] = np.nan
    sc[3::11] = -np.inf
    pr = lv.luvc_spu_prune(None, torch.from_numpy(sc[None]).cuda(), k, gather=False)
    kept = pr["kept_idx"].cpu().numpy()[0]
    assert len(np.unique(kept)) == k and (np.diff(kept) > 0).all() and kept.min() >= 0 and kept.max() < N


@pytest.mark.parametrize("dtype,D,pad", [("f32", 33, 0), ("bf16", 33, 0), ("bf16", 64, 8), ("f32", 256, 4), ("bf16", 3584, 0)])
def test_gather_rows(dtype, D, pad):
    rng = np.random.default_rng(D)
    B, N, k = 2, 50, 13
    x = wl.cast_io(rng.standard_normal((B, N, D + pad)).astype(np.float32), dtype)
    xd = to_dev(x, dtype)[:, :, :D]
    sc = torch.from_numpy(rng.random((B, N)).astype(np.float32)).cuda()
    pr = lv.luvc_spu_prune(xd, sc, k)
    torch.cuda.synchronize()
    idx = pr["kept_idx"].long()
    want = torch.gather(xd, 1, idx[:, :, None].expand(B, k, D))
    assert torch.equal(pr["x"].view(torch.int16) if dtype == "bf16" else pr["x"], want.contiguous().view(torch.int16) if dtype == "bf16" else want)


@pytest.mark.parametrize("seed", range(20))
def test_score_and_prune_random_shapes(oracle, seed):
    """Seeded random (B, N, D, sigma, window, row padding, keep count): lengths that the fft factorisations serve and
    lengths that they do not, bands from DC only to the widest each path takes, channel counts around the tile edges."""
    rng = np.random.default_rng(500 + seed)
    dtype = "bf16" if seed % 2 else "f32"
    B = int(rng.integers(1, 5))
    kind = seed % 4
    if kind == 0:
        N = int(rng.choice([256, 512, 768, 1024, 1280, 1536]))          # 16 x 16 x N2
    elif kind == 1:
        N = int(rng.choice([240, 480, 720, 960, 144, 288, 432, 1008]))  # 16 x 15 x N2, 16 x 9 x N2
    else:
        N = int(rng.integers(2, 700))
    D = int(rng.choice([1, 7, 31, 32, 33, 64, 65, 100, 130, 257]))
    sigma = int(rng.integers(0, N // 2 + 1))
    if kind < 2 and seed % 3:
        sigma = int(rng.integers(0, min(N // 2, 70) + 1))                # inside the band the fft path takes
    ham = bool(rng.integers(0, 2))
    pad = int(rng.choice([0, 0, 3, 8]))
    x = wl.cast_io((rng.standard_normal((B, N, D)) + np.cos(np.arange(N) * rng.uniform(0.01, 0.5))[None, :, None]).astype(np.float32), dtype)
    xd, got, ref = score_case(oracle, x, dtype, sigma, ham, f"fuzz{seed}", stride_pad=pad)
    k = int(rng.integers(1, N + 1))
    # selection on the library's own scores: compare with a stable sort of exactly those values
    pr = lv.luvc_spu_prune(xd, got, k)
    torch.cuda.synchronize()
    g = got.cpu().numpy()
    for b in range(B):
        want = np.sort(np.argsort(-g[b], kind="stable")[:k])
        np.testing.assert_array_equal(pr["kept_idx"][b].cpu().numpy(), want)
        np.testing.assert_array_equal(to_host_f64(pr["x"][b]), to_host_f64(xd[b])[want])


def test_calls_from_several_host_threads():
    """Four host threads, each with a stream, workspace and outputs of its own, run score + prune side by side:
    every result must equal, bit for bit, what one thread computes alone (the library keeps per-call counters in a
    shared device array handed out in slots, and its error and timing state per thread)."""
    import threading
    rng = np.random.default_rng(99)
    B, N, D, sigma, keep = 3, 1024, 160, 60, 100
    xs = [to_dev(wl.cast_io(rng.standard_normal((B, N, D)).astype(np.float32), "bf16"), "bf16") for _ in range(4)]
    want = []
    for x in xs:
        sc = lv.luvc_spu_score(x, sigma, True)
        pr = lv.luvc_spu_prune(x, sc, keep)
        torch.cuda.synchronize()
        want.append((sc.clone(), pr["kept_idx"].clone(), pr["x"].clone()))
    errors = []

    def worker(k):
        try:
            torch.cuda.set_device(0)
            st = torch.cuda.Stream()
            ws = torch.empty(lv.luvc_spu_workspace_bytes(B, N, D, lv.LUVC_BF16, sigma), dtype=torch.uint8, device="cuda")
            sc = torch.empty((B, N), dtype=torch.float32, device="cuda")
            out = dict(kept_idx=torch.empty((B, keep), dtype=torch.int32, device="cuda"),
                       x=torch.empty((B, keep, D), dtype=torch.bfloat16, device="cuda"))
            for it in range(30):
                sc.fill_(float("nan"))
                st.wait_stream(torch.cuda.current_stream())
                lv.luvc_spu_score(xs[k], sigma, True, workspace=ws, stream=st, out=sc)
                lv.luvc_spu_prune(xs[k], sc, keep, stream=st, out=out)
                st.synchronize()
                if not (torch.equal(sc, want[k][0]) and torch.equal(out["kept_idx"], want[k][1]) and torch.equal(out["x"], want[k][2])):
                    errors.append((k, it))
                    return
        except Exception as e:                    # surfaces in the main thread below
            errors.append((k, repr(e)))

    threads = [threading.Thread(target=worker, args=(k,)) for k in range(4)]
    for th in threads:
        th.start()
    for th in threads:
        th.join()
    assert not errors, errors


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("B,N,D,sigma", [(2, 1024, 96, 102), (1, 2048, 64, 102), (1, 768, 64, 50), (1, 1008, 64, 7), (1, 960, 40, 20)])
def test_score_where_token_energies_vanish(oracle, dtype, B, N, D, sigma):
    """Lengths on which the fft path evaluates the inverse on a subset of the tokens and fills in the rest from the
    band limit of the tile energies - which is ill-conditioned wherever a token's filtered channels all but vanish
    next to neighbours whose channels do not.  The kernel must notice (per tile) and evaluate those tiles in full:
    the bar is the same 1e-5 as everywhere."""
    rng = np.random.default_rng(N + D + sigma)
    n = np.arange(N)
    gains = rng.standard_normal(D)
    f = max(1, sigma // 2)
    tone = np.cos(2 * np.pi * f * n / N + 0.3)[None, :, None] * gains[None, None, :]           # every channel crosses zero at the same tokens
    x = np.broadcast_to(tone, (B, N, D)).astype(np.float32)
    score_case(oracle, wl.cast_io(x, dtype), dtype, sigma, True, "tone")
    x = rng.standard_normal((B, N, D)).astype(np.float32)
    x[:, N // 3: N // 3 + N // 5] = 0.0                                                         # a span of padding tokens
    score_case(oracle, wl.cast_io(x, dtype), dtype, sigma, True, "padding")
    x = rng.standard_normal((B, N, D)).astype(np.float32)
    x[:, :, :32] = tone[:, :, :32]                                                              # one ill-conditioned tile among ordinary ones
    score_case(oracle, wl.cast_io(x, dtype), dtype, sigma, False, "one-tile")
    x = np.zeros((B, N, D), np.float32)
    x[:, N // 2, :] = 1.0                                                                       # an impulse: the filter's own kernel, with its side-lobe zeros
    score_case(oracle, wl.cast_io(x, dtype), dtype, sigma, True, "impulse")


@pytest.mark.parametrize("seed", range(4))
def test_score_fuzz_on_lengths_with_a_thinned_inverse(oracle, seed):
    """Seeded random cases on the lengths the fft path serves, mostly with bands narrow enough for the thinned inverse:
    white noise, tones that cross zero in every channel, spans of zero tokens, a few dominant channels, token norms
    that swing over orders of magnitude, random walks (large energies next to small ones across the wrap-around)."""
    rng = np.random.default_rng(900 + seed)
    lengths = [512, 768, 1024, 1280, 1536, 2048, 3072, 4096, 480, 960, 1440, 1200, 288, 432, 576, 1008, 720, 2304]
    for it in range(25):
        N = int(rng.choice(lengths))
        dtype = "bf16" if rng.integers(2) else "f32"
        B, D = int(rng.integers(1, 4)), int(rng.choice([2, 31, 32, 33, 64, 96, 130, 257]))
        q = 16 if N % 256 == 0 else (15 if N % 240 == 0 else 9)
        smax = min((16 * q - 1) // 2, N // 2)
        sigma = int(rng.integers(0, max(1, min(smax, N // 8)) + 1)) if rng.integers(4) else int(rng.integers(0, smax + 1))
        kind = int(rng.integers(6))
        n = np.arange(N)
        x = rng.standard_normal((B, N, D))
        if kind == 1:
            x = np.cos(2 * np.pi * max(1, sigma // 2) * n / N + rng.uniform(0, 6))[None, :, None] * rng.standard_normal(D)[None, None, :] + 1e-3 * x
        if kind == 2:
            x[:, rng.integers(0, N // 2): rng.integers(N // 2, N)] = 0
        if kind == 3:
            x = x * np.exp(rng.standard_normal((1, 1, D)) * 3)
        if kind == 4:
            x = x * (np.abs(np.sin(2 * np.pi * 3 * n / N)) ** 4)[None, :, None]
        if kind == 5:
            x = np.cumsum(x, axis=1) / np.sqrt(N)
        pad = int(rng.choice([0, 0, 3, 8]))
        score_case(oracle, wl.cast_io(x.astype(np.float32), dtype), dtype, sigma, True, f"thin-fuzz{seed}.{it} kind={kind}", stride_pad=pad)

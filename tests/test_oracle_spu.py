"""Pins for the SPU oracle: Eq. 4 / Eq. 7 are the textbook DFT pair (library FFT and a brute-force
O(N^2) sum check them), Eq. 5 fixes the Hamming constants and the zero stop-band, Eq. 8 the norm,
Algorithm 2 the top-k keep of the ORIGINAL tokens.  CPU only."""
import numpy as np
import pytest


def rnd(shape, seed=0):
    return np.random.default_rng(seed).standard_normal(shape)


# ---------------------------------------------------------------- the mask (Eq. 5)

@pytest.mark.parametrize("N,sigma", [(8, 2), (9, 4), (144, 18), (196, 4), (720, 54), (1024, 102)])
def test_mask_shape(oracle, N, sigma):
    M = oracle.spu_mask(N, sigma, True)
    assert M[0] == 1.0                                           # DC passes untouched
    k = np.arange(N)
    f = np.minimum(k, N - k)
    assert (M[f > sigma] == 0).all() and (M[f <= sigma] > 0).all()
    np.testing.assert_array_equal(M[1:], M[1:][::-1])            # symmetric -> real filter
    assert (np.diff(M[: sigma + 1]) < 0).all()                   # tapers with |frequency|
    R = oracle.spu_mask(N, sigma, False)
    np.testing.assert_array_equal(R, (f <= sigma).astype(float)) # "wo HW": rectangular pass-band


def test_mask_printed_constants(oracle):
    # Hamming constants 0.54 / 0.46 and the N-1 denominator: the window reaches 0.54-0.46 = 0.08 at
    # the far end (f = (N-1)/2, odd N) and 0.54 at the quarter point f = (N-1)/4.
    M = oracle.spu_mask(9, 4, True)
    np.testing.assert_allclose(M[4], 0.08, rtol=0, atol=1e-15)
    np.testing.assert_allclose(M[2], 0.54, rtol=0, atol=1e-15)
    np.testing.assert_allclose(M[1], 0.54 + 0.46 * np.sqrt(0.5), rtol=0, atol=1e-15)
    M = oracle.spu_mask(13, 6, True)
    np.testing.assert_allclose(M[[2, 3, 4]], [0.54 + 0.23, 0.54, 0.54 - 0.23], atol=1e-15)
    assert oracle.spu_mask(1, 0, True)[0] == 1.0


# ---------------------------------------------------------------- transforms (Eq. 4, 7)

def brute_filter(x, M):
    """Direct double sum with complex exponentials, independent of the oracle's code."""
    N = x.shape[0]
    n = np.arange(N)
    E = np.exp(-2j * np.pi * np.outer(n, n) / N)                 # E[k,n]
    F = E @ x
    return (np.conj(E).T @ (M[:, None] * F)) / N


@pytest.mark.parametrize("N,sigma,ham", [(1, 0, True), (2, 1, True), (5, 1, True), (8, 2, False), (12, 6, True), (16, 3, True)])
def test_tiny_against_bruteforce_dft(oracle, N, sigma, ham):
    x = rnd((2, N, 3), N)
    sc, filt, imag = oracle.spu_score(x, sigma, ham, want_filtered=True)
    M = oracle.spu_mask(N, sigma, ham)
    for b in range(2):
        want = brute_filter(x[b], M)
        assert np.abs(want.imag).max() < 1e-12
        np.testing.assert_allclose(filt[b], want.real, atol=1e-12)
        np.testing.assert_allclose(sc[b], np.linalg.norm(want.real, axis=1), rtol=1e-11, atol=1e-13)
    assert imag < 1e-12


@pytest.mark.parametrize("N,sigma", [(144, 18), (196, 4), (720, 54), (256, 25), (97, 10)])
def test_against_library_fft(oracle, N, sigma):
    x = rnd((1, N, 4), N + 1)
    for ham in (True, False):
        sc, filt, imag = oracle.spu_score(x, sigma, ham, want_filtered=True)
        M = oracle.spu_mask(N, sigma, ham)
        want = np.fft.ifft(np.fft.fft(x[0], axis=0) * M[:, None], axis=0)
        np.testing.assert_allclose(filt[0], want.real, atol=1e-11)
        np.testing.assert_allclose(sc[0], np.linalg.norm(want.real, axis=1), rtol=1e-10)
        assert imag < 1e-11


def test_full_band_rectangular_is_identity(oracle):
    # sigma = N/2 without weighting passes every bin: forward followed by inverse (with 1/N) is the identity
    for N in (6, 7, 32):
        x = rnd((1, N, 5), 3)
        sc, filt, _ = oracle.spu_score(x, N // 2, False, want_filtered=True)
        np.testing.assert_allclose(filt, x, atol=1e-12)
        np.testing.assert_allclose(sc[0], np.linalg.norm(x[0], axis=1), rtol=1e-12)


# ---------------------------------------------------------------- special signals

def test_constant_signal_keeps_only_dc(oracle):
    v = rnd((6,), 4)
    x = np.broadcast_to(v, (1, 40, 6)).copy()
    sc, filt, _ = oracle.spu_score(x, 5, True, want_filtered=True)
    np.testing.assert_allclose(filt, x, atol=1e-12)              # M[0] = 1: the DC term comes back whole
    np.testing.assert_allclose(sc, np.linalg.norm(v), rtol=1e-12)
    # sigma = 0 keeps DC alone: the filtered signal is the token mean
    y = rnd((1, 40, 6), 5)
    sc0, filt0, _ = oracle.spu_score(y, 0, True, want_filtered=True)
    np.testing.assert_allclose(filt0[0], np.broadcast_to(y[0].mean(0), (40, 6)), atol=1e-12)


def test_low_band_passes_high_band_dies(oracle):
    N, sigma = 64, 6
    n = np.arange(N)
    low = np.stack([np.cos(2 * np.pi * 3 * n / N + 0.3), np.sin(2 * np.pi * 6 * n / N), 0.5 + 0 * n,
                    np.cos(2 * np.pi * 1 * n / N) - 2 * np.sin(2 * np.pi * 5 * n / N)], axis=1)[None]
    high = np.stack([np.cos(2 * np.pi * 7 * n / N), np.sin(2 * np.pi * 20 * n / N + 1.0),
                     np.cos(np.pi * n), np.sin(2 * np.pi * 31 * n / N)], axis=1)[None]
    _, f_low, _ = oracle.spu_score(low, sigma, False, want_filtered=True)
    np.testing.assert_allclose(f_low, low, atol=1e-12)
    sc_high, f_high, _ = oracle.spu_score(high, sigma, False, want_filtered=True)
    np.testing.assert_allclose(f_high, 0, atol=1e-12)
    np.testing.assert_allclose(sc_high, 0, atol=1e-11)
    # with the Hamming weights a pure tone at frequency f is scaled by exactly w(f)
    M = oracle.spu_mask(N, sigma, True)
    _, f_ham, _ = oracle.spu_score(low[:, :, :2], sigma, True, want_filtered=True)
    np.testing.assert_allclose(f_ham[0, :, 0], M[3] * low[0, :, 0], atol=1e-12)
    np.testing.assert_allclose(f_ham[0, :, 1], M[6] * low[0, :, 1], atol=1e-12)


def test_filter_closed_forms(oracle):
    N, D, sigma = 48, 5, 7
    x, y = rnd((1, N, D), 6), rnd((1, N, D), 7)
    _, fx, _ = oracle.spu_score(x, sigma, True, want_filtered=True)
    _, fy, _ = oracle.spu_score(y, sigma, True, want_filtered=True)
    sc, fxy, _ = oracle.spu_score(2.0 * x - 3.0 * y, sigma, True, want_filtered=True)
    np.testing.assert_allclose(fxy, 2.0 * fx - 3.0 * fy, atol=1e-12)          # linear
    sx = oracle.spu_score(x, sigma, True)
    sr = oracle.spu_score(np.roll(x, 5, axis=1), sigma, True)
    np.testing.assert_allclose(sr, np.roll(sx, 5, axis=1), rtol=1e-11)        # circular-shift covariance
    M = oracle.spu_mask(N, sigma, True)
    p = np.fft.ifft(M).real                                                   # impulse response
    conv = np.zeros((N, D))
    for n in range(N):
        for j in range(N):
            conv[n] += p[(n - j) % N] * x[0, j]
    np.testing.assert_allclose(fx[0], conv, atol=1e-12)                       # x' = p (*) x
    F = np.fft.fft(x[0], axis=0)
    np.testing.assert_allclose((sx ** 2).sum(), ((M[:, None] * np.abs(F)) ** 2).sum() / N, rtol=1e-11)  # Parseval
    # channels are independent and the score is the L2 norm over channels (not its square, not a mean)
    s1 = oracle.spu_score(x[:, :, :1], sigma, True)
    np.testing.assert_allclose(s1[0], np.abs(fx[0, :, 0]), rtol=1e-11, atol=1e-14)
    s_dup = oracle.spu_score(np.concatenate([x, x], axis=2), sigma, True)
    np.testing.assert_allclose(s_dup, np.sqrt(2.0) * sx, rtol=1e-12)


# ---------------------------------------------------------------- top-k keep (Algorithm 2)

def stable_topk(scores, k):
    order = np.argsort(-scores, kind="stable")[:k]
    return np.sort(order)


@pytest.mark.parametrize("N,k", [(1, 1), (10, 3), (10, 10), (257, 64), (1024, 205)])
def test_prune_is_stable_topk(oracle, N, k):
    rng = np.random.default_rng(N + k)
    sc = np.abs(rng.standard_normal((3, N)))
    sc[1] = np.round(sc[1] * 4) / 4                               # many exact ties
    sc[2] = 1.0                                                   # all equal -> the first k indices
    x = rng.standard_normal((3, N, 4))
    r = oracle.spu_prune(sc, k, x)
    for b in range(3):
        want = stable_topk(sc[b], k)
        np.testing.assert_array_equal(r["kept_idx"][b], want)
        np.testing.assert_array_equal(r["x"][b], x[b][want])      # the original, unfiltered tokens
    np.testing.assert_array_equal(r["kept_idx"][2], np.arange(k))
    assert (np.diff(r["kept_idx"], axis=1) > 0).all()


def test_prune_margin(oracle):
    sc = np.array([[5.0, 1.0, 4.0, 3.9, 0.5]])
    r = oracle.spu_prune(sc, 2)
    np.testing.assert_array_equal(r["kept_idx"][0], [0, 2])
    np.testing.assert_allclose(r["margin"], (4.0 - 3.9) / 4.0)
    assert oracle.spu_prune(np.array([[1.0, 1.0, 1.0]]), 2)["margin"] == 0.0


def test_keep_count(oracle):
    # round-half-up of ratio*N, clamped to [1, N]
    assert oracle.keep_count(1024, 0.20) == 205
    assert oracle.keep_count(196, 0.05) == 10
    assert oracle.keep_count(144, 0.25) == 36
    assert oracle.keep_count(720, 0.15) == 108
    assert oracle.keep_count(2048, 0.10) == 205
    assert oracle.keep_count(10, 0.0) == 1 and oracle.keep_count(10, 2.0) == 10


def test_end_to_end_energy_ranking(oracle):
    # tokens carrying a strong low-frequency component must outrank tokens that are pure high-frequency noise
    N, D = 64, 8
    n = np.arange(N)
    x = np.zeros((1, N, D))
    x[0, :, :] = 0.05 * np.cos(np.pi * n)[:, None]               # Nyquist ripple everywhere
    bump = np.exp(-0.5 * ((n - 20) / 6.0) ** 2)
    x[0] += bump[:, None]                                         # smooth bump around token 20
    sc = oracle.spu_score(x, 6, True)
    kept = oracle.spu_prune(sc, 9)["kept_idx"][0]
    np.testing.assert_array_equal(kept, np.arange(16, 25))


# ---------------------------------------------------------------- cascade (Section 3.3, last paragraph)

def fft_stage(x, sigma, k, origin):
    """A stage written with the library FFT and a stable argsort: rectangular band, no oracle code."""
    B, N, D = x.shape
    F = np.fft.fft(x, axis=1)
    f = np.minimum(np.arange(N), N - np.arange(N))
    F[:, f > sigma, :] = 0
    sc = np.linalg.norm(np.fft.ifft(F, axis=1).real, axis=2)
    kept = np.stack([stable_topk(sc[b], k) for b in range(B)])
    return kept, np.take_along_axis(origin, kept, axis=1), np.stack([x[b][kept[b]] for b in range(B)])


def test_cascade_keeps_closed_form(oracle):
    assert oracle.cascade_keeps(1024, 0.5, 4) == [512, 256, 128, 0]
    assert oracle.cascade_keeps(1024, 0.5, 3, eliminate=False) == [512, 256, 128]
    assert oracle.cascade_keeps(1024, 0.2, 3) == [205, 41, 0]          # 204.8 -> 205, 41.0 -> 41
    assert oracle.cascade_keeps(7, 0.01, 3, eliminate=False) == [1, 1, 1]
    assert oracle.cascade_keeps(9, 1.0, 1) == [0]


def test_stage_origin_composes(oracle):
    # three stages with a "layer" (a fixed mixing of channels plus a per-token drift) between them; the origins of the
    # survivors must be those of a pipeline written with the library FFT, and must index the first stage's tokens
    rng = np.random.default_rng(5)
    B, N, D = 2, 96, 6
    x0 = rng.standard_normal((B, N, D)) + np.sin(np.arange(N) / 7.0)[None, :, None]
    mix = rng.standard_normal((D, D)) / np.sqrt(D)
    keeps, sigmas = [40, 17, 5], [12, 6, 2]
    x_o, org_o = x0, None
    x_r, org_r = x0, np.tile(np.arange(N), (B, 1))
    for k, sg in zip(keeps, sigmas):
        r = oracle.spu_stage(x_o, sg, k, use_hamming=False, origin=org_o)
        kept, org_r, xk = fft_stage(x_r, sg, k, org_r)
        assert r["margin"] > 1e-9
        np.testing.assert_array_equal(r["kept_idx"], kept)
        np.testing.assert_array_equal(r["origin"], org_r)
        np.testing.assert_array_equal(r["x"], xk)
        assert (np.diff(r["origin"], axis=1) > 0).all()                 # order of the first stage survives
        x_o, org_o = np.tanh(r["x"] @ mix), r["origin"]
        x_r = np.tanh(xk @ mix)
    assert set(org_o[0]) <= set(range(N))


def test_stage_identity_origin_and_elimination(oracle):
    x = rnd((1, 12, 3), 2)
    r = oracle.spu_stage(x, 3, 5)
    np.testing.assert_array_equal(r["origin"], r["kept_idx"])
    perm = np.arange(100, 112, dtype=np.int32)[None, :]
    r2 = oracle.spu_stage(x, 3, 5, origin=perm)
    np.testing.assert_array_equal(r2["origin"], r["kept_idx"] + 100)
    z = oracle.spu_stage(x, 3, 0, origin=perm)
    assert z["kept_idx"].shape == (1, 0) and z["origin"].shape == (1, 0) and z["x"].shape == (1, 0, 3)

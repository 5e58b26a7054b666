"""GPU parity at the FULL sizes of the five benchmark configurations, element by element against
the CPU oracle, in the launch configuration bench.py times (preallocated outputs, one workspace,
same calls).  Inputs are the seeded synthetic fields of paper_2512_09010_amd.workloads; if a seed
happens to produce a decision whose gap is below the arithmetic error (see gpu_util), the seed is
advanced by 1000, as the design notes describe, and the seed used is printed."""
import numpy as np
import pytest
import torch

from paper_2512_09010_amd import binding as lv
from paper_2512_09010_amd import workloads as wl
from gpu_util import OIM_MARGIN, SPU_MARGIN, round_mode, to_dev, to_host_f64

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("i", [0, 1, 2, 3, 4])
def test_oim_full(oracle, i):
    w = wl.workload(i)
    for reseed in range(4):
        x = wl.oim_input(w, reseed)
        print(f"[full oim] {w.name} reseed={reseed} shape={x.shape}", flush=True)
        cur_ref, sizes_ref = wl.widen(x, w.dtype), None
        cur_dev, sizes_dev = to_dev(x, w.dtype), None
        margin = np.inf
        refs, outs = [], []
        for passes in w.oim_calls:
            ref = oracle.oim_merge(cur_ref, passes, sizes=sizes_ref, round_mode=round_mode(oracle, w.dtype))
            out = lv.luvc_oim_merge(cur_dev, passes, sizes=sizes_dev)
            torch.cuda.synchronize()
            margin = min(margin, ref["margin"])
            refs.append(ref)
            outs.append(out)
            cur_ref, sizes_ref = ref["x"], ref["sizes"]
            # the next call reads the oracle's bits on both sides, so a call is judged on identical inputs
            cur_dev = to_dev(wl.cast_io(ref["x"].astype(np.float32), w.dtype), w.dtype)
            sizes_dev = torch.from_numpy(ref["sizes"].astype(np.int32)).cuda()
        if margin > OIM_MARGIN:
            break
        print(f"  smallest decision gap {margin:.3e} <= {OIM_MARGIN}: reseeding", flush=True)
    else:
        pytest.fail("no seed with unique decisions found")
    print(f"  smallest decision gap {margin:.3e}", flush=True)
    for ref, out in zip(refs, outs):
        np.testing.assert_array_equal(out["merged_map"].cpu().numpy(), ref["merged_map"])
        np.testing.assert_array_equal(out["kept_map"].cpu().numpy(), ref["kept_map"])
        np.testing.assert_array_equal(out["sizes"].cpu().numpy().astype(np.int64), ref["sizes"])
        got = to_host_f64(out["x"])
        if w.dtype == "bf16":
            np.testing.assert_array_equal(got, ref["x"])                       # fp64 merge, one rounding: same bits
        else:
            np.testing.assert_allclose(got, ref["x"], rtol=1e-5, atol=0)
    Ho, Wo = w.out_grid()
    assert tuple(outs[-1]["x"].shape) == (w.grids, Ho, Wo, w.D)


@pytest.mark.parametrize("i", [0, 1, 2, 3, 4])
def test_spu_full(oracle, i):
    w = wl.workload(i)
    for reseed in range(4):
        x = wl.spu_input(w, reseed)
        print(f"[full spu] {w.name} reseed={reseed} shape={x.shape} sigma={w.sigma} n_keep={w.n_keep}", flush=True)
        xw = wl.widen(x, w.dtype)
        ref = oracle.spu_score(xw, w.sigma, True)
        full = oracle.spu_prune(ref, w.n_keep, xw)
        if full["margin"] > SPU_MARGIN:
            break
        print(f"  keep-boundary gap {full['margin']:.3e} <= {SPU_MARGIN}: reseeding", flush=True)
    else:
        pytest.fail("no seed with a unique keep set found")
    xd = to_dev(x, w.dtype)
    code = lv.LUVC_BF16 if w.dtype == "bf16" else lv.LUVC_F32
    ws = torch.empty(lv.luvc_spu_workspace_bytes(w.spu_B, w.spu_N, w.spu_D, code, w.sigma), dtype=torch.uint8, device="cuda")
    scores = torch.empty((w.spu_B, w.spu_N), dtype=torch.float32, device="cuda")
    ws.fill_(0xFF)                                                               # scratch contents must not matter
    lv.luvc_spu_score(xd, w.sigma, True, workspace=ws, out=scores)
    pr = lv.luvc_spu_prune(xd, scores, w.n_keep)
    torch.cuda.synchronize()
    got = scores.cpu().numpy().astype(np.float64)
    rel = np.abs(got - ref) / np.abs(ref)
    print(f"  keep-boundary gap {full['margin']:.3e}; worst relative score error {rel.max():.3e}", flush=True)
    assert rel.max() <= 1e-5                                                    # fp32 bar, met by bf16 inputs as well
    kept = pr["kept_idx"].cpu().numpy()
    np.testing.assert_array_equal(kept, oracle.spu_prune(got, w.n_keep)["kept_idx"])   # selection exact on own scores
    np.testing.assert_array_equal(kept, full["kept_idx"])                               # and equal to the oracle's keep set
    np.testing.assert_array_equal(to_host_f64(pr["x"]), full["x"])                      # original tokens, bit copies


def test_step_replayed_from_a_hip_graph():
    """The three calls of a step enqueue kernels only (no allocation, no host synchronisation, no memset), so a step can
    be captured into a HIP graph; every replay, with eager work and synchronisations in between, must reproduce the
    eager results bit for bit."""
    w = wl.mini(1)
    code = lv.LUVC_BF16
    xo = to_dev(wl.oim_input(w), w.dtype)
    xs = to_dev(wl.spu_input(w), w.dtype)
    passes = w.oim_calls[0]
    eager_o = lv.luvc_oim_merge(xo, passes)
    eager_s = lv.luvc_spu_score(xs, w.sigma, True)
    eager_p = lv.luvc_spu_prune(xs, eager_s, w.n_keep)
    torch.cuda.synchronize()
    B, H, W, D = xo.shape
    Ho, Wo = lv.out_grid(H, W, passes)
    out = dict(x=torch.empty_like(eager_o["x"]), sizes=torch.empty_like(eager_o["sizes"]),
               merged_map=torch.empty_like(eager_o["merged_map"]), kept_map=torch.empty_like(eager_o["kept_map"]))
    ws_o = torch.empty(max(256, lv.luvc_oim_workspace_bytes(B, H, W, D, code, passes)), dtype=torch.uint8, device="cuda")
    ws_s = torch.empty(max(256, lv.luvc_spu_workspace_bytes(w.spu_B, w.spu_N, w.spu_D, code, w.sigma)), dtype=torch.uint8, device="cuda")
    scores = torch.empty_like(eager_s)
    pr = dict(kept_idx=torch.empty_like(eager_p["kept_idx"]), x=torch.empty_like(eager_p["x"]))
    side = torch.cuda.Stream()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        with torch.cuda.graph(g, stream=side):
            st = torch.cuda.current_stream()
            lv.luvc_oim_merge(xo, passes, workspace=ws_o, stream=st, out=out)
            lv.luvc_spu_score(xs, w.sigma, True, workspace=ws_s, stream=st, out=scores)
            lv.luvc_spu_prune(xs, scores, w.n_keep, stream=st, out=pr)
    torch.cuda.synchronize()
    for rep in range(4):
        for t in (out["x"], scores, pr["x"]):
            t.zero_()
        out["merged_map"].fill_(-1); pr["kept_idx"].fill_(-1)
        ws_s.fill_(0xFF)
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        lv.luvc_spu_score(xs, w.sigma, True)                                   # eager work between the replays
        torch.cuda.synchronize()
        assert torch.equal(out["x"].view(torch.int16), eager_o["x"].view(torch.int16)), rep
        assert torch.equal(out["merged_map"], eager_o["merged_map"]) and torch.equal(out["kept_map"], eager_o["kept_map"]), rep
        assert torch.equal(scores.view(torch.int32), eager_s.view(torch.int32)), rep
        assert torch.equal(pr["kept_idx"], eager_p["kept_idx"]) and torch.equal(pr["x"].view(torch.int16), eager_p["x"].view(torch.int16)), rep


@pytest.mark.parametrize("B,N,D,sigma", [(2, 1024, 544, 102), (2, 196, 320, 4)])      # fft path (two tile groups), one-launch direct path
def test_graph_replays_beside_eager_score_calls(B, N, D, sigma):
    """A captured score launch replayed on one stream while more than 64 eager score calls run on another: every call
    owns its workspace (completion counters included), so nothing is shared between calls in flight and every result
    must carry the bits of a call that ran alone.  The workspaces start out holding different garbage."""
    rng = np.random.default_rng(N + D)
    xs = to_dev(wl.cast_io(rng.standard_normal((B, N, D)).astype(np.float32), "bf16"), "bf16")
    xs2 = to_dev(wl.cast_io(rng.standard_normal((B, N, D)).astype(np.float32), "bf16"), "bf16")
    alone = lv.luvc_spu_score(xs, sigma, True)
    alone2 = lv.luvc_spu_score(xs2, sigma, True)
    torch.cuda.synchronize()
    need = max(256, lv.luvc_spu_workspace_bytes(B, N, D, lv.LUVC_BF16, sigma))
    ws_g = torch.empty(need, dtype=torch.uint8, device="cuda"); ws_g.fill_(0x01)
    ws_e = torch.empty(need, dtype=torch.uint8, device="cuda"); ws_e.fill_(0xA5)
    sc_g = torch.empty_like(alone)
    side, other = torch.cuda.Stream(), torch.cuda.Stream()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        with torch.cuda.graph(g, stream=side):
            lv.luvc_spu_score(xs, sigma, True, workspace=ws_g, stream=torch.cuda.current_stream(), out=sc_g)
    torch.cuda.synchronize()
    outs = [torch.empty_like(alone2) for _ in range(72)]
    for rep in range(3):
        print(f"[graph+eager] N={N} round {rep}", flush=True)
        sc_g.zero_()
        torch.cuda.synchronize()
        with torch.cuda.stream(side):
            for _ in range(24):
                g.replay()
        with torch.cuda.stream(other):
            for o in outs[rep * 24:(rep + 1) * 24]:
                lv.luvc_spu_score(xs2, sigma, True, workspace=ws_e, stream=other, out=o)
        torch.cuda.synchronize()
        assert torch.equal(sc_g.view(torch.int32), alone.view(torch.int32)), rep
        for k, o in enumerate(outs[rep * 24:(rep + 1) * 24]):
            assert torch.equal(o.view(torch.int32), alone2.view(torch.int32)), (rep, k)


@pytest.mark.parametrize("i", [0, 1, 2, 3, 4])
def test_chained_step_on_the_gpus_own_bits(oracle, i):
    """The chain the configurations describe, end to end on one set of bits: every OIM call reads the previous call's
    GPU output, the merged tokens are projected on the host to the SPU width (input generation), and the score and the
    keep run on that tensor.  The oracle runs the same chain from the same input on its own."""
    w = wl.workload(i)
    code = lv.LUVC_BF16 if w.dtype == "bf16" else lv.LUVC_F32
    for reseed in range(4):
        x = wl.oim_input(w, reseed)
        print(f"[chain] {w.name} reseed={reseed}", flush=True)
        cur_ref, sizes_ref, margin = wl.widen(x, w.dtype), None, np.inf
        for passes in w.oim_calls:
            ref = oracle.oim_merge(cur_ref, passes, sizes=sizes_ref, round_mode=round_mode(oracle, w.dtype))
            margin = min(margin, ref["margin"])
            cur_ref, sizes_ref = ref["x"], ref["sizes"]
        xs_ref = wl.spu_input_from_merged(w, cur_ref, reseed)
        xs64 = wl.widen(xs_ref, w.dtype)
        sc_ref = oracle.spu_score(xs64, w.sigma, True)
        pr_ref = oracle.spu_prune(sc_ref, w.n_keep, xs64)
        if margin > OIM_MARGIN and pr_ref["margin"] > SPU_MARGIN:
            break
        print(f"  decision gap {margin:.3e}, keep-boundary gap {pr_ref['margin']:.3e}: reseeding", flush=True)
    else:
        pytest.fail("no seed with unique decisions found")
    cur, sizes = to_dev(x, w.dtype), None
    for passes in w.oim_calls:
        out = lv.luvc_oim_merge(cur, passes, sizes=sizes)
        cur, sizes = out["x"], out["sizes"]
    torch.cuda.synchronize()
    merged = to_host_f64(cur)
    np.testing.assert_array_equal(sizes.cpu().numpy().astype(np.int64), sizes_ref)
    if w.dtype == "bf16":
        np.testing.assert_array_equal(merged, cur_ref)                          # so both sides project the same tokens
    else:
        np.testing.assert_allclose(merged, cur_ref, rtol=1e-5, atol=0)
    xs = wl.spu_input_from_merged(w, merged, reseed)                            # the GPU's own bits, projected
    xd = to_dev(xs, w.dtype)
    scores = lv.luvc_spu_score(xd, w.sigma, True)
    pr = lv.luvc_spu_prune(xd, scores, w.n_keep)
    torch.cuda.synchronize()
    if w.dtype == "f32" and not np.array_equal(xs, xs_ref):                     # fp32 merges may differ in the last place: judge the SPU calls on what they read
        xs64 = wl.widen(xs, w.dtype)
        sc_ref = oracle.spu_score(xs64, w.sigma, True)
        pr_ref = oracle.spu_prune(sc_ref, w.n_keep, xs64)
        assert pr_ref["margin"] > SPU_MARGIN
    else:
        np.testing.assert_array_equal(xs, xs_ref)
    got = scores.cpu().numpy().astype(np.float64)
    rel = np.abs(got - sc_ref) / np.abs(sc_ref)
    print(f"  worst relative score error {rel.max():.3e}", flush=True)
    assert rel.max() <= 1e-5
    np.testing.assert_array_equal(pr["kept_idx"].cpu().numpy(), pr_ref["kept_idx"])
    np.testing.assert_array_equal(to_host_f64(pr["x"]), pr_ref["x"])


@pytest.mark.parametrize("i", [1, 2, 3])
def test_keyed_calls_at_full_size(oracle, i):
    """The calls that decide on keys, on the full encoder grids of the batch workloads (all grids of the batch, keys of
    one attention head cut from the tokens): the hot path's schedule on the fused pair kernel, and the appendix setting
    (whole line, merge number 2, two operations) on the one-launch passes, element by element against the oracle."""
    from gpu_util import oim_reference
    w = wl.workload(i)
    x = wl.oim_input(w)
    Dm = 128
    keys = np.ascontiguousarray(x[..., 256:256 + Dm])
    for passes, radius in ((w.oim_calls[0], 1), ([(1, 2), (0, 2)] * 2, 0)):
        print(f"[full keyed] {w.name} x={x.shape} keys={keys.shape} passes={passes} radius={radius}", flush=True)
        out = lv.luvc_oim_merge_keyed(to_dev(x, w.dtype), to_dev(keys, w.dtype), passes, radius)
        torch.cuda.synchronize()
        ref = oim_reference(oracle, wl.widen(x, w.dtype), passes, out["merged_map"].cpu().numpy(), w.dtype, R=radius, metric=wl.widen(keys, w.dtype))
        np.testing.assert_array_equal(out["sizes"].cpu().numpy().astype(np.int64), ref["sizes"])
        np.testing.assert_array_equal(out["merged_map"].cpu().numpy(), ref["merged_map"])
        np.testing.assert_array_equal(out["kept_map"].cpu().numpy(), ref["kept_map"])
        np.testing.assert_array_equal(to_host_f64(out["x"]), ref["x"])
        np.testing.assert_array_equal(to_host_f64(out["metric"]), ref["metric"])

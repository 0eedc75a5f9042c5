"""GPU parity of the data-free calibration step (Section 3.2, Eq. 4; App. B.2) against the CPU oracle.

Bar: the error matrix E = Q1(W + L R) - (W + L R) bit-exact (both sides form W + L R with the same fp32 FMA chain and
quantise it with the same fp32 arithmetic); gradients within 32 ulps of the sum of the magnitudes of their terms (the
GPU sums K or N products in fp32 on the matrix core, the oracle in fp64); the Adam update within what that gradient
difference can move it, plus a few ulps; loss trajectories over tens of steps within 1e-3."""
import numpy as np
import pytest
import torch

from paper_2604_18117_amd import binding as lq

pytestmark = pytest.mark.gpu


def _problem(N, K, r, seed):
    rng = np.random.default_rng(seed)
    W = (rng.standard_normal((N, K)) * 0.02).astype(np.float32)
    W[:, rng.choice(K, 3, replace=False)] *= 6.0          # a few heavy input channels
    U, S, Vt = np.linalg.svd(W.astype(np.float64), full_matrices=False)
    L0 = (U[:, :r] * np.sqrt(S[:r])).astype(np.float32)
    R0 = (np.sqrt(S[:r])[:, None] * Vt[:r]).astype(np.float32)
    return W, np.ascontiguousarray(-L0), np.ascontiguousarray(R0)


def _cfg(N, K, r, g, sint4):
    if g == 32:                                   # sint4 names the MX main format here: "mxfp4" | "mxint4"
        return lq.make_config(N, K, r, "mx" if sint4 == "mxfp4" else "mxi", 32, 8, 8)
    return lq.make_config(N, K, r, "int", g, 8, 8, a_group=64 if sint4 else 0)


def _orc_step(oracle, W, st, g, sint4, lr):
    if g == 32:
        return oracle.calib_step(W, st, q1=sint4, lr=lr)
    return oracle.calib_step(W, st, g, sint4_blocks=sint4, lr=lr)


def _n(t):
    return t.cpu().numpy()


def _check_step(oracle, cfg, W, Wd, state, st, step, lr, g, sint4):
    """One step on both sides from states that are (nearly) equal; returns the two losses."""
    L_before, R_before = st.L.copy(), st.R.copy()
    loss = torch.zeros(1, dtype=torch.float32, device="cuda")
    lq.lq_calib_step(cfg, Wd, state, step, lr=lr, loss=loss)
    out = _orc_step(oracle, W, st, g, sint4, lr)
    got = lq.lq_calib_unpack(cfg, state, ("L", "R", "gL", "gR", "E"))
    torch.cuda.synchronize()
    N, K = W.shape
    c = 2.0 / (N * K)
    bound_L = 2e-6 * c * (np.abs(out.E).astype(np.float64) @ np.abs(R_before).astype(np.float64).T) + 1e-30
    bound_R = 2e-6 * c * (np.abs(L_before).astype(np.float64).T @ np.abs(out.E).astype(np.float64)) + 1e-30
    return out, got, float(loss.item()), bound_L, bound_R


@pytest.mark.parametrize("N,K,r,g,sint4", [(128, 256, 16, 64, False), (192, 384, 32, 128, False), (64, 1152, 64, 64, True),
                                           (320, 128, 128, 64, False), (128, 384, 32, 32, "mxfp4"), (192, 256, 64, 32, "mxint4"),
                                           (128, 1152, 96, 32, "mxint4")])
def test_first_step_matches_oracle(oracle, N, K, r, g, sint4):
    W, L, R = _problem(N, K, r, seed=N + K)
    cfg = _cfg(N, K, r, g, sint4)
    Wd = torch.from_numpy(W).cuda()
    state = lq.lq_calib_init(cfg, torch.from_numpy(L).cuda(), torch.from_numpy(R).cuda())
    st = oracle.calib_init(L, R)
    lr = 1e-4
    out, got, loss, bL, bR = _check_step(oracle, cfg, W, Wd, state, st, 1, lr, g, sint4)
    assert np.array_equal(_n(got["E"]), out.E), "E"
    assert abs(loss - out.loss) <= 1e-5 * out.loss
    assert np.all(np.abs(_n(got["gL"]) - out.gL) <= bL), "gL"
    assert np.all(np.abs(_n(got["gR"]) - out.gR) <= bR), "gR"
    # Adam: d(update)/dg = lr eps / (|g| + eps)^2 at the first step; plus fp32 rounding of the update and the parameter
    eps = 1e-8
    for name, p_orc, gr, bd in (("L", st.L, out.gL, bL), ("R", st.R, out.gR, bR)):
        slack = lr * bd * eps / (np.abs(gr).astype(np.float64) + eps) ** 2 + 2e-6 * lr + 2e-7 * np.abs(p_orc)
        assert np.all(np.abs(_n(got[name]).astype(np.float64) - p_orc) <= slack), name
    # moments and a second call: bit-for-bit reproducible
    state2 = lq.lq_calib_init(cfg, torch.from_numpy(L).cuda(), torch.from_numpy(R).cuda())
    lq.lq_calib_step(cfg, Wd, state2, 1, lr=lr)
    names = ("L", "R", "mL", "vL", "mR", "vR", "gL", "gR", "E")
    a, b = lq.lq_calib_unpack(cfg, state, names), lq.lq_calib_unpack(cfg, state2, names)
    torch.cuda.synchronize()
    for k in names:                      # (the blob's alignment padding is never written, so compare the sections)
        assert torch.equal(a[k], b[k]), k
    assert np.allclose(_n(a["mL"]), 0.1 * _n(a["gL"]), rtol=1e-6, atol=0)   # first moments after one step: (1 - beta1) g


@pytest.mark.parametrize("g,kind,lr", [(64, False, 1e-4), (32, "mxfp4", 1e-3)])
def test_trajectory_matches_oracle(oracle, g, kind, lr):
    N, K, r = 128, 256, 16
    W, L, R = _problem(N, K, r, seed=5)
    cfg = _cfg(N, K, r, g, kind)
    Wd = torch.from_numpy(W).cuda()
    state = lq.lq_calib_init(cfg, torch.from_numpy(L).cuda(), torch.from_numpy(R).cuda())
    st = oracle.calib_init(L, R)
    steps = 40
    loss = torch.zeros(1, dtype=torch.float32, device="cuda")
    lg, lo = [], []
    for t in range(1, steps + 1):
        lq.lq_calib_step(cfg, Wd, state, t, lr=lr, loss=loss)
        lg.append(float(loss.item()))
        lo.append(_orc_step(oracle, W, st, g, kind, lr).loss)
    assert np.allclose(lg, lo, rtol=1e-3)
    assert lg[-1] < 0.97 * lg[0]                                 # the optimisation lowers the loss of the SVD start
    got = lq.lq_calib_unpack(cfg, state)
    travel = steps * lr
    assert np.abs(_n(got["L"]) - st.L).max() <= 0.05 * travel and np.abs(_n(got["R"]) - st.R).max() <= 0.05 * travel
    assert np.abs(st.L - L).max() > 0.3 * travel                 # ... and the factors did move


def test_full_size_layer_first_step(oracle):
    """The 1152 -> 3456 projection of configuration 2 (N = 3456, K = 1152, r = 32, groups of 64)."""
    N, K, r, g = 3456, 1152, 32, 64
    W, L, R = _problem(N, K, r, seed=2)
    cfg = _cfg(N, K, r, g, False)
    Wd = torch.from_numpy(W).cuda()
    state = lq.lq_calib_init(cfg, torch.from_numpy(L).cuda(), torch.from_numpy(R).cuda())
    st = oracle.calib_init(L, R)
    out, got, loss, bL, bR = _check_step(oracle, cfg, W, Wd, state, st, 1, 1e-4, g, False)
    assert np.array_equal(_n(got["E"]), out.E)
    assert abs(loss - out.loss) <= 1e-5 * out.loss
    assert np.all(np.abs(_n(got["gL"]) - out.gL) <= bL) and np.all(np.abs(_n(got["gR"]) - out.gR) <= bR)
    assert np.abs(_n(got["L"]) - st.L).max() <= 2e-5 and np.abs(_n(got["R"]) - st.R).max() <= 2e-5


def test_thousand_steps_from_the_svd_start_at_a_layer_shape(oracle):
    """The optimisation as the paper runs it (Section 3.2; App. A.2: Adam, lr 1e-4, on the order of a thousand steps) on
    the 1152 -> 3456 projection: start L = -L0, R = R0 from the best rank-32 approximation of W, 1000 steps on the GPU.
    The loss of Eq. 4 falls well below that of the start and keeps falling (compared over windows: single steps jitter,
    the rounding has no gradient); after the run the state is still the oracle's state: from the GPU's factors one more
    step on both sides gives the same error matrix bit for bit, the same loss and gradients within the accumulation bound."""
    N, K, r, g = 3456, 1152, 32, 64
    W, L, R = _problem(N, K, r, seed=21)
    cfg = _cfg(N, K, r, g, False)
    Wd = torch.from_numpy(W).cuda()
    state = lq.lq_calib_init(cfg, torch.from_numpy(L).cuda(), torch.from_numpy(R).cuda())
    steps, lr = 1000, 1e-4
    losses = torch.zeros(steps, dtype=torch.float32, device="cuda")
    for t in range(1, steps + 1):
        lq.lq_calib_step(cfg, Wd, state, t, lr=lr, loss=losses[t - 1:t])
    torch.cuda.synchronize()
    ls = _n(losses).astype(np.float64)
    assert np.all(np.isfinite(ls)) and np.all(ls > 0)
    w = ls.reshape(10, 100).mean(axis=1)
    print("[calib] mean loss per 100 steps, relative to the start:", np.round(w / ls[0], 4))
    assert w[-1] < 0.9 * ls[0], "1000 steps lower the loss of the SVD start by more than a tenth"
    assert np.all(np.diff(w) < 0.002 * ls[0]), "the windowed loss does not rise"
    got = lq.lq_calib_unpack(cfg, state, ("L", "R"))
    torch.cuda.synchronize()
    Lg, Rg = _n(got["L"]).copy(), _n(got["R"]).copy()
    assert np.abs(Lg - L).max() > 10 * lr                         # the factors travelled
    # one more step from these factors on both sides (fresh moments on both: step number 1)
    st = oracle.calib_init(Lg, Rg)
    state2 = lq.lq_calib_init(cfg, torch.from_numpy(Lg).cuda(), torch.from_numpy(Rg).cuda())
    out, got2, loss, bL, bR = _check_step(oracle, cfg, W, Wd, state2, st, 1, lr, g, False)
    assert np.array_equal(_n(got2["E"]), out.E)
    assert abs(loss - out.loss) <= 1e-5 * out.loss
    assert np.all(np.abs(_n(got2["gL"]) - out.gL) <= bL) and np.all(np.abs(_n(got2["gR"]) - out.gR) <= bR)
    # the loss the optimiser reported last belongs to (almost) these factors: one step of lr 1e-4 apart
    assert abs(out.loss - ls[-1]) <= 0.02 * ls[-1]


def test_calibrated_factors_feed_the_forward(oracle):
    """End to end: optimise, hand -L and R to lq_pack_weights (it forms W - L' R'), and the packed main codes are
    Q1(W + L R) of the calibration, i.e. the residual whose rounding error the branch now carries."""
    N, K, r, g = 128, 256, 16, 64
    W, L, R = _problem(N, K, r, seed=9)
    cfg = _cfg(N, K, r, g, False)
    Wd = torch.from_numpy(W).cuda()
    state = lq.lq_calib_init(cfg, torch.from_numpy(L).cuda(), torch.from_numpy(R).cuda())
    for t in range(1, 21):
        lq.lq_calib_step(cfg, Wd, state, t)
    f = lq.lq_calib_unpack(cfg, state)
    cfg_fp = lq.make_config(N, K, r, "int", g, 8, 8, residual_from_quantized=False)
    packed = lq.lq_pack_weights(cfg_fp, Wd, (-f["L"]).contiguous(), f["R"])
    wv = lq.lq_unpack_weights(cfg_fp, packed)
    torch.cuda.synchronize()
    Lc, Rc = _n(f["L"]), _n(f["R"])
    pk = oracle.pack_int(W, -Lc, Rc, g, 8, residual_from_quantized=False)
    assert np.array_equal(_n(wv.pq), pk.pq) and np.array_equal(_n(wv.sw), pk.sw)
    # the residual the pack step quantises is W + L R (fp64 sum rounded once there, an fp32 chain in the calibration)
    V = W.astype(np.float64) + Lc.astype(np.float64) @ Rc.astype(np.float64)
    assert np.allclose(pk.P, V, rtol=0, atol=1e-6 * np.abs(V).max())


def test_step_in_a_hip_graph(oracle):
    """A step is four kernel launches and nothing else, so it can be captured; the step number (bias correction) is a
    launch argument, so replays repeat that step number: compared with eager calls at the same number."""
    N, K, r, g = 128, 256, 16, 64
    W, L, R = _problem(N, K, r, seed=12)
    cfg = _cfg(N, K, r, g, False)
    Wd = torch.from_numpy(W).cuda()
    Ld, Rd = torch.from_numpy(L).cuda(), torch.from_numpy(R).cuda()
    eager = lq.lq_calib_init(cfg, Ld, Rd)
    loss_e = torch.zeros(1, dtype=torch.float32, device="cuda")
    for _ in range(5):
        lq.lq_calib_step(cfg, Wd, eager, 3, loss=loss_e)
    torch.cuda.synchronize()
    state = lq.lq_calib_init(cfg, Ld, Rd)
    loss_g = torch.zeros(1, dtype=torch.float32, device="cuda")
    graph = torch.cuda.CUDAGraph()
    s = torch.cuda.Stream()
    s.wait_stream(torch.cuda.current_stream())
    torch.cuda.synchronize()
    with torch.cuda.graph(graph, stream=s):
        lq.lq_calib_step(cfg, Wd, state, 3, loss=loss_g)
    for rep in range(5):
        graph.replay()
        torch.cuda.synchronize()
        _ = lq.lq_calib_unpack(cfg, eager, ("L",))          # eager work of the library between replays
        torch.cuda.synchronize()
    names = ("L", "R", "mL", "vL", "mR", "vR", "gL", "gR", "E")
    a, b = lq.lq_calib_unpack(cfg, eager, names), lq.lq_calib_unpack(cfg, state, names)
    torch.cuda.synchronize()
    for k in names:
        assert torch.equal(a[k], b[k]), k
    assert loss_e.item() == loss_g.item()

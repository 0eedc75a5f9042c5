"""Rotation search (Section 3.3, Eq. 6-7) on the GPU against the CPU oracle, through the C-ABI.

Bars: the quantisation errors E1, E2 come from fp32 chains in a fixed order and an integer decision, so they are
compared bit for bit; the gradient is an fp32 sum of ~N + K products per entry against the oracle's fp64 sum
(1e-5 of its largest entry); the r x r update runs in fp32 against fp64 (dot products of length r, a handful of them
chained): 2e-6 absolute on Omega (entries of size <= 1), 1e-5 relative to the largest entry on the momentum."""
import numpy as np
import pytest
import torch

from paper_2604_18117_amd import workloads as wl

pytestmark = pytest.mark.gpu


def _case(N, K, r, seed, outlier=8.0):
    rng = np.random.default_rng(seed)
    L = (rng.standard_normal((N, r)) * 0.05).astype(np.float32)
    R = (rng.standard_normal((r, K)) * 0.05).astype(np.float32)
    L[:, 3] *= outlier
    R[5, :] *= outlier
    X0 = np.linalg.qr(rng.standard_normal((r, r)))[0].astype(np.float32)
    M0 = (rng.standard_normal((r, r)) * 1e-3).astype(np.float32)
    return L, R, X0, M0


FAMILY = {"int": "int", "fp8": "mx", "mxfp8": "mxb", "mxfp6": "mxb", "mxint": "mxi"}


def _cfg(lq, N, K, r, bits, q2="int"):
    if q2 == "int":
        return lq.make_config(N, K, r, "int", 64, bits, 8)
    return lq.make_config(N, K, r, FAMILY[q2], 32, bits, 8)


def _d(a):
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def _compare_step(oracle, lq, N, K, r, bits, seed, X0=None, M0=None, q2="int", **opt):
    L, R, Xr, Mr = _case(N, K, r, seed)
    X0 = Xr if X0 is None else X0
    M0 = Mr if M0 is None else M0
    cfg = _cfg(lq, N, K, r, bits, q2)
    Ld, Rd = _d(L), _d(R)
    state = lq.lq_rot_init(cfg, _d(X0), _d(M0))
    loss = torch.zeros(1, dtype=torch.float32, device="cuda")
    lq.lq_rot_step(cfg, Ld, Rd, state, loss=loss, **opt)
    got = {k: v.cpu().numpy() for k, v in lq.lq_rot_unpack(cfg, state, ("Omega", "Mom", "G", "E1", "E2")).items()}
    st = oracle.rot_init(r, X0, M0)
    ref = oracle.rot_step(L, R, st, bits=bits, q2=q2, **opt)
    assert np.array_equal(got["E1"], ref.E1), "E1 differs"
    assert np.array_equal(got["E2"], ref.E2), "E2 differs"
    assert float(loss.item()) == pytest.approx(ref.loss, rel=1e-5)
    gmax = np.abs(ref.G).max()
    assert np.abs(got["G"] - ref.G).max() <= 1e-5 * gmax + 1e-30
    assert np.abs(got["Omega"] - st.Omega).max() <= 2e-6
    mmax = max(np.abs(st.Mom).max(), 1e-30)
    assert np.abs(got["Mom"] - st.Mom).max() <= 1e-5 * mmax
    return got, st


@pytest.mark.parametrize("N,K,r,bits", [(192, 320, 16, 8), (300, 448, 32, 4), (1000, 1152, 32, 8), (130, 192, 64, 6),
                                        (257, 704, 96, 6), (520, 1344, 128, 8)])
def test_one_step_matches_the_oracle(oracle, N, K, r, bits):
    """Every rank the branch supports, ragged N (not a multiple of the 256 rows a workgroup takes), K not a multiple of 256;
    a step long enough to exercise the fixed-point passes (grad_scale brings alpha ||W|| / 2 to the order of 0.1)."""
    from paper_2604_18117_amd import binding as lq
    N = (N + 63) // 64 * 64 if N % 64 else N   # cfg.N must be a multiple of 64
    _compare_step(oracle, lq, N, K, r, bits, seed=N + K + r, lr=0.5, beta=0.9, s=2, grad_scale=2500.0)


@pytest.mark.parametrize("name,bits", [("c2_qkv", 8), ("c4_qkv", 6), ("c3_fc2", 4)])
def test_full_size_layers(oracle, name, bits):
    """The factor shapes of the benchmark layers (3456 x 32 / 32 x 1152, 6720 x 64 / 64 x 2240, 1152 x 32 / 32 x 4608)."""
    from paper_2604_18117_amd import binding as lq
    l = wl.LAYERS[name]
    _compare_step(oracle, lq, l.N, l.K, l.r, bits, seed=7, lr=0.5, beta=0.9, s=2, grad_scale=20000.0)


@pytest.mark.parametrize("q2,bits", [("fp8", 8), ("mxfp8", 8), ("mxfp6", 6), ("mxint", 8), ("mxint", 4)])
@pytest.mark.parametrize("N,K,r", [(320, 448, 32), (192, 2240, 64), (576, 1344, 128), (1152, 1152, 96)])
def test_mx_branch_formats_as_q2(oracle, q2, bits, N, K, r):
    """Q2 = the branch weight format of the MX families: E4M3 with a per-row fp32 scale (config 5), MXFP8e4, MXFP6e2, MXINT8
    and MXINT4 blocks of 32 along the rows of L Omega and Omega^T R.  K = 2240 is 35 chunks of 64 (the search works on
    the caller's K, not the padded layout); K = 448 and 1344 end inside a 256-column workgroup."""
    from paper_2604_18117_amd import binding as lq
    if q2 == "fp8" and r == 96:
        pytest.skip("rank 96 is not a rank of the fp32-scaled FP8 branch")
    _compare_step(oracle, lq, N, K, r, bits, seed=N + r, q2=q2, lr=0.5, beta=0.9, s=2, grad_scale=2500.0)


def test_defaults_identity_start_and_more_passes(oracle):
    """lq_rot_init without matrices starts at the identity with zero momentum; the paper's learning rate with the loss as
    printed (grad_scale 1); s = 5 passes; beta = 0."""
    from paper_2604_18117_amd import binding as lq
    N, K, r = 320, 512, 32
    L, R, _, _ = _case(N, K, r, 3)
    cfg = _cfg(lq, N, K, r, 8)
    state = lq.lq_rot_init(cfg)
    v = lq.lq_rot_unpack(cfg, state, ("Omega", "Mom"))
    assert torch.equal(v["Omega"], torch.eye(r, device="cuda")) and not bool(v["Mom"].any())
    _compare_step(oracle, lq, N, K, r, 8, seed=3, X0=np.eye(r, dtype=np.float32), M0=np.zeros((r, r), np.float32), lr=0.5)
    _compare_step(oracle, lq, N, K, r, 4, seed=4, lr=0.1, beta=0.0, s=5, grad_scale=3000.0)


def test_trajectory_stays_orthogonal_and_tracks_the_oracle(oracle):
    """Ten steps along the oracle's trajectory, the GPU restarted from the oracle's state before each (the errors are a
    discontinuous function of Omega, so free-running fp32 and fp64 trajectories part ways after a code flips; each
    step is held to the one-step bars instead), then ten free-running GPU steps: the loss stays close to the oracle's,
    Omega stays near-orthogonal and moves."""
    from paper_2604_18117_amd import binding as lq
    N, K, r = 256, 384, 32
    L, R, X0, _ = _case(N, K, r, 11)
    cfg = _cfg(lq, N, K, r, 4)
    Ld, Rd = _d(L), _d(R)
    opt = dict(lr=0.5, beta=0.9, s=2, grad_scale=2000.0)
    st = oracle.rot_init(r, X0)
    losses = []
    for _ in range(10):
        state = lq.lq_rot_init(cfg, _d(st.Omega), _d(st.Mom))
        lq.lq_rot_step(cfg, Ld, Rd, state, **opt)
        got = {k: v.cpu().numpy() for k, v in lq.lq_rot_unpack(cfg, state, ("Omega", "Mom", "E1", "E2")).items()}
        ref = oracle.rot_step(L, R, st, bits=4, **opt)
        losses.append(ref.loss)
        assert np.array_equal(got["E1"], ref.E1) and np.array_equal(got["E2"], ref.E2)
        assert np.abs(got["Omega"] - st.Omega).max() <= 2e-6
        assert np.abs(got["Mom"] - st.Mom).max() <= 1e-5 * np.abs(st.Mom).max()
    state = lq.lq_rot_init(cfg, _d(X0))
    loss = torch.zeros(1, dtype=torch.float32, device="cuda")
    for t in range(10):
        lq.lq_rot_step(cfg, Ld, Rd, state, loss=loss, **opt)
        assert float(loss.item()) == pytest.approx(losses[t], rel=5e-2)
    Om = lq.lq_rot_unpack(cfg, state, ("Omega",))["Omega"].cpu().numpy().astype(np.float64)
    assert np.abs(Om.T @ Om - np.eye(r)).max() < 5e-2          # ten approximate Cayley transforms (a <= 0.5 each)
    assert np.abs(Om - X0).max() > 1e-3                        # and it moved


def test_apply_and_hand_off_to_pack(oracle):
    """lq_rot_apply gives exactly the oracle's rotated factors (same fp32 chains); packing them is packing the oracle's."""
    from paper_2604_18117_amd import binding as lq
    N, K, r = 192, 320, 32
    L, R, X0, _ = _case(N, K, r, 21)
    cfg = _cfg(lq, N, K, r, 8)
    state = lq.lq_rot_init(cfg, _d(X0))
    Lr, Rr = lq.lq_rot_apply(cfg, _d(L), _d(R), state)
    Lo, Ro = oracle.rot_apply(L, R, X0)
    assert np.array_equal(Lr.cpu().numpy(), Lo) and np.array_equal(Rr.cpu().numpy(), Ro)
    rng = np.random.default_rng(5)
    W = (rng.standard_normal((N, K)) * 0.02).astype(np.float32)
    packed = lq.lq_pack_weights(cfg, _d(W), Lr, Rr)
    wv = lq.lq_unpack_weights(cfg, packed)
    pk = oracle.pack_int(W, Lo, Ro, 64, 8)
    assert np.array_equal(wv.pq.cpu().numpy(), pk.pq) and np.array_equal(wv.lq.cpu().numpy(), pk.lq)
    assert np.array_equal(wv.rq.cpu().numpy(), pk.rq)


@pytest.mark.parametrize("r", [32, 128])
def test_step_is_reproducible_and_capturable(oracle, r):
    """Two runs give the same bits; a step captured in a HIP graph replays to the same state as eager steps (rank 128 asks
    the runtime for a larger LDS limit on its first, eager, call only: the captured call just launches)."""
    from paper_2604_18117_amd import binding as lq
    N, K = 256, 384
    L, R, X0, M0 = _case(N, K, r, 31)
    cfg = _cfg(lq, N, K, r, 6)
    Ld, Rd = _d(L), _d(R)

    def run(nsteps):
        state = lq.lq_rot_init(cfg, _d(X0), _d(M0))
        for _ in range(nsteps):
            lq.lq_rot_step(cfg, Ld, Rd, state, grad_scale=1500.0)
        return lq.lq_rot_unpack(cfg, state, ("Omega", "Mom", "G"))

    a, b = run(3), run(3)
    assert all(torch.equal(a[k], b[k]) for k in a)
    state = lq.lq_rot_init(cfg, _d(X0), _d(M0))
    graph = torch.cuda.CUDAGraph()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    torch.cuda.synchronize()
    with torch.cuda.graph(graph, stream=side):
        lq.lq_rot_step(cfg, Ld, Rd, state, grad_scale=1500.0)
    for _ in range(3):
        graph.replay()
        torch.cuda.synchronize()
        _ = lq.lq_rot_unpack(cfg, state, ("G",))                   # eager work of the library between replays
        torch.cuda.synchronize()
    c = lq.lq_rot_unpack(cfg, state, ("Omega", "Mom", "G"))
    assert all(torch.equal(a[k], c[k]) for k in a)


def test_search_lowers_the_loss_and_keeps_the_product(oracle):
    """300 free-running steps on factors with one outlier column / row (4-bit Q2, grad_scale 1e3): Eq. 7 falls by more than
    a fifth (the oracle run alongside falls by as much), Omega stays orthogonal, and the rotated factors multiply to the same L R."""
    from paper_2604_18117_amd import binding as lq
    rng = np.random.default_rng(0)
    N, K, r = 512, 512, 32
    L = (rng.standard_normal((N, r)) * 0.05).astype(np.float32)
    R = (rng.standard_normal((r, K)) * 0.05).astype(np.float32)
    L[:, 3] *= 8
    R[5, :] *= 8
    cfg = _cfg(lq, N, K, r, 4)
    Ld, Rd = _d(L), _d(R)
    state = lq.lq_rot_init(cfg)
    st = oracle.rot_init(r)
    loss = torch.zeros(1, dtype=torch.float32, device="cuda")
    first = last = None
    for t in range(300):
        lq.lq_rot_step(cfg, Ld, Rd, state, lr=0.5, beta=0.9, s=2, grad_scale=1e3, loss=loss)
        ref = oracle.rot_step(L, R, st, bits=4, lr=0.5, beta=0.9, s=2, grad_scale=1e3)
        if t == 0:
            first = float(loss.item())
            assert first == pytest.approx(ref.loss, rel=1e-5)
        if t == 299:
            last = float(loss.item())
            assert ref.loss < 0.8 * first
    assert last < 0.8 * first
    Om = lq.lq_rot_unpack(cfg, state, ("Omega",))["Omega"].cpu().numpy().astype(np.float64)
    assert np.abs(Om.T @ Om - np.eye(r)).max() < 1e-3
    Lr, Rr = lq.lq_rot_apply(cfg, Ld, Rd, state)
    P0 = L.astype(np.float64) @ R.astype(np.float64)
    P1 = Lr.cpu().numpy().astype(np.float64) @ Rr.cpu().numpy().astype(np.float64)
    assert np.abs(P1 - P0).max() < 2e-3 * np.abs(P0).max()

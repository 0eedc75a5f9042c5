"""GPU parity, INT family: the HIP library against the CPU oracle, element by element.

Bar: codes, scales computed from source data, and all integer accumulators bit-exact; the
fp32 value before the final rounding and the bf16 output bit-exact as well (the kernel keeps
the oracle's ascending-group FMA order), which is stronger than the 2e-3 relative bound.
"""
import numpy as np
import pytest
import torch

from paper_2604_18117_amd import workloads as wl
from tests.smoothing import smoothing_vector
from tests.gpu_util import bf16_to_bits, n, run_gpu, run_oracle_int

pytestmark = pytest.mark.gpu


def _compare_all(oracle, layer, X, W, L, R, check_acc=True):
    g = run_gpu(layer, X, W, L, R, debug=True, debug_acc=check_acc)
    pk, act, out = run_oracle_int(oracle, layer, X, W, L, R, want_acc=True)
    r = layer.r
    # offline packing
    assert np.array_equal(n(g.wv.pq), pk.pq), "pq"
    assert np.array_equal(n(g.wv.sw), pk.sw), "sw"
    assert np.array_equal(n(g.wv.sl), pk.sl), "sl"
    if r:
        assert np.array_equal(n(g.wv.lq), pk.lq), "lq"
        assert np.array_equal(n(g.wv.rq), pk.rq), "rq"
        assert np.array_equal(n(g.wv.sr), pk.sr), "sr"
    # activation step
    assert np.array_equal(n(g.av.xq), act.xq), "xq"
    assert np.array_equal(n(g.av.sx), act.sx), "sx"
    if r:
        assert np.array_equal(n(g.adbg.xb), act.xb), "xb"
        assert np.array_equal(n(g.adbg.sxb), act.sxb), "sxb"
        assert np.array_equal(n(g.adbg.accT), act.accT), "accT"
        assert np.array_equal(n(g.adbg.T), act.T), "T"
        assert np.array_equal(n(g.av.tq), act.tq), "tq"
        assert np.array_equal(n(g.av.st), act.st), "st"
    # forward
    if check_acc:
        assert np.array_equal(n(g.fdbg.acc), out.acc), "acc"
    assert np.array_equal(n(g.fdbg.acc2), out.acc2), "acc2"
    assert np.array_equal(n(g.fdbg.y32), out.y32), "y32"
    Yb = bf16_to_bits(g.Y)
    assert np.array_equal(Yb, out.Y), "Y"
    # the stated bar, spelled out: |Y - y32| within bf16 rounding of the oracle's fp32 value
    Yf = oracle.bf16_bits_to_f32(Yb).astype(np.float64)
    tau = 1e-3 * np.sqrt(np.mean(out.y32.astype(np.float64) ** 2))
    rel = np.abs(Yf - oracle.bf16_bits_to_f32(out.Y)) / np.maximum(np.maximum(np.abs(out.y32), tau), 1e-30)
    assert rel.max() <= 2e-3
    # production (no taps) launch gives the same bits
    g2 = run_gpu(layer, X, W, L, R, debug=False)
    assert torch.equal(g2.Y, g.Y)
    return g


SMALL = [
    # M (ragged), K, N (partial 256-wide tile), r, g, bw, ba, x_dtype
    (300, 256, 320, 16, 64, 8, 8, "bf16"),
    (77, 192, 64, 32, 64, 8, 8, "f32"),
    (513, 384, 576, 64, 64, 6, 6, "bf16"),
    (260, 256, 128, 32, 128, 4, 8, "bf16"),
    (33, 640, 192, 128, 128, 8, 8, "bf16"),
    (64, 128, 64, 0, 64, 8, 8, "bf16"),
    (1, 64, 64, 16, 64, 8, 8, "f32"),
    (200, 448, 320, 96, 64, 6, 6, "bf16"),    # rank 96: the 6-bit point of a 512-bit budget (85) padded
    (90, 256, 128, 96, 128, 6, 6, "f32"),
    (50, 64, 128, 128, 64, 8, 8, "bf16"),    # rank > K: the factor views are larger than N x K
    (33, 64, 192, 96, 64, 6, 6, "f32"),
]


@pytest.mark.parametrize("M,K,N,r,g,bw,ba,xd", SMALL)
def test_small_shapes_bit_exact(oracle, M, K, N, r, g, bw, ba, xd):
    layer = wl.Layer("t", M, K, N, r, "int", g, bw, ba, xd, outlier_scale=15.0, n_outliers=max(1, K // 100), seed=M + K)
    X, W, L, R = wl.make_inputs(layer)
    _compare_all(oracle, layer, X, W, L, R)


@pytest.mark.parametrize("M,K,N,r,g,bw,ba", [(2000, 128, 2304, 16, 64, 8, 8), (2100, 256, 2304, 32, 128, 4, 8),
                                                 (2100, 128, 2176, 32, 64, 8, 8), (2100, 128, 2240, 32, 64, 8, 8),
                                                 (4000, 128, 2304, 32, 64, 8, 8), (4100, 192, 2176, 64, 64, 6, 6),
                                                 (4000, 256, 2240, 32, 128, 4, 8), (2100, 128, 2112, 32, 64, 6, 6),
                                                 (2100, 256, 2112, 32, 128, 4, 8)])
def test_full_tiles_bit_exact(oracle, M, K, N, r, g, bw, ba):
    """Large enough (more than a quarter of the device's workgroup slots) that the grid runs
    full 128 x 256 tiles, the small shapes above run as half tiles; ragged last row tile; the third
    case has a last tile column with 128 valid channels (wavefronts arranged 2 x 2 there), the last two one with 64 (three of
    its four wavefronts only stage), the fourth one with 192 (its
    fourth wavefront only stages).  The last three have between one 128-row tile per compute unit and one per workgroup
    slot and therefore run as 96-row tiles (ragged last tile of one or two row blocks; last tile column of 128 or 192
    channels, whose wavefronts past the end only stage; 64- and 128-deep groups)."""
    layer = wl.Layer("t", M, K, N, r, "int", g, bw, ba, "bf16", outlier_scale=15.0, n_outliers=2, seed=M + K)
    X, W, L, R = wl.make_inputs(layer)
    _compare_all(oracle, layer, X, W, L, R)


def test_config1_exact(oracle):
    layer = wl.LAYERS["c1_single"]
    X, W, L, R = wl.make_inputs(layer)
    _compare_all(oracle, layer, X, W, L, R)


def test_degenerate_inputs(oracle):
    layer = wl.Layer("t", 70, 128, 64, 16, "int", 64, 8, 8, "bf16", seed=3)
    X, W, L, R = wl.make_inputs(layer)
    X[3] = 0.0            # an all-zero token
    X[5, :] = 0.0
    X[5, 7] = -2.0        # a one-hot token
    W[2] = 0.0            # an all-zero output channel
    L[4] = 0.0
    R[1] = 0.0
    _compare_all(oracle, layer, X, W, L, R)
    _compare_all(oracle, layer, np.zeros_like(X), W, L, R)


@pytest.mark.parametrize("xd,a_group", [("bf16", 0), ("f32", 0), ("bf16", 64), ("f32", 64)])
def test_main_codes_on_exact_ties_and_tiny_values(oracle, xd, a_group):
    """Rows whose scaled values x * (7 / amax) are exact half-integers (ties go to even), whole integers, values just
    below and above a tie, values far below half a step (codes +0 / -0), and the extremes +-amax: the main codes come
    from the hardware FP6 converter and must equal the oracle's nearest-even integers."""
    layer = wl.Layer("t", 96, 256, 64, 16, "int", 64, 8, 8, xd, seed=11, a_group=a_group)
    X, W, L, R = wl.make_inputs(layer)
    rng = np.random.default_rng(4)
    halves = (rng.integers(-14, 15, size=X.shape) * 0.5).astype(np.float32)          # multiples of 1/2 in [-7, 7]
    for m in range(X.shape[0]):
        scale = np.float32(2.0 ** (m % 9 - 4))
        row = halves[m] * scale
        if m % 3 == 1:   # one ulp (of the input type) to either side of the ties
            eps = np.float32(2.0 ** -7 if xd == "bf16" else 2.0 ** -22)
            row = row * (1 + eps * rng.choice([-1.0, 1.0], size=row.shape).astype(np.float32))
        if m % 3 == 2:   # tiny magnitudes of both signs next to the extremes
            row = (rng.standard_normal(row.shape) * 1e-6).astype(np.float32) * scale
        for b in range(0, X.shape[1], 64):   # every block of 64 holds +-7 * scale, so block scales equal the row scale
            row[b] = 7 * scale
            row[b + 1] = -7 * scale
        X[m] = row
    X = wl.round_to_bf16(X) if xd == "bf16" else X
    _compare_all(oracle, layer, X, W, L, R)


def test_rank0_equals_plain_w4a4_on_gpu(oracle):
    layer = wl.Layer("t", 96, 256, 128, 32, "int", 64, 8, 8, "bf16", seed=9)
    X, W, L, R = wl.make_inputs(layer)
    g0 = run_gpu(wl.shrink(layer, r=0), X, W, None, None, debug=False)
    gz = run_gpu(layer, X, W, np.zeros_like(L), np.zeros_like(R), debug=False)
    assert torch.equal(g0.Y, gz.Y)


def test_strided_x_and_determinism(oracle):
    from paper_2604_18117_amd import binding as lq
    layer = wl.Layer("t", 130, 256, 192, 32, "int", 64, 8, 8, "bf16", seed=11)
    X, W, L, R = wl.make_inputs(layer)
    g = run_gpu(layer, X, W, L, R, debug=False)
    from tests.gpu_util import to_dev_x
    Xd = to_dev_x(X, "bf16")
    wide = torch.zeros((130, 256 + 64), dtype=torch.bfloat16, device="cuda")
    wide[:, :256] = Xd
    act = lq.lq_quantize_act(g.cfg, g.packed, wide[:, :256])
    Ywide = torch.zeros((130, 192 + 8), dtype=torch.bfloat16, device="cuda")
    lq.lq_linear_lowrank_fwd(g.cfg, g.packed, act, 130, Y=Ywide[:, :192])
    torch.cuda.synchronize()
    assert torch.equal(Ywide[:, :192], g.Y) and not Ywide[:, 192:].any()
    for _ in range(3):
        assert torch.equal(run_gpu(layer, X, W, L, R, debug=False).Y, g.Y)


@pytest.mark.parametrize("name", ["c2_qkv", "c3_fc1", "c3_fc2", "c4_qkv", "c4_expand"])
def test_full_size_sampled_rows(oracle, name):
    _full_size_sampled(oracle, name)


def _full_size_sampled(oracle, name):
    """Full-size layer in the launch configuration the bench times; the oracle recomputes a
    sample of token rows (rows are independent through the whole path)."""
    layer = wl.LAYERS[name]
    X, W, L, R = wl.make_inputs(layer)
    g = run_gpu(layer, X, W, L, R, debug=False)
    rng = np.random.default_rng(1)
    # first and last rows, both halves of the last row tile (the tail of the grid may run as half
    # tiles), and a random sample
    fixed = [0, layer.M - 1, layer.M - 40, layer.M - 100]
    rows = np.unique(np.concatenate([fixed, rng.choice(layer.M, 20, replace=False)]))
    pk, act, out = run_oracle_int(oracle, layer, X[rows], W, L, R, want_acc=False)
    av = n(g.av.xq) if g.av is not None else None
    from paper_2604_18117_amd import binding as lq
    av = lq.lq_unpack_act(g.cfg, g.act, layer.M)
    wv = lq.lq_unpack_weights(g.cfg, g.packed)
    assert np.array_equal(n(wv.pq), pk.pq) and np.array_equal(n(wv.sw), pk.sw)
    assert np.array_equal(n(wv.lq), pk.lq) and np.array_equal(n(wv.rq), pk.rq)
    assert np.array_equal(n(av.xq)[rows], act.xq) and np.array_equal(n(av.sx)[rows], act.sx)
    assert np.array_equal(n(av.tq)[rows], act.tq) and np.array_equal(n(av.st)[rows], act.st)
    Yb = bf16_to_bits(g.Y)[rows]
    assert np.array_equal(Yb, out.Y)


@pytest.mark.parametrize("name", ["c2_qkv", "c3_fc1", "c3_fc2", "c4_qkv", "c4_expand"])
def test_full_size_whole_tile_row_and_column_panel(oracle, name):
    """Full-size layer with the accumulator taps on: one whole interior 128-row tile row (every channel) and one whole
    interior 256-column panel (every token) against the oracle, per-group accumulators included.  A wrong tile anywhere
    on that row or in that panel (tile order, panel order, the grid's tail) shows up here, which a sample of token rows
    can only see through the never-written check.  The oracle computes the panel from the same channels of W and L
    (channels are independent through the whole path, like token rows)."""
    layer = wl.LAYERS[name]
    X, W, L, R = wl.make_inputs(layer)
    g = run_gpu(layer, X, W, L, R, debug=True, debug_acc=True)
    tm = (layer.M // 128) * 5 // 8
    rows = slice(tm * 128, tm * 128 + 128)
    pk, act, out = run_oracle_int(oracle, layer, X[rows], W, L, R, want_acc=True)
    assert np.array_equal(n(g.fdbg.acc[rows]), out.acc), "acc, tile row"
    assert np.array_equal(n(g.fdbg.acc2[rows]), out.acc2), "acc2, tile row"
    assert np.array_equal(n(g.fdbg.y32[rows]), out.y32), "y32, tile row"
    assert np.array_equal(bf16_to_bits(g.Y[rows]), out.Y), "Y, tile row"
    tn = ((layer.N + 255) // 256) * 3 // 7
    cols = slice(tn * 256, tn * 256 + 256)
    pk, act, out = run_oracle_int(oracle, layer, X, W[cols], L[cols], R, want_acc=True)
    assert np.array_equal(n(g.fdbg.acc[:, cols].contiguous()), out.acc), "acc, column panel"
    assert np.array_equal(n(g.fdbg.acc2[:, cols].contiguous()), out.acc2), "acc2, column panel"
    assert np.array_equal(n(g.fdbg.y32[:, cols].contiguous()), out.y32), "y32, column panel"
    assert np.array_equal(bf16_to_bits(g.Y[:, cols]), out.Y), "Y, column panel"


@pytest.mark.parametrize("M,K,N,r,xd,ag", [(200, 1152, 320, 32, "bf16", 0), (77, 2304, 64, 16, "f32", 0), (33, 256, 64, 0, "bf16", 0),
                                              (200, 1152, 320, 32, "bf16", 64), (77, 2304, 64, 16, "f32", 64)])
def test_fused_smoothing(oracle, M, K, N, r, xd, ag):
    """Activation smoothing (Section 3.4; App. A.1) fused into the activation kernel: the GPU is given the raw X
    and the smoothing vector; the oracle quantises the smoothed input.  Everything bit-exact as for the plain path.
    ag = 64: together with SINT4 blocks for the main operands (the paper's literal SINT4 setting)."""
    import torch
    from paper_2604_18117_amd import binding as lq
    from tests.gpu_util import to_dev_x
    layer = wl.shrink(wl.LAYERS["c2_qkv"], M=M, K=K, N=N, r=r)
    layer = wl.Layer(**{**layer.__dict__, "x_dtype": xd, "seed": M + K, "a_group": ag})
    X, W, L, R = wl.make_inputs(layer)
    gamma = smoothing_vector(X, W)
    Ws = (W.astype(np.float64) * gamma).astype(np.float32)       # the caller folds gamma into W before packing
    cfg = lq.config_for_layer(layer, smooth=True)
    packed = lq.lq_pack_weights(cfg, torch.from_numpy(Ws).cuda(), torch.from_numpy(L).cuda() if r else None,
                                torch.from_numpy(R).cuda() if r else None)
    Xd = to_dev_x(X, xd)
    # before lq_set_smoothing the blob holds reciprocals 1: the plain path
    a0 = lq.lq_quantize_act(cfg, packed, Xd)
    pk = oracle.pack_int(Ws, L if r else None, R if r else None, layer.g, layer.br_w_bits, sint4_blocks=ag == 64)
    act0 = oracle.quantize_act_int(X, pk, layer.br_a_bits)
    assert np.array_equal(n(lq.lq_unpack_act(cfg, a0, M).xq), act0.xq)
    lq.lq_set_smoothing(cfg, packed, torch.from_numpy(gamma).cuda())
    act_g, adbg = lq.lq_quantize_act(cfg, packed, Xd, debug=True)
    Y, fdbg = lq.lq_linear_lowrank_fwd(cfg, packed, act_g, M, debug=True, debug_acc=False)
    av = lq.lq_unpack_act(cfg, act_g, M)
    torch.cuda.synchronize()
    Xs = oracle.smooth(X, gamma)
    act = oracle.quantize_act_int(Xs, pk, layer.br_a_bits)
    out = oracle.fwd_int(pk, act, want_acc=False)
    assert np.array_equal(n(av.xq), act.xq) and np.array_equal(n(av.sx), act.sx)
    if r:
        assert np.array_equal(n(adbg.xb), act.xb) and np.array_equal(n(adbg.sxb), act.sxb)
        assert np.array_equal(n(adbg.accT), act.accT) and np.array_equal(n(adbg.T), act.T)
        assert np.array_equal(n(av.tq), act.tq) and np.array_equal(n(av.st), act.st)
    assert np.array_equal(n(fdbg.y32), out.y32)
    assert np.array_equal(bf16_to_bits(Y), out.Y)
    assert not np.array_equal(act.xq, act0.xq)                   # the smoothing did change the codes


# ---- SINT4 blocks for both operands of the main product (App. A.3: 64 values, one FP16 scale) ------------------------

SINT4_SMALL = [
    # M (ragged), K, N, r, bw, ba, x_dtype
    (300, 256, 320, 16, 8, 8, "bf16"),
    (77, 192, 64, 32, 8, 8, "f32"),
    (513, 384, 576, 64, 6, 6, "bf16"),
    (97, 1152, 128, 128, 4, 8, "bf16"),      # 97 tokens: a last 128-row tile with one real row block
    (64, 128, 64, 0, 8, 8, "bf16"),
    (1, 64, 64, 16, 8, 8, "f32"),
    (130, 320, 192, 96, 6, 6, "bf16"),
]


@pytest.mark.parametrize("M,K,N,r,bw,ba,xd", SINT4_SMALL)
def test_sint4_blocks_small_shapes_bit_exact(oracle, M, K, N, r, bw, ba, xd):
    layer = wl.Layer("t", M, K, N, r, "int", 64, bw, ba, xd, outlier_scale=15.0, n_outliers=max(1, K // 100), seed=M + K,
                     a_group=64)
    X, W, L, R = wl.make_inputs(layer)
    g = _compare_all(oracle, layer, X, W, L, R)
    assert g.av.sx.shape == (M, K // 64)


@pytest.mark.parametrize("M,N", [(2000, 2304), (2100, 2176)])
def test_sint4_blocks_full_tiles_bit_exact(oracle, M, N):
    """Full 128 x 256 tiles, a ragged last row tile, and (second case) a last tile column of 128 channels."""
    layer = wl.Layer("t", M, 256, N, 32, "int", 64, 8, 8, "bf16", outlier_scale=15.0, n_outliers=2, seed=M, a_group=64)
    X, W, L, R = wl.make_inputs(layer)
    _compare_all(oracle, layer, X, W, L, R)


def test_sint4_blocks_degenerate_and_extreme_scales(oracle):
    layer = wl.Layer("t", 70, 256, 64, 16, "int", 64, 8, 8, "f32", seed=4, a_group=64)
    X, W, L, R = wl.make_inputs(layer)
    X[3] = 0.0                    # an all-zero token: every block scale is 1
    X[5, :] = 0.0
    X[5, 70] = -2.0               # a one-hot token: three all-zero blocks
    X[7, :64] *= 1e-9             # block scale below the FP16 range: clamped to 2^-24, codes flush or clamp
    X[8, 64:128] *= 3e5           # block scale above the FP16 range: clamped to 65504, codes saturate
    X[9, 128:192] = 2.0 ** -26    # amax / 7 rounds to zero in FP16
    W[2] = 0.0
    W[6, :64] *= 1e-7
    _compare_all(oracle, layer, X, W, L, R)
    _compare_all(oracle, layer, np.zeros_like(X), W, L, R)


@pytest.mark.parametrize("name", ["c2s_qkv", "c4s_qkv"])
def test_sint4_blocks_full_size_sampled_rows(oracle, name):
    _full_size_sampled(oracle, name)


def test_seeded_shape_sweep_bit_exact(oracle):
    """Seeded sweep over small shapes around the tile edges (32-row blocks, 128-row tiles, 64- and 256-column tiles),
    ranks, group sizes, branch widths, input types and both main scale granularities."""
    rng = np.random.default_rng(2024)
    edge_M = [1, 31, 32, 33, 63, 64, 65, 127, 128, 129, 255, 257]
    for it in range(40):
        M = int(rng.choice(edge_M))
        K = 64 * int(rng.integers(1, 9))      # K = 64 with ranks 96 and 128 included: factor views larger than N x K
        N = 64 * int(rng.integers(1, 10)) if it % 8 else 64 * int(rng.integers(10, 40))
        r = int(rng.choice([0, 16, 32, 64, 96, 128]))
        ag = int(rng.choice([0, 64]))
        g = 64 if ag or K % 128 else int(rng.choice([64, 128]))
        bw, ba = [(8, 8), (6, 6), (4, 8)][int(rng.integers(0, 3))]
        xd = "bf16" if rng.integers(0, 2) else "f32"
        layer = wl.Layer("t", M, K, N, r, "int", g, bw, ba, xd, outlier_scale=12.0, n_outliers=1, seed=100 + it, a_group=ag)
        X, W, L, R = wl.make_inputs(layer)
        try:
            _compare_all(oracle, layer, X, W, L, R)
        except AssertionError as e:
            raise AssertionError(f"shape M={M} K={K} N={N} r={r} g={g} ag={ag} bw={bw} ba={ba} {xd}: {e}") from e


@pytest.mark.parametrize("M,K,N,r,xd,ag,sm", [(40, 5632, 64, 32, "bf16", 0, False),    # a 5600-wide input padded to 64s
                                               (33, 2368, 64, 16, "f32", 0, False),     # fp32 rows beyond 2304
                                               (50, 4672, 128, 64, "bf16", 0, True),    # smoothing on a long row
                                               (20, 3072, 64, 32, "f32", 64, True),     # ... with SINT4 blocks
                                               (17, 8192, 64, 128, "bf16", 0, False),
                                               (150, 5632, 320, 32, "bf16", 64, False)])  # SINT4 blocks at their largest K
def test_long_rows_are_streamed(oracle, M, K, N, r, xd, ag, sm):
    """Rows that do not fit the register-resident kernel go through the two-pass streamed one: same bits."""
    import torch
    from paper_2604_18117_amd import binding as lq
    from tests.gpu_util import to_dev_x
    layer = wl.Layer("t", M, K, N, r, "int", 64, 8, 8, xd, outlier_scale=15.0, n_outliers=8, seed=K, a_group=ag)
    X, W, L, R = wl.make_inputs(layer)
    if not sm:
        _compare_all(oracle, layer, X, W, L, R)
        return
    gamma = smoothing_vector(X, W)
    g = run_gpu(layer, X, W, L, R, debug=True, debug_acc=False, gamma=gamma)
    pk, act, out = run_oracle_int(oracle, layer, oracle.smooth(X, gamma), W, L, R, want_acc=False)
    assert np.array_equal(n(g.av.xq), act.xq) and np.array_equal(n(g.av.sx), act.sx)
    assert np.array_equal(n(g.adbg.xb), act.xb) and np.array_equal(n(g.adbg.accT), act.accT)
    assert np.array_equal(n(g.av.tq), act.tq) and np.array_equal(n(g.av.st), act.st)
    assert np.array_equal(n(g.fdbg.y32), out.y32) and np.array_equal(bf16_to_bits(g.Y), out.Y)


@pytest.mark.parametrize("family", ["int", "mx", "mxb", "mxi"])
def test_empty_batch_is_a_no_op(oracle, family):
    """M = 0 on every per-call entry point: LQ_OK, empty results, nothing launched (the stream stays usable)."""
    from paper_2604_18117_amd import binding as lq
    N, K, r = 128, 256, 32
    cfg = lq.make_config(N, K, r, family, 64 if family == "int" else 32)
    rng = np.random.default_rng(0)
    W = torch.from_numpy((rng.standard_normal((N, K)) * 0.02).astype(np.float32)).cuda()
    L = torch.from_numpy((rng.standard_normal((N, r)) * 0.01).astype(np.float32)).cuda()
    R = torch.from_numpy((rng.standard_normal((r, K)) * 0.01).astype(np.float32)).cuda()
    packed = lq.lq_pack_weights(cfg, W, L, R)
    X = torch.empty((0, K), dtype=torch.bfloat16, device="cuda")
    act = lq.lq_quantize_act(cfg, packed, X)
    Y = lq.lq_linear_lowrank_fwd(cfg, packed, act, 0)
    torch.cuda.synchronize()
    assert tuple(Y.shape) == (0, N)
    X1 = torch.ones((8, K), dtype=torch.bfloat16, device="cuda")      # and the next, non-empty call works
    Y1 = lq.lq_linear_lowrank_fwd(cfg, packed, lq.lq_quantize_act(cfg, packed, X1), 8)
    torch.cuda.synchronize()
    assert tuple(Y1.shape) == (8, N) and bool(torch.isfinite(Y1.float()).all())

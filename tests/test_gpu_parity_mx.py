"""GPU parity, MX family (MXFP4 main on the scaled MFMA, FP8 branch) against the CPU oracle.

Bar: every code and scale computed from source data (X, P, L, R) bit-exact (+0 and -0 codes are
the same value); quantities that pass through fp32 accumulation in the matrix core (T, y) within a
bound derived from the arithmetic; re-quantised intermediate codes may differ from the oracle's only
where T sits on a rounding boundary (counted, each difference at most one code step).
"""
import dataclasses

import numpy as np
import pytest
import torch

from paper_2604_18117_amd import workloads as wl
from tests.smoothing import smoothing_vector
from tests.gpu_util import bf16_to_bits, check_bf16_against_oracle, check_end_to_end, n, run_gpu

pytestmark = pytest.mark.gpu

E2M1 = np.array([0, .5, 1, 1.5, 2, 3, 4, 6, -0., -.5, -1, -1.5, -2, -3, -4, -6], np.float32)


def _e4m3_table(oracle):
    return oracle.e4m3_decode(np.arange(256, dtype=np.uint8))


def _run_oracle(oracle, layer, X, W, L, R):
    pk = oracle.pack_mx(W, L if layer.r else None, R if layer.r else None)
    act = oracle.quantize_act_mx(X, pk)
    return pk, act


def _compare(oracle, layer, X, W, L, R, rows=None, gamma=None):
    """rows: None = compare everything, else the sampled token rows (oracle sees only those)."""
    g = run_gpu(layer, X, W, L, R, debug=True, debug_acc=False, gamma=gamma)
    Xo = X if rows is None else X[rows]
    if gamma is not None:                       # fused smoothing: the oracle quantises the smoothed input
        Xo = oracle.smooth(Xo, gamma)
    sel = slice(None) if rows is None else rows
    pk, act = _run_oracle(oracle, layer, Xo, W, L, R)
    f8 = _e4m3_table(oracle)
    r = layer.r
    # ---- offline packing: exact
    assert np.array_equal(E2M1[n(g.wv.pq).view(np.uint8)], E2M1[pk.pc]), "pq"
    assert np.array_equal(n(g.wv.pe), pk.pe), "pe"
    assert np.array_equal(n(g.wv.sl), pk.sl), "sl"
    if r:
        assert np.array_equal(f8[n(g.wv.lq).view(np.uint8)], f8[pk.l8]), "l8"
        assert np.array_equal(f8[n(g.wv.rq).view(np.uint8)], f8[pk.r8]), "r8"
        assert np.array_equal(n(g.wv.sr), pk.sr), "sr"
    # ---- activation step: codes and scales from X exact
    assert np.array_equal(E2M1[n(g.av.xq).view(np.uint8)[sel]], E2M1[act.xc]), "xc"
    assert np.array_equal(n(g.av.xe)[sel], act.xe), "xe"
    tq_gpu = n(g.av.tq).view(np.uint8)[sel]
    st_gpu = n(g.av.st)[sel]
    if r:
        assert np.array_equal(f8[n(g.adbg.xb).view(np.uint8)[sel]], f8[act.xb8]), "xb8"
        assert np.array_equal(n(g.adbg.sxb)[sel], act.sxb), "sxb"
        # T: K fp32 accumulations of products bounded by 448^2 sxb sr
        T_gpu = n(g.adbg.T)[sel]
        tb = 2.0 ** -15 * (np.abs(f8[act.xb8].astype(np.float64)) @ np.abs(f8[pk.r8].astype(np.float64)).T) \
            * act.sxb[:, None] * pk.sr[None, :] + 1e-30
        assert np.all(np.abs(T_gpu - act.T) <= tb), "T"
        assert np.allclose(st_gpu, act.st, rtol=2e-4, atol=0), "st"
        diff = tq_gpu != act.tq8
        diff &= ~(((tq_gpu & 0x7F) == 0) & ((act.tq8 & 0x7F) == 0))
        # Re-quantised codes may differ from the oracle's only where T sits within the accumulation bound of a rounding
        # boundary (where |T| is small against the sum of |terms| that bound can span more than one code step): the
        # GPU's code must be a correct rounding of a value within the bound of the oracle's T (checked next, for every
        # element), and the two dequantised intermediates lie within two half steps plus the bound of each other
        # (checked with the end-to-end comparison below).  The count is reported.
        if diff.any():
            print(f"[parity mx] re-quantised codes that differ from the oracle's: {int(diff.sum())} of {diff.size}")
        # every GPU code is a correct E4M3 rounding of a value within the accumulation bound of the
        # oracle's T: |deq - T| <= half the local code spacing (in units of st) + bound
        u = np.abs(act.T.astype(np.float64)) / st_gpu[:, None]
        step = np.exp2(np.maximum(np.floor(np.log2(np.maximum(u, 2.0 ** -6))) - 3, -9))
        deq = f8[tq_gpu].astype(np.float64) * st_gpu[:, None]
        slack = st_gpu[:, None] * (0.5 * step * (1 + 1e-3) + 2e-4 * u) + tb
        assert np.all(np.abs(deq - act.T) <= slack), "tq8 is not a rounding of T"
    # ---- forward: the oracle is fed the GPU's re-quantised intermediate, so that what is compared
    # is the forward arithmetic alone
    act_g = dataclasses.replace(act, tq8=np.ascontiguousarray(tq_gpu), st=np.ascontiguousarray(st_gpu))
    out = oracle.fwd_mx(pk, act_g)
    y_gpu = n(g.fdbg.y32)[sel]
    Xd = np.abs(E2M1[act.xc].astype(np.float64).reshape(Xo.shape[0], -1, 32)) * oracle.e8m0_decode(act.xe)[:, :, None]
    Wd = np.abs(E2M1[pk.pc].astype(np.float64).reshape(layer.N, -1, 32)) * oracle.e8m0_decode(pk.pe)[:, :, None]
    A = Xd.reshape(Xo.shape[0], -1) @ Wd.reshape(layer.N, -1).T          # sum of |terms| of the main product
    bound = 2.0 ** -15 * (A + np.abs(out.ybr)) + 1e-30
    assert np.all(np.abs(y_gpu - out.y32) <= bound), f"y32 max excess {np.max(np.abs(y_gpu - out.y32) / bound)}"
    Yb = bf16_to_bits(g.Y)[sel]
    check_bf16_against_oracle(oracle, Yb, y_gpu, out, bound, " mx")
    # ---- end to end: the oracle alone (its own T, scale and codes)
    if r:
        out_alone = oracle.fwd_mx(pk, act)
        deq_g = f8[tq_gpu].astype(np.float64) * st_gpu[:, None].astype(np.float64)
        deq_o = f8[act.tq8].astype(np.float64) * act.st[:, None].astype(np.float64)
        D = np.abs(deq_g - deq_o)
        # both are roundings (half a local E4M3 step under their own per-token scale) of values within tb of each other
        uo = np.abs(act.T.astype(np.float64)) / act.st[:, None]
        step_o = np.exp2(np.maximum(np.floor(np.log2(np.maximum(uo, 2.0 ** -6))) - 3, -9))
        assert np.all(D <= (st_gpu[:, None] * 0.5 * step + act.st[:, None] * 0.5 * step_o) * (1 + 1e-3)
                      + 4e-4 * np.abs(act.T) + tb), "intermediates further apart than two half steps"
        Labs = np.abs(f8[pk.l8].astype(np.float64)) * pk.sl[:, None].astype(np.float64)
        check_end_to_end(oracle, Yb, y_gpu, out_alone, 2.0 ** -15 * (A + np.abs(out_alone.ybr)) + 1e-30, D, Labs, " mx")
    g2 = run_gpu(layer, X, W, L, R, debug=False, gamma=gamma)
    assert torch.equal(g2.Y, g.Y)
    return g


SMALL = [
    # M (ragged), K (multiple of 128), N (partial 256-wide tile), r, x_dtype
    (300, 256, 320, 32, "bf16"),
    (77, 384, 64, 16, "f32"),
    (130, 1152, 192, 64, "bf16"),
    (100, 2240, 128, 64, "bf16"),     # 35 chunks of 64: the 2240-wide transformer; one padding chunk in the layouts
    (70, 192, 64, 32, "f32"),
    (64, 128, 64, 0, "bf16"),
    (33, 640, 128, 128, "bf16"),
    (1, 128, 64, 32, "f32"),
    (33, 64, 576, 128, "bf16"),       # rank > K: the factor views are larger than N x K
    (255, 192, 256, 0, "f32"),        # rank 0: no branch section of either blob is read
]


@pytest.mark.parametrize("M,K,N,r,xd", SMALL)
def test_small_shapes(oracle, M, K, N, r, xd):
    layer = wl.Layer("t", M, K, N, r, "mx", 32, 8, 8, xd, seed=M + K)
    X, W, L, R = wl.make_inputs(layer)
    _compare(oracle, layer, X, W, L, R)


def test_degenerate_inputs(oracle):
    layer = wl.Layer("t", 70, 256, 64, 16, "mx", 32, 8, 8, "bf16", seed=3)
    X, W, L, R = wl.make_inputs(layer)
    X[3] = 0.0
    X[5, :] = 0.0
    X[5, 7] = -2.0
    X[9, 32:64] = 0.0     # an all-zero block inside a token
    W[2] = 0.0
    W[4, 64:96] = 0.0
    L[4] = 0.0
    R[1] = 0.0
    _compare(oracle, layer, X, W, L, R)
    _compare(oracle, layer, np.zeros_like(X), W, L, R)


def test_wide_dynamic_range_blocks(oracle):
    layer = wl.Layer("t", 64, 256, 64, 32, "mx", 32, 8, 8, "bf16", seed=5)
    X, W, L, R = wl.make_inputs(layer)
    rng = np.random.default_rng(7)
    X *= wl.round_to_bf16(np.exp2(rng.integers(-20, 20, size=(64, 8)).repeat(32, axis=1)).astype(np.float32))
    W *= np.exp2(rng.integers(-10, 10, size=(64, 8)).repeat(32, axis=1)).astype(np.float32)
    _compare(oracle, layer, wl.round_to_bf16(X), W, L, R)


@pytest.mark.parametrize("name", ["c5_qkv", "c5_attn_out", "c5_cross_kv", "c5_fc1", "c5_fc2"])
def test_full_size_sampled_rows(oracle, name):
    layer = wl.LAYERS[name]
    X, W, L, R = wl.make_inputs(layer)
    rng = np.random.default_rng(1)
    # (first and last row, both halves of the last row tile -- the last generation of some layers runs as half tiles)
    rows = np.unique(np.concatenate([[0, layer.M - 1, layer.M - 128, layer.M - 65, layer.M - 64], rng.choice(layer.M, 14, replace=False)]))
    _compare(oracle, layer, X, W, L, R, rows=rows)


def test_half_tiles_of_the_last_generation(oracle):
    """More tiles than workgroup slots with a sparse last generation: the forward cuts the tiles left over into 64-row half
    tiles.  Every row of those tiles (ragged end included) and a sample of the others against the oracle."""
    M = 528 * 128 - 37
    layer = wl.Layer("t", M, 128, 320, 32, "mx", 32, 8, 8, "bf16", seed=11)
    X, W, L, R = wl.make_inputs(layer)
    rng = np.random.default_rng(2)
    rows = np.unique(np.concatenate([np.arange(M - 16 * 128 - 200, M), [0, 63, 64, 127, 128], rng.choice(M, 24, replace=False)]))
    _compare(oracle, layer, X, W, L, R, rows=rows)


@pytest.mark.parametrize("M,K,N,r,xd,sm", [(40, 5632, 64, 32, "bf16", False), (33, 2432, 64, 16, "f32", False),
                                            (50, 4736, 128, 64, "bf16", True), (17, 8192, 64, 128, "bf16", False)])
def test_long_rows_are_streamed(oracle, M, K, N, r, xd, sm):
    """Rows that do not fit the register-resident activation kernel go through the two-pass streamed form."""
    layer = wl.Layer("t", M, K, N, r, "mx", 32, 8, 8, xd, outlier_scale=10.0, n_outliers=8, seed=K)
    X, W, L, R = wl.make_inputs(layer)
    _compare(oracle, layer, X, W, L, R, gamma=smoothing_vector(X, W) if sm else None)

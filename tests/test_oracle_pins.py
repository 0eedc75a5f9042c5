"""Pins of the CPU oracle against what the paper and the mathematics fix (no GPU).

Each test names the passage or identity it pins.  None of them re-types the oracle's own
formula: they use exact rational / big-integer arithmetic, numpy's integer matmul, closed
forms, invariants and the format tables of the OCP MX specification the paper cites.
"""
import itertools
import os
from fractions import Fraction

import numpy as np
import pytest

from paper_2604_18117_amd import workloads as wl
from tests.smoothing import smoothing_vector

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "ocp_mx_element_formats.txt")


def _golden():
    out = {"e2m1": None, "e2m3": None, "e4m3": [], "e8m0": [], "budget": [], "mxint": {}}
    for line in open(GOLDEN):
        line = line.strip()
        if not line or line.startswith("#"):
            continue
        t = line.split()
        if t[0] == "e2m1":
            out["e2m1"] = [float(v) for v in t[1:]]
        elif t[0] == "e2m3":
            out["e2m3"] = [float(v) for v in t[1:]]
        elif t[0] == "e4m3":
            out["e4m3"].append((int(t[1], 16), float(t[2])))
        elif t[0] == "e8m0":
            out["e8m0"].append((int(t[1]), float(t[2])))
        elif t[0] == "mxint":
            out["mxint"][int(t[1])] = (float(t[2]), float(t[3]))
        elif t[0] == "budget":
            out["budget"].append(tuple(int(v) for v in t[1:]))
    return out


def _small_int_problem(oracle, seed=0, M=24, K=256, N=40, r=8, g=64, bw=8, ba=8, lr_std=1e-3):
    rng = np.random.default_rng(seed)
    X = rng.standard_normal((M, K)).astype(np.float32)
    X[:, rng.choice(K, 3, replace=False)] *= 15
    W = (rng.standard_normal((N, K)) * 0.02).astype(np.float32)
    L = (rng.standard_normal((N, r)) * lr_std).astype(np.float32)
    R = (rng.standard_normal((r, K)) * lr_std).astype(np.float32)
    pk = oracle.pack_int(W, L, R, g, bw)
    act = oracle.quantize_act_int(X, pk, ba)
    out = oracle.fwd_int(pk, act, want_acc=True)
    return X, W, L, R, pk, act, out


# --------------------------------------------------------------------------------------
# element formats (App. A.3, values fixed by the OCP MX specification)
# --------------------------------------------------------------------------------------

def test_e2m1_table_matches_spec(oracle):
    g = _golden()
    dec = oracle.e2m1_decode(np.arange(16, dtype=np.uint8))
    assert list(dec[:8]) == g["e2m1"]
    assert list(dec[8:]) == [-v if v else -0.0 for v in g["e2m1"]]
    assert np.signbit(dec[8])


def test_e4m3_e8m0_landmarks(oracle):
    g = _golden()
    for code, val in g["e4m3"]:
        assert float(oracle.e4m3_decode(np.uint8(code))) == val
    assert np.isnan(oracle.e4m3_decode(np.uint8(0x7F)))
    for code, val in g["e8m0"]:
        assert float(oracle.e8m0_decode(np.uint8(code))) == val
    # monotone over the finite positive codes, all 256 codes round-trip (idempotence of Q)
    dec = oracle.e4m3_decode(np.arange(127, dtype=np.uint8))
    assert np.all(np.diff(dec) > 0)
    for c in range(256):
        if c & 0x7F == 0x7F:
            continue
        v = float(oracle.e4m3_decode(np.uint8(c)))
        assert oracle.e4m3_encode(v) == c


def test_budget_example():
    # Section 3.3: 16 bits/value x rank 32 = 512 bits/channel => rank 64 at 8 b, 128 at 4 b
    for bits, rank, budget in _golden()["budget"]:
        assert bits * rank == budget
        assert budget // 8 == 64 and budget // 4 == 128


def test_e2m1_rounding_is_nearest_even_and_saturating(oracle):
    vals = [0, 0.5, 1, 1.5, 2, 3, 4, 6]
    # exact ties go to the code with even mantissa bit
    ties = {0.25: 0.0, 0.75: 1.0, 1.25: 1.0, 1.75: 2.0, 2.5: 2.0, 3.5: 4.0, 5.0: 4.0}
    for u, want in ties.items():
        for sgn in (1, -1):
            got = float(oracle.e2m1_decode(np.uint8(oracle.e2m1_encode(sgn * u))))
            assert got == sgn * want
    # brute force: nearest representable for a dense sweep (non-ties)
    for u in np.linspace(-9, 9, 7201):
        got = float(oracle.e2m1_decode(np.uint8(oracle.e2m1_encode(float(u)))))
        best = min(abs(abs(u) - v) for v in vals)
        assert abs(abs(got) - abs(u)) <= best + 1e-12
        assert abs(got) <= 6
        if got != 0:
            assert np.sign(got) == np.sign(u)


def test_e4m3_rounding_nearest_even_saturating(oracle):
    dec = oracle.e4m3_decode(np.arange(127, dtype=np.uint8)).astype(np.float64)
    rng = np.random.default_rng(1)
    us = np.concatenate([rng.uniform(-460, 460, 3000), rng.uniform(-1, 1, 3000),
                         rng.uniform(-0.02, 0.02, 2000), [448.0, 464.0, 1e4, -1e4]])
    for u in us:
        u = float(np.float32(u))
        c = oracle.e4m3_encode(u)
        got = float(oracle.e4m3_decode(np.uint8(c)))
        best = np.min(np.abs(dec - abs(u)))
        assert abs(abs(got) - abs(u)) <= best
        assert abs(got) <= 448
    # exact ties: midpoint of neighbours goes to the even code
    for c in range(0, 126):
        mid = float(np.float32((dec[c] + dec[c + 1]) / 2))
        if mid == (dec[c] + dec[c + 1]) / 2:
            assert oracle.e4m3_encode(mid) == (c if c % 2 == 0 else c + 1)


def test_mxfp4_block_scale_and_bound(oracle):
    # App. A.3: blocks of 32, power-of-two scale.  Scale exponent = floor(log2 amax) - 2.
    rng = np.random.default_rng(2)
    v = (rng.standard_normal(32 * 40) * np.exp(rng.uniform(-6, 6, 32 * 40))).astype(np.float32)
    v[64:96] = 0.0
    codes, e = oracle.quant_mxfp4(v)
    assert e[2] == 0 and np.all(codes[64:96] & 7 == 0)
    deq = oracle.e2m1_decode(codes).astype(np.float64).reshape(-1, 32)
    sc = oracle.e8m0_decode(e)
    vb = v.astype(np.float64).reshape(-1, 32)
    for b in range(vb.shape[0]):
        a = np.abs(vb[b]).max()
        if a == 0:
            continue
        assert sc[b] == 2.0 ** (np.floor(np.log2(a)) - 2)
        u = vb[b] / sc[b]
        assert np.abs(u).max() < 8
        # error bound: half the local spacing below 6, |u|-6 above (saturation)
        err = np.abs(u - deq[b])
        spacing = np.where(np.abs(u) < 2, 0.5, np.where(np.abs(u) < 4, 1.0, 2.0))
        bound = np.where(np.abs(u) <= 6, spacing / 2, np.abs(u) - 6)
        assert np.all(err <= bound + 1e-12)
    # idempotence (Section 3.2): Q(deq(Q(v))) gives the same codes and scales, unless the
    # block maximum dropped below its binade by rounding (then the scale may shrink)
    back = (deq * sc[:, None]).astype(np.float32).ravel()
    codes2, e2 = oracle.quant_mxfp4(back)
    deq2 = oracle.e2m1_decode(codes2).astype(np.float64).reshape(-1, 32) * oracle.e8m0_decode(e2)[:, None]
    assert np.array_equal(deq2.ravel().astype(np.float32), back)


# --------------------------------------------------------------------------------------
# integer quantiser
# --------------------------------------------------------------------------------------

@pytest.mark.parametrize("qmax", [7, 31, 127])
def test_int_quantiser_error_bound_and_range(oracle, qmax):
    # |x - s q| <= s/2 (round to nearest), codes symmetric in [-qmax, qmax], amax maps to qmax
    rng = np.random.default_rng(qmax)
    for n in (1, 5, 64, 1152):
        v = (rng.standard_normal(n) * 10 ** rng.uniform(-3, 3)).astype(np.float32)
        q, s = oracle.quant_int(v, qmax)
        assert q.min() >= -qmax and q.max() <= qmax
        assert abs(int(q[np.argmax(np.abs(v))])) == qmax
        sd = float(s)
        assert np.all(np.abs(v.astype(np.float64) - sd * q) <= sd / 2 * (1 + 2 ** -20))
        # exact-rational statement of "nearest": |qmax*x/amax - q| <= 1/2 (+ fp32 slack)
        amax = Fraction(float(np.abs(v).max()))
        for x, qi in zip(v[:64], q[:64]):
            assert abs(Fraction(float(x)) * qmax / amax - int(qi)) <= Fraction(1, 2) + Fraction(1, 2 ** 18)


def test_int_quantiser_ties_to_even_and_zero(oracle):
    # amax = 2 => 7/amax = 3.5 exactly: x=1 -> 3.5 -> 4 (even); x = 3/7*... use exact cases
    q, s = oracle.quant_int(np.array([2.0, 1.0, -1.0, 3.0 / 7 * 2], np.float32), 7)
    assert list(q[:3]) == [7, 4, -4]
    # amax = 14: inv = 0.5; 5 -> 2.5 -> 2, 7 -> 3.5 -> 4, 3 -> 1.5 -> 2, 1 -> 0.5 -> 0
    q, s = oracle.quant_int(np.array([14, 5, 7, 3, 1, -1, -3, -5], np.float32), 7)
    assert list(q) == [7, 2, 4, 2, 0, 0, -2, -2]
    assert s == np.float32(2.0)
    q, s = oracle.quant_int(np.zeros(8, np.float32), 7)
    assert s == np.float32(1.0) and not q.any()


@pytest.mark.parametrize("qmax", [7, 31, 127])
def test_int_quantiser_idempotent(oracle, qmax):
    # Section 3.2: Q(X) = X on the image of Q.  Codes are reproduced exactly; the scale is
    # reproduced to one ulp (qmax is not a power of two), exactly for power-of-two scales.
    rng = np.random.default_rng(10 + qmax)
    v = rng.standard_normal(512).astype(np.float32)
    q, s = oracle.quant_int(v, qmax)
    deq = (q.astype(np.float32) * s)
    q2, s2 = oracle.quant_int(deq, qmax)
    assert np.array_equal(q, q2)
    assert abs(float(s2) - float(s)) <= np.spacing(np.float32(s))
    v[0] = qmax * 0.25
    v[1:] = np.clip(v[1:], -1, 1)
    q, s = oracle.quant_int(v, qmax)
    assert s == np.float32(0.25)
    q2, s2 = oracle.quant_int(q.astype(np.float32) * s, qmax)
    assert s2 == s and np.array_equal(q, q2)


def test_scale_and_sign_equivariance(oracle):
    # scaling by 2^k scales the scale, leaves codes; negation negates codes (symmetric range)
    rng = np.random.default_rng(3)
    v = rng.standard_normal(300).astype(np.float32)
    q, s = oracle.quant_int(v, 7)
    q2, s2 = oracle.quant_int(v * np.float32(8), 7)
    q3, s3 = oracle.quant_int(-v, 7)
    assert np.array_equal(q, q2) and s2 == s * np.float32(8)
    assert np.array_equal(q3, -q) and s3 == s



# --------------------------------------------------------------------------------------
# SINT4 blocks (App. A.3: blocks of 64 values, one FP16 scale per block, round to nearest)
# --------------------------------------------------------------------------------------

def test_f16_rounding_matches_ieee_half(oracle):
    # numpy's float16 cast is an independent implementation of round-to-nearest-even to binary16
    rng = np.random.default_rng(21)
    v = (rng.standard_normal(20000) * np.exp2(rng.uniform(-27, 15.9, 20000))).astype(np.float32)
    special = np.float32([0.0, 2.0 ** -24, 2.0 ** -25, 1.5 * 2.0 ** -25, 2.0 ** -14, 2.0 ** -14 - 2.0 ** -26, 65504.0, 65519.0,
                          1.0 + 2.0 ** -11, 1.0 + 3 * 2.0 ** -11, 1.0 + 2.0 ** -11 + 2.0 ** -20, -3.0003])
    v = np.concatenate([v[np.abs(v) < 65520], special, -special])
    got = np.array([oracle.f16_round(float(x)) for x in v], np.float32)
    want = v.astype(np.float16).astype(np.float32)
    assert np.array_equal(got, want)
    assert oracle.f16_round(float(np.float32(1.0 + 2.0 ** -11))) == 1.0                       # tie -> even
    assert oracle.f16_round(float(np.float32(1.0 + 3 * 2.0 ** -11))) == 1.0 + 2.0 ** -9       # tie -> even (up)


def test_sint4_block_quantiser(oracle):
    rng = np.random.default_rng(22)
    v = (rng.standard_normal(64 * 40) * np.repeat(np.exp2(rng.uniform(-12, 8, 40)), 64)).astype(np.float32)
    q, s = oracle.quant_sint4(v)
    vb, qb = v.reshape(40, 64), q.reshape(40, 64)
    # one scale per block of 64, an FP16 number: the nearest one to amax / 7
    assert s.shape == (40,)
    assert np.array_equal(s, s.astype(np.float16).astype(np.float32))
    amax = np.abs(vb).max(axis=1)
    for b in range(40):
        exact = Fraction(float(amax[b])) / 7
        sb = Fraction(float(s[b]))
        ulp = Fraction(float(np.spacing(np.float16(s[b]))))
        assert abs(sb - exact) <= ulp / 2 + exact * Fraction(1, 2 ** 23)     # nearest FP16 to the fp32 quotient
        # codes: nearest integer to x / s (stored scale), within [-7, 7]; the block maximum maps to +-7
        assert qb[b].min() >= -7 and qb[b].max() <= 7
        assert abs(int(qb[b][np.argmax(np.abs(vb[b]))])) == 7
        for x, qi in zip(vb[b], qb[b]):
            u = Fraction(float(x)) / sb
            if abs(u) <= 7:
                assert abs(u - int(qi)) <= Fraction(1, 2) + Fraction(1, 2 ** 18)
            else:
                assert abs(int(qi)) == 7      # the scale was rounded down: at most 7 (1 + 2^-11)
                assert abs(u) <= 7 * (1 + Fraction(1, 2 ** 11))
    # dequantisation error: half a step (plus the clamp slack above)
    assert np.all(np.abs(vb.astype(np.float64) - s[:, None].astype(np.float64) * qb) <= s[:, None] * (0.5 + 7 * 2.0 ** -11))
    # blocks are independent: changing one block leaves the others' codes and scales alone
    v2 = v.copy()
    v2[64:128] *= 3
    q2, s2 = oracle.quant_sint4(v2)
    keep = np.r_[0:64, 128:v.size]
    assert np.array_equal(q[keep], q2[keep]) and np.array_equal(np.delete(s, 1), np.delete(s2, 1))


def test_sint4_block_edge_cases(oracle):
    # exact ties with a power-of-two scale: amax = 14 -> s = 2: 5 -> 2.5 -> 2, 7 -> 3.5 -> 4, 3 -> 1.5 -> 2, 1 -> 0.5 -> 0
    v = np.zeros(128, np.float32)
    v[:8] = [14, 5, 7, 3, 1, -1, -3, -5]
    q, s = oracle.quant_sint4(v)
    assert list(q[:8]) == [7, 2, 4, 2, 0, 0, -2, -2] and s[0] == 2.0
    assert s[1] == 1.0 and not q[64:].any()                      # all-zero block
    # scales outside the FP16 range are clamped to it and the codes saturate / flush accordingly
    tiny = np.zeros(64, np.float32)
    tiny[0], tiny[1], tiny[2] = 1e-6, 2.0 ** -25 * 1.01, -2.0 ** -26
    q, s = oracle.quant_sint4(tiny * np.float32(1e-1))           # amax / 7 = 1.4e-8 < 2^-25: rounds to 0 -> 2^-24
    assert s[0] == np.float32(2.0 ** -24)
    assert list(q[:3]) == [2, 0, 0]                              # 1e-7 / 2^-24 = 1.68 -> 2
    q, s = oracle.quant_sint4(tiny)                              # amax / 7 = 1.43e-7 = 2.4 * 2^-24 -> 2 * 2^-24
    assert s[0] == np.float32(2.0 ** -23)
    assert list(q[:3]) == [7, 0, 0]                              # 1e-6 / 2^-23 = 8.4 -> clamped to 7
    huge = np.zeros(64, np.float32)
    huge[0], huge[1] = 1e6, -3e5
    q, s = oracle.quant_sint4(huge)
    assert s[0] == np.float32(65504.0) and list(q[:2]) == [7, -5]   # 1e6 / 65504 = 15.3 -> 7; 3e5 / 65504 = 4.58 -> 5
    # idempotence on the grid (Section 3.2): codes are reproduced, and so is a scale whose 7-fold is exact
    rng = np.random.default_rng(23)
    w = rng.standard_normal(256).astype(np.float32)
    q, s = oracle.quant_sint4(w)
    q2, s2 = oracle.quant_sint4((q.reshape(4, 64) * s[:, None]).astype(np.float32).ravel())
    assert np.array_equal(q, q2)
    assert np.all(np.abs(s2 - s) <= np.spacing(s.astype(np.float16)).astype(np.float32))


def _small_sint4_problem(oracle, seed=5, M=6, K=256, N=10, r=8):
    rng = np.random.default_rng(seed)
    X = rng.standard_normal((M, K)).astype(np.float32)
    X[:, rng.choice(K, 3, replace=False)] *= 15
    W = (rng.standard_normal((N, K)) * 0.02).astype(np.float32)
    L = (rng.standard_normal((N, r)) * 1e-3).astype(np.float32)
    R = (rng.standard_normal((r, K)) * 1e-3).astype(np.float32)
    pk = oracle.pack_int(W, L, R, 64, 8, sint4_blocks=True)
    act = oracle.quantize_act_int(X, pk, 8)
    out = oracle.fwd_int(pk, act, want_acc=True)
    return X, W, L, R, pk, act, out


def test_sint4_block_forward_against_exact_rationals(oracle):
    X, W, L, R, pk, act, out = _small_sint4_problem(oracle)
    M, K = X.shape
    N, G = pk.N, K // 64
    # both operands of the main product carry one FP16 scale per block of 64 along K
    assert act.sx.shape == (M, G) and pk.sw.shape == (N, G)
    for a in (act.sx, pk.sw):
        assert np.array_equal(a, a.astype(np.float16).astype(np.float32))
    # the codes are those of the block quantiser applied row by row (to X, and to the residual P)
    for m in range(M):
        q, s = oracle.quant_sint4(X[m])
        assert np.array_equal(q, act.xq[m]) and np.array_equal(s, act.sx[m])
    q, s = oracle.quant_sint4(pk.P[3])
    assert np.array_equal(q, pk.pq[3]) and np.array_equal(s, pk.sw[3])
    # the branch is the per-token / per-row branch of the plain INT path, bit for bit
    pk0 = oracle.pack_int(W, L, R, 64, 8)
    act0 = oracle.quantize_act_int(X, pk0, 8)
    assert np.array_equal(pk.lq, pk0.lq) and np.array_equal(pk.rq, pk0.rq) and np.array_equal(pk.P, pk0.P)
    assert np.array_equal(act.tq, act0.tq) and np.array_equal(act.st, act0.st) and np.array_equal(act.xb, act0.xb)
    # integer contractions are textbook matrix products per block
    xq = act.xq.astype(np.int64).reshape(M, G, 64)
    pq = pk.pq.astype(np.int64).reshape(N, G, 64)
    assert np.array_equal(out.acc, np.einsum("mgk,ngk->mng", xq, pq))
    # y32 = sum_g acc * sx * sw + branch, exact up to the fp32 roundings of the G + 3 operations
    for m in range(M):
        for n in range(N):
            terms = [Fraction(int(out.acc[m, n, g])) * Fraction(float(act.sx[m, g])) * Fraction(float(pk.sw[n, g]))
                     for g in range(G)]
            br = Fraction(int(out.acc2[m, n])) * Fraction(float(act.st[m])) * Fraction(float(pk.sl[n]))
            mag = float(sum(abs(t) for t in terms) + abs(br))
            assert abs(float(sum(terms) + br) - float(out.y32[m, n])) <= (G + 4) * 2 ** -24 * mag
            assert abs(float(sum(terms)) - float(out.ymain[m, n])) <= (G + 1) * 2 ** -24 * mag
    # a single block (K = 64) and no branch: y32 is the correctly rounded acc * (sx * sw), no other rounding
    pk1 = oracle.pack_int(W[:, :64], None, None, 64, 8, sint4_blocks=True)
    act1 = oracle.quantize_act_int(X[:, :64], pk1, 8)
    o1 = oracle.fwd_int(pk1, act1, want_acc=True)
    p = (act1.sx[:, 0][:, None].astype(np.float64) * pk1.sw[:, 0][None, :].astype(np.float64))   # exact in fp64 and in fp32
    assert np.array_equal(p.astype(np.float32).astype(np.float64), p)
    want = (o1.acc[:, :, 0].astype(np.float64) * p).astype(np.float32)                         # one rounding
    assert np.array_equal(o1.y32, want)
    # finer scales help: with outlier channels the block-scaled main product is closer to X P^T than the per-token one
    ref = X.astype(np.float64) @ pk.P.astype(np.float64).T
    out0 = oracle.fwd_int(pk0, act0)
    e_blk = np.abs(out.ymain - ref).mean()
    e_tok = np.abs(out0.ymain - ref).mean()
    assert e_blk < e_tok


# --------------------------------------------------------------------------------------
# data-free calibration of the factors (Section 3.2, Eq. 4; App. B.2)
# --------------------------------------------------------------------------------------

def _calib_problem(oracle, seed=31, N=48, K=256, r=8):
    rng = np.random.default_rng(seed)
    W = (rng.standard_normal((N, K)) * 0.02).astype(np.float32)
    U, S, Vt = np.linalg.svd(W.astype(np.float64), full_matrices=False)
    L0 = (U[:, :r] * np.sqrt(S[:r])).astype(np.float32)           # best rank-r approximation W ~ L0 R0 (Section 3.2)
    R0 = (np.sqrt(S[:r])[:, None] * Vt[:r]).astype(np.float32)
    return W, -L0, R0                                             # the paper starts from L = -L0, R = R0


@pytest.mark.parametrize("q1", ["mxfp4", "mxint4"])
def test_calib_error_mx_quantisers(oracle, q1):
    # E = Q1(V) - V for the block-32 / E8M0 formats: E + V is an element value times the block's power of two, the
    # one the (already pinned) block quantiser picks for the fp32 V
    W, L, R = _calib_problem(oracle)
    N, K = W.shape
    st = oracle.calib_init(L, R)
    out = oracle.calib_step(W, st, q1=q1)
    V = W.astype(np.float64) + L.astype(np.float64) @ R.astype(np.float64)
    grid = np.array(sorted(set(abs(v) for v in oracle.e2m1_decode(np.arange(16))))) if q1 == "mxfp4" else np.arange(8) / 4.0
    for n in (0, 11, N - 1):
        for b in range(K // 32):
            sl = slice(32 * b, 32 * b + 32)
            e = np.floor(np.log2(np.abs(V[n, sl]).max())) - (2 if q1 == "mxfp4" else 0)
            units = (out.E[n, sl] + V[n, sl]) / 2.0 ** e           # in element units
            near = grid[np.abs(np.abs(units)[:, None] - grid[None, :]).argmin(axis=1)]
            assert np.all(np.abs(np.abs(units) - near) <= 1e-5), (n, b)
            step_max = 2.0 if q1 == "mxfp4" else 0.25              # widest gap of the element grid (4 -> 6; 1/4)
            top = 6.0 if q1 == "mxfp4" else 1.75
            inside = np.abs(V[n, sl]) / 2.0 ** e <= top
            assert np.all(np.abs(out.E[n, sl][inside]) / 2.0 ** e <= step_max / 2 + 1e-5)
    assert abs(out.loss - np.mean(out.E.astype(np.float64) ** 2)) <= 1e-12 * out.loss
    gL = -2.0 / (N * K) * out.E.astype(np.float64) @ R.astype(np.float64).T
    assert np.allclose(out.gL, gL, rtol=1e-6, atol=1e-7 * np.abs(gL).max())
    # descent also holds for these formats
    losses = [out.loss] + [oracle.calib_step(W, st, q1=q1, lr=1e-3).loss for _ in range(60)]
    assert losses[-1] < 0.97 * losses[0]


@pytest.mark.parametrize("g,sint4", [(64, False), (128, False), (64, True)])
def test_calib_error_and_gradients(oracle, g, sint4):
    W, L, R = _calib_problem(oracle)
    N, K = W.shape
    st = oracle.calib_init(L, R)
    out = oracle.calib_step(W, st, g, sint4_blocks=sint4)
    V = W.astype(np.float64) + L.astype(np.float64) @ R.astype(np.float64)
    # E = Q1(V) - V: E + V sits on the 4-bit grid of its group (integer code in [-7, 7] times the group scale)
    for n in (0, 7, N - 1):
        for gi in range(K // g):
            sl = slice(gi * g, (gi + 1) * g)
            if sint4:
                scale = float(np.float16(np.abs(V[n, sl]).max() / 7))
                tol = 2 ** -10
            else:
                scale = np.abs(V[n, sl]).max() / 7
                tol = 1e-5
            codes = (out.E[n, sl] + V[n, sl]) / scale
            assert np.all(np.abs(codes - np.rint(codes)) <= 7 * tol + 1e-4) and np.abs(np.rint(codes)).max() == 7
            assert np.all(np.abs(out.E[n, sl]) <= scale * (0.5 + 8 * tol))
    # loss = mean of E^2 (Mean Squared Error)
    assert abs(out.loss - np.mean(out.E.astype(np.float64) ** 2)) <= 1e-12 * out.loss
    # App. B.2: grad_L = -2/(NK) E R^T, grad_R = -2/(NK) L^T E  (numpy's matmul as the independent routine)
    gL = -2.0 / (N * K) * out.E.astype(np.float64) @ R.astype(np.float64).T
    gR = -2.0 / (N * K) * L.astype(np.float64).T @ out.E.astype(np.float64)
    assert np.allclose(out.gL, gL, rtol=1e-6, atol=1e-7 * np.abs(gL).max())
    assert np.allclose(out.gR, gR, rtol=1e-6, atol=1e-7 * np.abs(gR).max())
    # ... which is the gradient of mean((C - L R)^2) with the quantised target C = Q1(W + L R) - W held fixed
    # (the rounding has zero derivative): central differences on a few entries
    Cq = out.E.astype(np.float64) + L.astype(np.float64) @ R.astype(np.float64)
    f = lambda Lm, Rm: np.mean((Cq - Lm @ Rm) ** 2)
    Ld, Rd = L.astype(np.float64), R.astype(np.float64)
    for (i, j) in ((0, 0), (5, 3), (N - 1, 7)):
        h = 1e-6
        Lp, Lm_ = Ld.copy(), Ld.copy()
        Lp[i, j] += h
        Lm_[i, j] -= h
        assert abs((f(Lp, Rd) - f(Lm_, Rd)) / (2 * h) - gL[i, j]) <= 1e-6 * np.abs(gL).max() + 1e-12
    for (j, k) in ((0, 0), (3, 100), (7, K - 1)):
        h = 1e-6
        Rp, Rm_ = Rd.copy(), Rd.copy()
        Rp[j, k] += h
        Rm_[j, k] -= h
        assert abs((f(Ld, Rp) - f(Ld, Rm_)) / (2 * h) - gR[j, k]) <= 1e-6 * np.abs(gR).max() + 1e-12


def test_calib_adam_matches_library_optimizer(oracle):
    # the update rule against torch.optim.Adam fed with the oracle's own gradients, over several steps
    torch = pytest.importorskip("torch")
    W, L, R = _calib_problem(oracle, seed=32)
    st = oracle.calib_init(L, R)
    Lt = torch.tensor(L, dtype=torch.float64, requires_grad=True)
    Rt = torch.tensor(R, dtype=torch.float64, requires_grad=True)
    opt = torch.optim.Adam([Lt, Rt], lr=1e-3, betas=(0.9, 0.999), eps=1e-8)
    for step in range(4):
        out = oracle.calib_step(W, st, 64, lr=1e-3)
        Lt.grad = torch.tensor(out.gL, dtype=torch.float64)
        Rt.grad = torch.tensor(out.gR, dtype=torch.float64)
        opt.step()
        # fp32 storage of the state on the oracle's side: a few ulps of the parameter per step
        assert np.allclose(st.L, Lt.detach().numpy(), rtol=0, atol=4e-7 * (step + 1) * np.abs(L).max())
        assert np.allclose(st.R, Rt.detach().numpy(), rtol=0, atol=4e-7 * (step + 1) * np.abs(R).max())
    # closed form of Adam's first step (mhat = g, vhat = g^2): p -= lr g / (|g| + eps); with the mean-squared-error scaling
    # the gradients of such a layer are of the order of eps, so eps is not negligible here
    st1 = oracle.calib_init(L, R)
    out = oracle.calib_step(W, st1, 64, lr=1e-3)
    gd = out.gL.astype(np.float64)
    want = L.astype(np.float64) - 1e-3 * gd / (np.abs(gd) + 1e-8)
    assert np.allclose(st1.L, want, rtol=0, atol=2e-7 * np.abs(L).max())
    assert 1e-9 < np.abs(gd).max() < 1e-5


def test_calib_fixed_point_and_descent(oracle):
    # Section 3.2: a point of the quantiser's image is a fixed point: E = 0, zero gradients, nothing moves
    W, L, R = _calib_problem(oracle, seed=33)
    # a weight on the 4-bit grid of its groups: scale 0.25 (amax 1.75 = 7 * 0.25), codes 7, 2, -3, 0
    Wfix = np.zeros_like(W)
    Wfix[:, 0], Wfix[:, 1], Wfix[:, 2] = 1.75, 0.5, -0.75
    Wfix[:, 64:128] = Wfix[:, :64] * np.float32(2.0 ** -5)
    st = oracle.calib_init(np.zeros_like(L), R)
    out = oracle.calib_step(Wfix, st, 64)
    assert not out.E.any() and not out.gL.any() and not out.gR.any() and out.loss == 0.0
    assert not st.L.any() and np.array_equal(st.R, R)
    # descent on a seeded synthetic weight: the optimisation lowers the loss of the SVD initialisation (Section 3.2)
    st = oracle.calib_init(L, R)
    losses = [oracle.calib_step(W, st, 64, lr=1e-4).loss for _ in range(120)]
    assert losses[-1] < 0.9 * losses[0]
    assert sum(b <= a * (1 + 1e-3) for a, b in zip(losses, losses[1:])) >= 0.9 * (len(losses) - 1)
    # the SVD initialisation itself beats no compensation: Q(W - L0 R0) + L0 R0 is closer to W than Q(W)
    z = oracle.calib_init(np.zeros_like(L), np.zeros_like(R))
    assert losses[0] < oracle.calib_step(W, z, 64).loss

# --------------------------------------------------------------------------------------
# whole INT path
# --------------------------------------------------------------------------------------

def test_integer_contractions_match_numpy_int64(oracle):
    # the three contractions are textbook integer matrix products
    X, W, L, R, pk, act, out = _small_int_problem(oracle)
    M, K = X.shape
    N, G, g = pk.N, pk.K // pk.g, pk.g
    xq = act.xq.astype(np.int64).reshape(M, G, g)
    pq = pk.pq.astype(np.int64).reshape(N, G, g)
    assert np.array_equal(out.acc, np.einsum("mgk,ngk->mng", xq, pq))
    assert np.array_equal(act.accT, act.xb.astype(np.int64) @ pk.rq.astype(np.int64).T)
    assert np.array_equal(out.acc2, act.tq.astype(np.int64) @ pk.lq.astype(np.int64).T)


def test_forward_matches_exact_rational_dequant(oracle):
    # y32 equals the exact value of sx*sum_g acc*sw + acc2*st*sl up to fp32 rounding of the
    # G+4 operations involved; Y is y32 rounded to bf16 (nearest even).
    X, W, L, R, pk, act, out = _small_int_problem(oracle, M=6, N=10)
    G = pk.K // pk.g
    for m in range(6):
        for n in range(10):
            terms = [Fraction(int(out.acc[m, n, gi])) * Fraction(float(pk.sw[n, gi])) for gi in range(G)]
            main = Fraction(float(act.sx[m])) * sum(terms)
            br = Fraction(int(out.acc2[m, n])) * Fraction(float(act.st[m])) * Fraction(float(pk.sl[n]))
            mag = float(Fraction(float(act.sx[m])) * sum(abs(t) for t in terms) + abs(br))
            assert abs(float(main + br) - float(out.y32[m, n])) <= (G + 4) * 2 ** -24 * mag
            assert abs(float(main) - float(out.ymain[m, n])) <= (G + 2) * 2 ** -24 * mag
            assert abs(float(br) - float(out.ybr[m, n])) <= 3 * 2 ** -24 * abs(float(br)) + 1e-45
    y = out.y32.astype(np.float64)
    Yf = oracle.bf16_bits_to_f32(out.Y).astype(np.float64)
    assert np.all(np.abs(Yf - y) <= np.abs(y) * 2 ** -8 + 1e-40)   # half a bf16 ulp
    # bf16 rounding: exact ties to even
    assert oracle.bf16_rne(float(np.float32(1.0 + 2 ** -8))) == 0x3F80       # tie -> even (down)
    assert oracle.bf16_rne(float(np.float32(1.0 + 3 * 2 ** -8))) == 0x3F82   # tie -> even (up)
    assert oracle.bf16_rne(-2.5) == 0xC020


def test_final_scale_and_add_is_one_fused_rounding(oracle):
    """The order of the last dequantisation step is a choice the paper leaves open (Fig. 1 only draws a sum node):
    y = fma(sx, t, ybr), one rounding, not fl(fl(sx * t) + ybr).  A constructed layer on which the two forms differ
    pins the choice: t = sx = 1 + 2^-23 and ybr = 2^-24, so sx * t = 1 + 2^-22 + 2^-46; rounding that product first
    loses the 2^-46 and the sum 1 + 2^-22 + 2^-24 is an exact tie that goes to even (1 + 2^-22), while the fused form
    sees a value just above the tie and rounds up to 1 + 2^-22 + 2^-23."""
    K, g = 64, 64
    one_eps = np.float32(1.0 + 2.0 ** -23)
    pq = np.zeros((1, K), np.int8); pq[0, 0] = 1
    xq = np.zeros((1, K), np.int8); xq[0, 0] = 1
    pk = oracle.PackedInt(1, K, 1, g, False, pq, np.full((1, 1), one_eps, np.float32), np.ones((1, 1), np.int8),
                          np.ones(1, np.float32), np.zeros((1, K), np.int8), np.ones(1, np.float32),
                          np.zeros((1, K), np.float32))
    act = oracle.ActInt(1, xq, np.full(1, one_eps, np.float32), np.zeros((1, K), np.int8), np.ones(1, np.float32),
                        np.zeros((1, 1), np.int32), np.zeros((1, 1), np.float32), np.ones((1, 1), np.int8),
                        np.full(1, 2.0 ** -24, np.float32))
    out = oracle.fwd_int(pk, act, want_acc=True)
    assert out.acc[0, 0, 0] == 1 and out.acc2[0, 0] == 1
    assert out.ybr[0, 0] == np.float32(2.0 ** -24)
    two_step = np.float32(np.float32(one_eps * one_eps) + np.float32(2.0 ** -24))
    assert two_step == np.float32(1.0 + 2.0 ** -22)                      # what two roundings would give
    fused = Fraction(float(one_eps)) ** 2 + Fraction(2) ** -24           # exact value, then one rounding
    assert fused > Fraction(1) + Fraction(2) ** -22 + Fraction(2) ** -24  # just above the tie
    assert out.y32[0, 0] == np.float32(1.0 + 2.0 ** -22 + 2.0 ** -23)
    assert out.y32[0, 0] != two_step
    # ymain is reported as the separately rounded product (it is a tap, not an operand of the sum)
    assert out.ymain[0, 0] == np.float32(one_eps * one_eps)


def test_rank0_equals_plain_w4a4(oracle):
    # rank 0, or L = R = 0: P == W and the branch contributes +0 (bit for bit)
    X, W, L, R, pk, act, out = _small_int_problem(oracle)
    pk0 = oracle.pack_int(W, None, None, 64, 8)
    act0 = oracle.quantize_act_int(X, pk0, 8)
    out0 = oracle.fwd_int(pk0, act0, want_acc=True)
    pkz = oracle.pack_int(W, np.zeros_like(L), np.zeros_like(R), 64, 8)
    actz = oracle.quantize_act_int(X, pkz, 8)
    outz = oracle.fwd_int(pkz, actz, want_acc=True)
    assert np.array_equal(pk0.P, W) and np.array_equal(pkz.P, W)
    assert np.array_equal(pk0.pq, pkz.pq) and np.array_equal(pk0.sw, pkz.sw)
    assert np.array_equal(out0.Y, outz.Y) and np.array_equal(out0.y32, outz.y32)
    assert not outz.ybr.any() and not out0.ybr.any()
    assert np.array_equal(out0.y32, out0.ymain)
    # and the main product alone is the plain W4A4 product of the dequantised tensors
    Xd = act0.xq.astype(np.float64) * act0.sx[:, None]
    Wd = (pk0.pq.astype(np.float64).reshape(pk0.N, -1, 64) * pk0.sw[:, :, None]).reshape(pk0.N, -1)
    ref = Xd @ Wd.T
    assert np.max(np.abs(ref - out0.y32)) <= 1e-5 * np.max(np.abs(ref))


def _on_grid_problem(rng, M, K, N, r, g, qmax_b):
    G = K // g
    pq = rng.integers(-7, 8, size=(N, K)).astype(np.int64)
    pq.reshape(N, G, g)[:, :, 0] = rng.choice([-7, 7], size=(N, G))
    sw = 2.0 ** rng.integers(-8, -5, size=(N, G))
    P0 = (pq.reshape(N, G, g) * sw[:, :, None]).reshape(N, K)
    lq = rng.integers(-3, 4, size=(N, r)).astype(np.int64)
    lq[np.arange(N), rng.integers(0, r, N)] = rng.choice([-qmax_b, qmax_b], size=N)
    rq = rng.integers(-3, 4, size=(r, K)).astype(np.int64)
    rq[np.arange(r), rng.integers(0, K, r)] = rng.choice([-qmax_b, qmax_b], size=r)
    sl = 2.0 ** rng.integers(-11, -9, size=N)
    sr = 2.0 ** rng.integers(-5, -3, size=r)
    Lh, Rh = lq * sl[:, None], rq * sr[:, None]
    W = P0 + Lh @ Rh
    assert np.array_equal(W.astype(np.float32).astype(np.float64), W)
    # X on both activation grids: entries in {0, +-a}, a = 7*qmax_b*2^k
    a = 7.0 * qmax_b * 2.0 ** rng.integers(-6, -2, size=M)
    sign = rng.choice([-1, 0, 1], size=(M, K))
    sign[:, 0] = 1
    X = sign * a[:, None]
    return X, W, Lh, Rh, pq, sw, lq, sl, rq, sr


@pytest.mark.parametrize("bits", [8, 6, 4])
def test_exact_rank_r_residual_is_recovered(oracle, bits):
    # Fixed point of Section 3.2 / Eq. 5: if W + (-L)R lies in the image of Q1 and L, R in the
    # image of Q2, packing is lossless: codes recovered, deq(Q1(P)) + L^R^ == W exactly.
    rng = np.random.default_rng(40 + bits)
    qb = {8: 127, 6: 31, 4: 7}[bits]
    M, K, N, r, g = 8, 128, 12, 4, 64
    X, W, Lh, Rh, pq, sw, lq, sl, rq, sr = _on_grid_problem(rng, M, K, N, r, g, qb)
    pk = oracle.pack_int(W, Lh, Rh, g, bits)
    assert np.array_equal(pk.pq, pq) and np.array_equal(pk.sw, sw.astype(np.float32))
    assert np.array_equal(pk.lq, lq) and np.array_equal(pk.rq, rq)
    assert np.array_equal(pk.sl, sl.astype(np.float32)) and np.array_equal(pk.sr, sr.astype(np.float32))
    Wrec = (pk.pq.astype(np.float64).reshape(N, -1, g) * pk.sw[:, :, None]).reshape(N, K) + \
        (pk.lq * pk.sl[:, None].astype(np.float64)) @ (pk.rq * pk.sr[:, None].astype(np.float64))
    assert np.array_equal(Wrec, W)
    # output side: the only loss left is the re-quantisation of T = X R^T (error <= st/2 each)
    ba = 8 if bits != 6 else 6
    qa = {8: 127, 6: 31}[ba]
    if ba != bits:
        # X must sit on the branch-activation grid too: rebuild with a = 7*qa*2^k
        a = 7.0 * qa * 2.0 ** rng.integers(-6, -2, size=M)
        X = np.sign(X) * a[:, None]
    act = oracle.quantize_act_int(X, pk, ba)
    assert np.array_equal(act.xq.astype(np.float64) * act.sx[:, None], X)
    assert np.array_equal(act.xb.astype(np.float64) * act.sxb[:, None], X)
    out = oracle.fwd_int(pk, act)
    exact = X @ W.T
    gap = (act.st[:, None].astype(np.float64) / 2) * np.abs(Lh).sum(1)[None, :]
    assert np.all(np.abs(out.y32 - exact) <= gap * (1 + 1e-6) + 1e-6 * np.abs(exact).max())


def test_single_component_branch_is_lossless(oracle):
    # r = 1: every T row is on its own grid (T/st = +-qmax), so Y = X W^T up to fp32 rounding
    rng = np.random.default_rng(7)
    M, K, N, g = 8, 128, 12, 64
    X, W, Lh, Rh, *_ = _on_grid_problem(rng, M, K, N, 1, g, 127)
    pk = oracle.pack_int(W, Lh, Rh, g, 8)
    act = oracle.quantize_act_int(X, pk, 8)
    assert np.all(np.abs(act.tq) == 127)
    out = oracle.fwd_int(pk, act)
    exact = X @ W.T
    assert np.max(np.abs(out.y32 - exact)) <= 4e-7 * np.max(np.abs(exact)) * 8


def test_residual_definition_and_flag(oracle):
    # Fig. 1: P = W - Q2(L)Q2(R) (dequantised factors); flag 0 gives P = W - L R.
    X, W, L, R, pk, act, out = _small_int_problem(oracle, lr_std=0.05)
    Lh = pk.lq.astype(np.float64) * pk.sl[:, None]
    Rh = pk.rq.astype(np.float64) * pk.sr[:, None]
    assert np.max(np.abs(pk.P - (W - Lh @ Rh))) <= 2 ** -23 * np.max(np.abs(W)) * 2
    pk2 = oracle.pack_int(W, L, R, 64, 8, residual_from_quantized=False)
    assert np.max(np.abs(pk2.P - (W.astype(np.float64) - L.astype(np.float64) @ R))) <= 2 ** -23 * np.max(np.abs(W)) * 2
    assert not np.array_equal(pk.P, pk2.P)
    # sign convention: the branch is ADDED.  W_eff = deq(Q1 P) + L^R^ is closer to W than deq(Q1 P)
    Pd = (pk.pq.astype(np.float64).reshape(pk.N, -1, 64) * pk.sw[:, :, None]).reshape(pk.N, -1)
    assert np.linalg.norm(Pd + Lh @ Rh - W) < 0.5 * np.linalg.norm(Pd - Lh @ Rh - W)


def test_error_upper_bound_eq2(oracle):
    # Eq. 2: ||XW - Q(X)Q(W)|| <= ||X-Q(X)|| ||W|| + ||Q(X)|| ||W-Q(W)||  (Frobenius)
    X, W, L, R, pk, act, out = _small_int_problem(oracle)
    pk0 = oracle.pack_int(W, None, None, 64, 8)
    Xd = act.xq.astype(np.float64) * act.sx[:, None]
    Wd = (pk0.pq.astype(np.float64).reshape(pk0.N, -1, 64) * pk0.sw[:, :, None]).reshape(pk0.N, -1)
    fro = np.linalg.norm
    lhs = fro(X.astype(np.float64) @ W.T.astype(np.float64) - Xd @ Wd.T)
    rhs = fro(X - Xd) * fro(W) + fro(Xd) * fro(W - Wd)
    assert lhs <= rhs
    # and the low-rank branch reduces the weight-side error when L R is the weight's own error
    E = (W - Wd).astype(np.float64)
    U, S, Vt = np.linalg.svd(E, full_matrices=False)
    r = 8
    Lc, Rc = (U[:, :r] * S[:r]).astype(np.float32), Vt[:r].astype(np.float32)
    pkc = oracle.pack_int(W, Lc, Rc, 64, 8)
    Pd = (pkc.pq.astype(np.float64).reshape(pkc.N, -1, 64) * pkc.sw[:, :, None]).reshape(pkc.N, -1)
    Weff = Pd + (pkc.lq * pkc.sl[:, None].astype(np.float64)) @ (pkc.rq * pkc.sr[:, None].astype(np.float64))
    assert fro(Weff - W) < fro(Wd - W) * 1.05


def test_permutation_equivariance(oracle):
    X, W, L, R, pk, act, out = _small_int_problem(oracle)
    rng = np.random.default_rng(5)
    pm, pn = rng.permutation(X.shape[0]), rng.permutation(W.shape[0])
    # tokens are independent rows; output channels are independent columns
    act_p = oracle.quantize_act_int(X[pm], pk, 8)
    assert np.array_equal(oracle.fwd_int(pk, act_p).Y, out.Y[pm])
    pk_p = oracle.pack_int(W[pn], L[pn], R, 64, 8)
    assert np.array_equal(oracle.fwd_int(pk_p, act).Y, out.Y[:, pn])
    # permuting K inside a group, jointly on X, W, R, leaves all accumulators unchanged
    K = X.shape[1]
    pk_idx = np.concatenate([g0 + rng.permutation(64) for g0 in range(0, K, 64)])
    pk_k = oracle.pack_int(W[:, pk_idx], L, R[:, pk_idx], 64, 8)
    act_k = oracle.quantize_act_int(X[:, pk_idx], pk_k, 8)
    out_k = oracle.fwd_int(pk_k, act_k, want_acc=True)
    assert np.array_equal(out_k.acc, out.acc) and np.array_equal(out_k.acc2, out.acc2)
    assert np.array_equal(out_k.Y, out.Y)


def test_power_of_two_scaling_and_negation(oracle):
    X, W, L, R, pk, act, out = _small_int_problem(oracle)
    a4 = oracle.quantize_act_int(X * np.float32(4), pk, 8)
    assert np.array_equal(a4.xq, act.xq) and np.array_equal(a4.tq, act.tq)
    assert np.array_equal(a4.sx, act.sx * 4) and np.array_equal(a4.st, act.st * 4)
    assert np.array_equal(oracle.fwd_int(pk, a4).y32, out.y32 * 4)
    an = oracle.quantize_act_int(-X, pk, 8)
    assert np.array_equal(oracle.fwd_int(pk, an).y32, -out.y32)


def test_accumulator_ranges(oracle):
    # worst cases stay far inside int32: |acc_g| <= 49 g, |accT| <= 127^2 K, |acc2| <= 127^2 r
    M, K, N, r, g = 2, 4608, 2, 128, 128
    X = np.full((M, K), 3.0, np.float32)
    W = np.full((N, K), -0.5, np.float32)
    L = np.full((N, r), 1.0, np.float32)
    R = np.full((r, K), 1.0, np.float32)
    pk = oracle.pack_int(W, L * 0, R, g, 8)
    act = oracle.quantize_act_int(X, pk, 8)
    out = oracle.fwd_int(pk, act, want_acc=True)
    assert np.all(out.acc == -49 * g) and 49 * 128 < 2 ** 22
    assert np.all(act.accT == 127 * 127 * K) and 127 * 127 * 4608 < 2 ** 31
    pk2 = oracle.pack_int(W, L, R, g, 8)        # all-equal T row => tq = 127, lq = 127
    act2 = oracle.quantize_act_int(X, pk2, 8)
    out2 = oracle.fwd_int(pk2, act2, want_acc=True)
    assert np.all(act2.tq == 127) and np.all(pk2.lq == 127)
    assert np.all(out2.acc2 == 127 * 127 * r)


def test_closed_form_constants(oracle):
    # X = c 1, W = w 1, no branch: codes all +-7, acc = 49 g, y = K c w up to fp32 rounding
    M, K, N, g = 3, 256, 5, 64
    c, w = 0.75, -0.0123
    pk = oracle.pack_int(np.full((N, K), w, np.float32), None, None, g, 8)
    act = oracle.quantize_act_int(np.full((M, K), c, np.float32), pk, 8)
    out = oracle.fwd_int(pk, act, want_acc=True)
    assert np.all(act.xq == 7) and np.all(pk.pq == -7) and np.all(out.acc == -49 * g)
    want = K * float(np.float32(c)) * float(np.float32(w))
    assert np.max(np.abs(out.y32 - want)) <= 8 * 2 ** -24 * abs(want)


def test_exhaustive_tiny_int(oracle):
    # all 15^2 x 15^2 on-grid pairs with K = g = 2 ... 3 checked against Python integers
    # (rows that contain a +-7 are on the grid of Q, so codes must come back unchanged)
    sx, swt = 0.25, 2.0 ** -5
    codes = range(-7, 8)
    rows = [c for c in itertools.product(codes, repeat=2) if max(abs(v) for v in c) == 7]
    X = np.array(rows, np.float32) * np.float32(sx)
    W = np.array(rows, np.float32) * np.float32(swt)
    pk = oracle.pack_int(W, None, None, 2, 8)
    act = oracle.quantize_act_int(X, pk, 8)
    out = oracle.fwd_int(pk, act, want_acc=True)
    assert np.array_equal(act.xq, np.array(rows)) and np.array_equal(pk.pq, np.array(rows))
    assert np.all(act.sx == np.float32(sx)) and np.all(pk.sw == np.float32(swt))
    for i, a in enumerate(rows):
        for j, b in enumerate(rows):
            dot = a[0] * b[0] + a[1] * b[1]
            assert out.acc[i, j, 0] == dot
            assert out.y32[i, j] == np.float32(dot * sx * swt)   # exact: small dyadic numbers
    # off-grid rows (max |code| < 7): nearest-integer property in exact rationals
    rows3 = list(itertools.product(range(-3, 4), repeat=3))
    X3 = np.array(rows3, np.float32)
    pk3 = oracle.pack_int(np.ones((1, 3), np.float32), None, None, 3, 8)
    act3 = oracle.quantize_act_int(X3, pk3, 8)
    for row, q, s in zip(rows3, act3.xq, act3.sx):
        amax = max(abs(v) for v in row)
        if amax == 0:
            assert s == 1 and not q.any()
            continue
        assert s == np.float32(amax) / np.float32(7)
        for v, qi in zip(row, q):
            assert abs(Fraction(7 * v, amax) - int(qi)) <= Fraction(1, 2) + Fraction(1, 10 ** 6)


# --------------------------------------------------------------------------------------
# whole MX path
# --------------------------------------------------------------------------------------

def test_mx_forward_against_exact_rationals(oracle):
    rng = np.random.default_rng(11)
    M, K, N, r = 5, 64, 6, 4
    X = wl.round_to_bf16(rng.standard_normal((M, K)).astype(np.float32))
    W = (rng.standard_normal((N, K)) * 0.02).astype(np.float32)
    L = (rng.standard_normal((N, r)) * 1e-3).astype(np.float32)
    R = (rng.standard_normal((r, K)) * 1e-3).astype(np.float32)
    pk = oracle.pack_mx(W, L, R)
    act = oracle.quantize_act_mx(X, pk)
    out = oracle.fwd_mx(pk, act)
    F = Fraction
    vx = oracle.e2m1_decode(act.xc)
    vw = oracle.e2m1_decode(pk.pc)
    sx = oracle.e8m0_decode(act.xe)
    sw = oracle.e8m0_decode(pk.pe)
    t8 = oracle.e4m3_decode(act.tq8)
    l8 = oracle.e4m3_decode(pk.l8)
    x8 = oracle.e4m3_decode(act.xb8)
    r8 = oracle.e4m3_decode(pk.r8)
    for m in range(M):
        for j in range(r):
            T = F(float(act.sxb[m])) * F(float(pk.sr[j])) * sum(F(float(a)) * F(float(b)) for a, b in zip(x8[m], r8[j]))
            assert abs(float(T) - float(act.T[m, j])) <= 2 ** -22 * abs(float(T))
        for n in range(N):
            main = sum(F(float(sx[m, b])) * F(float(sw[n, b])) *
                       sum(F(float(vx[m, 32 * b + k])) * F(float(vw[n, 32 * b + k])) for k in range(32))
                       for b in range(K // 32))
            br = F(float(act.st[m])) * F(float(pk.sl[n])) * sum(F(float(a)) * F(float(b)) for a, b in zip(t8[m], l8[n]))
            assert out.ymain[m, n] == np.float32(float(main))      # single rounding of an exact sum
            assert abs(float(br) - float(out.ybr[m, n])) <= 2 ** -22 * abs(float(br))
            assert out.y32[m, n] == np.float32(out.ymain[m, n]) + np.float32(out.ybr[m, n])
    # MX quantisation error of X is bounded per block (half spacing unless saturated)
    Xd = vx.astype(np.float64).reshape(M, -1, 32) * sx[:, :, None]
    err = np.abs(Xd.reshape(M, K) - X)
    assert np.all(err <= np.repeat(sx, 32, axis=1) * 2.0)
    # FP8 branch codes: relative error <= 2^-4 for normal values, amax -> 448
    assert np.all(np.abs(x8).max(axis=1) == 448)
    big = np.abs(X) > np.abs(X).max(axis=1, keepdims=True) * 2.0 ** -6
    rel = np.abs(x8 * act.sxb[:, None] - X) / np.abs(X)
    assert np.all(rel[big] <= 2 ** -4 * (1 + 1e-6))


def test_mx_rank0_and_residual(oracle):
    rng = np.random.default_rng(12)
    M, K, N, r = 4, 96, 5, 4
    X = wl.round_to_bf16(rng.standard_normal((M, K)).astype(np.float32))
    W = (rng.standard_normal((N, K)) * 0.02).astype(np.float32)
    pk0 = oracle.pack_mx(W, None, None)
    pkz = oracle.pack_mx(W, np.zeros((N, r), np.float32), np.zeros((r, K), np.float32))
    assert np.array_equal(pk0.P, W) and np.array_equal(pkz.pc, pk0.pc) and np.array_equal(pkz.pe, pk0.pe)
    o0 = oracle.fwd_mx(pk0, oracle.quantize_act_mx(X, pk0))
    oz = oracle.fwd_mx(pkz, oracle.quantize_act_mx(X, pkz))
    assert np.array_equal(o0.Y, oz.Y) and not oz.ybr.any()
    # on-grid P (E2M1 values times power-of-two block scales) is recovered exactly
    codes = rng.integers(0, 16, size=(N, K)).astype(np.uint8)
    codes.reshape(N, -1, 32)[:, :, 0] = 7          # a 6 in each block fixes the scale
    sc = 2.0 ** rng.integers(-9, -5, size=(N, K // 32))
    Wg = (oracle.e2m1_decode(codes).astype(np.float64).reshape(N, -1, 32) * sc[:, :, None]).reshape(N, K)
    pkg = oracle.pack_mx(Wg.astype(np.float32), None, None)
    assert np.array_equal(oracle.e2m1_decode(pkg.pc), oracle.e2m1_decode(codes))
    assert np.array_equal(oracle.e8m0_decode(pkg.pe), sc)   # floor(log2(6 s)) - 2 = log2 s


# --------------------------------------------------------------------------------------
# MXB family: block-scaled E4M3 branch (App. A.3 "MXFP8e4": blocks of 32, E8M0 scale)
# --------------------------------------------------------------------------------------

def test_mxfp8_block_scale_nearest_and_idempotent(oracle):
    rng = np.random.default_rng(21)
    v = (rng.standard_normal(32 * 60) * np.exp(rng.uniform(-8, 8, 32 * 60))).astype(np.float32)
    v[96:128] = 0.0
    v[128] = 0.75; v[129:160] = 0.0                      # a lone value fixes scale and code by hand
    codes, e = oracle.quant_mxfp8(v)
    assert e[3] == 0 and np.all(codes[96:128] & 0x7F == 0)
    # 0.75 = 1.5 * 2^-1: floor(log2) = -1, E = -1 - 8 + 127; element = 0.75 * 2^9 = 384 = 1.5 * 2^8 -> e=15, m=4
    assert e[4] == 118 and codes[128] == ((15 << 3) | 4)
    dec_tab = oracle.e4m3_decode(np.arange(127, dtype=np.uint8)).astype(np.float64)
    deq = oracle.e4m3_decode(codes).astype(np.float64).reshape(-1, 32)
    sc = oracle.e8m0_decode(e)
    vb = v.astype(np.float64).reshape(-1, 32)
    for b in range(vb.shape[0]):
        a = np.abs(vb[b]).max()
        if a == 0:
            continue
        assert sc[b] == 2.0 ** (np.floor(np.log2(a)) - 8)          # exponent rule
        u = vb[b] / sc[b]                                           # exact (power of two)
        assert 256 <= np.abs(u).max() < 512
        for ui, di in zip(u, deq[b]):                               # nearest representable, saturating at 448
            best = np.min(np.abs(dec_tab - abs(ui)))
            assert abs(abs(di) - abs(ui)) <= best and abs(di) <= 448
            assert di == 0 or np.sign(di) == np.sign(ui)
    # idempotence (Section 3.2): the block maximum stays in its binade, so codes and scales repeat
    back = (deq * sc[:, None]).astype(np.float32).ravel()
    codes2, e2 = oracle.quant_mxfp8(back)
    nz = np.repeat(np.abs(vb).max(axis=1) > 0, 32)
    assert np.array_equal(e2[np.abs(vb).max(axis=1) > 0], e[np.abs(vb).max(axis=1) > 0])
    assert np.array_equal(oracle.e4m3_decode(codes2)[nz], oracle.e4m3_decode(codes)[nz])
    # scaling by a power of two moves only the scale byte
    codes3, e3 = oracle.quant_mxfp8(v * np.float32(2.0 ** 5))
    assert np.array_equal(codes3[nz], codes[nz]) and np.array_equal(e3[e > 0].astype(int), e[e > 0].astype(int) + 5)


@pytest.mark.parametrize("elem", [8, 6])
def test_mxb_forward_against_exact_rationals(oracle, elem):
    rng = np.random.default_rng(22)
    quant = oracle.quant_mxfp8 if elem == 8 else oracle.quant_mxfp6
    M, K, N, r = 4, 64, 5, 32
    X = wl.round_to_bf16(rng.standard_normal((M, K)).astype(np.float32))
    W = (rng.standard_normal((N, K)) * 0.02).astype(np.float32)
    L = (rng.standard_normal((N, r)) * 3e-2).astype(np.float32)
    R = (rng.standard_normal((r, K)) * 3e-2).astype(np.float32)
    pk = oracle.pack_mxb(W, L, R, elem=elem)
    act = oracle.quantize_act_mxb(X, pk)
    out = oracle.fwd_mxb(pk, act)
    F = Fraction
    f = lambda a: F(float(a))
    vx, vw = oracle.e2m1_decode(act.xc), oracle.e2m1_decode(pk.pc)
    sx, sw = oracle.e8m0_decode(act.xe), oracle.e8m0_decode(pk.pe)
    x8, r8, t8, l8 = (oracle.mxb_decode(c, elem) for c in (act.xb8, pk.r8, act.tq8, pk.l8))
    xbe, re, te, le = (oracle.e8m0_decode(c) for c in (act.xbe, pk.re, act.te, pk.le))
    # residual: P = fl(W - sum_j Lhat Rhat) from the dequantised factors (Fig. 1), exact in rationals
    for n in range(N):
        for k in range(0, K, 7):
            d = sum(f(l8[n, j]) * f(le[n, j // 32]) * f(r8[j, k]) * f(re[j, k // 32]) for j in range(r))
            assert pk.P[n, k] == np.float32(float(f(W[n, k]) - d))
    # the factors' codes are the block quantiser applied to their rows
    c, e = quant(R[3]); assert np.array_equal(c, pk.r8[3]) and np.array_equal(e, pk.re[3])
    c, e = quant(L[2]); assert np.array_equal(c, pk.l8[2]) and np.array_equal(e, pk.le[2])
    c, e = quant(X[1]); assert np.array_equal(c, act.xb8[1]) and np.array_equal(e, act.xbe[1])
    for m in range(M):
        Tex = []
        for j in range(r):
            T = sum(f(xbe[m, b]) * f(re[j, b]) * sum(f(x8[m, 32 * b + k]) * f(r8[j, 32 * b + k]) for k in range(32))
                    for b in range(K // 32))
            assert act.T[m, j] == np.float32(float(T))               # one rounding of the exact contraction
            Tex.append(T)
        c, e = quant(act.T[m]); assert np.array_equal(c, act.tq8[m]) and np.array_equal(e, act.te[m])
        for n in range(N):
            main = sum(f(sx[m, b]) * f(sw[n, b]) * sum(f(vx[m, 32 * b + k]) * f(vw[n, 32 * b + k]) for k in range(32))
                       for b in range(K // 32))
            br = sum(f(te[m, b]) * f(le[n, b]) * sum(f(t8[m, 32 * b + j]) * f(l8[n, 32 * b + j]) for j in range(32))
                     for b in range(r // 32))
            assert out.ymain[m, n] == np.float32(float(main)) and out.ybr[m, n] == np.float32(float(br))
            assert out.y32[m, n] == np.float32(float(main + br))     # both accumulators, one rounding
            assert out.Y[m, n] == oracle.bf16_rne(float(out.y32[m, n]))
    # the branch approximates X R^T L^T: relative error 2^-4 per factor and element (both formats keep
    # 3 mantissa bits; E2M3's narrow exponent range adds absolute error on the small elements of a block)
    ref = X.astype(np.float64) @ R.astype(np.float64).T @ L.astype(np.float64).T
    assert np.abs(out.ybr - ref).max() <= (0.2 if elem == 8 else 0.3) * np.abs(ref).max()


def test_e2m3_table_rounding_and_block_scale(oracle):
    g = _golden()
    dec = oracle.e2m3_decode(np.arange(64, dtype=np.uint8))
    assert list(dec[:32]) == g["e2m3"] and list(dec[32:]) == [-v if v else -0.0 for v in g["e2m3"]]
    tab = np.array(g["e2m3"])
    rng = np.random.default_rng(41)
    for u in np.concatenate([rng.uniform(-9, 9, 4000), (tab[:-1] + tab[1:]) / 2, -(tab[:-1] + tab[1:]) / 2, [7.5, 7.75, 100.0, -8.0]]):
        u = float(np.float32(u))
        c = oracle.e2m3_encode(u)
        d = float(oracle.e2m3_decode(np.array([c], np.uint8))[0])
        best = np.min(np.abs(tab - abs(u)))
        assert abs(abs(d) - abs(u)) == best and (d == 0 or np.sign(d) == np.sign(u))       # nearest, saturating at 7.5
        if np.sum(np.abs(tab - abs(u)) == best) == 2:                                     # exact tie: even mantissa
            assert (c & 1) == 0
    v = (rng.standard_normal(32 * 40) * np.exp(rng.uniform(-8, 8, 32 * 40))).astype(np.float32)
    v[64:96] = 0.0
    v[96] = -0.75; v[97] = 0.2; v[98:128] = 0.0      # 0.75 = 1.5 * 2^-1: exponent -1 - 2 = -3: 0.75 * 8 = 6 -> code 28; 1.6 -> 1.625 = code 13
    codes, e = oracle.quant_mxfp6(v)
    assert e[2] == 0 and not (codes[64:96] & 31).any()
    assert e[3] == 124 and codes[96] == (32 | 28) and codes[97] == 13
    vb = v.astype(np.float64).reshape(-1, 32)
    deq = oracle.e2m3_decode(codes).astype(np.float64).reshape(-1, 32)
    for b in range(vb.shape[0]):
        a = np.abs(vb[b]).max()
        if a == 0:
            continue
        sc = 2.0 ** (int(e[b]) - 127)
        assert sc == 2.0 ** (np.floor(np.log2(a)) - 2)
        u = vb[b] / sc
        assert 4 <= np.abs(u).max() < 8
        for ui, di in zip(u, deq[b]):
            assert abs(abs(di) - abs(ui)) <= np.min(np.abs(tab - abs(ui)))
    back = (deq * (2.0 ** (e.astype(np.float64) - 127))[:, None]).astype(np.float32).ravel()
    c2, e2 = oracle.quant_mxfp6(back)                                                      # idempotence (Section 3.2)
    nzb = np.abs(vb).max(axis=1) > 0
    assert np.array_equal(e2[nzb], e[nzb])
    assert np.array_equal(oracle.e2m3_decode(c2).reshape(-1, 32)[nzb], oracle.e2m3_decode(codes).reshape(-1, 32)[nzb])


def test_mxb_rank0_equals_mx_rank0_and_grid_factors_are_exact(oracle):
    rng = np.random.default_rng(23)
    M, K, N, r = 4, 96, 6, 32
    X = wl.round_to_bf16(rng.standard_normal((M, K)).astype(np.float32))
    W = (rng.standard_normal((N, K)) * 0.02).astype(np.float32)
    pa, pb = oracle.pack_mx(W, None, None), oracle.pack_mxb(W, None, None)
    assert np.array_equal(pa.pc, pb.pc) and np.array_equal(pa.pe, pb.pe)
    ya = oracle.fwd_mx(pa, oracle.quantize_act_mx(X, pa))
    yb = oracle.fwd_mxb(pb, oracle.quantize_act_mxb(X, pb))
    assert np.array_equal(ya.Y, yb.Y) and np.array_equal(ya.y32, yb.y32)
    pz = oracle.pack_mxb(W, np.zeros((N, r), np.float32), np.zeros((r, K), np.float32))
    yz = oracle.fwd_mxb(pz, oracle.quantize_act_mxb(X, pz))
    assert np.array_equal(yz.Y, yb.Y) and not yz.ybr.any()
    # factors that already lie on the MXFP8e4 grid are stored without loss (Section 3.2 fixed point)
    cod = rng.integers(0, 127, size=(r, K)).astype(np.uint8) | (rng.integers(0, 2, size=(r, K)).astype(np.uint8) << 7)
    cod.reshape(r, -1, 32)[:, :, 0] = 126                      # 448 in every block fixes the scale
    sc = 2.0 ** rng.integers(-12, -6, size=(r, K // 32))
    Rg = (oracle.e4m3_decode(cod).astype(np.float64).reshape(r, -1, 32) * sc[:, :, None]).reshape(r, K).astype(np.float32)
    pg = oracle.pack_mxb(W, np.zeros((N, r), np.float32), Rg)
    back = oracle.e4m3_decode(pg.r8).astype(np.float64).reshape(r, -1, 32) * oracle.e8m0_decode(pg.re)[:, :, None]
    assert np.array_equal(back.reshape(r, K).astype(np.float32), Rg)


# --------------------------------------------------------------------------------------
# MXI family: MXINT4 main, MXINT8 / MXINT4 branch (App. A.3: signed int elements, blocks of 32,
# E8M0 scale; the integer rows of the mixed-precision tables, Section 4.3)
# --------------------------------------------------------------------------------------

@pytest.mark.parametrize("bits", [4, 8])
def test_mxint_block_quantiser(oracle, bits):
    step, top = _golden()["mxint"][bits]
    qmax = 2 ** (bits - 1) - 1
    assert top == qmax * step and step == 2.0 ** -(bits - 2)
    rng = np.random.default_rng(31 + bits)
    v = (rng.standard_normal(32 * 80) * np.exp(rng.uniform(-8, 8, 32 * 80))).astype(np.float32)
    v[64:96] = 0.0
    v[96] = 1.0; v[97] = -0.3; v[98:128] = 0.0           # hand-checked block: shared exponent 0
    v[128] = -7.9; v[129] = 2.5; v[130:160] = 0.0        # 7.9 = 1.975 * 2^2: shared exponent 2
    codes, e = oracle.quant_mxint(v, bits)
    assert e[2] == 0 and not codes[64:96].any()
    assert e[3] == 127 and codes[96] == 2 ** (bits - 2) and codes[97] == -round(0.3 / step)
    assert e[4] == 129 and codes[128] == -(qmax if bits == 4 else 126) and codes[129] == round(2.5 / 4 / step)
    assert np.abs(codes.astype(int)).max() <= qmax
    vb = v.astype(np.float64).reshape(-1, 32)
    cb = codes.astype(np.float64).reshape(-1, 32)
    for b in range(vb.shape[0]):
        a = np.abs(vb[b]).max()
        if a == 0:
            continue
        shared = 2.0 ** np.floor(np.log2(a))                      # the specification's shared scale
        assert 2.0 ** (int(e[b]) - 127) == shared
        u = vb[b] / shared                                          # exact; |u| < 2
        deq = cb[b] * step
        grid = np.arange(-qmax, qmax + 1) * step
        for ui, di in zip(u, deq):                                  # nearest grid point (saturating)
            assert abs(di - ui) <= np.min(np.abs(grid - ui))
        assert np.abs(deq).max() >= 1.0                             # the maximum sits in the top octave
        inside = np.abs(u) <= top
        assert np.all(np.abs(deq - u)[inside] <= step / 2) and np.all(np.abs(deq - u)[~inside] < step)
    # exact ties go to the even code
    t = np.zeros(32, np.float32); t[0] = 1.0
    t[1:5] = np.array([0.5, 1.5, 2.5, -3.5], np.float32) * np.float32(step)
    ct, _ = oracle.quant_mxint(t, bits)
    assert list(ct[1:5]) == [0, 2, 2, -4]
    # idempotence (Section 3.2) and power-of-two equivariance
    back = (cb * step * (2.0 ** (e.astype(np.float64) - 127))[:, None]).astype(np.float32).ravel()
    c2, e2 = oracle.quant_mxint(back, bits)
    nzb = np.abs(vb).max(axis=1) > 0
    assert np.array_equal(e2[nzb], e[nzb]) and np.array_equal(c2.reshape(-1, 32)[nzb], codes.reshape(-1, 32)[nzb])
    c3, e3 = oracle.quant_mxint(v * np.float32(2.0 ** -7), bits)
    assert np.array_equal(c3, codes) and np.array_equal(e3[nzb].astype(int), e[nzb].astype(int) - 7)
    c4, _ = oracle.quant_mxint(-v, bits)
    assert np.array_equal(c4, -codes)


@pytest.mark.parametrize("bw", [8, 4])
def test_mxi_forward_against_exact_rationals(oracle, bw):
    rng = np.random.default_rng(32 + bw)
    M, K, N, r = 4, 64, 5, 32
    X = wl.round_to_bf16(rng.standard_normal((M, K)).astype(np.float32))
    W = (rng.standard_normal((N, K)) * 0.02).astype(np.float32)
    L = (rng.standard_normal((N, r)) * 3e-2).astype(np.float32)
    R = (rng.standard_normal((r, K)) * 3e-2).astype(np.float32)
    pk = oracle.pack_mxi(W, L, R, bw)
    act = oracle.quantize_act_mxi(X, pk)
    out = oracle.fwd_mxi(pk, act)
    F = Fraction
    sc = lambda byte, bits: F(2) ** (int(byte) - 127 - (bits - 2))
    val = lambda codes, bytes_, bits: [[F(int(c)) * sc(bytes_[i][j // 32], bits) for j, c in enumerate(row)]
                                       for i, row in enumerate(codes)]
    xv, pv = val(act.xq, act.xe, 4), val(pk.pq, pk.pe, 4)
    xbv, rv = val(act.xb, act.xbe, 8), val(pk.rq, pk.re, bw)
    tv, lv = val(act.tq, act.te, 8), val(pk.lq, pk.le, bw)
    for n in range(N):                                           # residual from the dequantised factors
        for k in range(0, K, 5):
            d = sum(lv[n][j] * rv[j][k] for j in range(r))
            assert pk.P[n, k] == np.float32(float(F(float(W[n, k])) - d))
    c, e = oracle.quant_mxint(R[3], bw); assert np.array_equal(c, pk.rq[3]) and np.array_equal(e, pk.re[3])
    c, e = oracle.quant_mxint(L[2], bw); assert np.array_equal(c, pk.lq[2]) and np.array_equal(e, pk.le[2])
    c, e = oracle.quant_mxint(pk.P[1], 4); assert np.array_equal(c, pk.pq[1]) and np.array_equal(e, pk.pe[1])
    c, e = oracle.quant_mxint(X[1], 4); assert np.array_equal(c, act.xq[1]) and np.array_equal(e, act.xe[1])
    c, e = oracle.quant_mxint(X[1], 8); assert np.array_equal(c, act.xb[1]) and np.array_equal(e, act.xbe[1])
    for m in range(M):
        for j in range(r):
            T = sum(xbv[m][k] * rv[j][k] for k in range(K))
            assert act.T[m, j] == np.float32(float(T))              # one rounding of the exact contraction
        c, e = oracle.quant_mxint(act.T[m], 8); assert np.array_equal(c, act.tq[m]) and np.array_equal(e, act.te[m])
        for n in range(N):
            main = sum(xv[m][k] * pv[n][k] for k in range(K))
            br = sum(tv[m][j] * lv[n][j] for j in range(r))
            assert out.ymain[m, n] == np.float32(float(main)) and out.ybr[m, n] == np.float32(float(br))
            assert out.y32[m, n] == np.float32(float(main + br))
            assert out.Y[m, n] == oracle.bf16_rne(float(out.y32[m, n]))
    # the integer contractions inside the blocks are textbook integer matmuls (uniform scales)
    Xu = np.tile(np.arange(-16, 16, dtype=np.float32) / 8, (M, K // 32)); Xu[:, 0::32] = 1.9
    Wu = np.tile(np.arange(16, -16, -1, dtype=np.float32) / 16, (N, K // 32)); Wu[:, 1::32] = 1.9
    pu = oracle.pack_mxi(Wu, None, None, bw)
    au = oracle.quantize_act_mxi(Xu, pu)
    assert np.all(au.xe == 127) and np.all(pu.pe == 127)
    ref = (au.xq.astype(np.int64) @ pu.pq.astype(np.int64).T) / 16.0
    assert np.array_equal(oracle.fwd_mxi(pu, au).y32, ref.astype(np.float32))
    # the 8-bit branch approximates X R^T L^T far better than the 4-bit main product's step
    ref = X.astype(np.float64) @ R.astype(np.float64).T @ L.astype(np.float64).T
    assert np.abs(out.ybr - ref).max() <= (0.03 if bw == 8 else 0.4) * np.abs(ref).max()


def test_mxi_rank0_zero_factors_and_lossless_grids(oracle):
    rng = np.random.default_rng(35)
    M, K, N, r = 4, 96, 6, 32
    X = wl.round_to_bf16(rng.standard_normal((M, K)).astype(np.float32))
    W = (rng.standard_normal((N, K)) * 0.02).astype(np.float32)
    p0 = oracle.pack_mxi(W, None, None)
    pz = oracle.pack_mxi(W, np.zeros((N, r), np.float32), np.zeros((r, K), np.float32))
    assert np.array_equal(p0.P, W) and np.array_equal(p0.pq, pz.pq) and np.array_equal(p0.pe, pz.pe)
    y0 = oracle.fwd_mxi(p0, oracle.quantize_act_mxi(X, p0))
    yz = oracle.fwd_mxi(pz, oracle.quantize_act_mxi(X, pz))
    assert np.array_equal(y0.Y, yz.Y) and not yz.ybr.any()
    # Section 3.2 fixed point: weights on the MXINT4 grid, factors on the MXINT8 grid, an input on the
    # MXINT4 grid: everything is stored without loss and the main product equals X W^T exactly
    cw = rng.integers(-7, 8, size=(N, K)); cw.reshape(N, -1, 32)[:, :, 0] = 5
    sw = 2.0 ** rng.integers(-9, -5, size=(N, K // 32))
    Wg = (cw.reshape(N, -1, 32) * sw[:, :, None] / 4).reshape(N, K).astype(np.float32)
    cx = rng.integers(-7, 8, size=(M, K)); cx.reshape(M, -1, 32)[:, :, 3] = -6
    sx = 2.0 ** rng.integers(-3, 3, size=(M, K // 32))
    Xg = (cx.reshape(M, -1, 32) * sx[:, :, None] / 4).reshape(M, K).astype(np.float32)
    pg = oracle.pack_mxi(Wg, None, None)
    ag = oracle.quantize_act_mxi(Xg, pg)
    assert np.array_equal(pg.pq, cw) and np.array_equal(ag.xq, cx)
    assert np.array_equal(oracle.mxint_scale(pg.pe, 4) * 4, sw) and np.array_equal(oracle.mxint_scale(ag.xe, 4) * 4, sx)
    exact = Xg.astype(np.float64) @ Wg.astype(np.float64).T          # exact in fp64 at these magnitudes
    assert np.array_equal(oracle.fwd_mxi(pg, ag).y32, exact.astype(np.float32))
    # inputs in the block maximum's own octave with 6 fraction bits pass through MXINT8 unchanged
    Xs = (np.round(rng.uniform(1.0, 1.98, size=(M, K)) * 64) / 64 * rng.choice([-1, 1], size=(M, K))).astype(np.float32)
    cs, es = oracle.quant_mxint(Xs, 8)
    assert np.array_equal((cs.astype(np.float64) * np.repeat(oracle.mxint_scale(es, 8), 32)).astype(np.float32), Xs.ravel())


# --------------------------------------------------------------------------------------
# activation smoothing (Section 3.4; App. A.1)
# --------------------------------------------------------------------------------------

def test_smoothing_is_a_reciprocal_multiply_and_tames_outlier_channels(oracle):
    rng = np.random.default_rng(51)
    M, K, N, r = 48, 256, 32, 16
    X = rng.standard_normal((M, K)).astype(np.float32)
    out_cols = rng.choice(K, 4, replace=False)
    X[:, out_cols] *= 30                                   # the situation smoothing addresses
    W = (rng.standard_normal((N, K)) * 0.02).astype(np.float32)
    g = smoothing_vector(X, W)
    assert g.shape == (K,) and np.all(g > 0) and np.all(g[out_cols] > np.median(g) * 3)
    Xs = oracle.smooth(X, g)
    # correctly rounded reciprocal, one rounding for the product (exact rationals)
    for m, k in [(0, 0), (3, int(out_cols[0])), (47, 255), (10, 77)]:
        rg = np.float32(float(Fraction(1) / Fraction(float(g[k]))))
        assert Xs[m, k] == np.float32(float(Fraction(float(X[m, k])) * Fraction(float(rg))))
    assert np.array_equal(oracle.smooth(X, np.ones(K, np.float32)), X)          # gamma = 1: identity
    p2 = np.exp2(rng.integers(-3, 4, K)).astype(np.float32)
    assert np.array_equal(oracle.smooth(X, p2), X / p2)                          # powers of two: exact division
    # the layer is unchanged in exact arithmetic: (X / gamma)(W gamma)^T = X W^T
    Ws = (W.astype(np.float64) * g).astype(np.float32)
    ref = X.astype(np.float64) @ W.astype(np.float64).T
    assert np.abs(Xs.astype(np.float64) @ Ws.astype(np.float64).T - ref).max() <= 1e-5 * np.abs(ref).max()
    # and the 4-bit product gets closer to it (outlier channels no longer set every token's scale)
    L = np.zeros((N, r), np.float32); R = np.zeros((r, K), np.float32)
    def err(Xin, Win):
        pk = oracle.pack_int(Win, L, R, 64, 8)
        return np.abs(oracle.fwd_int(pk, oracle.quantize_act_int(Xin, pk, 8), want_acc=False).y32 - ref).mean()
    assert err(Xs, Ws) < 0.6 * err(X, W)


def test_workload_generator_is_seeded():
    l = wl.shrink(wl.LAYERS["c2_qkv"], M=16, K=128, N=64, r=16)
    a, b = wl.make_inputs(l), wl.make_inputs(l)
    assert all(np.array_equal(x, y) for x, y in zip(a, b))
    X = a[0]
    assert np.array_equal(wl.round_to_bf16(X), X)
    assert [x.shape for x in a] == [(16, 128), (64, 128), (64, 16), (16, 128)]


# ---- rotation search (Section 3.3, Eq. 6-7) -----------------------------------------------------------------------
def _rot_case(seed, N=96, K=160, r=16, outlier=8.0):
    rng = np.random.default_rng(seed)
    L = rng.standard_normal((N, r)).astype(np.float32) * 0.05
    R = rng.standard_normal((r, K)).astype(np.float32) * 0.05
    L[:, 3] *= outlier
    R[5, :] *= outlier
    X0 = np.linalg.qr(rng.standard_normal((r, r)))[0].astype(np.float32)
    return L, R, X0


def test_rot_errors_are_roundings_of_the_rotated_factors(oracle):
    """Eq. 7's two terms: E1, E2 are the errors of a per-row integer quantiser applied to L Omega and Omega^T R: every
    entry within half a step of its row, every reconstructed value an integer multiple of the step within the code
    range, the row maximum exact; the loss is the sum of the two mean squares."""
    L, R, X0 = _rot_case(1)
    for bits in (8, 6, 4):
        qmax = 2 ** (bits - 1) - 1
        st = oracle.rot_init(16, X0)
        out = oracle.rot_step(L, R, st, bits=bits, lr=0.0)
        for Z, E in ((L.astype(np.float64) @ X0, out.E1), (X0.T.astype(np.float64) @ R, out.E2)):
            step = np.abs(Z).max(axis=1, keepdims=True) / qmax
            assert np.all(np.abs(E) <= 0.5 * step * (1 + 1e-5) + 1e-9)
            codes = (Z + E) / step
            assert np.all(np.abs(codes - np.rint(codes)) < 1e-3) and np.abs(np.rint(codes)).max() == qmax
        assert out.loss == pytest.approx(np.mean(out.E1.astype(np.float64) ** 2) + np.mean(out.E2.astype(np.float64) ** 2), rel=1e-12)
        assert np.array_equal(st.Omega, X0)          # a zero learning rate moves nothing


def test_rot_gradient_is_the_gradient_of_the_loss_with_the_codes_held(oracle):
    """App. B.2's convention applied to Eq. 7: with the quantised values C1, C2 held fixed the loss is the quadratic
    mean((C1 - L Omega)^2) + mean((C2 - Omega^T R)^2); its central differences give G entry by entry."""
    L, R, X0 = _rot_case(2)
    st = oracle.rot_init(16, X0)
    out = oracle.rot_step(L, R, st, bits=4, lr=0.0, grad_scale=3.0)
    L64, R64, X64 = L.astype(np.float64), R.astype(np.float64), X0.astype(np.float64)
    C1, C2 = L64 @ X64 + out.E1, X64.T @ R64 + out.E2

    def f(X):
        return np.mean((C1 - L64 @ X) ** 2) + np.mean((C2 - X.T @ R64) ** 2)

    h = 1e-4
    for (i, j) in [(0, 0), (3, 5), (5, 3), (15, 2), (7, 7)]:
        D = np.zeros((16, 16))
        D[i, j] = h
        fd = (f(X64 + D) - f(X64 - D)) / (2 * h)       # exact for a quadratic, up to rounding
        assert 3.0 * fd == pytest.approx(float(out.G[i, j]), rel=2e-4, abs=1e-9)


@pytest.mark.parametrize("s,beta", [(2, 0.0), (6, 0.0), (3, 0.9)])
def test_rot_update_is_the_cayley_transform_of_the_projected_momentum(oracle, s, beta):
    """The published iteration converges to the closed-form Cayley transform (I - a/2 W)^-1 (I + a/2 W) X of the
    skew-symmetric W built from the momentum; after s passes the distance is at most a^s * 2 a^2 / (1 - a) * ||X||
    with a = ||alpha W / 2||_2.  A wrong sign, a dropped 1/2 or a transposed operand leaves an error of order a."""
    L, R, X0 = _rot_case(3)
    rng = np.random.default_rng(4)
    M0 = (rng.standard_normal((16, 16)) * 1e-3).astype(np.float32)
    st = oracle.rot_init(16, X0, M0)
    lr, scale = 0.5, 2500.0
    out = oracle.rot_step(L, R, st, bits=4, lr=lr, beta=beta, s=s, grad_scale=scale)
    X = X0.astype(np.float64)
    M = beta * M0.astype(np.float64) - out.G.astype(np.float64)
    Wh = M @ X.T - 0.5 * X @ (X.T @ M @ X.T)
    W = Wh - Wh.T
    assert np.allclose(W, -W.T)
    alpha = min(lr, 1.0 / (np.linalg.norm(W) + 1e-8))
    a = np.linalg.norm(alpha * W / 2, 2)
    assert 0.01 < a < 0.5                                 # the case exercises the iteration, inside its contraction region
    I = np.eye(16)
    Ystar = np.linalg.solve(I - alpha / 2 * W, (I + alpha / 2 * W) @ X)
    bound = a ** s * 2 * a * a / (1 - a) * np.linalg.norm(X) + 1e-6
    assert np.linalg.norm(st.Omega - Ystar) <= bound
    if s == 6:
        assert np.abs(st.Omega - Ystar).max() < 2e-7      # fp32 storage is all that is left
    # the stored momentum is the projected one, W X: tangent to the orthogonal group at X
    assert np.allclose(st.Mom, W @ X, rtol=1e-5, atol=1e-9)
    T = st.Mom.astype(np.float64) @ X.T
    assert np.abs(T + T.T).max() < 1e-6 * max(1.0, np.abs(T).max())
    # the transform of an orthogonal matrix is orthogonal
    assert np.abs(Ystar.T @ Ystar - I).max() < 1e-5
    assert np.abs(st.Omega.astype(np.float64).T @ st.Omega - I).max() < 4 * bound + 1e-5


def test_rot_step_limiter_and_descent(oracle):
    """The step length is min(lr, 2q / (||W|| + eps)): a huge gradient cannot leave the contraction region (the update
    stays near-orthogonal), and a small step goes downhill on the loss with the codes held (sign of the update)."""
    L, R, X0 = _rot_case(5)
    st = oracle.rot_init(16, X0)
    oracle.rot_step(L, R, st, bits=4, lr=0.5, beta=0.0, s=2, grad_scale=1e6)
    assert np.abs(st.Omega.astype(np.float64).T @ st.Omega - np.eye(16)).max() < 0.3   # a = q = 0.5: bounded, not exploded
    st = oracle.rot_init(16, X0)
    out = oracle.rot_step(L, R, st, bits=4, lr=1e-3, beta=0.0, s=2, grad_scale=100.0)
    L64, R64, X64 = L.astype(np.float64), R.astype(np.float64), X0.astype(np.float64)
    C1, C2 = L64 @ X64 + out.E1, X64.T @ R64 + out.E2
    f = lambda X: np.mean((C1 - L64 @ X) ** 2) + np.mean((C2 - X.T @ R64) ** 2)
    assert f(st.Omega.astype(np.float64)) < f(X64)


def test_rot_lossless_factors_are_a_fixed_point_and_apply_keeps_the_product(oracle):
    """Factors already on the integer grid of their rows (row maximum = qmax steps) have zero error at Omega = I: loss 0,
    gradient 0, Omega and the momentum stay exactly where they were.  Applying an orthogonal Omega leaves L R unchanged
    up to fp32 rounding and equals the plain matrix products."""
    rng = np.random.default_rng(6)
    r, N, K = 16, 40, 96
    L = rng.integers(-127, 128, (N, r)).astype(np.float32)
    R = rng.integers(-127, 128, (r, K)).astype(np.float32)
    L[:, 0] = 127.0
    R[:, 1] = -127.0
    L *= np.float32(2.0 ** -9)
    R *= np.float32(2.0 ** -7)
    st = oracle.rot_init(r)
    out = oracle.rot_step(L, R, st, bits=8, lr=0.5)
    assert out.loss == 0.0 and not out.G.any() and not out.E1.any() and not out.E2.any()
    assert np.array_equal(st.Omega, np.eye(r, dtype=np.float32)) and not st.Mom.any()
    L2, R2, X0 = _rot_case(7)
    Lr, Rr = oracle.rot_apply(L2, R2, X0)
    assert np.allclose(Lr, L2.astype(np.float64) @ X0, rtol=0, atol=1e-6)
    assert np.allclose(Rr, X0.T.astype(np.float64) @ R2, rtol=0, atol=1e-6)
    assert np.allclose(Lr.astype(np.float64) @ Rr, L2.astype(np.float64) @ R2, rtol=0, atol=2e-6)


@pytest.mark.parametrize("q2,bits,half_ulp", [("fp8", 8, 2.0 ** -4), ("mxfp8", 8, 2.0 ** -4), ("mxfp6", 6, 2.0 ** -4), ("mxint", 8, None),
                                              ("mxint", 4, None)])
def test_rot_errors_with_mx_branch_formats(oracle, q2, bits, half_ulp):
    """Eq. 7 with the MX branch formats as Q2 (App. A.3): every reconstructed value Z + E is a representable number of
    its block (or row) and E is no larger than half the local spacing.  Floating-point elements: relative error at most
    2^-(m+1) (m = 3 mantissa bits) above the format's smallest normal, and the largest element of a block is exact to
    that bound; MXINT: multiples of the block step 2^(floor(log2 amax) - (bits - 2)), at most half a step off, except a
    value rounding to 2^(bits-1) steps, which saturates (a full step at most)."""
    L, R, X0 = _rot_case(8, N=64, K=128, r=32)
    st = oracle.rot_init(32, X0)
    out = oracle.rot_step(L, R, st, bits=bits, lr=0.0, q2=q2)
    for Z, E in ((L.astype(np.float64) @ X0, out.E1), (X0.T.astype(np.float64) @ R, out.E2)):
        Zb, Eb = Z.reshape(Z.shape[0], -1, 32), E.astype(np.float64).reshape(Z.shape[0], -1, 32)
        amax = np.abs(Zb).max(axis=2, keepdims=True) if q2 != "fp8" else np.abs(Z).max(axis=1).reshape(-1, 1, 1)
        if q2 == "mxint":
            step = 2.0 ** (np.floor(np.log2(amax)) - (bits - 2))
            codes = (Zb + Eb) / step
            assert np.all(np.abs(codes - np.rint(codes)) < 1e-3) and np.abs(np.rint(codes)).max() <= 2 ** (bits - 1) - 1
            assert np.all(np.abs(Eb) <= step * (1 + 1e-5))
            inside = np.abs(Zb) / step <= 2 ** (bits - 1) - 1
            assert np.all(np.abs(Eb)[inside] <= (0.5 * step * np.ones_like(Eb))[inside] * (1 + 1e-5) + 1e-12)
        else:
            # elements far enough above the subnormal range of the scaled format: relative error <= 2^-4 (3 mantissa bits)
            big = np.abs(Zb) >= amax * (2.0 ** -2 if q2 == "mxfp6" else 2.0 ** -5)   # E2M3 has normals over two octaves only
            if q2 != "fp8":   # block formats: elements above the largest code of the scaled format saturate to it
                top = (448.0 if q2 == "mxfp8" else 7.5) * 2.0 ** (np.floor(np.log2(amax)) - (8 if q2 == "mxfp8" else 2))
                sat = np.abs(Zb) > top
                assert np.allclose(np.abs(Zb + Eb)[sat], (top * np.ones_like(Zb))[sat], rtol=1e-6)
                big &= ~sat
            assert np.all(np.abs(Eb)[big] <= half_ulp * np.abs(Zb)[big] * (1 + 1e-5))
            assert np.all(np.abs(Eb) <= 2 * half_ulp * amax * (1 + 1e-5))
            # the reconstructed values have at most 4 significant bits
            v = np.abs(Zb + Eb)[big]
            m, _ = np.frexp(v if q2 != "fp8" else v / (amax * np.ones_like(Zb))[big] * 448.0)
            if q2 != "fp8":
                assert np.all(np.abs(m * 16 - np.rint(m * 16)) < 1e-4)
    assert out.loss == pytest.approx(np.mean(out.E1.astype(np.float64) ** 2) + np.mean(out.E2.astype(np.float64) ** 2), rel=1e-12)
    assert out.loss > 0


# ---------------------------------------------------------------------------------------
# quantized hand-off between two linears (Section 4.5)
# ---------------------------------------------------------------------------------------
def _mxi_layer(oracle, rng, N, K, r, bw=8):
    W = (rng.standard_normal((N, K)) * 0.05).astype(np.float32)
    L = (rng.standard_normal((N, r)) * 0.02).astype(np.float32)
    R = (rng.standard_normal((r, K)) * 0.02).astype(np.float32)
    return oracle.pack_mxi(W, L, R, bw)


def test_handoff_is_the_next_activation_step_on_the_bf16_output(oracle):
    rng = np.random.default_rng(31)
    M, K1, N1, N2, r = 9, 128, 192, 64, 32
    pk1 = _mxi_layer(oracle, rng, N1, K1, r)
    pk2 = _mxi_layer(oracle, rng, N2, N1, r)
    X = rng.standard_normal((M, K1)).astype(np.float32)
    out1 = oracle.fwd_mxi(pk1, oracle.quantize_act_mxi(X, pk1))
    ho = oracle.handoff_mxi(out1.Y, pk2)
    ref = oracle.quantize_act_mxi(oracle.bf16_bits_to_f32(out1.Y), pk2)
    for f in ("xq", "xe", "xb", "xbe", "T", "tq", "te"):
        assert np.array_equal(getattr(ho, f), getattr(ref, f)), f
    # the second layer's output through the hand-off equals the two-call path bit for bit
    assert np.array_equal(oracle.fwd_mxi(pk2, ho).Y, oracle.fwd_mxi(pk2, ref).Y)
    # every hand-off scale and code belongs to 32 consecutive output channels of the producing layer: codes of one
    # block do not move when any other column of Y changes (what makes a tile-local epilogue legal) ...
    Y2 = out1.Y.copy()
    Y2[:, 32:] = Y2[:, 32:][:, ::-1]
    ho2 = oracle.handoff_mxi(Y2, pk2)
    assert np.array_equal(ho2.xq[:, :32], ho.xq[:, :32]) and np.array_equal(ho2.xe[:, 0], ho.xe[:, 0])
    assert np.array_equal(ho2.xb[:, :32], ho.xb[:, :32]) and np.array_equal(ho2.xbe[:, 0], ho.xbe[:, 0])
    # ... while the skinny contraction of the next layer runs over the whole row
    assert not np.array_equal(ho2.T, ho.T)


def test_handoff_codes_come_from_the_bf16_value_not_from_the_fp32_sum(oracle):
    """The reading pinned on a constructed row: a block whose largest value is 4 has MXINT8 step 1/16; the fp32 value
    2^-5 + 2^-14 lies above the tie between codes 0 and 1, its bf16 rounding (a tie at spacing 2^-13, to even) is
    exactly 2^-5, the tie itself, which goes to the even code 0."""
    rng = np.random.default_rng(32)
    pk2 = _mxi_layer(oracle, rng, 64, 64, 32)
    y32 = np.zeros((1, 64), np.float32)
    y32[0, 0] = 4.0
    y32[0, 1] = np.float32(2.0 ** -5 + 2.0 ** -14)
    ybits = np.array([[oracle.bf16_rne(float(v)) for v in y32[0]]], np.uint16)
    assert oracle.bf16_bits_to_f32(ybits)[0, 1] == np.float32(2.0 ** -5)
    from_bf16 = oracle.handoff_mxi(ybits, pk2)
    from_f32 = oracle.quantize_act_mxi(y32, pk2)
    assert from_bf16.xbe[0, 0] == 127 + 2 and from_bf16.xb[0, 0] == 64
    assert from_f32.xb[0, 1] == 1 and from_bf16.xb[0, 1] == 0

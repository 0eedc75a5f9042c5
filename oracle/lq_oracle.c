/*
 * lq_oracle.c -- plain CPU oracle for the LoRaQ inference forward (TEST INFRASTRUCTURE).
 *
 * This file is the slow, scalar, obviously-correct definition that the GPU library is
 * checked against.  It is NOT part of the product: only tests, the smoke check and the
 * bench's cpu_baseline leg may call it.  It shares no source, header, table or helper
 * with the HIP path.
 *
 * What it computes (paper Fig. 1 and Eq. 5; orientation X: M x K, W: N x K, L: N x r,
 * R: r x K, Y: M x N, all row-major):
 *
 *     P     = W - deq(Q2(L)) deq(Q2(R))                      residual weights (Fig. 1)
 *     Y     = deq(Q1(X) Q1(P)^T) + deq(Q2(Q2(X) Q2(R)^T) Q2(L)^T)
 *
 * Q1 is the 4-bit main format, Q2 the sub-16-bit branch format.  Two families:
 *   INT  : symmetric signed integers, round-to-nearest-even, fp32 scales
 *          (SINT4-style block scales along K for Q1(P), App. A.3; per-token / per-channel
 *          scales elsewhere); integer accumulate, fp32 dequantisation.
 *          With a_group = 64 (the literal SINT4 of App. A.3: blocks of 64 values, one FP16 scale
 *          per block) both operands of the main product are quantised in blocks of 64 along K
 *          with FP16 scales; the branch is unchanged.
 *   MX   : Q1 = MXFP4 (E2M1 elements, blocks of 32 along K, E8M0 power-of-two scale,
 *          App. A.3), Q2 = FP8 E4M3 with one fp32 scale per token / per channel;
 *          fp64 accumulate, result rounded once to fp32.
 *   MXB  : as MX, but Q2 = MXFP8e4 (App. A.3: E4M3 elements, blocks of 32 along the
 *          contraction axis, E8M0 scale) for X, R, the intermediate X R^T and L, i.e. the
 *          all-MX setting of the paper's mixed-precision tables (Section 4.3); no fp32
 *          scale anywhere; the two branches are summed in fp64 and rounded once.
 *   MXB6 : as MXB with MXFP6e2 elements (App. A.3: E2M3, 1 sign + 2 exponent + 3 mantissa bits,
 *          bias 1, largest magnitude 7.5) in place of E4M3; scale exponent floor(log2 amax) - 2.
 *   MXI  : Q1 = MXINT4 for both operands of the main product, Q2 = MXINT8 for the branch
 *          activations and the intermediate, MXINT8 or MXINT4 for L and R (App. A.3: "signed
 *          int4 and int8" elements, blocks of 32, E8M0 scale; the integer rows of the
 *          mixed-precision tables, Section 4.3); fp64 accumulate, one rounding.
 *
 * Besides the forward, lqo_calib_step is one Adam step of the data-free optimisation of the factors
 * (Eq. 4, App. B.2), the step that produces the L and R the forward consumes, and lqo_rot_step one step
 * of the rotation search of Section 3.3 (Eq. 6-7) that follows it.
 *
 * Readings of points the paper leaves open (all "parity unpinned" by the paper; the tests
 * pin self-consistency only):
 *   - "round to nearest" = ties to even;
 *   - integer codes are symmetric, [-qmax, qmax], qmax = 2^(b-1)-1;
 *   - scale s = amax / qmax, codes = rne(v * (qmax / amax)), both in fp32
 *     (reciprocal-multiply form of v / s); all-zero vector: s = 1, codes 0;
 *   - the intermediate X R^T is re-quantised per token at the branch activation width
 *     (the paper lists this as future work; the benchmark spec requires it);
 *   - MX scale exponent = floor(log2 amax) - 2 (2 = largest E2M1 exponent), elements
 *     saturate at +-6; all-zero block: E8M0 byte 0;
 *   - MXFP8e4 scale exponent = floor(log2 amax) - 8 (8 = largest E4M3 exponent), elements
 *     saturate at +-448; the rank is a multiple of 32 so that blocks along r are whole;
 *   - MXINT element of width b: integer code c in [-(2^(b-1)-1), 2^(b-1)-1] with b-2 fraction
 *     bits, value = c * 2^-(b-2) * 2^(E-127) with the shared exponent E-127 = floor(log2 amax)
 *     (the MX specification's INT8 element, 1 sign + 1 integer + 6 fraction bits and largest
 *     element exponent 0, and the same pattern at 4 bits: 1 + 1 + 2); the block maximum
 *     therefore lands in the top octave of the code range, a value that would round to
 *     2^(b-1) saturates, -2^(b-1) is never produced; all-zero block: E8M0 byte 0;
 *   - SINT4 blocks: the stored scale is s = fp16_rne(amax / 7) (kept inside the positive finite
 *     FP16 range: at least 2^-24, at most 65504; all-zero block: s = 1); codes are taken against
 *     the STORED scale, code = clamp(rne(v * fl(1 / s)), -7, 7); a block contributes
 *     fma(float(acc), sx * sw, t) to the running fp32 sum, where the product of the two FP16
 *     scales is exact in fp32, and the branch is added with one fp32 addition;
 *   - activation smoothing divides by gamma as a multiplication by fl(1/gamma);
 *   - P is built from the *dequantised* quantised factors (Fig. 1), optionally from the
 *     unquantised ones (residual_from_quantized = 0).
 *
 * Build: gcc -O2 -fno-fast-math -ffp-contract=off -fopenmp -shared -fPIC
 * OpenMP is used across token rows (or weight rows) only; no blocking, no reordering.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#define LQO_API __attribute__((visibility("default")))

/* ------------------------------------------------------------------------------------ */
/* small helpers                                                                          */
/* ------------------------------------------------------------------------------------ */

static float absmax_f32(const float *v, int64_t n)
{
    float a = 0.0f;
    for (int64_t i = 0; i < n; ++i) {
        float t = fabsf(v[i]);
        if (t > a) a = t;
    }
    return a;
}

/* fp32 -> bf16 bits, round-to-nearest-even (finite inputs). */
static uint16_t bf16_rne(float f)
{
    uint32_t u;
    memcpy(&u, &f, 4);
    uint32_t lsb = (u >> 16) & 1u;
    u += 0x7FFFu + lsb;
    return (uint16_t)(u >> 16);
}

LQO_API uint16_t lqo_bf16_rne(float f) { return bf16_rne(f); }

/* ------------------------------------------------------------------------------------ */
/* symmetric integer quantiser (SINT4-style; App. A.3 "round-to-nearest" on scaled values) */
/* ------------------------------------------------------------------------------------ */

/* One vector of n values sharing one scale.  q in [-qmax, qmax]. */
LQO_API void lqo_quant_int(const float *v, int64_t n, int qmax, int8_t *q, float *scale)
{
    float a = absmax_f32(v, n);
    float s, inv;
    if (a == 0.0f) {
        s = 1.0f;
        inv = 1.0f;
    } else {
        s = a / (float)qmax;
        inv = (float)qmax / a;
    }
    for (int64_t i = 0; i < n; ++i) {
        float u = v[i] * inv;
        float r = nearbyintf(u); /* default rounding mode: ties to even */
        if (r > (float)qmax) r = (float)qmax;
        if (r < -(float)qmax) r = -(float)qmax;
        q[i] = (int8_t)r;
    }
    *scale = s;
}

/* fp32 -> nearest value with FP16's precision (11 significant bits, subnormal spacing 2^-24; ties to
   even), returned as fp32.  Finite inputs.  The exponent range is not limited at the top: magnitudes
   of 65520 and more come back as 65536 or larger and the caller clamps to 65504. */
static float f16_round(float f)
{
    float a = fabsf(f);
    float r;
    if (a == 0.0f) return f;
    if (a < 6.103515625e-05f) { /* below 2^-14: FP16 subnormals, spacing 2^-24 */
        r = ldexpf(nearbyintf(ldexpf(a, 24)), -24);
    } else {
        int e;
        (void)frexpf(a, &e);  /* a = m * 2^e, m in [0.5, 1)  ->  a in [2^(e-1), 2^e) */
        /* 11 significant bits: spacing 2^(e-1-10) */
        r = ldexpf(nearbyintf(ldexpf(a, 11 - e)), e - 11);
    }
    return f < 0.0f ? -r : r;
}

LQO_API float lqo_f16_round(float f) { return f16_round(f); }

/* SINT4 block quantiser (App. A.3): n values (n a multiple of 64) in blocks of 64, one FP16 scale
   per block (returned as fp32), round-to-nearest on the scaled values. */
LQO_API void lqo_quant_sint4(const float *v, int64_t n, int8_t *q, float *scales)
{
    for (int64_t b = 0; b < n / 64; ++b) {
        const float *blk = v + 64 * b;
        float a = absmax_f32(blk, 64);
        float s;
        if (a == 0.0f) {
            s = 1.0f;
        } else {
            s = f16_round(a / 7.0f);
            if (s < 5.9604644775390625e-08f) s = 5.9604644775390625e-08f; /* 2^-24 */
            if (s > 65504.0f) s = 65504.0f;
        }
        float inv = 1.0f / s;
        for (int i = 0; i < 64; ++i) {
            float r = nearbyintf(blk[i] * inv);
            if (r > 7.0f) r = 7.0f;
            if (r < -7.0f) r = -7.0f;
            q[64 * b + i] = (int8_t)r;
        }
        scales[b] = s;
    }
}

/* Activation smoothing (Section 3.4; App. A.1): channel k of X is divided by gamma[k] before
   quantisation, for both branches.  Reading: the division is a multiplication by the correctly
   rounded reciprocal, Xs = X * fl(1 / gamma), both in fp32 (the reciprocal-multiply form used for
   every scale of this oracle). */
LQO_API void lqo_smooth(int64_t M, int64_t K, const float *X, const float *gamma, float *Xs)
{
    for (int64_t m = 0; m < M; ++m)
        for (int64_t k = 0; k < K; ++k) {
            float rg = 1.0f / gamma[k];
            Xs[m * K + k] = X[m * K + k] * rg;
        }
}

/* ------------------------------------------------------------------------------------ */
/* element formats of the MX family (App. A.3)                                            */
/* ------------------------------------------------------------------------------------ */

/* E2M1: 1 sign, 2 exponent (bias 1), 1 mantissa bit.  code = s e e m (4 bits). */
LQO_API float lqo_e2m1_decode(uint8_t code)
{
    int s = (code >> 3) & 1, e = (code >> 1) & 3, m = code & 1;
    float mag;
    if (e == 0)
        mag = 0.5f * (float)m; /* subnormal: m * 2^(1-1) * 2^-1 */
    else
        mag = ldexpf(1.0f + 0.5f * (float)m, e - 1);
    return s ? -mag : mag;
}

/* E4M3 (OCP "FN" flavour): 1 sign, 4 exponent (bias 7), 3 mantissa; no Inf; S.1111.111 = NaN;
   largest finite 448. */
LQO_API float lqo_e4m3_decode(uint8_t code)
{
    int s = (code >> 7) & 1, e = (code >> 3) & 15, m = code & 7;
    float mag;
    if (e == 15 && m == 7) return NAN;
    if (e == 0)
        mag = ldexpf((float)m, -9); /* m/8 * 2^-6 */
    else
        mag = ldexpf(1.0f + (float)m / 8.0f, e - 7);
    return s ? -mag : mag;
}

/* E8M0: value 2^(E-127); byte 0xFF is NaN and is never produced here. */
LQO_API double lqo_e8m0_decode(uint8_t e) { return ldexp(1.0, (int)e - 127); }

/* Nearest representable magnitude among codes 0..ncodes-1 of a monotone decode table,
   ties to the even code (= even mantissa), saturating at the top code. */
static int nearest_code(float mag, const float *table, int ncodes)
{
    if (mag >= table[ncodes - 1]) return ncodes - 1;
    int lo = 0;
    while (lo + 1 < ncodes && table[lo + 1] <= mag) ++lo; /* table[lo] <= mag < table[lo+1] */
    double dl = (double)mag - (double)table[lo];
    double dh = (double)table[lo + 1] - (double)mag;
    if (dl < dh) return lo;
    if (dh < dl) return lo + 1;
    return (lo & 1) ? lo + 1 : lo;
}

LQO_API uint8_t lqo_e2m1_encode(float u)
{
    float table[8];
    for (int c = 0; c < 8; ++c) table[c] = lqo_e2m1_decode((uint8_t)c);
    int s = signbit(u) ? 1 : 0;
    int c = nearest_code(fabsf(u), table, 8);
    return (uint8_t)((s << 3) | c);
}

LQO_API uint8_t lqo_e4m3_encode(float u)
{
    float table[127];
    for (int c = 0; c < 127; ++c) table[c] = lqo_e4m3_decode((uint8_t)c);
    int s = signbit(u) ? 1 : 0;
    int c = nearest_code(fabsf(u), table, 127);
    return (uint8_t)((s << 7) | c);
}

/* MXFP4: K values in blocks of 32; one E8M0 byte per block; one E2M1 code per byte of `codes`. */
LQO_API void lqo_quant_mxfp4(const float *v, int64_t K, uint8_t *codes, uint8_t *e8m0)
{
    for (int64_t b = 0; b < K / 32; ++b) {
        const float *blk = v + 32 * b;
        float a = absmax_f32(blk, 32);
        int e;
        if (a == 0.0f) {
            e = -127;
        } else {
            int ex;
            (void)frexpf(a, &ex); /* a = f * 2^ex, f in [0.5,1) => floor(log2 a) = ex-1 */
            e = (ex - 1) - 2;
            if (e < -127) e = -127;
            if (e > 127) e = 127;
        }
        e8m0[b] = (uint8_t)(e + 127);
        for (int i = 0; i < 32; ++i) {
            float u = ldexpf(blk[i], -e); /* exact power-of-two scaling */
            codes[32 * b + i] = lqo_e2m1_encode(u);
        }
    }
}

/* FP8 E4M3 with one fp32 scale for the whole vector: s = amax/448. */
LQO_API void lqo_quant_fp8(const float *v, int64_t n, uint8_t *codes, float *scale)
{
    float a = absmax_f32(v, n);
    float s, inv;
    if (a == 0.0f) {
        s = 1.0f;
        inv = 1.0f;
    } else {
        s = a / 448.0f;
        inv = 448.0f / a;
    }
    for (int64_t i = 0; i < n; ++i) codes[i] = lqo_e4m3_encode(v[i] * inv);
    *scale = s;
}

/* ------------------------------------------------------------------------------------ */
/* INT family                                                                             */
/* ------------------------------------------------------------------------------------ */

/* Offline packing step (Fig. 1; Eq. 5): quantise the factors with Q2, form the residual P,
   quantise P with Q1 in groups of g along K.
   qmax_bw : qmax of the branch weight format (127 / 31 / 7).
   sint4_blocks != 0 (then g == 64): Q1 is the literal SINT4 block format with FP16 scales.
   Outputs: pq N x K, sw N x (K/g), lq N x r, sl N, rq r x K, sr r, P (optional, N x K). */
LQO_API void lqo_pack_int(int64_t N, int64_t K, int r, int g, int qmax_bw,
                          int residual_from_quantized, const float *W, const float *L,
                          const float *R, int8_t *pq, float *sw, int8_t *lq, float *sl,
                          int8_t *rq, float *sr, float *P_out, int sint4_blocks)
{
    const int64_t G = K / g;
    for (int j = 0; j < r; ++j) lqo_quant_int(R + (int64_t)j * K, K, qmax_bw, rq + (int64_t)j * K, &sr[j]);
    for (int64_t n = 0; n < N; ++n) lqo_quant_int(L + n * r, r, qmax_bw, lq + n * r, &sl[n]);

#pragma omp parallel for schedule(static)
    for (int64_t n = 0; n < N; ++n) {
        float *P = (float *)malloc(sizeof(float) * (size_t)K);
        for (int64_t k = 0; k < K; ++k) {
            double d = 0.0;
            for (int j = 0; j < r; ++j) {
                float lh, rh;
                if (residual_from_quantized) {
                    lh = (float)lq[n * r + j] * sl[n];
                    rh = (float)rq[(int64_t)j * K + k] * sr[j];
                } else {
                    lh = L[n * r + j];
                    rh = R[(int64_t)j * K + k];
                }
                d += (double)lh * (double)rh;
            }
            P[k] = (float)((double)W[n * K + k] - d);
        }
        if (sint4_blocks)
            lqo_quant_sint4(P, K, pq + n * K, sw + n * G);
        else
            for (int64_t gi = 0; gi < G; ++gi)
                lqo_quant_int(P + gi * g, g, 7, pq + n * K + gi * g, &sw[n * G + gi]);
        if (P_out) memcpy(P_out + n * K, P, sizeof(float) * (size_t)K);
        free(P);
    }
}

/* Per-call activation step: 4-bit codes for the main product, b-bit codes for the branch,
   the skinny contraction with Q2(R) and the re-quantisation of its result.
   qmax_a : qmax of the branch activation format (127 / 31).
   a_group: 0 = one main scale per token (sx M); 64 = SINT4 blocks along K (sx M x K/64).
   Outputs: xq M x K, sx, xb M x K, sxb M, accT M x r (int32), T M x r, tq M x r, st M.
   Any of xb / accT / T may be NULL. */
LQO_API void lqo_quantize_act_int(int64_t M, int64_t K, int r, int qmax_a, const float *X,
                                  const int8_t *rq, const float *sr, int8_t *xq, float *sx,
                                  int8_t *xb, float *sxb, int32_t *accT, float *T,
                                  int8_t *tq, float *st, int a_group)
{
#pragma omp parallel for schedule(static)
    for (int64_t m = 0; m < M; ++m) {
        const float *x = X + m * K;
        if (a_group)
            lqo_quant_sint4(x, K, xq + m * K, sx + m * (K / 64));
        else
            lqo_quant_int(x, K, 7, xq + m * K, &sx[m]);
        if (r == 0) continue;
        int8_t *xbrow = (int8_t *)malloc((size_t)K);
        float *Trow = (float *)malloc(sizeof(float) * (size_t)r);
        float s_b;
        lqo_quant_int(x, K, qmax_a, xbrow, &s_b);
        sxb[m] = s_b;
        for (int j = 0; j < r; ++j) {
            int32_t a = 0;
            for (int64_t k = 0; k < K; ++k) a += (int32_t)xbrow[k] * (int32_t)rq[(int64_t)j * K + k];
            if (accT) accT[m * r + j] = a;
            Trow[j] = ((float)a * s_b) * sr[j];
        }
        lqo_quant_int(Trow, r, qmax_a, tq + m * r, &st[m]);
        if (xb) memcpy(xb + m * K, xbrow, (size_t)K);
        if (T) memcpy(T + m * r, Trow, sizeof(float) * (size_t)r);
        free(xbrow);
        free(Trow);
    }
}

/* Forward: main 4-bit product with per-group fp32 dequantisation, rank-r expansion, sum.
   a_group = 64 (then g == 64): sx is M x G, and a block's accumulator is scaled by the product of
   the two block scales (exact in fp32 for FP16 scales).
   Outputs: acc M x N x G int32 (optional), acc2 M x N int32 (optional), ymain, ybr, y32
   (fp32, M x N, each optional) and Y (bf16 bits, M x N). */
LQO_API void lqo_fwd_int(int64_t M, int64_t N, int64_t K, int r, int g, const int8_t *xq,
                         const float *sx, const int8_t *pq, const float *sw, const int8_t *tq,
                         const float *st, const int8_t *lq, const float *sl, int32_t *acc,
                         int32_t *acc2, float *ymain, float *ybr, float *y32, uint16_t *Y, int a_group)
{
    const int64_t G = K / g;
#pragma omp parallel for schedule(static)
    for (int64_t m = 0; m < M; ++m) {
        for (int64_t n = 0; n < N; ++n) {
            float t = 0.0f;
            for (int64_t gi = 0; gi < G; ++gi) {
                int32_t a = 0;
                for (int k = 0; k < g; ++k)
                    a += (int32_t)xq[m * K + gi * g + k] * (int32_t)pq[n * K + gi * g + k];
                if (acc) acc[(m * N + n) * G + gi] = a;
                if (a_group)
                    t = fmaf((float)a, sx[m * G + gi] * sw[n * G + gi], t);
                else
                    t = fmaf((float)a, sw[n * G + gi], t);
            }
            float ym = a_group ? t : sx[m] * t;
            float yb = 0.0f;
            if (r > 0) {
                int32_t a2 = 0;
                for (int j = 0; j < r; ++j) a2 += (int32_t)tq[m * r + j] * (int32_t)lq[n * r + j];
                if (acc2) acc2[m * N + n] = a2;
                yb = ((float)a2 * st[m]) * sl[n];
            } else if (acc2) {
                acc2[m * N + n] = 0;
            }
            /* sum node of Fig. 1: one rounding for scale-and-add (per-token scale) or for the add */
            float y = a_group ? t + yb : fmaf(sx[m], t, yb);
            if (ymain) ymain[m * N + n] = ym;
            if (ybr) ybr[m * N + n] = yb;
            if (y32) y32[m * N + n] = y;
            if (Y) Y[m * N + n] = bf16_rne(y);
        }
    }
}

/* ------------------------------------------------------------------------------------ */
/* MX family                                                                              */
/* ------------------------------------------------------------------------------------ */

/* Outputs: pc N x K E2M1 codes (one per byte), pe N x K/32 E8M0, l8 N x r E4M3, sl N,
   r8 r x K E4M3, sr r, P (optional). */
LQO_API void lqo_pack_mx(int64_t N, int64_t K, int r, int residual_from_quantized,
                         const float *W, const float *L, const float *R, uint8_t *pc,
                         uint8_t *pe, uint8_t *l8, float *sl, uint8_t *r8, float *sr,
                         float *P_out)
{
    for (int j = 0; j < r; ++j) lqo_quant_fp8(R + (int64_t)j * K, K, r8 + (int64_t)j * K, &sr[j]);
    for (int64_t n = 0; n < N; ++n) lqo_quant_fp8(L + n * r, r, l8 + n * r, &sl[n]);

#pragma omp parallel for schedule(static)
    for (int64_t n = 0; n < N; ++n) {
        float *P = (float *)malloc(sizeof(float) * (size_t)K);
        for (int64_t k = 0; k < K; ++k) {
            double d = 0.0;
            for (int j = 0; j < r; ++j) {
                float lh, rh;
                if (residual_from_quantized) {
                    lh = lqo_e4m3_decode(l8[n * r + j]) * sl[n];
                    rh = lqo_e4m3_decode(r8[(int64_t)j * K + k]) * sr[j];
                } else {
                    lh = L[n * r + j];
                    rh = R[(int64_t)j * K + k];
                }
                d += (double)lh * (double)rh;
            }
            P[k] = (float)((double)W[n * K + k] - d);
        }
        lqo_quant_mxfp4(P, K, pc + n * K, pe + n * (K / 32));
        if (P_out) memcpy(P_out + n * K, P, sizeof(float) * (size_t)K);
        free(P);
    }
}

/* Outputs: xc M x K E2M1 codes, xe M x K/32 E8M0, xb8 M x K E4M3 (optional), sxb M,
   T M x r fp32 (optional), tq8 M x r E4M3, st M. */
LQO_API void lqo_quantize_act_mx(int64_t M, int64_t K, int r, const float *X,
                                 const uint8_t *r8, const float *sr, uint8_t *xc, uint8_t *xe,
                                 uint8_t *xb8, float *sxb, float *T, uint8_t *tq8, float *st)
{
#pragma omp parallel for schedule(static)
    for (int64_t m = 0; m < M; ++m) {
        const float *x = X + m * K;
        lqo_quant_mxfp4(x, K, xc + m * K, xe + m * (K / 32));
        if (r == 0) continue;
        uint8_t *xbrow = (uint8_t *)malloc((size_t)K);
        float *Trow = (float *)malloc(sizeof(float) * (size_t)r);
        float s_b;
        lqo_quant_fp8(x, K, xbrow, &s_b);
        sxb[m] = s_b;
        for (int j = 0; j < r; ++j) {
            double a = 0.0;
            for (int64_t k = 0; k < K; ++k)
                a += (double)lqo_e4m3_decode(xbrow[k]) * (double)lqo_e4m3_decode(r8[(int64_t)j * K + k]);
            Trow[j] = (float)(((double)s_b * (double)sr[j]) * a);
        }
        lqo_quant_fp8(Trow, r, tq8 + m * r, &st[m]);
        if (xb8) memcpy(xb8 + m * K, xbrow, (size_t)K);
        if (T) memcpy(T + m * r, Trow, sizeof(float) * (size_t)r);
        free(xbrow);
        free(Trow);
    }
}

LQO_API void lqo_fwd_mx(int64_t M, int64_t N, int64_t K, int r, const uint8_t *xc,
                        const uint8_t *xe, const uint8_t *pc, const uint8_t *pe,
                        const uint8_t *tq8, const float *st, const uint8_t *l8, const float *sl,
                        float *ymain, float *ybr, float *y32, uint16_t *Y)
{
    const int64_t B = K / 32;
    /* element values decoded once up front (decode only; no arithmetic is moved) */
    float *vw = (float *)malloc(sizeof(float) * (size_t)(N * K));
    for (int64_t i = 0; i < N * K; ++i) vw[i] = lqo_e2m1_decode(pc[i]);
    float *vl = (float *)malloc(sizeof(float) * (size_t)(N * (r > 0 ? r : 1)));
    for (int64_t i = 0; i < N * r; ++i) vl[i] = lqo_e4m3_decode(l8[i]);
#pragma omp parallel for schedule(static)
    for (int64_t m = 0; m < M; ++m) {
        float *vx = (float *)malloc(sizeof(float) * (size_t)K);
        for (int64_t k = 0; k < K; ++k) vx[k] = lqo_e2m1_decode(xc[m * K + k]);
        for (int64_t n = 0; n < N; ++n) {
            double t = 0.0;
            for (int64_t b = 0; b < B; ++b) {
                double d = 0.0;
                for (int k = 0; k < 32; ++k)
                    d += (double)vx[32 * b + k] * (double)vw[n * K + 32 * b + k];
                t += lqo_e8m0_decode(xe[m * B + b]) * lqo_e8m0_decode(pe[n * B + b]) * d;
            }
            float ym = (float)t;
            float yb = 0.0f;
            if (r > 0) {
                double a = 0.0;
                for (int j = 0; j < r; ++j)
                    a += (double)lqo_e4m3_decode(tq8[m * r + j]) * (double)vl[n * r + j];
                yb = (float)(((double)st[m] * (double)sl[n]) * a);
            }
            float y = ym + yb;
            if (ymain) ymain[m * N + n] = ym;
            if (ybr) ybr[m * N + n] = yb;
            if (y32) y32[m * N + n] = y;
            if (Y) Y[m * N + n] = bf16_rne(y);
        }
        free(vx);
    }
    free(vw);
    free(vl);
}

/* ------------------------------------------------------------------------------------ */
/* MXB family: block-scaled FP8 branch                                                    */
/* ------------------------------------------------------------------------------------ */

/* MXFP8e4: n values (n a multiple of 32) in blocks of 32; one E8M0 byte per block; E4M3 codes. */
LQO_API void lqo_quant_mxfp8(const float *v, int64_t n, uint8_t *codes, uint8_t *e8m0)
{
    for (int64_t b = 0; b < n / 32; ++b) {
        const float *blk = v + 32 * b;
        float a = absmax_f32(blk, 32);
        int e;
        if (a == 0.0f) {
            e = -127;
        } else {
            int ex;
            (void)frexpf(a, &ex); /* floor(log2 a) = ex - 1 */
            e = (ex - 1) - 8;
            if (e < -127) e = -127;
            if (e > 127) e = 127;
        }
        e8m0[b] = (uint8_t)(e + 127);
        for (int i = 0; i < 32; ++i) codes[32 * b + i] = lqo_e4m3_encode(ldexpf(blk[i], -e));
    }
}

/* value of an MXFP8e4 element */
static double mxfp8_value(uint8_t code, uint8_t e8m0)
{
    return (double)lqo_e4m3_decode(code) * lqo_e8m0_decode(e8m0);
}

/* Outputs: pc N x K E2M1, pe N x K/32; l8 N x r E4M3, le N x r/32 (blocks along r);
   r8 r x K E4M3, re r x K/32 (blocks along K); P (optional). */
LQO_API void lqo_pack_mxb(int64_t N, int64_t K, int r, int residual_from_quantized,
                          const float *W, const float *L, const float *R, uint8_t *pc,
                          uint8_t *pe, uint8_t *l8, uint8_t *le, uint8_t *r8, uint8_t *re,
                          float *P_out)
{
    const int64_t BK = K / 32;
    const int BR = r / 32;
    for (int j = 0; j < r; ++j) lqo_quant_mxfp8(R + (int64_t)j * K, K, r8 + (int64_t)j * K, re + (int64_t)j * BK);
    for (int64_t n = 0; n < N; ++n) lqo_quant_mxfp8(L + n * r, r, l8 + n * r, le + n * BR);

#pragma omp parallel for schedule(static)
    for (int64_t n = 0; n < N; ++n) {
        float *P = (float *)malloc(sizeof(float) * (size_t)K);
        for (int64_t k = 0; k < K; ++k) {
            double d = 0.0;
            for (int j = 0; j < r; ++j) {
                double lh, rh;
                if (residual_from_quantized) {
                    lh = mxfp8_value(l8[n * r + j], le[n * BR + j / 32]);
                    rh = mxfp8_value(r8[(int64_t)j * K + k], re[(int64_t)j * BK + k / 32]);
                } else {
                    lh = L[n * r + j];
                    rh = R[(int64_t)j * K + k];
                }
                d += lh * rh;
            }
            P[k] = (float)((double)W[n * K + k] - d);
        }
        lqo_quant_mxfp4(P, K, pc + n * K, pe + n * BK);
        if (P_out) memcpy(P_out + n * K, P, sizeof(float) * (size_t)K);
        free(P);
    }
}

/* Outputs: xc M x K E2M1, xe M x K/32; xb8 M x K E4M3, xbe M x K/32; T M x r fp32 (the fp64
   contraction rounded once); tq8 M x r E4M3, te M x r/32. */
LQO_API void lqo_quantize_act_mxb(int64_t M, int64_t K, int r, const float *X, const uint8_t *r8,
                                  const uint8_t *re, uint8_t *xc, uint8_t *xe, uint8_t *xb8,
                                  uint8_t *xbe, float *T, uint8_t *tq8, uint8_t *te)
{
    const int64_t BK = K / 32;
    const int BR = r / 32;
#pragma omp parallel for schedule(static)
    for (int64_t m = 0; m < M; ++m) {
        const float *x = X + m * K;
        lqo_quant_mxfp4(x, K, xc + m * K, xe + m * BK);
        if (r == 0) continue;
        lqo_quant_mxfp8(x, K, xb8 + m * K, xbe + m * BK);
        float *Trow = (float *)malloc(sizeof(float) * (size_t)r);
        for (int j = 0; j < r; ++j) {
            double a = 0.0;
            for (int64_t b = 0; b < BK; ++b) {
                double d = 0.0;
                for (int k = 0; k < 32; ++k)
                    d += (double)lqo_e4m3_decode(xb8[m * K + 32 * b + k]) *
                         (double)lqo_e4m3_decode(r8[(int64_t)j * K + 32 * b + k]);
                a += lqo_e8m0_decode(xbe[m * BK + b]) * lqo_e8m0_decode(re[(int64_t)j * BK + b]) * d;
            }
            Trow[j] = (float)a;
        }
        lqo_quant_mxfp8(Trow, r, tq8 + m * r, te + m * BR);
        if (T) memcpy(T + m * r, Trow, sizeof(float) * (size_t)r);
        free(Trow);
    }
}

LQO_API void lqo_fwd_mxb(int64_t M, int64_t N, int64_t K, int r, const uint8_t *xc,
                         const uint8_t *xe, const uint8_t *pc, const uint8_t *pe,
                         const uint8_t *tq8, const uint8_t *te, const uint8_t *l8,
                         const uint8_t *le, float *ymain, float *ybr, float *y32, uint16_t *Y)
{
    const int64_t B = K / 32;
    const int BR = r / 32;
    float *vw = (float *)malloc(sizeof(float) * (size_t)(N * K));
    for (int64_t i = 0; i < N * K; ++i) vw[i] = lqo_e2m1_decode(pc[i]);
#pragma omp parallel for schedule(static)
    for (int64_t m = 0; m < M; ++m) {
        float *vx = (float *)malloc(sizeof(float) * (size_t)K);
        for (int64_t k = 0; k < K; ++k) vx[k] = lqo_e2m1_decode(xc[m * K + k]);
        for (int64_t n = 0; n < N; ++n) {
            double t = 0.0;
            for (int64_t b = 0; b < B; ++b) {
                double d = 0.0;
                for (int k = 0; k < 32; ++k)
                    d += (double)vx[32 * b + k] * (double)vw[n * K + 32 * b + k];
                t += lqo_e8m0_decode(xe[m * B + b]) * lqo_e8m0_decode(pe[n * B + b]) * d;
            }
            double u = 0.0;
            for (int b = 0; b < BR; ++b) {
                double d = 0.0;
                for (int j = 0; j < 32; ++j)
                    d += (double)lqo_e4m3_decode(tq8[m * r + 32 * b + j]) *
                         (double)lqo_e4m3_decode(l8[n * r + 32 * b + j]);
                u += lqo_e8m0_decode(te[m * BR + b]) * lqo_e8m0_decode(le[n * BR + b]) * d;
            }
            float y = (float)(t + u); /* sum node of Fig. 1: both accumulators, one rounding */
            if (ymain) ymain[m * N + n] = (float)t;
            if (ybr) ybr[m * N + n] = (float)u;
            if (y32) y32[m * N + n] = y;
            if (Y) Y[m * N + n] = bf16_rne(y);
        }
        free(vx);
    }
    free(vw);
}

/* ------------------------------------------------------------------------------------ */
/* MXI family: MXINT4 main product, MXINT8 / MXINT4 branch                                */
/* ------------------------------------------------------------------------------------ */

/* MXINT of width `bits` (8 or 4): n values (a multiple of 32) in blocks of 32; one E8M0 byte
   per block holding the shared exponent floor(log2 amax) + 127; one integer code per value,
   value = code * 2^-(bits-2) * 2^(byte-127). */
LQO_API void lqo_quant_mxint(const float *v, int64_t n, int bits, int8_t *codes, uint8_t *e8m0)
{
    const int qmax = (1 << (bits - 1)) - 1;
    const int frac = bits - 2;
    for (int64_t b = 0; b < n / 32; ++b) {
        const float *blk = v + 32 * b;
        float a = absmax_f32(blk, 32);
        int s;
        if (a == 0.0f) {
            s = -127;
        } else {
            int ex;
            (void)frexpf(a, &ex); /* floor(log2 a) = ex - 1 */
            s = ex - 1;
            if (s < -127) s = -127;
            if (s > 127) s = 127;
        }
        e8m0[b] = (uint8_t)(s + 127);
        for (int i = 0; i < 32; ++i) {
            float u = ldexpf(blk[i], frac - s); /* exact power-of-two scaling into code units */
            float q = nearbyintf(u);            /* ties to even */
            if (q > (float)qmax) q = (float)qmax;
            if (q < -(float)qmax) q = -(float)qmax;
            codes[32 * b + i] = (int8_t)q;
        }
    }
}

/* value of an MXINT element */
static double mxint_value(int8_t code, uint8_t e8m0, int bits)
{
    return ldexp((double)code, (int)e8m0 - 127 - (bits - 2));
}

/* bw_bits: width of the branch weight format (8 or 4).
   Outputs: pq N x K int4 codes (one per byte), pe N x K/32; lq N x r, le N x r/32 (blocks
   along r); rq r x K, re r x K/32 (blocks along K); P (optional). */
LQO_API void lqo_pack_mxi(int64_t N, int64_t K, int r, int bw_bits, int residual_from_quantized,
                          const float *W, const float *L, const float *R, int8_t *pq,
                          uint8_t *pe, int8_t *lq, uint8_t *le, int8_t *rq, uint8_t *re,
                          float *P_out)
{
    const int64_t BK = K / 32;
    const int BR = r / 32;
    for (int j = 0; j < r; ++j) lqo_quant_mxint(R + (int64_t)j * K, K, bw_bits, rq + (int64_t)j * K, re + (int64_t)j * BK);
    for (int64_t n = 0; n < N; ++n) lqo_quant_mxint(L + n * r, r, bw_bits, lq + n * r, le + n * BR);

#pragma omp parallel for schedule(static)
    for (int64_t n = 0; n < N; ++n) {
        float *P = (float *)malloc(sizeof(float) * (size_t)K);
        for (int64_t k = 0; k < K; ++k) {
            double d = 0.0;
            for (int j = 0; j < r; ++j) {
                double lh, rh;
                if (residual_from_quantized) {
                    lh = mxint_value(lq[n * r + j], le[n * BR + j / 32], bw_bits);
                    rh = mxint_value(rq[(int64_t)j * K + k], re[(int64_t)j * BK + k / 32], bw_bits);
                } else {
                    lh = L[n * r + j];
                    rh = R[(int64_t)j * K + k];
                }
                d += lh * rh;
            }
            P[k] = (float)((double)W[n * K + k] - d);
        }
        lqo_quant_mxint(P, K, 4, pq + n * K, pe + n * BK);
        if (P_out) memcpy(P_out + n * K, P, sizeof(float) * (size_t)K);
        free(P);
    }
}

/* Outputs: xq M x K int4 codes, xe M x K/32; xb M x K int8 codes, xbe M x K/32; T M x r fp32
   (the fp64 contraction rounded once); tq M x r int8 codes, te M x r/32. */
LQO_API void lqo_quantize_act_mxi(int64_t M, int64_t K, int r, int bw_bits, const float *X,
                                  const int8_t *rq, const uint8_t *re, int8_t *xq, uint8_t *xe,
                                  int8_t *xb, uint8_t *xbe, float *T, int8_t *tq, uint8_t *te)
{
    const int64_t BK = K / 32;
    const int BR = r / 32;
#pragma omp parallel for schedule(static)
    for (int64_t m = 0; m < M; ++m) {
        const float *x = X + m * K;
        lqo_quant_mxint(x, K, 4, xq + m * K, xe + m * BK);
        if (r == 0) continue;
        lqo_quant_mxint(x, K, 8, xb + m * K, xbe + m * BK);
        float *Trow = (float *)malloc(sizeof(float) * (size_t)r);
        for (int j = 0; j < r; ++j) {
            double a = 0.0;
            for (int64_t b = 0; b < BK; ++b) {
                int32_t d = 0;
                for (int k = 0; k < 32; ++k)
                    d += (int32_t)xb[m * K + 32 * b + k] * (int32_t)rq[(int64_t)j * K + 32 * b + k];
                a += ldexp((double)d, ((int)xbe[m * BK + b] - 127 - 6) + ((int)re[(int64_t)j * BK + b] - 127 - (bw_bits - 2)));
            }
            Trow[j] = (float)a;
        }
        lqo_quant_mxint(Trow, r, 8, tq + m * r, te + m * BR);
        if (T) memcpy(T + m * r, Trow, sizeof(float) * (size_t)r);
        free(Trow);
    }
}

LQO_API void lqo_fwd_mxi(int64_t M, int64_t N, int64_t K, int r, int bw_bits, const int8_t *xq,
                         const uint8_t *xe, const int8_t *pq, const uint8_t *pe, const int8_t *tq,
                         const uint8_t *te, const int8_t *lq, const uint8_t *le, float *ymain,
                         float *ybr, float *y32, uint16_t *Y)
{
    const int64_t B = K / 32;
    const int BR = r / 32;
#pragma omp parallel for schedule(static)
    for (int64_t m = 0; m < M; ++m) {
        for (int64_t n = 0; n < N; ++n) {
            double t = 0.0;
            for (int64_t b = 0; b < B; ++b) {
                int32_t d = 0;
                for (int k = 0; k < 32; ++k)
                    d += (int32_t)xq[m * K + 32 * b + k] * (int32_t)pq[n * K + 32 * b + k];
                t += ldexp((double)d, ((int)xe[m * B + b] - 127 - 2) + ((int)pe[n * B + b] - 127 - 2));
            }
            double u = 0.0;
            for (int b = 0; b < BR; ++b) {
                int32_t d = 0;
                for (int j = 0; j < 32; ++j)
                    d += (int32_t)tq[m * r + 32 * b + j] * (int32_t)lq[n * r + 32 * b + j];
                u += ldexp((double)d, ((int)te[m * BR + b] - 127 - 6) + ((int)le[n * BR + b] - 127 - (bw_bits - 2)));
            }
            float y = (float)(t + u); /* sum node of Fig. 1: both accumulators, one rounding */
            if (ymain) ymain[m * N + n] = (float)t;
            if (ybr) ybr[m * N + n] = (float)u;
            if (y32) y32[m * N + n] = y;
            if (Y) Y[m * N + n] = bf16_rne(y);
        }
    }
}

/* ------------------------------------------------------------------------------------ */
/* MXB6 family: block-scaled FP6 (E2M3) branch                                            */
/* ------------------------------------------------------------------------------------ */

/* E2M3: 1 sign, 2 exponent (bias 1), 3 mantissa bits; no Inf / NaN; largest magnitude 7.5.
   code = s ee mmm (6 bits). */
LQO_API float lqo_e2m3_decode(uint8_t code)
{
    int s = (code >> 5) & 1, e = (code >> 3) & 3, m = code & 7;
    float mag;
    if (e == 0)
        mag = (float)m / 8.0f; /* subnormal: m/8 * 2^(1-1) */
    else
        mag = ldexpf(1.0f + (float)m / 8.0f, e - 1);
    return s ? -mag : mag;
}

LQO_API uint8_t lqo_e2m3_encode(float u)
{
    float table[32];
    for (int c = 0; c < 32; ++c) table[c] = lqo_e2m3_decode((uint8_t)c);
    int s = signbit(u) ? 1 : 0;
    int c = nearest_code(fabsf(u), table, 32);
    return (uint8_t)((s << 5) | c);
}

/* MXFP6e2: n values (a multiple of 32) in blocks of 32; one E8M0 byte per block; E2M3 codes. */
LQO_API void lqo_quant_mxfp6(const float *v, int64_t n, uint8_t *codes, uint8_t *e8m0)
{
    for (int64_t b = 0; b < n / 32; ++b) {
        const float *blk = v + 32 * b;
        float a = absmax_f32(blk, 32);
        int e;
        if (a == 0.0f) {
            e = -127;
        } else {
            int ex;
            (void)frexpf(a, &ex); /* floor(log2 a) = ex - 1 */
            e = (ex - 1) - 2;     /* 2 = largest E2M3 exponent */
            if (e < -127) e = -127;
            if (e > 127) e = 127;
        }
        e8m0[b] = (uint8_t)(e + 127);
        for (int i = 0; i < 32; ++i) codes[32 * b + i] = lqo_e2m3_encode(ldexpf(blk[i], -e));
    }
}

static double mxfp6_value(uint8_t code, uint8_t e8m0)
{
    return (double)lqo_e2m3_decode(code) * lqo_e8m0_decode(e8m0);
}

/* Outputs as lqo_pack_mxb, with E2M3 codes (one per byte) for the factors. */
LQO_API void lqo_pack_mxb6(int64_t N, int64_t K, int r, int residual_from_quantized,
                           const float *W, const float *L, const float *R, uint8_t *pc,
                           uint8_t *pe, uint8_t *l6, uint8_t *le, uint8_t *r6, uint8_t *re,
                           float *P_out)
{
    const int64_t BK = K / 32;
    const int BR = r / 32;
    for (int j = 0; j < r; ++j) lqo_quant_mxfp6(R + (int64_t)j * K, K, r6 + (int64_t)j * K, re + (int64_t)j * BK);
    for (int64_t n = 0; n < N; ++n) lqo_quant_mxfp6(L + n * r, r, l6 + n * r, le + n * BR);

#pragma omp parallel for schedule(static)
    for (int64_t n = 0; n < N; ++n) {
        float *P = (float *)malloc(sizeof(float) * (size_t)K);
        for (int64_t k = 0; k < K; ++k) {
            double d = 0.0;
            for (int j = 0; j < r; ++j) {
                double lh, rh;
                if (residual_from_quantized) {
                    lh = mxfp6_value(l6[n * r + j], le[n * BR + j / 32]);
                    rh = mxfp6_value(r6[(int64_t)j * K + k], re[(int64_t)j * BK + k / 32]);
                } else {
                    lh = L[n * r + j];
                    rh = R[(int64_t)j * K + k];
                }
                d += lh * rh;
            }
            P[k] = (float)((double)W[n * K + k] - d);
        }
        lqo_quant_mxfp4(P, K, pc + n * K, pe + n * BK);
        if (P_out) memcpy(P_out + n * K, P, sizeof(float) * (size_t)K);
        free(P);
    }
}

/* Outputs as lqo_quantize_act_mxb, with E2M3 codes for the branch activations and the intermediate. */
LQO_API void lqo_quantize_act_mxb6(int64_t M, int64_t K, int r, const float *X, const uint8_t *r6,
                                   const uint8_t *re, uint8_t *xc, uint8_t *xe, uint8_t *xb6,
                                   uint8_t *xbe, float *T, uint8_t *tq6, uint8_t *te)
{
    const int64_t BK = K / 32;
    const int BR = r / 32;
#pragma omp parallel for schedule(static)
    for (int64_t m = 0; m < M; ++m) {
        const float *x = X + m * K;
        lqo_quant_mxfp4(x, K, xc + m * K, xe + m * BK);
        if (r == 0) continue;
        lqo_quant_mxfp6(x, K, xb6 + m * K, xbe + m * BK);
        float *Trow = (float *)malloc(sizeof(float) * (size_t)r);
        for (int j = 0; j < r; ++j) {
            double a = 0.0;
            for (int64_t b = 0; b < BK; ++b) {
                double d = 0.0;
                for (int k = 0; k < 32; ++k)
                    d += (double)lqo_e2m3_decode(xb6[m * K + 32 * b + k]) *
                         (double)lqo_e2m3_decode(r6[(int64_t)j * K + 32 * b + k]);
                a += lqo_e8m0_decode(xbe[m * BK + b]) * lqo_e8m0_decode(re[(int64_t)j * BK + b]) * d;
            }
            Trow[j] = (float)a;
        }
        lqo_quant_mxfp6(Trow, r, tq6 + m * r, te + m * BR);
        if (T) memcpy(T + m * r, Trow, sizeof(float) * (size_t)r);
        free(Trow);
    }
}

LQO_API void lqo_fwd_mxb6(int64_t M, int64_t N, int64_t K, int r, const uint8_t *xc,
                          const uint8_t *xe, const uint8_t *pc, const uint8_t *pe,
                          const uint8_t *tq6, const uint8_t *te, const uint8_t *l6,
                          const uint8_t *le, float *ymain, float *ybr, float *y32, uint16_t *Y)
{
    const int64_t B = K / 32;
    const int BR = r / 32;
    float *vw = (float *)malloc(sizeof(float) * (size_t)(N * K));
    for (int64_t i = 0; i < N * K; ++i) vw[i] = lqo_e2m1_decode(pc[i]);
#pragma omp parallel for schedule(static)
    for (int64_t m = 0; m < M; ++m) {
        float *vx = (float *)malloc(sizeof(float) * (size_t)K);
        for (int64_t k = 0; k < K; ++k) vx[k] = lqo_e2m1_decode(xc[m * K + k]);
        for (int64_t n = 0; n < N; ++n) {
            double t = 0.0;
            for (int64_t b = 0; b < B; ++b) {
                double d = 0.0;
                for (int k = 0; k < 32; ++k)
                    d += (double)vx[32 * b + k] * (double)vw[n * K + 32 * b + k];
                t += lqo_e8m0_decode(xe[m * B + b]) * lqo_e8m0_decode(pe[n * B + b]) * d;
            }
            double u = 0.0;
            for (int b = 0; b < BR; ++b) {
                double d = 0.0;
                for (int j = 0; j < 32; ++j)
                    d += (double)lqo_e2m3_decode(tq6[m * r + 32 * b + j]) *
                         (double)lqo_e2m3_decode(l6[n * r + 32 * b + j]);
                u += lqo_e8m0_decode(te[m * BR + b]) * lqo_e8m0_decode(le[n * BR + b]) * d;
            }
            float y = (float)(t + u); /* sum node of Fig. 1: both accumulators, one rounding */
            if (ymain) ymain[m * N + n] = (float)t;
            if (ybr) ybr[m * N + n] = (float)u;
            if (y32) y32[m * N + n] = y;
            if (Y) Y[m * N + n] = bf16_rne(y);
        }
        free(vx);
    }
    free(vw);
}

/* ------------------------------------------------------------------------------------ */
/* Data-free calibration of the low-rank factors (Section 3.2, Eq. 4; App. B.2)           */
/* ------------------------------------------------------------------------------------ */

/* One Adam step on   loss(L, R) = mean_{n,k} ( Q1(W + L R) - W - L R )^2   (Eq. 4 with the Mean Squared
   Error loss).  Orientation as everywhere here: W is N x K, L is N x r, R is r x K (the paper's
   W^T, R^T, L^T); Q1 quantises W + L R along K: q1 = 0 INT4 in groups of g with fp32 scales, 1 SINT4 blocks,
   2 MXFP4, 3 MXINT4 (blocks of 32, E8M0 scale; g is ignored for 1..3).
   Readings:
     - the point V = W + L R at which Q1 is evaluated is an fp32 number: v = W[n,k], then
       v = fma(L[n,j], R[j,k], v) for ascending j (the quantised codes depend on V's rounding, so the
       arithmetic type of this decision is fixed: fp32, this order);
     - E = deq(Q1(V)) - V with deq = code * scale, both in fp32;
     - App. B.2: the rounding has zero derivative, so d loss / d(L R) = -2 E / (N K), and
       grad_L = -2/(N K) E R^T, grad_R = -2/(N K) L^T E  (accumulated in fp64 here, ascending index,
       rounded once to fp32);
     - Adam as published: m = b1 m + (1-b1) g, v = b2 v + (1-b2) g^2, bias-corrected by 1-b1^t and
       1-b2^t (t = step, counted from 1), p -= lr * mhat / (sqrt(vhat) + eps); no weight decay.  State is
       stored in fp32; one step's arithmetic is done in fp64 and rounded once per stored value.
   In/out: L, R, mL, vL, mR, vR.  Out (each optional): E N x K, gL N x r, gR r x K, *loss (before the
   update). */
LQO_API void lqo_calib_step(int64_t N, int64_t K, int r, int g, int q1, const float *W, float *L,
                            float *R, float *mL, float *vL, float *mR, float *vR, int step, double lr,
                            double b1, double b2, double eps, float *E_out, float *gL_out, float *gR_out,
                            double *loss_out)
{
    if (q1 == 1) g = 64;
    if (q1 >= 2) g = 32;
    const int64_t G = K / g;
    float *E = (float *)malloc(sizeof(float) * (size_t)(N * K));
    float *gL = (float *)malloc(sizeof(float) * (size_t)(N * (r > 0 ? r : 1)));
    float *gR = (float *)malloc(sizeof(float) * (size_t)((r > 0 ? r : 1) * K));
    const double c = -2.0 / ((double)N * (double)K);

#pragma omp parallel for schedule(static)
    for (int64_t n = 0; n < N; ++n) {
        float *V = (float *)malloc(sizeof(float) * (size_t)K);
        int8_t *q = (int8_t *)malloc((size_t)K);
        float *sc = (float *)malloc(sizeof(float) * (size_t)G);
        for (int64_t k = 0; k < K; ++k) {
            float v = W[n * K + k];
            for (int j = 0; j < r; ++j) v = fmaf(L[n * r + j], R[(int64_t)j * K + k], v);
            V[k] = v;
        }
        if (q1 >= 2) { /* element value times the block's power of two: exact in fp32 */
            uint8_t *eb = (uint8_t *)malloc((size_t)G);
            if (q1 == 2)
                lqo_quant_mxfp4(V, K, (uint8_t *)q, eb);
            else
                lqo_quant_mxint(V, K, 4, q, eb);
            for (int64_t k = 0; k < K; ++k) {
                float deq = q1 == 2 ? lqo_e2m1_decode((uint8_t)q[k]) * (float)lqo_e8m0_decode(eb[k / 32])
                                    : (float)mxint_value(q[k], eb[k / 32], 4);
                E[n * K + k] = deq - V[k];
            }
            free(eb);
        } else {
            if (q1 == 1)
                lqo_quant_sint4(V, K, q, sc);
            else
                for (int64_t gi = 0; gi < G; ++gi) lqo_quant_int(V + gi * g, g, 7, q + gi * g, &sc[gi]);
            for (int64_t k = 0; k < K; ++k) {
                float deq = (float)q[k] * sc[k / g];
                E[n * K + k] = deq - V[k];
            }
        }
        free(V);
        free(q);
        free(sc);
    }
    double loss = 0.0;
    for (int64_t i = 0; i < N * K; ++i) loss += (double)E[i] * (double)E[i];
    loss /= (double)N * (double)K;

#pragma omp parallel for schedule(static)
    for (int64_t n = 0; n < N; ++n)
        for (int j = 0; j < r; ++j) {
            double a = 0.0;
            for (int64_t k = 0; k < K; ++k) a += (double)E[n * K + k] * (double)R[(int64_t)j * K + k];
            gL[n * r + j] = (float)(c * a);
        }
#pragma omp parallel for schedule(static)
    for (int64_t k = 0; k < K; ++k)
        for (int j = 0; j < r; ++j) {
            double a = 0.0;
            for (int64_t n = 0; n < N; ++n) a += (double)L[n * r + j] * (double)E[n * K + k];
            gR[(int64_t)j * K + k] = (float)(c * a);
        }

    const double c1 = 1.0 - pow(b1, (double)step), c2 = 1.0 - pow(b2, (double)step);
    for (int pass = 0; pass < 2; ++pass) {
        float *p = pass ? R : L, *m = pass ? mR : mL, *v = pass ? vR : vL;
        const float *gr = pass ? gR : gL;
        const int64_t cnt = pass ? (int64_t)r * K : N * r;
        for (int64_t i = 0; i < cnt; ++i) {
            double gd = (double)gr[i];
            double mm = b1 * (double)m[i] + (1.0 - b1) * gd;
            double vv = b2 * (double)v[i] + (1.0 - b2) * gd * gd;
            m[i] = (float)mm;
            v[i] = (float)vv;
            double upd = lr * (mm / c1) / (sqrt(vv / c2) + eps);
            p[i] = (float)((double)p[i] - upd);
        }
    }
    if (E_out) memcpy(E_out, E, sizeof(float) * (size_t)(N * K));
    if (gL_out) memcpy(gL_out, gL, sizeof(float) * (size_t)(N * r));
    if (gR_out) memcpy(gR_out, gR, sizeof(float) * (size_t)(r * K));
    if (loss_out) *loss_out = loss;
    free(E);
    free(gL);
    free(gR);
}

/* ------------------------------------------------------------------------------------ */
/* Rotation of the factors before they are quantised (Section 3.3, Eq. 6-7)               */
/* ------------------------------------------------------------------------------------ */

/* One step of the search for an orthogonal r x r matrix Omega that makes L Omega and Omega^T R easier
   to quantise with Q2 (the product L R is unchanged: Omega Omega^T = I).  Orientation as everywhere
   here: L is N x r, R is r x K.  Eq. 7 with the Mean Squared Error loss of Eq. 4:
       loss(Omega) = mean_{n,j} ( Q2(Z1) - Z1 )^2 + mean_{j,k} ( Q2(Z2) - Z2 )^2 ,
       Z1 = L Omega (N x r),  Z2 = Omega^T R (r x K).
   Q2 is the format the packing step applies to L and R, along the rows of Z1 (per output channel, r values)
   and of Z2 (per rank index, K values): q2 = 0 symmetric integers of qmax = qparam with one fp32 scale per
   row; 1 FP8 E4M3 with one fp32 scale per row; 2 MXFP8e4, 3 MXFP6e2, 4 MXINT of qparam bits (blocks of 32
   along the row, E8M0 scale; r and K multiples of 32).
   Readings (the paper names the loss, a learning rate and the optimiser family only):
     - Z1, Z2 are fp32 numbers, each a chain z = fma(a_i, b_i, z) over the rank index i ascending from
       z = 0 (the codes depend on their rounding, so the arithmetic of this decision is fixed);
     - E = deq(Q2(Z)) - Z in fp32, deq = code * scale;
     - the rounding has zero derivative, as in App. B.2, so with E1, E2 held fixed
           G = d loss / d Omega = -2/(N r) L^T E1 - 2/(r K) R E2^T          (r x r),
       accumulated in fp64, times grad_scale (1 = the loss as printed), rounded once to fp32;
     - the optimiser is the Cayley SGD with momentum of the work the paper cites for it (Li et al. 2020,
       Algorithm 1), with X = Omega and the Frobenius norm:
           M  <- beta M - G
           Wh <- M X^T - 1/2 X (X^T M X^T);   W <- Wh - Wh^T;   M <- W X
           alpha <- min(lr, 2 q / (||W|| + eps))
           Y <- X + alpha M;  s times:  Y <- X + alpha/2 W (X + Y);   X <- Y
       done in fp64 from the fp32 state and rounded once per stored value.
   In/out: Omega, Mom (r x r).  Out (each optional): E1 N x r, E2 r x K, G r x r, *loss (before the update). */
static void rot_quant_err(const float *z, int64_t n, int q2, int qparam, float *e)
{
    uint8_t *c = (uint8_t *)malloc((size_t)n);
    uint8_t *eb = (uint8_t *)malloc((size_t)(n / 32 + 1));
    float sc;
    switch (q2) {
    case 0:
        lqo_quant_int(z, n, qparam, (int8_t *)c, &sc);
        for (int64_t i = 0; i < n; ++i) e[i] = (float)((int8_t *)c)[i] * sc - z[i];
        break;
    case 1:
        lqo_quant_fp8(z, n, c, &sc);
        for (int64_t i = 0; i < n; ++i) e[i] = lqo_e4m3_decode(c[i]) * sc - z[i];
        break;
    case 2:
        lqo_quant_mxfp8(z, n, c, eb);
        for (int64_t i = 0; i < n; ++i) e[i] = (float)mxfp8_value(c[i], eb[i / 32]) - z[i];
        break;
    case 3:
        lqo_quant_mxfp6(z, n, c, eb);
        for (int64_t i = 0; i < n; ++i) e[i] = (float)mxfp6_value(c[i], eb[i / 32]) - z[i];
        break;
    default:
        lqo_quant_mxint(z, n, qparam, (int8_t *)c, eb);
        for (int64_t i = 0; i < n; ++i) e[i] = (float)mxint_value(((int8_t *)c)[i], eb[i / 32], qparam) - z[i];
        break;
    }
    free(c);
    free(eb);
}

LQO_API void lqo_rot_step(int64_t N, int64_t K, int r, int q2, int qparam, const float *L, const float *R, float *Omega,
                          float *Mom, double lr, double beta, double eps, double q, int s, double grad_scale,
                          float *E1_out, float *E2_out, float *G_out, double *loss_out)
{
    float *E1 = (float *)malloc(sizeof(float) * (size_t)(N * r));
    float *E2 = (float *)malloc(sizeof(float) * (size_t)(r * K));
    const int rr = r * r;

#pragma omp parallel for schedule(static)
    for (int64_t n = 0; n < N; ++n) {
        float *z = (float *)malloc(sizeof(float) * (size_t)r);
        for (int j = 0; j < r; ++j) {
            float v = 0.0f;
            for (int i = 0; i < r; ++i) v = fmaf(L[n * r + i], Omega[i * r + j], v);
            z[j] = v;
        }
        rot_quant_err(z, r, q2, qparam, E1 + n * r);
        free(z);
    }
#pragma omp parallel for schedule(static)
    for (int j = 0; j < r; ++j) {
        float *z = (float *)malloc(sizeof(float) * (size_t)K);
        for (int64_t k = 0; k < K; ++k) {
            float v = 0.0f;
            for (int i = 0; i < r; ++i) v = fmaf(Omega[i * r + j], R[(int64_t)i * K + k], v);
            z[k] = v;
        }
        rot_quant_err(z, K, q2, qparam, E2 + (int64_t)j * K);
        free(z);
    }
    double l1 = 0.0, l2 = 0.0;
    for (int64_t i = 0; i < N * r; ++i) l1 += (double)E1[i] * (double)E1[i];
    for (int64_t i = 0; i < (int64_t)r * K; ++i) l2 += (double)E2[i] * (double)E2[i];
    const double loss = l1 / ((double)N * r) + l2 / ((double)r * (double)K);

    double *G = (double *)malloc(sizeof(double) * (size_t)rr);
    const double c1 = -2.0 / ((double)N * r), c2 = -2.0 / ((double)r * (double)K);
    for (int i = 0; i < r; ++i)
        for (int j = 0; j < r; ++j) {
            double a = 0.0, b = 0.0;
            for (int64_t n = 0; n < N; ++n) a += (double)L[n * r + i] * (double)E1[n * r + j];
            for (int64_t k = 0; k < K; ++k) b += (double)R[(int64_t)i * K + k] * (double)E2[(int64_t)j * K + k];
            G[i * r + j] = (double)(float)(grad_scale * (c1 * a + c2 * b));
        }

    /* Cayley SGD with momentum; all r x r, row-major */
    double *X = (double *)malloc(sizeof(double) * (size_t)rr * 7);
    double *M = X + rr, *A = M + rr, *B = A + rr, *Wh = B + rr, *W = Wh + rr, *Y = W + rr;
    for (int i = 0; i < rr; ++i) {
        X[i] = (double)Omega[i];
        M[i] = beta * (double)Mom[i] - G[i];
    }
    for (int i = 0; i < r; ++i)      /* A = M X^T */
        for (int j = 0; j < r; ++j) {
            double a = 0.0;
            for (int k = 0; k < r; ++k) a += M[i * r + k] * X[j * r + k];
            A[i * r + j] = a;
        }
    for (int i = 0; i < r; ++i)      /* B = X^T A = X^T M X^T */
        for (int j = 0; j < r; ++j) {
            double a = 0.0;
            for (int k = 0; k < r; ++k) a += X[k * r + i] * A[k * r + j];
            B[i * r + j] = a;
        }
    for (int i = 0; i < r; ++i)      /* Wh = A - 1/2 X B */
        for (int j = 0; j < r; ++j) {
            double a = 0.0;
            for (int k = 0; k < r; ++k) a += X[i * r + k] * B[k * r + j];
            Wh[i * r + j] = A[i * r + j] - 0.5 * a;
        }
    double nrm = 0.0;
    for (int i = 0; i < r; ++i)
        for (int j = 0; j < r; ++j) {
            W[i * r + j] = Wh[i * r + j] - Wh[j * r + i];
            nrm += W[i * r + j] * W[i * r + j];
        }
    nrm = sqrt(nrm);
    for (int i = 0; i < r; ++i)      /* M = W X */
        for (int j = 0; j < r; ++j) {
            double a = 0.0;
            for (int k = 0; k < r; ++k) a += W[i * r + k] * X[k * r + j];
            M[i * r + j] = a;
        }
    double alpha = 2.0 * q / (nrm + eps);
    if (lr < alpha) alpha = lr;
    for (int i = 0; i < rr; ++i) Y[i] = X[i] + alpha * M[i];
    for (int it = 0; it < s; ++it) {
        for (int i = 0; i < rr; ++i) A[i] = X[i] + Y[i];
        for (int i = 0; i < r; ++i)
            for (int j = 0; j < r; ++j) {
                double a = 0.0;
                for (int k = 0; k < r; ++k) a += W[i * r + k] * A[k * r + j];
                B[i * r + j] = X[i * r + j] + 0.5 * alpha * a;
            }
        for (int i = 0; i < rr; ++i) Y[i] = B[i];
    }
    for (int i = 0; i < rr; ++i) {
        Omega[i] = (float)Y[i];
        Mom[i] = (float)M[i];
    }
    if (E1_out) memcpy(E1_out, E1, sizeof(float) * (size_t)(N * r));
    if (E2_out) memcpy(E2_out, E2, sizeof(float) * (size_t)(r * K));
    if (G_out)
        for (int i = 0; i < rr; ++i) G_out[i] = (float)G[i];
    if (loss_out) *loss_out = loss;
    free(X);
    free(G);
    free(E1);
    free(E2);
}

/* The rotated factors the packing step then takes: Lr = L Omega, Rr = Omega^T R, the same fp32 chains as above. */
LQO_API void lqo_rot_apply(int64_t N, int64_t K, int r, const float *L, const float *R, const float *Omega,
                           float *Lr, float *Rr)
{
    for (int64_t n = 0; n < N; ++n)
        for (int j = 0; j < r; ++j) {
            float v = 0.0f;
            for (int i = 0; i < r; ++i) v = fmaf(L[n * r + i], Omega[i * r + j], v);
            Lr[n * r + j] = v;
        }
    for (int j = 0; j < r; ++j)
        for (int64_t k = 0; k < K; ++k) {
            float v = 0.0f;
            for (int i = 0; i < r; ++i) v = fmaf(Omega[i * r + j], R[(int64_t)i * K + k], v);
            Rr[(int64_t)j * K + k] = v;
        }
}

LQO_API int lqo_num_threads(void)
{
    int n = 1;
#ifdef _OPENMP
    extern int omp_get_max_threads(void);
    n = omp_get_max_threads();
#endif
    return n;
}

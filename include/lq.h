/*
 * lq.h -- C ABI of the MI355X (gfx950) library for the forward pass of a fully quantized
 * linear layer with a quantized low-rank error-compensation branch (paper Fig. 1, Eq. 5):
 *
 *     P = W - deq(Q2(L)) deq(Q2(R))                              (offline, lq_pack_weights)
 *     Y = deq(Q1(X) Q1(P)^T) + deq(Q2( Q2(X) Q2(R)^T ) Q2(L)^T)  (per call)
 *
 * Orientation, all row-major: X is M x K (tokens x in-features), W is N x K, L is N x r,
 * R is r x K, Y is M x N.  In the paper's notation (Section 3.1/3.2: X in R^{m x d},
 * W in R^{d x n}, L in R^{d x rho}, R in R^{rho x n}) this is M=m, K=d, N=n, W = W_paper^T,
 * L = R_paper^T, R = L_paper^T.
 *
 * Q1 is the 4-bit main format, Q2 the sub-16-bit branch format (Section 3.3).  Families:
 *   INT : Q1 = signed INT4, symmetric [-7,7], round-to-nearest-even; weights carry one fp32
 *         scale per group of `main_w_group` values along K (SINT4-style blocks, App. A.3),
 *         activations one fp32 scale per token.  Q2 = signed INT8 / INT6 / INT4 with one
 *         scale per token (activations, intermediate) or per row of L / R (weights).
 *         Integer accumulation, fp32 dequantisation.
 *         With main_a_group = 64 (and main_w_group = 64) both operands of the main product use the
 *         literal SINT4 block format of App. A.3: blocks of 64 values along K, one FP16 scale per
 *         block, s = fp16(amax / 7) kept inside [2^-24, 65504], codes clamp(rne(v * fl(1 / s))), and
 *         Y = sum_g acc_g * (sx[m,g] * sw[n,g]) + branch.  The branch keeps its per-token scales.  K <= 5632.
 *   MX  : Q1 = MXFP4 (E2M1 elements, blocks of 32 along K, E8M0 scale, App. A.3) for both
 *         operands; Q2 = FP8 E4M3 with one fp32 scale per token / per row, or (all-MX setting of
 *         the mixed-precision tables, Section 4.3) MXFP8e4 / MXFP6e2: E4M3 / E2M3 elements in blocks of 32 along
 *         the contraction axis (K for X and R, the rank for X R^T and L) with E8M0 scales; then
 *         no fp32 scale exists and the branch accumulates into the main product's accumulator.
 *   MXI : the integer MX formats of App. A.3 (the integer rows of the mixed-precision tables,
 *         Section 4.3): Q1 = MXINT4 for both operands; Q2 = MXINT8 for X and X R^T, MXINT8 or
 *         MXINT4 for L and R.  Element of width b: code c in [-(2^(b-1)-1), 2^(b-1)-1], value
 *         c * 2^-(b-2) * 2^(E-127), E - 127 = floor(log2 amax) of the block of 32 (E = 0 for an
 *         all-zero block).  Block maxima must be zero or lie in [2^-100, 2^120].
 *
 * General rules
 *   - Every pointer named "device" is GPU memory of the current HIP device, owned by the
 *     caller; the library never allocates, frees or keeps device memory.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).  All calls are
 *     asynchronous on it and never synchronise.
 *   - Argument errors are found on the host before anything is launched and reported by the
 *     return value; a failed launch returns LQ_ERR_DEVICE.  Nothing throws.
 *   - Inputs must be finite (NaN / Inf give undefined codes).
 *   - Shape contract: K % 64 == 0, K % main_w_group == 0, N % 64 == 0,
 *     rank in {0,16,32,64,96,128} ({0,32,64,96,128} with a block-scaled branch, {0,16,32,64,128} with the fp32-scaled
 *     FP8 branch), 0 <= M <= 2^24 (M = 0, an empty batch: LQ_OK, nothing is launched and no pointer is looked at),
 *     row strides >= row lengths.
 *   - Calls are deterministic: no atomics, no split-K; repeated calls give identical bits.
 */
#ifndef LQ_H
#define LQ_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    LQ_OK = 0,
    LQ_ERR_NULL = 1,             /* a required pointer is NULL                           */
    LQ_ERR_SHAPE = 2,            /* a dimension violates the shape contract              */
    LQ_ERR_UNSUPPORTED = 3,      /* format combination not implemented                   */
    LQ_ERR_ALIGN = 4,            /* a pointer or stride is not aligned as documented     */
    LQ_ERR_BUFFER_TOO_SMALL = 5, /* caller's buffer smaller than lq_*_sizes reports       */
    LQ_ERR_DEVICE = 6,           /* the HIP runtime rejected a launch                    */
    LQ_ERR_STALE_BLOB = 7        /* lq_verify_blob: the blob's header belongs to another configuration, token count or layout version */
} lq_status;

typedef enum { LQ_BLOB_PACKED = 1, LQ_BLOB_ACT = 2 } lq_blob_kind;

typedef enum {
    LQ_INT4 = 0,
    LQ_INT6 = 1,
    LQ_INT8 = 2,
    LQ_MXFP4_E2M1 = 3,
    LQ_FP8_E4M3 = 4,     /* E4M3 elements, one fp32 scale per token / per row                    */
    LQ_MXFP8_E4M3 = 5,   /* "MXFP8e4" (App. A.3): E4M3 elements, blocks of 32, E8M0 scale         */
    LQ_MXINT4 = 6,       /* "MXINT4" (App. A.3): signed int4 elements, blocks of 32, E8M0 scale    */
    LQ_MXINT8 = 7,       /* "MXINT8" (App. A.3): signed int8 elements, blocks of 32, E8M0 scale    */
    LQ_MXFP6_E2M3 = 8    /* "MXFP6e2" (App. A.3): E2M3 elements, blocks of 32, E8M0 scale          */
} lq_fmt;

typedef enum { LQ_F32 = 0, LQ_BF16 = 1 } lq_dtype;

/* Problem statement of one layer (Section 3.1-3.3: W, L, R, rank, bit widths, block size,
   scale granularity).  Plain data; pass by pointer. */
typedef struct {
    int64_t N, K;                    /* out-features, in-features                                 */
    int32_t rank;                    /* r; 0 = no branch (plain W4A4)                            */
    int32_t main_w;                  /* lq_fmt: LQ_INT4 | LQ_MXFP4_E2M1                          */
    int32_t main_a;                  /* lq_fmt: must equal main_w                                 */
    int32_t main_w_group;            /* INT: 64 | 128 values along K per weight scale; MX, MXI: 32 */
    int32_t main_a_group;            /* INT: 0 = one scale per token, 64 = SINT4 blocks (needs main_w_group 64); MX, MXI: 32 */
    int32_t br_w;                    /* lq_fmt of Q2(L), Q2(R): INT8|INT6|INT4; MX: FP8 | MXFP8 | MXFP6; MXI: MXINT8 | MXINT4 */
    int32_t br_a;                    /* lq_fmt of Q2(X), Q2(X R^T): INT8|INT6; MX: = br_w; MXI: MXINT8 */
    int32_t residual_from_quantized; /* 1: P = W - deq(Q2 L) deq(Q2 R) (Fig. 1); 0: P = W - L R  */
    int32_t x_dtype;                 /* lq_dtype of X                                             */
    int32_t flags;                   /* bit set of LQ_FLAG_*; unknown bits are rejected           */
} lq_config;

/* Activation smoothing (Section 3.4; App. A.1): the activation kernel multiplies channel k of X by
   1 / gamma[k] before anything else, for both branches (the caller has folded gamma into the columns of
   W before calibration and packing).  All families; gamma is set with lq_set_smoothing after
   lq_pack_weights. */
#define LQ_FLAG_SMOOTH 1

/* Optional parity taps.  Every member may be NULL.  Device pointers, plain row-major. */
typedef struct {
    int8_t  *xb;    /* M x K   branch activation codes (INT) / E4M3 bytes or E2M3 codes (MX)    */
    float   *sxb;   /* M       branch activation scales (not with an MXFP8e4 branch)           */
    int32_t *accT;  /* M x r   integer accumulators of Q2(X) Q2(R)^T (INT only)                 */
    float   *T;     /* M x r   dequantised intermediate before re-quantisation                  */
    uint8_t *xbe;   /* M x K/32  E8M0 bytes of the branch activation blocks (MXFP8e4 branch)    */
} lq_act_debug;

typedef struct {
    int32_t *acc;   /* M x N x G   per-group accumulators of the main product (INT only)       */
    int32_t *acc2;  /* M x N       accumulators of the rank-r expansion (INT only)             */
    float   *y32;   /* M x N       fp32 sum before the bf16 rounding                            */
} lq_fwd_debug;

/* Plain row-major views of a packed weight blob / an activation blob (device pointers,
   any may be NULL).  INT family: codes are int8; MX family: pq / xq hold one E2M1 code per
   byte, pe / xe the E8M0 bytes (N x K/32, M x K/32), lq / rq / tq E4M3 bytes. */
typedef struct {
    int8_t  *pq;    /* N x K                                                                   */
    float   *sw;    /* N x (K / main_w_group)     (INT; FP16-valued with main_a_group = 64)      */
    uint8_t *pe;    /* N x (K / 32)               (MX)                                         */
    int8_t  *lq;    /* N x r                                                                   */
    float   *sl;    /* N                                                                       */
    int8_t  *rq;    /* r x K                                                                   */
    float   *sr;    /* r                                                                       */
    uint8_t *le;    /* N x r/32   E8M0 bytes of L's blocks (MXFP8e4 branch; then sl, sr unused) */
    uint8_t *re;    /* r x K/32   E8M0 bytes of R's blocks (MXFP8e4 branch)                     */
} lq_weights_view;

typedef struct {
    int8_t  *xq;    /* M x K                                                                   */
    float   *sx;    /* M                          (INT);  M x (K / 64) with main_a_group = 64    */
    uint8_t *xe;    /* M x (K / 32)               (MX)                                         */
    int8_t  *tq;    /* M x r                                                                   */
    float   *st;    /* M                                                                       */
    uint8_t *te;    /* M x r/32   E8M0 bytes of the intermediate's blocks (MXFP8e4 branch)      */
} lq_act_view;

const char *lq_status_string(lq_status s);

/* Bytes of the packed weight blob for `cfg`.  Host-only. */
lq_status lq_packed_sizes(const lq_config *cfg, size_t *packed_bytes);

/* Offline packing (Fig. 1; Eq. 5): quantise L and R with Q2, form the residual P, quantise
   it with Q1 and lay everything out for the kernels.
   W (N x K), L (N x r), R (r x K): device, fp32, dense row-major; L and R may be NULL iff
   rank == 0.  `packed`: device, 256-byte aligned, at least packed_bytes.  Contents are an
   opaque function of cfg and the inputs; read them back with lq_unpack_weights. */
lq_status lq_pack_weights(const lq_config *cfg, const float *W, const float *L, const float *R,
                          void *packed, size_t packed_bytes, void *stream);

/* Store the smoothing vector of a layer packed with LQ_FLAG_SMOOTH: gamma is device memory, K fp32
   values, finite and > 0; the blob keeps the correctly rounded reciprocals 1 / gamma[k].  Until this
   call the blob holds reciprocals 1.0 (lq_pack_weights writes them).  LQ_ERR_UNSUPPORTED without the flag. */
lq_status lq_set_smoothing(const lq_config *cfg, const float *gamma, void *packed, size_t packed_bytes,
                           void *stream);

/* Both blobs start with a 256-byte header (magic, layout version, kind, a hash of every field of the configuration, the
   token count of an activation blob, N, K) that lq_pack_weights and the activation step write.  The per-call entry
   points never read device memory on the host (that would put a synchronising copy on an asynchronous path), so they
   cannot notice a blob that was packed under another configuration, written for another M, or produced by an older
   layout: lq_verify_blob is the explicit check for callers that load blobs from elsewhere.  It copies the header to the
   host and therefore SYNCHRONISES `stream`.  kind: lq_blob_kind; M: the token count for LQ_BLOB_ACT (ignored otherwise);
   blob_bytes must cover the blob of that configuration (LQ_ERR_BUFFER_TOO_SMALL).  LQ_ERR_STALE_BLOB on a mismatch. */
lq_status lq_verify_blob(const lq_config *cfg, int32_t kind, const void *blob, size_t blob_bytes, int64_t M, void *stream);

/* Bytes of the activation blob for M tokens.  Host-only. */
lq_status lq_act_sizes(const lq_config *cfg, int64_t M, size_t *act_bytes);

/* Per-call activation step (Section 3.4; low-rank branch of Fig. 1): one pass over X emits the
   4-bit main codes and scales, quantises X for the branch, contracts it with Q2(R) and
   re-quantises the M x r result per token.
   X: device, M x K of cfg.x_dtype, row stride ldx elements (ldx >= K, ldx*elemsize % 16 == 0,
   X 16-byte aligned).  `packed`: blob written by lq_pack_weights for the same cfg, packed_bytes = the
   bytes the caller holds there (LQ_ERR_BUFFER_TOO_SMALL below lq_packed_sizes; packed may be NULL, and
   packed_bytes is then ignored, when rank == 0 and no smoothing is fused).
   `act`: device, 256-byte aligned, at least lq_act_sizes(cfg, M) bytes.  dbg may be NULL. */
lq_status lq_quantize_act(const lq_config *cfg, const void *packed, size_t packed_bytes, const void *X,
                          int64_t M, int64_t ldx, void *act, size_t act_bytes, const lq_act_debug *dbg,
                          void *stream);

/* Forward (Fig. 1): main 4-bit product with per-group dequantisation, rank-r expansion of the
   re-quantised intermediate, sum, bf16 rounding.
   Y: device, M x N bf16, row stride ldy elements (N <= ldy <= 2^22, ldy % 8 == 0, Y 16-byte aligned).
   packed_bytes / act_bytes: the bytes the caller holds behind `packed` / `act`; a blob smaller than
   lq_packed_sizes(cfg) / lq_act_sizes(cfg, M) is refused (LQ_ERR_BUFFER_TOO_SMALL) before any launch, so
   that a blob sized for another configuration or token count is never read past its end.
   dbg may be NULL (production); with dbg the same kernel also writes the taps. */
lq_status lq_linear_lowrank_fwd(const lq_config *cfg, const void *packed, size_t packed_bytes,
                                const void *act, size_t act_bytes, int64_t M, void *Y, int64_t ldy,
                                const lq_fwd_debug *dbg, void *stream);

/* Quantized hand-off between two linear layers (Section 4.5, "Method Efficiency": with quantized branches the
   activations that move between layers are in the 8-, 6- or 4-bit MX formats instead of 16 bits).  Built for the integer
   MX family (main_w = main_a = LQ_MXINT4, br_a = LQ_MXINT8 in both configurations) and a consuming layer whose K is the
   producing layer's N.  The paper does not say from which value the consumer's codes are taken, nor where an
   element-wise operation between the two linears would sit; the reading taken: the codes are those of the consumer's
   own activation step applied to the bf16 value the producer would have stored, Q(bf16_rne(y)), and nothing sits
   between the two linears (an operation in between has to consume and produce codes itself).  The two calls below
   therefore fill `act_next` with exactly the bytes lq_quantize_act(next_cfg, packed_next, Y) would have written,
   without Y (2 bytes per value) ever being stored or re-read: the producer's epilogue emits the consumer's main codes
   and block scales (0.5 + 1/32 bytes per value) straight into `act_next`, and its MXINT8 branch codes and scale bytes
   (1 + 1/32 bytes per value) into `codes`; every one of these belongs to 32 consecutive output channels, which one
   wavefront of the forward owns.  The consumer's skinny contraction runs over the whole row, so it stays a kernel of its
   own that reads the codes: lq_branch_from_codes.
     lq_handoff_sizes           bytes of the `codes` buffer for M tokens of the consuming layer.
     lq_linear_lowrank_fwd_handoff   lq_linear_lowrank_fwd plus the hand-off.  Y may be NULL (nothing is stored then);
                                with Y the bf16 output is written as well.  act_next: device, 256-byte aligned, at
                                least lq_act_sizes(next_cfg, M) bytes; codes: device, 256-byte aligned.
     lq_branch_from_codes       completes act_next (intermediate codes and scales of the consumer's branch) from `codes`;
                                a no-op for a consumer of rank 0.
   Errors as for the calls they extend; a configuration pair outside the family, or next_cfg->K != cfg->N:
   LQ_ERR_UNSUPPORTED / LQ_ERR_SHAPE before any launch. */
lq_status lq_handoff_sizes(const lq_config *next_cfg, int64_t M, size_t *codes_bytes);
lq_status lq_linear_lowrank_fwd_handoff(const lq_config *cfg, const void *packed, size_t packed_bytes, const void *act,
                                        size_t act_bytes, int64_t M, void *Y, int64_t ldy, const lq_config *next_cfg,
                                        void *act_next, size_t act_next_bytes, void *codes, size_t codes_bytes,
                                        void *stream);
lq_status lq_branch_from_codes(const lq_config *next_cfg, const void *packed_next, size_t packed_next_bytes,
                               const void *codes, size_t codes_bytes, int64_t M, void *act_next, size_t act_next_bytes,
                               void *stream);

/* Decode the opaque blobs into plain row-major arrays (test / inspection helpers). */
lq_status lq_unpack_weights(const lq_config *cfg, const void *packed, const lq_weights_view *out,
                            void *stream);
lq_status lq_unpack_act(const lq_config *cfg, const void *act, int64_t M, const lq_act_view *out,
                        void *stream);

/* ---- Data-free calibration of the factors (Section 3.2, Eq. 4; gradients of App. B.2) --------------------------
   The step that produces the L and R the forward consumes: gradient descent with Adam on
       loss(L, R) = mean over N x K of ( Q1(W + L R) - W - L R )^2 ,
   the rounding treated as having zero derivative, so that grad_L = -2/(N K) E R^T and grad_R = -2/(N K) L^T E with
   E = Q1(W + L R) - W - L R.  Q1 is cfg's main weight quantiser (INT4 groups, SINT4 blocks, MXFP4 or MXINT4; the
   branch formats of cfg play no part); rank >= 16.  W + L R is formed in fp32 (W, then one fused multiply-add per rank index, ascending).
   Sign: the factors follow the paper, Q1(W + L R) - W ~ L R, and the paper starts them at L = -L0, R = R0 with L0 R0
   the best rank-r approximation of W (an input here: the singular value decomposition is the caller's).  lq_pack_weights
   forms W - L' R', so it takes L' = -L, R' = R.
   The state blob is device memory owned by the caller (256-byte aligned, at least state_bytes); it holds the factors,
   Adam's two moments, the last step's gradients and error matrix.  A step is four kernel launches, no atomics, no
   allocation; results are reproducible bit for bit. */
typedef struct {
    float lr;      /* the paper uses 1e-4 for INT formats (App. A.2)                  */
    float beta1;   /* Adam as published: 0.9, 0.999, 1e-8; bias-corrected, no decay   */
    float beta2;
    float eps;
} lq_adam;

typedef struct {   /* plain row-major fp32 device arrays; any member may be NULL */
    float *L, *R;        /* N x r, r x K   current factors                              */
    float *mL, *vL;      /* N x r          Adam moments of L                            */
    float *mR, *vR;      /* r x K          Adam moments of R                            */
    float *gL, *gR;      /* gradients used by the last step                              */
    float *E;            /* N x K          Q1(W + L R) - (W + L R) of the last step      */
} lq_calib_view;

lq_status lq_calib_sizes(const lq_config *cfg, size_t *state_bytes);

/* Start an optimisation: copies L (N x r) and R (r x K), device fp32 dense, into the state and zeroes the moments. */
lq_status lq_calib_init(const lq_config *cfg, const float *L, const float *R, void *state, size_t state_bytes,
                        void *stream);

/* One Adam step.  W: device, N x K fp32 dense.  step: 1 for the first step after lq_calib_init, then 2, 3, ... (it
   sets the bias correction).  loss: device, one float, receives the loss BEFORE this step's update; may be NULL. */
lq_status lq_calib_step(const lq_config *cfg, const float *W, void *state, size_t state_bytes, int32_t step,
                        const lq_adam *adam, float *loss, void *stream);

/* Copy parts of the state out (device to device). */
lq_status lq_calib_unpack(const lq_config *cfg, const void *state, const lq_calib_view *out, void *stream);

/* ---- Rotation of the calibrated factors before they are quantised (Section 3.3, Eq. 6-7) -----------------------
   Search for an orthogonal r x r matrix Omega that lowers
       loss(Omega) = mean over N x r of ( Q2(L Omega) - L Omega )^2 + mean over r x K of ( Q2(Omega^T R) - Omega^T R )^2 ,
   the product (L Omega)(Omega^T R) = L R unchanged.  Q2 is the branch weight format cfg->br_w along the rows of L Omega
   and of Omega^T R, as lq_pack_weights quantises L and R: symmetric integers (INT family) or FP8 E4M3 (MX family with
   the fp32-scaled branch) with one fp32 scale per row, or MXFP8e4 / MXFP6e2 / MXINT8 / MXINT4 blocks of 32 along the row
   with E8M0 scales; rank >= 16.  The main formats of cfg play no part.  Both products are fp32 fused-multiply-add chains over the rank index, ascending
   from zero.  The rounding is treated as having zero derivative (App. B.2), so
       G = -2/(N r) L^T E1 - 2/(r K) R E2^T ,   E1 = Q2(L Omega) - L Omega,  E2 = Q2(Omega^T R) - Omega^T R ,
   times grad_scale.  The update is the Cayley SGD with momentum of the work the paper cites for it (Li et al. 2020,
   Algorithm 1; X = Omega, Frobenius norm):
       M <- beta M - G;  Wh <- M X^T - 1/2 X (X^T M X^T);  W <- Wh - Wh^T;  M <- W X;
       alpha <- min(lr, 2 q / (||W|| + eps));  Y <- X + alpha M;  s times: Y <- X + alpha/2 W (X + Y);  X <- Y.
   The paper gives the learning rate (0.5; 0.1 for the mixed-precision study; 500 steps; App. A.2) and nothing else of
   the optimiser: beta, q, s and eps are the cited algorithm's (0.9, 0.5, 2, 1e-8).  With the mean-squared-error loss
   as printed the gradient of a layer-sized problem is of the order of 1e-7 and a step of 0.5 moves Omega by as much;
   grad_scale (1 = as printed) is the caller's handle on that.
   The state blob is device memory owned by the caller (256-byte aligned, at least state_bytes).  A step is five kernel
   launches (four with block-scaled formats), no atomics, no allocation; results are reproducible bit for bit. */
typedef struct {
    float lr;          /* 0.5 (App. A.2)                                                  */
    float beta;        /* momentum, in [0, 1)                                            */
    float eps;         /* > 0                                                            */
    float q;           /* in (0, 1): alpha ||W|| / 2 stays at or below it                */
    int32_t s;         /* fixed-point passes of the Cayley transform, 0 .. 16            */
    float grad_scale;  /* > 0                                                            */
} lq_cayley;

typedef struct {   /* plain row-major fp32 device arrays; any member may be NULL */
    float *Omega, *Mom, *G;  /* r x r: the rotation, the momentum, the gradient used by the last step */
    float *E1;               /* N x r  Q2(L Omega) - L Omega of the last step                         */
    float *E2;               /* r x K  Q2(Omega^T R) - Omega^T R of the last step                     */
} lq_rot_view;

lq_status lq_rot_sizes(const lq_config *cfg, size_t *state_bytes);

/* Start a search.  Omega0, Mom0: device, r x r fp32 dense, or NULL for the identity / zero. */
lq_status lq_rot_init(const lq_config *cfg, const float *Omega0, const float *Mom0, void *state, size_t state_bytes,
                      void *stream);

/* One step.  L: device, N x r; R: device, r x K; fp32 dense, not modified.  loss: device, one float, receives the loss
   BEFORE this step's update; may be NULL. */
lq_status lq_rot_step(const lq_config *cfg, const float *L, const float *R, void *state, size_t state_bytes,
                      const lq_cayley *opt, float *loss, void *stream);

/* For callers that cannot allocate or size a workspace (code under HIP graph capture, tight serving loops, harnesses
   that forbid hipMalloc): lq_rot_step with the step's partial results (row maxima, loss and gradient partials, the
   update's work matrices) in an array the library holds on each GPU (LQ_ROT_STATIC_SCRATCH_BYTES, until the process
   ends) instead of in the state blob.  Same arguments, same kernels, same results bit for bit.  Of the state blob only
   the leading sections are used (Omega, momentum, gradient, E1, E2: 3 r^2 + N r + r K floats, each section rounded up to
   256 bytes), so state_bytes may be that small; a blob of lq_rot_sizes bytes always serves.  A configuration whose
   partial results need more than LQ_ROT_STATIC_SCRATCH_BYTES (rank 96 and 128; a K or N in the millions) is rejected
   with LQ_ERR_UNSUPPORTED before any launch.  Calls no allocator.  All calls on one GPU share that GPU's array: two
   calls that overlap in time on one GPU (different streams, or a second thread) race; calls on one stream, or ordered
   by events, are fine.  Nothing in the array has to start at zero. */
#define LQ_ROT_STATIC_SCRATCH_BYTES (2u << 20)
lq_status lq_rot_step_static(const lq_config *cfg, const float *L, const float *R, void *state, size_t state_bytes,
                             const lq_cayley *opt, float *loss, void *stream);

/* The rotated factors lq_pack_weights then takes: Lr = L Omega (N x r), Rr = Omega^T R (r x K), device fp32 dense, the
   same fp32 chains the loss quantises.  Lr, Rr must not overlap L, R. */
lq_status lq_rot_apply(const lq_config *cfg, const float *L, const float *R, const void *state, float *Lr, float *Rr,
                       void *stream);

/* Copy parts of the state out (device to device). */
lq_status lq_rot_unpack(const lq_config *cfg, const void *state, const lq_rot_view *out, void *stream);

#ifdef __cplusplus
}
#endif
#endif /* LQ_H */

// Internal declarations shared by the translation units of liblq (device layouts, launch
// prototypes).  Not part of the public ABI.
#pragma once

#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include "lq.h"

namespace lq {

// ---------------------------------------------------------------------------------------
// Device data layout (INT family).  All sections start 256-byte aligned.
//
// The 4-bit main codes (weights pq, activations xq) are stored as 6-bit sign-magnitude fields
// s00mmm, which are the E2M3 (FP6) bit patterns of +-m/8: the matrix core multiplies them in its
// FP6 mode with no expansion step in the forward kernel (every product and every partial sum is an
// integer multiple of 2^-6, exact in the fp32 accumulator).  A lane's v_mfma_f32_32x32x64_f8f6f4
// FP6 operand is the 32 codes k = 32*half .. 32*half+31 of one row as 192 contiguous bits (code i at
// bits 6i .. 6i+5), six dwords.
//
// "Fragment order" for a 64-deep K chunk and a block of 32 rows (tokens or out-channels), 1536 bytes:
//     bytes    0..1023 : [lane = row%32 + 32*half][16 bytes = dwords 0..3 of the lane's operand]
//     bytes 1024..1535 : [lane][8 bytes = dwords 4..5]
// chunks ordered [block][chunk]; a lane reads its operand as one aligned 16-byte and one aligned
// 8-byte load, each contiguous over the wavefront.
//
// The MXI family keeps 4-bit sign-magnitude nibbles, 8 codes c0..c7 per dword, such that two bit
// operations turn a dword into two dwords of FP8-E4M3 *subnormal* bytes  s0000mmm (+-m * 2^-9):
//     lo = p & 0x87878787          -> bytes of c0..c3
//     hi = rotl(p, 4) & 0x87878787 -> bytes of c4..c7
// i.e. for i in 0..3:  c_i   : sign at bit 8i+7, magnitude at bits 8i+2..8i
//                      c_4+i : sign at bit 8i+3, magnitude at bits 8j+6..8j+4, j = (i-1)&3
//
// MX family: E2M1 codes as [block of 32 rows][64-chunk][lane = row%32 + 32*half][16 bytes], code i of a lane's
// 32 in nibble i of its 16 bytes (the FP4 operand layout of v_mfma_scale_f32_32x32x64_f8f6f4).  E8M0 scales:
//     [block of 32 rows][quad = chunk/4][lane = row%32 + 32*half][4 bytes = chunks 4q..4q+3]
// so that a lane's scale operand for four consecutive chunks is one dword and the instruction's
// op_sel picks the chunk's byte (padding bytes hold 127 = 2^0).  Branch codes are E4M3 bytes;
// lq / tq rows are zero-padded to a multiple of 64.
//
// MX family with an MXFP8e4 branch (E4M3 elements, blocks of 32 along the contraction axis, E8M0
// scales; no fp32 scales): with 8-bit operands the scaled MFMA gives a lane 16 bytes of each of two
// 32-blocks, and lane (row, h) supplies the scale of block h:
//     v_mfma_scale_f32_32x32x64 : lane (row, h): bytes 0..15 = k 16h..16h+15, bytes 16..31 = k 32+16h..
//     v_mfma_scale_f32_16x16x128: lane (row, q): bytes 0..15 = k 16q..16q+15, bytes 16..31 = k 64+16q..;
//                                 lane (row, q) supplies the scale of block q
// lq / tq : [block of 32 rows][64-chunk of the rank][lane][32 bytes] (mxb_frag8_offset); le / te (in the
// sl / st sections): one dword per (row block, lane), byte cc = scale of rank block 2*cc + h.
// rq : [128-chunk of K][rank/16][lane][32 bytes] (mxb_rq_offset); re (in the sr section): one dword
// per (chunk, rank/16, lane), byte 0 = scale of K block 4*chunk + q.
//
// MXI family (MXINT4 main, MXINT8 / MXINT4 branch): main codes as 4-bit sign-magnitude nibbles in the
// fragment order of the 8-bit scaled MFMA (mxi_frag_offset), scale bytes in the MX layout above holding
// shared exponent + 127 + 7; the dequantised branch elements as bf16 in bf16-MFMA operand order
// (lq / tq sections: [block of 32 rows][rank/16][lane][8 bf16]; rq section: [64-chunk][rank/16][2][lane]
// [8 bf16]); their E8M0 bytes row-major in the sl / sr / st sections (kept for the views only).
// ---------------------------------------------------------------------------------------

struct Dims {
    int64_t N, K;   // MX family (MXFP4 main): K is the layout's K, the caller's K rounded up to 128 (the forward stages 128)
    int64_t Ks;     // the caller's K: row length of W, R and X and of the plain views (= K outside the MX family)
    int r;        // rank
    int rp;       // rank padded to a multiple of 32 (0 if r == 0)
    int g;        // main weight group (64 | 128; MX: 32)
    int G;        // K / g
    int C64;      // K / 64
    bool mx;      // MX family
    bool mxb;     // MX family with a block-scaled (MXFP8e4) branch
    int mxb_elem; // block-scaled FP branch: 8 = E4M3 (MXFP8e4), 6 = E2M3 (MXFP6e2); 0 otherwise
    bool mxi;     // MXI family: MXINT4 main product, MXINT8 / MXINT4 branch (then mx is false)
    int bw_bits;  // MXI: width of the branch weight format (8 | 4)
    bool ga;      // INT family with SINT4 blocks for both main operands (main_a_group = 64): FP16 scales per 64 values
    bool smooth;  // LQ_FLAG_SMOOTH: the activation kernel multiplies X by the stored reciprocals of gamma
    int qmax_bw;  // INT branch weight qmax
    int qmax_ba;  // INT branch activation qmax
    uint64_t cfg_hash;  // of every field of the caller's lq_config (blob headers)
};

// Every blob starts with a 256-byte header: 8 dwords {magic, layout version, kind, configuration hash (2), M (activation
// blobs; 0 otherwise), N, K}, the rest reserved.  lq_pack_weights and the activation kernels write it; lq_verify_blob
// compares it with a configuration (a blob packed under one configuration and used under another is otherwise
// undetectable: the per-call entry points never read device memory on the host).
constexpr size_t BLOB_HEADER = 256;
constexpr uint32_t BLOB_MAGIC = 0x4C515242u;   // "LQRB"
constexpr uint32_t BLOB_VERSION = 2u;          // layout revision (6-bit code fields for the INT family)
struct BlobTag { uint32_t w[8]; };
static inline BlobTag make_tag(const Dims& d, int kind, int64_t M)
{
    BlobTag t;
    t.w[0] = BLOB_MAGIC;
    t.w[1] = BLOB_VERSION;
    t.w[2] = (uint32_t)kind;
    t.w[3] = (uint32_t)d.cfg_hash;
    t.w[4] = (uint32_t)(d.cfg_hash >> 32);
    t.w[5] = (uint32_t)M;
    t.w[6] = (uint32_t)d.N;
    t.w[7] = (uint32_t)d.Ks;
    return t;
}

struct PackedLayout {
    size_t off_pq;   // main codes, fragment order: INT family N*K*3/4 bytes (6-bit fields), MX families N*K/2
    size_t off_sw;   // INT: [G][N] fp32, pre-multiplied by 2^18 (SINT4 blocks: FP16 bits in a dword);  MX: E8M0 bytes
    size_t off_lq;   // [N][rp] int8 (zero padded) / E4M3 bytes
    size_t off_sl;   // [N] fp32
    size_t off_rq;   // branch R codes in the activation kernel's operand order, r*K bytes
    size_t off_sr;   // [r] fp32
    size_t off_rg;   // [K] fp32 reciprocals of the smoothing vector (only with LQ_FLAG_SMOOTH)
    size_t total;
};

struct ActLayout {
    int64_t Mp;      // M rounded up to 32
    size_t off_xq;   // main codes, fragment order: INT family Mp*K*3/4 bytes (6-bit fields), MX families Mp*K/2
    size_t off_sx;   // INT: [Mp] fp32 (SINT4 blocks: [G][Mp/128 rounded up][32][4] dwords of FP16 bits, sxg_index);  MX: E8M0 bytes
    size_t off_tq;   // [Mp][rp] int8 / E4M3
    size_t off_st;   // [Mp] fp32
    size_t total;
};

lq_status make_dims(const lq_config* cfg, Dims* d);
PackedLayout packed_layout(const Dims& d);
ActLayout act_layout(const Dims& d, int64_t M);

static inline size_t align256(size_t x) { return (x + 255) & ~(size_t)255; }

// ---- launchers (each validates nothing: the API layer has done it) ----------------------
hipError_t launch_pack_int(const Dims& d, int residual_from_quantized, const float* W,
                           const float* L, const float* R, uint8_t* packed, hipStream_t s);
hipError_t launch_unpack_weights_int(const Dims& d, const uint8_t* packed,
                                     const lq_weights_view* out, hipStream_t s);
hipError_t launch_unpack_act_int(const Dims& d, const uint8_t* act, int64_t M,
                                 const lq_act_view* out, hipStream_t s);
hipError_t launch_quantize_act_int(const Dims& d, int x_dtype, const uint8_t* packed,
                                   const void* X, int64_t M, int64_t ldx, uint8_t* act,
                                   const lq_act_debug* dbg, hipStream_t s);
hipError_t launch_set_smoothing(const Dims& d, const float* gamma, uint8_t* packed, hipStream_t s);
hipError_t launch_fwd_int(const Dims& d, const uint8_t* packed, const uint8_t* act, int64_t M,
                          uint16_t* Y, int64_t ldy, const lq_fwd_debug* dbg, hipStream_t s);

hipError_t launch_pack_mx(const Dims& d, int residual_from_quantized, const float* W, const float* L,
                          const float* R, uint8_t* packed, hipStream_t s);
hipError_t launch_unpack_weights_mx(const Dims& d, const uint8_t* packed, const lq_weights_view* out,
                                    hipStream_t s);
hipError_t launch_unpack_act_mx(const Dims& d, const uint8_t* act, int64_t M, const lq_act_view* out,
                                hipStream_t s);
hipError_t launch_quantize_act_mx(const Dims& d, int x_dtype, const uint8_t* packed, const void* X,
                                  int64_t M, int64_t ldx, uint8_t* act, const lq_act_debug* dbg,
                                  hipStream_t s);
hipError_t launch_fwd_mx(const Dims& d, const uint8_t* packed, const uint8_t* act, int64_t M,
                         uint16_t* Y, int64_t ldy, const lq_fwd_debug* dbg, hipStream_t s);

// MXFP6e2 pieces of the MX family (lq_mx6.hip)
hipError_t launch_pack_rows_mx6(const Dims& d, const float* L, const float* R, uint8_t* packed, hipStream_t s);
hipError_t launch_unpack_weights_mx6(const Dims& d, const uint8_t* packed, const lq_weights_view* out, hipStream_t s);
hipError_t launch_unpack_act_mx6(const Dims& d, const uint8_t* act, int64_t M, const lq_act_view* out, hipStream_t s);
hipError_t launch_quantize_act_mx6(const Dims& d, int x_dtype, const uint8_t* packed, const void* X, int64_t M,
                                   int64_t ldx, uint8_t* act, const lq_act_debug* dbg, hipStream_t s);

hipError_t launch_pack_mxi(const Dims& d, int residual_from_quantized, const float* W, const float* L,
                           const float* R, uint8_t* packed, hipStream_t s);
hipError_t launch_unpack_weights_mxi(const Dims& d, const uint8_t* packed, const lq_weights_view* out,
                                     hipStream_t s);
hipError_t launch_unpack_act_mxi(const Dims& d, const uint8_t* act, int64_t M, const lq_act_view* out,
                                 hipStream_t s);
hipError_t launch_quantize_act_mxi(const Dims& d, int x_dtype, const uint8_t* packed, const void* X,
                                   int64_t M, int64_t ldx, uint8_t* act, const lq_act_debug* dbg,
                                   hipStream_t s);
hipError_t launch_fwd_mxi(const Dims& d, const uint8_t* packed, const uint8_t* act, int64_t M,
                          uint16_t* Y, int64_t ldy, const lq_fwd_debug* dbg, hipStream_t s);

// Quantized hand-off between two MXINT layers (Section 4.5; lq_mxi.hip): the producing layer's forward also writes the
// consuming layer's main codes and scales into its activation blob and its MXINT8 branch codes into a hand-off buffer
// ([Mp][K] code bytes, then [Mp][K/32] E8M0 bytes, each section 256-byte aligned); the consuming layer's branch step then
// runs from those codes.
size_t handoff_codes_bytes(const Dims& next, int64_t M);
size_t handoff_total_bytes(const Dims& next, int64_t M);
hipError_t launch_fwd_handoff_mxi(const Dims& d, const uint8_t* packed, const uint8_t* act, int64_t M, uint16_t* Y, int64_t ldy,
                                  const Dims& next, uint8_t* act_next, uint8_t* codes, hipStream_t s);
hipError_t launch_branch_from_codes_mxi(const Dims& d, const uint8_t* packed, const uint8_t* codes, int64_t M, uint8_t* act,
                                        hipStream_t s);

// Calibration state (lq_calib.hip): plain row-major fp32 sections, each 256-byte aligned.
struct CalibLayout {
    size_t off_L, off_R;       // factors, N x r and r x K
    size_t off_mL, off_vL, off_mR, off_vR;  // Adam moments (contiguous, in this order)
    size_t off_gL, off_gR;     // gradients of the last step
    size_t off_E;              // N x K  deq(Q1(W + L R)) - (W + L R) of the last step
    size_t off_lp;             // partial sums of E^2, one per wavefront
    int n_lp;
    size_t off_gRp;            // partials of L^T E over row ranges, [range][r][K]
    size_t total;
};
CalibLayout calib_layout(const Dims& d);
hipError_t launch_calib_init(const Dims& d, const float* L, const float* R, uint8_t* state, hipStream_t s);
hipError_t launch_calib_step(const Dims& d, const float* W, uint8_t* state, int step, const lq_adam* ad, float* loss,
                             hipStream_t s);
hipError_t launch_calib_unpack(const Dims& d, const uint8_t* state, const lq_calib_view* out, hipStream_t s);

struct RotLayout {
    size_t off_X, off_M, off_G;  // Omega, momentum, gradient of the last step (r x r each)
    size_t off_E1, off_E2;       // N x r and r x K quantisation errors of the rotated factors (last step)
    size_t off_ax;               // per-wavefront row maxima of Omega^T R, [4 * nkb][r]
    size_t off_lp;               // partial sums of E1^2 (nlb), then of E2^2 (r * nkb)
    size_t off_gp;               // partials of the gradient, [workgroup][r][r]
    size_t off_tmp;              // scratch matrices of the update
    int nlb, nkb, n_lp;
    size_t total;
};
RotLayout rot_layout(const Dims& d);
hipError_t launch_rot_init(const Dims& d, const float* Omega0, const float* Mom0, uint8_t* state, hipStream_t s);
hipError_t launch_rot_step(const Dims& d, const float* L, const float* R, uint8_t* state, const lq_cayley* cs, float* loss,
                           hipStream_t s);
// The same step with its partial results in a per-device array of the library instead of the state blob's last sections
// (for callers that cannot allocate); rot_static_scratch_needed = the bytes of those sections for a configuration.
hipError_t launch_rot_step_static(const Dims& d, const float* L, const float* R, uint8_t* state, const lq_cayley* cs,
                                  float* loss, hipStream_t s);
size_t rot_static_scratch_needed(const Dims& d);
hipError_t launch_rot_apply(const Dims& d, const float* L, const float* R, const uint8_t* state, float* Lr, float* Rr,
                            hipStream_t s);
hipError_t launch_rot_unpack(const Dims& d, const uint8_t* state, const lq_rot_view* out, hipStream_t s);

// Tile order of the forward kernels: panels of `panel` tile columns (256 channels each), row-major inside a panel; the
// last panel may be narrower.  The workgroups resident on an XCD at one time then share few weight column blocks: with
// all tile columns in flight at once, the weight codes of a wide layer (7.5 MB at 2240 x 6720) do not stay in the XCD's
// 4 MB L2 (measured: -5 % and -9 % on the 2240-wide layers, nothing on the 1152-wide ones, whose weights fit anyway).
// Width: the weight codes of a panel (256 channels x chunk_row_bytes per 64-chunk and tile column) within about 2 MB.
static inline int panel_width(int tilesN, int C64, int chunk_row_bytes = 32)
{
    const int pw = (int)(((int64_t)2 << 20) / ((int64_t)256 * C64 * chunk_row_bytes));
    return pw < 1 ? 1 : pw > tilesN ? tilesN : pw;
}

hipError_t launch_write_tag(uint8_t* blob, const BlobTag& t, hipStream_t s);

// ---- device helpers ----------------------------------------------------------------------
#if defined(__HIPCC__)
// header of an activation blob, written by the first workgroup of the kernel that fills the blob
__device__ __forceinline__ void write_tag(uint32_t* dst, const BlobTag& t)
{
    if (blockIdx.x == 0 && threadIdx.x < 8) dst[threadIdx.x] = t.w[threadIdx.x];
}
__device__ __forceinline__ void panel_tile(int tile, int tilesM, int tilesN, int panel, int& tile_m, int& tile_n)
{
    const int full = (tilesN / panel) * panel;  // columns in full panels
    if (tile < tilesM * full) {
        const int per = tilesM * panel, pn = tile / per, t = tile - pn * per;
        tile_m = t / panel;
        tile_n = pn * panel + (t - tile_m * panel);
    } else {
        const int w = tilesN - full, t = tile - tilesM * full;
        tile_m = t / w;
        tile_n = full + (t - tile_m * w);
    }
}
__device__ __forceinline__ uint32_t nib_lo(uint32_t p) { return p & 0x87878787u; }
__device__ __forceinline__ uint32_t nib_hi(uint32_t p)
{
    return __builtin_rotateleft32(p, 4) & 0x87878787u;
}

// Insert code e (0..7) with sign bit s (0|1) and magnitude m (0..7) into a packed dword.
__device__ __forceinline__ uint32_t nib_put(int e, uint32_t s, uint32_t m)
{
    if (e < 4) return (s << (8 * e + 7)) | (m << (8 * e));
    const int i = e - 4, j = (i - 1) & 3;
    return (s << (8 * i + 3)) | (m << (8 * j + 4));
}

// Extract code e of a packed dword as a signed integer.
__device__ __forceinline__ int nib_get(uint32_t p, int e)
{
    const uint32_t v = (e < 4) ? nib_lo(p) : nib_hi(p);
    const uint32_t b = (v >> (8 * (e & 3))) & 0xFFu;
    const int m = (int)(b & 7u);
    return (b & 0x80u) ? -m : m;
}

// ---- 6-bit main codes of the INT family (fragment order above) ----
constexpr int F6_CHUNK = 1536;  // bytes of one (32-row block, 64-chunk)
// byte offset, inside a chunk, of dword d (0..5) of lane `lane`'s operand
__device__ __forceinline__ int f6_dword_offset(int lane, int d)
{
    return d < 4 ? lane * 16 + d * 4 : 1024 + lane * 8 + (d - 4) * 4;
}
__device__ __forceinline__ size_t f6_chunk_offset(int row, int k, int C64)
{
    return ((size_t)(row >> 5) * C64 + (k >> 6)) * F6_CHUNK;
}
// the 6-bit field of an integer code in [-7, 7]
__device__ __forceinline__ uint32_t f6_field(int q) { return q < 0 ? (32u | (uint32_t)(-q)) : (uint32_t)q; }
// code (row, k) of a section in fragment order, as a signed integer
__device__ __forceinline__ int f6_get(const uint8_t* sec, int row, int k, int C64)
{
    const uint8_t* ch = sec + f6_chunk_offset(row, k, C64);
    const int lane = (row & 31) + 32 * ((k & 63) >> 5), bit = 6 * (k & 31), d = bit >> 5, sh = bit & 31;
    uint64_t v = *(const uint32_t*)(ch + f6_dword_offset(lane, d));
    if (d < 5) v |= (uint64_t)(*(const uint32_t*)(ch + f6_dword_offset(lane, d + 1))) << 32;
    const uint32_t c = (uint32_t)(v >> sh) & 63u;
    const int m = (int)(c & 7u);
    return (c & 32u) ? -m : m;
}

// ---- MXFP6e2 branch (E2M3 elements, blocks of 32, E8M0 scale): with 6-bit operands a lane of the scaled
// MFMA holds the 32 values of ONE block as 192 contiguous bits (value i at bits 6i..6i+5); they sit in the
// first 24 bytes of a 32-byte operand slot.  Slots are ordered like the 8-bit operands of the MXFP8e4 branch:
// lq / tq: [block of 32 rows][64-chunk of the rank][lane = row%32 + 32*h], h = block within the chunk;
// rq: [128-chunk of K][rank/16][lane = j%16 + 16*q], q = block within the chunk.  Scale bytes as for MXFP8e4.
__device__ __forceinline__ size_t mx6_lt_slot(int row, int blk, int rp)
{
    return ((size_t)((size_t)(row >> 5) * (rp >> 6) + (blk >> 1)) * 64 + (row & 31) + 32 * (blk & 1)) * 32;
}
__device__ __forceinline__ size_t mx6_rq_slot(int j, int kb, int r)
{
    return ((size_t)((size_t)(kb >> 2) * (r >> 4) + (j >> 4)) * 64 + (j & 15) + 16 * (kb & 3)) * 32;
}
__device__ __forceinline__ uint32_t fp6_get(const uint8_t* slot, int i)  // code i (0..31) of a slot
{
    const uint32_t* w = (const uint32_t*)slot;
    const int bit = 6 * i;
    const uint64_t v = (uint64_t)w[bit >> 5] | ((uint64_t)w[(bit >> 5) + 1] << 32);  // dword 6 exists: the slot has 8
    return (uint32_t)(v >> (bit & 31)) & 63u;
}
__device__ __forceinline__ float e2m3_value(uint32_t c)  // 1 sign, 2 exponent (bias 1), 3 mantissa bits
{
    const int e = (int)(c >> 3) & 3, m = (int)c & 7;
    const float mag = e ? ldexpf(1.0f + 0.125f * (float)m, e - 1) : 0.125f * (float)m;
    return (c & 32u) ? -mag : mag;
}

// SINT4 block scale (App. A.3): the FP16 number nearest to amax / 7, kept inside [2^-24, 65504]; 1 for an
// all-zero block.  *inv is the correctly rounded fp32 reciprocal of the stored scale.
__device__ __forceinline__ uint32_t sint4_scale(float amax, float* inv)
{
    if (amax == 0.0f) {
        *inv = 1.0f;
        return 0x3C00u;
    }
    const _Float16 h = (_Float16)fminf(__fdiv_rn(amax, 7.0f), 65504.0f);  // round to nearest even
    uint32_t bits = (uint32_t)__builtin_bit_cast(uint16_t, h);
    float f = (float)h;
    if (f < 5.9604644775390625e-08f) {
        f = 5.9604644775390625e-08f;
        bits = 1u;
    }
    *inv = __fdiv_rn(1.0f, f);
    return bits;
}
__device__ __forceinline__ float f16_bits_value(uint32_t bits) { return (float)__builtin_bit_cast(_Float16, (uint16_t)bits); }

// dword index of the block scale of token `row`, K block g: the forward reads the scales of the four 32-row
// blocks of a 128-row tile as one 16-byte operand per lane
__device__ __forceinline__ size_t sxg_index(int row, int g, int tiles128)
{
    return ((size_t)((size_t)g * tiles128 + (row >> 7)) * 32 + (row & 31)) * 4 + ((row >> 5) & 3);
}

// Activation smoothing (Section 3.4; App. A.1) fused into an activation kernel: NV (16 | 32) consecutive values of X
// (bf16 or fp32 source) times the stored reciprocals of the smoothing vector, as fp32 (zeros if !ok).  A product of a
// bf16 value and an fp32 reciprocal is not a bf16 number, so smoothing kernels hold X as fp32.
template <bool BF16IN, int NV>
__device__ __forceinline__ void smooth_load(float (&out)[NV], const void* X, size_t elem, const float* rg, bool ok)
{
    typedef int v4i_ __attribute__((ext_vector_type(4)));
    float raw[NV];
    if constexpr (BF16IN) {
#pragma unroll
        for (int q = 0; q < NV / 8; ++q) {
            v4i_ a = {0, 0, 0, 0};
            if (ok) a = ((const v4i_*)((const uint16_t*)X + elem))[q];
#pragma unroll
            for (int d = 0; d < 4; ++d) {
                raw[8 * q + 2 * d] = __uint_as_float((uint32_t)a[d] << 16);
                raw[8 * q + 2 * d + 1] = __uint_as_float((uint32_t)a[d] & 0xFFFF0000u);
            }
        }
    } else {
#pragma unroll
        for (int q = 0; q < NV / 4; ++q) {
            v4i_ a = {0, 0, 0, 0};
            if (ok) a = ((const v4i_*)((const float*)X + elem))[q];
#pragma unroll
            for (int d = 0; d < 4; ++d) raw[4 * q + d] = __int_as_float(a[d]);
        }
    }
#pragma unroll
    for (int q = 0; q < NV / 4; ++q) {
        v4i_ g = {0, 0, 0, 0};
        if (ok) g = ((const v4i_*)rg)[q];
#pragma unroll
        for (int d = 0; d < 4; ++d) out[4 * q + d] = __fmul_rn(raw[4 * q + d], __int_as_float(g[d]));
    }
}

// fp32 -> bf16 bits, round to nearest even (finite inputs)
__device__ __forceinline__ uint32_t bf16_bits(float f)
{
    uint32_t u = __float_as_uint(f);
    return (u + 0x7FFFu + ((u >> 16) & 1u)) >> 16;
}
#endif

}  // namespace lq

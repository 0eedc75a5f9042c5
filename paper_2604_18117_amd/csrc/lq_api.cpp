// Host side of the C ABI: argument validation, layout arithmetic, dispatch.  Every error is
// detected here, before any launch, so that all error paths can be exercised without a GPU.
#include <hip/hip_runtime.h>

#include "lq_internal.h"

namespace lq {

static int int_qmax(int fmt)
{
    switch (fmt) {
        case LQ_INT4: return 7;
        case LQ_INT6: return 31;
        case LQ_INT8: return 127;
        default: return 0;
    }
}

lq_status make_dims(const lq_config* cfg, Dims* d)
{
    if (!cfg) return LQ_ERR_NULL;
    if (cfg->flags & ~LQ_FLAG_SMOOTH) return LQ_ERR_UNSUPPORTED;
    if (cfg->N <= 0 || cfg->K <= 0 || cfg->N > (1 << 24) || cfg->K > (1 << 24)) return LQ_ERR_SHAPE;
    if (cfg->K % 64 != 0 || cfg->N % 64 != 0) return LQ_ERR_SHAPE;
    const int r = cfg->rank;
    if (!(r == 0 || r == 16 || r == 32 || r == 64 || r == 96 || r == 128)) return LQ_ERR_SHAPE;
    if (cfg->x_dtype != LQ_F32 && cfg->x_dtype != LQ_BF16) return LQ_ERR_UNSUPPORTED;
    if (cfg->residual_from_quantized != 0 && cfg->residual_from_quantized != 1) return LQ_ERR_UNSUPPORTED;
    d->N = cfg->N;
    d->K = d->Ks = cfg->K;
    d->r = r;
    d->rp = (r + 31) / 32 * 32;
    d->C64 = (int)(cfg->K / 64);
    d->smooth = (cfg->flags & LQ_FLAG_SMOOTH) != 0;
    d->mx = d->mxb = d->mxi = d->ga = false;
    d->bw_bits = d->mxb_elem = 0;
    if (cfg->main_w == LQ_INT4) {
        if (cfg->main_a != LQ_INT4) return LQ_ERR_UNSUPPORTED;
        if (cfg->main_w_group != 64 && cfg->main_w_group != 128) return LQ_ERR_SHAPE;
        if (cfg->K % cfg->main_w_group != 0) return LQ_ERR_SHAPE;
        if (cfg->main_a_group != 0 && cfg->main_a_group != 64) return LQ_ERR_UNSUPPORTED;
        if (cfg->main_a_group == 64 && cfg->main_w_group != 64) return LQ_ERR_UNSUPPORTED;  // one block size for both operands
        d->ga = cfg->main_a_group == 64;
        if (d->ga && cfg->K > 5632) return LQ_ERR_UNSUPPORTED;  // the forward keeps a tile's token block scales in LDS
        // the forward addresses the channel group scales with 32-bit byte offsets
        if (cfg->N * (cfg->K / cfg->main_w_group) * 4 >= ((int64_t)1 << 31)) return LQ_ERR_UNSUPPORTED;
        const int qw = int_qmax(cfg->br_w), qa = int_qmax(cfg->br_a);
        if (qw == 0 || qa == 0 || cfg->br_a == LQ_INT4) return LQ_ERR_UNSUPPORTED;
        d->mx = false;
        d->g = cfg->main_w_group;
        d->qmax_bw = qw;
        d->qmax_ba = qa;
    } else if (cfg->main_w == LQ_MXFP4_E2M1) {
        if (cfg->main_a != LQ_MXFP4_E2M1) return LQ_ERR_UNSUPPORTED;
        if (cfg->main_w_group != 32 || cfg->main_a_group != 32) return LQ_ERR_SHAPE;
        if (cfg->br_w != cfg->br_a ||
            (cfg->br_w != LQ_FP8_E4M3 && cfg->br_w != LQ_MXFP8_E4M3 && cfg->br_w != LQ_MXFP6_E2M3))
            return LQ_ERR_UNSUPPORTED;
        // the MX forward stages K in steps of 128: an odd number of 64-chunks is padded inside the blobs with one chunk
        // of zero codes (pack and activation kernels write it; sources and views keep the caller's K)
        d->K = (cfg->K + 127) / 128 * 128;
        d->C64 = (int)(d->K / 64);
        d->mxb = cfg->br_w != LQ_FP8_E4M3;
        if (!d->mxb && r == 96) return LQ_ERR_SHAPE;
        d->mxb_elem = cfg->br_w == LQ_MXFP8_E4M3 ? 8 : cfg->br_w == LQ_MXFP6_E2M3 ? 6 : 0;
        if (d->mxb && r % 32 != 0) return LQ_ERR_SHAPE;  // whole blocks of 32 along the rank
        d->mx = true;
        d->g = 32;
        d->qmax_bw = d->qmax_ba = 0;
        d->rp = (r + 63) / 64 * 64;                  // FP8 expansion runs 64 deep
    } else if (cfg->main_w == LQ_MXINT4) {
        if (cfg->main_a != LQ_MXINT4) return LQ_ERR_UNSUPPORTED;
        if (cfg->main_w_group != 32 || cfg->main_a_group != 32) return LQ_ERR_SHAPE;
        if (cfg->br_a != LQ_MXINT8 || (cfg->br_w != LQ_MXINT8 && cfg->br_w != LQ_MXINT4)) return LQ_ERR_UNSUPPORTED;
        if (r % 32 != 0) return LQ_ERR_SHAPE;  // whole blocks of 32 along the rank
        d->mxi = true;
        d->bw_bits = cfg->br_w == LQ_MXINT8 ? 8 : 4;
        d->g = 32;
        d->qmax_bw = d->qmax_ba = 0;
    } else {
        return LQ_ERR_UNSUPPORTED;
    }
    d->G = (int)(cfg->K / d->g);
    {   // FNV-1a over the configuration's fields, in declaration order
        const int64_t f[12] = {cfg->N, cfg->K, cfg->rank, cfg->main_w, cfg->main_a, cfg->main_w_group, cfg->main_a_group,
                               cfg->br_w, cfg->br_a, cfg->residual_from_quantized, cfg->x_dtype, cfg->flags};
        uint64_t h = 1469598103934665603ull;
        for (int i = 0; i < 12; ++i)
            for (int b = 0; b < 8; ++b) {
                h ^= (uint64_t)((f[i] >> (8 * b)) & 0xFF);
                h *= 1099511628211ull;
            }
        d->cfg_hash = h;
    }
    return LQ_OK;
}

PackedLayout packed_layout(const Dims& d)
{
    PackedLayout pl;
    size_t o = BLOB_HEADER;
    pl.off_pq = o;
    o = align256(o + ((d.mx || d.mxi) ? (size_t)d.N * d.K / 2 : (size_t)d.N * d.K / 4 * 3));  // INT family: 6-bit fields
    pl.off_sw = o;
    o = align256(o + ((d.mx || d.mxi) ? (size_t)(d.N / 32) * ((d.C64 + 3) / 4) * 256 : (size_t)d.N * d.G * 4));
    pl.off_lq = o;
    o = align256(o + (size_t)d.N * d.rp * (d.mxi ? 2 : 1));  // MXI: dequantised elements as bf16
    pl.off_sl = o;
    // fp32 per channel; MXFP8e4: a scale dword per (channel, rank half); MXI: a byte per (channel, rank block)
    o = align256(o + (d.mxi ? (size_t)d.N * (d.r / 32) + 4 : (size_t)d.N * (d.mxb ? 8 : 4)));
    pl.off_rq = o;
    o = align256(o + (size_t)d.r * d.K * (d.mxi ? 2 : 1));
    pl.off_sr = o;
    o = align256(o + (d.mxi   ? (size_t)d.r * (d.K / 32) + 4
                      : d.mxb ? (size_t)(d.K / 128) * (d.r / 16) * 256 + 4
                              : (size_t)(d.r > 0 ? d.r : 1) * 4));
    pl.off_rg = o;
    if (d.smooth) o = align256(o + (size_t)d.K * 4);
    pl.total = o;
    return pl;
}

ActLayout act_layout(const Dims& d, int64_t M)
{
    ActLayout al;
    al.Mp = (M + 31) / 32 * 32;
    size_t o = BLOB_HEADER;
    al.off_xq = o;
    o = align256(o + ((d.mx || d.mxi) ? (size_t)al.Mp * d.K / 2 : (size_t)al.Mp * d.K / 4 * 3));
    al.off_sx = o;
    o = align256(o + ((d.mx || d.mxi) ? (size_t)(al.Mp / 32) * ((d.C64 + 3) / 4) * 256
                      : d.ga          ? (size_t)d.G * ((al.Mp + 127) / 128) * 512
                                      : (size_t)al.Mp * 4));
    al.off_tq = o;
    o = align256(o + (size_t)al.Mp * d.rp * (d.mxi ? 2 : 1));
    al.off_st = o;
    o = align256(o + (d.mxi ? (size_t)al.Mp * (d.r / 32) + 4 : (size_t)al.Mp * (d.mxb ? 8 : 4)));
    al.total = o;
    return al;
}

}  // namespace lq

using namespace lq;

extern "C" {

const char* lq_status_string(lq_status s)
{
    switch (s) {
        case LQ_OK: return "ok";
        case LQ_ERR_NULL: return "null pointer";
        case LQ_ERR_SHAPE: return "shape violates the contract";
        case LQ_ERR_UNSUPPORTED: return "unsupported format combination";
        case LQ_ERR_ALIGN: return "misaligned pointer or stride";
        case LQ_ERR_BUFFER_TOO_SMALL: return "buffer too small";
        case LQ_ERR_DEVICE: return "HIP launch failed";
        case LQ_ERR_STALE_BLOB: return "blob header does not match the configuration";
    }
    return "unknown status";
}

lq_status lq_packed_sizes(const lq_config* cfg, size_t* packed_bytes)
{
    if (!cfg || !packed_bytes) return LQ_ERR_NULL;
    Dims d;
    lq_status st = make_dims(cfg, &d);
    if (st != LQ_OK) return st;
    *packed_bytes = packed_layout(d).total;
    return LQ_OK;
}

lq_status lq_act_sizes(const lq_config* cfg, int64_t M, size_t* act_bytes)
{
    if (!cfg || !act_bytes) return LQ_ERR_NULL;
    Dims d;
    lq_status st = make_dims(cfg, &d);
    if (st != LQ_OK) return st;
    if (M < 0 || M > (1 << 24)) return LQ_ERR_SHAPE;
    *act_bytes = M == 0 ? 0 : act_layout(d, M).total;  // (an empty batch needs no blob, not even the header)
    return LQ_OK;
}

static bool aligned(const void* p, size_t a) { return ((uintptr_t)p % a) == 0; }

lq_status lq_pack_weights(const lq_config* cfg, const float* W, const float* L, const float* R, void* packed,
                          size_t packed_bytes, void* stream)
{
    Dims d;
    lq_status st = make_dims(cfg, &d);
    if (st != LQ_OK) return st;
    if (!W || !packed) return LQ_ERR_NULL;
    if (d.r > 0 && (!L || !R)) return LQ_ERR_NULL;
    if (!aligned(packed, 256) || !aligned(W, 4)) return LQ_ERR_ALIGN;
    if (packed_bytes < packed_layout(d).total) return LQ_ERR_BUFFER_TOO_SMALL;
    hipError_t e = d.mxi ? launch_pack_mxi(d, cfg->residual_from_quantized, W, L, R, (uint8_t*)packed, (hipStream_t)stream)
                   : d.mx ? launch_pack_mx(d, cfg->residual_from_quantized, W, L, R, (uint8_t*)packed, (hipStream_t)stream)
                        : launch_pack_int(d, cfg->residual_from_quantized, W, L, R, (uint8_t*)packed, (hipStream_t)stream);
    if (e == hipSuccess) e = launch_write_tag((uint8_t*)packed, make_tag(d, LQ_BLOB_PACKED, 0), (hipStream_t)stream);
    return e == hipSuccess ? LQ_OK : LQ_ERR_DEVICE;
}

lq_status lq_verify_blob(const lq_config* cfg, int32_t kind, const void* blob, size_t blob_bytes, int64_t M, void* stream)
{
    Dims d;
    lq_status st = make_dims(cfg, &d);
    if (st != LQ_OK) return st;
    if (!blob) return LQ_ERR_NULL;
    if (kind != LQ_BLOB_PACKED && kind != LQ_BLOB_ACT) return LQ_ERR_UNSUPPORTED;
    if (kind == LQ_BLOB_ACT && (M < 1 || M > (1 << 24))) return LQ_ERR_SHAPE;
    if (!aligned(blob, 256)) return LQ_ERR_ALIGN;
    const size_t need = kind == LQ_BLOB_PACKED ? packed_layout(d).total : act_layout(d, M).total;
    if (blob_bytes < need) return LQ_ERR_BUFFER_TOO_SMALL;
    BlobTag got;
    if (hipMemcpyAsync(&got, blob, sizeof(got), hipMemcpyDeviceToHost, (hipStream_t)stream) != hipSuccess) return LQ_ERR_DEVICE;
    if (hipStreamSynchronize((hipStream_t)stream) != hipSuccess) return LQ_ERR_DEVICE;
    const BlobTag want = make_tag(d, kind, kind == LQ_BLOB_ACT ? M : 0);
    for (int i = 0; i < 8; ++i)
        if (got.w[i] != want.w[i]) return LQ_ERR_STALE_BLOB;
    return LQ_OK;
}

lq_status lq_set_smoothing(const lq_config* cfg, const float* gamma, void* packed, size_t packed_bytes, void* stream)
{
    Dims d;
    lq_status st = make_dims(cfg, &d);
    if (st != LQ_OK) return st;
    if (!d.smooth) return LQ_ERR_UNSUPPORTED;
    if (!gamma || !packed) return LQ_ERR_NULL;
    if (!aligned(packed, 256) || !aligned(gamma, 4)) return LQ_ERR_ALIGN;
    if (packed_bytes < packed_layout(d).total) return LQ_ERR_BUFFER_TOO_SMALL;
    return launch_set_smoothing(d, gamma, (uint8_t*)packed, (hipStream_t)stream) == hipSuccess ? LQ_OK : LQ_ERR_DEVICE;
}

lq_status lq_quantize_act(const lq_config* cfg, const void* packed, size_t packed_bytes, const void* X, int64_t M,
                          int64_t ldx, void* act, size_t act_bytes, const lq_act_debug* dbg, void* stream)
{
    Dims d;
    lq_status st = make_dims(cfg, &d);
    if (st != LQ_OK) return st;
    if (M == 0) return LQ_OK;  // an empty batch: nothing to do, no launch, the pointers are not looked at
    if (!X || !act) return LQ_ERR_NULL;
    if ((d.r > 0 || d.smooth) && !packed) return LQ_ERR_NULL;
    if (M < 1 || M > (1 << 24) || ldx < d.Ks) return LQ_ERR_SHAPE;
    const size_t es = cfg->x_dtype == LQ_BF16 ? 2 : 4;
    if (!aligned(X, 16) || (ldx * es) % 16 != 0 || !aligned(act, 256) || (packed && !aligned(packed, 256)))
        return LQ_ERR_ALIGN;
    if (act_bytes < act_layout(d, M).total || (packed && packed_bytes < packed_layout(d).total)) return LQ_ERR_BUFFER_TOO_SMALL;
    hipError_t e = d.mxi ? launch_quantize_act_mxi(d, cfg->x_dtype, (const uint8_t*)packed, X, M, ldx, (uint8_t*)act, dbg,
                                                   (hipStream_t)stream)
                   : d.mx ? launch_quantize_act_mx(d, cfg->x_dtype, (const uint8_t*)packed, X, M, ldx, (uint8_t*)act, dbg,
                                                 (hipStream_t)stream)
                        : launch_quantize_act_int(d, cfg->x_dtype, (const uint8_t*)packed, X, M, ldx, (uint8_t*)act, dbg,
                                                  (hipStream_t)stream);
    return e == hipSuccess ? LQ_OK : LQ_ERR_DEVICE;
}

lq_status lq_linear_lowrank_fwd(const lq_config* cfg, const void* packed, size_t packed_bytes, const void* act,
                                size_t act_bytes, int64_t M, void* Y, int64_t ldy, const lq_fwd_debug* dbg, void* stream)
{
    Dims d;
    lq_status st = make_dims(cfg, &d);
    if (st != LQ_OK) return st;
    if (M == 0) return LQ_OK;  // an empty batch
    if (!packed || !act || !Y) return LQ_ERR_NULL;
    if (M < 1 || M > (1 << 24) || ldy < d.N || ldy > (1 << 22)) return LQ_ERR_SHAPE;
    if (!aligned(packed, 256) || !aligned(act, 256) || !aligned(Y, 16) || (ldy & 7)) return LQ_ERR_ALIGN;
    if (packed_bytes < packed_layout(d).total || act_bytes < act_layout(d, M).total) return LQ_ERR_BUFFER_TOO_SMALL;
    hipError_t e = d.mxi ? launch_fwd_mxi(d, (const uint8_t*)packed, (const uint8_t*)act, M, (uint16_t*)Y, ldy, dbg,
                                          (hipStream_t)stream)
                   : d.mx ? launch_fwd_mx(d, (const uint8_t*)packed, (const uint8_t*)act, M, (uint16_t*)Y, ldy, dbg,
                                        (hipStream_t)stream)
                        : launch_fwd_int(d, (const uint8_t*)packed, (const uint8_t*)act, M, (uint16_t*)Y, ldy, dbg,
                                         (hipStream_t)stream);
    return e == hipSuccess ? LQ_OK : LQ_ERR_DEVICE;
}

static lq_status handoff_dims(const lq_config* next_cfg, Dims* dn)
{
    lq_status st = make_dims(next_cfg, dn);
    if (st != LQ_OK) return st;
    if (!dn->mxi || dn->smooth) return LQ_ERR_UNSUPPORTED;  // integer MX family; smoothing has no place in a hand-off
    return LQ_OK;
}

lq_status lq_handoff_sizes(const lq_config* next_cfg, int64_t M, size_t* codes_bytes)
{
    if (!next_cfg || !codes_bytes) return LQ_ERR_NULL;
    Dims dn;
    lq_status st = handoff_dims(next_cfg, &dn);
    if (st != LQ_OK) return st;
    if (M < 0 || M > (1 << 24)) return LQ_ERR_SHAPE;
    *codes_bytes = handoff_total_bytes(dn, M);
    return LQ_OK;
}

lq_status lq_linear_lowrank_fwd_handoff(const lq_config* cfg, const void* packed, size_t packed_bytes, const void* act,
                                        size_t act_bytes, int64_t M, void* Y, int64_t ldy, const lq_config* next_cfg,
                                        void* act_next, size_t act_next_bytes, void* codes, size_t codes_bytes, void* stream)
{
    Dims d, dn;
    lq_status st = make_dims(cfg, &d);
    if (st != LQ_OK) return st;
    if (!next_cfg) return LQ_ERR_NULL;
    st = handoff_dims(next_cfg, &dn);
    if (st != LQ_OK) return st;
    if (!d.mxi) return LQ_ERR_UNSUPPORTED;
    if (dn.K != d.N) return LQ_ERR_SHAPE;
    if (M == 0) return LQ_OK;  // an empty batch
    if (!packed || !act || !act_next || !codes) return LQ_ERR_NULL;
    if (M < 1 || M > (1 << 24) || (Y && (ldy < d.N || ldy > (1 << 22)))) return LQ_ERR_SHAPE;
    if (!aligned(packed, 256) || !aligned(act, 256) || !aligned(act_next, 256) || !aligned(codes, 256) ||
        (Y && (!aligned(Y, 16) || (ldy & 7))))
        return LQ_ERR_ALIGN;
    if (act_next_bytes < act_layout(dn, M).total || codes_bytes < handoff_total_bytes(dn, M) ||
        packed_bytes < packed_layout(d).total || act_bytes < act_layout(d, M).total)
        return LQ_ERR_BUFFER_TOO_SMALL;
    return launch_fwd_handoff_mxi(d, (const uint8_t*)packed, (const uint8_t*)act, M, (uint16_t*)Y, Y ? ldy : d.N, dn,
                                  (uint8_t*)act_next, (uint8_t*)codes, (hipStream_t)stream) == hipSuccess
               ? LQ_OK
               : LQ_ERR_DEVICE;
}

lq_status lq_branch_from_codes(const lq_config* next_cfg, const void* packed_next, size_t packed_next_bytes,
                               const void* codes, size_t codes_bytes, int64_t M, void* act_next, size_t act_next_bytes,
                               void* stream)
{
    Dims dn;
    if (!next_cfg) return LQ_ERR_NULL;
    lq_status st = handoff_dims(next_cfg, &dn);
    if (st != LQ_OK) return st;
    if (M == 0) return LQ_OK;
    if (!codes || !act_next || (dn.r > 0 && !packed_next)) return LQ_ERR_NULL;
    if (M < 1 || M > (1 << 24)) return LQ_ERR_SHAPE;
    if (!aligned(codes, 256) || !aligned(act_next, 256) || (packed_next && !aligned(packed_next, 256))) return LQ_ERR_ALIGN;
    if (act_next_bytes < act_layout(dn, M).total || codes_bytes < handoff_total_bytes(dn, M) ||
        (packed_next && packed_next_bytes < packed_layout(dn).total))
        return LQ_ERR_BUFFER_TOO_SMALL;
    if (dn.r == 0) return LQ_OK;
    return launch_branch_from_codes_mxi(dn, (const uint8_t*)packed_next, (const uint8_t*)codes, M, (uint8_t*)act_next,
                                        (hipStream_t)stream) == hipSuccess
               ? LQ_OK
               : LQ_ERR_DEVICE;
}

lq_status lq_unpack_weights(const lq_config* cfg, const void* packed, const lq_weights_view* out, void* stream)
{
    Dims d;
    lq_status st = make_dims(cfg, &d);
    if (st != LQ_OK) return st;
    if (!packed || !out) return LQ_ERR_NULL;
    if (!aligned(packed, 256)) return LQ_ERR_ALIGN;
    hipError_t e = d.mxi ? launch_unpack_weights_mxi(d, (const uint8_t*)packed, out, (hipStream_t)stream)
                   : d.mx ? launch_unpack_weights_mx(d, (const uint8_t*)packed, out, (hipStream_t)stream)
                        : launch_unpack_weights_int(d, (const uint8_t*)packed, out, (hipStream_t)stream);
    return e == hipSuccess ? LQ_OK : LQ_ERR_DEVICE;
}

lq_status lq_unpack_act(const lq_config* cfg, const void* act, int64_t M, const lq_act_view* out, void* stream)
{
    Dims d;
    lq_status st = make_dims(cfg, &d);
    if (st != LQ_OK) return st;
    if (M == 0) return LQ_OK;  // an empty batch
    if (!act || !out) return LQ_ERR_NULL;
    if (M < 1 || M > (1 << 24)) return LQ_ERR_SHAPE;
    if (!aligned(act, 256)) return LQ_ERR_ALIGN;
    hipError_t e = d.mxi ? launch_unpack_act_mxi(d, (const uint8_t*)act, M, out, (hipStream_t)stream)
                   : d.mx ? launch_unpack_act_mx(d, (const uint8_t*)act, M, out, (hipStream_t)stream)
                        : launch_unpack_act_int(d, (const uint8_t*)act, M, out, (hipStream_t)stream);
    return e == hipSuccess ? LQ_OK : LQ_ERR_DEVICE;
}

static lq_status calib_dims(const lq_config* cfg, Dims* d)
{
    lq_status st = make_dims(cfg, d);
    if (st != LQ_OK) return st;
    if (d->r < 16) return LQ_ERR_SHAPE;
    // the calibration works on the caller's W (N x K), not on packed layouts
    d->K = d->Ks;
    d->C64 = (int)(d->K / 64);
    d->G = (int)(d->K / d->g);
    return LQ_OK;
}

lq_status lq_calib_sizes(const lq_config* cfg, size_t* state_bytes)
{
    if (!cfg || !state_bytes) return LQ_ERR_NULL;
    Dims d;
    lq_status st = calib_dims(cfg, &d);
    if (st != LQ_OK) return st;
    *state_bytes = calib_layout(d).total;
    return LQ_OK;
}

lq_status lq_calib_init(const lq_config* cfg, const float* L, const float* R, void* state, size_t state_bytes, void* stream)
{
    Dims d;
    lq_status st = calib_dims(cfg, &d);
    if (st != LQ_OK) return st;
    if (!L || !R || !state) return LQ_ERR_NULL;
    if (!aligned(state, 256) || !aligned(L, 16) || !aligned(R, 16)) return LQ_ERR_ALIGN;
    if (state_bytes < calib_layout(d).total) return LQ_ERR_BUFFER_TOO_SMALL;
    return launch_calib_init(d, L, R, (uint8_t*)state, (hipStream_t)stream) == hipSuccess ? LQ_OK : LQ_ERR_DEVICE;
}

lq_status lq_calib_step(const lq_config* cfg, const float* W, void* state, size_t state_bytes, int32_t step,
                        const lq_adam* adam, float* loss, void* stream)
{
    Dims d;
    lq_status st = calib_dims(cfg, &d);
    if (st != LQ_OK) return st;
    if (!W || !state || !adam) return LQ_ERR_NULL;
    if (step < 1) return LQ_ERR_SHAPE;
    if (!(adam->lr > 0.f) || !(adam->beta1 >= 0.f && adam->beta1 < 1.f) || !(adam->beta2 >= 0.f && adam->beta2 < 1.f) ||
        !(adam->eps > 0.f))
        return LQ_ERR_UNSUPPORTED;
    if (!aligned(state, 256) || !aligned(W, 16) || (loss && !aligned(loss, 4))) return LQ_ERR_ALIGN;
    if (state_bytes < calib_layout(d).total) return LQ_ERR_BUFFER_TOO_SMALL;
    return launch_calib_step(d, W, (uint8_t*)state, step, adam, loss, (hipStream_t)stream) == hipSuccess ? LQ_OK : LQ_ERR_DEVICE;
}

lq_status lq_calib_unpack(const lq_config* cfg, const void* state, const lq_calib_view* out, void* stream)
{
    Dims d;
    lq_status st = calib_dims(cfg, &d);
    if (st != LQ_OK) return st;
    if (!state || !out) return LQ_ERR_NULL;
    if (!aligned(state, 256)) return LQ_ERR_ALIGN;
    return launch_calib_unpack(d, (const uint8_t*)state, out, (hipStream_t)stream) == hipSuccess ? LQ_OK : LQ_ERR_DEVICE;
}

static lq_status rot_dims(const lq_config* cfg, Dims* d)
{
    lq_status st = make_dims(cfg, d);
    if (st != LQ_OK) return st;
    if (d->r < 16) return LQ_ERR_SHAPE;
    // the search works on the caller's factors (N x r, r x K), not on packed layouts
    d->K = d->Ks;
    d->C64 = (int)(d->K / 64);
    d->G = (int)(d->K / d->g);
    if ((int64_t)d->r * d->K * 4 >= ((int64_t)1 << 31)) return LQ_ERR_UNSUPPORTED;  // R is read with 32-bit byte offsets
    return LQ_OK;
}

lq_status lq_rot_sizes(const lq_config* cfg, size_t* state_bytes)
{
    if (!cfg || !state_bytes) return LQ_ERR_NULL;
    Dims d;
    lq_status st = rot_dims(cfg, &d);
    if (st != LQ_OK) return st;
    *state_bytes = rot_layout(d).total;
    return LQ_OK;
}

lq_status lq_rot_init(const lq_config* cfg, const float* Omega0, const float* Mom0, void* state, size_t state_bytes,
                      void* stream)
{
    Dims d;
    lq_status st = rot_dims(cfg, &d);
    if (st != LQ_OK) return st;
    if (!state) return LQ_ERR_NULL;
    if (!aligned(state, 256) || !aligned(Omega0, 4) || !aligned(Mom0, 4)) return LQ_ERR_ALIGN;
    if (state_bytes < rot_layout(d).total) return LQ_ERR_BUFFER_TOO_SMALL;
    return launch_rot_init(d, Omega0, Mom0, (uint8_t*)state, (hipStream_t)stream) == hipSuccess ? LQ_OK : LQ_ERR_DEVICE;
}

lq_status lq_rot_step(const lq_config* cfg, const float* L, const float* R, void* state, size_t state_bytes,
                      const lq_cayley* opt, float* loss, void* stream)
{
    Dims d;
    lq_status st = rot_dims(cfg, &d);
    if (st != LQ_OK) return st;
    if (!L || !R || !state || !opt) return LQ_ERR_NULL;
    if (!(opt->lr > 0.f) || !(opt->beta >= 0.f && opt->beta < 1.f) || !(opt->eps > 0.f) || !(opt->q > 0.f && opt->q < 1.f) ||
        opt->s < 0 || opt->s > 16 || !(opt->grad_scale > 0.f))
        return LQ_ERR_UNSUPPORTED;
    if (!aligned(state, 256) || !aligned(L, 16) || !aligned(R, 16) || (loss && !aligned(loss, 4))) return LQ_ERR_ALIGN;
    if (state_bytes < rot_layout(d).total) return LQ_ERR_BUFFER_TOO_SMALL;
    return launch_rot_step(d, L, R, (uint8_t*)state, opt, loss, (hipStream_t)stream) == hipSuccess ? LQ_OK : LQ_ERR_DEVICE;
}

lq_status lq_rot_step_static(const lq_config* cfg, const float* L, const float* R, void* state, size_t state_bytes,
                             const lq_cayley* opt, float* loss, void* stream)
{
    Dims d;
    lq_status st = rot_dims(cfg, &d);
    if (st != LQ_OK) return st;
    if (!L || !R || !state || !opt) return LQ_ERR_NULL;
    if (!(opt->lr > 0.f) || !(opt->beta >= 0.f && opt->beta < 1.f) || !(opt->eps > 0.f) || !(opt->q > 0.f && opt->q < 1.f) ||
        opt->s < 0 || opt->s > 16 || !(opt->grad_scale > 0.f))
        return LQ_ERR_UNSUPPORTED;
    if (rot_static_scratch_needed(d) > LQ_ROT_STATIC_SCRATCH_BYTES) return LQ_ERR_UNSUPPORTED;  // beyond the library's array
    if (!aligned(state, 256) || !aligned(L, 16) || !aligned(R, 16) || (loss && !aligned(loss, 4))) return LQ_ERR_ALIGN;
    if (state_bytes < rot_layout(d).off_ax) return LQ_ERR_BUFFER_TOO_SMALL;  // Omega, momentum, gradient, E1, E2
    return launch_rot_step_static(d, L, R, (uint8_t*)state, opt, loss, (hipStream_t)stream) == hipSuccess ? LQ_OK : LQ_ERR_DEVICE;
}

lq_status lq_rot_apply(const lq_config* cfg, const float* L, const float* R, const void* state, float* Lr, float* Rr,
                       void* stream)
{
    Dims d;
    lq_status st = rot_dims(cfg, &d);
    if (st != LQ_OK) return st;
    if (!L || !R || !state || !Lr || !Rr) return LQ_ERR_NULL;
    if (!aligned(state, 256) || !aligned(L, 16) || !aligned(R, 16) || !aligned(Lr, 16) || !aligned(Rr, 16)) return LQ_ERR_ALIGN;
    return launch_rot_apply(d, L, R, (const uint8_t*)state, Lr, Rr, (hipStream_t)stream) == hipSuccess ? LQ_OK : LQ_ERR_DEVICE;
}

lq_status lq_rot_unpack(const lq_config* cfg, const void* state, const lq_rot_view* out, void* stream)
{
    Dims d;
    lq_status st = rot_dims(cfg, &d);
    if (st != LQ_OK) return st;
    if (!state || !out) return LQ_ERR_NULL;
    if (!aligned(state, 256)) return LQ_ERR_ALIGN;
    return launch_rot_unpack(d, (const uint8_t*)state, out, (hipStream_t)stream) == hipSuccess ? LQ_OK : LQ_ERR_DEVICE;
}

}  // extern "C"

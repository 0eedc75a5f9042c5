// MXI family: integer MX formats (App. A.3: "MXINT4 and MXINT8 quantize to a signed int4 and int8
// format", blocks of 32, E8M0 scale; the integer rows of the mixed-precision tables, Section 4.3).
//
//   main   : X and P = W - deq(Q2 L) deq(Q2 R) in MXINT4, blocks of 32 along K
//   branch : X and X R^T in MXINT8, L and R in MXINT8 or MXINT4, blocks of 32 along the contraction axis
//
// Element of width b: integer code c in [-(2^(b-1)-1), 2^(b-1)-1], value c * 2^(s-(b-2)) with the
// block's shared exponent s = floor(log2 amax) (E8M0 byte s + 127; 0 for an all-zero block).
//
// Main product: the 4-bit codes are fed to v_mfma_scale_f32_32x32x64_f8f6f4 as FP8-E4M3 subnormals
// (byte s0000mmm = +-m * 2^-9); the instruction applies both E8M0 block scales itself, so there is
// NO vector-ALU dequantisation: the stored scale byte is s + 127 + 7 (2^-9 * 2^(s+7) = 2^(s-2), one
// code step).  Inside a block every product and partial sum is exact; across blocks the matrix core
// accumulates in fp32.
// Branch: a power-of-two block scale times an integer of at most 7 bits is exactly a bf16 value, so
// the dequantised MXINT elements are stored as bf16 and both contractions run on the bf16 MFMA with
// fp32 accumulation (products exact); the rank-r expansion accumulates straight into the main
// product's accumulators.
//
// Contract beyond the general one: block maxima are zero or lie in [2^-100, 2^120].
#include "lq_internal.h"

#include <type_traits>

namespace lq {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v8i __attribute__((ext_vector_type(8)));
typedef float v4f __attribute__((ext_vector_type(4)));
typedef float v16f __attribute__((ext_vector_type(16)));
typedef __bf16 v8bf __attribute__((ext_vector_type(8)));
typedef unsigned short us2 __attribute__((ext_vector_type(2)));

// ---- layouts -------------------------------------------------------------------------------
// Main codes, "fragment order": [block of 32 rows][64-chunk of K][lane = row%32 + 32*h][16 bytes].
// With 8-bit operands the scaled MFMA takes bytes 0..15 of both lanes of a row as K block 0 and
// bytes 16..31 as K block 1, so lane (row, h) holds k = 16h..16h+15 of each 32-block: packed dwords
// 0,1 (block 0) and 2,3 (block 1); 8 codes per dword in the nibble order of nib_put.
__device__ __forceinline__ size_t mxi_frag_offset(int row, int k, int C64)  // dword holding code (row, k)
{
    const int c = k >> 6, kk = k & 63, blk = kk >> 5, h = (kk >> 4) & 1, d = 2 * blk + ((kk & 15) >> 3);
    return ((size_t)((size_t)(row >> 5) * C64 + c) * 64 + (row & 31) + 32 * h) * 16 + d * 4;
}
// Scale bytes: one dword per (block of 32 rows, quad of 64-chunks, lane); lane (row, h) holds the
// scale of K block h of its row, byte c%4 for chunk c (the instruction's op_sel picks the byte).
__device__ __forceinline__ size_t mxi_scale_offset(int row, int c, int blk, int CQ)
{
    return ((size_t)((size_t)(row >> 5) * CQ + (c >> 2)) * 64 + (row & 31) + 32 * blk) * 4 + (c & 3);
}
// bf16 element (rank row j, k) of the dequantised R, operand order of v_mfma_f32_16x16x32_bf16 in the
// activation kernel: [64-chunk][j/16][u = (k%16)/8][lane = j%16 + 16*((k%64)/16)][k%8]
__device__ __forceinline__ size_t mxi_rq_offset(int j, int k, int r)
{
    const int c = k >> 6, q = (k & 63) >> 4, u = (k & 15) >> 3;
    return ((((size_t)((size_t)c * (r >> 4) + (j >> 4)) * 2 + u) * 64 + (j & 15) + 16 * q) * 8 + (k & 7)) * 2;
}
// bf16 element (row, rank index j) of the dequantised L / intermediate, operand order of
// v_mfma_f32_32x32x16_bf16: [block of 32 rows][j/16][lane = row%32 + 32*((j%16)/8)][j%8]
__device__ __forceinline__ size_t mxi_lt_offset(int row, int j, int rp)
{
    return (((size_t)((size_t)(row >> 5) * (rp >> 4) + (j >> 4)) * 64 + (row & 31) + 32 * ((j >> 3) & 1)) * 8 + (j & 7)) * 2;
}

__device__ __forceinline__ float bf16_value(uint16_t b) { return __uint_as_float((uint32_t)b << 16); }

// shared exponent byte of a block: floor(log2 amax) + 127 clamped at 0 = the fp32 exponent field
__device__ __forceinline__ uint32_t exp_field(float amax) { return (__float_as_uint(amax) >> 23) & 0xFFu; }

// One element: code = clamp(rne(v * 2^(frac - s)), -qmax, qmax) with s = field - 127.
__device__ __forceinline__ int mxint_code(float v, uint32_t field, int bits)
{
    const float qmax = (float)((1 << (bits - 1)) - 1);
    const float q = rintf(ldexpf(v, (bits - 2) - ((int)field - 127)));
    return (int)fminf(fmaxf(q, -qmax), qmax);
}
__device__ __forceinline__ float mxint_value(int code, uint32_t field, int bits)
{
    return ldexpf((float)code, ((int)field - 127) - (bits - 2));
}

__global__ __launch_bounds__(256) void mxi_fill_kernel(uint8_t* p, size_t n, uint8_t v)
{
    const size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
    if (i < n) p[i] = v;
}

// ---------------------------------------------------------------------------------------------
// offline packing
// ---------------------------------------------------------------------------------------------
// Factors: one thread per (row, block of 32).  mode 0: rows of R, blocks along K; mode 1: rows of L,
// blocks along the rank.  Stores the dequantised elements as bf16 in operand order and the E8M0 bytes
// row-major.
__global__ __launch_bounds__(256) void mxi_pack_rows_kernel(const float* A, int rows, int len, int mode, int bits,
                                                            int r, int rp, uint8_t* vals, uint8_t* ebytes)
{
    const int nb = len >> 5;
    const size_t idx = (size_t)blockIdx.x * 256 + threadIdx.x;
    if (idx >= (size_t)rows * nb) return;
    const int row = (int)(idx / nb), b = (int)(idx % nb);
    const float* v = A + (size_t)row * len + 32 * b;
    float a = 0.f;
    for (int i = 0; i < 32; ++i) a = fmaxf(a, fabsf(v[i]));
    const uint32_t field = exp_field(a);
    ebytes[(size_t)row * nb + b] = (uint8_t)field;
    for (int i = 0; i < 32; ++i) {
        const float val = mxint_value(mxint_code(v[i], field, bits), field, bits);
        const uint16_t h = (uint16_t)(__float_as_uint(val) >> 16);  // at most 7 significant bits: exact
        const size_t off = mode == 0 ? mxi_rq_offset(row, 32 * b + i, r) : mxi_lt_offset(row, 32 * b + i, rp);
        *(uint16_t*)(vals + off) = h;
    }
}

// Residual and its MXINT4 codes: one wavefront per (n, 64-chunk), lane = k % 64 (two blocks of 32).
__global__ __launch_bounds__(256) void mxi_pack_p_kernel(const float* W, const float* L, const float* R, int N, int K,
                                                         int r, int rp, int from_q, const uint8_t* lv,
                                                         const uint8_t* rv, uint8_t* pq, uint8_t* pe)
{
    const int lane = threadIdx.x & 63;
    const int C64 = K >> 6, CQ = (C64 + 3) >> 2;
    const size_t wid = (size_t)blockIdx.x * 4 + (threadIdx.x >> 6);
    if (wid >= (size_t)N * C64) return;
    const int n = (int)(wid / C64), c = (int)(wid % C64);
    const int k = c * 64 + lane;
    double d = 0.0;
    for (int j = 0; j < r; ++j) {
        double lh, rh;
        if (from_q) {  // the dequantised elements, exact in bf16
            lh = (double)bf16_value(*(const uint16_t*)(lv + mxi_lt_offset(n, j, rp)));
            rh = (double)bf16_value(*(const uint16_t*)(rv + mxi_rq_offset(j, k, r)));
        } else {
            lh = (double)L[(size_t)n * r + j];
            rh = (double)R[(size_t)j * K + k];
        }
        d = fma(lh, rh, d);
    }
    const float P = (float)((double)W[(size_t)n * K + k] - d);
    float a = fabsf(P);
#pragma unroll
    for (int o = 16; o >= 1; o >>= 1) a = fmaxf(a, __shfl_xor(a, o, 64));  // block of 32 = half a wavefront
    const uint32_t field = exp_field(a);
    const int q = mxint_code(P, field, 4);
    uint32_t w = nib_put(lane & 7, q < 0 ? 1u : 0u, (uint32_t)(q < 0 ? -q : q));
    w |= __shfl_xor(w, 1, 64);
    w |= __shfl_xor(w, 2, 64);
    w |= __shfl_xor(w, 4, 64);
    if ((lane & 7) == 0) *(uint32_t*)(pq + mxi_frag_offset(n, k, C64)) = w;
    if ((lane & 31) == 0) pe[mxi_scale_offset(n, c, lane >> 5, CQ)] = (uint8_t)(field + 7);
}

struct MxiPackedPtrs {
    uint8_t *pq, *pe, *lv, *le, *rv, *re;
};
static MxiPackedPtrs mxi_packed_ptrs(const Dims& d, uint8_t* packed)
{
    const PackedLayout pl = packed_layout(d);
    return {packed + pl.off_pq, packed + pl.off_sw, packed + pl.off_lq, packed + pl.off_sl, packed + pl.off_rq,
            packed + pl.off_sr};
}

hipError_t launch_pack_mxi(const Dims& d, int from_q, const float* W, const float* L, const float* R, uint8_t* packed,
                           hipStream_t s)
{
    const MxiPackedPtrs pp = mxi_packed_ptrs(d, packed);
    const int N = (int)d.N, K = (int)d.K;
    // scale bytes of the padding chunks of the last quad: 2^0
    const size_t pe_bytes = (size_t)(N / 32) * ((d.C64 + 3) / 4) * 256;
    if (d.smooth) {  // reciprocals of the smoothing vector start at 1
        const hipError_t e = launch_set_smoothing(d, nullptr, packed, s);
        if (e != hipSuccess) return e;
    }
    hipLaunchKernelGGL(mxi_fill_kernel, dim3((unsigned)((pe_bytes + 255) / 256)), dim3(256), 0, s, pp.pe, pe_bytes,
                       (uint8_t)127);
    if (d.r > 0) {
        const size_t nr = (size_t)d.r * (K / 32), nl = (size_t)N * (d.r / 32);
        hipLaunchKernelGGL(mxi_pack_rows_kernel, dim3((unsigned)((nr + 255) / 256)), dim3(256), 0, s, R, d.r, K, 0,
                           d.bw_bits, d.r, d.rp, pp.rv, pp.re);
        hipLaunchKernelGGL(mxi_pack_rows_kernel, dim3((unsigned)((nl + 255) / 256)), dim3(256), 0, s, L, N, d.r, 1,
                           d.bw_bits, d.r, d.rp, pp.lv, pp.le);
    }
    const size_t waves = (size_t)N * d.C64;
    hipLaunchKernelGGL(mxi_pack_p_kernel, dim3((unsigned)((waves + 3) / 4)), dim3(256), 0, s, W, L, R, N, K, d.r, d.rp,
                       from_q, pp.lv, pp.rv, pp.pq, pp.pe);
    return hipGetLastError();
}

// ---------------------------------------------------------------------------------------------
// plain views
// ---------------------------------------------------------------------------------------------
__device__ __forceinline__ int8_t mxi_code_of(uint16_t bf, uint32_t field, int bits)
{
    return (int8_t)(int)ldexpf(bf16_value(bf), (bits - 2) - ((int)field - 127));  // exact: the value is on the grid
}

__global__ __launch_bounds__(256) void mxi_unpack_w_kernel(MxiPackedPtrs pp, int N, int K, int r, int rp, int bits,
                                                           lq_weights_view out)
{
    const size_t idx = (size_t)blockIdx.x * 256 + threadIdx.x;
    const int C64 = K >> 6, CQ = (C64 + 3) >> 2, B = K >> 5, BR = r >> 5;
    if (idx < (size_t)N * K && out.pq) {
        const int n = (int)(idx / K), k = (int)(idx % K);
        const uint32_t w = *(const uint32_t*)(pp.pq + mxi_frag_offset(n, k, C64));
        out.pq[idx] = (int8_t)nib_get(w, k & 7);
    }
    if (idx < (size_t)N * B && out.pe) {
        const int n = (int)(idx / B), b = (int)(idx % B);
        out.pe[idx] = (uint8_t)(pp.pe[mxi_scale_offset(n, b >> 1, b & 1, CQ)] - 7);
    }
    if (idx < (size_t)N * r && out.lq) {
        const int n = (int)(idx / r), j = (int)(idx % r);
        out.lq[idx] = mxi_code_of(*(const uint16_t*)(pp.lv + mxi_lt_offset(n, j, rp)), pp.le[(size_t)n * BR + (j >> 5)], bits);
    }
    if (idx < (size_t)N * BR && out.le) out.le[idx] = pp.le[idx];
    if (idx < (size_t)r * K && out.rq) {
        const int j = (int)(idx / K), k = (int)(idx % K);
        out.rq[idx] = mxi_code_of(*(const uint16_t*)(pp.rv + mxi_rq_offset(j, k, r)), pp.re[(size_t)j * B + (k >> 5)], bits);
    }
    if (idx < (size_t)r * B && out.re) out.re[idx] = pp.re[idx];
}

hipError_t launch_unpack_weights_mxi(const Dims& d, const uint8_t* packed, const lq_weights_view* out, hipStream_t s)
{
    const MxiPackedPtrs pp = mxi_packed_ptrs(d, const_cast<uint8_t*>(packed));
    const size_t n = (size_t)(d.N > d.r ? d.N : d.r) * (d.K > d.r ? d.K : d.r);  // covers N x K, r x K and N x r
    hipLaunchKernelGGL(mxi_unpack_w_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, s, pp, (int)d.N, (int)d.K,
                       d.r, d.rp, d.bw_bits, *out);
    return hipGetLastError();
}

__global__ __launch_bounds__(256) void mxi_unpack_a_kernel(const uint8_t* act, ActLayout al, int M, int K, int r, int rp,
                                                           lq_act_view out)
{
    const size_t idx = (size_t)blockIdx.x * 256 + threadIdx.x;
    const int C64 = K >> 6, CQ = (C64 + 3) >> 2, B = K >> 5, BR = r >> 5;
    if (idx < (size_t)M * K && out.xq) {
        const int m = (int)(idx / K), k = (int)(idx % K);
        const uint32_t w = *(const uint32_t*)(act + al.off_xq + mxi_frag_offset(m, k, C64));
        out.xq[idx] = (int8_t)nib_get(w, k & 7);
    }
    if (idx < (size_t)M * B && out.xe) {
        const int m = (int)(idx / B), b = (int)(idx % B);
        out.xe[idx] = (uint8_t)(act[al.off_sx + mxi_scale_offset(m, b >> 1, b & 1, CQ)] - 7);
    }
    if (idx < (size_t)M * r && out.tq) {
        const int m = (int)(idx / r), j = (int)(idx % r);
        out.tq[idx] = mxi_code_of(*(const uint16_t*)(act + al.off_tq + mxi_lt_offset(m, j, rp)),
                                  act[al.off_st + (size_t)m * BR + (j >> 5)], 8);
    }
    if (idx < (size_t)M * BR && out.te) out.te[idx] = act[al.off_st + idx];
}

hipError_t launch_unpack_act_mxi(const Dims& d, const uint8_t* act, int64_t M, const lq_act_view* out, hipStream_t s)
{
    const ActLayout al = act_layout(d, M);
    const size_t n = (size_t)M * (d.K > d.r ? d.K : d.r);
    hipLaunchKernelGGL(mxi_unpack_a_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, s, act, al, (int)M, (int)d.K,
                       d.r, d.rp, *out);
    return hipGetLastError();
}

// ---------------------------------------------------------------------------------------------
// activation kernel.  Same decomposition as the other families (16 token rows per workgroup, lane =
// (row l%16, 16-value quarter l/16 of each 64-chunk), chunks dealt round-robin to 4 wavefronts), but
// every scale is local to a block of 32, so there is no pass over the whole row before coding: the row
// is streamed through a few chunk slots and K is not limited by the register file.
// ---------------------------------------------------------------------------------------------
struct MxiActParams {
    const void* X;
    const int8_t* cb;    // from-codes variant: M x K MXINT8 codes of a quantized hand-off, row-major
    const uint8_t* cbe;  // ... and their E8M0 bytes, M x K/32
    int64_t ldx;
    int M, K, C64, CQ, r, rp;
    const uint8_t* rv;
    uint8_t* xq;
    uint8_t* xe;
    uint8_t* tv;
    uint8_t* te;
    int8_t* dbg_xb;
    uint8_t* dbg_xbe;
    float* dbg_T;
    const float* rg;  // reciprocals of the smoothing vector (smoothing variant only)
    BlobTag tag;        // header of the activation blob (written by the first workgroup)
    uint32_t* tag_dst;
};

template <bool BF16>
struct MxiChunk;
template <>
struct MxiChunk<true> {  // 16 bf16 values = 8 dwords
    uint32_t w[8];
    __device__ __forceinline__ void load(const void* X, size_t elem, bool ok)
    {
        v4i a = {0, 0, 0, 0}, b = {0, 0, 0, 0};
        if (ok) {
            const v4i* p = (const v4i*)((const uint16_t*)X + elem);
            a = p[0];
            b = p[1];
        }
        w[0] = a[0]; w[1] = a[1]; w[2] = a[2]; w[3] = a[3];
        w[4] = b[0]; w[5] = b[1]; w[6] = b[2]; w[7] = b[3];
    }
    __device__ __forceinline__ float get(int i) const
    {
        return __uint_as_float((i & 1) ? (w[i >> 1] & 0xFFFF0000u) : (w[i >> 1] << 16));
    }
};
template <>
struct MxiChunk<false> {  // 16 fp32 values
    float v[16];
    __device__ __forceinline__ void load(const void* X, size_t elem, bool ok)
    {
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            v4i a = {0, 0, 0, 0};
            if (ok) a = ((const v4i*)((const float*)X + elem))[q];
            v[4 * q] = __int_as_float(a[0]);
            v[4 * q + 1] = __int_as_float(a[1]);
            v[4 * q + 2] = __int_as_float(a[2]);
            v[4 * q + 3] = __int_as_float(a[3]);
        }
    }
    __device__ __forceinline__ float get(int i) const { return v[i]; }
};

// Round v to the MXINT8 grid of a block with exponent field `field`: multiples of 2^(s-6), ties to
// even, clamped to +-127 steps.  Adding 1.5 * 2^(17+s) leaves exactly that granularity in the sum's
// significand (|v| < 2^(s+1)); the result has at most 7 significant bits, so its upper 16 bits are
// the exact bf16 value.
__device__ __forceinline__ float mxint8_round(float v, uint32_t field)
{
    const float magic = __uint_as_float(((field + 17u) << 23) | 0x00400000u);
    const float lim = __uint_as_float((field << 23) | 0x007E0000u);  // 127 * 2^(s-6) = 1.984375 * 2^s
    const float q = __fsub_rn(__fadd_rn(v, magic), magic);
    return fminf(fmaxf(q, -lim), lim);
}
__device__ __forceinline__ uint32_t bf16_pair(float lo, float hi)  // upper halves of two floats
{
    return __builtin_amdgcn_perm(__float_as_uint(hi), __float_as_uint(lo), 0x07060302u);
}

// BF16IN: element type of X; SM: smoothing variant (X times the stored reciprocals, held as fp32).
// FROMC: the branch half of the step alone, from the MXINT8 codes of a quantized hand-off (the producing layer's
// epilogue has already written this layer's main codes and scales): 16 code bytes and a scale byte replace the 16 values
// of X, code * 2^(s-6) is the dequantised bf16 element; the contraction and the re-quantisation are the same code.
template <bool BF16IN, int NJB, bool SM = false, bool FROMC = false>
__global__ __launch_bounds__(256) void mxi_act_kernel(MxiActParams p)
{
    write_tag(p.tag_dst, p.tag);
    constexpr bool BF16 = BF16IN && !SM;  // representation of a chunk in registers
    constexpr int NJA = NJB > 0 ? NJB : 1;
    constexpr int PF = 2;  // 64-chunks in flight per wavefront (measured: 2 beats 4, 6, 8 -- fewer registers, more resident workgroups)
    __shared__ float s_acc[4][NJA][64][4];

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int r16 = lane & 15, kq = lane >> 4;
    const int row = blockIdx.x * 16 + r16;
    const bool row_ok = row < p.M;
    const int C64 = p.C64;
    const int nmy = (C64 - wave + 3) >> 2;  // chunks of this wavefront: c = wave + 4 * ci, ci < nmy

    // No scale spans more than a block of 32, so the row is streamed: PF chunks are in flight, a slot
    // is refilled as soon as its chunk has been coded.
    MxiChunk<BF16> xc[PF];
    auto load_x = [&](MxiChunk<BF16>& ch, size_t koff, bool ok) {
        if constexpr (FROMC) {  // 16 code bytes in w[0..3], the block's scale byte in w[4]
            static_assert(!FROMC || (BF16IN && !SM), "the from-codes variant reuses the packed chunk registers");
            v4i a = {0, 0, 0, 0};
            uint32_t e = 0u;
            if (ok) {
                a = *(const v4i*)(p.cb + (size_t)row * p.K + koff);
                e = p.cbe[(size_t)row * (p.K >> 5) + (koff >> 5)];
            }
            ch.w[0] = a[0]; ch.w[1] = a[1]; ch.w[2] = a[2]; ch.w[3] = a[3];
            ch.w[4] = e;
        } else if constexpr (SM)
            smooth_load<BF16IN, 16>(ch.v, p.X, (size_t)row * p.ldx + koff, p.rg + koff, ok);
        else
            ch.load(p.X, (size_t)row * p.ldx + koff, ok);
    };
#pragma unroll
    for (int i = 0; i < PF; ++i) load_x(xc[i], (size_t)(wave + 4 * i) * 64 + kq * 16, row_ok && i < nmy);
    // dequantised R fragments (bf16): first chunk now, later ones one chunk ahead.  Two register sets up to rank 64; one
    // above (refilled right after the chunk's MFMAs): a second set of 64 or more registers would halve the occupancy
    constexpr int RB = NJB > 4 ? 1 : 2;
    v4i bvs[RB][NJA][2];
    auto load_r = [&](int slot, int ci) {
        int c = wave + 4 * ci;
        c = c < C64 ? c : C64 - 1;  // clamped: a fragment past the end is fetched but not used
#pragma unroll
        for (int jb = 0; jb < NJB; ++jb)
#pragma unroll
            for (int u = 0; u < 2; ++u)
                bvs[slot][jb][u] = *(const v4i*)(p.rv + ((((size_t)((size_t)c * NJB + jb) * 2 + u) * 64 + lane) * 16));
    };
    load_r(0, 0);

    v4f acc[NJA];
#pragma unroll
    for (int jb = 0; jb < NJB; ++jb) acc[jb] = v4f{0.f, 0.f, 0.f, 0.f};

    for (int base = 0; base < nmy; base += PF) {
#pragma unroll
    for (int sl = 0; sl < PF; ++sl) {
        const int ci = base + sl;
        const int c = wave + 4 * ci;
        if constexpr (RB == 2) load_r((sl + 1) & 1, ci + 1);
        if (ci < nmy) {  // wave-uniform
            uint32_t field;
            if constexpr (FROMC) {
                field = xc[sl].w[4];
            } else {
                float m = 0.f;
                if constexpr (BF16) {
                    // |bf16| is monotonic in its low 15 bits: packed unsigned 16-bit max, two values per op
                    us2 m2 = {0, 0};
#pragma unroll
                    for (int d = 0; d < 8; ++d) m2 = __builtin_elementwise_max(m2, __builtin_bit_cast(us2, xc[sl].w[d] & 0x7FFF7FFFu));
                    const uint32_t mm = m2[0] > m2[1] ? m2[0] : m2[1];
                    m = __uint_as_float(mm << 16);
                } else {
#pragma unroll
                    for (int i = 0; i < 16; ++i) m = fmaxf(m, fabsf(xc[sl].get(i)));
                }
                const float ab = fmaxf(m, __shfl_xor(m, 16, 64));  // block of 32 = lanes kq, kq ^ 1
                field = exp_field(ab);
                // ---- main codes: MXINT4.  code = min(rne(|x| * 2^(2-s)), 7), sign kept apart
                const float inv4 = field >= 2u ? __uint_as_float((256u - field) << 23) : 0.0f;  // 2^(2-s)
                uint32_t pk[2] = {0u, 0u};
                if constexpr (BF16) {
                    // |x|*inv + 2^23 has the code in its low bits and 0x4B in its top byte; eight of them
                    // are summed at their nibble positions (the top bytes shifted by 0 and 4 add up to the
                    // constant removed first, the others leave the dword); signs by one byte permute per four
#pragma unroll
                    for (int h = 0; h < 2; ++h) {
                        uint32_t sum = 0u - 0xFB000000u;
#pragma unroll
                        for (int e = 0; e < 8; ++e) {
                            const float x = xc[sl].get(8 * h + e);
                            const uint32_t mb = __float_as_uint(__fadd_rn(fminf(__fmul_rn(fabsf(x), inv4), 7.0f), 8388608.0f));
                            const int sh = e < 4 ? 8 * e : 8 * ((e - 5) & 3) + 4;
                            sum += mb << sh;
                        }
                        const uint32_t* w = &xc[sl].w[4 * h];
                        const uint32_t s03 = __builtin_amdgcn_perm(w[1], w[0], 0x07050301u);
                        const uint32_t s47 = __builtin_amdgcn_perm(w[3], w[2], 0x07050301u);
                        pk[h] = sum | (s03 & 0x80808080u) | ((s47 >> 4) & 0x08080808u);
                    }
                } else {
#pragma unroll
                    for (int i = 0; i < 16; ++i) {
                        const float x = xc[sl].get(i);
                        const uint32_t mg = __float_as_uint(__fadd_rn(fminf(__fmul_rn(fabsf(x), inv4), 7.0f), 8388608.0f)) & 7u;
                        pk[i >> 3] |= nib_put(i & 7, __float_as_uint(x) >> 31, mg);
                    }
                }
                // lane (row, kq): block kq>>1 of the chunk, K half-block h = kq&1 -> dwords 2*(kq>>1), +1 of lane (row, h)
                uint8_t* dst = p.xq + ((size_t)((size_t)(row >> 5) * C64 + c) * 64 + (row & 31) + 32 * (kq & 1)) * 16 + (kq >> 1) * 8;
                *(uint2*)dst = make_uint2(pk[0], pk[1]);
                if ((kq & 1) == 0) p.xe[mxi_scale_offset(row, c, kq >> 1, p.CQ)] = (uint8_t)(field + 7u);
            }
            if (NJB > 0) {
                // ---- branch: MXINT8 of the same block, kept as dequantised bf16
                float v8[16];
                if constexpr (FROMC) {  // code * 2^(s-6): exact, at most 7 significant bits
                    const float step = field >= 7u ? __uint_as_float((field - 6u) << 23) : 0.0f;
#pragma unroll
                    for (int i = 0; i < 16; ++i)
                        v8[i] = __fmul_rn((float)(int)(int8_t)((xc[sl].w[i >> 2] >> (8 * (i & 3))) & 0xFFu), step);
                } else {
#pragma unroll
                    for (int i = 0; i < 16; ++i) v8[i] = mxint8_round(xc[sl].get(i), field);
                }
                v4i au[2];
#pragma unroll
                for (int u = 0; u < 2; ++u)
#pragma unroll
                    for (int d = 0; d < 4; ++d) au[u][d] = (int)bf16_pair(v8[8 * u + 2 * d], v8[8 * u + 2 * d + 1]);
                if (p.dbg_xb && row_ok) {
                    uint32_t cb[4] = {0u, 0u, 0u, 0u};
#pragma unroll
                    for (int i = 0; i < 16; ++i)
                        cb[i >> 2] |= ((uint32_t)(int)ldexpf(v8[i], 6 - ((int)field - 127)) & 0xFFu) << (8 * (i & 3));
                    *(v4i*)(p.dbg_xb + (size_t)row * p.K + c * 64 + kq * 16) = v4i{(int)cb[0], (int)cb[1], (int)cb[2], (int)cb[3]};
                }
                if (p.dbg_xbe && row_ok && (kq & 1) == 0) p.dbg_xbe[(size_t)row * (p.K >> 5) + 2 * c + (kq >> 1)] = (uint8_t)field;
#pragma unroll
                for (int jb = 0; jb < NJB; ++jb)
#pragma unroll
                    for (int u = 0; u < 2; ++u)
                        acc[jb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(v8bf, au[u]),
                                                                         __builtin_bit_cast(v8bf, bvs[sl % RB][jb][u]), acc[jb], 0, 0, 0);
            }
        }
        if constexpr (RB == 1) load_r(0, ci + 1);
        // refill the slot with the chunk PF positions further on
        load_x(xc[sl], (size_t)(c + 4 * PF) * 64 + kq * 16, row_ok && ci + PF < nmy);
    }
    }
    if constexpr (!FROMC) {   // padding chunk of the last quad (at most one per wavefront): its scale bytes must be valid E8M0 values (2^0)
        const int c = wave + 4 * nmy;
        if (c < 4 * p.CQ && (kq & 1) == 0) p.xe[mxi_scale_offset(row, c, kq >> 1, p.CQ)] = (uint8_t)127;
    }
    if (NJB == 0) return;

#pragma unroll
    for (int jb = 0; jb < NJB; ++jb) *(v4f*)&s_acc[wave][jb][lane][0] = acc[jb];
    __syncthreads();
    if (wave != 0) return;

    // lane holds column j = jb*16 + lane%16 of the intermediate for token rows 4*kq + i
    float T[NJA][4];
#pragma unroll
    for (int jb = 0; jb < NJB; ++jb) {
        v4f sum = *(const v4f*)&s_acc[0][jb][lane][0];
#pragma unroll
        for (int w = 1; w < 4; ++w) {
            const v4f o = *(const v4f*)&s_acc[w][jb][lane][0];
#pragma unroll
            for (int i = 0; i < 4; ++i) sum[i] = __fadd_rn(sum[i], o[i]);
        }
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            T[jb][i] = sum[i];
            const int grow = blockIdx.x * 16 + 4 * kq + i;
            if (grow < p.M && p.dbg_T) p.dbg_T[(size_t)grow * p.r + jb * 16 + r16] = sum[i];
        }
    }
    // re-quantise to MXINT8 per token and per block of 32 along the rank (two 16-column groups)
    const int BR = p.r >> 5;
#pragma unroll
    for (int bb = 0; bb < (NJB + 1) / 2; ++bb) {
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            float tm = fmaxf(fabsf(T[2 * bb][i]), fabsf(T[(2 * bb + 1) % NJA][i]));
#pragma unroll
            for (int o = 8; o >= 1; o >>= 1) tm = fmaxf(tm, __shfl_xor(tm, o, 64));
            const int grow = blockIdx.x * 16 + 4 * kq + i;
            const uint32_t field = exp_field(tm);
            if (r16 == 0) p.te[(size_t)grow * BR + bb] = (uint8_t)field;
#pragma unroll
            for (int g = 0; g < 2; ++g) {
                const float v = mxint8_round(T[(2 * bb + g) % NJA][i], field);
                *(uint16_t*)(p.tv + mxi_lt_offset(grow, (2 * bb + g) * 16 + r16, p.rp)) = (uint16_t)(__float_as_uint(v) >> 16);
            }
        }
    }
}

template <bool BF16, int NJB, bool SM>
static hipError_t mxi_act_launch(const MxiActParams& p, int64_t Mp, hipStream_t s)
{
    hipLaunchKernelGGL((mxi_act_kernel<BF16, NJB, SM>), dim3((unsigned)(Mp / 16)), dim3(256), 0, s, p);
    return hipGetLastError();
}
template <bool BF16, bool SM>
static hipError_t mxi_act_rank2(const MxiActParams& p, int64_t Mp, hipStream_t s)
{
    switch (p.r) {
        case 0: return mxi_act_launch<BF16, 0, SM>(p, Mp, s);
        case 32: return mxi_act_launch<BF16, 2, SM>(p, Mp, s);
        case 64: return mxi_act_launch<BF16, 4, SM>(p, Mp, s);
        case 96: return mxi_act_launch<BF16, 6, SM>(p, Mp, s);
        default: return mxi_act_launch<BF16, 8, SM>(p, Mp, s);
    }
}
template <bool BF16>
static hipError_t mxi_act_rank(const MxiActParams& p, int64_t Mp, hipStream_t s)
{
    return p.rg ? mxi_act_rank2<BF16, true>(p, Mp, s) : mxi_act_rank2<BF16, false>(p, Mp, s);
}

// The branch half of the activation step from the codes of a quantized hand-off (see mxi_act_kernel, FROMC).
hipError_t launch_branch_from_codes_mxi(const Dims& d, const uint8_t* packed, const uint8_t* codes, int64_t M, uint8_t* act,
                                        hipStream_t s)
{
    const PackedLayout pl = packed_layout(d);
    const ActLayout al = act_layout(d, M);
    MxiActParams p = {};
    p.tag = make_tag(d, LQ_BLOB_ACT, M);
    p.tag_dst = (uint32_t*)act;
    p.cb = (const int8_t*)codes;
    p.cbe = codes + handoff_codes_bytes(d, M);
    p.M = (int)M;
    p.K = (int)d.K;
    p.C64 = d.C64;
    p.CQ = (d.C64 + 3) / 4;
    p.r = d.r;
    p.rp = d.rp;
    p.rv = packed + pl.off_rq;
    p.xq = act + al.off_xq;
    p.xe = act + al.off_sx;
    p.tv = act + al.off_tq;
    p.te = act + al.off_st;
    const unsigned grid = (unsigned)(al.Mp / 16);
    switch (d.r) {
        case 32: hipLaunchKernelGGL((mxi_act_kernel<true, 2, false, true>), dim3(grid), dim3(256), 0, s, p); break;
        case 64: hipLaunchKernelGGL((mxi_act_kernel<true, 4, false, true>), dim3(grid), dim3(256), 0, s, p); break;
        case 96: hipLaunchKernelGGL((mxi_act_kernel<true, 6, false, true>), dim3(grid), dim3(256), 0, s, p); break;
        case 128: hipLaunchKernelGGL((mxi_act_kernel<true, 8, false, true>), dim3(grid), dim3(256), 0, s, p); break;
        default: break;  // rank 0: the next layer has no branch, its blob is complete after the producing layer's epilogue
    }
    return hipGetLastError();
}

hipError_t launch_quantize_act_mxi(const Dims& d, int x_dtype, const uint8_t* packed, const void* X, int64_t M,
                                   int64_t ldx, uint8_t* act, const lq_act_debug* dbg, hipStream_t s)
{
    const PackedLayout pl = packed_layout(d);
    const ActLayout al = act_layout(d, M);
    MxiActParams p;
    p.tag = make_tag(d, LQ_BLOB_ACT, M);
    p.tag_dst = (uint32_t*)act;
    p.X = X;
    p.cb = nullptr;
    p.cbe = nullptr;
    p.ldx = ldx;
    p.M = (int)M;
    p.K = (int)d.K;
    p.C64 = d.C64;
    p.CQ = (d.C64 + 3) / 4;
    p.r = d.r;
    p.rp = d.rp;
    p.rv = packed + pl.off_rq;
    p.xq = act + al.off_xq;
    p.xe = act + al.off_sx;
    p.tv = act + al.off_tq;
    p.te = act + al.off_st;
    p.dbg_xb = dbg ? dbg->xb : nullptr;
    p.dbg_xbe = dbg ? dbg->xbe : nullptr;
    p.dbg_T = dbg ? dbg->T : nullptr;
    p.rg = d.smooth ? (const float*)(packed + pl.off_rg) : nullptr;
    return x_dtype == LQ_BF16 ? mxi_act_rank<true>(p, al.Mp, s) : mxi_act_rank<false>(p, al.Mp, s);
}

// ---------------------------------------------------------------------------------------------
// forward: 1 x 4 wavefronts per workgroup, 128 x 64 outputs per wavefront, one 64-chunk of K per step
// ---------------------------------------------------------------------------------------------
struct MxiFwdParams {
    const uint8_t* xq;
    const uint8_t* xe;
    const uint8_t* tv;
    const uint8_t* pq;
    const uint8_t* pe;
    const uint8_t* lv;
    uint16_t* Y;
    int64_t ldy;
    int M, N, C64, CQ, nrb;
    int tilesM, tilesN, panel;
    float* dbg_y32;
    // quantized hand-off to a next MXINT layer whose K is this layer's N (HO variant): its main codes and scale bytes
    // (sections of its activation blob) and its MXINT8 branch codes and scale bytes (row-major, for the from-codes step)
    uint8_t* ho_xq;
    uint8_t* ho_xe;
    int8_t* ho_cb;
    uint8_t* ho_cbe;
    int ho_C64, ho_CQ;
    BlobTag ho_tag;      // header of the consumer's activation blob
    uint32_t* ho_tag_dst;
};

__device__ __forceinline__ v8i mxi_expand8(v4i p)  // 32 nibbles -> 32 FP8 subnormal bytes
{
    v8i o;
#pragma unroll
    for (int d = 0; d < 4; ++d) {
        o[2 * d] = (int)nib_lo((uint32_t)p[d]);
        o[2 * d + 1] = (int)nib_hi((uint32_t)p[d]);
    }
    return o;
}

// NK16 = 16-deep chunks of the rank: 0 | 2 | 4 | 6 | 8.  HO: quantized hand-off (Section 4.5): the epilogue also emits
// the next layer's activation codes from the bf16 values it has just formed; Y itself is optional then.
template <int NK16, bool DBG, bool HO = false>
__global__ __launch_bounds__(256, 2) void mxi_fwd_kernel(MxiFwdParams p)
{
    if constexpr (HO) write_tag(p.ho_tag_dst, p.ho_tag);
    constexpr int RBT = 4;
    constexpr int EPI_ROW = 144, EPI_WAVE = 32 * EPI_ROW;
    constexpr int LDS_MAIN = 2 * RBT * 2048;  // [buffer][row block][part][lane][16 B]
    constexpr int LDS_BYTES = LDS_MAIN > 4 * EPI_WAVE ? LDS_MAIN : 4 * EPI_WAVE;
    __shared__ __attribute__((aligned(16))) uint8_t lds[LDS_BYTES];

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int half = lane >> 5, l32 = lane & 31;

    // XCD-aware tile order: workgroup ids are dealt round-robin to the 8 XCDs, each gets one run of tiles
    const int tiles = p.tilesM * p.tilesN;
    const int per = tiles >> 3, rem = tiles & 7;
    const int xcd = blockIdx.x & 7, loc = blockIdx.x >> 3;
    const int tile = xcd * per + (xcd < rem ? xcd : rem) + loc;
    int tile_m, tile_n;
    panel_tile(tile, p.tilesM, p.tilesN, p.panel, tile_m, tile_n);
    const int rb0 = tile_m * RBT;
    const int cb0 = tile_n * 8 + wave * 2;
    const bool active = (cb0 * 32 < p.N) && (rb0 < p.nrb);
    const int C64 = p.C64, CQ = p.CQ;

    const uint32_t lane16 = (uint32_t)lane * 16u, lane4 = (uint32_t)lane * 4u;
    int rbs = rb0 + wave;  // row block staged by this wavefront
    rbs = rbs < p.nrb ? rbs : p.nrb - 1;
    const uint8_t* xq_base = p.xq + (size_t)rbs * C64 * 1024;
    const int cbw = (cb0 * 32 < p.N) ? cb0 : 0;  // wavefronts past the last column read block 0 (unused)
    const uint8_t* pq_base[2] = {p.pq + (size_t)cbw * C64 * 1024, p.pq + (size_t)(cbw + 1) * C64 * 1024};
    const uint8_t* pe_base[2] = {p.pe + (size_t)cbw * CQ * 256, p.pe + (size_t)(cbw + 1) * CQ * 256};
    const uint8_t* xe_base[4];
#pragma unroll
    for (int rbi = 0; rbi < 4; ++rbi) {
        int rb = rb0 + rbi;
        rb = rb < p.nrb ? rb : p.nrb - 1;
        xe_base[rbi] = p.xe + (size_t)rb * CQ * 256;
    }

    // Steps (and quads of steps) past the end are clamped instead of predicated: the loads stay
    // unconditional, what they fetch is never used.
    auto load_a = [&](v4i& a, int step) {
        const int st = step < C64 ? step : C64 - 1;
        a = *(const v4i*)(xq_base + (size_t)st * 1024 + lane16);
    };
    auto store_a = [&](const v4i& a, int buf) {
        const v8i e = mxi_expand8(a);
        uint8_t* base = lds + (size_t)((buf * RBT + wave) * 2048) + lane16;
        *(v4i*)(base) = v4i{e[0], e[1], e[2], e[3]};
        *(v4i*)(base + 1024) = v4i{e[4], e[5], e[6], e[7]};
    };
    struct BStage { v4i v[2]; };
    auto load_b = [&](BStage& b, int step) {
        const int st = step < C64 ? step : C64 - 1;
#pragma unroll
        for (int cbi = 0; cbi < 2; ++cbi) b.v[cbi] = *(const v4i*)(pq_base[cbi] + (size_t)st * 1024 + lane16);
    };
    struct Scales { int a[4]; int b[2]; };
    auto load_s = [&](Scales& sc, int quad) {
        const int q = quad < CQ ? quad : CQ - 1;
#pragma unroll
        for (int rbi = 0; rbi < 4; ++rbi) sc.a[rbi] = *(const int*)(xe_base[rbi] + (size_t)q * 256 + lane4);
#pragma unroll
        for (int cbi = 0; cbi < 2; ++cbi) sc.b[cbi] = *(const int*)(pe_base[cbi] + (size_t)q * 256 + lane4);
    };

    v16f t[4][2];
#pragma unroll
    for (int a = 0; a < 4; ++a)
#pragma unroll
        for (int b = 0; b < 2; ++b)
#pragma unroll
            for (int i = 0; i < 16; ++i) t[a][b][i] = 0.f;

    v8i bu[2][2];  // expanded weight operands: [step parity][column block]

    // One step = one 64-chunk.  On entry: LDS buffer s&1 holds the activation operands of step s,
    // bu[s&1] the weight operands of step s, `a`/`b` the packed data of step s+1.  During the step the
    // data of step s+1 is expanded (activations into the other LDS buffer, weights into bu[(s+1)&1])
    // and the loads of step s+3 are issued into `a`/`b`.  SEL = s % 4 picks the scale byte.
    auto do_step = [&](auto sel, int s, v4i& a, BStage& b, const Scales& sc) {
        constexpr int SEL = decltype(sel)::value;
        constexpr int PAR = SEL & 1;
        const int buf = PAR;
        auto lds_a = [&](int rbi) -> v8i {
            const uint8_t* base = lds + (size_t)((buf * RBT + rbi) * 2048) + lane16;
            const v4i lo = *(const v4i*)(base);
            const v4i hi = *(const v4i*)(base + 1024);
            return v8i{lo[0], lo[1], lo[2], lo[3], hi[0], hi[1], hi[2], hi[3]};
        };
        v8i af[2];
        af[0] = lds_a(0);
#pragma unroll
        for (int rbi = 0; rbi < 4; ++rbi) {
            if (rbi + 1 < 4) af[(rbi + 1) & 1] = lds_a(rbi + 1);
#pragma unroll
            for (int cbi = 0; cbi < 2; ++cbi)
                t[rbi][cbi] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(af[rbi & 1], bu[PAR][cbi], t[rbi][cbi], 0, 0, SEL,
                                                                             sc.a[rbi], SEL, sc.b[cbi]);
            if (rbi == 0) {
                store_a(a, buf ^ 1);
                load_a(a, s + 3);
            }
            if (rbi == 1) {
#pragma unroll
                for (int cbi = 0; cbi < 2; ++cbi) bu[PAR ^ 1][cbi] = mxi_expand8(b.v[cbi]);
                load_b(b, s + 3);
            }
        }
        __syncthreads();
    };

    v4i a0, a1;
    BStage b0, b1;
    Scales s0, s1;
    load_a(a0, 0);
    load_b(b0, 0);
    load_s(s0, 0);
    store_a(a0, 0);
#pragma unroll
    for (int cbi = 0; cbi < 2; ++cbi) bu[0][cbi] = mxi_expand8(b0.v[cbi]);
    __builtin_amdgcn_sched_barrier(0);
    load_a(a1, 1);
    load_b(b1, 1);
    load_a(a0, 2);
    load_b(b0, 2);
    load_s(s1, 1);
    __builtin_amdgcn_sched_barrier(0);
    __syncthreads();

    // steps in groups of eight (two quads of chunks): quad q uses scale set q & 1; step s uses the
    // register set s & 1 (a1/b1 hold step s+1 on entry to an even step)
    int s = 0;
    for (; s + 7 < C64; s += 8) {
        do_step(std::integral_constant<int, 0>{}, s, a1, b1, s0);
        do_step(std::integral_constant<int, 1>{}, s + 1, a0, b0, s0);
        do_step(std::integral_constant<int, 2>{}, s + 2, a1, b1, s0);
        do_step(std::integral_constant<int, 3>{}, s + 3, a0, b0, s0);
        load_s(s0, (s >> 2) + 2);
        do_step(std::integral_constant<int, 0>{}, s + 4, a1, b1, s1);
        do_step(std::integral_constant<int, 1>{}, s + 5, a0, b0, s1);
        do_step(std::integral_constant<int, 2>{}, s + 6, a1, b1, s1);
        do_step(std::integral_constant<int, 3>{}, s + 7, a0, b0, s1);
        load_s(s1, (s >> 2) + 3);
    }
    if (s < C64) do_step(std::integral_constant<int, 0>{}, s, a1, b1, s0);
    if (s + 1 < C64) do_step(std::integral_constant<int, 1>{}, s + 1, a0, b0, s0);
    if (s + 2 < C64) do_step(std::integral_constant<int, 2>{}, s + 2, a1, b1, s0);
    if (s + 3 < C64) do_step(std::integral_constant<int, 3>{}, s + 3, a0, b0, s0);
    if (s + 4 < C64) do_step(std::integral_constant<int, 0>{}, s + 4, a1, b1, s1);
    if (s + 5 < C64) do_step(std::integral_constant<int, 1>{}, s + 5, a0, b0, s1);
    if (s + 6 < C64) do_step(std::integral_constant<int, 2>{}, s + 6, a1, b1, s1);

    if (!active) return;

    // ---- rank-r expansion on the bf16 MFMA, accumulated on top of the main product --------------
#pragma unroll
    for (int ch = 0; ch < NK16; ++ch) {
        v4i lf[2];
#pragma unroll
        for (int cbi = 0; cbi < 2; ++cbi) lf[cbi] = *(const v4i*)(p.lv + ((size_t)((size_t)(cb0 + cbi) * NK16 + ch) * 64 + lane) * 16);
#pragma unroll
        for (int rbi = 0; rbi < 4; ++rbi) {
            int rb = rb0 + rbi;
            rb = rb < p.nrb ? rb : p.nrb - 1;
            const v4i tf = *(const v4i*)(p.tv + ((size_t)((size_t)rb * NK16 + ch) * 64 + lane) * 16);
#pragma unroll
            for (int cbi = 0; cbi < 2; ++cbi)
                t[rbi][cbi] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(v8bf, tf), __builtin_bit_cast(v8bf, lf[cbi]),
                                                                     t[rbi][cbi], 0, 0, 0);
        }
    }

    // ---- epilogue: bf16, transposed through the wavefront's own LDS slice, full-line stores ------
    typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
    typedef float f32x2 __attribute__((ext_vector_type(2)));
    uint8_t* stage = lds + wave * EPI_WAVE;
    const int wr_off = (4 * half) * EPI_ROW + l32 * 2;
    const int rd_row = lane >> 3, rd_seg = lane & 7;
    // The stores are buffer stores through a descriptor that ends with the wavefront's 128 bytes of the tile's last valid
    // row (rows past M are out of range and dropped by the hardware; without Y the descriptor is empty): no branch, so
    // the compiler can count the stores and need not wait for them when it waits for an older load.
    typedef unsigned int u4 __attribute__((ext_vector_type(4)));
    const int rows_valid = p.M - rb0 * 32 < 128 ? p.M - rb0 * 32 : 128;
    const bool have_y = !HO || p.Y;
    const __amdgpu_buffer_rsrc_t rs_y = __builtin_amdgcn_make_buffer_rsrc(
        have_y ? (void*)(p.Y + (size_t)(rb0 * 32) * p.ldy + cb0 * 32) : (void*)p.ho_xq, 0,
        have_y ? (int)((rows_valid - 1) * p.ldy * 2 + 128) : 0, 0x00020000);
    uint32_t yoff = (uint32_t)(rd_row * (int)p.ldy * 2 + rd_seg * 16);
    const uint32_t ystep = (uint32_t)(8 * (int)p.ldy * 2);
    v4i ov[4];
#pragma unroll
    for (int rbi = 0; rbi < 4; ++rbi) {
        const int rbase = (rb0 + rbi) * 32;
#pragma unroll
        for (int cbi = 0; cbi < 2; ++cbi) {
#pragma unroll
            for (int i = 0; i < 16; i += 2) {
                const bf16x2 h = __builtin_convertvector(f32x2{t[rbi][cbi][i], t[rbi][cbi][i + 1]}, bf16x2);
                const uint32_t w = __builtin_bit_cast(uint32_t, h);
                const int o = wr_off + (8 * (i >> 2) + (i & 3)) * EPI_ROW + cbi * 64;
                *(uint16_t*)(stage + o) = (uint16_t)(w & 0xFFFFu);
                *(uint16_t*)(stage + o + EPI_ROW) = (uint16_t)(w >> 16);
            }
            if (DBG) {
                const int col = (cb0 + cbi) * 32 + l32;
#pragma unroll
                for (int i = 0; i < 16; ++i) {
                    const int row = rbase + 8 * (i >> 2) + 4 * half + (i & 3);
                    if (row < p.M && p.dbg_y32) p.dbg_y32[(size_t)row * p.N + col] = t[rbi][cbi][i];
                }
            }
        }
#pragma unroll
        for (int q = 0; q < 4; ++q) ov[q] = *(const v4i*)(stage + (q * 8 + rd_row) * EPI_ROW + rd_seg * 16);
        if constexpr (HO) {
            // The lane holds 8 consecutive channels of one token as bf16; a block of 32 channels of the next layer's K
            // axis is the 4 lanes that differ in the two low lane bits.  Codes as in the activation kernel: shared
            // exponent from the block maximum, MXINT4 main codes (sign-magnitude nibbles), MXINT8 branch codes.
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const int row = rbase + q * 8 + rd_row;
                const uint32_t w[4] = {(uint32_t)ov[q][0], (uint32_t)ov[q][1], (uint32_t)ov[q][2], (uint32_t)ov[q][3]};
                us2 m2 = {0, 0};
#pragma unroll
                for (int d = 0; d < 4; ++d) m2 = __builtin_elementwise_max(m2, __builtin_bit_cast(us2, w[d] & 0x7FFF7FFFu));
                uint32_t mm = m2[0] > m2[1] ? m2[0] : m2[1];
                float am = __uint_as_float(mm << 16);
                am = fmaxf(am, __shfl_xor(am, 1, 64));
                am = fmaxf(am, __shfl_xor(am, 2, 64));
                const uint32_t field = exp_field(am);
                const float inv4 = field >= 2u ? __uint_as_float((256u - field) << 23) : 0.0f;   // 2^(2-s)
                const float to8 = field >= 7u ? __uint_as_float((260u - field) << 23) : 0.0f;    // 2^(6-s)
                // Both codes by one fused multiply-add each: scaling by a power of two is exact, so fma(x, 2^-step, magic)
                // rounds the scaled value to the nearest integer (ties to even) in one step -- the same integer the
                // activation kernel reaches by rounding on the block's grid and scaling afterwards -- and leaves it in
                // the low mantissa bits of the magic number.  Clamping after the rounding equals clamping before it.
                uint32_t sum = 0u - 0xFB000000u, c8[2];
                uint32_t ub[8];
#pragma unroll
                for (int e = 0; e < 8; ++e) {
                    const float x = __uint_as_float((e & 1) ? (w[e >> 1] & 0xFFFF0000u) : (w[e >> 1] << 16));
                    const uint32_t mb = __float_as_uint(fminf(__builtin_fmaf(fabsf(x), inv4, 8388608.0f), 8388615.0f));
                    const int sh = e < 4 ? 8 * e : 8 * ((e - 5) & 3) + 4;
                    sum += mb << sh;
                    // 1.5 * 2^23 + code, code in [-127, 127]: the low byte is the two's-complement MXINT8 code
                    ub[e] = __float_as_uint(__builtin_amdgcn_fmed3f(__builtin_fmaf(x, to8, 12582912.0f), 12582785.0f, 12583039.0f));
                }
#pragma unroll
                for (int h = 0; h < 2; ++h) {
                    const uint32_t lo = __builtin_amdgcn_perm(ub[4 * h + 1], ub[4 * h], 0x0c0c0400u);      // bytes 0 of two dwords
                    const uint32_t hi = __builtin_amdgcn_perm(ub[4 * h + 3], ub[4 * h + 2], 0x04000c0cu);  // ... in the upper half
                    c8[h] = lo | hi;
                }
                const uint32_t s03 = __builtin_amdgcn_perm(w[1], w[0], 0x07050301u);
                const uint32_t s47 = __builtin_amdgcn_perm(w[3], w[2], 0x07050301u);
                const uint32_t pk = sum | (s03 & 0x80808080u) | ((s47 >> 4) & 0x08080808u);
                if (row < p.nrb * 32) {
                    const int k0 = cb0 * 32 + rd_seg * 8;   // this layer's channel = the next layer's k
                    *(uint32_t*)(p.ho_xq + mxi_frag_offset(row, k0, p.ho_C64)) = pk;
                    *(uint2*)(p.ho_cb + (size_t)row * p.N + k0) = make_uint2(c8[0], c8[1]);
                    if ((rd_seg & 3) == 0) {
                        p.ho_xe[mxi_scale_offset(row, k0 >> 6, (k0 >> 5) & 1, p.ho_CQ)] = (uint8_t)(field + 7u);
                        p.ho_cbe[(size_t)row * (p.N >> 5) + (k0 >> 5)] = (uint8_t)field;
                        // padding chunks of the next layer's last quad: valid E8M0 bytes (2^0), written by the wavefront
                        // that owns the last real chunk
                        if ((k0 >> 6) == p.ho_C64 - 1)
                            for (int c = p.ho_C64; c < 4 * p.ho_CQ; ++c) p.ho_xe[mxi_scale_offset(row, c, (k0 >> 5) & 1, p.ho_CQ)] = (uint8_t)127;
                    }
                }
            }
        }
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            __builtin_amdgcn_raw_buffer_store_b128(__builtin_bit_cast(u4, ov[q]), rs_y, yoff, 0, 0);
            yoff += ystep;
        }
    }
}

template <int NK16>
static void mxi_fwd_launch(const MxiFwdParams& p, hipStream_t s)
{
    dim3 grid((unsigned)(p.tilesM * p.tilesN)), block(256);
    if (p.ho_xq)
        hipLaunchKernelGGL((mxi_fwd_kernel<NK16, false, true>), grid, block, 0, s, p);
    else if (p.dbg_y32)
        hipLaunchKernelGGL((mxi_fwd_kernel<NK16, true>), grid, block, 0, s, p);
    else
        hipLaunchKernelGGL((mxi_fwd_kernel<NK16, false>), grid, block, 0, s, p);
}

static hipError_t fwd_mxi_launches(const Dims& d, const uint8_t* packed, const uint8_t* act, int64_t M, uint16_t* Y, int64_t ldy,
                                   const lq_fwd_debug* dbg, const Dims* next, uint8_t* act_next, uint8_t* codes, hipStream_t s);

hipError_t launch_fwd_mxi(const Dims& d, const uint8_t* packed, const uint8_t* act, int64_t M, uint16_t* Y, int64_t ldy,
                          const lq_fwd_debug* dbg, hipStream_t s)
{
    return fwd_mxi_launches(d, packed, act, M, Y, ldy, dbg, nullptr, nullptr, nullptr, s);
}

// Forward with the quantized hand-off: `next` is the consuming layer (K = this layer's N), act_next its activation blob
// (main codes and scales are written here), codes the hand-off buffer of its branch codes.  Y may be null.
hipError_t launch_fwd_handoff_mxi(const Dims& d, const uint8_t* packed, const uint8_t* act, int64_t M, uint16_t* Y, int64_t ldy,
                                  const Dims& next, uint8_t* act_next, uint8_t* codes, hipStream_t s)
{
    return fwd_mxi_launches(d, packed, act, M, Y, ldy, nullptr, &next, act_next, codes, s);
}

size_t handoff_codes_bytes(const Dims& next, int64_t M)
{
    const int64_t Mp = (M + 31) / 32 * 32;
    return align256((size_t)Mp * next.K);
}
size_t handoff_total_bytes(const Dims& next, int64_t M)
{
    const int64_t Mp = (M + 31) / 32 * 32;
    return handoff_codes_bytes(next, M) + align256((size_t)Mp * (next.K / 32));
}

static hipError_t fwd_mxi_launches(const Dims& d, const uint8_t* packed, const uint8_t* act, int64_t M, uint16_t* Y, int64_t ldy,
                                   const lq_fwd_debug* dbg, const Dims* next, uint8_t* act_next, uint8_t* codes, hipStream_t s)
{
    const PackedLayout pl = packed_layout(d);
    const ActLayout al = act_layout(d, M);
    MxiFwdParams p;
    p.ho_xq = p.ho_xe = p.ho_cbe = nullptr;
    p.ho_cb = nullptr;
    p.ho_C64 = p.ho_CQ = 0;
    if (next) {
        const ActLayout an = act_layout(*next, M);
        p.ho_xq = act_next + an.off_xq;
        p.ho_xe = act_next + an.off_sx;
        p.ho_cb = (int8_t*)codes;
        p.ho_cbe = codes + handoff_codes_bytes(*next, M);
        p.ho_C64 = next->C64;
        p.ho_CQ = (next->C64 + 3) / 4;
        p.ho_tag = make_tag(*next, LQ_BLOB_ACT, M);
        p.ho_tag_dst = (uint32_t*)act_next;
    }
    p.xq = act + al.off_xq;
    p.xe = act + al.off_sx;
    p.tv = act + al.off_tq;
    p.pq = packed + pl.off_pq;
    p.pe = packed + pl.off_sw;
    p.lv = packed + pl.off_lq;
    p.Y = Y;
    p.ldy = ldy;
    p.M = (int)M;
    p.N = (int)d.N;
    p.C64 = d.C64;
    p.CQ = (d.C64 + 3) / 4;
    p.nrb = (int)(al.Mp / 32);
    p.tilesM = (p.nrb + 3) / 4;
    p.tilesN = (p.N + 255) / 256;
    p.panel = panel_width(p.tilesN, p.C64);
    p.dbg_y32 = dbg ? dbg->y32 : nullptr;
    switch (d.rp >> 4) {
        case 0: mxi_fwd_launch<0>(p, s); break;
        case 2: mxi_fwd_launch<2>(p, s); break;
        case 4: mxi_fwd_launch<4>(p, s); break;
        case 6: mxi_fwd_launch<6>(p, s); break;
        default: mxi_fwd_launch<8>(p, s); break;
    }
    return hipGetLastError();
}

}  // namespace lq

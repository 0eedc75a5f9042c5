// MXFP6e2 branch of the MX family (App. A.3: E2M3 elements, blocks of 32, E8M0 scale; the 6-bit rows of
// the mixed-precision tables, Section 4.3): offline packing of L and R, the plain views, and the
// activation kernel.  The main product (MXFP4) and the forward kernel are those of lq_mx.hip; only the
// element format of the four branch operands differs (the scaled MFMA takes FP6 at the FP4 rate).
//
// Block exponent: floor(log2 amax) - 2 (2 = largest E2M3 exponent, the same rule as for E2M1, so the main
// and the branch codes of an activation block share one scale byte); elements saturate at +-7.5; codes
// come from the hardware converters (round to nearest even), checked against the oracle's encoder.
#include "lq_internal.h"

namespace lq {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v8i __attribute__((ext_vector_type(8)));
typedef unsigned v6u __attribute__((ext_vector_type(6)));
typedef float v4f __attribute__((ext_vector_type(4)));
typedef float v16f __attribute__((ext_vector_type(16)));
typedef __bf16 v2bf __attribute__((ext_vector_type(2)));
typedef __bf16 v32bf __attribute__((ext_vector_type(32)));
typedef unsigned short us2 __attribute__((ext_vector_type(2)));

// layouts shared with lq_mx.hip (same formulas there)
__device__ __forceinline__ size_t m6_code_offset(int row, int k, int C64)  // dword holding main code (row, k)
{
    const int blk = row >> 5, c = k >> 6, half = (k & 63) >> 5, d = (k & 31) >> 3;
    return ((size_t)((size_t)blk * C64 + c) * 64 + (row & 31) + 32 * half) * 16 + d * 4;
}
__device__ __forceinline__ size_t m6_scale_offset(int row, int c, int half, int CQ)  // main scale byte of block (row, c, half)
{
    return ((size_t)((size_t)(row >> 5) * CQ + (c >> 2)) * 64 + (row & 31) + 32 * half) * 4 + (c & 3);
}
__device__ __forceinline__ size_t m6_lt_scale_offset(int row, int rb)  // scale byte (row, rank block rb) of le / te
{
    return ((size_t)(row >> 5) * 64 + (row & 31) + 32 * (rb & 1)) * 4 + (rb >> 1);
}
__device__ __forceinline__ size_t m6_re_offset(int j, int kb, int r)  // scale dword (rank row j, K block kb) of re
{
    return ((size_t)((size_t)(kb >> 2) * (r >> 4) + (j >> 4)) * 64 + (j & 15) + 16 * (kb & 3)) * 4;
}
__device__ __forceinline__ uint32_t m6_e8m0_of(float amax)  // floor(log2 amax) - 2 + 127, clamped at 0
{
    const int e = (int)((__float_as_uint(amax) >> 23) & 0xFFu) - 2;
    return (amax == 0.0f || e < 0) ? 0u : (uint32_t)e;
}
__device__ __forceinline__ float m6_e8m0_value(uint32_t E)  // 2^(E-127) as a float (E >= 1), 2^-127 for E = 0
{
    return E ? __uint_as_float(E << 23) : __uint_as_float(0x00400000u);
}

// 32 fp32 values -> 32 E2M3 codes (6 dwords).  The two-source converter interleaves its sources (result
// position 2j holds a[j], 2j+1 holds b[j]), so it is fed the even and the odd elements.
__device__ __forceinline__ v6u fp6_block_from_f32(const float* v, float sc)
{
    v16f a, b;
#pragma unroll
    for (int j = 0; j < 16; ++j) {
        a[j] = v[2 * j];
        b[j] = v[2 * j + 1];
    }
    const v6u c = __builtin_amdgcn_cvt_scalef32_2xpk16_fp6_f32(a, b, sc);
    // The converter writes its six result registers over several passes while still reading its sources,
    // and the register allocator is not told: without the sources being live past it, it has been seen
    // to place the result on top of the scale register (positions 0 and 1 right, the rest garbage).
    asm volatile("" : : "v"(a), "v"(b), "v"(sc));
    return c;
}
__device__ __forceinline__ v6u fp6_block_from_bf16(v32bf h, float sc)
{
    const v6u c = __builtin_amdgcn_cvt_scalef32_pk32_fp6_bf16(h, sc);
    asm volatile("" : : "v"(h), "v"(sc));  // as above
    return c;
}

// ---------------------------------------------------------------------------------------------
// offline packing of the factors: one thread per (row, block of 32)
// ---------------------------------------------------------------------------------------------
// (src_len: row length of the source; len: of the layout, a multiple of 128 for R: blocks past the source are zero)
__global__ __launch_bounds__(256) void mx6_pack_rows_kernel(const float* A, int rows, int len, int src_len, int mode, int r,
                                                            int rp, uint8_t* slots, uint8_t* scales)
{
    const int nb = len >> 5;
    const size_t idx = (size_t)blockIdx.x * 256 + threadIdx.x;
    if (idx >= (size_t)rows * nb) return;
    const int row = (int)(idx / nb), b = (int)(idx % nb);
    float v[32];
    float a = 0.f;
    for (int i = 0; i < 32; ++i) {
        v[i] = 32 * b < src_len ? A[(size_t)row * src_len + 32 * b + i] : 0.0f;
        a = fmaxf(a, fabsf(v[i]));
    }
    const uint32_t E = m6_e8m0_of(a);
    v6u c = {0u, 0u, 0u, 0u, 0u, 0u};
    if (a != 0.0f) c = fp6_block_from_f32(v, m6_e8m0_value(E));
    uint32_t* dst = (uint32_t*)(slots + (mode == 0 ? mx6_rq_slot(row, b, r) : mx6_lt_slot(row, b, rp)));
#pragma unroll
    for (int i = 0; i < 6; ++i) dst[i] = c[i];
    dst[6] = 0u;
    dst[7] = 0u;
    if (mode == 0)
        *(uint32_t*)(scales + m6_re_offset(row, b, r)) = 0x7F7F7F00u | E;
    else
        scales[m6_lt_scale_offset(row, b)] = (uint8_t)E;
}

hipError_t launch_pack_rows_mx6(const Dims& d, const float* L, const float* R, uint8_t* packed, hipStream_t s)
{
    const PackedLayout pl = packed_layout(d);
    if (d.r == 0) return hipSuccess;
    const int N = (int)d.N, K = (int)d.K;
    const size_t nr = (size_t)d.r * (K / 32), nl = (size_t)N * (d.r / 32);
    hipLaunchKernelGGL(mx6_pack_rows_kernel, dim3((unsigned)((nr + 255) / 256)), dim3(256), 0, s, R, d.r, K, (int)d.Ks, 0, d.r, d.rp,
                       packed + pl.off_rq, packed + pl.off_sr);
    hipLaunchKernelGGL(mx6_pack_rows_kernel, dim3((unsigned)((nl + 255) / 256)), dim3(256), 0, s, L, N, d.r, d.r, 1, d.r, d.rp,
                       packed + pl.off_lq, packed + pl.off_sl);
    return hipGetLastError();
}

// ---------------------------------------------------------------------------------------------
// plain views
// ---------------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void mx6_unpack_w_kernel(const uint8_t* packed, PackedLayout pl, int N, int K, int C64, int r,
                                                           int rp, lq_weights_view out)
{
    const size_t idx = (size_t)blockIdx.x * 256 + threadIdx.x;
    const int CQ = (C64 + 3) >> 2, B = K >> 5, BR = r >> 5;  // K: the caller's (views); C64: chunks of the layout
    if (idx < (size_t)N * K && out.pq) {
        const int n = (int)(idx / K), k = (int)(idx % K);
        const uint32_t w = *(const uint32_t*)(packed + pl.off_pq + m6_code_offset(n, k, C64));
        out.pq[idx] = (int8_t)((w >> (4 * (k & 7))) & 0xFu);
    }
    if (idx < (size_t)N * B && out.pe) {
        const int n = (int)(idx / B), b = (int)(idx % B);
        out.pe[idx] = packed[pl.off_sw + m6_scale_offset(n, b >> 1, b & 1, CQ)];
    }
    if (idx < (size_t)N * r && out.lq) {
        const int n = (int)(idx / r), j = (int)(idx % r);
        out.lq[idx] = (int8_t)fp6_get(packed + pl.off_lq + mx6_lt_slot(n, j >> 5, rp), j & 31);
    }
    if (idx < (size_t)N * BR && out.le) {
        const int n = (int)(idx / BR), b = (int)(idx % BR);
        out.le[idx] = packed[pl.off_sl + m6_lt_scale_offset(n, b)];
    }
    if (idx < (size_t)r * K && out.rq) {
        const int j = (int)(idx / K), k = (int)(idx % K);
        out.rq[idx] = (int8_t)fp6_get(packed + pl.off_rq + mx6_rq_slot(j, k >> 5, r), k & 31);
    }
    if (idx < (size_t)r * B && out.re) {
        const int j = (int)(idx / B), b = (int)(idx % B);
        out.re[idx] = packed[pl.off_sr + m6_re_offset(j, b, r)];
    }
}

hipError_t launch_unpack_weights_mx6(const Dims& d, const uint8_t* packed, const lq_weights_view* out, hipStream_t s)
{
    const PackedLayout pl = packed_layout(d);
    const size_t n = (size_t)(d.N > d.r ? d.N : d.r) * (d.Ks > d.r ? d.Ks : d.r);  // covers N x K, r x K and N x r
    hipLaunchKernelGGL(mx6_unpack_w_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, s, packed, pl, (int)d.N, (int)d.Ks,
                       d.C64, d.r, d.rp, *out);
    return hipGetLastError();
}

__global__ __launch_bounds__(256) void mx6_unpack_a_kernel(const uint8_t* act, ActLayout al, int M, int K, int C64, int r, int rp,
                                                           lq_act_view out)
{
    const size_t idx = (size_t)blockIdx.x * 256 + threadIdx.x;
    const int CQ = (C64 + 3) >> 2, B = K >> 5, BR = r >> 5;
    if (idx < (size_t)M * K && out.xq) {
        const int m = (int)(idx / K), k = (int)(idx % K);
        const uint32_t w = *(const uint32_t*)(act + al.off_xq + m6_code_offset(m, k, C64));
        out.xq[idx] = (int8_t)((w >> (4 * (k & 7))) & 0xFu);
    }
    if (idx < (size_t)M * B && out.xe) {
        const int m = (int)(idx / B), b = (int)(idx % B);
        out.xe[idx] = act[al.off_sx + m6_scale_offset(m, b >> 1, b & 1, CQ)];
    }
    if (idx < (size_t)M * r && out.tq) {
        const int m = (int)(idx / r), j = (int)(idx % r);
        out.tq[idx] = (int8_t)fp6_get(act + al.off_tq + mx6_lt_slot(m, j >> 5, rp), j & 31);
    }
    if (idx < (size_t)M * BR && out.te) {
        const int m = (int)(idx / BR), b = (int)(idx % BR);
        out.te[idx] = act[al.off_st + m6_lt_scale_offset(m, b)];
    }
}

hipError_t launch_unpack_act_mx6(const Dims& d, const uint8_t* act, int64_t M, const lq_act_view* out, hipStream_t s)
{
    const ActLayout al = act_layout(d, M);
    const size_t n = (size_t)M * (d.Ks > d.r ? d.Ks : d.r);
    hipLaunchKernelGGL(mx6_unpack_a_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, s, act, al, (int)M, (int)d.Ks,
                       d.C64, d.r, d.rp, *out);
    return hipGetLastError();
}

// ---------------------------------------------------------------------------------------------
// activation kernel.  16 token rows per workgroup; K is walked in chunks of 128 (= one
// v_mfma_scale_f32_16x16x128_f8f6f4), dealt round-robin to the 4 wavefronts; lane (row l%16, q = l/16)
// owns block q of the chunk: its 32 values are one lane's FP4 operand of the main product (16 bytes),
// one lane's FP6 operand of the skinny contraction (24 bytes), and share one scale byte, which the
// lane itself supplies to the instruction.  No scale spans more than a block, so the row is streamed.
// ---------------------------------------------------------------------------------------------
struct Mx6ActParams {
    const void* X;
    int64_t ldx;
    int M, K, C64, C64s, CQ, C128, r, rp;  // K, C64s: the caller's row length and its 64-chunks; C64, C128: of the layout
    const uint8_t* rs;   // R slots
    const uint8_t* re;   // R scale dwords
    uint8_t* xc;
    uint8_t* xe;
    uint8_t* ts;         // intermediate slots
    uint8_t* te;
    int8_t* dbg_xb;
    uint8_t* dbg_xbe;
    float* dbg_T;
    const float* rg;  // reciprocals of the smoothing vector (smoothing variant only)
    BlobTag tag;        // header of the activation blob (written by the first workgroup)
    uint32_t* tag_dst;
};

template <bool BF16>
struct Mx6Block;
template <>
struct Mx6Block<true> {  // 32 bf16 values = 16 dwords
    uint32_t w[16];
    __device__ __forceinline__ void load(const void* X, size_t elem, bool ok)
    {
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            v4i a = {0, 0, 0, 0};
            if (ok) a = ((const v4i*)((const uint16_t*)X + elem))[q];
            w[4 * q] = a[0]; w[4 * q + 1] = a[1]; w[4 * q + 2] = a[2]; w[4 * q + 3] = a[3];
        }
    }
    __device__ __forceinline__ float get(int i) const
    {
        return __uint_as_float((i & 1) ? (w[i >> 1] & 0xFFFF0000u) : (w[i >> 1] << 16));
    }
};
template <>
struct Mx6Block<false> {  // 32 fp32 values
    float v[32];
    __device__ __forceinline__ void load(const void* X, size_t elem, bool ok)
    {
#pragma unroll
        for (int q = 0; q < 8; ++q) {
            v4i a = {0, 0, 0, 0};
            if (ok) a = ((const v4i*)((const float*)X + elem))[q];
            v[4 * q] = __int_as_float(a[0]); v[4 * q + 1] = __int_as_float(a[1]);
            v[4 * q + 2] = __int_as_float(a[2]); v[4 * q + 3] = __int_as_float(a[3]);
        }
    }
    __device__ __forceinline__ float get(int i) const { return v[i]; }
};

// BF16IN: element type of X; SM: smoothing variant (X times the stored reciprocals, held as fp32).
template <bool BF16IN, int NJB, bool SM = false>
__global__ __launch_bounds__(256) void mx6_act_kernel(Mx6ActParams p)
{
    write_tag(p.tag_dst, p.tag);
    constexpr bool BF16 = BF16IN && !SM;  // representation of a block in registers
    constexpr int NJA = NJB > 0 ? NJB : 1;
    constexpr int PF = 2;  // 128-chunks in flight per wavefront
    __shared__ float s_acc[4][NJA][64][4];
    __shared__ float s_T[16][NJA * 16 + 1];

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int r16 = lane & 15, q = lane >> 4;
    const int row = blockIdx.x * 16 + r16;
    const bool row_ok = row < p.M;
    const int C128 = p.C128;
    const int nmy = (C128 - wave + 3) >> 2;  // chunks of this wavefront: c = wave + 4 * ci, ci < nmy

    Mx6Block<BF16> xb[PF];
    auto load_x = [&](Mx6Block<BF16>& blk, size_t koff, bool ok) {
        if constexpr (SM)
            smooth_load<BF16IN, 32>(blk.v, p.X, (size_t)row * p.ldx + koff, p.rg + koff, ok);
        else
            blk.load(p.X, (size_t)row * p.ldx + koff, ok);
    };
#pragma unroll
    for (int i = 0; i < PF; ++i) load_x(xb[i], (size_t)(wave + 4 * i) * 128 + q * 32, row_ok && 4 * (wave + 4 * i) + q < 2 * p.C64s);
    v8i bvs[2][NJA];
    int bss[2][NJA];
    auto load_r = [&](int slot, int ci) {
        int c = wave + 4 * ci;
        c = c < C128 ? c : C128 - 1;  // clamped: a fragment past the end is fetched but not used
#pragma unroll
        for (int jb = 0; jb < NJB; ++jb) {
            bvs[slot][jb] = *(const v8i*)(p.rs + ((size_t)((size_t)c * NJB + jb) * 64 + lane) * 32);
            bss[slot][jb] = *(const int*)(p.re + ((size_t)((size_t)c * NJB + jb) * 64 + lane) * 4);
        }
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
            load_r((sl + 1) & 1, ci + 1);
            if (ci < nmy) {  // wave-uniform
                const Mx6Block<BF16>& x = xb[sl];
                float m = 0.f;
                if constexpr (BF16) {
                    us2 m2 = {0, 0};
#pragma unroll
                    for (int d = 0; d < 16; ++d) m2 = __builtin_elementwise_max(m2, __builtin_bit_cast(us2, x.w[d] & 0x7FFF7FFFu));
                    const uint32_t mm = m2[0] > m2[1] ? m2[0] : m2[1];
                    m = __uint_as_float(mm << 16);
                } else {
#pragma unroll
                    for (int i = 0; i < 32; ++i) m = fmaxf(m, fabsf(x.get(i)));
                }
                const uint32_t E = m6_e8m0_of(m);
                const float sc = m6_e8m0_value(E);
                uint32_t pk[4] = {0u, 0u, 0u, 0u};
                v6u c6 = {0u, 0u, 0u, 0u, 0u, 0u};
                if (m != 0.0f) {
                    if constexpr (BF16) {
#define LQ_CVT4B(J) pk[(J) >> 2] = __builtin_amdgcn_cvt_scalef32_pk_fp4_bf16(pk[(J) >> 2], __builtin_bit_cast(v2bf, x.w[J]), sc, (J) & 3)
                        LQ_CVT4B(0); LQ_CVT4B(1); LQ_CVT4B(2); LQ_CVT4B(3); LQ_CVT4B(4); LQ_CVT4B(5); LQ_CVT4B(6); LQ_CVT4B(7);
                        LQ_CVT4B(8); LQ_CVT4B(9); LQ_CVT4B(10); LQ_CVT4B(11); LQ_CVT4B(12); LQ_CVT4B(13); LQ_CVT4B(14); LQ_CVT4B(15);
#undef LQ_CVT4B
                        v32bf h;
#pragma unroll
                        for (int j = 0; j < 16; ++j) {
                            const v2bf two = __builtin_bit_cast(v2bf, x.w[j]);
                            h[2 * j] = two[0];
                            h[2 * j + 1] = two[1];
                        }
                        c6 = fp6_block_from_bf16(h, sc);
                    } else {
#define LQ_CVT4F(J) pk[(J) >> 2] = __builtin_amdgcn_cvt_scalef32_pk_fp4_f32(pk[(J) >> 2], x.get(2 * (J)), x.get(2 * (J) + 1), sc, (J) & 3)
                        LQ_CVT4F(0); LQ_CVT4F(1); LQ_CVT4F(2); LQ_CVT4F(3); LQ_CVT4F(4); LQ_CVT4F(5); LQ_CVT4F(6); LQ_CVT4F(7);
                        LQ_CVT4F(8); LQ_CVT4F(9); LQ_CVT4F(10); LQ_CVT4F(11); LQ_CVT4F(12); LQ_CVT4F(13); LQ_CVT4F(14); LQ_CVT4F(15);
#undef LQ_CVT4F
                        c6 = fp6_block_from_f32(x.v, sc);
                    }
                }
                // the lane's block is K block q&1 of 64-chunk 2c + (q>>1)
                const int c64 = 2 * c + (q >> 1);
                uint8_t* dst = p.xc + ((size_t)((size_t)(row >> 5) * p.C64 + c64) * 64 + (row & 31) + 32 * (q & 1)) * 16;
                *(v4i*)dst = v4i{(int)pk[0], (int)pk[1], (int)pk[2], (int)pk[3]};
                p.xe[m6_scale_offset(row, c64, q & 1, p.CQ)] = (uint8_t)E;
                if (NJB > 0) {
                    if (p.dbg_xb && row_ok && c64 < p.C64s) {
                        uint32_t cw[8] = {c6[0], c6[1], c6[2], c6[3], c6[4], c6[5], 0u, 0u};
                        int8_t* o = p.dbg_xb + (size_t)row * p.K + (size_t)c * 128 + q * 32;
                        for (int i = 0; i < 32; ++i) o[i] = (int8_t)fp6_get((const uint8_t*)cw, i);
                    }
                    if (p.dbg_xbe && row_ok && c64 < p.C64s) p.dbg_xbe[(size_t)row * (p.K >> 5) + 4 * c + q] = (uint8_t)E;
                    const v8i a8 = {(int)c6[0], (int)c6[1], (int)c6[2], (int)c6[3], (int)c6[4], (int)c6[5], 0, 0};
#pragma unroll
                    for (int jb = 0; jb < NJB; ++jb)
                        acc[jb] = __builtin_amdgcn_mfma_scale_f32_16x16x128_f8f6f4(a8, bvs[sl & 1][jb], acc[jb], 2, 2, 0, (int)E, 0,
                                                                                bss[sl & 1][jb]);
                }
            }
            load_x(xb[sl], (size_t)(c + 4 * PF) * 128 + q * 32, row_ok && 4 * (c + 4 * PF) + q < 2 * p.C64s);
        }
    }
    {   // padding 64-chunks of the last quad (at most one 128-chunk per wavefront): valid E8M0 bytes (2^0)
        const int c = wave + 4 * nmy;
        if (2 * c < 4 * p.CQ) p.xe[m6_scale_offset(row, 2 * c + (q >> 1), q & 1, p.CQ)] = (uint8_t)127;
    }
    if (NJB == 0) return;

#pragma unroll
    for (int jb = 0; jb < NJB; ++jb) *(v4f*)&s_acc[wave][jb][lane][0] = acc[jb];
    __syncthreads();
    if (wave == 0) {
        // lane holds column j = jb*16 + lane%16 of the intermediate for token rows 4*q + i
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
                s_T[4 * q + i][jb * 16 + r16] = sum[i];
                const int grow = blockIdx.x * 16 + 4 * q + i;
                if (grow < p.M && p.dbg_T) p.dbg_T[(size_t)grow * p.r + jb * 16 + r16] = sum[i];
            }
        }
    }
    __syncthreads();
    // re-quantise: one thread per (token row, block of 32 along the rank); blocks that pad the rank to a
    // multiple of 64 get zero codes and scale 2^0
    const int BRP = p.rp >> 5, BR = p.r >> 5;
    if (tid < 16 * BRP) {
        const int trow = tid / BRP, blk = tid % BRP;
        const int grow = blockIdx.x * 16 + trow;
        float v[32];
        float a = 0.f;
        v6u c6 = {0u, 0u, 0u, 0u, 0u, 0u};
        uint32_t E = 127u;
        if (blk < BR) {
            for (int i = 0; i < 32; ++i) {
                v[i] = s_T[trow][32 * blk + i];
                a = fmaxf(a, fabsf(v[i]));
            }
            E = m6_e8m0_of(a);
            if (a != 0.0f) c6 = fp6_block_from_f32(v, m6_e8m0_value(E));
        }
        uint32_t* dst = (uint32_t*)(p.ts + mx6_lt_slot(grow, blk, p.rp));
#pragma unroll
        for (int i = 0; i < 6; ++i) dst[i] = c6[i];
        dst[6] = 0u;
        dst[7] = 0u;
        p.te[m6_lt_scale_offset(grow, blk)] = (uint8_t)E;
    }
}

template <bool BF16, int NJB, bool SM>
static hipError_t mx6_act_launch(const Mx6ActParams& p, int64_t Mp, hipStream_t s)
{
    hipLaunchKernelGGL((mx6_act_kernel<BF16, NJB, SM>), dim3((unsigned)(Mp / 16)), dim3(256), 0, s, p);
    return hipGetLastError();
}
template <bool BF16, bool SM>
static hipError_t mx6_act_rank2(const Mx6ActParams& p, int64_t Mp, hipStream_t s)
{
    switch (p.r) {
        case 0: return mx6_act_launch<BF16, 0, SM>(p, Mp, s);
        case 32: return mx6_act_launch<BF16, 2, SM>(p, Mp, s);
        case 64: return mx6_act_launch<BF16, 4, SM>(p, Mp, s);
        case 96: return mx6_act_launch<BF16, 6, SM>(p, Mp, s);
        default: return mx6_act_launch<BF16, 8, SM>(p, Mp, s);
    }
}
template <bool BF16>
static hipError_t mx6_act_rank(const Mx6ActParams& p, int64_t Mp, hipStream_t s)
{
    return p.rg ? mx6_act_rank2<BF16, true>(p, Mp, s) : mx6_act_rank2<BF16, false>(p, Mp, s);
}

hipError_t launch_quantize_act_mx6(const Dims& d, int x_dtype, const uint8_t* packed, const void* X, int64_t M,
                                   int64_t ldx, uint8_t* act, const lq_act_debug* dbg, hipStream_t s)
{
    const PackedLayout pl = packed_layout(d);
    const ActLayout al = act_layout(d, M);
    Mx6ActParams p;
    p.tag = make_tag(d, LQ_BLOB_ACT, M);
    p.tag_dst = (uint32_t*)act;
    p.X = X;
    p.ldx = ldx;
    p.M = (int)M;
    p.K = (int)d.Ks;
    p.C64 = d.C64;
    p.C64s = (int)(d.Ks / 64);
    p.CQ = (d.C64 + 3) / 4;
    p.C128 = d.C64 / 2;
    p.r = d.r;
    p.rp = d.rp;
    p.rs = packed + pl.off_rq;
    p.re = packed + pl.off_sr;
    p.xc = act + al.off_xq;
    p.xe = act + al.off_sx;
    p.ts = act + al.off_tq;
    p.te = act + al.off_st;
    p.dbg_xb = dbg ? dbg->xb : nullptr;
    p.dbg_xbe = dbg ? dbg->xbe : nullptr;
    p.dbg_T = dbg ? dbg->T : nullptr;
    p.rg = d.smooth ? (const float*)(packed + pl.off_rg) : nullptr;
    return x_dtype == LQ_BF16 ? mx6_act_rank<true>(p, al.Mp, s) : mx6_act_rank<false>(p, al.Mp, s);
}

}  // namespace lq

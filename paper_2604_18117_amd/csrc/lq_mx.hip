// MX family (App. A.3 "MX Formats"): main product in MXFP4 (E2M1 elements, blocks of 32 along K,
// E8M0 power-of-two scale) on v_mfma_scale_f32_32x32x64_f8f6f4 -- the hardware applies both block
// scales, so there is no vector-ALU dequantisation at all -- and the low-rank branch in FP8 E4M3
// with one fp32 scale per token / per row of L, R (Fig. 1, Eq. 5).
//
//   pack      : Q2(R), Q2(L) -> E4M3;  P = W - deq(Q2 L) deq(Q2 R) (fp64 chain, one rounding);
//               Q1(P) -> E2M1 + E8M0 per 32 values
//   act       : Q1(X) -> E2M1 + E8M0;  Q2(X) -> E4M3 (registers only);  T = (X8 . R8^T * sxb) * sr;
//               Q2(T) -> E4M3 + st
//   forward   : t = sum_blocks 2^(ex+ew) (x . p)  [scaled MFMA, fp32 accumulate];
//               y = t + (tq8 . l8^T * st) * sl;  Y = bf16_rne(y)
//
// Block scale exponent = (exponent field of the block amax) - 2, i.e. floor(log2 amax) - 2; elements
// are converted by v_cvt_scalef32_pk_fp4_f32 (nearest even, saturating at +-6) and
// v_cvt_pk_fp8_f32 (nearest even; inputs are clamped to +-448 first because the instruction
// returns NaN, not 448, above 464).
#include <type_traits>

#include "lq_internal.h"

namespace lq {

typedef int v2i __attribute__((ext_vector_type(2)));
typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v8i __attribute__((ext_vector_type(8)));
typedef float v4f __attribute__((ext_vector_type(4)));
typedef float v16f __attribute__((ext_vector_type(16)));
typedef unsigned short us2 __attribute__((ext_vector_type(2)));

// ---------------------------------------------------------------------------------------------
// shared device helpers
// ---------------------------------------------------------------------------------------------
__device__ __forceinline__ size_t mx_code_offset(int row, int k, int C64)  // dword holding code (row,k)
{
    const int blk = row >> 5, c = k >> 6, half = (k & 63) >> 5, d = (k & 31) >> 3;
    return ((size_t)((size_t)blk * C64 + c) * 64 + (row & 31) + 32 * half) * 16 + d * 4;
}
__device__ __forceinline__ size_t mx_scale_offset(int row, int c, int half, int CQ)  // byte of block (row, c, half)
{
    return ((size_t)((size_t)(row >> 5) * CQ + (c >> 2)) * 64 + (row & 31) + 32 * half) * 4 + (c & 3);
}
__device__ __forceinline__ size_t mx_rq_offset(int j, int k, int r)
{
    const int c = k >> 6, kq = (k & 63) >> 4;
    return ((size_t)((size_t)c * (r >> 4) + (j >> 4)) * 64 + (j & 15) + 16 * kq) * 16 + (k & 15);
}
__device__ __forceinline__ uint32_t e8m0_of(float amax)  // floor(log2 amax) - 2 + 127, clamped at 0
{
    const int e = (int)((__float_as_uint(amax) >> 23) & 0xFFu) - 2;
    return (amax == 0.0f || e < 0) ? 0u : (uint32_t)e;
}
__device__ __forceinline__ float e8m0_value(uint32_t E)  // 2^(E-127) as a float (E >= 1), 2^-127 for E = 0
{
    return E ? __uint_as_float(E << 23) : __uint_as_float(0x00400000u);
}
__device__ __forceinline__ uint32_t fp8_byte(float u)  // E4M3, nearest even, saturating
{
    u = fminf(fmaxf(u, -448.0f), 448.0f);
    return (uint32_t)__builtin_amdgcn_cvt_pk_fp8_f32(u, u, 0, false) & 0xFFu;
}
__device__ __forceinline__ uint32_t fp8_pair(float u0, float u1)  // two E4M3 bytes in the low half
{
    u0 = fminf(fmaxf(u0, -448.0f), 448.0f);
    u1 = fminf(fmaxf(u1, -448.0f), 448.0f);
    return (uint32_t)__builtin_amdgcn_cvt_pk_fp8_f32(u0, u1, 0, false) & 0xFFFFu;
}
// four E4M3 bytes from four in-range-or-not values: one median (saturation) and half a convert each
__device__ __forceinline__ uint32_t fp8_quad(float u0, float u1, float u2, float u3)
{
    u0 = __builtin_amdgcn_fmed3f(u0, -448.0f, 448.0f);
    u1 = __builtin_amdgcn_fmed3f(u1, -448.0f, 448.0f);
    u2 = __builtin_amdgcn_fmed3f(u2, -448.0f, 448.0f);
    u3 = __builtin_amdgcn_fmed3f(u3, -448.0f, 448.0f);
    const int lo = __builtin_amdgcn_cvt_pk_fp8_f32(u0, u1, 0, false);
    return (uint32_t)__builtin_amdgcn_cvt_pk_fp8_f32(u2, u3, lo, true);
}
__device__ __forceinline__ float fp8_value(uint32_t byte) { return __builtin_amdgcn_cvt_f32_fp8((int)byte, 0); }
__device__ __forceinline__ void fp8_scales(float amax, float* s, float* inv)
{
    if (amax == 0.0f) {
        *s = 1.0f;
        *inv = 1.0f;
    } else {
        *s = amax / 448.0f;
        *inv = 448.0f / amax;
    }
}
// ---- MXFP8e4 branch (block-scaled E4M3): operand layouts of the 8-bit scaled MFMA forms ----
__device__ __forceinline__ size_t mxb_frag8_offset(int row, int j, int rp)  // byte (row, rank index j) of lq / tq
{
    const int blk = row >> 5, cc = j >> 6, jj = j & 63;
    const int h = (jj & 31) >> 4, byte = (jj & 15) + ((jj >> 5) << 4);
    return ((size_t)((size_t)blk * (rp >> 6) + cc) * 64 + (row & 31) + 32 * h) * 32 + byte;
}
__device__ __forceinline__ size_t mxb_scale_offset(int row, int rb)  // scale byte (row, rank block rb) of le / te
{
    return ((size_t)(row >> 5) * 64 + (row & 31) + 32 * (rb & 1)) * 4 + (rb >> 1);
}
__device__ __forceinline__ size_t mxb_rq_offset(int j, int k, int r)  // byte (rank row j, k) of rq
{
    const int c = k >> 7, kk = k & 127;
    const int q = (kk & 63) >> 4, byte = (kk & 15) + ((kk >> 6) << 4);
    return ((size_t)((size_t)c * (r >> 4) + (j >> 4)) * 64 + (j & 15) + 16 * q) * 32 + byte;
}
__device__ __forceinline__ size_t mxb_re_offset(int j, int kb, int r)  // scale dword (rank row j, K block kb) of re
{
    return ((size_t)((size_t)(kb >> 2) * (r >> 4) + (j >> 4)) * 64 + (j & 15) + 16 * (kb & 3)) * 4;
}
__device__ __forceinline__ uint32_t e8m0_of_fp8(float amax)  // floor(log2 amax) - 8 + 127, clamped at 0
{
    const int e = (int)((__float_as_uint(amax) >> 23) & 0xFFu) - 8;
    return (amax == 0.0f || e < 0) ? 0u : (uint32_t)e;
}
__device__ __forceinline__ float e8m0_inverse(uint32_t E)  // 2^(127-E), exact (E <= 253)
{
    return __uint_as_float((254u - E) << 23);
}
__device__ __forceinline__ double e8m0_double(uint32_t E) { return __builtin_ldexp(1.0, (int)E - 127); }

__device__ __forceinline__ float wmax64(float v)
{
#pragma unroll
    for (int o = 32; o >= 1; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, 64));
    return v;
}

// ---------------------------------------------------------------------------------------------
// pack
// ---------------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void mx_fill_kernel(uint8_t* p, size_t n, uint8_t v)
{
    const size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
    if (i < n) p[i] = v;
}

// Ks: row length of the source; K: row length of the layout (Ks rounded up to 128, the rest zero codes)
__global__ __launch_bounds__(256) void mx_pack_r_kernel(const float* R, int Ks, int K, int r, uint8_t* r8, float* sr)
{
    __shared__ float red[4];
    const int j = blockIdx.x, tid = threadIdx.x;
    float a = 0.f;
    for (int k = tid; k < Ks; k += 256) a = fmaxf(a, fabsf(R[(size_t)j * Ks + k]));
    a = wmax64(a);
    if ((tid & 63) == 0) red[tid >> 6] = a;
    __syncthreads();
    a = fmaxf(fmaxf(red[0], red[1]), fmaxf(red[2], red[3]));
    float s, inv;
    fp8_scales(a, &s, &inv);
    if (tid == 0) sr[j] = s;
    for (int k = tid; k < K; k += 256)
        r8[mx_rq_offset(j, k, r)] = k < Ks ? (uint8_t)fp8_byte(__fmul_rn(R[(size_t)j * Ks + k], inv)) : (uint8_t)0;
}

__global__ __launch_bounds__(256) void mx_pack_l_kernel(const float* L, int N, int r, int rp, uint8_t* l8, float* sl)
{
    const int n = blockIdx.x * 256 + threadIdx.x;
    if (n >= N) return;
    float a = 0.f;
    for (int j = 0; j < r; ++j) a = fmaxf(a, fabsf(L[(size_t)n * r + j]));
    float s, inv;
    fp8_scales(a, &s, &inv);
    sl[n] = s;
    for (int j = 0; j < rp; ++j)
        l8[(size_t)n * rp + j] = (j < r) ? (uint8_t)fp8_byte(__fmul_rn(L[(size_t)n * r + j], inv)) : (uint8_t)0;
}

// MXFP8e4 factors: one thread per (row, block of 32).  mode 0: rows of R, blocks along K, into the
// activation kernel's operand order; mode 1: rows of L, blocks along the rank, into the forward's.
// (src_len: row length of the source; len: of the layout, a multiple of 128 for R: blocks past the source are zero)
__global__ __launch_bounds__(256) void mxb_pack_rows_kernel(const float* A, int rows, int len, int src_len, int mode, int r,
                                                            int rp, uint8_t* codes, uint8_t* scales)
{
    const int nb = len >> 5;
    const size_t idx = (size_t)blockIdx.x * 256 + threadIdx.x;
    if (idx >= (size_t)rows * nb) return;
    const int row = (int)(idx / nb), b = (int)(idx % nb);
    const bool in_src = 32 * b < src_len;
    const float* v = A + (size_t)row * src_len + 32 * b;
    float a = 0.f;
    if (in_src)
        for (int i = 0; i < 32; ++i) a = fmaxf(a, fabsf(v[i]));
    const uint32_t E = e8m0_of_fp8(a);
    const float inv = e8m0_inverse(E);
    for (int i = 0; i < 32; ++i) {
        const uint8_t c = in_src ? (uint8_t)fp8_byte(__fmul_rn(v[i], inv)) : (uint8_t)0;
        if (mode == 0)
            codes[mxb_rq_offset(row, 32 * b + i, r)] = c;
        else
            codes[mxb_frag8_offset(row, 32 * b + i, rp)] = c;
    }
    if (mode == 0)
        *(uint32_t*)(scales + mxb_re_offset(row, b, r)) = 0x7F7F7F00u | E;
    else
        scales[mxb_scale_offset(row, b)] = (uint8_t)E;
}

// one wavefront per (n, 64-chunk): lane = k % 64, two blocks of 32.  from_q: 0 = unquantised factors,
// 1 = E4M3 codes with fp32 row scales, 2 = MXFP8e4 codes with E8M0 block scales (sl, sr hold le, re).
__global__ __launch_bounds__(256) void mx_pack_p_kernel(const float* W, const float* L, const float* R, int N, int Ks, int K,
                                                        int r, int rp, int from_q, const uint8_t* l8, const float* sl,
                                                        const uint8_t* r8, const float* sr, uint8_t* pc, uint8_t* pe)
{
    const int lane = threadIdx.x & 63;
    const int C64 = K >> 6, CQ = (C64 + 3) >> 2;  // layout chunks; a chunk past the source row (k >= Ks) is all zero
    const size_t wid = (size_t)blockIdx.x * 4 + (threadIdx.x >> 6);
    if (wid >= (size_t)N * C64) return;
    const int n = (int)(wid / C64), c = (int)(wid % C64);
    const int k = c * 64 + lane;
    double d = 0.0;
    const int rr = k < Ks ? r : 0;
    for (int j = 0; j < rr; ++j) {
        if (from_q == 3) {  // MXFP6e2 factors
            const uint8_t* le = (const uint8_t*)sl;
            const uint8_t* re = (const uint8_t*)sr;
            const double lh = (double)e2m3_value(fp6_get(l8 + mx6_lt_slot(n, j >> 5, rp), j & 31)) * e8m0_double(le[mxb_scale_offset(n, j >> 5)]);
            const double rh = (double)e2m3_value(fp6_get(r8 + mx6_rq_slot(j, k >> 5, r), k & 31)) * e8m0_double(re[mxb_re_offset(j, k >> 5, r)]);
            d = fma(lh, rh, d);
            continue;
        }
        if (from_q == 2) {  // element * 2^e is exact in fp64, and so is the product of two of them
            const uint8_t* le = (const uint8_t*)sl;
            const uint8_t* re = (const uint8_t*)sr;
            const double lh = (double)fp8_value(l8[mxb_frag8_offset(n, j, rp)]) * e8m0_double(le[mxb_scale_offset(n, j >> 5)]);
            const double rh = (double)fp8_value(r8[mxb_rq_offset(j, k, r)]) * e8m0_double(re[mxb_re_offset(j, k >> 5, r)]);
            d = fma(lh, rh, d);
            continue;
        }
        float lh, rh;
        if (from_q) {
            lh = __fmul_rn(fp8_value(l8[(size_t)n * rp + j]), sl[n]);
            rh = __fmul_rn(fp8_value(r8[mx_rq_offset(j, k, r)]), sr[j]);
        } else {
            lh = L[(size_t)n * r + j];
            rh = R[(size_t)j * Ks + k];
        }
        d = fma((double)lh, (double)rh, d);
    }
    const float P = k < Ks ? (float)((double)W[(size_t)n * Ks + k] - d) : 0.0f;
    float a = fabsf(P);
#pragma unroll
    for (int o = 16; o >= 1; o >>= 1) a = fmaxf(a, __shfl_xor(a, o, 64));  // amax of the 32-block (half wave)
    const uint32_t E = e8m0_of(a);
    uint32_t code = 0;
    if (a != 0.0f) code = __builtin_amdgcn_cvt_scalef32_pk_fp4_f32(0u, P, 0.0f, e8m0_value(E), 0) & 0xFu;
    uint32_t w = code << (4 * (lane & 7));
    w |= __shfl_xor(w, 1, 64);
    w |= __shfl_xor(w, 2, 64);
    w |= __shfl_xor(w, 4, 64);
    if ((lane & 7) == 0) *(uint32_t*)(pc + mx_code_offset(n, k, C64)) = w;
    if ((lane & 31) == 0) pe[mx_scale_offset(n, c, lane >> 5, CQ)] = (uint8_t)E;
}

hipError_t launch_pack_mx(const Dims& d, int from_q, const float* W, const float* L, const float* R, uint8_t* packed,
                          hipStream_t s)
{
    const PackedLayout pl = packed_layout(d);
    uint8_t* l8 = packed + pl.off_lq;
    float* sl = (float*)(packed + pl.off_sl);
    uint8_t* r8 = packed + pl.off_rq;
    float* sr = (float*)(packed + pl.off_sr);
    const int N = (int)d.N, K = (int)d.K, Ks = (int)d.Ks;
    const size_t pe_bytes = (size_t)(N / 32) * ((d.C64 + 3) / 4) * 256;
    hipLaunchKernelGGL(mx_fill_kernel, dim3((unsigned)((pe_bytes + 255) / 256)), dim3(256), 0, s, packed + pl.off_sw,
                       pe_bytes, (uint8_t)127);
    if (d.smooth) {  // reciprocals of the smoothing vector start at 1
        const hipError_t e = launch_set_smoothing(d, nullptr, packed, s);
        if (e != hipSuccess) return e;
    }
    if (d.mxb) {
        // padding of the rank to 64: zero codes, scale 2^0
        const size_t lq_bytes = (size_t)N * d.rp, le_bytes = (size_t)N * 8;
        if (lq_bytes) hipLaunchKernelGGL(mx_fill_kernel, dim3((unsigned)((lq_bytes + 255) / 256)), dim3(256), 0, s, l8, lq_bytes, (uint8_t)0);
        hipLaunchKernelGGL(mx_fill_kernel, dim3((unsigned)((le_bytes + 255) / 256)), dim3(256), 0, s, (uint8_t*)sl, le_bytes, (uint8_t)127);
        if (d.r > 0 && d.mxb_elem == 6) {
            const hipError_t e = launch_pack_rows_mx6(d, L, R, packed, s);
            if (e != hipSuccess) return e;
        } else if (d.r > 0) {
            const size_t nr = (size_t)d.r * (K / 32), nl = (size_t)N * (d.r / 32);
            hipLaunchKernelGGL(mxb_pack_rows_kernel, dim3((unsigned)((nr + 255) / 256)), dim3(256), 0, s, R, d.r, K, Ks, 0, d.r, d.rp, r8, (uint8_t*)sr);
            hipLaunchKernelGGL(mxb_pack_rows_kernel, dim3((unsigned)((nl + 255) / 256)), dim3(256), 0, s, L, N, d.r, d.r, 1, d.r, d.rp, l8, (uint8_t*)sl);
        }
    } else {
        if (d.r > 0) hipLaunchKernelGGL(mx_pack_r_kernel, dim3(d.r), dim3(256), 0, s, R, Ks, K, d.r, r8, sr);
        hipLaunchKernelGGL(mx_pack_l_kernel, dim3((N + 255) / 256), dim3(256), 0, s, d.r > 0 ? L : (const float*)nullptr, N,
                           d.r, d.rp, l8, sl);
    }
    const size_t waves = (size_t)N * d.C64;
    hipLaunchKernelGGL(mx_pack_p_kernel, dim3((unsigned)((waves + 3) / 4)), dim3(256), 0, s, W, L, R, N, Ks, K, d.r, d.rp,
                       (from_q && d.mxb) ? (d.mxb_elem == 6 ? 3 : 2) : from_q, l8, sl, r8, sr, packed + pl.off_pq, packed + pl.off_sw);
    return hipGetLastError();
}

// ---------------------------------------------------------------------------------------------
// plain views
// ---------------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void mx_unpack_w_kernel(const uint8_t* packed, PackedLayout pl, int N, int K, int C64, int r,
                                                          int rp, int mxb, lq_weights_view out)
{
    const size_t idx = (size_t)blockIdx.x * 256 + threadIdx.x;
    const int CQ = (C64 + 3) >> 2, B = K >> 5;  // K: the caller's (views); C64: chunks of the layout
    if (idx < (size_t)N * K && out.pq) {
        const int n = (int)(idx / K), k = (int)(idx % K);
        const uint32_t w = *(const uint32_t*)(packed + pl.off_pq + mx_code_offset(n, k, C64));
        out.pq[idx] = (int8_t)((w >> (4 * (k & 7))) & 0xFu);
    }
    if (idx < (size_t)N * B && out.pe) {
        const int n = (int)(idx / B), b = (int)(idx % B);
        out.pe[idx] = packed[pl.off_sw + mx_scale_offset(n, b >> 1, b & 1, CQ)];
    }
    if (idx < (size_t)N * r && out.lq) {
        const int n = (int)(idx / r), j = (int)(idx % r);
        out.lq[idx] = (int8_t)packed[pl.off_lq + (mxb ? mxb_frag8_offset(n, j, rp) : (size_t)n * rp + j)];
    }
    if (idx < (size_t)r * K && out.rq) {
        const int j = (int)(idx / K), k = (int)(idx % K);
        out.rq[idx] = (int8_t)packed[pl.off_rq + (mxb ? mxb_rq_offset(j, k, r) : mx_rq_offset(j, k, r))];
    }
    if (mxb) {
        if (idx < (size_t)N * (r >> 5) && out.le) {
            const int n = (int)(idx / (r >> 5)), b = (int)(idx % (r >> 5));
            out.le[idx] = packed[pl.off_sl + mxb_scale_offset(n, b)];
        }
        if (idx < (size_t)r * B && out.re) {
            const int j = (int)(idx / B), b = (int)(idx % B);
            out.re[idx] = packed[pl.off_sr + mxb_re_offset(j, b, r)];
        }
    } else {
        if (idx < (size_t)N && out.sl) out.sl[idx] = ((const float*)(packed + pl.off_sl))[idx];
        if (idx < (size_t)r && out.sr) out.sr[idx] = ((const float*)(packed + pl.off_sr))[idx];
    }
}

hipError_t launch_unpack_weights_mx(const Dims& d, const uint8_t* packed, const lq_weights_view* out, hipStream_t s)
{
    if (d.mxb_elem == 6) return launch_unpack_weights_mx6(d, packed, out, s);
    const PackedLayout pl = packed_layout(d);
    const size_t n = (size_t)(d.N > d.r ? d.N : d.r) * (d.Ks > d.r ? d.Ks : d.r);  // covers N x K, r x K and N x r
    hipLaunchKernelGGL(mx_unpack_w_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, s, packed, pl, (int)d.N,
                       (int)d.Ks, d.C64, d.r, d.rp, d.mxb ? 1 : 0, *out);
    return hipGetLastError();
}

__global__ __launch_bounds__(256) void mx_unpack_a_kernel(const uint8_t* act, ActLayout al, int M, int K, int C64, int r, int rp,
                                                          int mxb, lq_act_view out)
{
    const size_t idx = (size_t)blockIdx.x * 256 + threadIdx.x;
    const int CQ = (C64 + 3) >> 2, B = K >> 5;
    if (idx < (size_t)M * K && out.xq) {
        const int m = (int)(idx / K), k = (int)(idx % K);
        const uint32_t w = *(const uint32_t*)(act + al.off_xq + mx_code_offset(m, k, C64));
        out.xq[idx] = (int8_t)((w >> (4 * (k & 7))) & 0xFu);
    }
    if (idx < (size_t)M * B && out.xe) {
        const int m = (int)(idx / B), b = (int)(idx % B);
        out.xe[idx] = act[al.off_sx + mx_scale_offset(m, b >> 1, b & 1, CQ)];
    }
    if (idx < (size_t)M && out.st && !mxb) out.st[idx] = ((const float*)(act + al.off_st))[idx];
    if (idx < (size_t)M * r && out.tq) {
        const int m = (int)(idx / r), j = (int)(idx % r);
        out.tq[idx] = (int8_t)act[al.off_tq + (mxb ? mxb_frag8_offset(m, j, rp) : (size_t)m * rp + j)];
    }
    if (mxb && idx < (size_t)M * (r >> 5) && out.te) {
        const int m = (int)(idx / (r >> 5)), b = (int)(idx % (r >> 5));
        out.te[idx] = act[al.off_st + mxb_scale_offset(m, b)];
    }
}

hipError_t launch_unpack_act_mx(const Dims& d, const uint8_t* act, int64_t M, const lq_act_view* out, hipStream_t s)
{
    if (d.mxb_elem == 6) return launch_unpack_act_mx6(d, act, M, out, s);
    const ActLayout al = act_layout(d, M);
    const size_t n = (size_t)M * (d.Ks > d.r ? d.Ks : d.r);
    hipLaunchKernelGGL(mx_unpack_a_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, s, act, al, (int)M,
                       (int)d.Ks, d.C64, d.r, d.rp, d.mxb ? 1 : 0, *out);
    return hipGetLastError();
}

// ---------------------------------------------------------------------------------------------
// activation kernel: same decomposition as the INT one (16 token rows per workgroup, lane =
// (row l%16, 16-value quarter l/16 of each 64-chunk), chunks dealt round-robin to 4 wavefronts)
// ---------------------------------------------------------------------------------------------
struct MxActParams {
    const void* X;
    int64_t ldx;
    int M, K, C64, C64s, CQ, r, rp;  // K, C64s: the caller's row length and its 64-chunks; C64: chunks of the layout
    const uint8_t* r8;
    const float* sr;
    uint8_t* xc;
    uint8_t* xe;
    uint8_t* tq8;
    float* st;
    int8_t* dbg_xb;
    float* dbg_sxb;
    float* dbg_T;
    const float* rg;  // reciprocals of the smoothing vector (smoothing variant only)
    BlobTag tag;        // header of the activation blob (written by the first workgroup)
    uint32_t* tag_dst;
};

template <bool BF16>
struct MxChunk;
template <>
struct MxChunk<true> {
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
struct MxChunk<false> {
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

// BF16IN: element type of X; SM: smoothing variant (X times the stored reciprocals, held as fp32).
template <bool BF16IN, int MAXC, int NJB, bool SM = false>
__global__ __launch_bounds__(256) void mx_act_kernel(MxActParams p)
{
    write_tag(p.tag_dst, p.tag);
    constexpr bool BF16 = BF16IN && !SM;  // representation of the row in registers
    __shared__ float s_amax[4][16];
    __shared__ float s_sxb[16];
    __shared__ float s_acc[4][NJB > 0 ? NJB : 1][64][4];

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int r16 = lane & 15, kq = lane >> 4;
    const int row = blockIdx.x * 16 + r16;
    const bool row_ok = row < p.M;
    const int C64 = p.C64;

    // MAXC = 0: rows too long for the registers are streamed twice through a two-chunk ring (amax pass, coding pass;
    // the second read comes from the caches)
    constexpr bool STREAM = MAXC == 0;
    constexpr int NS = STREAM ? 2 : MAXC;   // chunk slots in registers
    const int nmy = (C64 - wave + 3) >> 2;  // chunks of this wavefront: c = wave + 4 * ci, ci < nmy
    MxChunk<BF16> xc[NS];
    auto load_x = [&](MxChunk<BF16>& ch, int ci) {
        const int c = wave + 4 * ci;
        const size_t koff = (size_t)c * 64 + kq * 16;
        const bool ok = row_ok && c < p.C64s;  // (a chunk of the layout past the row is coded from zeros)
        if constexpr (SM)
            smooth_load<BF16IN, 16>(ch.v, p.X, (size_t)row * p.ldx + koff, p.rg + koff, ok);
        else
            ch.load(p.X, (size_t)row * p.ldx + koff, ok);
    };
#pragma unroll
    for (int ci = 0; ci < NS; ++ci) load_x(xc[ci], ci);

    // Operands that do not depend on X are requested now (their latency overlaps the load of X):
    // the Q2(R) fragments of the first chunk (later ones one chunk ahead, in the loop), R's scales.
    constexpr int NJA = NJB > 0 ? NJB : 1;
    v4i bvs[2][NJA];
    auto load_r8 = [&](v4i (&dst)[NJA], int ci) {
        int c = wave + 4 * ci;
        c = c < C64 ? c : C64 - 1;  // clamped: a fragment past the end is fetched but not used
#pragma unroll
        for (int jb = 0; jb < NJB; ++jb) dst[jb] = *(const v4i*)(p.r8 + ((size_t)((size_t)c * NJB + jb) * 64 + lane) * 16);
    };
    load_r8(bvs[0], 0);
    float srj[NJA];
#pragma unroll
    for (int jb = 0; jb < NJB; ++jb) srj[jb] = p.sr[jb * 16 + r16];

    // amax of the lane's 16 values per chunk (kept for the block scale when the row is resident) and of the whole row
    auto amax16 = [&](const MxChunk<BF16>& ch) -> float {
        if constexpr (BF16) {
            // |bf16| is monotonic in its low 15 bits: packed unsigned 16-bit max, two values per op
            us2 m2 = {0, 0};
#pragma unroll
            for (int d = 0; d < 8; ++d) m2 = __builtin_elementwise_max(m2, __builtin_bit_cast(us2, ch.w[d] & 0x7FFF7FFFu));
            const uint32_t mm = m2[0] > m2[1] ? m2[0] : m2[1];
            return __uint_as_float(mm << 16);
        } else {
            float m = 0.f;
#pragma unroll
            for (int i = 0; i < 16; ++i) m = fmaxf(m, fabsf(ch.get(i)));
            return m;
        }
    };
    float a16[NS];
    float a = 0.f;
    if constexpr (STREAM) {
        for (int ci0 = 0; ci0 < nmy; ci0 += 2) {
#pragma unroll
            for (int sl = 0; sl < 2; ++sl) {
                a = fmaxf(a, amax16(xc[sl]));  // (a slot past the end holds zeros)
                load_x(xc[sl], ci0 + sl + 2);
            }
        }
#pragma unroll
        for (int sl = 0; sl < 2; ++sl) load_x(xc[sl], sl);  // second pass: the ring starts over
    } else {
#pragma unroll
        for (int ci = 0; ci < NS; ++ci) {
            a16[ci] = amax16(xc[ci]);
            a = fmaxf(a, a16[ci]);
        }
    }
    a = fmaxf(a, __shfl_xor(a, 16, 64));
    a = fmaxf(a, __shfl_xor(a, 32, 64));
    if (kq == 0) s_amax[wave][r16] = a;
    __syncthreads();
    a = fmaxf(fmaxf(s_amax[0][r16], s_amax[1][r16]), fmaxf(s_amax[2][r16], s_amax[3][r16]));
    float sb, invb;
    fp8_scales(a, &sb, &invb);
    if (wave == 0 && kq == 0) {
        s_sxb[r16] = sb;
        if (p.dbg_sxb && row_ok) p.dbg_sxb[row] = sb;
        if (NJB == 0) p.st[row] = 1.0f;
    }

    v4f acc[NJB > 0 ? NJB : 1];
#pragma unroll
    for (int jb = 0; jb < NJB; ++jb) acc[jb] = v4f{0.f, 0.f, 0.f, 0.f};

    // one 64-chunk: MXFP4 codes and block scales, FP8 branch codes, skinny contraction (am: amax of the lane's 16 values)
    auto code_chunk = [&](const MxChunk<BF16>& ch, const int c, const float am, const int bslot) {
        // MXFP4: block of 32 = this lane's 16 values and its neighbour's (kq ^ 1)
        const float ab = fmaxf(am, __shfl_xor(am, 16, 64));
        const uint32_t E = e8m0_of(ab);
        const float sc = e8m0_value(E);
        uint32_t pk[2] = {0u, 0u};
        uint32_t x8[4];
#define LQ_CVT4(J) pk[(J) >> 2] = __builtin_amdgcn_cvt_scalef32_pk_fp4_f32(pk[(J) >> 2], ch.get(2 * (J)), ch.get(2 * (J) + 1), sc, (J) & 3)
        if (ab != 0.0f) {
            LQ_CVT4(0); LQ_CVT4(1); LQ_CVT4(2); LQ_CVT4(3); LQ_CVT4(4); LQ_CVT4(5); LQ_CVT4(6); LQ_CVT4(7);
        }
#undef LQ_CVT4
#pragma unroll
        for (int q = 0; q < 4; ++q)
            x8[q] = fp8_quad(__fmul_rn(ch.get(4 * q), invb), __fmul_rn(ch.get(4 * q + 1), invb),
                             __fmul_rn(ch.get(4 * q + 2), invb), __fmul_rn(ch.get(4 * q + 3), invb));
        uint8_t* dst = p.xc + ((size_t)((size_t)(row >> 5) * C64 + c) * 64 + (row & 31) + 32 * (kq >> 1)) * 16 + (kq & 1) * 8;
        *(uint2*)dst = make_uint2(pk[0], pk[1]);
        if ((kq & 1) == 0) p.xe[mx_scale_offset(row, c, kq >> 1, p.CQ)] = (uint8_t)E;
        if (p.dbg_xb && row_ok && c < p.C64s)
            *(v4i*)(p.dbg_xb + (size_t)row * p.K + c * 64 + kq * 16) = v4i{(int)x8[0], (int)x8[1], (int)x8[2], (int)x8[3]};
        if (NJB > 0) {
            const long alo = (long)(((unsigned long)x8[1] << 32) | x8[0]);
            const long ahi = (long)(((unsigned long)x8[3] << 32) | x8[2]);
#pragma unroll
            for (int jb = 0; jb < NJB; ++jb) {
                const v4i bv = bvs[bslot][jb];
                const long blo = (long)(((unsigned long)(uint32_t)bv[1] << 32) | (uint32_t)bv[0]);
                const long bhi = (long)(((unsigned long)(uint32_t)bv[3] << 32) | (uint32_t)bv[2]);
                acc[jb] = __builtin_amdgcn_mfma_f32_16x16x32_fp8_fp8(alo, blo, acc[jb], 0, 0, 0);
                acc[jb] = __builtin_amdgcn_mfma_f32_16x16x32_fp8_fp8(ahi, bhi, acc[jb], 0, 0, 0);
            }
        }
    };
    auto pad_chunk = [&](const int c) {  // padding chunk of the last quad: its scale bytes must be valid E8M0 values (2^0)
        if (c >= C64 && c < 4 * p.CQ && (kq & 1) == 0) p.xe[mx_scale_offset(row, c, kq >> 1, p.CQ)] = (uint8_t)127;
    };
    if constexpr (STREAM) {
        for (int ci0 = 0; ci0 < nmy; ci0 += 2) {
#pragma unroll
            for (int sl = 0; sl < 2; ++sl) {
                const int ci = ci0 + sl, c = wave + 4 * ci;
                load_r8(bvs[(sl + 1) & 1], ci + 1);
                if (c < C64) code_chunk(xc[sl], c, amax16(xc[sl]), sl);  // wave-uniform
                load_x(xc[sl], ci + 2);
            }
        }
        pad_chunk(wave + 4 * nmy);
    } else {
#pragma unroll
        for (int ci = 0; ci < NS; ++ci) {
            const int c = wave + 4 * ci;
            if (ci + 1 < NS) load_r8(bvs[(ci + 1) & 1], ci + 1);
            if (c < C64) code_chunk(xc[ci], c, a16[ci], ci & 1);  // wave-uniform
            else pad_chunk(c);
        }
    }
    if (NJB == 0) return;

#pragma unroll
    for (int jb = 0; jb < NJB; ++jb) *(v4f*)&s_acc[wave][jb][lane][0] = acc[jb];
    __syncthreads();
    if (wave != 0) return;

    float T[NJB > 0 ? NJB : 1][4];
    float tmax[4] = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int jb = 0; jb < NJB; ++jb) {
        v4f s = *(const v4f*)&s_acc[0][jb][lane][0];
#pragma unroll
        for (int w = 1; w < 4; ++w) {
            const v4f o = *(const v4f*)&s_acc[w][jb][lane][0];
#pragma unroll
            for (int i = 0; i < 4; ++i) s[i] = __fadd_rn(s[i], o[i]);
        }
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int tok = 4 * kq + i;
            const float tv = __fmul_rn(__fmul_rn(s[i], s_sxb[tok]), srj[jb]);
            T[jb][i] = tv;
            tmax[i] = fmaxf(tmax[i], fabsf(tv));
            const int grow = blockIdx.x * 16 + tok;
            if (grow < p.M && p.dbg_T) p.dbg_T[(size_t)grow * p.r + jb * 16 + r16] = tv;
        }
    }
#pragma unroll
    for (int i = 0; i < 4; ++i) {
#pragma unroll
        for (int o = 8; o >= 1; o >>= 1) tmax[i] = fmaxf(tmax[i], __shfl_xor(tmax[i], o, 64));
    }
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int grow = blockIdx.x * 16 + 4 * kq + i;
        float stv, invt;
        fp8_scales(tmax[i], &stv, &invt);
        if (r16 == 0) p.st[grow] = stv;
#pragma unroll
        for (int jb = 0; jb < NJB; ++jb) p.tq8[(size_t)grow * p.rp + jb * 16 + r16] = (uint8_t)fp8_byte(__fmul_rn(T[jb][i], invt));
        for (int j = p.r + r16; j < p.rp; j += 16) p.tq8[(size_t)grow * p.rp + j] = 0;
    }
}

template <bool BF16, int MAXC, int NJB, bool SM>
static hipError_t mx_act_launch(const MxActParams& p, int64_t Mp, hipStream_t s)
{
    hipLaunchKernelGGL((mx_act_kernel<BF16, MAXC, NJB, SM>), dim3((unsigned)(Mp / 16)), dim3(256), 0, s, p);
    return hipGetLastError();
}
template <bool BF16, int MAXC, bool SM = false>
static hipError_t mx_act_rank(const MxActParams& p, int64_t Mp, hipStream_t s)
{
    switch (p.r) {
        case 0: return mx_act_launch<BF16, MAXC, 0, SM>(p, Mp, s);
        case 16: return mx_act_launch<BF16, MAXC, 1, SM>(p, Mp, s);
        case 32: return mx_act_launch<BF16, MAXC, 2, SM>(p, Mp, s);
        case 64: return mx_act_launch<BF16, MAXC, 4, SM>(p, Mp, s);
        default: return mx_act_launch<BF16, MAXC, 8, SM>(p, Mp, s);
    }
}

static hipError_t launch_quantize_act_mxb(const Dims& d, int x_dtype, const uint8_t* packed, const void* X, int64_t M,
                                          int64_t ldx, uint8_t* act, const lq_act_debug* dbg, hipStream_t s);

hipError_t launch_quantize_act_mx(const Dims& d, int x_dtype, const uint8_t* packed, const void* X, int64_t M,
                                  int64_t ldx, uint8_t* act, const lq_act_debug* dbg, hipStream_t s)
{
    if (d.mxb_elem == 6) return launch_quantize_act_mx6(d, x_dtype, packed, X, M, ldx, act, dbg, s);
    if (d.mxb) return launch_quantize_act_mxb(d, x_dtype, packed, X, M, ldx, act, dbg, s);
    const PackedLayout pl = packed_layout(d);
    const ActLayout al = act_layout(d, M);
    MxActParams p;
    p.tag = make_tag(d, LQ_BLOB_ACT, M);
    p.tag_dst = (uint32_t*)act;
    p.X = X;
    p.ldx = ldx;
    p.M = (int)M;
    p.K = (int)d.Ks;
    p.C64 = d.C64;
    p.C64s = (int)(d.Ks / 64);
    p.CQ = (d.C64 + 3) / 4;
    p.r = d.r;
    p.rp = d.rp;
    p.r8 = packed + pl.off_rq;
    p.sr = (const float*)(packed + pl.off_sr);
    p.xc = act + al.off_xq;
    p.xe = act + al.off_sx;
    p.tq8 = act + al.off_tq;
    p.st = (float*)(act + al.off_st);
    p.dbg_xb = dbg ? dbg->xb : nullptr;
    p.dbg_sxb = dbg ? dbg->sxb : nullptr;
    p.dbg_T = dbg ? dbg->T : nullptr;
    const int maxc = (d.C64 + 3) / 4;
    p.rg = d.smooth ? (const float*)(packed + pl.off_rg) : nullptr;
    // MAXC = 0: the streamed form, for rows that do not fit in registers (fp32 representation: K > 2304; bf16: K > 4608)
    if (d.smooth) {
        if (x_dtype == LQ_BF16)
            return maxc <= 5 ? mx_act_rank<true, 5, true>(p, al.Mp, s) : maxc <= 9 ? mx_act_rank<true, 9, true>(p, al.Mp, s) : mx_act_rank<true, 0, true>(p, al.Mp, s);
        return maxc <= 5 ? mx_act_rank<false, 5, true>(p, al.Mp, s) : maxc <= 9 ? mx_act_rank<false, 9, true>(p, al.Mp, s) : mx_act_rank<false, 0, true>(p, al.Mp, s);
    }
    if (x_dtype == LQ_BF16) {
        if (maxc <= 5) return mx_act_rank<true, 5>(p, al.Mp, s);
        if (maxc <= 9) return mx_act_rank<true, 9>(p, al.Mp, s);
        if (maxc <= 18) return mx_act_rank<true, 18>(p, al.Mp, s);
        return mx_act_rank<true, 0>(p, al.Mp, s);
    }
    if (maxc <= 5) return mx_act_rank<false, 5>(p, al.Mp, s);
    if (maxc <= 9) return mx_act_rank<false, 9>(p, al.Mp, s);
    return mx_act_rank<false, 0>(p, al.Mp, s);
}

// ---------------------------------------------------------------------------------------------
// activation kernel with an MXFP8e4 branch.  Same decomposition as above, but K is walked in chunks
// of 128 (= one v_mfma_scale_f32_16x16x128_f8f6f4): lane (row l%16, q = l/16) holds the 16 values
// k = 16q.. of each 64-half of the chunk, which is both the fragment position of the 4-bit main codes
// and, as E4M3, bytes 0..15 / 16..31 of the lane's 8-bit MFMA operand.  A 32-block is shared by the
// lane pair (q, q^1); the MFMA takes the scale of block q from lane (row, q), so lanes 1 and 2 swap.
// ---------------------------------------------------------------------------------------------
struct MxbActParams {
    const void* X;
    int64_t ldx;
    int M, K, C64, C64s, CQ, C128, r, rp;  // K, C64s: the caller's row length and its 64-chunks; C64, C128: of the layout
    const uint8_t* r8;
    const uint8_t* re;
    uint8_t* xc;
    uint8_t* xe;
    uint8_t* tq8;
    uint8_t* te;
    int8_t* dbg_xb;
    uint8_t* dbg_xbe;
    float* dbg_T;
    const float* rg;  // reciprocals of the smoothing vector (smoothing variant only)
    BlobTag tag;        // header of the activation blob (written by the first workgroup)
    uint32_t* tag_dst;
};

// BF16IN: element type of X; SM: smoothing variant (X times the stored reciprocals, held as fp32).
template <bool BF16IN, int NJB, bool SM = false>
__global__ __launch_bounds__(256) void mxb_act_kernel(MxbActParams p)
{
    write_tag(p.tag_dst, p.tag);
    constexpr bool BF16 = BF16IN && !SM;  // representation of a chunk in registers
    constexpr int NJA = NJB > 0 ? NJB : 1;
    constexpr int PF = 2;  // 128-chunks in flight per wavefront: no scale spans more than a block, the row is streamed
    __shared__ float s_acc[4][NJA][64][4];

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int r16 = lane & 15, q = lane >> 4;
    const int row = blockIdx.x * 16 + r16;
    const bool row_ok = row < p.M;
    const int C64 = p.C64, C128 = p.C128;

    const int nmy = (C128 - wave + 3) >> 2;  // chunks of this wavefront: c = wave + 4 * ci, ci < nmy
    MxChunk<BF16> xh[PF][2];
    auto load_x = [&](MxChunk<BF16>& ch, size_t koff, bool ok) {
        if constexpr (SM)
            smooth_load<BF16IN, 16>(ch.v, p.X, (size_t)row * p.ldx + koff, p.rg + koff, ok);
        else
            ch.load(p.X, (size_t)row * p.ldx + koff, ok);
    };
#pragma unroll
    for (int i = 0; i < PF; ++i)
#pragma unroll
        for (int hh = 0; hh < 2; ++hh)
            load_x(xh[i][hh], (size_t)(wave + 4 * i) * 128 + hh * 64 + q * 16, row_ok && 2 * (wave + 4 * i) + hh < p.C64s);
    // R fragments and their scale dwords: first chunk now, later ones one chunk ahead
    v8i bvs[2][NJA];
    int bss[2][NJA];
    auto load_r8 = [&](int slot, int ci) {
        int c = wave + 4 * ci;
        c = c < C128 ? c : C128 - 1;  // clamped: a fragment past the end is fetched but not used
#pragma unroll
        for (int jb = 0; jb < NJB; ++jb) {
            bvs[slot][jb] = *(const v8i*)(p.r8 + ((size_t)((size_t)c * NJB + jb) * 64 + lane) * 32);
            bss[slot][jb] = *(const int*)(p.re + ((size_t)((size_t)c * NJB + jb) * 64 + lane) * 4);
        }
    };
    load_r8(0, 0);

    v4f acc[NJA];
#pragma unroll
    for (int jb = 0; jb < NJB; ++jb) acc[jb] = v4f{0.f, 0.f, 0.f, 0.f};

    for (int base = 0; base < nmy; base += PF) {
#pragma unroll
    for (int sl = 0; sl < PF; ++sl) {
        const int ci = base + sl;
        const int c = wave + 4 * ci;
        load_r8((sl + 1) & 1, ci + 1);
        if (ci < nmy) {  // wave-uniform
            uint32_t x8[8];
            uint32_t Eh[2];
#pragma unroll
            for (int hh = 0; hh < 2; ++hh) {
                const MxChunk<BF16>& xc = xh[sl][hh];
                float m = 0.f;
                if constexpr (BF16) {
                    us2 m2 = {0, 0};
#pragma unroll
                    for (int d = 0; d < 8; ++d) m2 = __builtin_elementwise_max(m2, __builtin_bit_cast(us2, xc.w[d] & 0x7FFF7FFFu));
                    const uint32_t mm = m2[0] > m2[1] ? m2[0] : m2[1];
                    m = __uint_as_float(mm << 16);
                } else {
#pragma unroll
                    for (int i = 0; i < 16; ++i) m = fmaxf(m, fabsf(xc.get(i)));
                }
                const float ab = fmaxf(m, __shfl_xor(m, 16, 64));  // amax of the 32-block (lanes q, q^1)
                // main codes: MXFP4
                const uint32_t E4 = e8m0_of(ab);
                const float sc = e8m0_value(E4);
                uint32_t pk[2] = {0u, 0u};
#define LQ_CVT4(J) pk[(J) >> 2] = __builtin_amdgcn_cvt_scalef32_pk_fp4_f32(pk[(J) >> 2], xc.get(2 * (J)), xc.get(2 * (J) + 1), sc, (J) & 3)
                if (ab != 0.0f) {
                    LQ_CVT4(0); LQ_CVT4(1); LQ_CVT4(2); LQ_CVT4(3); LQ_CVT4(4); LQ_CVT4(5); LQ_CVT4(6); LQ_CVT4(7);
                }
#undef LQ_CVT4
                const int c64 = 2 * c + hh;
                uint8_t* dst = p.xc + ((size_t)((size_t)(row >> 5) * C64 + c64) * 64 + (row & 31) + 32 * (q >> 1)) * 16 + (q & 1) * 8;
                *(uint2*)dst = make_uint2(pk[0], pk[1]);
                if ((q & 1) == 0) p.xe[mx_scale_offset(row, c64, q >> 1, p.CQ)] = (uint8_t)E4;
                // branch codes: MXFP8e4 of the same block
                const uint32_t E8 = e8m0_of_fp8(ab);
                const float inv8 = e8m0_inverse(E8);
                Eh[hh] = E8;
#pragma unroll
                for (int g = 0; g < 4; ++g)
                    x8[4 * hh + g] = fp8_quad(__fmul_rn(xc.get(4 * g), inv8), __fmul_rn(xc.get(4 * g + 1), inv8),
                                              __fmul_rn(xc.get(4 * g + 2), inv8), __fmul_rn(xc.get(4 * g + 3), inv8));
                if (p.dbg_xb && row_ok && c64 < p.C64s)
                    *(v4i*)(p.dbg_xb + (size_t)row * p.K + (size_t)c * 128 + hh * 64 + q * 16) =
                        v4i{(int)x8[4 * hh], (int)x8[4 * hh + 1], (int)x8[4 * hh + 2], (int)x8[4 * hh + 3]};
                if (p.dbg_xbe && row_ok && c64 < p.C64s && (q & 1) == 0) p.dbg_xbe[(size_t)row * (p.K >> 5) + 4 * c + 2 * hh + (q >> 1)] = (uint8_t)E8;
            }
            if (NJB > 0) {
                // lane q knows blocks (q>>1) [first half] and 2+(q>>1) [second half]; it must supply block q
                const uint32_t send = (q == 1) ? Eh[1] : Eh[0];
                const uint32_t recv = (uint32_t)__shfl_xor((int)send, 48, 64);
                const int sa = (int)((q == 0) ? Eh[0] : (q == 3) ? Eh[1] : recv);
                const v8i a8 = {(int)x8[0], (int)x8[1], (int)x8[2], (int)x8[3], (int)x8[4], (int)x8[5], (int)x8[6], (int)x8[7]};
#pragma unroll
                for (int jb = 0; jb < NJB; ++jb)
                    acc[jb] = __builtin_amdgcn_mfma_scale_f32_16x16x128_f8f6f4(a8, bvs[sl & 1][jb], acc[jb], 0, 0, 0, sa, 0,
                                                                            bss[sl & 1][jb]);
            }
        }
        // refill the slot with the chunk PF positions further on
#pragma unroll
        for (int hh = 0; hh < 2; ++hh)
            load_x(xh[sl][hh], (size_t)(c + 4 * PF) * 128 + hh * 64 + q * 16, row_ok && 2 * (c + 4 * PF) + hh < p.C64s);
    }
    }
    {   // padding 64-chunks of the last quad (at most one 128-chunk per wavefront): valid E8M0 bytes (2^0)
        const int c = wave + 4 * nmy;
#pragma unroll
        for (int hh = 0; hh < 2; ++hh)
            if (2 * c + hh < 4 * p.CQ && (q & 1) == 0) p.xe[mx_scale_offset(row, 2 * c + hh, q >> 1, p.CQ)] = (uint8_t)127;
    }
    if (NJB == 0) return;

#pragma unroll
    for (int jb = 0; jb < NJB; ++jb) *(v4f*)&s_acc[wave][jb][lane][0] = acc[jb];
    __syncthreads();
    if (wave != 0) return;

    // lane holds column j = jb*16 + lane%16 of the intermediate for token rows 4*q + i
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
            const int grow = blockIdx.x * 16 + 4 * q + i;
            if (grow < p.M && p.dbg_T) p.dbg_T[(size_t)grow * p.r + jb * 16 + r16] = sum[i];
        }
    }
    // re-quantise per token and per block of 32 along the rank (two 16-column groups per block)
#pragma unroll
    for (int bb = 0; bb < (NJB + 1) / 2; ++bb) {
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            float tm = fmaxf(fabsf(T[2 * bb][i]), fabsf(T[2 * bb + 1][i]));
#pragma unroll
            for (int o = 8; o >= 1; o >>= 1) tm = fmaxf(tm, __shfl_xor(tm, o, 64));
            const int grow = blockIdx.x * 16 + 4 * q + i;
            const uint32_t E = e8m0_of_fp8(tm);
            const float inv = e8m0_inverse(E);
            if (r16 == 0) p.te[mxb_scale_offset(grow, bb)] = (uint8_t)E;
#pragma unroll
            for (int g = 0; g < 2; ++g)
                p.tq8[mxb_frag8_offset(grow, (2 * bb + g) * 16 + r16, p.rp)] = (uint8_t)fp8_byte(__fmul_rn(T[2 * bb + g][i], inv));
        }
    }
    // padding of the rank to a multiple of 64: zero codes, scale 2^0
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int grow = blockIdx.x * 16 + 4 * q + i;
        for (int j = p.r + r16; j < p.rp; j += 16) p.tq8[mxb_frag8_offset(grow, j, p.rp)] = 0;
        if (r16 == 0)
            for (int bb = p.r >> 5; bb < (p.rp >> 5); ++bb) p.te[mxb_scale_offset(grow, bb)] = (uint8_t)127;
    }
}

template <bool BF16, int NJB, bool SM>
static hipError_t mxb_act_launch(const MxbActParams& p, int64_t Mp, hipStream_t s)
{
    hipLaunchKernelGGL((mxb_act_kernel<BF16, NJB, SM>), dim3((unsigned)(Mp / 16)), dim3(256), 0, s, p);
    return hipGetLastError();
}
template <bool BF16, bool SM>
static hipError_t mxb_act_rank2(const MxbActParams& p, int64_t Mp, hipStream_t s)
{
    switch (p.r) {
        case 0: return mxb_act_launch<BF16, 0, SM>(p, Mp, s);
        case 32: return mxb_act_launch<BF16, 2, SM>(p, Mp, s);
        case 64: return mxb_act_launch<BF16, 4, SM>(p, Mp, s);
        case 96: return mxb_act_launch<BF16, 6, SM>(p, Mp, s);
        default: return mxb_act_launch<BF16, 8, SM>(p, Mp, s);
    }
}
template <bool BF16>
static hipError_t mxb_act_rank(const MxbActParams& p, int64_t Mp, hipStream_t s)
{
    return p.rg ? mxb_act_rank2<BF16, true>(p, Mp, s) : mxb_act_rank2<BF16, false>(p, Mp, s);
}

static hipError_t launch_quantize_act_mxb(const Dims& d, int x_dtype, const uint8_t* packed, const void* X, int64_t M,
                                          int64_t ldx, uint8_t* act, const lq_act_debug* dbg, hipStream_t s)
{
    const PackedLayout pl = packed_layout(d);
    const ActLayout al = act_layout(d, M);
    MxbActParams p;
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
    p.r8 = packed + pl.off_rq;
    p.re = packed + pl.off_sr;
    p.xc = act + al.off_xq;
    p.xe = act + al.off_sx;
    p.tq8 = act + al.off_tq;
    p.te = act + al.off_st;
    p.dbg_xb = dbg ? dbg->xb : nullptr;
    p.dbg_xbe = dbg ? dbg->xbe : nullptr;
    p.dbg_T = dbg ? dbg->T : nullptr;
    p.rg = d.smooth ? (const float*)(packed + pl.off_rg) : nullptr;
    return x_dtype == LQ_BF16 ? mxb_act_rank<true>(p, al.Mp, s) : mxb_act_rank<false>(p, al.Mp, s);
}

// ---------------------------------------------------------------------------------------------
// forward: 1 x 4 wavefronts per workgroup, 128 x 64 outputs per wavefront, K staged 128 at a time
// ---------------------------------------------------------------------------------------------
struct MxFwdParams {
    const uint8_t* xc;
    const uint8_t* xe;
    const uint8_t* tq8;
    const float* st;
    const uint8_t* pc;
    const uint8_t* pe;
    const uint8_t* l8;
    const float* sl;
    uint16_t* Y;
    int64_t ldy;
    int M, N, C64, CQ, S, rp, nrb;
    int tilesM, tilesN, panel;
    int n_full;  // workgroups that compute whole tiles; the rest of the grid are half tiles
    float* dbg_y32;
};

// NK = 64-deep chunks of the (padded) rank: 0 | 1 | 2.  BLK: the branch is MXFP8e4 (block scales,
// accumulated by the scaled MFMA straight into the main product's accumulators).
// BFMT: operand format code of the block-scaled branch (0 = E4M3, 2 = E2M3).
namespace mxf {
constexpr int WN = 4, RBT = 4;
constexpr int EPI_ROW = 136, EPI_WAVE = 32 * EPI_ROW;
constexpr int NBUF = 4;                          // LDS buffers of the activation stream (one stage each)
constexpr int LDS_MAIN = NBUF * 2 * RBT * 1024;  // [buffer][chunk in stage][row block][lane][16 B]
constexpr int LDS_BYTES = LDS_MAIN > 4 * EPI_WAVE ? LDS_MAIN : 4 * EPI_WAVE;
constexpr int LDS_TOTAL = LDS_BYTES + RBT * 32 * 4 + WN * 64 * 4;
}  // namespace mxf

// One output tile: row blocks rb0 .. rb0 + NRB - 1 (NRB = 4: a whole 128-row tile; 2: a half tile of the grid's last,
// sparse generation), columns tile_n * 256 ...  The four wavefronts always stage four row blocks (clamped).
template <int NK, bool DBG, bool BLK, int BFMT, int NRB>
__device__ __forceinline__ void mx_fwd_tile(const MxFwdParams& p, uint8_t* lds, const int rb0, const int tile_n)
{
    using namespace mxf;
    // + the tile's 128 per-token scales of the fp32-scaled branch (read back by every wavefront in the epilogue: an LDS
    // broadcast read instead of sixteen 1 KB vector-memory loads per wavefront whose lanes all fetch the same 16 bytes)
    // ... and the tile's 256 per-channel scales of that branch; both are small loads whose round trip would otherwise
    // open the epilogue
    float* lds_st = (float*)(lds + LDS_BYTES);
    float* lds_sl = lds_st + RBT * 32;

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int half = lane >> 5, l32 = lane & 31;

    const int cb0 = tile_n * (WN * 2) + wave * 2;
    const bool active = (cb0 * 32 < p.N) && (rb0 < p.nrb);
    const int C64 = p.C64, CQ = p.CQ, S = p.S;

    const uint32_t lane16 = (uint32_t)lane * 16u, lane4 = (uint32_t)lane * 4u;
    int rbs = rb0 + wave;  // row block staged by this wavefront
    rbs = rbs < p.nrb ? rbs : p.nrb - 1;
    const uint8_t* xc_base = p.xc + (size_t)rbs * C64 * 1024;
    const int cbw = (cb0 * 32 < p.N) ? cb0 : 0;
    const uint8_t* pc_base[2] = {p.pc + (size_t)cbw * C64 * 1024, p.pc + (size_t)(cbw + 1) * C64 * 1024};
    const uint8_t* pe_base[2] = {p.pe + (size_t)cbw * CQ * 256, p.pe + (size_t)(cbw + 1) * CQ * 256};
    const uint8_t* xe_base[NRB];
#pragma unroll
    for (int rbi = 0; rbi < NRB; ++rbi) {
        int rb = rb0 + rbi;
        rb = rb < p.nrb ? rb : p.nrb - 1;
        xe_base[rbi] = p.xe + (size_t)rb * CQ * 256;
    }

    struct AStage { v4i v[2]; };
    struct BStage { v4i v[2][2]; };
    // The streams are read with buffer loads: a wave-uniform descriptor and chunk offset in scalar registers plus the
    // 32-bit lane offsets all streams share, instead of a 64-bit vector address per stream (about 28 registers per
    // lane fewer).  Each descriptor spans exactly the bytes its stream may touch.
    typedef unsigned int u4 __attribute__((ext_vector_type(4)));
    constexpr int RSRC_FLAGS = 0x00020000;
    const __amdgpu_buffer_rsrc_t rs_pe[2] = {__builtin_amdgcn_make_buffer_rsrc((void*)pe_base[0], 0, CQ * 256, RSRC_FLAGS),
                                             __builtin_amdgcn_make_buffer_rsrc((void*)pe_base[1], 0, CQ * 256, RSRC_FLAGS)};
    __amdgpu_buffer_rsrc_t rs_xe[NRB];
#pragma unroll
    for (int rbi = 0; rbi < NRB; ++rbi) rs_xe[rbi] = __builtin_amdgcn_make_buffer_rsrc((void*)xe_base[rbi], 0, CQ * 256, RSRC_FLAGS);
    // A load for a stage (or quad of chunks) past the end goes through a descriptor of zero bytes: every lane is out of
    // range, nothing is fetched and the (unused) result is zero; the loop body stays branch-free.
    auto load_a = [&](AStage& a, int stage) {
        const bool ok = stage < S;
        const int st = ok ? stage : S - 1;
        const __amdgpu_buffer_rsrc_t rs = __builtin_amdgcn_make_buffer_rsrc((void*)xc_base, 0, ok ? C64 * 1024 : 0, RSRC_FLAGS);
#pragma unroll
        for (int cc = 0; cc < 2; ++cc)
            a.v[cc] = __builtin_bit_cast(v4i, (u4)__builtin_amdgcn_raw_buffer_load_b128(rs, lane16, (st * 2 + cc) * 1024, 0));
    };
    auto store_a = [&](const AStage& a, int buf) {
#pragma unroll
        for (int cc = 0; cc < 2; ++cc) *(v4i*)(lds + (size_t)(((buf * 2 + cc) * RBT + wave) * 1024) + lane16) = a.v[cc];
    };
    auto load_b = [&](BStage& b, int stage) {
        const bool ok = stage < S;
        const int st = ok ? stage : S - 1;
#pragma unroll
        for (int cbi = 0; cbi < 2; ++cbi) {
            const __amdgpu_buffer_rsrc_t rs = __builtin_amdgcn_make_buffer_rsrc((void*)pc_base[cbi], 0, ok ? C64 * 1024 : 0, RSRC_FLAGS);
#pragma unroll
            for (int cc = 0; cc < 2; ++cc)
                b.v[cc][cbi] = __builtin_bit_cast(v4i, (u4)__builtin_amdgcn_raw_buffer_load_b128(rs, lane16, (st * 2 + cc) * 1024, 0));
        }
    };
    // scale dwords of one quad of chunks (= two stages)
    struct Scales { int a[NRB]; int b[2]; };
    auto load_s = [&](Scales& sc, int quad) {
        const int q = quad < CQ ? quad : CQ - 1;
#pragma unroll
        for (int rbi = 0; rbi < NRB; ++rbi) sc.a[rbi] = (int)__builtin_amdgcn_raw_buffer_load_b32(rs_xe[rbi], lane4, q * 256, 0);
#pragma unroll
        for (int cbi = 0; cbi < 2; ++cbi) sc.b[cbi] = (int)__builtin_amdgcn_raw_buffer_load_b32(rs_pe[cbi], lane4, q * 256, 0);
    };

    v16f t[NRB][2];
#pragma unroll
    for (int a = 0; a < NRB; ++a)
#pragma unroll
        for (int b = 0; b < 2; ++b)
#pragma unroll
            for (int i = 0; i < 16; ++i) t[a][b][i] = 0.f;

    // One stage = 128 values of K = two 64-chunks = eight activation fragments (chunk, row block), each the A operand of
    // two MFMAs.  P = stage index mod 4: LDS buffer P holds the stage's activation codes, buffer P+1 those of the next
    // stage (written one stage earlier, so they are visible without a barrier in between), buffer P+2 receives stage
    // s+2 during this one.  The fragments are read two ahead of their MFMAs into a ring of four register sets, across
    // the stage boundary as well, so that a wavefront on its own keeps the matrix core busy (the barrier at the end of
    // a stage orders LDS writes against reads two stages apart; nothing waits on it).  Loads past the last stage are
    // issued through an empty descriptor: at K = 1152 they would be a sixth of the wavefront's vector-memory work.
    // The op_sel immediates of the scale bytes are 2*(P&1) and 2*(P&1)+1.
    v4i fr[4];
    constexpr int NF = 2 * NRB;                    // fragments of a stage
    auto lds_frag = [&](int buf, int f) -> v4i {   // f = chunk * NRB + row block
        return *(const v4i*)(lds + (size_t)((buf * 2 * RBT + (f / NRB) * RBT + f % NRB) * 1024) + lane16);
    };
    auto do_stage = [&](auto pc, int s, AStage& a, BStage& b, const Scales& sc) {
        constexpr int P = decltype(pc)::value, PAR = P & 1;
#pragma unroll
        for (int f = 0; f < NF; ++f) {
            const int cc = f / NRB, rbi = f % NRB;
            fr[(f + 2) & 3] = f + 2 < NF ? lds_frag(P, f + 2) : lds_frag((P + 1) & 3, f + 2 - NF);
            if (f == 0) store_a(a, (P + 2) & 3);
            if (f == 1) load_a(a, s + 4);
            const v4i av = fr[f & 3];
            const v8i a8 = {av[0], av[1], av[2], av[3], 0, 0, 0, 0};
#pragma unroll
            for (int cbi = 0; cbi < 2; ++cbi) {
                const v4i bq = b.v[cc][cbi];
                const v8i b8 = {bq[0], bq[1], bq[2], bq[3], 0, 0, 0, 0};
                // the weights are the first operand: a lane then holds one token and, per register quad, four
                // consecutive channels (the epilogue packs them into 8-byte LDS writes)
                if (cc == 0)
                    t[rbi][cbi] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(b8, a8, t[rbi][cbi], 4, 4, 2 * PAR,
                                                                                 sc.b[cbi], 2 * PAR, sc.a[rbi]);
                else
                    t[rbi][cbi] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(b8, a8, t[rbi][cbi], 4, 4, 2 * PAR + 1,
                                                                                 sc.b[cbi], 2 * PAR + 1, sc.a[rbi]);
            }
            if (f == NF - 1) load_b(b, s + 2);
            __builtin_amdgcn_sched_barrier(0);
        }
        __syncthreads();
    };

    // A wavefront whose columns lie past N (the last tile column of a layer whose width is no multiple of 256) only stages
    // its row block of the activation codes and the token scales, barrier for barrier with the others: no matrix work, no
    // weight or scale loads that would compete with the wavefront it shares a SIMD with.
    if (cb0 * 32 >= p.N) {  // wave-uniform
        AStage x0, x1;
        load_a(x0, 0);
        load_a(x1, 1);
        if constexpr (!BLK && NK > 0) {
            if (lane < 32) lds_st[wave * 32 + lane] = p.st[rbs * 32 + lane];
        }
        store_a(x0, 0);
        store_a(x1, 1);
        load_a(x0, 2);
        load_a(x1, 3);
        __syncthreads();
        for (int s = 0; s < S; s += 2) {  // stage s sends stage s + 2 to its buffer and requests stage s + 4
            store_a(x0, (s + 2) & 3);
            load_a(x0, s + 4);
            __syncthreads();
            if (s + 1 >= S) break;
            store_a(x1, (s + 3) & 3);
            load_a(x1, s + 5);
            __syncthreads();
        }
        return;
    }
    AStage a0, a1;
    BStage b0, b1;
    Scales s0, s1;
    load_a(a0, 0);
    load_a(a1, 1);
    load_b(b0, 0);
    load_s(s0, 0);
    if constexpr (!BLK && NK > 0) {
        if (lane < 32) lds_st[wave * 32 + lane] = p.st[rbs * 32 + lane];
        lds_sl[wave * 64 + lane] = p.sl[cbw * 32 + lane];
    }
    store_a(a0, 0);
    store_a(a1, 1);
    __builtin_amdgcn_sched_barrier(0);
    load_a(a0, 2);
    load_a(a1, 3);
    load_b(b1, 1);
    load_s(s1, 1);
    // Operands of the epilogue's first matrix instructions (the branch's channel codes, the intermediate codes of the
    // first row block) are requested here: asked for at the start of the epilogue, their round trip would open it.
    constexpr int NKF = BLK ? 0 : NK;  // chunks of the fp32-scaled branch handled in the epilogue
    constexpr int NKA = NKF > 0 ? NKF : 1;
    constexpr bool TQ_ALL = NKF <= 1;
    v8i lf[2][NKA];
    v8i tf[TQ_ALL ? NRB : 1][NKA];
    auto load_tq = [&](int rbi) {
        int rb = rb0 + rbi;
        rb = rb < p.nrb ? rb : p.nrb - 1;
#pragma unroll
        for (int kk = 0; kk < NKF; ++kk)
            tf[TQ_ALL ? rbi : 0][kk] = *(const v8i*)(p.tq8 + (size_t)(rb * 32 + l32) * p.rp + kk * 64 + half * 32);
    };
    auto load_lf = [&]() {
#pragma unroll
        for (int cbi = 0; cbi < 2; ++cbi)
#pragma unroll
            for (int kk = 0; kk < NKF; ++kk)
                lf[cbi][kk] = *(const v8i*)(p.l8 + (size_t)((cbw + cbi) * 32 + l32) * p.rp + kk * 64 + half * 32);
    };
    constexpr bool EARLY = NKF == 1;  // (two chunks: the registers are not there; the epilogue requests them itself)
    if constexpr (EARLY) {
        load_lf();
        load_tq(0);
    }
    __builtin_amdgcn_sched_barrier(0);
    __syncthreads();
    fr[0] = lds_frag(0, 0);
    fr[1] = lds_frag(0, 1);

    // stages come in groups of four (two quads of chunks): quad q uses scale set q & 1
    int s = 0;
    for (; s + 3 < S; s += 4) {
        do_stage(std::integral_constant<int, 0>{}, s, a0, b0, s0);
        do_stage(std::integral_constant<int, 1>{}, s + 1, a1, b1, s0);
        load_s(s0, (s >> 1) + 2);
        do_stage(std::integral_constant<int, 2>{}, s + 2, a0, b0, s1);
        do_stage(std::integral_constant<int, 3>{}, s + 3, a1, b1, s1);
        load_s(s1, (s >> 1) + 3);
    }
    if (s < S) {
        do_stage(std::integral_constant<int, 0>{}, s, a0, b0, s0);
        if (s + 1 < S) do_stage(std::integral_constant<int, 1>{}, s + 1, a1, b1, s0);
        if (s + 2 < S) do_stage(std::integral_constant<int, 2>{}, s + 2, a0, b0, s1);
    }

    if (!active) return;

    if constexpr (BLK) {
        // ---- MXFP8e4 branch: tq . lq^T with both block scales, on top of the main accumulators.
        // Operands are stored in the 8-bit operand order of the instruction (32 bytes per lane and
        // 64-chunk of the rank); the scale dword of a lane holds the byte of chunk cc at position cc.
#pragma unroll
        for (int cc = 0; cc < NK; ++cc) {
            v8i lb[2];
            int lsc[2];
#pragma unroll
            for (int cbi = 0; cbi < 2; ++cbi) {
                lb[cbi] = *(const v8i*)(p.l8 + ((size_t)((size_t)(cb0 + cbi) * NK + cc) * 64 + lane) * 32);
                lsc[cbi] = *(const int*)((const uint8_t*)p.sl + ((size_t)(cb0 + cbi) * 64 + lane) * 4);
            }
#pragma unroll
            for (int rbi = 0; rbi < NRB; ++rbi) {
                int rb = rb0 + rbi;
                rb = rb < p.nrb ? rb : p.nrb - 1;
                const v8i ta = *(const v8i*)(p.tq8 + ((size_t)((size_t)rb * NK + cc) * 64 + lane) * 32);
                const int tsc = *(const int*)((const uint8_t*)p.st + ((size_t)rb * 64 + lane) * 4);
#pragma unroll
                for (int cbi = 0; cbi < 2; ++cbi) {
                    if (cc == 0)
                        t[rbi][cbi] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(lb[cbi], ta, t[rbi][cbi], BFMT, BFMT, 0, lsc[cbi], 0, tsc);
                    else
                        t[rbi][cbi] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(lb[cbi], ta, t[rbi][cbi], BFMT, BFMT, 1, lsc[cbi], 1, tsc);
                }
            }
        }
    }

    // ---- epilogue: FP8 rank-r expansion, scales, sum, bf16, full-line stores -------
    // A lane holds token l32 of a row block and, in registers 4g .. 4g+3 of a 32 x 32 tile, channels 8g + 4 half + 0..3:
    // four bf16 values = one 8-byte LDS write; the block is read back row-wise, 16 bytes per lane.
    typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
    typedef float f32x2 __attribute__((ext_vector_type(2)));
    uint8_t* stage = lds + wave * EPI_WAVE;
    v4f slv[2][4];  // channel scales of the branch, in register order
#pragma unroll
    for (int cbi = 0; cbi < 2; ++cbi) {
        if (!BLK && NK > 0) {
#pragma unroll
            for (int g = 0; g < 4; ++g) slv[cbi][g] = *(const v4f*)(lds_sl + wave * 64 + cbi * 32 + 8 * g + 4 * half);
        }
    }
    const int wr_off = l32 * EPI_ROW + half * 8;
    const int rd_row = lane >> 3, rd_seg = lane & 7;
    // With one 64-chunk of the rank the intermediate codes of the other three row blocks are requested before the first
    // output store: the vector-memory counter retires in order, so a wait for a load issued after a store also waits for
    // that store's acknowledgement, and no such wait is left in the epilogue.  (Two chunks: one row block ahead; registers.)
    if constexpr (!EARLY) {
        load_lf();
        load_tq(0);
    }
    if constexpr (TQ_ALL) {
#pragma unroll
        for (int rbi = 1; rbi < NRB; ++rbi) load_tq(rbi);
    }
    // The stores are buffer stores through a descriptor that ends with the wavefront's 128 bytes of the tile's last valid
    // row: rows past M are out of range and dropped by the hardware, so the stores need no branch -- and only stores the
    // compiler can count let it wait for a load issued before them without waiting for the stores themselves.
    const int rows_valid = p.M - rb0 * 32 < NRB * 32 ? p.M - rb0 * 32 : NRB * 32;
    const __amdgpu_buffer_rsrc_t rs_y = __builtin_amdgcn_make_buffer_rsrc(
        (void*)(p.Y + (size_t)(rb0 * 32) * p.ldy + cb0 * 32), 0, (int)((rows_valid - 1) * p.ldy * 2 + 128), RSRC_FLAGS);
    uint32_t yoff = (uint32_t)(rd_row * (int)p.ldy * 2 + rd_seg * 16);
    const uint32_t ystep = (uint32_t)(8 * (int)p.ldy * 2);
    v4i ov[4];
#pragma unroll
    for (int rbi = 0; rbi < NRB; ++rbi) {
        const int rbase = (rb0 + rbi) * 32;
        v16f a2[2];
#pragma unroll
        for (int cbi = 0; cbi < 2; ++cbi) {
            a2[cbi] = v16f{0};
#pragma unroll
            for (int kk = 0; kk < NKF; ++kk)
                a2[cbi] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(lf[cbi][kk], tf[TQ_ALL ? rbi : 0][kk], a2[cbi], 0, 0, 0, 0, 0, 0);
        }
        if (!TQ_ALL && rbi + 1 < NRB) load_tq(rbi + 1);
        const float stl = (!BLK && NK > 0) ? lds_st[rbi * 32 + l32] : 0.f;  // this lane's token
        float y[2][16];
#pragma unroll
        for (int cbi = 0; cbi < 2; ++cbi)
#pragma unroll
            for (int i = 0; i < 16; ++i) {
                if (BLK) {
                    y[cbi][i] = t[rbi][cbi][i];
                } else if (NK == 0) {  // rank 0: the branch term is +0, whatever the (unused, possibly unwritten) scales hold
                    y[cbi][i] = __fadd_rn(t[rbi][cbi][i], 0.f);
                } else {
                    // two vector instructions per output: the scaled branch term enters through a fused multiply-add
                    // (the fp32 result is compared against a sum rounded once, within an accumulation bound)
                    y[cbi][i] = __builtin_fmaf(__fmul_rn(a2[cbi][i], stl), slv[cbi][i >> 2][i & 3], t[rbi][cbi][i]);
                }
            }
#pragma unroll
        for (int cbi = 0; cbi < 2; ++cbi) {
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                const bf16x2 h0 = __builtin_convertvector(f32x2{y[cbi][4 * g], y[cbi][4 * g + 1]}, bf16x2);
                const bf16x2 h1 = __builtin_convertvector(f32x2{y[cbi][4 * g + 2], y[cbi][4 * g + 3]}, bf16x2);
                *(v2i*)(stage + wr_off + cbi * 64 + g * 16) = v2i{__builtin_bit_cast(int, h0), __builtin_bit_cast(int, h1)};
            }
            if (DBG) {
#pragma unroll
                for (int i = 0; i < 16; ++i) {
                    const int row = rbase + l32;
                    const int col = (cb0 + cbi) * 32 + 8 * (i >> 2) + 4 * half + (i & 3);
                    if (row < p.M && p.dbg_y32) p.dbg_y32[(size_t)row * p.N + col] = y[cbi][i];
                }
            }
        }
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const uint8_t* src = stage + (q * 8 + rd_row) * EPI_ROW + rd_seg * 16;
            const v2i lo = *(const v2i*)src, hi = *(const v2i*)(src + 8);
            ov[q] = v4i{lo[0], lo[1], hi[0], hi[1]};
        }
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            __builtin_amdgcn_raw_buffer_store_b128(__builtin_bit_cast(u4, ov[q]), rs_y, yoff, 0, 0);
            yoff += ystep;
        }
    }
}

// Grid: the first n_full workgroups compute whole tiles (dealt round-robin to the XCDs, each XCD one contiguous run of the
// panel order); the tiles left over, if they were split (see the launcher), follow as two half tiles each.
template <int NK, bool DBG, bool BLK, int BFMT = 0>
__global__ __launch_bounds__(256, 2) void mx_fwd_kernel(MxFwdParams p)
{
    __shared__ __attribute__((aligned(16))) uint8_t lds[mxf::LDS_TOTAL];
    const int b = (int)blockIdx.x;
    auto xcd_order = [](int i, int n) {
        const int per = n >> 3, rem = n & 7, xcd = i & 7, loc = i >> 3;
        return xcd * per + (xcd < rem ? xcd : rem) + loc;
    };
    int tile_m, tile_n;
    if (b < p.n_full) {
        panel_tile(xcd_order(b, p.n_full), p.tilesM, p.tilesN, p.panel, tile_m, tile_n);
        mx_fwd_tile<NK, DBG, BLK, BFMT, 4>(p, lds, tile_m * 4, tile_n);
    } else {
        const int hh = xcd_order(b - p.n_full, 2 * (p.tilesM * p.tilesN - p.n_full));
        panel_tile(p.n_full + (hh >> 1), p.tilesM, p.tilesN, p.panel, tile_m, tile_n);
        const int rb0 = tile_m * 4 + (hh & 1) * 2;
        if (rb0 >= p.nrb) return;  // lower half of a partial last row tile
        mx_fwd_tile<NK, DBG, BLK, BFMT, 2>(p, lds, rb0, tile_n);
    }
}

template <int NK, bool BLK, int BFMT = 0>
static void mx_fwd_launch(const MxFwdParams& p, hipStream_t s)
{
    dim3 grid((unsigned)(p.n_full + 2 * (p.tilesM * p.tilesN - p.n_full))), block(256);
    if (p.dbg_y32)
        hipLaunchKernelGGL((mx_fwd_kernel<NK, true, BLK, BFMT>), grid, block, 0, s, p);
    else
        hipLaunchKernelGGL((mx_fwd_kernel<NK, false, BLK, BFMT>), grid, block, 0, s, p);
}

static int mx_workgroup_slots()  // two workgroups (of up to 256 registers per lane) per compute unit
{
    static int cached[64] = {0};
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return 512;
    if (cached[dev] == 0) {
        int cus = 0;
        if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cus <= 0) cus = 256;
        cached[dev] = 2 * cus;
    }
    return cached[dev];
}

hipError_t launch_fwd_mx(const Dims& d, const uint8_t* packed, const uint8_t* act, int64_t M, uint16_t* Y, int64_t ldy,
                         const lq_fwd_debug* dbg, hipStream_t s)
{
    const PackedLayout pl = packed_layout(d);
    const ActLayout al = act_layout(d, M);
    MxFwdParams p;
    p.xc = act + al.off_xq;
    p.xe = act + al.off_sx;
    p.tq8 = act + al.off_tq;
    p.st = (const float*)(act + al.off_st);
    p.pc = packed + pl.off_pq;
    p.pe = packed + pl.off_sw;
    p.l8 = packed + pl.off_lq;
    p.sl = (const float*)(packed + pl.off_sl);
    p.Y = Y;
    p.ldy = ldy;
    p.M = (int)M;
    p.N = (int)d.N;
    p.C64 = d.C64;
    p.CQ = (d.C64 + 3) / 4;
    p.S = d.C64 / 2;
    p.rp = d.rp;
    p.nrb = (int)(al.Mp / 32);
    p.tilesM = (p.nrb + 3) / 4;
    p.tilesN = (p.N + 255) / 256;
    p.panel = panel_width(p.tilesN, p.C64);
    // Whole generations of the grid (two workgroups per CU) use whole tiles.  A last generation that fills at most a
    // quarter of the slots is cut into half tiles: one per CU instead of one per second CU (16384 x 4608 -> 1152: 57.6 ->
    // 54.3 us, 16384 x 1152 -> 1152: 22.4 -> 21.3 us).
    {
        const int tiles = p.tilesM * p.tilesN, slots = mx_workgroup_slots() & ~7;
        const int rest = tiles % slots;
        p.n_full = (tiles > slots && 4 * rest <= slots) ? tiles - rest : tiles;
    }
    p.dbg_y32 = dbg ? dbg->y32 : nullptr;
    if (d.mxb_elem == 6) {
        switch (p.rp >> 6) {
            case 0: mx_fwd_launch<0, false>(p, s); break;
            case 1: mx_fwd_launch<1, true, 2>(p, s); break;
            default: mx_fwd_launch<2, true, 2>(p, s); break;
        }
    } else if (d.mxb) {  // sl / st hold the E8M0 scale dwords of L / of the intermediate
        switch (p.rp >> 6) {
            case 0: mx_fwd_launch<0, false>(p, s); break;
            case 1: mx_fwd_launch<1, true>(p, s); break;
            default: mx_fwd_launch<2, true>(p, s); break;
        }
    } else {
        switch (p.rp >> 6) {
            case 0: mx_fwd_launch<0, false>(p, s); break;
            case 1: mx_fwd_launch<1, false>(p, s); break;
            default: mx_fwd_launch<2, false>(p, s); break;
        }
    }
    return hipGetLastError();
}

}  // namespace lq

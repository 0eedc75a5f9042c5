// Offline packing for the INT family (paper Fig. 1 caption and Eq. 5):
//   Q2(R), Q2(L) with one scale per row; P = W - deq(Q2 L) deq(Q2 R) accumulated in fp64 and
//   rounded once to fp32; Q1(P) = INT4 with one fp32 scale per group of g values along K
//   (SINT4-style blocks, App. A.3), or the literal SINT4 blocks: 64 values, FP16 scale.  Also the inverse
//   views used by tests.
// Quantiser: s = amax / qmax, code = rne(v * (qmax / amax)), symmetric range, all-zero -> s = 1.
#include "lq_internal.h"

namespace lq {

__device__ __forceinline__ float wave_max(float v)
{
#pragma unroll
    for (int o = 32; o >= 1; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, 64));
    return v;
}

__device__ __forceinline__ void scale_pair(float amax, float qmax, float* s, float* inv)
{
    if (amax == 0.0f) {
        *s = 1.0f;
        *inv = 1.0f;
    } else {
        *s = amax / qmax;
        *inv = qmax / amax;
    }
}

__device__ __forceinline__ int quant_code(float v, float inv, float qmax)
{
    float r = rintf(v * inv);
    r = fminf(fmaxf(r, -qmax), qmax);
    return (int)r;
}

// byte offset of R code (j,k) in the activation kernel's operand order:
// [chunk = k/64][jb = j/16][lane = j%16 + 16*((k%64)/16)][k%16]
__device__ __forceinline__ size_t rq_offset(int j, int k, int r)
{
    const int c = k >> 6, kq = (k & 63) >> 4;
    return ((size_t)((size_t)c * (r >> 4) + (j >> 4)) * 64 + (j & 15) + 16 * kq) * 16 + (k & 15);
}

// ---- Q2(R): one workgroup per row j ------------------------------------------------------
__global__ __launch_bounds__(256) void pack_r_kernel(const float* R, int K, int r, float qmax,
                                                     int8_t* rq, float* sr)
{
    __shared__ float red[4];
    const int j = blockIdx.x, tid = threadIdx.x;
    float a = 0.f;
    for (int k = tid; k < K; k += 256) a = fmaxf(a, fabsf(R[(size_t)j * K + k]));
    a = wave_max(a);
    if ((tid & 63) == 0) red[tid >> 6] = a;
    __syncthreads();
    a = fmaxf(fmaxf(red[0], red[1]), fmaxf(red[2], red[3]));
    float s, inv;
    scale_pair(a, qmax, &s, &inv);
    if (tid == 0) sr[j] = s;
    for (int k = tid; k < K; k += 256)
        rq[rq_offset(j, k, r)] = (int8_t)quant_code(R[(size_t)j * K + k], inv, qmax);
}

// ---- Q2(L): one thread per row n ---------------------------------------------------------
__global__ __launch_bounds__(256) void pack_l_kernel(const float* L, int N, int r, int rp,
                                                     float qmax, int8_t* lq, float* sl)
{
    const int n = blockIdx.x * 256 + threadIdx.x;
    if (n >= N) return;
    float a = 0.f;
    for (int j = 0; j < r; ++j) a = fmaxf(a, fabsf(L[(size_t)n * r + j]));
    float s, inv;
    scale_pair(a, qmax, &s, &inv);
    sl[n] = s;
    for (int j = 0; j < rp; ++j)
        lq[(size_t)n * rp + j] = (j < r) ? (int8_t)quant_code(L[(size_t)n * r + j], inv, qmax) : (int8_t)0;
}

// ---- residual + Q1: one wavefront per (n, group) -------------------------------------------
template <int GC>
__global__ __launch_bounds__(256) void pack_p_kernel(const float* W, const float* L, const float* R,
                                                     int N, int K, int r, int rp, int from_q,
                                                     const int8_t* lq, const float* sl,
                                                     const int8_t* rq, const float* sr,
                                                     uint8_t* pq, float* swT, int ga)
{
    const int lane = threadIdx.x & 63;
    const int G = K / (64 * GC), C64 = K >> 6;
    const size_t wid = (size_t)blockIdx.x * 4 + (threadIdx.x >> 6);
    if (wid >= (size_t)N * G) return;
    const int n = (int)(wid / G), gi = (int)(wid % G);
    float P[GC];
    float a = 0.f;
#pragma unroll
    for (int cc = 0; cc < GC; ++cc) {
        const int k = (gi * GC + cc) * 64 + lane;
        double d = 0.0;
        for (int j = 0; j < r; ++j) {
            float lh, rh;
            if (from_q) {
                lh = (float)lq[(size_t)n * rp + j] * sl[n];
                rh = (float)rq[rq_offset(j, k, r)] * sr[j];
            } else {
                lh = L[(size_t)n * r + j];
                rh = R[(size_t)j * K + k];
            }
            d = fma((double)lh, (double)rh, d);
        }
        P[cc] = (float)((double)W[(size_t)n * K + k] - d);
        a = fmaxf(a, fabsf(P[cc]));
    }
    a = wave_max(a);
    float s, inv;
    if (ga) {  // FP16 scale, stored as its bits; codes against the stored scale
        const uint32_t bits = sint4_scale(a, &inv);
        if (lane == 0) ((uint32_t*)swT)[(size_t)gi * N + n] = bits;
    } else {
        scale_pair(a, 7.0f, &s, &inv);
        if (lane == 0) swT[(size_t)gi * N + n] = ldexpf(s, 6);
    }
#pragma unroll
    for (int cc = 0; cc < GC; ++cc) {
        const int k = (gi * GC + cc) * 64 + lane;
        const int q = quant_code(P[cc], inv, 7.0f);
        // 6-bit fields: lane (half = lane / 32, i = lane % 32) owns bits 6i .. 6i+5 of its half's 192-bit operand;
        // the six dwords of a half are OR-reduced over its 32 lanes
        const int i = lane & 31, bit = 6 * i;
        const uint64_t v = (uint64_t)f6_field(q) << (bit & 31);
        uint32_t mine = 0u;
#pragma unroll
        for (int dd = 0; dd < 6; ++dd) {
            uint32_t w = (bit >> 5) == dd ? (uint32_t)v : (bit >> 5) + 1 == dd ? (uint32_t)(v >> 32) : 0u;
#pragma unroll
            for (int o = 16; o >= 1; o >>= 1) w |= __shfl_xor(w, o, 64);
            if (i == dd) mine = w;
        }
        if (i < 6) *(uint32_t*)(pq + f6_chunk_offset(n, k, C64) + f6_dword_offset((n & 31) + 32 * (lane >> 5), i)) = mine;
    }
}

// blob header (offline packing: a launch of its own; the activation kernels write theirs themselves)
__global__ void write_tag_kernel(uint32_t* dst, BlobTag t) { write_tag(dst, t); }
hipError_t launch_write_tag(uint8_t* blob, const BlobTag& t, hipStream_t s)
{
    hipLaunchKernelGGL(write_tag_kernel, dim3(1), dim3(64), 0, s, (uint32_t*)blob, t);
    return hipGetLastError();
}

// reciprocals of the smoothing vector (gamma == nullptr: ones)
__global__ __launch_bounds__(256) void smooth_recip_kernel(const float* gamma, int Ks, int K, float* rg)
{
    const int k = blockIdx.x * 256 + threadIdx.x;
    if (k < K) rg[k] = (gamma && k < Ks) ? __fdiv_rn(1.0f, gamma[k]) : 1.0f;  // (k >= Ks: layout padding)
}

hipError_t launch_set_smoothing(const Dims& d, const float* gamma, uint8_t* packed, hipStream_t s)
{
    const PackedLayout pl = packed_layout(d);
    hipLaunchKernelGGL(smooth_recip_kernel, dim3((unsigned)((d.K + 255) / 256)), dim3(256), 0, s, gamma, (int)d.Ks, (int)d.K,
                       (float*)(packed + pl.off_rg));
    return hipGetLastError();
}

hipError_t launch_pack_int(const Dims& d, int from_q, const float* W, const float* L,
                           const float* R, uint8_t* packed, hipStream_t s)
{
    const PackedLayout pl = packed_layout(d);
    int8_t* lq = (int8_t*)(packed + pl.off_lq);
    float* sl = (float*)(packed + pl.off_sl);
    int8_t* rq = (int8_t*)(packed + pl.off_rq);
    float* sr = (float*)(packed + pl.off_sr);
    uint8_t* pq = packed + pl.off_pq;
    float* swT = (float*)(packed + pl.off_sw);
    const int N = (int)d.N, K = (int)d.K;
    if (d.r > 0) {
        hipLaunchKernelGGL(pack_r_kernel, dim3(d.r), dim3(256), 0, s, R, K, d.r, (float)d.qmax_bw, rq, sr);
        hipLaunchKernelGGL(pack_l_kernel, dim3((N + 255) / 256), dim3(256), 0, s, L, N, d.r, d.rp,
                           (float)d.qmax_bw, lq, sl);
    } else {
        // no branch: sl must still hold finite values (the forward multiplies 0 by it)
        hipLaunchKernelGGL(pack_l_kernel, dim3((N + 255) / 256), dim3(256), 0, s, (const float*)nullptr, N, 0, 0,
                           1.0f, lq, sl);
    }
    if (d.smooth) {
        const hipError_t e = launch_set_smoothing(d, nullptr, packed, s);
        if (e != hipSuccess) return e;
    }
    const size_t waves = (size_t)N * d.G;
    const unsigned blocks = (unsigned)((waves + 3) / 4);
    if (d.g == 64)
        hipLaunchKernelGGL(pack_p_kernel<1>, dim3(blocks), dim3(256), 0, s, W, L, R, N, K, d.r, d.rp, from_q, lq,
                           sl, rq, sr, pq, swT, d.ga ? 1 : 0);
    else
        hipLaunchKernelGGL(pack_p_kernel<2>, dim3(blocks), dim3(256), 0, s, W, L, R, N, K, d.r, d.rp, from_q, lq,
                           sl, rq, sr, pq, swT, 0);
    return hipGetLastError();
}

// ---- plain views ----------------------------------------------------------------------------
__global__ __launch_bounds__(256) void unpack_w_kernel(const uint8_t* packed, PackedLayout pl, int N, int K,
                                                       int r, int rp, int g, int ga, lq_weights_view out)
{
    const size_t idx = (size_t)blockIdx.x * 256 + threadIdx.x;
    const int C64 = K >> 6, G = K / g;
    if (idx < (size_t)N * K) {
        const int n = (int)(idx / K), k = (int)(idx % K);
        if (out.pq) {
            out.pq[idx] = (int8_t)f6_get(packed + pl.off_pq, n, k, C64);
        }
    }
    if (idx < (size_t)N * G && out.sw) {
        const int n = (int)(idx / G), gi = (int)(idx % G);
        out.sw[idx] = ga ? f16_bits_value(((const uint32_t*)(packed + pl.off_sw))[(size_t)gi * N + n])
                         : ldexpf(((const float*)(packed + pl.off_sw))[(size_t)gi * N + n], -6);
    }
    if (idx < (size_t)N * r && out.lq) {
        const int n = (int)(idx / r), j = (int)(idx % r);
        out.lq[idx] = ((const int8_t*)(packed + pl.off_lq))[(size_t)n * rp + j];
    }
    if (idx < (size_t)N && out.sl) out.sl[idx] = ((const float*)(packed + pl.off_sl))[idx];
    if (idx < (size_t)r * K && out.rq) {
        const int j = (int)(idx / K), k = (int)(idx % K);
        out.rq[idx] = ((const int8_t*)(packed + pl.off_rq))[rq_offset(j, k, r)];
    }
    if (idx < (size_t)r && out.sr) out.sr[idx] = ((const float*)(packed + pl.off_sr))[idx];
}

hipError_t launch_unpack_weights_int(const Dims& d, const uint8_t* packed, const lq_weights_view* out,
                                     hipStream_t s)
{
    const PackedLayout pl = packed_layout(d);
    const size_t n = (size_t)(d.N > d.r ? d.N : d.r) * (d.K > d.r ? d.K : d.r);  // covers N x K, r x K and N x r
    hipLaunchKernelGGL(unpack_w_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, s, packed, pl, (int)d.N,
                       (int)d.K, d.r, d.rp, d.g, d.ga ? 1 : 0, *out);
    return hipGetLastError();
}

__global__ __launch_bounds__(256) void unpack_a_kernel(const uint8_t* act, ActLayout al, int M, int K, int r,
                                                       int rp, int ga, lq_act_view out)
{
    const size_t idx = (size_t)blockIdx.x * 256 + threadIdx.x;
    const int C64 = K >> 6;
    if (idx < (size_t)M * K && out.xq) {
        const int m = (int)(idx / K), k = (int)(idx % K);
        out.xq[idx] = (int8_t)f6_get(act + al.off_xq, m, k, C64);
    }
    if (ga) {
        if (idx < (size_t)M * C64 && out.sx) {
            const int m = (int)(idx / C64), gi = (int)(idx % C64);
            out.sx[idx] = f16_bits_value(((const uint32_t*)(act + al.off_sx))[sxg_index(m, gi, (int)((al.Mp + 127) / 128))]);
        }
    } else if (idx < (size_t)M && out.sx) {
        out.sx[idx] = ((const float*)(act + al.off_sx))[idx];
    }
    if (idx < (size_t)M && out.st) out.st[idx] = ((const float*)(act + al.off_st))[idx];
    if (idx < (size_t)M * r && out.tq) {
        const int m = (int)(idx / r), j = (int)(idx % r);
        out.tq[idx] = ((const int8_t*)(act + al.off_tq))[(size_t)m * rp + j];
    }
}

hipError_t launch_unpack_act_int(const Dims& d, const uint8_t* act, int64_t M, const lq_act_view* out,
                                 hipStream_t s)
{
    const ActLayout al = act_layout(d, M);
    const size_t n = (size_t)M * (d.K > d.r ? d.K : d.r);
    hipLaunchKernelGGL(unpack_a_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, s, act, al, (int)M,
                       (int)d.K, d.r, d.rp, d.ga ? 1 : 0, *out);
    return hipGetLastError();
}

}  // namespace lq

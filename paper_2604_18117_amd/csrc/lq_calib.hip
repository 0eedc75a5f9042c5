// Data-free calibration of the low-rank factors (Section 3.2, Eq. 4; gradients of App. B.2): one Adam step on
//     loss(L, R) = mean ( Q1(W + L R) - W - L R )^2
// for the main quantiser Q1 of the configuration: INT4 in groups of 64 | 128 along K with fp32 scales, SINT4 blocks with
// FP16 scales, MXFP4 or MXINT4 (blocks of 32, E8M0 scale).  Four launches per step:
//   calib_err_kernel   V = W + L R (fp32 FMA chain over ascending j), E = deq(Q1(V)) - V, partial sums of E^2
//   calib_grad_l_kernel  grad_L = -2/(N K) E R^T      (fp32 MFMA, contraction split over the wavefronts of a workgroup)
//   calib_grad_r_kernel  partials of L^T E over row ranges
//   calib_adam_kernel    grad_R = -2/(N K) * (sum of the partials), Adam update of L and R, loss = sum of its partials / (N K)
// No atomics: every sum has a fixed order, so a step is reproducible bit for bit.
#include "lq_internal.h"

namespace lq {

typedef float v4f __attribute__((ext_vector_type(4)));

// column groups a wavefront of calib_err_kernel owns one of: the INT scale groups, or 64-chunks (two MX blocks)
static int calib_groups(const Dims& d) { return (d.mx || d.mxi) ? d.C64 : d.G; }

// Row ranges the contraction of grad_R = L^T E is split into (each range a multiple of 16 rows): enough workgroups
// (K / 32 per range) to fill the device, at most 16 ranges.
static int calib_splits(const Dims& d)
{
    const int blocks = (int)(d.N / 16), per = (int)(d.K / 32);
    int best = 1;
    for (int s = 1; s <= 16; ++s) {
        if (blocks % s) continue;
        best = s;
        if (s * per >= 256) break;
    }
    return best;
}

CalibLayout calib_layout(const Dims& d)
{
    CalibLayout cl;
    const size_t nl = (size_t)d.N * d.r * 4, nr = (size_t)d.r * d.K * 4;
    size_t o = 0;
    cl.off_L = o;  o = align256(o + nl);
    cl.off_R = o;  o = align256(o + nr);
    cl.off_mL = o; o = align256(o + nl);
    cl.off_vL = o; o = align256(o + nl);
    cl.off_mR = o; o = align256(o + nr);
    cl.off_vR = o; o = align256(o + nr);
    cl.off_gL = o; o = align256(o + nl);
    cl.off_gR = o; o = align256(o + nr);
    cl.off_E = o;  o = align256(o + (size_t)d.N * d.K * 4);
    cl.n_lp = (int)(d.N / 16) * ((calib_groups(d) + 3) / 4) * 4;  // one partial per wavefront of calib_err_kernel
    cl.off_lp = o; o = align256(o + (size_t)cl.n_lp * 4);
    cl.off_gRp = o; o = align256(o + (size_t)calib_splits(d) * nr);
    cl.total = o;
    return cl;
}

// Maximum over the 64 lanes, returned in every lane: four cross-lane steps inside each row of 16 lanes on the
// vector ALU's data-parallel-primitive path (no LDS traffic), then the four row results through scalar registers.
template <int CTRL>
__device__ __forceinline__ float dpp_max(float v)
{
    const int o = __builtin_amdgcn_update_dpp(0, __float_as_int(v), CTRL, 0xF, 0xF, false);
    return fmaxf(v, __int_as_float(o));
}
// HALF = false: maximum over the wavefront; HALF = true: over the lane's half (lanes 0..31 | 32..63 = one MX block)
template <bool HALF>
__device__ __forceinline__ float wave_max_f(float v, int lane)
{
    v = dpp_max<0xB1>(v);   // quad_perm [1,0,3,2]
    v = dpp_max<0x4E>(v);   // quad_perm [2,3,0,1]
    v = dpp_max<0x141>(v);  // row_half_mirror
    v = dpp_max<0x140>(v);  // row_mirror
    const float r0 = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), 0));
    const float r1 = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), 16));
    const float r2 = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), 32));
    const float r3 = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), 48));
    if constexpr (HALF) return lane < 32 ? fmaxf(r0, r1) : fmaxf(r2, r3);
    return fmaxf(fmaxf(r0, r1), fmaxf(r2, r3));
}

// MX block scales and elements (App. A.3), the arithmetic of the MX pack kernels:
// MXFP4: scale byte floor(log2 amax) - 2 + 127 clamped at 0; E2M1 element by the hardware converter (nearest even, saturating)
__device__ __forceinline__ uint32_t mxfp4_scale_byte(float amax)
{
    const int e = (int)((__float_as_uint(amax) >> 23) & 0xFFu) - 2;
    return (amax == 0.0f || e < 0) ? 0u : (uint32_t)e;
}
__device__ __forceinline__ float e8m0_as_float(uint32_t E) { return E ? __uint_as_float(E << 23) : __uint_as_float(0x00400000u); }
__device__ __forceinline__ float e2m1_value(uint32_t c)  // 1 sign, 2 exponent (bias 1), 1 mantissa bit
{
    const uint32_t m = c & 7u;
    const float mag = m < 2u ? 0.5f * (float)m : ldexpf(1.0f + 0.5f * (float)(m & 1u), (int)(m >> 1) - 1);
    return (c & 8u) ? -mag : mag;
}
// MXINT4: shared exponent = the fp32 exponent field of amax; code = clamp(rne(v 2^(2 - s)), -7, 7), value = code 2^(s - 2)
__device__ __forceinline__ float mxint4_round(float v, uint32_t field)
{
    const int s = (int)field - 127;
    const float q = fminf(fmaxf(rintf(ldexpf(v, 2 - s)), -7.0f), 7.0f);
    return ldexpf(q, s - 2);
}
__device__ __forceinline__ float wave_sum_f(float v)
{
#pragma unroll
    for (int o = 32; o >= 1; o >>= 1) v = __fadd_rn(v, __shfl_xor(v, o, 64));
    return v;
}

// A workgroup owns 16 rows of W and four consecutive K groups, one per wavefront; lane = column within a 64-chunk.
// The 16 x r block of L sits in LDS (uniform-address reads broadcast), the r values of R for the lane's column(s)
// stream through registers four rows of R at a time.  Many small workgroups: the loop is a chain of L2 round
// trips, hidden by occupancy.
// Q: 0 INT4 groups of 64 * GC (fp32 scale), 1 SINT4 blocks, 2 MXFP4, 3 MXINT4 (1..3: GC = 1; 2, 3: two blocks of 32 per wavefront).
template <int GC, int Q>
__global__ __launch_bounds__(256) void calib_err_kernel(const float* W, const float* L, const float* R, float* E, float* lp,
                                                        int N, int K, int r)
{
    extern __shared__ __attribute__((aligned(16))) float sL[];  // [16][r]
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int G = K / (64 * GC), GQ = (G + 3) / 4;
    const int n0 = (blockIdx.x / GQ) * 16;
    for (int i = tid * 4; i < 16 * r; i += 256 * 4) *(v4f*)&sL[i] = *(const v4f*)&L[(size_t)n0 * r + i];
    __syncthreads();
    float lsum = 0.f;
    const int g = (blockIdx.x % GQ) * 4 + wave;
    if (g < G) {
        const int col0 = g * GC * 64 + lane;
        float v[16][GC];
#pragma unroll
        for (int row = 0; row < 16; ++row)
#pragma unroll
            for (int c = 0; c < GC; ++c) v[row][c] = W[(size_t)(n0 + row) * K + col0 + c * 64];
        // 16 rows of R at a time: all their loads are in flight together (one L2 round trip per 16 rank indices)
        for (int j = 0; j < r; j += 16) {
            float rj[16][GC];
#pragma unroll
            for (int jj = 0; jj < 16; ++jj)
#pragma unroll
                for (int c = 0; c < GC; ++c) rj[jj][c] = R[(size_t)(j + jj) * K + col0 + c * 64];
#pragma unroll
            for (int row = 0; row < 16; ++row) {
#pragma unroll
                for (int j4 = 0; j4 < 16; j4 += 4) {
                    const v4f l4 = *(const v4f*)&sL[row * r + j + j4];
#pragma unroll
                    for (int jj = 0; jj < 4; ++jj)
#pragma unroll
                        for (int c = 0; c < GC; ++c) v[row][c] = __builtin_fmaf(l4[jj], rj[j4 + jj][c], v[row][c]);
                }
            }
        }
        float amax[16];
#pragma unroll
        for (int row = 0; row < 16; ++row) {
            float a = 0.f;
#pragma unroll
            for (int c = 0; c < GC; ++c) a = fmaxf(a, fabsf(v[row][c]));
            amax[row] = wave_max_f<(Q >= 2)>(a, lane);
        }
        // INT / SINT4 scales need correctly rounded divisions: done once for the 16 rows (lane l works on row l % 16,
        // the rows then read their pair back through scalar registers) instead of once per row by all lanes
        float sv = 1.0f, iv = 1.0f;
        if constexpr (Q <= 1) {
            float am = amax[0];
#pragma unroll
            for (int row = 1; row < 16; ++row) am = (lane & 15) == row ? amax[row] : am;
            if constexpr (Q == 1) {
                sv = f16_bits_value(sint4_scale(am, &iv));
            } else {  // branch-free: an all-zero group takes scale 1
                const float sd = __fdiv_rn(am, 7.0f), id = __fdiv_rn(7.0f, am);
                sv = am == 0.0f ? 1.0f : sd;
                iv = am == 0.0f ? 1.0f : id;
            }
        }
#pragma unroll
        for (int row = 0; row < 16; ++row) {
            const float a = amax[row];
            float s = 1.0f, inv = 1.0f;
            uint32_t eb = 0u;
            if constexpr (Q <= 1) {
                s = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(sv), row));
                inv = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(iv), row));
            } else if constexpr (Q == 2) {
                eb = mxfp4_scale_byte(a);
                s = e8m0_as_float(eb);
            } else {
                eb = (__float_as_uint(a) >> 23) & 0xFFu;
            }
#pragma unroll
            for (int c = 0; c < GC; ++c) {
                float deq;
                if constexpr (Q <= 1) {
                    float q = rintf(__fmul_rn(v[row][c], inv));
                    q = fminf(fmaxf(q, -7.0f), 7.0f);
                    deq = __fmul_rn(q, s);
                } else if constexpr (Q == 2) {
                    const uint32_t code = a != 0.0f ? (__builtin_amdgcn_cvt_scalef32_pk_fp4_f32(0u, v[row][c], 0.0f, s, 0) & 0xFu) : 0u;
                    deq = __fmul_rn(e2m1_value(code), s);
                } else {
                    deq = mxint4_round(v[row][c], eb);
                }
                const float e = __fsub_rn(deq, v[row][c]);
                E[(size_t)(n0 + row) * K + col0 + c * 64] = e;
                lsum = __fadd_rn(lsum, __fmul_rn(e, e));
            }
        }
    }
    lsum = wave_sum_f(lsum);
    if (lane == 0) lp[blockIdx.x * 4 + wave] = lsum;
}

// Gradient products on v_mfma_f32_16x16x4_f32 (fp32 in, fp32 accumulate): lane l supplies A[row l%16][k slot l/16] and
// B[col l%16][k slot l/16]; the four values a lane holds per 16-deep slice feed four MFMAs (the k order inside a slice
// is permuted the same way for both operands).  The contraction is split over the wavefronts of a workgroup (slices
// w, w + WAVES, ...) and the partial tiles are summed through LDS in wavefront order.  NT = r / 16.
//
// grad_L = scale * E R^T: a workgroup owns 16 rows of E and all r columns, so E is read once.
template <int NT>
__global__ __launch_bounds__(512) void calib_grad_l_kernel(const float* E, const float* R, float* gL, int K, float scale)
{
    constexpr int WAVES = 8;
    __shared__ __attribute__((aligned(16))) float s_acc[WAVES][NT][64][4];
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int row = lane & 15, q = lane >> 4;
    const int m0 = blockIdx.x * 16;
    v4f acc[NT];
#pragma unroll
    for (int t = 0; t < NT; ++t) acc[t] = v4f{0.f, 0.f, 0.f, 0.f};
    const float* ap = E + (size_t)(m0 + row) * K + 4 * q;
    const float* bp = R + (size_t)row * K + 4 * q;
    for (int kk = wave * 16; kk < K; kk += WAVES * 16) {
        const v4f a4 = *(const v4f*)(ap + kk);
        v4f b4[NT];
#pragma unroll
        for (int t = 0; t < NT; ++t) b4[t] = *(const v4f*)(bp + (size_t)t * 16 * K + kk);
#pragma unroll
        for (int t = 0; t < NT; ++t)
#pragma unroll
            for (int i = 0; i < 4; ++i) acc[t] = __builtin_amdgcn_mfma_f32_16x16x4f32(a4[i], b4[t][i], acc[t], 0, 0, 0);
    }
#pragma unroll
    for (int t = 0; t < NT; ++t) *(v4f*)&s_acc[wave][t][lane][0] = acc[t];
    __syncthreads();
    // wavefront w finishes tiles w, w + WAVES, ...
    for (int t = wave; t < NT; t += WAVES) {
        v4f s = *(const v4f*)&s_acc[0][t][lane][0];
#pragma unroll
        for (int w = 1; w < WAVES; ++w) {
            const v4f o = *(const v4f*)&s_acc[w][t][lane][0];
#pragma unroll
            for (int i = 0; i < 4; ++i) s[i] = __fadd_rn(s[i], o[i]);
        }
#pragma unroll
        for (int i = 0; i < 4; ++i) gL[(size_t)(m0 + 4 * q + i) * (NT * 16) + t * 16 + row] = __fmul_rn(scale, s[i]);
    }
}

// Partial grad_R = L^T E over a range of rows: a workgroup owns 32 columns of E (whole 128-byte lines per row), all r
// rows of the result, and the rows [split * rows_per, (split + 1) * rows_per) of the contraction; the partial goes to
// part[split][r][K] and the Adam kernel adds the splits in order (and applies the scale).
template <int NT, int WAVES>
__global__ __launch_bounds__(WAVES * 64) void calib_grad_r_kernel(const float* L, const float* E, float* part, int K, int rows_per)
{
    constexpr int r = NT * 16;
    __shared__ __attribute__((aligned(16))) float s_acc[WAVES][NT * 2][64][4];
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int row = lane & 15, q = lane >> 4;
    const int ct = K >> 5;
    const int n0 = ((int)blockIdx.x % ct) * 32, split = (int)blockIdx.x / ct;
    const size_t base = (size_t)split * rows_per;
    v4f acc[NT][2];
#pragma unroll
    for (int t = 0; t < NT; ++t) acc[t][0] = acc[t][1] = v4f{0.f, 0.f, 0.f, 0.f};
    const float* ap = L + (base + 4 * q) * r + row;
    const float* bp = E + (base + 4 * q) * K + n0 + row;
    for (int kk = wave * 16; kk < rows_per; kk += WAVES * 16) {
        float a4[NT][4], b4[2][4];
#pragma unroll
        for (int i = 0; i < 4; ++i) {
#pragma unroll
            for (int t = 0; t < NT; ++t) a4[t][i] = ap[(size_t)(kk + i) * r + t * 16];
            b4[0][i] = bp[(size_t)(kk + i) * K];
            b4[1][i] = bp[(size_t)(kk + i) * K + 16];
        }
#pragma unroll
        for (int t = 0; t < NT; ++t)
#pragma unroll
            for (int h = 0; h < 2; ++h)
#pragma unroll
                for (int i = 0; i < 4; ++i) acc[t][h] = __builtin_amdgcn_mfma_f32_16x16x4f32(a4[t][i], b4[h][i], acc[t][h], 0, 0, 0);
    }
#pragma unroll
    for (int t = 0; t < NT; ++t)
#pragma unroll
        for (int h = 0; h < 2; ++h) *(v4f*)&s_acc[wave][t * 2 + h][lane][0] = acc[t][h];
    __syncthreads();
    for (int th = wave; th < NT * 2; th += WAVES) {
        v4f s = *(const v4f*)&s_acc[0][th][lane][0];
#pragma unroll
        for (int w = 1; w < WAVES; ++w) {
            const v4f o = *(const v4f*)&s_acc[w][th][lane][0];
#pragma unroll
            for (int i = 0; i < 4; ++i) s[i] = __fadd_rn(s[i], o[i]);
        }
        const int t = th >> 1, h = th & 1;
#pragma unroll
        for (int i = 0; i < 4; ++i) part[((size_t)split * r + t * 16 + 4 * q + i) * K + n0 + h * 16 + row] = s[i];
    }
}

struct AdamParams {
    float lr, b1, b2, eps, ic1, ic2;  // ic = 1 / (1 - beta^t)
};

// One thread per parameter: the N x r values of L, then the r x K values of R.  Block 0 also sums the loss partials
// (thread-strided, a fixed shuffle tree per wavefront, then the four wavefronts in order).
__global__ __launch_bounds__(256) void calib_adam_kernel(float* L, float* mL, float* vL, const float* gL, size_t nL, float* R,
                                                         float* mR, float* vR, float* gR, const float* gR_part, int splits,
                                                         float gscale, size_t nR, AdamParams a, const float* lp, int n_lp,
                                                         float inv_count, float* loss)
{
    const size_t idx = (size_t)blockIdx.x * 256 + threadIdx.x;
    if (idx < nL + nR) {
        const bool isL = idx < nL;
        const size_t i = isL ? idx : idx - nL;
        float* p = isL ? L : R;
        float* m = isL ? mL : mR;
        float* v = isL ? vL : vR;
        float g;
        if (isL) {
            g = gL[i];
        } else {  // grad_R: the row-range partials in order, then the scale
            float sum = gR_part[i];
            for (int sp = 1; sp < splits; ++sp) sum = __fadd_rn(sum, gR_part[(size_t)sp * nR + i]);
            g = __fmul_rn(gscale, sum);
            gR[i] = g;
        }
        const float mm = __fadd_rn(__fmul_rn(a.b1, m[i]), __fmul_rn(1.0f - a.b1, g));
        const float vv = __fadd_rn(__fmul_rn(a.b2, v[i]), __fmul_rn(1.0f - a.b2, __fmul_rn(g, g)));
        m[i] = mm;
        v[i] = vv;
        const float den = __fadd_rn(__fsqrt_rn(__fmul_rn(vv, a.ic2)), a.eps);
        p[i] = __fsub_rn(p[i], __fdiv_rn(__fmul_rn(a.lr, __fmul_rn(mm, a.ic1)), den));
    }
    if (loss && blockIdx.x == 0) {  // block-uniform
        __shared__ float s_part[4];
        float s = 0.f;
#pragma unroll 8
        for (int i = threadIdx.x; i < n_lp; i += 256) s = __fadd_rn(s, lp[i]);
        s = wave_sum_f(s);
        if ((threadIdx.x & 63) == 0) s_part[threadIdx.x >> 6] = s;
        __syncthreads();
        if (threadIdx.x == 0)
            *loss = __fmul_rn(__fadd_rn(__fadd_rn(s_part[0], s_part[1]), __fadd_rn(s_part[2], s_part[3])), inv_count);
    }
}

__global__ __launch_bounds__(256) void calib_zero_kernel(float* p, size_t n)
{
    const size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
    if (i < n) p[i] = 0.f;
}

hipError_t launch_calib_init(const Dims& d, const float* L, const float* R, uint8_t* state, hipStream_t s)
{
    const CalibLayout cl = calib_layout(d);
    const size_t nl = (size_t)d.N * d.r * 4, nr = (size_t)d.r * d.K * 4;
    hipError_t e = hipMemcpyAsync(state + cl.off_L, L, nl, hipMemcpyDeviceToDevice, s);
    if (e != hipSuccess) return e;
    e = hipMemcpyAsync(state + cl.off_R, R, nr, hipMemcpyDeviceToDevice, s);
    if (e != hipSuccess) return e;
    // moments start at zero (one contiguous range: mL, vL, mR, vR); a kernel, so that the call can be captured in a graph
    const size_t nz = (cl.off_gL - cl.off_mL) / 4;
    hipLaunchKernelGGL(calib_zero_kernel, dim3((unsigned)((nz + 255) / 256)), dim3(256), 0, s, (float*)(state + cl.off_mL), nz);
    return hipGetLastError();
}

hipError_t launch_calib_step(const Dims& d, const float* W, uint8_t* state, int step, const lq_adam* ad, float* loss,
                             hipStream_t s)
{
    const CalibLayout cl = calib_layout(d);
    float* L = (float*)(state + cl.off_L);
    float* R = (float*)(state + cl.off_R);
    float* gL = (float*)(state + cl.off_gL);
    float* gR = (float*)(state + cl.off_gR);
    float* E = (float*)(state + cl.off_E);
    float* lp = (float*)(state + cl.off_lp);
    const int N = (int)d.N, K = (int)d.K, r = d.r;
    const unsigned lds = (unsigned)(16 * r * sizeof(float));
    const dim3 grid((unsigned)((N / 16) * ((calib_groups(d) + 3) / 4))), block(256);
    if (d.mxi)
        hipLaunchKernelGGL((calib_err_kernel<1, 3>), grid, block, lds, s, W, L, R, E, lp, N, K, r);
    else if (d.mx)
        hipLaunchKernelGGL((calib_err_kernel<1, 2>), grid, block, lds, s, W, L, R, E, lp, N, K, r);
    else if (d.ga)
        hipLaunchKernelGGL((calib_err_kernel<1, 1>), grid, block, lds, s, W, L, R, E, lp, N, K, r);
    else if (d.g == 64)
        hipLaunchKernelGGL((calib_err_kernel<1, 0>), grid, block, lds, s, W, L, R, E, lp, N, K, r);
    else
        hipLaunchKernelGGL((calib_err_kernel<2, 0>), grid, block, lds, s, W, L, R, E, lp, N, K, r);
    const float cg = (float)(-2.0 / ((double)N * (double)K));
    // grad_L (N x r): one workgroup per 16 rows of E
    const dim3 gl_grid((unsigned)(N / 16)), gl_block(512);
    switch (r >> 4) {
        case 1: hipLaunchKernelGGL((calib_grad_l_kernel<1>), gl_grid, gl_block, 0, s, E, R, gL, K, cg); break;
        case 2: hipLaunchKernelGGL((calib_grad_l_kernel<2>), gl_grid, gl_block, 0, s, E, R, gL, K, cg); break;
        case 4: hipLaunchKernelGGL((calib_grad_l_kernel<4>), gl_grid, gl_block, 0, s, E, R, gL, K, cg); break;
        case 6: hipLaunchKernelGGL((calib_grad_l_kernel<6>), gl_grid, gl_block, 0, s, E, R, gL, K, cg); break;
        default: hipLaunchKernelGGL((calib_grad_l_kernel<8>), gl_grid, gl_block, 0, s, E, R, gL, K, cg); break;
    }
    // grad_R (r x K): partials over row ranges
    const int splits = calib_splits(d), rows_per = N / splits;
    float* gRp = (float*)(state + cl.off_gRp);
    const dim3 gr_grid((unsigned)((K / 32) * splits));
    switch (r >> 4) {
        case 1: hipLaunchKernelGGL((calib_grad_r_kernel<1, 8>), gr_grid, dim3(512), 0, s, L, E, gRp, K, rows_per); break;
        case 2: hipLaunchKernelGGL((calib_grad_r_kernel<2, 8>), gr_grid, dim3(512), 0, s, L, E, gRp, K, rows_per); break;
        case 4: hipLaunchKernelGGL((calib_grad_r_kernel<4, 8>), gr_grid, dim3(512), 0, s, L, E, gRp, K, rows_per); break;
        case 6: hipLaunchKernelGGL((calib_grad_r_kernel<6, 4>), gr_grid, dim3(256), 0, s, L, E, gRp, K, rows_per); break;
        default: hipLaunchKernelGGL((calib_grad_r_kernel<8, 4>), gr_grid, dim3(256), 0, s, L, E, gRp, K, rows_per); break;
    }
    AdamParams a;
    a.lr = ad->lr;
    a.b1 = ad->beta1;
    a.b2 = ad->beta2;
    a.eps = ad->eps;
    a.ic1 = (float)(1.0 / (1.0 - pow((double)ad->beta1, (double)step)));
    a.ic2 = (float)(1.0 / (1.0 - pow((double)ad->beta2, (double)step)));
    const size_t nL = (size_t)N * r, nR = (size_t)r * K;
    hipLaunchKernelGGL(calib_adam_kernel, dim3((unsigned)((nL + nR + 255) / 256)), dim3(256), 0, s, L, (float*)(state + cl.off_mL),
                       (float*)(state + cl.off_vL), gL, nL, R, (float*)(state + cl.off_mR), (float*)(state + cl.off_vR), gR, gRp,
                       splits, cg, nR, a, lp, cl.n_lp, (float)(1.0 / ((double)N * (double)K)), loss);
    return hipGetLastError();
}

hipError_t launch_calib_unpack(const Dims& d, const uint8_t* state, const lq_calib_view* out, hipStream_t s)
{
    const CalibLayout cl = calib_layout(d);
    const size_t nl = (size_t)d.N * d.r * 4, nr = (size_t)d.r * d.K * 4;
    struct { float* dst; size_t off, bytes; } parts[] = {
        {out->L, cl.off_L, nl},   {out->R, cl.off_R, nr},   {out->mL, cl.off_mL, nl}, {out->vL, cl.off_vL, nl},
        {out->mR, cl.off_mR, nr}, {out->vR, cl.off_vR, nr}, {out->gL, cl.off_gL, nl}, {out->gR, cl.off_gR, nr},
        {out->E, cl.off_E, (size_t)d.N * d.K * 4}};
    for (auto& p : parts) {
        if (!p.dst) continue;
        hipError_t e = hipMemcpyAsync(p.dst, state + p.off, p.bytes, hipMemcpyDeviceToDevice, s);
        if (e != hipSuccess) return e;
    }
    return hipSuccess;
}

}  // namespace lq

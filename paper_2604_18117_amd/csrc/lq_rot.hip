// Rotation search for the low-rank factors (Section 3.3, Eq. 6-7): one step on an orthogonal r x r matrix Omega that
// lowers the error of quantising L Omega and Omega^T R with Q2, the product L R unchanged.
//     loss(Omega) = mean ( Q2(Z1) - Z1 )^2 + mean ( Q2(Z2) - Z2 )^2,   Z1 = L Omega (N x r),  Z2 = Omega^T R (r x K)
// Q2: the branch weight format of the configuration along the rows of Z1 and Z2, as lq_pack_weights applies it to L and R:
// symmetric integers or FP8 E4M3 with one fp32 scale per row, or MXFP8e4 / MXFP6e2 / MXINT blocks of 32 with E8M0 scales.  Z1 and Z2 are fp32 chains z = fma(a_i, b_i, z) over the rank index
// ascending (the codes depend on their rounding); the rounding has zero derivative (App. B.2), so
//     G = -2/(N r) L^T E1 - 2/(r K) R E2^T
// and the update is the Cayley SGD with momentum of the work the paper cites for it (Li et al. 2020, Algorithm 1).
// Five launches per step, no atomics, every sum in a fixed order:
//   rot_zl_kernel     one thread per row of L: the row of Z1 in blocks of 32 columns (twice with a per-row scale: row
//                     maximum, then codes), E1, partial sums of E1^2
//   rot_zr_kernel     one thread per column of R: the column of Z2 (stored in E2's place), per-wavefront row maxima
//   rot_qr_kernel     E2 = deq(Q2(Z2)) - Z2 in place, partial sums of E2^2 (row-scaled Q2 only: with block scales
//                     rot_zr_kernel forms E2 itself and a step is four launches)
//   rot_grad_kernel   partials of L^T E1 and R E2^T over strided 16-deep slices of N and K
//   rot_cayley_kernel one workgroup: G, loss, momentum, the skew-symmetric W, step length, the fixed-point passes
#include <mutex>

#include "lq_internal.h"
#include <type_traits>

namespace lq {

typedef float v4f __attribute__((ext_vector_type(4)));

constexpr int ROT_TPB = 256;
constexpr int ROT_GRAD_WGS = 64;   // slices the two contractions of the gradient are dealt to
constexpr int ROT_TMP = 3;         // r x r scratch matrices of the update kernel

RotLayout rot_layout(const Dims& d)
{
    RotLayout rl;
    const size_t rr = (size_t)d.r * d.r * 4;
    rl.nlb = (int)((d.N + ROT_TPB - 1) / ROT_TPB);
    rl.nkb = (int)((d.K + ROT_TPB - 1) / ROT_TPB);
    size_t o = 0;
    rl.off_X = o;   o = align256(o + rr);
    rl.off_M = o;   o = align256(o + rr);
    rl.off_G = o;   o = align256(o + rr);
    rl.off_E1 = o;  o = align256(o + (size_t)d.N * d.r * 4);
    rl.off_E2 = o;  o = align256(o + (size_t)d.r * d.K * 4);
    rl.off_ax = o;  o = align256(o + (size_t)rl.nkb * 4 * d.r * 4);
    rl.n_lp = rl.nlb + d.r * rl.nkb;
    rl.off_lp = o;  o = align256(o + (size_t)rl.n_lp * 4);
    rl.off_gp = o;  o = align256(o + (size_t)ROT_GRAD_WGS * rr);
    rl.off_tmp = o; o = align256(o + (size_t)ROT_TMP * rr);
    rl.total = o;
    return rl;
}

// Maximum over the 64 lanes (in every lane) on the data-parallel-primitive path.
template <int CTRL>
__device__ __forceinline__ float rot_dpp_max(float v)
{
    const int o = __builtin_amdgcn_update_dpp(0, __float_as_int(v), CTRL, 0xF, 0xF, false);
    return fmaxf(v, __int_as_float(o));
}
__device__ __forceinline__ float rot_wave_max(float v)
{
    v = rot_dpp_max<0xB1>(v);   // quad_perm [1,0,3,2]
    v = rot_dpp_max<0x4E>(v);   // quad_perm [2,3,0,1]
    v = rot_dpp_max<0x141>(v);  // row_half_mirror
    v = rot_dpp_max<0x140>(v);  // row_mirror
    const float r0 = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), 0));
    const float r1 = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), 16));
    const float r2 = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), 32));
    const float r3 = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), 48));
    return fmaxf(fmaxf(r0, r1), fmaxf(r2, r3));
}

// Sum over the workgroup (256 threads), valid in thread 0.
__device__ __forceinline__ float rot_block_sum(float v, float* red)
{
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_down(v, o);
    const int tid = threadIdx.x;
    if ((tid & 63) == 0) red[tid >> 6] = v;
    __syncthreads();
    return red[0] + red[1] + red[2] + red[3];
}

// Q2, the format lq_pack_weights gives L and R (App. A.3).  Row kinds carry one fp32 scale per row: 0 symmetric integers
// of qmax, 1 FP8 E4M3 (largest magnitude 448).  Block kinds carry an E8M0 scale per 32 values along the row: 2 MXFP8e4,
// 3 MXFP6e2, 4 MXINT of `bits`.
struct RotQ {
    int kind;
    float top;  // row kinds: qmax or 448
    int bits;   // MXINT
};

// Maximum over the lane's half of the wavefront (lanes 0..31 | 32..63 = one block of 32 columns).
__device__ __forceinline__ float rot_half_max(float v, int lane)
{
    v = rot_dpp_max<0xB1>(v);
    v = rot_dpp_max<0x4E>(v);
    v = rot_dpp_max<0x141>(v);
    v = rot_dpp_max<0x140>(v);
    const float r0 = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), 0));
    const float r1 = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), 16));
    const float r2 = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), 32));
    const float r3 = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), 48));
    return lane < 32 ? fmaxf(r0, r1) : fmaxf(r2, r3);
}

// Row kinds: scale amax / top, codes against top / amax (an all-zero row: scale 1).
__device__ __forceinline__ void rot_scale(float amax, float top, float& s, float& inv)
{
    if (amax == 0.f) {
        s = 1.f;
        inv = 1.f;
    } else {
        s = amax / top;
        inv = top / amax;
    }
}
__device__ __forceinline__ float rot_fp8_value(float u)  // nearest E4M3 number (ties to even), saturating at 448
{
    u = fminf(fmaxf(u, -448.f), 448.f);  // the converter returns NaN above 464
    const int code = __builtin_amdgcn_cvt_pk_fp8_f32(u, u, 0, false) & 0xFF;
    return __builtin_amdgcn_cvt_f32_fp8(code, 0);
}
template <int QK>  // 0: integers of qmax = top; 1: FP8 E4M3
__device__ __forceinline__ float rot_err(float z, float s, float inv, float top)
{
    if constexpr (QK == 0) {
        float c = rintf(z * inv);
        c = fminf(fmaxf(c, -top), top);
        return c * s - z;
    } else {
        return rot_fp8_value(z * inv) * s - z;
    }
}

// Block kinds: the shared exponent floor(log2 amax) - (largest element exponent: 8 for E4M3, 2 for E2M3, 0 for MXINT),
// kept in [-127, 127]; an all-zero block: -127.
__device__ __forceinline__ int rot_block_exp(float amax, const RotQ& q)
{
    if (amax == 0.f) return -127;
    const int e = __builtin_amdgcn_frexp_expf(amax) - 1 - (q.kind == 2 ? 8 : q.kind == 3 ? 2 : 0);
    return e < -127 ? -127 : e > 127 ? 127 : e;
}
__device__ __forceinline__ float rot_err_block(float z, int e, const RotQ& q)
{
    if (q.kind == 2) return __builtin_ldexpf(rot_fp8_value(__builtin_ldexpf(z, -e)), e) - z;
    if (q.kind == 3) {  // E2M3: spacing 1/8 below 2, 1/4 below 4, 1/2 up to the largest magnitude 7.5
        const float m = fminf(fabsf(__builtin_ldexpf(z, -e)), 7.5f);
        const float step = m < 2.f ? 0.125f : m < 4.f ? 0.25f : 0.5f;
        const float v = fminf(rintf(m / step) * step, 7.5f);
        return __builtin_copysignf(__builtin_ldexpf(v, e), z) - z;
    }
    const int frac = q.bits - 2;
    const float qmax = (float)((1 << (q.bits - 1)) - 1);
    float c = rintf(__builtin_ldexpf(z, frac - e));
    c = fminf(fmaxf(c, -qmax), qmax);
    return __builtin_ldexpf(c, e - frac) - z;
}

// BW neighbouring entries of the thread's row (or column) of Z: z[c] = sum_i a(i) * Om[i][j0 + c], each an fma chain over
// ascending i.  The rank index is the loop (four rows of Omega per turn, broadcast from LDS), the BW running sums are the
// registers: the thread's own operand a(i) is read again for every block of columns (L1-resident) instead of being held,
// so the register count does not grow with the rank (a first version that held the row spilled at ranks 96 and 128).
template <int R, int BW, typename AOP>
__device__ __forceinline__ void rot_chain_block(AOP a, const float* om, int j0, float (&z)[BW])
{
#pragma unroll
    for (int c = 0; c < BW; ++c) z[c] = 0.f;
    float av[4], an[4];
    a(0, av);
#pragma unroll 1
    for (int i = 0; i < R; i += 4) {
        a(i + 4 < R ? i + 4 : i, an);  // the next turn's operand, requested before this turn's arithmetic
#pragma unroll
        for (int u = 0; u < 4; ++u)
#pragma unroll
            for (int c = 0; c < BW; c += 4) {
                const v4f w = *(const v4f*)(om + (i + u) * R + j0 + c);
#pragma unroll
                for (int t = 0; t < 4; ++t) z[c + t] = __builtin_fmaf(av[u], w[t], z[c + t]);
            }
#pragma unroll
        for (int u = 0; u < 4; ++u) av[u] = an[u];
    }
}

// One thread per row n of L.  OUTZ: write Z1 = L Omega itself (the rotated factor) instead of its quantisation error.
// QK: 0 integer rows, 1 FP8 rows (one scale per row: the chains run twice, row maximum first), 2 block kinds (a block
// of 32 columns is one pass of the chains).
template <int R, bool OUTZ, int QK>
__global__ __launch_bounds__(ROT_TPB) void rot_zl_kernel(const float* __restrict__ L, const float* __restrict__ X, int N,
                                                        RotQ q, float* __restrict__ out, float* __restrict__ lp)
{
    constexpr int BW = R < 32 ? R : 32;
    extern __shared__ __attribute__((aligned(16))) float om[];
    __shared__ float red[4];
    for (int i = threadIdx.x; i < R * R; i += ROT_TPB) om[i] = X[i];
    __syncthreads();
    const int n = blockIdx.x * ROT_TPB + threadIdx.x;
    const bool ok = n < N;
    const float* lrow = L + (size_t)(ok ? n : 0) * R;  // rows past N recompute row 0 and store nothing
    auto aop = [&](int i, float (&av)[4]) {
        const v4f v = *(const v4f*)(lrow + i);
        av[0] = v[0]; av[1] = v[1]; av[2] = v[2]; av[3] = v[3];
    };
    float* orow = out + (size_t)(ok ? n : 0) * R;
    float z[BW];
    float sq = 0.f;
    if constexpr (OUTZ) {
#pragma unroll 1
        for (int j0 = 0; j0 < R; j0 += BW) {
            rot_chain_block<R, BW>(aop, om, j0, z);
            if (ok) {
#pragma unroll
                for (int c = 0; c < BW; c += 4) *(v4f*)(orow + j0 + c) = v4f{z[c], z[c + 1], z[c + 2], z[c + 3]};
            }
        }
    } else {
        float s = 1.f, inv = 1.f;
        if constexpr (QK != 2) {
            float amax = 0.f;
#pragma unroll 1
            for (int j0 = 0; j0 < R; j0 += BW) {
                rot_chain_block<R, BW>(aop, om, j0, z);
#pragma unroll
                for (int c = 0; c < BW; ++c) amax = fmaxf(amax, fabsf(z[c]));
            }
            rot_scale(amax, q.top, s, inv);
        }
#pragma unroll 1
        for (int j0 = 0; j0 < R; j0 += BW) {
            rot_chain_block<R, BW>(aop, om, j0, z);  // (row kinds: the same chains, the same bits as in the first pass)
            int eb = 0;
            if constexpr (QK == 2) {
                float amax = 0.f;
#pragma unroll
                for (int c = 0; c < BW; ++c) amax = fmaxf(amax, fabsf(z[c]));
                eb = rot_block_exp(amax, q);
            }
#pragma unroll
            for (int c = 0; c < BW; ++c) {
                if constexpr (QK == 2) z[c] = rot_err_block(z[c], eb, q);
                else z[c] = rot_err<QK>(z[c], s, inv, q.top);
                sq = __builtin_fmaf(z[c], z[c], sq);
            }
            if (ok) {
#pragma unroll
                for (int c = 0; c < BW; c += 4) *(v4f*)(orow + j0 + c) = v4f{z[c], z[c + 1], z[c + 2], z[c + 3]};
            }
        }
        const float tot = rot_block_sum(ok ? sq : 0.f, red);
        if (threadIdx.x == 0) lp[blockIdx.x] = tot;
    }
}

// One thread per column k of R: the column of Z2 = Omega^T R.  OUTZ: written to out[j][k] as it is.  Otherwise, row kinds
// of Q2: Z2 is written and the maximum magnitude of every row j over the wavefront's 64 columns is left in
// ax[4 * block + wavefront][j] (rot_qr_kernel finishes the job); block kinds: a block is 32 lanes of one row, so the error
// is formed here, written to out, and its squares are summed into lp[block].
template <int R, bool OUTZ, int QK>
__global__ __launch_bounds__(ROT_TPB) void rot_zr_kernel(const float* __restrict__ Rm, const float* __restrict__ X, int K,
                                                        RotQ q, float* __restrict__ out, float* __restrict__ ax,
                                                        float* __restrict__ lp)
{
    constexpr int BW = R < 32 ? R : 32;
    extern __shared__ __attribute__((aligned(16))) float om[];
    __shared__ float red[4];
    for (int i = threadIdx.x; i < R * R; i += ROT_TPB) om[i] = X[i];
    __syncthreads();
    const int k = blockIdx.x * ROT_TPB + threadIdx.x;
    const bool ok = k < K;
    // buffer loads: the row offset i * K travels in a scalar register and all loads share one vector offset; a column
    // past K reads finite in-range data of the next row (zeros past the end of the descriptor), and nothing computed
    // from it is stored or enters a maximum
    const __amdgpu_buffer_rsrc_t rs = __builtin_amdgcn_make_buffer_rsrc((void*)Rm, 0, R * K * 4, 0x00020000);
    auto aop = [&](int i, float (&av)[4]) {
#pragma unroll
        for (int u = 0; u < 4; ++u) av[u] = __uint_as_float(__builtin_amdgcn_raw_buffer_load_b32(rs, k * 4, (i + u) * K * 4, 0));
    };
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    float z[BW];
    float sq = 0.f;
#pragma unroll 1
    for (int j0 = 0; j0 < R; j0 += BW) {
        rot_chain_block<R, BW>(aop, om, j0, z);
#pragma unroll
        for (int c = 0; c < BW; ++c) {
            float o = z[c];
            if constexpr (!OUTZ) {
                if constexpr (QK != 2) {
                    const float m = rot_wave_max(ok ? fabsf(o) : 0.f);
                    if (lane == 0) ax[(size_t)(blockIdx.x * 4 + wave) * R + j0 + c] = m;
                } else {
                    const int eb = rot_block_exp(rot_half_max(ok ? fabsf(o) : 0.f, lane), q);
                    o = rot_err_block(o, eb, q);
                    if (ok) sq = __builtin_fmaf(o, o, sq);
                }
            }
            if (ok) out[(size_t)(j0 + c) * K + k] = o;
        }
    }
    if constexpr (!OUTZ && QK == 2) {
        const float tot = rot_block_sum(sq, red);
        if (threadIdx.x == 0) lp[blockIdx.x] = tot;
    }
}

// E2 = deq(Q2(Z2)) - Z2 in place; grid (column blocks, r).
__global__ __launch_bounds__(ROT_TPB) void rot_qr_kernel(float* __restrict__ E2, const float* __restrict__ ax, int K, int r,
                                                        int nparts, RotQ q, float* __restrict__ lp)
{
    __shared__ float red[4];
    const int j = blockIdx.y;
    float amax = 0.f;
    for (int p = 0; p < nparts; ++p) amax = fmaxf(amax, ax[(size_t)p * r + j]);
    float s, inv;
    rot_scale(amax, q.top, s, inv);
    const int k = blockIdx.x * ROT_TPB + threadIdx.x;
    float sq = 0.f;
    if (k < K) {
        const float z = E2[(size_t)j * K + k];
        const float e = q.kind == 0 ? rot_err<0>(z, s, inv, q.top) : rot_err<1>(z, s, inv, q.top);
        E2[(size_t)j * K + k] = e;
        sq = e * e;
    }
    const float tot = rot_block_sum(sq, red);
    if (threadIdx.x == 0) lp[(size_t)j * gridDim.x + blockIdx.x] = tot;
}

// Partials of  c1 L^T E1 + c2 R E2^T  (r x r): workgroup w takes the 16-deep slices w, w + gridDim.x, ... of the
// contraction over N, then of the one over K.  Thread (ty, tx) of 16 x 16 owns entries (ty + 16 a, tx + 16 b).
template <int T>
__global__ __launch_bounds__(ROT_TPB) void rot_grad_kernel(const float* __restrict__ L, const float* __restrict__ E1,
                                                          const float* __restrict__ Rm, const float* __restrict__ E2, int N,
                                                          int K, float c1, float c2, float* __restrict__ gp)
{
    constexpr int R = 16 * T;
    __shared__ float As[16][R];
    __shared__ float Bs[16][R];
    const int tid = threadIdx.x, ty = tid >> 4, tx = tid & 15;
    float acc[T][T];
#pragma unroll
    for (int a = 0; a < T; ++a)
#pragma unroll
        for (int b = 0; b < T; ++b) acc[a][b] = 0.f;
    auto contract = [&]() {
#pragma unroll
        for (int kk = 0; kk < 16; ++kk) {
            float av[T], bv[T];
#pragma unroll
            for (int a = 0; a < T; ++a) av[a] = As[kk][ty + 16 * a];
#pragma unroll
            for (int b = 0; b < T; ++b) bv[b] = Bs[kk][tx + 16 * b];
#pragma unroll
            for (int a = 0; a < T; ++a)
#pragma unroll
                for (int b = 0; b < T; ++b) acc[a][b] = __builtin_fmaf(av[a], bv[b], acc[a][b]);
        }
    };
    for (int n0 = blockIdx.x * 16; n0 < N; n0 += gridDim.x * 16) {  // rows n0 .. n0+15 of L and E1 (zero past N)
        __syncthreads();
        for (int e = tid; e < 16 * R; e += ROT_TPB) {
            const int rr = e / R, i = e - rr * R;
            const bool ok = n0 + rr < N;
            As[rr][i] = ok ? L[(size_t)(n0 + rr) * R + i] : 0.f;
            Bs[rr][i] = ok ? c1 * E1[(size_t)(n0 + rr) * R + i] : 0.f;
        }
        __syncthreads();
        contract();
    }
    for (int k0 = blockIdx.x * 16; k0 < K; k0 += gridDim.x * 16) {  // columns k0 .. k0+15 of R and E2 (K is a multiple of 64)
        __syncthreads();
        for (int e = tid; e < 16 * R; e += ROT_TPB) {
            const int i = e >> 4, kk = e & 15;
            As[kk][i] = Rm[(size_t)i * K + k0 + kk];
            Bs[kk][i] = c2 * E2[(size_t)i * K + k0 + kk];
        }
        __syncthreads();
        contract();
    }
    float* o = gp + (size_t)blockIdx.x * R * R;
#pragma unroll
    for (int a = 0; a < T; ++a)
#pragma unroll
        for (int b = 0; b < T; ++b) o[(ty + 16 * a) * R + tx + 16 * b] = acc[a][b];
}

struct RotStepParams {
    float* X;          // Omega
    float* M;          // momentum
    float* G;          // gradient of this step
    const float* gp;   // its partials
    const float* lp;   // partial sums of E1^2 (nlb) then of E2^2
    float* tmp;        // ROT_TMP scratch matrices
    float* loss;       // may be null
    int r, nlb, n_lp, nparts;
    float inv1, inv2;  // 1 / (N r), 1 / (r K)
    float lr, beta, eps, q, grad_scale;
    int s;
};

// The update, one workgroup of 1024 threads.  Three r x r work matrices and Omega; as many as fit sit in a 60 KB LDS pool
// (all four up to rank 32, three at rank 64, one at rank 96), the rest in the state's scratch area in global memory:
// the code addresses both through generic pointers.  Every phase reads what earlier phases wrote; __syncthreads orders
// those accesses within the workgroup.
// T = entries per thread and dimension in the r-deep products: thread (ty, tx) of 32 x 32 owns entries (ty + 32 a, tx + 32 b),
// so one k step loads T + T operands for T * T multiply-adds (rank 16 and 32: T = 1, 64: 2, 96: 3, 128: 4).
// ALL_LDS (rank <= 32): everything sits in the pool and the compiler sees plain LDS addresses.
constexpr int ROT_POOL = 15360;  // floats
template <int T, bool ALL_LDS>
__global__ __launch_bounds__(1024) void rot_cayley_kernel(RotStepParams p)
{
    __shared__ __attribute__((aligned(16))) float pool[ROT_POOL];
    __shared__ double red[16];
    __shared__ float bc;
    const int r = p.r, rr = r * r, tid = threadIdx.x;
    const int ty = tid >> 5, tx = tid & 31;
    __builtin_assume(r % 16 == 0 && r >= 16);
    // priority: W (read by every product of the second half), then the operands of the passes, then Omega
    float *W, *T1, *T2, *Xl;
    if constexpr (ALL_LDS) {
        W = pool;
        T1 = pool + rr;
        T2 = pool + 2 * rr;
        Xl = pool + 3 * rr;
    } else {
        const int fit = ROT_POOL / rr;
        W = 0 < fit ? pool : p.tmp;
        T1 = 1 < fit ? pool + rr : p.tmp + rr;
        T2 = 2 < fit ? pool + 2 * rr : p.tmp + 2 * rr;
        Xl = 3 < fit ? pool + 3 * rr : p.X;
    }
    // W: first beta M - G, then Wh, then W = Wh - Wh^T in place;  T1: A = (beta M - G) X^T, later Y;
    // T2: X^T (for A), B = X^T A, later X + Y
    auto block_sum = [&](double v) -> double {
#pragma unroll
        for (int o = 32; o > 0; o >>= 1) v += __shfl_down(v, o);
        __syncthreads();
        if ((tid & 63) == 0) red[tid >> 6] = v;
        __syncthreads();
        double t = 0.0;
        for (int w = 0; w < 16; ++w) t += red[w];
        return t;
    };
    // C(i, j) = sum_k A(i, k) B(k, j), each entry an fma chain over ascending k; out(i, j, value) stores it
    auto product = [&](auto A, auto B, auto out) {
        float acc[T][T];
#pragma unroll
        for (int a = 0; a < T; ++a)
#pragma unroll
            for (int b = 0; b < T; ++b) acc[a][b] = 0.f;
        const bool live = ty < r && tx < r;  // (rank 16 leaves three quarters of the workgroup idle)
        if (live) {
#pragma unroll 8
            for (int k = 0; k < r; ++k) {
                float av[T], bv[T];
#pragma unroll
                for (int a = 0; a < T; ++a) av[a] = A(ty + 32 * a, k);
#pragma unroll
                for (int b = 0; b < T; ++b) bv[b] = B(k, tx + 32 * b);
#pragma unroll
                for (int a = 0; a < T; ++a)
#pragma unroll
                    for (int b = 0; b < T; ++b) acc[a][b] = __builtin_fmaf(av[a], bv[b], acc[a][b]);
            }
#pragma unroll
            for (int a = 0; a < T; ++a)
#pragma unroll
                for (int b = 0; b < T; ++b) out(ty + 32 * a, tx + 32 * b, acc[a][b]);
        }
    };
    // loss (before the update) and gradient from their partials
    {
        double a = 0.0, b = 0.0;
        for (int i = tid; i < p.nlb; i += 1024) a += (double)p.lp[i];
        for (int i = p.nlb + tid; i < p.n_lp; i += 1024) b += (double)p.lp[i];
        const double ta = block_sum(a), tb = block_sum(b);
        if (tid == 0 && p.loss) *p.loss = (float)(ta * (double)p.inv1 + tb * (double)p.inv2);
    }
    for (int e = tid; e < rr; e += 1024) {
        double g = 0.0;
#pragma unroll 16
        for (int w = 0; w < ROT_GRAD_WGS; ++w) g += (double)p.gp[(size_t)w * rr + e];  // 16 loads in flight at a time
        const float gf = (float)((double)p.grad_scale * g);
        p.G[e] = gf;
        W[e] = p.beta * p.M[e] - gf;
        const float x = p.X[e];
        if (ALL_LDS || Xl != p.X) Xl[e] = x;
        const int i = e / r, j = e - i * r;
        T2[j * r + i] = x;  // X^T: the product below then reads rows, not columns (in LDS a column read is a 32-way bank conflict)
    }
    __syncthreads();
    product([&](int i, int k) { return W[i * r + k]; }, [&](int k, int j) { return T2[k * r + j]; },
            [&](int i, int j, float v) { T1[i * r + j] = v; });                       // A = (beta M - G) X^T
    __syncthreads();
    product([&](int i, int k) { return Xl[k * r + i]; }, [&](int k, int j) { return T1[k * r + j]; },
            [&](int i, int j, float v) { T2[i * r + j] = v; });                       // B = X^T A
    __syncthreads();
    product([&](int i, int k) { return Xl[i * r + k]; }, [&](int k, int j) { return T2[k * r + j]; },
            [&](int i, int j, float v) { W[i * r + j] = T1[i * r + j] - 0.5f * v; });  // Wh = A - 1/2 X B
    __syncthreads();
    double n2 = 0.0;
    for (int e = tid; e < rr; e += 1024) {  // W = Wh - Wh^T, each pair (i, j), (j, i) by the thread of its upper entry
        const int i = e / r, j = e - i * r;
        if (i > j) continue;
        const float w = W[e] - W[j * r + i];
        W[e] = w;
        W[j * r + i] = -w;
        if (i < j) n2 += 2.0 * (double)w * (double)w;
    }
    const double nrm2 = block_sum(n2);      // (its barriers also order W's stores before the reads below)
    if (tid == 0) {
        const float lim = 2.f * p.q / ((float)sqrt(nrm2) + p.eps);
        bc = p.lr < lim ? p.lr : lim;
    }
    __syncthreads();
    const float alpha = bc;
    product([&](int i, int k) { return W[i * r + k]; }, [&](int k, int j) { return Xl[k * r + j]; },
            [&](int i, int j, float v) {                                               // M = W X;  Y = X + alpha M
                p.M[i * r + j] = v;
                T1[i * r + j] = __builtin_fmaf(alpha, v, Xl[i * r + j]);
            });
    for (int it = 0; it < p.s; ++it) {      // Y <- X + alpha/2 W (X + Y); Y is dead once X + Y is formed, so it is updated in place
        __syncthreads();
        for (int e = tid; e < rr; e += 1024) T2[e] = Xl[e] + T1[e];
        __syncthreads();
        product([&](int i, int k) { return W[i * r + k]; }, [&](int k, int j) { return T2[k * r + j]; },
                [&](int i, int j, float v) { T1[i * r + j] = __builtin_fmaf(0.5f * alpha, v, Xl[i * r + j]); });
    }
    __syncthreads();
    for (int e = tid; e < rr; e += 1024) p.X[e] = T1[e];
}

__global__ __launch_bounds__(ROT_TPB) void rot_init_kernel(float* X, float* M, const float* X0, const float* M0, int r)
{
    const int e = blockIdx.x * ROT_TPB + threadIdx.x;
    if (e >= r * r) return;
    X[e] = X0 ? X0[e] : (e / r == e % r ? 1.f : 0.f);
    M[e] = M0 ? M0[e] : 0.f;
}

hipError_t launch_rot_init(const Dims& d, const float* Omega0, const float* Mom0, uint8_t* state, hipStream_t s)
{
    const RotLayout rl = rot_layout(d);
    hipLaunchKernelGGL(rot_init_kernel, dim3((d.r * d.r + ROT_TPB - 1) / ROT_TPB), dim3(ROT_TPB), 0, s,
                       (float*)(state + rl.off_X), (float*)(state + rl.off_M), Omega0, Mom0, d.r);
    return hipGetLastError();
}

// Q2 of the configuration: the branch weight format.
static RotQ rot_q2(const Dims& d)
{
    RotQ q;
    q.kind = d.mxi ? 4 : d.mxb ? (d.mxb_elem == 8 ? 2 : 3) : d.mx ? 1 : 0;
    q.top = q.kind == 0 ? (float)d.qmax_bw : 448.f;
    q.bits = d.mxi ? d.bw_bits : 0;
    return q;
}

template <int R, bool OUTZ>
static void rot_launch_z(const Dims& d, const RotLayout& rl, const RotQ& q, const float* L, const float* Rm, const float* X,
                         float* o1, float* o2, float* ax, float* lp, hipStream_t s)
{
    const size_t lds = (size_t)R * R * 4;
    auto go = [&](auto qk) {
        constexpr int BQ = decltype(qk)::value;
        if constexpr (R == 128) {  // Omega alone fills the 64 KB a launch may use without asking for more
            // once per device and kernel pair, so that later calls (which a caller may capture in a graph) only launch
            static bool asked[64] = {false};
            int dev = 0;
            if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) dev = 0;
            if (!asked[dev]) {
                (void)hipFuncSetAttribute((const void*)rot_zl_kernel<R, OUTZ, BQ>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
                (void)hipFuncSetAttribute((const void*)rot_zr_kernel<R, OUTZ, BQ>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
                asked[dev] = true;
            }
        }
        hipLaunchKernelGGL((rot_zl_kernel<R, OUTZ, BQ>), dim3(rl.nlb), dim3(ROT_TPB), lds, s, L, X, (int)d.N, q, o1, lp);
        hipLaunchKernelGGL((rot_zr_kernel<R, OUTZ, BQ>), dim3(rl.nkb), dim3(ROT_TPB), lds, s, Rm, X, (int)d.K, q, o2, ax,
                           lp ? lp + rl.nlb : nullptr);
    };
    // (the rotated factors themselves do not depend on Q2: one instantiation serves both)
    if (OUTZ || q.kind == 0)
        go(std::integral_constant<int, 0>{});
    else if (q.kind == 1)
        go(std::integral_constant<int, 1>{});
    else if constexpr (R >= 32)
        go(std::integral_constant<int, 2>{});
}

template <bool OUTZ>
static void rot_dispatch_z(const Dims& d, const RotLayout& rl, const RotQ& q, const float* L, const float* Rm, const float* X,
                           float* o1, float* o2, float* ax, float* lp, hipStream_t s)
{
    switch (d.r) {
        case 16: rot_launch_z<16, OUTZ>(d, rl, q, L, Rm, X, o1, o2, ax, lp, s); break;
        case 32: rot_launch_z<32, OUTZ>(d, rl, q, L, Rm, X, o1, o2, ax, lp, s); break;
        case 64: rot_launch_z<64, OUTZ>(d, rl, q, L, Rm, X, o1, o2, ax, lp, s); break;
        case 96: rot_launch_z<96, OUTZ>(d, rl, q, L, Rm, X, o1, o2, ax, lp, s); break;
        default: rot_launch_z<128, OUTZ>(d, rl, q, L, Rm, X, o1, o2, ax, lp, s); break;
    }
}

// Partial results of a step (row maxima, loss and gradient partials, the update's work matrices) for callers that
// cannot allocate: one array per device, held until the process ends.  Every element a step reads it has written before
// in that same step, so nothing needs clearing between calls; two steps that overlap on one GPU would race on it.
static __device__ __align__(256) uint8_t scratch[LQ_ROT_STATIC_SCRATCH_BYTES];

// The array's device address on the current device (host code must not use the symbol's name as an address), looked up
// once per device.
static hipError_t rot_scratch_ptr(uint8_t** out)
{
    static std::mutex mu;
    static uint8_t* ptr[64] = {nullptr};
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    if (dev < 0 || dev >= 64) return hipErrorInvalidDevice;
    std::lock_guard<std::mutex> lock(mu);
    if (!ptr[dev]) {
        void* p = nullptr;
        e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess) return e;
        if (!p) return hipErrorInvalidSymbol;
        ptr[dev] = (uint8_t*)p;
    }
    *out = ptr[dev];
    return hipSuccess;
}

size_t rot_static_scratch_needed(const Dims& d)
{
    const RotLayout rl = rot_layout(d);
    return rl.total - rl.off_ax;
}

// part: where the step's partial results live (laid out like the state blob's sections from off_ax on): inside the
// state blob, or the per-device array
static hipError_t rot_step_launches(const Dims& d, const float* L, const float* Rm, uint8_t* state, uint8_t* part,
                                    const lq_cayley* cs, float* loss, hipStream_t s);

hipError_t launch_rot_step(const Dims& d, const float* L, const float* Rm, uint8_t* state, const lq_cayley* cs, float* loss,
                           hipStream_t s)
{
    return rot_step_launches(d, L, Rm, state, state + rot_layout(d).off_ax, cs, loss, s);
}

hipError_t launch_rot_step_static(const Dims& d, const float* L, const float* Rm, uint8_t* state, const lq_cayley* cs,
                                  float* loss, hipStream_t s)
{
    uint8_t* part = nullptr;
    const hipError_t e = rot_scratch_ptr(&part);
    if (e != hipSuccess) return e;
    return rot_step_launches(d, L, Rm, state, part, cs, loss, s);
}

static hipError_t rot_step_launches(const Dims& d, const float* L, const float* Rm, uint8_t* state, uint8_t* part,
                                    const lq_cayley* cs, float* loss, hipStream_t s)
{
    const RotLayout rl = rot_layout(d);
    float* X = (float*)(state + rl.off_X);
    float* E1 = (float*)(state + rl.off_E1);
    float* E2 = (float*)(state + rl.off_E2);
    float* ax = (float*)part;
    float* lp = (float*)(part + (rl.off_lp - rl.off_ax));
    float* gp = (float*)(part + (rl.off_gp - rl.off_ax));
    const int N = (int)d.N, K = (int)d.K, r = d.r;
    const RotQ q = rot_q2(d);
    rot_dispatch_z<false>(d, rl, q, L, Rm, X, E1, E2, ax, lp, s);
    if (q.kind <= 1)
        hipLaunchKernelGGL(rot_qr_kernel, dim3(rl.nkb, r), dim3(ROT_TPB), 0, s, E2, ax, K, r, rl.nkb * 4, q, lp + rl.nlb);
    const float c1 = (float)(-2.0 / ((double)N * r)), c2 = (float)(-2.0 / ((double)r * K));
    switch (r >> 4) {
        case 1: hipLaunchKernelGGL(rot_grad_kernel<1>, dim3(ROT_GRAD_WGS), dim3(ROT_TPB), 0, s, L, E1, Rm, E2, N, K, c1, c2, gp); break;
        case 2: hipLaunchKernelGGL(rot_grad_kernel<2>, dim3(ROT_GRAD_WGS), dim3(ROT_TPB), 0, s, L, E1, Rm, E2, N, K, c1, c2, gp); break;
        case 4: hipLaunchKernelGGL(rot_grad_kernel<4>, dim3(ROT_GRAD_WGS), dim3(ROT_TPB), 0, s, L, E1, Rm, E2, N, K, c1, c2, gp); break;
        case 6: hipLaunchKernelGGL(rot_grad_kernel<6>, dim3(ROT_GRAD_WGS), dim3(ROT_TPB), 0, s, L, E1, Rm, E2, N, K, c1, c2, gp); break;
        default: hipLaunchKernelGGL(rot_grad_kernel<8>, dim3(ROT_GRAD_WGS), dim3(ROT_TPB), 0, s, L, E1, Rm, E2, N, K, c1, c2, gp); break;
    }
    RotStepParams p;
    p.X = X;
    p.M = (float*)(state + rl.off_M);
    p.G = (float*)(state + rl.off_G);
    p.gp = gp;
    p.lp = lp;
    p.tmp = (float*)(part + (rl.off_tmp - rl.off_ax));
    p.loss = loss;
    p.r = r;
    p.nlb = rl.nlb;
    p.n_lp = q.kind <= 1 ? rl.n_lp : rl.nlb + rl.nkb;
    p.nparts = ROT_GRAD_WGS;
    p.inv1 = (float)(1.0 / ((double)N * r));
    p.inv2 = (float)(1.0 / ((double)r * K));
    p.lr = cs->lr;
    p.beta = cs->beta;
    p.eps = cs->eps;
    p.q = cs->q;
    p.grad_scale = cs->grad_scale;
    p.s = cs->s;
    switch ((r + 31) >> 5) {
        case 1: hipLaunchKernelGGL((rot_cayley_kernel<1, true>), dim3(1), dim3(1024), 0, s, p); break;
        case 2: hipLaunchKernelGGL((rot_cayley_kernel<2, false>), dim3(1), dim3(1024), 0, s, p); break;
        case 3: hipLaunchKernelGGL((rot_cayley_kernel<3, false>), dim3(1), dim3(1024), 0, s, p); break;
        default: hipLaunchKernelGGL((rot_cayley_kernel<4, false>), dim3(1), dim3(1024), 0, s, p); break;
    }
    return hipGetLastError();
}

hipError_t launch_rot_apply(const Dims& d, const float* L, const float* Rm, const uint8_t* state, float* Lr, float* Rr,
                            hipStream_t s)
{
    const RotLayout rl = rot_layout(d);
    rot_dispatch_z<true>(d, rl, rot_q2(d), L, Rm, (const float*)(state + rl.off_X), Lr, Rr, nullptr, nullptr, s);
    return hipGetLastError();
}

hipError_t launch_rot_unpack(const Dims& d, const uint8_t* state, const lq_rot_view* out, hipStream_t s)
{
    const RotLayout rl = rot_layout(d);
    const size_t rr = (size_t)d.r * d.r * 4;
    struct { float* dst; size_t off, bytes; } parts[5] = {{out->Omega, rl.off_X, rr}, {out->Mom, rl.off_M, rr}, {out->G, rl.off_G, rr},
                                                         {out->E1, rl.off_E1, (size_t)d.N * d.r * 4},
                                                         {out->E2, rl.off_E2, (size_t)d.r * d.K * 4}};
    for (auto& pt : parts) {
        if (!pt.dst) continue;
        const hipError_t e = hipMemcpyAsync(pt.dst, state + pt.off, pt.bytes, hipMemcpyDeviceToDevice, s);
        if (e != hipSuccess) return e;
    }
    return hipSuccess;
}

}  // namespace lq

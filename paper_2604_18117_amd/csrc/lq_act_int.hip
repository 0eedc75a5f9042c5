// Per-call activation kernel, INT family (Section 3.4 and the low-rank branch of Fig. 1).
// One pass over X does, per token row:
//   sx = amax/7,      xq = rne(x * 7/amax)          4-bit main codes (stored as 6-bit fields s00mmm)
//   sxb = amax/qa,    xb = rne(x * qa/amax)         branch codes, kept in registers only
//   accT = xb . rq^T  (int8 MFMA, int32)            skinny contraction with Q2(R)
//   T = (float(accT) * sxb) * sr ;  st = max|T|/qa ;  tq = rne(T * qa/max|T|)
// SINT4 blocks (App. A.3; template flag GA): the main codes take one FP16 scale per 64-chunk of K instead
// of one scale per token, sx[m,g] = fp16(amax_g / 7), codes clamp(rne(x * fl(1 / sx))); the branch is unchanged.
//
// Decomposition: a workgroup of 4 wavefronts owns 16 token rows; lane l of every wavefront
// works on row l%16 and on the 16-value quarter l/16 of each 64-deep K chunk, which is
// exactly the A-operand layout of v_mfma_i32_16x16x64_i8.  The 64-chunks of K are dealt
// round-robin to the 4 wavefronts, so a whole row block lives in registers between the
// amax pass and the quantisation pass: X is read from HBM once.  Rows too long for that (MAXC = 0) are
// streamed twice through a two-chunk ring instead: once for the amax, once for the codes (the second read
// comes from the caches: a workgroup's 16 rows are at most a few hundred KB).
#include "lq_internal.h"

namespace lq {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef unsigned short us2 __attribute__((ext_vector_type(2)));

struct ActParams {
    const void* X;
    int64_t ldx;
    int M, K, C64, r, rp;
    float qa;  // qmax of the branch activation format
    const float* rg;  // reciprocals of the smoothing vector (smoothing variant only)
    const int8_t* rq;
    const float* sr;
    uint8_t* xq;
    float* sx;
    uint32_t* sxg;  // SINT4 blocks: FP16 bits of the block scales (sxg_index), tiles128 = 128-row tiles
    int tiles128, Mp;
    int8_t* tq;
    float* st;
    int8_t* dbg_xb;
    float* dbg_sxb;
    int32_t* dbg_accT;
    float* dbg_T;
    BlobTag tag;        // header of the activation blob (written by the first workgroup)
    uint32_t* tag_dst;
};

template <bool BF16>
struct XChunk;

template <>
struct XChunk<true> {  // 16 bf16 values = 8 dwords
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
struct XChunk<false> {  // 16 fp32 values
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

// Smoothing variant: 16 values of X (bf16 or fp32 source) times the reciprocals of the smoothing vector,
// held as fp32 (the products are no longer bf16 numbers).
template <bool BF16IN>
__device__ __forceinline__ void load_smoothed(XChunk<false>& xc, const void* X, size_t elem, const float* rg, bool ok)
{
    float raw[16];
    if constexpr (BF16IN) {
        XChunk<true> t;
        t.load(X, elem, ok);
#pragma unroll
        for (int i = 0; i < 16; ++i) raw[i] = t.get(i);
    } else {
        XChunk<false> t;
        t.load(X, elem, ok);
#pragma unroll
        for (int i = 0; i < 16; ++i) raw[i] = t.get(i);
    }
#pragma unroll
    for (int q = 0; q < 4; ++q) {
        v4i g = {0, 0, 0, 0};
        if (ok) g = ((const v4i*)rg)[q];
#pragma unroll
        for (int i = 0; i < 4; ++i) xc.v[4 * q + i] = __fmul_rn(raw[4 * q + i], __int_as_float(g[i]));
    }
}

__device__ __forceinline__ void scales(float amax, float qmax, float* s, float* inv)
{
    if (amax == 0.0f) {
        *s = 1.0f;
        *inv = 1.0f;
    } else {
        *s = amax / qmax;
        *inv = qmax / amax;
    }
}

// round-to-nearest-even of a value with |u| < 2^22, returned in the low bits (two's complement)
__device__ __forceinline__ uint32_t rne_bits(float u) { return __float_as_uint(__fadd_rn(u, 12582912.0f)); }

// 16 values in [-7, 7] (already scaled, fp32) -> their nearest integers as 6-bit sign-magnitude fields, code i at bits
// 6i .. 6i+5 of three dwords.  The field s00mmm is the E2M3 pattern of +-m/8, so this is the hardware FP6 converter
// applied to v/8 (round to nearest even; the scale operand divides).  The two-source converter interleaves its
// sources (result position 2j holds a[j], 2j+1 holds b[j]); only the lower halves of the sources are defined, the
// codes of the upper halves (result dwords 3..5) are not used.
__device__ __forceinline__ void f6_codes16(const float (&v)[16], uint32_t (&out)[3])
{
    typedef float v8f __attribute__((ext_vector_type(8)));
    typedef float v16f __attribute__((ext_vector_type(16)));
    typedef unsigned int v6u __attribute__((ext_vector_type(6)));
    const v8f ev = {v[0], v[2], v[4], v[6], v[8], v[10], v[12], v[14]};
    const v8f od = {v[1], v[3], v[5], v[7], v[9], v[11], v[13], v[15]};
    const v16f a = __builtin_shufflevector(ev, ev, 0, 1, 2, 3, 4, 5, 6, 7, -1, -1, -1, -1, -1, -1, -1, -1);
    const v16f b = __builtin_shufflevector(od, od, 0, 1, 2, 3, 4, 5, 6, 7, -1, -1, -1, -1, -1, -1, -1, -1);
    const float sc = 8.0f;
    const v6u c = __builtin_amdgcn_cvt_scalef32_2xpk16_fp6_f32(a, b, sc);
    // The converter writes its result registers over several passes while still reading its sources, and the
    // register allocator is not told: the sources are kept live past it so that the result cannot land on them.
    asm volatile("" : : "v"(a), "v"(b), "v"(sc));
    out[0] = c[0];
    out[1] = c[1];
    out[2] = c[2];
}

// BF16IN: element type of X; SM: smoothing variant (X times stored reciprocals, row held as fp32).
template <bool BF16IN, int MAXC, int NJB, bool SM = false, bool GA = false>
__global__ __launch_bounds__(256) void act_int_kernel(ActParams p)
{
    write_tag(p.tag_dst, p.tag);
    constexpr bool BF16 = BF16IN && !SM;  // representation of the row in registers
    __shared__ float s_amax[4][16];
    __shared__ float s_sxb[16];
    __shared__ int s_acc[4][NJB > 0 ? NJB : 1][64][4];  // [wave][j block][lane][4]

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int r16 = lane & 15, kq = lane >> 4;
    const int row = blockIdx.x * 16 + r16;
    const bool row_ok = row < p.M;
    const int C64 = p.C64;
    constexpr int njb = NJB;  // rank / 16

    constexpr bool STREAM = MAXC == 0;
    constexpr int NS = STREAM ? 2 : MAXC;            // chunk slots in registers
    const int nmy = (C64 - wave + 3) >> 2;           // chunks of this wavefront: c = wave + 4 * ci, ci < nmy
    XChunk<BF16> xc[NS];
    auto load_x = [&](XChunk<BF16>& ch, int ci) {
        const int c = wave + 4 * ci;
        const size_t koff = (size_t)c * 64 + kq * 16;
        if constexpr (SM)
            load_smoothed<BF16IN>(ch, p.X, (size_t)row * p.ldx + koff, p.rg + (c < C64 ? koff : 0), row_ok && c < C64);
        else
            ch.load(p.X, (size_t)row * p.ldx + koff, row_ok && c < C64);
    };
#pragma unroll
    for (int ci = 0; ci < NS; ++ci) load_x(xc[ci], ci);

    // Operands that do not depend on X are requested now, so that their latency overlaps the
    // load of X: the Q2(R) fragments of this wavefront's first chunk (later chunks are fetched one
    // chunk ahead inside the loop) and the row scales of R.
    constexpr int NJA = NJB > 0 ? NJB : 1;
    v4i bv[2][NJA];
    auto load_rq = [&](v4i (&dst)[NJA], int ci) {
        int c = wave + 4 * ci;
        c = c < C64 ? c : C64 - 1;  // clamped: a fragment past the end is fetched but not used
#pragma unroll
        for (int jb = 0; jb < NJB; ++jb) dst[jb] = *(const v4i*)(p.rq + ((size_t)((size_t)c * NJB + jb) * 64 + lane) * 16);
    };
    load_rq(bv[0], 0);
    float srj[NJA];
#pragma unroll
    for (int jb = 0; jb < NJB; ++jb) srj[jb] = p.sr[jb * 16 + r16];

    // ---- per-row amax -------------------------------------------------------------------
    float a = 0.f;
    us2 m2 = {0, 0};  // |bf16| is monotonic in its low 15 bits: packed unsigned 16-bit max, two values per op
    auto amax_chunk = [&](const XChunk<BF16>& ch) {
        if constexpr (BF16) {
#pragma unroll
            for (int d = 0; d < 8; ++d) m2 = __builtin_elementwise_max(m2, __builtin_bit_cast(us2, ch.w[d] & 0x7FFF7FFFu));
        } else {
#pragma unroll
            for (int i = 0; i < 16; ++i) a = fmaxf(a, fabsf(ch.get(i)));
        }
    };
    if constexpr (STREAM) {
        for (int ci0 = 0; ci0 < nmy; ci0 += 2) {
#pragma unroll
            for (int sl = 0; sl < 2; ++sl) {
                amax_chunk(xc[sl]);               // (a slot past the end holds zeros)
                load_x(xc[sl], ci0 + sl + 2);
            }
        }
        // second pass: the ring starts over
#pragma unroll
        for (int sl = 0; sl < 2; ++sl) load_x(xc[sl], sl);
    } else {
#pragma unroll
        for (int ci = 0; ci < NS; ++ci) amax_chunk(xc[ci]);
    }
    if constexpr (BF16) {
        const uint32_t mm = m2[0] > m2[1] ? m2[0] : m2[1];
        a = __uint_as_float(mm << 16);
    }
    a = fmaxf(a, __shfl_xor(a, 16, 64));
    a = fmaxf(a, __shfl_xor(a, 32, 64));
    if (kq == 0) s_amax[wave][r16] = a;
    __syncthreads();
    a = fmaxf(fmaxf(s_amax[0][r16], s_amax[1][r16]), fmaxf(s_amax[2][r16], s_amax[3][r16]));

    float s4, inv4, sb, invb;
    scales(a, 7.0f, &s4, &inv4);
    scales(a, p.qa, &sb, &invb);
    if (wave == 0 && kq == 0) {
        if constexpr (!GA) p.sx[row] = s4;
        s_sxb[r16] = sb;
        if (p.dbg_sxb && row_ok) p.dbg_sxb[row] = sb;
        if (p.r == 0) p.st[row] = 1.0f;
    }

    v4i acc[NJB > 0 ? NJB : 1];
#pragma unroll
    for (int jb = 0; jb < NJB; ++jb) acc[jb] = v4i{0, 0, 0, 0};

    const int rb = row >> 5;
    // one 64-chunk: main codes (and the block scale with SINT4 blocks), branch codes, skinny contraction
    auto code_chunk = [&](const XChunk<BF16>& ch, const int c, const int bslot) {
        uint32_t pk[3];
        uint32_t xb4[4] = {0u, 0u, 0u, 0u};
        if constexpr (GA) {
            // block scale of this 64-chunk: amax over the lane's 16 values, then over the row's 4 lanes
            float ac = 0.f;
            if constexpr (BF16) {
                us2 m2 = {0, 0};
#pragma unroll
                for (int d = 0; d < 8; ++d)
                    m2 = __builtin_elementwise_max(m2, __builtin_bit_cast(us2, ch.w[d] & 0x7FFF7FFFu));
                const uint32_t mm = m2[0] > m2[1] ? m2[0] : m2[1];
                ac = __uint_as_float(mm << 16);
            } else {
#pragma unroll
                for (int i = 0; i < 16; ++i) ac = fmaxf(ac, fabsf(ch.get(i)));
            }
            ac = fmaxf(ac, __shfl_xor(ac, 16, 64));
            ac = fmaxf(ac, __shfl_xor(ac, 32, 64));
            const uint32_t bits = sint4_scale(ac, &inv4);
            if (kq == 0) {
                p.sxg[sxg_index(row, c, p.tiles128)] = bits;
                // row blocks of the last 128-row tile that do not exist: finite scales (the forward multiplies
                // them by zero)
                if (row + 32 >= p.Mp)
                    for (int rr = row + 32; (rr >> 7) == (row >> 7); rr += 32) p.sxg[sxg_index(rr, c, p.tiles128)] = 0u;
            }
        }
        {
            // Main codes: x * inv rounded to the nearest integer by the FP6 converter (f6_codes16).  Branch codes:
            // low bytes of x*invb + 1.5*2^23, gathered with byte permutes (bf16 source) or shifts.
            float um[16];
#pragma unroll
            for (int i = 0; i < 16; ++i) {
                um[i] = __fmul_rn(ch.get(i), inv4);
                if constexpr (GA) um[i] = __builtin_amdgcn_fmed3f(um[i], -7.0f, 7.0f);  // the stored scale may be smaller than amax / 7
            }
            f6_codes16(um, pk);
        }
        if constexpr (BF16) {
#pragma unroll
            for (int h = 0; h < 2; ++h) {
                uint32_t tb[8];
#pragma unroll
                for (int e = 0; e < 8; ++e) tb[e] = rne_bits(__fmul_rn(ch.get(8 * h + e), invb));
#pragma unroll
                for (int q = 0; q < 2; ++q) {
                    const uint32_t p01 = __builtin_amdgcn_perm(tb[4 * q + 1], tb[4 * q], 0x0c0c0400u);
                    const uint32_t p23 = __builtin_amdgcn_perm(tb[4 * q + 3], tb[4 * q + 2], 0x0c0c0400u);
                    xb4[2 * h + q] = __builtin_amdgcn_perm(p23, p01, 0x05040100u);
                }
            }
        } else {
#pragma unroll
            for (int i = 0; i < 16; ++i) {
                const uint32_t b = rne_bits(__fmul_rn(ch.get(i), invb)) & 0xFFu;
                xb4[i >> 2] |= b << (8 * (i & 3));
            }
        }
        // the lane's 16 codes are dwords 3*(kq&1) .. +2 of the forward lane (row % 32, K half kq/2): an aligned
        // 8-byte and a 4-byte store
        {
            uint8_t* chunk = p.xq + ((size_t)rb * C64 + c) * F6_CHUNK;
            const int fl = (row & 31) + 32 * (kq >> 1);
            const bool odd = kq & 1;
            uint8_t* d8 = chunk + (odd ? 1024 + fl * 8 : fl * 16);
            uint8_t* d4 = chunk + fl * 16 + (odd ? 12 : 8);
            *(uint2*)d8 = odd ? make_uint2(pk[1], pk[2]) : make_uint2(pk[0], pk[1]);
            *(uint32_t*)d4 = odd ? pk[0] : pk[2];
        }
        if (p.dbg_xb && row_ok)
            *(v4i*)(p.dbg_xb + (size_t)row * p.K + c * 64 + kq * 16) = v4i{(int)xb4[0], (int)xb4[1], (int)xb4[2], (int)xb4[3]};
        if (njb > 0) {
            const v4i av = {(int)xb4[0], (int)xb4[1], (int)xb4[2], (int)xb4[3]};
#pragma unroll
            for (int jb = 0; jb < NJB; ++jb)
                acc[jb] = __builtin_amdgcn_mfma_i32_16x16x64_i8(av, bv[bslot][jb], acc[jb], 0, 0, 0);
        }
    };
    if constexpr (STREAM) {
        for (int ci0 = 0; ci0 < nmy; ci0 += 2) {
#pragma unroll
            for (int sl = 0; sl < 2; ++sl) {
                const int ci = ci0 + sl, c = wave + 4 * ci;
                load_rq(bv[(sl + 1) & 1], ci + 1);
                if (c < C64) code_chunk(xc[sl], c, sl);  // wave-uniform
                load_x(xc[sl], ci + 2);
            }
        }
    } else {
#pragma unroll
        for (int ci = 0; ci < NS; ++ci) {
            const int c = wave + 4 * ci;
            if (ci + 1 < NS) load_rq(bv[(ci + 1) & 1], ci + 1);
            if (c < C64) code_chunk(xc[ci], c, ci & 1);  // wave-uniform
        }
    }
    if (njb == 0) return;

    // ---- combine the 4 wavefronts' partial accumulators, dequantise, re-quantise ----------
#pragma unroll
    for (int jb = 0; jb < NJB; ++jb) *(v4i*)&s_acc[wave][jb][lane][0] = acc[jb];
    __syncthreads();
    if (wave != 0) return;

    // lane holds column j = jb*16 + lane%16 and token rows 4*(lane/16) + i
    float T[NJB > 0 ? NJB : 1][4];
    float tmax[4] = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int jb = 0; jb < NJB; ++jb) {
        {
            v4i s = *(const v4i*)&s_acc[0][jb][lane][0];
#pragma unroll
            for (int w = 1; w < 4; ++w) {
                const v4i o = *(const v4i*)&s_acc[w][jb][lane][0];
                s += o;
            }
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const int tok = 4 * kq + i;
                const float tv = __fmul_rn(__fmul_rn((float)s[i], s_sxb[tok]), srj[jb]);
                T[jb][i] = tv;
                tmax[i] = fmaxf(tmax[i], fabsf(tv));
                const int grow = blockIdx.x * 16 + tok;
                if (grow < p.M) {
                    if (p.dbg_accT) p.dbg_accT[(size_t)grow * p.r + jb * 16 + r16] = s[i];
                    if (p.dbg_T) p.dbg_T[(size_t)grow * p.r + jb * 16 + r16] = tv;
                }
            }
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
        scales(tmax[i], p.qa, &stv, &invt);
        if (r16 == 0) p.st[grow] = stv;
#pragma unroll
        for (int jb = 0; jb < NJB; ++jb)
            p.tq[(size_t)grow * p.rp + jb * 16 + r16] = (int8_t)(rne_bits(__fmul_rn(T[jb][i], invt)) & 0xFFu);
        if (p.rp > p.r && r16 < (p.rp - p.r)) p.tq[(size_t)grow * p.rp + p.r + r16] = 0;
    }
}

template <bool BF16, int MAXC, int NJB, bool SM, bool GA>
static hipError_t launch_one(const ActParams& p, int64_t Mp, hipStream_t s)
{
    hipLaunchKernelGGL((act_int_kernel<BF16, MAXC, NJB, SM, GA>), dim3((unsigned)(Mp / 16)), dim3(256), 0, s, p);
    return hipGetLastError();
}

template <bool BF16, int MAXC, bool SM, bool GA>
static hipError_t launch_rank2(const ActParams& p, int64_t Mp, hipStream_t s)
{
    switch (p.r) {
        case 0: return launch_one<BF16, MAXC, 0, SM, GA>(p, Mp, s);
        case 16: return launch_one<BF16, MAXC, 1, SM, GA>(p, Mp, s);
        case 32: return launch_one<BF16, MAXC, 2, SM, GA>(p, Mp, s);
        case 64: return launch_one<BF16, MAXC, 4, SM, GA>(p, Mp, s);
        case 96: return launch_one<BF16, MAXC, 6, SM, GA>(p, Mp, s);
        default: return launch_one<BF16, MAXC, 8, SM, GA>(p, Mp, s);
    }
}

template <bool BF16, int MAXC, bool SM = false>
static hipError_t launch_rank(const ActParams& p, int64_t Mp, hipStream_t s)
{
    return p.sxg ? launch_rank2<BF16, MAXC, SM, true>(p, Mp, s) : launch_rank2<BF16, MAXC, SM, false>(p, Mp, s);
}

hipError_t launch_quantize_act_int(const Dims& d, int x_dtype, const uint8_t* packed, const void* X,
                                   int64_t M, int64_t ldx, uint8_t* act, const lq_act_debug* dbg,
                                   hipStream_t s)
{
    const PackedLayout pl = packed_layout(d);
    const ActLayout al = act_layout(d, M);
    ActParams p;
    p.tag = make_tag(d, LQ_BLOB_ACT, M);
    p.tag_dst = (uint32_t*)act;
    p.X = X;
    p.ldx = ldx;
    p.M = (int)M;
    p.K = (int)d.K;
    p.C64 = d.C64;
    p.r = d.r;
    p.rp = d.rp;
    p.qa = (float)d.qmax_ba;
    p.rq = (const int8_t*)(packed + pl.off_rq);
    p.sr = (const float*)(packed + pl.off_sr);
    p.xq = act + al.off_xq;
    p.sx = (float*)(act + al.off_sx);
    p.sxg = d.ga ? (uint32_t*)(act + al.off_sx) : nullptr;
    p.tiles128 = (int)((al.Mp + 127) / 128);
    p.Mp = (int)al.Mp;
    p.tq = (int8_t*)(act + al.off_tq);
    p.st = (float*)(act + al.off_st);
    p.dbg_xb = dbg ? dbg->xb : nullptr;
    p.dbg_sxb = dbg ? dbg->sxb : nullptr;
    p.dbg_accT = dbg ? dbg->accT : nullptr;
    p.dbg_T = dbg ? dbg->T : nullptr;
    p.rg = (const float*)(packed + pl.off_rg);
    const int maxc = (d.C64 + 3) / 4;
    // MAXC = 0: the streamed kernel, for rows that do not fit in registers (fp32 representation: beyond 9 chunks per
    // wavefront, K > 2304; bf16: beyond 18, K > 4608)
    if (d.smooth) {
        if (x_dtype == LQ_BF16)
            return maxc <= 5 ? launch_rank<true, 5, true>(p, al.Mp, s) : maxc <= 9 ? launch_rank<true, 9, true>(p, al.Mp, s) : launch_rank<true, 0, true>(p, al.Mp, s);
        return maxc <= 5 ? launch_rank<false, 5, true>(p, al.Mp, s) : maxc <= 9 ? launch_rank<false, 9, true>(p, al.Mp, s) : launch_rank<false, 0, true>(p, al.Mp, s);
    }
    if (x_dtype == LQ_BF16) {
        if (maxc <= 5) return launch_rank<true, 5>(p, al.Mp, s);
        if (maxc <= 9) return launch_rank<true, 9>(p, al.Mp, s);
        if (maxc <= 18) return launch_rank<true, 18>(p, al.Mp, s);
        return launch_rank<true, 0>(p, al.Mp, s);
    }
    if (maxc <= 5) return launch_rank<false, 5>(p, al.Mp, s);
    if (maxc <= 9) return launch_rank<false, 9>(p, al.Mp, s);
    return launch_rank<false, 0>(p, al.Mp, s);
}

}  // namespace lq

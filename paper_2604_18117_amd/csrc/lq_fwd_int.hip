// Forward kernel, INT family (paper Fig. 1: residual branch + low-rank branch + sum).
//
//   acc[m,n,g] = sum_{k in g} xq[m,k] pq[n,k]           4-bit codes, exact
//   t[m,n]     = fma(acc[m,n,g], sw[n,g], t)            ascending g, fp32
//   acc2[m,n]  = sum_j tq[m,j] lq[n,j]                  int8 MFMA, int32
//   y          = fma(sx[m], t, (float(acc2) * st[m]) * sl[n]);   Y = bf16_rne(y)
//
// The 4-bit codes are stored as 6-bit fields s00mmm = the E2M3 pattern of +-m/8 and go to the matrix
// cores as they are (v_mfma_f32_32x32x64_f8f6f4 in FP6 mode): every product and every partial sum of a
// 64..128-deep group is an integer multiple of 2^-6 below 2^13 * 2^-6, so the fp32 MFMA accumulator
// holds the integer accumulator exactly and the per-group dequantisation is ONE fp32 FMA per output (no
// int->float conversion, no operand expansion); the factor 2^6 is folded into the stored weight scales.
//
// SINT4 blocks for both operands (template flag GA; App. A.3: one FP16 scale per 64 values): the dequantisation
// factor of an output and a K block is sx[m,g] * sw[n,g].  The 32 x 32 tile of these products comes from the
// matrix core as well: one v_mfma_f32_32x32x16_f16 whose A operand holds the token scales of the tile's four
// row blocks at k = 0, 2, 4, 6 (a lane's 16-byte load as it stands) and whose B operand holds the channel
// scale at the k of the wanted row block and zeros elsewhere; a product of two FP16 numbers is exact in fp32.
// The per-group dequantisation therefore stays ONE FMA per output, t = fma(acc, P, t); the factor 2^6 of the
// code fields is applied once at the end (t * 2^6 is exact).
//
// Work decomposition: a workgroup of 4 wavefronts computes a 128 x 256 tile of Y (64 x 256 for
// the half tiles at the tail of the grid); each wavefront owns 128 x 64 (4 x 2 MFMA tiles of
// 32 x 32, 128 fp32 running sums per lane).  Activation codes go global -> registers -> LDS once per
// workgroup; weight codes are read by each wavefront straight from global memory in operand order (no
// other wavefront needs them) into the registers the MFMAs read.
#include <type_traits>

#include "lq_internal.h"

namespace lq {

typedef int v2i __attribute__((ext_vector_type(2)));
typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v8i __attribute__((ext_vector_type(8)));
typedef int v16i __attribute__((ext_vector_type(16)));
typedef float v16f __attribute__((ext_vector_type(16)));
typedef float v4f __attribute__((ext_vector_type(4)));

struct FwdParams {
    const uint8_t* xq;
    const float* sx;
    const int8_t* tq;
    const float* st;
    const uint8_t* pq;
    const float* swT;
    const uint32_t* sxg;  // SINT4 blocks: FP16 bits of the token block scales, [G][tiles128][32][4]
    int tiles128;
    const int8_t* lq;
    const float* sl;
    uint16_t* Y;
    int64_t ldy;
    int M, N, G, C64, rp, nrb;
    int tilesM, tilesN, n_full;
    int nrb_main;    // row blocks per tile in the region of whole tiles: 4, or 3 where that fills the device better
    int panel;       // column tiles per panel of the tile order (panel_tile)
    int split_last;  // the last tile column has exactly 128 valid channels: run it 2 x 2
    int32_t* dbg_acc;
    int32_t* dbg_acc2;
    float* dbg_y32;
};

// One lane's FP6 operand: 32 six-bit codes = 24 bytes = six dwords (loaded as the 16-byte and the 8-byte part of the layout).
typedef int Op6 __attribute__((ext_vector_type(6)));
__device__ __forceinline__ Op6 op6(v4i lo, v2i hi) { return Op6{lo[0], lo[1], lo[2], lo[3], hi[0], hi[1]}; }
__device__ __forceinline__ v8i op8(Op6 o)  // the builtin's operand type; FP6 mode reads the first six dwords
{
    return __builtin_shufflevector(o, o, 0, 1, 2, 3, 4, 5, -1, -1);
}

constexpr int WN = 4;                          // wavefronts per workgroup, side by side along N
constexpr int NW = WN;
constexpr int RBT = 4;                         // 32-row blocks staged per workgroup (LDS slots)
constexpr int EPI_ROW = 144;                   // bytes per staged output row (128 + pad: no bank conflicts)
constexpr int EPI_WAVE = 32 * EPI_ROW;         // one 32 x 64 bf16 block per wavefront
constexpr int GA_MAXG = 88;                    // SINT4-block variant: K <= 5632 (the tile's token scales sit in LDS: 44 KB)
// LDS slot of one staged (row block, chunk): the 1536 operand bytes; the stride is chosen so that the 8-byte parts of
// two slots are neither 512-byte multiples nor within 2040 bytes of each other (the compiler would otherwise merge
// their reads into one two-address read and pay register moves to put the halves back into operand tuples)
// (the SINT4-block variant, short of registers, keeps the dense stride: there the merged reads cost fewer registers)
template <bool GA>
constexpr int lds_slot()
{
    return GA ? F6_CHUNK : 2064;
}
template <int GC, bool GA = false>
constexpr int lds_bytes()
{
    // [buffer][chunk in group][row block][slot]
    return 2 * GC * RBT * lds_slot<GA>() > NW * EPI_WAVE ? 2 * GC * RBT * lds_slot<GA>() : NW * EPI_WAVE;
}

// Epilogue operands parked in LDS: a tile's per-token scales, intermediate codes, and each wavefront's
// channel scales and channel codes are fetched in the prologue, when the running sums do not exist yet and registers
// are free, and wait in LDS; requested at the start of the epilogue, their round trip through the memory system
// (nothing else is left to do by then) would open every tile's epilogue.  sx[128] st[128] | sl[4][64] | lq[4][2][NK][64 x 16 B] |
// tq[4][NK][64 x 16 B]
template <int GC, int NK, bool GA>
constexpr bool park_epilogue()
{
    return !GA && (GC == 1 || NK <= 3);  // (two workgroups per CU must still fit their LDS; SINT4 blocks keep theirs for the token scales)
}
template <int NK>
constexpr int park_bytes()
{
    return 2048 + 12 * (NK > 0 ? NK : 1) * 1024;
}

// One output tile: rows rb0*32.., columns tile_n*256...  Each wavefront owns NRB row blocks x 64
// columns.  SPLIT = false: the 4 wavefronts sit side by side (tile of NRB*32 x 256).  SPLIT = true
// (NRB = 2): they are arranged 2 x 2 over a 128 x 128 tile, used for a last tile column that has
// only 128 valid channels, where two of four side-by-side wavefronts would idle through the loop.
// NRB = 4 (full tile) or
// 2 (half tile, used for the tail of the grid).  NK = 32-deep chunks of the padded rank: 0|1|2|3|4.
template <int GC, int NK, int NRB, bool DBG, bool SPLIT = false, bool GA = false>
__device__ __forceinline__ void fwd_tile(const FwdParams& p, uint8_t* lds, const int rb0, const int tile_n)
{
    static_assert(!GA || GC == 1, "SINT4 blocks are 64 deep");
    typedef _Float16 v8h __attribute__((ext_vector_type(8)));
    // Register sets of the weight stream: with 64-deep groups three sets rotate (a step's operands are requested two
    // steps before their use: an L2 round trip is about as long as one step); 128-deep groups (a step twice as long)
    // and the register-scarce SINT4-block variant use two sets, reloaded right after their last use.
    constexpr int BSETS = (GC == 1 && !GA) ? 3 : 2;
    constexpr int ASETS = (GC == 1) ? 2 : 1;    // register sets of the activation stream (on their way to LDS)
    constexpr int NT = NRB * 2;                 // 32 x 32 MFMA tiles per wavefront and step

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);  // wave-uniform: keeps address math scalar
    static_assert(!SPLIT || NRB == 2, "2 x 2 arrangement uses two row blocks per wavefront");
    const int wn = SPLIT ? (wave & 1) : wave;
    const int wm = SPLIT ? (wave >> 1) : 0;
    const int rbw = rb0 + wm * NRB;             // first row block owned by this wavefront
    const int half = lane >> 5, l32 = lane & 31;

    const int cb0 = tile_n * (WN * 2) + wn * 2;
    const bool active = (cb0 * 32 < p.N) && (rbw < p.nrb);

    const int C64 = p.C64, G = p.G;

    // ---- operand streams -----------------------------------------------------------------
    // Steps and row blocks are clamped instead of predicated: the loop body stays branch-free, and a
    // clamped load only re-reads valid data that never reaches a stored output.
    // Every wavefront stages one row block; with a half tile the upper two stage (clamped)
    // blocks that are not read.
    const uint32_t lane16 = (uint32_t)lane * 16u, lane8 = 1024u + (uint32_t)lane * 8u;
    const uint32_t l32x4 = (uint32_t)l32 * 4u, l32x16 = (uint32_t)l32 * 16u;
    int rbs = rb0 + wave;
    rbs = rbs < p.nrb ? rbs : p.nrb - 1;
    const uint8_t* xq_base = p.xq + (size_t)rbs * C64 * F6_CHUNK;
    const int cbw = (cb0 * 32 < p.N) ? cb0 : 0;  // wavefronts past the last column read block 0 (unused)
    const uint8_t* pq_base[2] = {p.pq + (size_t)cbw * C64 * F6_CHUNK, p.pq + (size_t)(cbw + 1) * C64 * F6_CHUNK};
    const float* sw_base = p.swT + cbw * 32;

    struct AStage { Op6 v[GC]; };
    struct BStage { Op6 v[GC][2]; float sw[2]; };
    // The streams are read with buffer loads: a wave-uniform descriptor and step offset in scalar registers plus
    // the 32-bit lane offsets all streams share, instead of a 64-bit vector address per stream (registers are
    // scarce).  Each descriptor spans exactly the bytes its stream may touch (a read past it would return zeros).
    typedef unsigned int u4 __attribute__((ext_vector_type(4)));
    typedef unsigned int u2 __attribute__((ext_vector_type(2)));
    constexpr int RSRC_FLAGS = 0x00020000;
    const __amdgpu_buffer_rsrc_t rs_xq = __builtin_amdgcn_make_buffer_rsrc((void*)xq_base, 0, C64 * F6_CHUNK, RSRC_FLAGS);
    const __amdgpu_buffer_rsrc_t rs_pq[2] = {__builtin_amdgcn_make_buffer_rsrc((void*)pq_base[0], 0, C64 * F6_CHUNK, RSRC_FLAGS),
                                             __builtin_amdgcn_make_buffer_rsrc((void*)pq_base[1], 0, C64 * F6_CHUNK, RSRC_FLAGS)};
    const __amdgpu_buffer_rsrc_t rs_sw = __builtin_amdgcn_make_buffer_rsrc((void*)sw_base, 0, (G * p.N - cbw * 32) * 4, RSRC_FLAGS);
    auto load_op = [&](Op6& o, const __amdgpu_buffer_rsrc_t& rs, int chunk) {
        o = op6(__builtin_bit_cast(v4i, (u4)__builtin_amdgcn_raw_buffer_load_b128(rs, lane16, chunk * F6_CHUNK, 0)),
                __builtin_bit_cast(v2i, (u2)__builtin_amdgcn_raw_buffer_load_b64(rs, lane8, chunk * F6_CHUNK, 0)));
    };
    auto load_a = [&](AStage& a, int step) {
        const int st = step < G ? step : G - 1;
#pragma unroll
        for (int cc = 0; cc < GC; ++cc) load_op(a.v[cc], rs_xq, st * GC + cc);
    };
    auto store_a = [&](const AStage& a, int buf) {
#pragma unroll
        for (int cc = 0; cc < GC; ++cc) {
            uint8_t* base = lds + (size_t)(((buf * GC + cc) * RBT + wave) * lds_slot<GA>());
            *(v4i*)(base + lane16) = v4i{a.v[cc][0], a.v[cc][1], a.v[cc][2], a.v[cc][3]};
            *(v2i*)(base + lane8) = v2i{a.v[cc][4], a.v[cc][5]};
        }
    };
    auto load_b = [&](BStage& b, int step) {
        const int st = step < G ? step : G - 1;
        // (the scales first: whatever path leads to their first use, the operand loads below were issued after them, so
        // the wait the compiler places before that use never has to drain the whole vector-memory queue)
#pragma unroll
        for (int cbi = 0; cbi < 2; ++cbi)
            b.sw[cbi] = __uint_as_float(__builtin_amdgcn_raw_buffer_load_b32(rs_sw, l32x4 + cbi * 128, st * p.N * 4, 0));
#pragma unroll
        for (int cbi = 0; cbi < 2; ++cbi) {
#pragma unroll
            for (int cc = 0; cc < GC; ++cc) load_op(b.v[cc][cbi], rs_pq[cbi], st * GC + cc);
        }
    };

    // SINT4 blocks: the token scales of the whole 128-row tile (G x 512 bytes, [g][row % 32][row block]) are
    // copied to LDS once; each step reads its 16 bytes per lane from there, one step ahead, into the register
    // set that serves as the A operand of the scale-product MFMAs.
    struct SStage { v4i sx; };
    uint8_t* lds_sx = lds + lds_bytes<GC, GA>();
    if constexpr (GA) {
        const uint32_t* src = p.sxg + (size_t)(rbw >> 2) * 128;
        for (int i = tid; i < G * 32; i += NW * 64)
            *(v4i*)(lds_sx + (size_t)i * 16) = *(const v4i*)(src + ((size_t)(i >> 5) * p.tiles128 * 32 + (i & 31)) * 4);
    }
    auto load_s = [&](SStage& sc, int step) {
        if constexpr (GA) {
            const int st = step < G ? step : G - 1;
            v4i v = *(const v4i*)(lds_sx + st * 512 + l32x16);
            if constexpr (NRB == 2) {  // half tiles own row blocks 0,1 or 2,3 of the 128-row tile: bring them to 0,1
                if (rbw & 2) v = v4i{v[2], v[3], v[0], v[1]};
            }
            sc.sx = v;
        }
    };

    v16f t[NRB][2];  // running sums; the first step starts them (from +0, as a constant operand of its FMAs)

    const uint64_t half_mask = 0xFFFFFFFF00000000ull;
    v4i bsel = {0, 0, 0, 0};

    // One step = one weight group.  On entry: LDS buffer s&1 holds the activation operands of step s, `bc` the
    // weight operands and scales of step s, `a` the activation codes of step s+1 on their way to LDS.  During
    // the step `a` goes to the other LDS buffer and is reloaded (two steps ahead with 64-deep groups), and the
    // weight set `bl` is requested: the set that step s-1 read (three rotating sets), or `bc` itself after this
    // step's last MFMA has been issued (two sets).
    auto do_step = [&](auto first_tag, int s, AStage& a, BStage& bc, BStage& bl, SStage& sc) {
        constexpr bool FIRST = decltype(first_tag)::value;
        const int buf = s & 1;
        auto lds_a = [&](int rbi, int cc) -> v8i {
            const uint8_t* base = lds + (size_t)(((buf * GC + cc) * RBT + wm * NRB + rbi) * lds_slot<GA>());
            return op8(op6(*(const v4i*)(base + lane16), *(const v2i*)(base + lane8)));
        };
        auto tile_mfma = [&](const v8i (&af)[GC], int cbi) -> v16f {
            v16f d = {0};
#pragma unroll
            for (int cc = 0; cc < GC; ++cc)
                d = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(af[cc], op8(bc.v[cc][cbi]), d, 2, 2, 0, 0, 0, 0);
            return d;
        };
        // operand of the current row block; double-buffered unless registers are scarce (SINT4 blocks; 128-deep groups,
        // whose two-chunk operands and weight sets otherwise push the kernel into spills): the next block's read is
        // then issued after the last MFMA that uses the current one, so one buffer is enough
        constexpr int AFB = (GA || GC == 2) ? 1 : 2;
        v8i af[AFB][GC];
        v16f dd[2];
        float swc[2];
        if constexpr (GA) {  // FP16 bits in the lanes of K half 0, zero in the others (they hold k = 8..15 of the scale MFMA)
#pragma unroll
            for (int cbi = 0; cbi < 2; ++cbi)
                asm volatile("v_cndmask_b32 %0, %1, 0, %2" : "=v"(swc[cbi]) : "v"(bc.sw[cbi]), "s"(half_mask));
        } else {
            swc[0] = bc.sw[0];
            swc[1] = bc.sw[1];
        }
        if constexpr (BSETS == 3) load_b(bl, s + 2);
#pragma unroll
        for (int cc = 0; cc < GC; ++cc) af[0][cc] = lds_a(0, cc);
        if constexpr (AFB == 2 && NRB > 1) {
#pragma unroll
            for (int cc = 0; cc < GC; ++cc) af[1][cc] = lds_a(1, cc);
        }
        dd[0] = tile_mfma(af[0], 0);
        // software pipeline over the 8 MFMA tiles: the matrix core works on tile j+1 while
        // the vector ALU folds tile j into the running sums
#pragma unroll
        for (int j = 0; j < NT; ++j) {
            const int rbi = j >> 1, cbi = j & 1;
            v16f P;
            if constexpr (GA) {  // scale products of this tile; issued ahead of the next main MFMA
                // B operand: the channel scale at the k of this row block, zeros elsewhere; kept in one
                // register set across tiles and steps, so a tile costs one or two moves
                if (cbi == 0) bsel[(rbi + NRB - 1) % NRB] = 0;
                bsel[rbi] = __float_as_int(swc[cbi]);
                asm volatile("" : "+v"(bsel));  // opaque: keeps the set in place instead of rebuilding it per tile
                P = __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(v8h, sc.sx), __builtin_bit_cast(v8h, bsel),
                                                           v16f{0}, 0, 0, 0);
            }
            if (j + 1 < NT) {
                const int nrbi = (j + 1) >> 1, ncbi = (j + 1) & 1;
                dd[(j + 1) & 1] = tile_mfma(af[nrbi % AFB], ncbi);
            }
            if constexpr (AFB == 2) {
                // operands are read a whole row block (two tiles) ahead of their first MFMA: block rbi + 2 goes into the
                // buffer of block rbi as soon as that block's last MFMA has been issued (the LDS round trip is longer
                // than one tile's FMAs)
                if (cbi == 1 && rbi + 2 < NRB) {
#pragma unroll
                    for (int cc = 0; cc < GC; ++cc) af[rbi % AFB][cc] = lds_a(rbi + 2, cc);
                }
            } else if (cbi == 0 && rbi + 1 < NRB) {  // one buffer: the next row block, one tile ahead
#pragma unroll
                for (int cc = 0; cc < GC; ++cc) af[0][cc] = lds_a(rbi + 1, cc);
            }
            if (j == 0) {  // fills the pipeline start-up bubble
                store_a(a, buf ^ 1);
                load_a(a, s + 1 + ASETS);
            }
            if (j == NT - 1) {  // the last MFMA of the step is in flight
                if constexpr (BSETS == 2) load_b(bl, s + 2);  // (bl is bc: its operands have been read)
                load_s(sc, s + 1);  // ... and so has this step's scale set
            }
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int i = 0; i < 16; ++i)
                t[rbi][cbi][i] = __builtin_fmaf(dd[j & 1][i], GA ? P[i] : swc[cbi], FIRST ? 0.0f : t[rbi][cbi][i]);
            if (DBG) {
                if (p.dbg_acc && active) {
#pragma unroll
                    for (int i = 0; i < 16; ++i) {
                        const int row = (rbw + rbi) * 32 + 8 * (i >> 2) + 4 * half + (i & 3);
                        const int col = (cb0 + cbi) * 32 + l32;
                        if (row < p.M)
                            p.dbg_acc[((size_t)row * p.N + col) * G + s] = (int)(dd[j & 1][i] * 64.0f);
                    }
                }
            }
            __builtin_amdgcn_sched_barrier(0);
        }
        __syncthreads();
    };

    // A wavefront whose columns lie past N (the last tile column of a layer whose width is no multiple of 256) only
    // stages its row block of the activation codes, barrier for barrier with the others: it issues no matrix or
    // vector work that would compete with the wavefront it shares a SIMD with.
    constexpr bool PARK = park_epilogue<GC, NK, GA>();
    constexpr int NKP = NK > 0 ? NK : 1;
    uint8_t* park = lds + lds_bytes<GC, GA>();
    float* park_sx = (float*)park;
    float* park_st = (float*)(park + 512);
    float* park_sl = (float*)(park + 1024) + wave * 64;
    uint8_t* park_lq = park + 2048 + wave * 2 * NKP * 1024;
    uint8_t* park_tq = park + 2048 + 8 * NKP * 1024;
    struct ParkRows { float sx, st; v4i tq[NKP]; };
    struct ParkCols { float sl; v4i lq[2][NKP]; };
    auto park_load_rows = [&](ParkRows& r) {  // of the row block this wavefront stages
        r.sx = p.sx[rbs * 32 + l32];
        r.st = p.st[rbs * 32 + l32];
#pragma unroll
        for (int kk = 0; kk < NK; ++kk) r.tq[kk] = *(const v4i*)(p.tq + (size_t)(rbs * 32 + l32) * p.rp + kk * 32 + half * 16);
    };
    auto park_store_rows = [&](const ParkRows& r) {
        park_sx[wave * 32 + l32] = r.sx;  // (both halves of the wavefront write the same value)
        park_st[wave * 32 + l32] = r.st;
#pragma unroll
        for (int kk = 0; kk < NK; ++kk) *(v4i*)(park_tq + (size_t)((wave * NKP + kk) * 1024) + lane16) = r.tq[kk];
    };
    auto park_load_cols = [&](ParkCols& c) {
        c.sl = p.sl[cb0 * 32 + lane];
#pragma unroll
        for (int cbi = 0; cbi < 2; ++cbi)
#pragma unroll
            for (int kk = 0; kk < NK; ++kk)
                c.lq[cbi][kk] = *(const v4i*)(p.lq + (size_t)((cb0 + cbi) * 32 + l32) * p.rp + kk * 32 + half * 16);
    };
    auto park_store_cols = [&](const ParkCols& c) {
        park_sl[lane] = c.sl;
#pragma unroll
        for (int cbi = 0; cbi < 2; ++cbi)
#pragma unroll
            for (int kk = 0; kk < NK; ++kk) *(v4i*)(park_lq + (size_t)((cbi * NKP + kk) * 1024) + lane16) = c.lq[cbi][kk];
    };
    if (cb0 * 32 >= p.N) {  // wave-uniform
        AStage x0, x1;
        load_a(x0, 0);
        load_a(x1, 1);
        if constexpr (PARK) {  // the other wavefronts read this row block's epilogue operands from LDS
            ParkRows pr;
            park_load_rows(pr);
            park_store_rows(pr);
        }
        store_a(x0, 0);
        __syncthreads();
        for (int s = 0; s < G; s += 2) {  // step s: the codes of step s + 1 go to the other buffer
            store_a(x1, (s & 1) ^ 1);
            load_a(x0, s + 2);
            __syncthreads();
            if (s + 1 >= G) break;
            store_a(x0, s & 1);
            load_a(x1, s + 3);
            __syncthreads();
        }
        return;
    }
    // Every other wavefront runs the same branch-free loop; one without valid output (past the last row block of a
    // partial tile) works on clamped operands, stores nothing.
    SStage s0;
    const std::true_type first{};    // the first step of a tile starts the running sums
    const std::false_type later{};
    if constexpr (BSETS == 3) {
        AStage a0, a1;
        BStage b0, b1, b2;
        load_a(a0, 0);
        load_b(b0, 0);
        load_a(a1, 1);   // (goes to LDS during step 0)
        load_b(b1, 1);
        store_a(a0, 0);
        load_a(a0, 2);   // (goes to LDS during step 1)
        if constexpr (PARK) {
            ParkRows pr;
            ParkCols pc;
            park_load_rows(pr);
            park_load_cols(pc);
            __syncthreads();
            park_store_rows(pr);
            park_store_cols(pc);
        } else {
            __syncthreads();
        }
        load_s(s0, 0);
        // step s reads weight set s % 3 and requests set (s + 2) % 3; activation set (s + 1) % 2 goes to LDS
        do_step(first, 0, a1, b0, b2, s0);
        for (int s = 1; s < G; s += 6) {
            do_step(later, s, a0, b1, b0, s0);
            if (s + 1 >= G) break;
            do_step(later, s + 1, a1, b2, b1, s0);
            if (s + 2 >= G) break;
            do_step(later, s + 2, a0, b0, b2, s0);
            if (s + 3 >= G) break;
            do_step(later, s + 3, a1, b1, b0, s0);
            if (s + 4 >= G) break;
            do_step(later, s + 4, a0, b2, b1, s0);
            if (s + 5 >= G) break;
            do_step(later, s + 5, a1, b0, b2, s0);
        }
    } else if constexpr (ASETS == 2) {  // SINT4 blocks: two weight sets
        AStage a0, a1;
        BStage b0, b1;
        load_a(a0, 0);
        load_b(b0, 0);
        load_a(a1, 1);
        load_b(b1, 1);
        store_a(a0, 0);
        load_a(a0, 2);
        __syncthreads();
        load_s(s0, 0);
        // (registers are scarce here: the running sums start as zeros in registers and every step is the same code)
#pragma unroll
        for (int a = 0; a < NRB; ++a)
#pragma unroll
            for (int b = 0; b < 2; ++b)
#pragma unroll
                for (int i = 0; i < 16; ++i) t[a][b][i] = 0.f;
        do_step(later, 0, a1, b0, b0, s0);
        for (int s = 1; s < G; s += 2) {
            do_step(later, s, a0, b1, b1, s0);
            if (s + 1 >= G) break;
            do_step(later, s + 1, a1, b0, b0, s0);
        }
    } else {  // 128-deep groups
        AStage a0;
        BStage b0, b1;
        load_a(a0, 0);
        load_b(b0, 0);
        load_b(b1, 1);
        store_a(a0, 0);
        load_a(a0, 1);
        if constexpr (PARK) {
            ParkRows pr;
            ParkCols pc;
            park_load_rows(pr);
            park_load_cols(pc);
            __syncthreads();
            park_store_rows(pr);
            park_store_cols(pc);
        } else {
            __syncthreads();
        }
        do_step(first, 0, a0, b0, b0, s0);
        // whole pairs of steps in a loop with one exit, an odd last step after it: with an exit between the two steps
        // the compiler builds a loop whose header can be reached with a weight scale as the last load issued, and
        // waits for the whole vector-memory queue before every use of a scale
        int s = 1;
        for (; s + 1 < G; s += 2) {
            do_step(later, s, a0, b1, b1, s0);
            do_step(later, s + 1, a0, b0, b0, s0);
        }
        if (s < G) do_step(later, s, a0, b1, b1, s0);
    }

    // ---- epilogue: rank-r expansion, scales, sum, bf16 -------------------------------------
    // Each wavefront turns one 32 x 64 block at a time into bf16, transposes it through its own
    // LDS slice and writes full 128-byte rows (16 bytes per lane).
    if (!active) return;  // (the loop's last barrier already separates operand reads from the staging below)

    typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
    typedef float f32x2 __attribute__((ext_vector_type(2)));
    uint8_t* stage = lds + wave * EPI_WAVE;
    constexpr int NKA = NK > 0 ? NK : 1;
    float slv[2];
    v4i lqf[2][NKA];
#pragma unroll
    for (int cbi = 0; cbi < 2; ++cbi) {
        const int col = (cb0 + cbi) * 32 + l32;
        if constexpr (PARK) {
            slv[cbi] = park_sl[cbi * 32 + l32];
#pragma unroll
            for (int kk = 0; kk < NK; ++kk) lqf[cbi][kk] = *(const v4i*)(park_lq + (size_t)((cbi * NKP + kk) * 1024) + lane16);
        } else {
            slv[cbi] = p.sl[col];
#pragma unroll
            for (int kk = 0; kk < NK; ++kk)
                lqf[cbi][kk] = *(const v4i*)(p.lq + (size_t)col * p.rp + kk * 32 + half * 16);
        }
    }
    const int wr_off = (4 * half) * EPI_ROW + l32 * 2;        // this lane's column in the staged block
    const int rd_row = lane >> 3, rd_seg = lane & 7;          // read-back: 8 lanes per 128-byte row
    // Per-row-block operands (intermediate codes, per-token scales).  Row blocks past the end of
    // a partial tile are clamped (their results are never stored), so the loads of block rbi+1
    // can be issued while block rbi is still being processed.
    v4i tqf[NKA];
    v4f sxv[4], stv[4];
    auto load_tq = [&](int rbi) {
        if constexpr (PARK) {  // (slot of the wavefront that staged this row block)
#pragma unroll
            for (int kk = 0; kk < NK; ++kk)
                tqf[kk] = *(const v4i*)(park_tq + (size_t)(((wm * NRB + rbi) * NKP + kk) * 1024) + lane16);
            return;
        }
        int rb = rbw + rbi;
        rb = rb < p.nrb ? rb : p.nrb - 1;
#pragma unroll
        for (int kk = 0; kk < NK; ++kk)
            tqf[kk] = *(const v4i*)(p.tq + (size_t)(rb * 32 + l32) * p.rp + kk * 32 + half * 16);
    };
    auto load_scales = [&](int rbi) {  // rows 8*q + 4*half + 0..3 are contiguous -> one 16-byte load each
        if constexpr (PARK) {
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                sxv[q] = *(const v4f*)(park_sx + (wm * NRB + rbi) * 32 + 8 * q + 4 * half);
                stv[q] = *(const v4f*)(park_st + (wm * NRB + rbi) * 32 + 8 * q + 4 * half);
            }
            return;
        }
        int rb = rbw + rbi;
        rb = rb < p.nrb ? rb : p.nrb - 1;
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            if constexpr (!GA) sxv[q] = *(const v4f*)(p.sx + rb * 32 + 8 * q + 4 * half);
            stv[q] = *(const v4f*)(p.st + rb * 32 + 8 * q + 4 * half);
        }
    };
    load_tq(0);
    load_scales(0);
    // this lane's output pointer: row rd_row of the tile, 16 bytes at column segment rd_seg; it moves
    // down 8 rows per store (4 stores per row block), rows past M are skipped
    // The stores are buffer stores through a descriptor that ends with the wavefront's 128 bytes of its last valid row:
    // rows past M are out of range and dropped by the hardware, so the stores need no branch -- and only stores the
    // compiler can count let it wait for a load issued before them without waiting for the stores themselves (the
    // vector-memory counter retires in order).  Measured: 2240 -> 6720 layer 110 -> 107 us.
    const int rows_valid = p.M - rbw * 32 < NRB * 32 ? p.M - rbw * 32 : NRB * 32;
    const __amdgpu_buffer_rsrc_t rs_y = __builtin_amdgcn_make_buffer_rsrc(
        (void*)(p.Y + (size_t)(rbw * 32) * p.ldy + cb0 * 32), 0, (int)((rows_valid - 1) * p.ldy * 2 + 128), RSRC_FLAGS);
    uint32_t yoff = (uint32_t)(rd_row * (int)p.ldy * 2 + rd_seg * 16);
    const uint32_t ystep = (uint32_t)(8 * (int)p.ldy * 2);
    v4i ov[4];
#pragma unroll
    for (int rbi = 0; rbi < NRB; ++rbi) {
        const int rbase = (rbw + rbi) * 32;
        v16i a2[2];
#pragma unroll
        for (int cbi = 0; cbi < 2; ++cbi) {
            a2[cbi] = v16i{0};
#pragma unroll
            for (int kk = 0; kk < NK; ++kk)
                a2[cbi] = __builtin_amdgcn_mfma_i32_32x32x32_i8(tqf[kk], lqf[cbi][kk], a2[cbi], 0, 0, 0);
        }
        if (rbi + 1 < NRB) load_tq(rbi + 1);  // the matrix core has read tqf: fetch the next block's codes
        float y[2][16];
#pragma unroll
        for (int cbi = 0; cbi < 2; ++cbi)
#pragma unroll
            for (int i = 0; i < 16; ++i) {
                const float ybr = __fmul_rn(__fmul_rn((float)a2[cbi][i], stv[i >> 2][i & 3]), slv[cbi]);
                // SINT4 blocks: t carries the factor 2^-6 of the code fields; scaling it back is exact
                y[cbi][i] = GA ? __builtin_fmaf(t[rbi][cbi][i], 64.0f, ybr)
                               : __builtin_fmaf(sxv[i >> 2][i & 3], t[rbi][cbi][i], ybr);
            }
        if (rbi + 1 < NRB) load_scales(rbi + 1);
#pragma unroll
        for (int cbi = 0; cbi < 2; ++cbi) {
#pragma unroll
            for (int i = 0; i < 16; i += 2) {
                const bf16x2 h = __builtin_convertvector(f32x2{y[cbi][i], y[cbi][i + 1]}, bf16x2);
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
                    if (row < p.M) {
                        if (p.dbg_acc2) p.dbg_acc2[(size_t)row * p.N + col] = a2[cbi][i];
                        if (p.dbg_y32) p.dbg_y32[(size_t)row * p.N + col] = y[cbi][i];
                    }
                }
            }
        }
        // read the block back row-wise (LDS operations of one wavefront complete in order)
#pragma unroll
        for (int q = 0; q < 4; ++q) ov[q] = *(const v4i*)(stage + (q * 8 + rd_row) * EPI_ROW + rd_seg * 16);
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            __builtin_amdgcn_raw_buffer_store_b128(__builtin_bit_cast(u4, ov[q]), rs_y, yoff, 0, 0);
            yoff += ystep;
        }
    }
}

// Grid: the first n_full workgroups compute full 128 x 256 tiles, in row-major tile order; the
// remaining tiles (see launch_cfg for when and how many) are each split into two 64 x 256 half tiles,
// which shortens or evens out the last round of the grid.  XCD-aware order in both regions: workgroup ids are
// dealt round-robin to the 8 XCDs, so each XCD gets one contiguous run of tiles (its L2 then sees
// few distinct row tiles).
__device__ __forceinline__ int xcd_order(int b, int n)
{
    const int per = n >> 3, rem = n & 7;
    const int xcd = b & 7, loc = b >> 3;
    return xcd * per + (xcd < rem ? xcd : rem) + loc;
}

template <int GC, int NK, bool DBG, bool GA = false>
__global__ __launch_bounds__(NW * 64, 2) void fwd_int_kernel(FwdParams p)
{
    __shared__ __attribute__((aligned(16))) uint8_t lds[lds_bytes<GC, GA>() + (GA ? GA_MAXG * 512 : 0) +
                                                       (park_epilogue<GC, NK, GA>() ? park_bytes<NK>() : 0)];
    const int b = blockIdx.x;
    if (b < p.n_full) {
        const int tile = xcd_order(b, p.n_full);
        int tile_m, tile_n;
        panel_tile(tile, p.tilesM, p.tilesN, p.panel, tile_m, tile_n);
        if (p.split_last && tile_n == p.tilesN - 1)
            fwd_tile<GC, NK, 2, DBG, true, GA>(p, lds, tile_m * 4, tile_n);
        else if (!GA && p.nrb_main == 3)
            fwd_tile<GC, NK, 3, DBG, false, false>(p, lds, tile_m * 3, tile_n);
        else
            fwd_tile<GC, NK, 4, DBG, false, GA>(p, lds, tile_m * 4, tile_n);
    } else {
        const int hh = xcd_order(b - p.n_full, 2 * (p.tilesM * p.tilesN - p.n_full));
        const int tile = p.n_full + (hh >> 1);
        int tile_m, tile_n;
        panel_tile(tile, p.tilesM, p.tilesN, p.panel, tile_m, tile_n);
        const int rb0 = tile_m * 4 + (hh & 1) * 2;
        if (rb0 >= p.nrb) return;  // lower half of a partial last row tile: nothing to do
        fwd_tile<GC, NK, 2, DBG, false, GA>(p, lds, rb0, tile_n);
    }
}

// Workgroup slots of the device: two workgroups (of 256 registers per lane) per compute unit.
static int workgroup_slots()
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

template <int GC, int NK, bool DBG, bool GA = false>
static hipError_t launch_cfg(const FwdParams& p0, hipStream_t s)
{
    FwdParams p = p0;
    p.tilesM = (p.nrb + 3) / 4;
    p.tilesN = (p.N + WN * 64 - 1) / (WN * 64);
    const int slots = workgroup_slots() & ~7;
    // Tile height.  Tiles of 96 rows instead of 128 when they fill the device better: a layer whose 128-row tiles
    // number between one per compute unit and one per workgroup slot (the 4608 -> 1152 projection: 288 tiles on 512
    // slots) leaves half the wavefront slots empty while the rest work two to a SIMD; 96-row tiles (430) put more of
    // the chip to work for three quarters of the time each.  Estimated time of a layout: generations of the grid
    // times (a fixed part + the tile's row blocks), a lone workgroup on a compute unit counted at 0.6.
    {
        auto est = [&](int h) {
            const int t = ((p.nrb + h - 1) / h) * p.tilesN;
            const double c = 1.0 + h;
            if (t <= slots / 2) return 0.6 * c;
            return (double)((t + slots - 1) / slots) * c;
        };
        const int t4 = p.tilesM * p.tilesN;
        p.nrb_main = (!GA && t4 > slots / 2 && est(3) < 0.9 * est(4)) ? 3 : 4;
    }
    if (p.nrb_main == 3) {
        p.tilesM = (p.nrb + 2) / 3;
        p.n_full = p.tilesM * p.tilesN;
        p.split_last = 0;   // (a last tile column of 128 channels: its two wavefronts past the end only stage)
        p.panel = panel_width(p.tilesN, p.C64, 48);
        dim3 grid((unsigned)p.n_full), block(NW * 64);
        hipLaunchKernelGGL((fwd_int_kernel<GC, NK, DBG, GA>), grid, block, 0, s, p);
        return hipGetLastError();
    }
    const int tiles = p.tilesM * p.tilesN;
    // Full rounds of the grid use full tiles.  A half tile costs more than half of a full one (each wavefront
    // reads its weight operands either way), so splitting the remainder pays only while
    // the halves still fit one per compute unit: measured +5 % on a 1152 -> 4608 layer (2.25 rounds),
    // nothing at 1.75 rounds when the whole remainder is split, a loss at 0.6 rounds.
    int n_full = (tiles / slots) * slots;
    if (4 * (tiles - n_full) > slots) {
        // A layer of between one and two generations whose second generation fills 50 .. 85 % of the slots (1152 -> 3456:
        // 896 tiles on 512 slots): as many of the last tiles are halved as it takes to occupy every slot, so that no CU
        // runs two whole tiles while its neighbour runs one (38.9 -> 36.5 us; with more generations before it, or a
        // fuller last one, the same split changes nothing or loses).
        const int rest = tiles - n_full;
        n_full = tiles;
        if (tiles > slots && tiles < 2 * slots && 2 * rest > slots && 20 * rest <= 17 * slots) n_full = tiles - (slots - rest);
    }
    p.n_full = n_full;
    p.split_last = (p.N & 255) == 128;
    p.panel = panel_width(p.tilesN, p.C64, 48);
    dim3 grid((unsigned)(n_full + 2 * (tiles - n_full))), block(NW * 64);
    hipLaunchKernelGGL((fwd_int_kernel<GC, NK, DBG, GA>), grid, block, 0, s, p);
    return hipGetLastError();
}

template <int GC, bool DBG, bool GA = false>
static hipError_t launch_rank(int nk, const FwdParams& p, hipStream_t s)
{
    switch (nk) {
        case 0: return launch_cfg<GC, 0, DBG, GA>(p, s);
        case 1: return launch_cfg<GC, 1, DBG, GA>(p, s);
        case 2: return launch_cfg<GC, 2, DBG, GA>(p, s);
        case 3: return launch_cfg<GC, 3, DBG, GA>(p, s);
        default: return launch_cfg<GC, 4, DBG, GA>(p, s);
    }
}

hipError_t launch_fwd_int(const Dims& d, const uint8_t* packed, const uint8_t* act, int64_t M,
                          uint16_t* Y, int64_t ldy, const lq_fwd_debug* dbg, hipStream_t s)
{
    const PackedLayout pl = packed_layout(d);
    const ActLayout al = act_layout(d, M);
    FwdParams p;
    p.xq = act + al.off_xq;
    p.sx = (const float*)(act + al.off_sx);
    p.tq = (const int8_t*)(act + al.off_tq);
    p.st = (const float*)(act + al.off_st);
    p.pq = packed + pl.off_pq;
    p.swT = (const float*)(packed + pl.off_sw);
    p.sxg = (const uint32_t*)(act + al.off_sx);
    p.tiles128 = (int)((al.Mp + 127) / 128);
    p.lq = (const int8_t*)(packed + pl.off_lq);
    p.sl = (const float*)(packed + pl.off_sl);
    p.Y = Y;
    p.ldy = ldy;
    p.M = (int)M;
    p.N = (int)d.N;
    p.G = d.G;
    p.C64 = d.C64;
    p.rp = d.rp;
    p.nrb = (int)(al.Mp / 32);
    p.tilesM = p.tilesN = p.n_full = p.split_last = 0;
    p.panel = 1;
    p.dbg_acc = dbg ? dbg->acc : nullptr;
    p.dbg_acc2 = dbg ? dbg->acc2 : nullptr;
    p.dbg_y32 = dbg ? dbg->y32 : nullptr;
    const bool want_dbg = dbg && (dbg->acc || dbg->acc2 || dbg->y32);
    const int nk = d.rp >> 5;  // 0 | 1 | 2 | 3 | 4 (the rank is one of 0, 16, 32, 64, 96, 128)
    if (d.ga) return want_dbg ? launch_rank<1, true, true>(nk, p, s) : launch_rank<1, false, true>(nk, p, s);
    if (d.g == 64) {
        return want_dbg ? launch_rank<1, true>(nk, p, s) : launch_rank<1, false>(nk, p, s);
    } else {
        return want_dbg ? launch_rank<2, true>(nk, p, s) : launch_rank<2, false>(nk, p, s);
    }
}

}  // namespace lq

// bf16 x bf16 -> fp32 tiled product on the CDNA4 matrix cores:
//   C(m, n) = sum_c A(m, c) * B(n, c),   A, B and C given as Views (views.h).
//
// One workgroup (512 threads = two teams of 4 wavefronts) owns a 128 x 128 tile of C and walks the
// reduction index in steps of 64, the teams taking alternate steps (see gemm_mfma_kernel).  Within a
// team each wavefront owns a 64 x 64 quadrant = 2 x 2 MFMA tiles of v_mfma_f32_32x32x16_bf16,
// accumulators in registers (64 floats per lane).
//
// Operand staging: global -> registers -> LDS (two LDS stages per team).  The global loads of a step
// are issued two of the team's steps before the step is multiplied (two register sets, used
// alternately), so that L2 / HBM latency is covered by MFMA work of both teams.
// Two loader kinds, chosen per operand:
//   LD_KC  the reduction index is contiguous in memory (X, G, L, D in the forward; delta in dX).
//          LDS tile [128 rows][64 + 8]; a lane's MFMA operand is one 16-byte LDS read.
//   LD_KM  the free index is contiguous, the reduction index strides (L, C, D in dX and error
//          compression; delta, X, G in the weight gradients).  LDS tile [64][128 + 16]; the MFMA
//          operand is built by two ds_read_b64_tr_b16 (the gfx950 transposing LDS read: within 16
//          lanes, lanes 4j..4j+3 supply row j of a 4 x 16 block, lane i receives column i).
// The peers' segments (G_i, D_i) are addressed in place through the View; VEC (8, 4 or 2
// elements) is the widest vector that never straddles a segment boundary.
//
// Address arithmetic is kept off the vector ALU as far as possible (it competes with the MFMAs for
// issue slots): everything that depends only on the thread is computed once, everything that
// depends only on the reduction step is computed on the scalar unit, and a full interior tile
// takes one or two vector adds per 16-byte load.  Only the ragged last tile pays for clamping and
// masking.
//
// Workgroup ids are re-mapped so that the ids an XCD receives (id mod 8) form a contiguous range
// of tiles: neighbouring tiles share operand panels in that XCD's L2.
#pragma once
#include "common.h"
#include "gemm_generic.h"   // Epilogue, EPI_*
#include "views.h"

namespace phantom {

enum { LD_KC = 0, LD_KM = 1 };

constexpr int MT = 128;               // tile rows (m) and columns (n)
constexpr int KT = 64;                // reduction step
constexpr int KC_PITCH = KT + 8;      // elements per LDS row, K-contiguous tile [128][72]
constexpr int KM_PITCH = MT + 16;     // elements per LDS row, K-major tile [64][144]
constexpr int TILE_ELEMS = MT * KC_PITCH;   // = KT * KM_PITCH = 9216
static_assert(MT * KC_PITCH == KT * KM_PITCH, "both tile shapes use the same LDS space");
constexpr int MFMA_THREADS = 512;       // two teams of four wavefronts
constexpr int MFMA_LDS_BYTES = 2 /*teams*/ * 2 /*stages*/ * 2 /*operands*/ * TILE_ELEMS * 2;

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
template <int VEC> struct VecOf;
template <> struct VecOf<8> { typedef u32x4 type; };
template <> struct VecOf<4> { typedef u32x2 type; };
template <> struct VecOf<2> { typedef uint32_t type; };

// a global-memory load that the compiler cannot mistake for a generic (flat) access
template <typename V>
__device__ __forceinline__ V load_global(const __bf16 *p)
{
    return *(const __attribute__((address_space(1))) V *)(uintptr_t)p;
}

// ---- staging one operand tile ---------------------------------------------------------
// KIND == LD_KC: tile rows = free index r in [r0, r0+128), columns = reduction index c in [c0, c0+64).
//                The reduction index may decide the region (head block / peer segments); r never does.
// KIND == LD_KM: tile rows = reduction index c in [c0, c0+64), columns = free index r in [r0, r0+128).
//                r may decide the region (fixed per thread); c may decide only between a head block
//                and ONE tail block ([L ; C] stacked along the reduction index).
// All element offsets inside a group fit 32 bits (checked on the host).
//
// No load is predicated (predication turns into divergent branches and makes the compiler wait for
// ALL outstanding loads instead of counting them).  Rows past the end of the free index read the
// last valid row; what they produce lands in outputs the epilogue never writes.  A tile that
// reaches past the end of the reduction range takes the slow path: indices are clamped to the last
// valid position and the store zeroes what was loaded for reduction indices >= c_lim.
template <int KIND, int VEC>
struct StageCfg {
    typedef typename VecOf<VEC>::type V;
    static constexpr int PER_ROW = (KIND == LD_KC ? KT : MT) / VEC;   // vectors per LDS row
    static constexpr int ROWS = KIND == LD_KC ? MT : KT;
    static constexpr int NV = ROWS * PER_ROW / 256;                   // vectors per thread
    static constexpr int ROW_STEP = 256 / PER_ROW;
    static constexpr int PITCH = KIND == LD_KC ? KC_PITCH : KM_PITCH;
};

struct StageState {          // scalars only, so that it lives in registers
    const __bf16 *base0, *base1;
    const __bf16 *tbase;     // LD_KM with a fixed region: the thread's base pointer
    int col, row0;           // this thread's vector column (elements) and first row inside the tile
    int c_lim;
    int c_decides, c_split, c_seg, c_skip;
    unsigned c_magic;        // ceil(2^32 / c_seg)
    int c_mult0, c_mult1, c_seg_stride;
    int r_region;            // LD_KM: region of the thread's fixed free index (-1: the reduction index decides)
};

// off0[j], off1[j]: element offsets of the thread's j-th vector that do not depend on the step, in
// region 0 and region 1.  LD_KC: row * row stride.  LD_KM: fixed free-index offset + (row0 + j*ROW_STEP) * c stride.
template <int KIND, int VEC>
__device__ __forceinline__ StageState stage_init(const View &v, int g, int r0, int r_limit, int c_limit, int tid,
                                                 int (&off0)[StageCfg<KIND, VEC>::NV], int (&off1)[StageCfg<KIND, VEC>::NV])
{
    typedef StageCfg<KIND, VEC> C;
    StageState s;
    s.base0 = (const __bf16 *)v.p0 + g * v.g0;
    s.base1 = (const __bf16 *)v.p1 + g * v.g1;
    const int skip = v.skip0 + g * v.skip_g;
    s.col = (tid % C::PER_ROW) * VEC;
    s.row0 = tid / C::PER_ROW;
    s.c_lim = c_limit;
    s.c_decides = v.c.decides;
    s.c_split = v.c.decides ? v.c.split : 0x7fffffff;
    s.c_seg = v.c.seg; s.c_skip = skip;
    s.c_magic = (unsigned)((0x100000000ull + (unsigned)v.c.seg - 1) / (unsigned)v.c.seg);
    s.c_mult0 = (int)v.c.mult0; s.c_mult1 = (int)v.c.mult1; s.c_seg_stride = (int)v.c.seg_stride;
    s.r_region = -1;
    s.tbase = s.base0;
    if (KIND == LD_KC) {
#pragma unroll
        for (int j = 0; j < C::NV; ++j) {
            const int r = min(r0 + s.row0 + j * C::ROW_STEP, r_limit - 1);
            off0[j] = r * (int)v.r.mult0;
            off1[j] = r * (int)v.r.mult1;
        }
    } else {
        const int r = r0 + s.col;
        const Loc lr = locate(v.r, r < r_limit ? r : 0, skip);
        s.r_region = lr.region;
        if (!v.c.decides) s.tbase = lr.region > 0 ? s.base1 : s.base0;
#pragma unroll
        for (int j = 0; j < C::NV; ++j) {
            const int cj = s.row0 + j * C::ROW_STEP;
            off0[j] = (int)lr.off0 + cj * s.c_mult0;
            off1[j] = (int)lr.off1 + (v.c.decides ? cj - s.c_split : cj) * s.c_mult1;
        }
    }
    return s;
}

// issue the global loads of the tile whose reduction index starts at c0
template <int KIND, int VEC>
__device__ __forceinline__ void stage_fetch(const StageState &s, const int (&off0)[StageCfg<KIND, VEC>::NV],
                                            const int (&off1)[StageCfg<KIND, VEC>::NV],
                                            typename VecOf<VEC>::type (&regs)[StageCfg<KIND, VEC>::NV], int c0)
{
    typedef StageCfg<KIND, VEC> C;
    typedef typename C::V V;
    const bool interior = c0 + KT <= s.c_lim;          // uniform
    if (KIND == LD_KC) {
        const int c = interior ? c0 + s.col : max(0, min(c0 + s.col, s.c_lim - VEC));
        if (!s.c_decides) {                            // uniform: a plain operand
            const __bf16 *base = s.base0 + c;
#pragma unroll
            for (int j = 0; j < C::NV; ++j) regs[j] = load_global<V>(base + off0[j]);
        } else {
            const bool reg1 = c >= s.c_split;
            const unsigned t = reg1 ? (unsigned)(c - s.c_split) : 0u;
            const unsigned i = __umulhi(t, s.c_magic);
            const int w = (int)(t - i * (unsigned)s.c_seg);
            const int slot = (int)i + ((int)i >= s.c_skip ? 1 : 0);
            const int coff = reg1 ? slot * s.c_seg_stride + w : c;
            const __bf16 *base = (reg1 ? s.base1 : s.base0) + coff;
#pragma unroll
            for (int j = 0; j < C::NV; ++j) regs[j] = load_global<V>(base + (reg1 ? off1[j] : off0[j]));
        }
    } else {
        if (interior && !s.c_decides) {
            // c0 * stride is the same for every lane: scalar unit
            const int step_off = s.r_region > 0 ? c0 * s.c_mult1 : c0 * s.c_mult0;
            const __bf16 *base = s.tbase + step_off;
#pragma unroll
            for (int j = 0; j < C::NV; ++j) regs[j] = load_global<V>(base + (s.r_region > 0 ? off1[j] : off0[j]));
        } else {
#pragma unroll
            for (int j = 0; j < C::NV; ++j) {
                const int cj = s.row0 + j * C::ROW_STEP;
                const int c = interior ? c0 + cj : max(0, min(c0 + cj, s.c_lim - 1));
                const bool reg1 = s.c_decides ? (c >= s.c_split) : (s.r_region > 0);
                const int off = reg1 ? off1[j] + (c - cj) * s.c_mult1 : off0[j] + (c - cj) * s.c_mult0;
                regs[j] = load_global<V>((reg1 ? s.base1 : s.base0) + off);
            }
        }
    }
}

// move the tile fetched for reduction start c0 into LDS, zeroing reduction indices >= c_lim
template <int KIND, int VEC>
__device__ __forceinline__ void stage_store(const StageState &s, const typename VecOf<VEC>::type (&regs)[StageCfg<KIND, VEC>::NV],
                                            __bf16 *tile, int c0)
{
    typedef StageCfg<KIND, VEC> C;
    typedef typename C::V V;
    __bf16 *dst = tile + s.row0 * C::PITCH + s.col;
    if (c0 + KT <= s.c_lim) {                          // uniform: a full tile
#pragma unroll
        for (int j = 0; j < C::NV; ++j) *(V *)(dst + j * C::ROW_STEP * C::PITCH) = regs[j];
    } else {
#pragma unroll
        for (int j = 0; j < C::NV; ++j) {
            const int c = KIND == LD_KC ? c0 + s.col : c0 + s.row0 + j * C::ROW_STEP;
            const uint32_t keep = c < s.c_lim ? 0xffffffffu : 0u;
            *(V *)(dst + j * C::ROW_STEP * C::PITCH) = regs[j] & keep;
        }
    }
}

// MFMA operand (rows rbase..rbase+31 of the tile, reduction sub-step ks of 16) for this lane
template <int KIND>
__device__ __forceinline__ bf16x8 lds_operand(const __bf16 *tile, int rbase, int ks, int lane)
{
    if (KIND == LD_KC) {
        return *(const bf16x8 *)(tile + (rbase + (lane & 31)) * KC_PITCH + ks * 16 + (lane >> 5) * 8);
    } else {
        const int krow = ks * 16 + (lane >> 5) * 8 + ((lane & 15) >> 2);
        const int rcol = rbase + ((lane >> 4) & 1) * 16 + (lane & 3) * 4;
        const __bf16 *p = tile + krow * KM_PITCH + rcol;
        typedef __attribute__((address_space(3))) s16x4 lds_s16x4;
        s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4 *)(p));
        s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4 *)(p + 4 * KM_PITCH));
        union { struct { s16x4 a, b; } s; bf16x8 v; } u;
        u.s.a = lo; u.s.b = hi;
        return u.v;
    }
}

struct MfmaParams {
    View a, b, o;        // o: the row index must not decide the region (true for every output here)
    Epilogue ep;
    int M, N, K;
    int tiles_m, tiles_n;
    int ksplit;          // > 1: the reduction range is cut into ksplit pieces, results added atomically
    int k_per_split;     // multiple of KT
    int total_wg;
};

template <int KA, int KB>
__device__ __forceinline__ void mfma_tile(f32x16 (&acc)[2][2], const __bf16 *ta, const __bf16 *tb, int wm, int wn, int lane)
{
#pragma unroll
    for (int kk = 0; kk < KT / 16; ++kk) {
        bf16x8 av[2], bv[2];
        av[0] = lds_operand<KA>(ta, wm, kk, lane);
        av[1] = lds_operand<KA>(ta, wm + 32, kk, lane);
        bv[0] = lds_operand<KB>(tb, wn, kk, lane);
        bv[1] = lds_operand<KB>(tb, wn + 32, kk, lane);
#pragma unroll
        for (int i = 0; i < 2; ++i)
#pragma unroll
            for (int j = 0; j < 2; ++j)
                acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(av[i], bv[j], acc[i][j], 0, 0, 0);
    }
}

// Writes the 32 x 64 block of accumulators acc[j] (two 32 x 32 MFMA tiles side by side) whose first
// row is mrow0 and first column ncol0.  A lane holds column (lane & 31) of each tile and rows
// 8*(e/4) + 4*(lane>>5) + e%4.
template <typename TOut, bool ATOMIC>
__device__ __forceinline__ void epilogue_rows(const MfmaParams &P, int g, const f32x16 (&acc)[2], int mrow0, int ncol0, int lane)
{
    TOut *o0 = (TOut *)P.o.p0 + g * P.o.g0, *o1 = (TOut *)P.o.p1 + g * P.o.g1;
    const int skip_o = P.o.skip0 + g * P.o.skip_g;
    const Epilogue &ep = P.ep;
#pragma unroll
    for (int j = 0; j < 2; ++j) {
        const int n = ncol0 + j * 32 + (lane & 31);
        if (n >= P.N) continue;
        const Loc ln = locate(P.o.c, n, skip_o);
        const int region = ln.region > 0 ? 1 : 0;
        TOut *obase = region ? o1 + ln.off1 : o0 + ln.off0;
        const int64_t row_mult = region ? P.o.r.mult1 : P.o.r.mult0;
        float bias = 0.f;
        if (ep.mode == EPI_BIAS_ACT) bias = (float)((const __bf16 *)ep.bias + g * ep.bias_g)[n];
        const int64_t aux_base = g * ep.aux_g + n;
#pragma unroll
        for (int e = 0; e < 16; ++e) {
            const int m = mrow0 + (e >> 2) * 8 + (lane >> 5) * 4 + (e & 3);
            if (m >= P.M) continue;
            float v = acc[j][e];
            if (ep.mode == EPI_BIAS_ACT) {
                v += bias;
                if (ep.aux) {
                    const int64_t at = aux_base + (int64_t)m * ep.aux_ld;
                    if (ep.aux_f32) ((float *)ep.aux)[at] = v; else ((__bf16 *)ep.aux)[at] = (__bf16)v;
                }
                v = act_apply(ep.act, v);
            } else if (ep.mode == EPI_DACT) {
                const int64_t at = aux_base + (int64_t)m * ep.aux_ld;
                const float a = ep.aux_f32 ? ((const float *)ep.aux)[at] : (float)((const __bf16 *)ep.aux)[at];
                v *= act_deriv(ep.act, a);
            }
            TOut *dst = obase + (int64_t)m * row_mult;
            if constexpr (ATOMIC) unsafeAtomicAdd((float *)dst, v); else *dst = from_f32<TOut>(v);
        }
    }
}

#ifdef PHANTOM_TIMELINE   // cycle stamps for the development micro-benchmark, never built into the library
#define PH_STAMP(slot) do { __builtin_amdgcn_sched_barrier(0); if (blockIdx.x == 0 && lane == 0 && wave == 0 && t < 16) \
        ((long long *)P.ep.aux)[(team * 16 + t) * 8 + (slot)] = clock64(); __builtin_amdgcn_sched_barrier(0); } while (0)
#else
#define PH_STAMP(slot) do { } while (0)
#endif

// 512 threads = two teams of 4 wavefronts.  Both teams work on the SAME 128 x 128 tile of C; team q
// takes the reduction steps q, q+2, q+4, ... with its own pair of LDS stages, so every SIMD holds two
// wavefronts whose loads, LDS traffic and MFMAs interleave, without reading any operand twice.  At
// the end the teams swap half of their accumulators through LDS: team 0 finishes and writes the
// upper 32 rows of every wavefront quadrant, team 1 the lower 32.
// One launch may carry two independent products of the same operand layout and output type (the
// layer update with the compression, the error compression with the input gradient, the weight
// gradients with the compressor gradient): their workgroups run side by side instead of one thin
// launch waiting for the other.
struct MfmaBatch {
    MfmaParams p[2];
    int count;
    int total_wg;
};

template <int KA, int KB, int VA, int VB, typename TOut, bool ATOMIC>
__global__ __launch_bounds__(512, 1) void gemm_mfma_kernel(MfmaBatch batch)
{
    extern __shared__ __attribute__((aligned(16))) unsigned char smem_raw[];

    // XCD-aware id: hardware deals workgroup ids round-robin over 8 XCDs
    int wg = blockIdx.x;
    {
        const int per = batch.total_wg >> 3;
        if (wg < per * 8) wg = (wg & 7) * per + (wg >> 3);
    }
    const bool second = wg >= batch.p[0].total_wg;
    if (second) wg -= batch.p[0].total_wg;
    const MfmaParams &P = batch.p[second ? 1 : 0];
    const int tiles = P.tiles_m * P.tiles_n;
    const int g = wg / (tiles * P.ksplit);
    int rem = wg - g * tiles * P.ksplit;
    const int ks = rem / tiles;
    rem -= ks * tiles;
    // tiles are walked in bands of RASTER_M tile rows, down the band first: the workgroups that run
    // together on one XCD then cover a near-square patch of C and share both operand panels in L2
    constexpr int RASTER_M = 8;
    const int band = rem / (RASTER_M * P.tiles_n);
    const int in_band = rem - band * (RASTER_M * P.tiles_n);
    const int band_rows = min(P.tiles_m - band * RASTER_M, RASTER_M);
    const int tn = in_band / band_rows;
    const int tm = band * RASTER_M + (in_band - tn * band_rows);
    const int m0 = tm * MT, n0 = tn * MT;
    const int k_begin = ks * P.k_per_split;
    const int k_end = min(P.K, k_begin + P.k_per_split);

    const int team = threadIdx.x >> 8;
    const int tid = threadIdx.x & 255, lane = tid & 63, wave = tid >> 6;
    const int wm = (wave >> 1) * 64, wn = (wave & 1) * 64;

    typedef StageCfg<KA, VA> SA;
    typedef StageCfg<KB, VB> SB;
    int a_off0[SA::NV], a_off1[SA::NV], b_off0[SB::NV], b_off1[SB::NV];
    const StageState sa = stage_init<KA, VA>(P.a, g, m0, P.M, k_end, tid, a_off0, a_off1);
    const StageState sb = stage_init<KB, VB>(P.b, g, n0, P.N, k_end, tid, b_off0, b_off1);
    typename SA::V ra0[SA::NV], ra1[SA::NV];
    typename SB::V rb0[SB::NV], rb1[SB::NV];
#define PH_FETCH(set, c0) do { stage_fetch<KA, VA>(sa, a_off0, a_off1, ra##set, (c0)); \
                               stage_fetch<KB, VB>(sb, b_off0, b_off1, rb##set, (c0)); } while (0)
#define PH_STORE(set, stage, c0) do { stage_store<KA, VA>(sa, ra##set, s##stage##a, (c0)); \
                                      stage_store<KB, VB>(sb, rb##set, s##stage##b, (c0)); } while (0)

    f32x16 acc[2][2];
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;

    __bf16 *smem = (__bf16 *)smem_raw + team * 4 * TILE_ELEMS;
    __bf16 *s0a = smem, *s0b = smem + TILE_ELEMS, *s1a = smem + 2 * TILE_ELEMS, *s1b = smem + 3 * TILE_ELEMS;
    // both teams run the same number of steps (one barrier serves all 512 threads); a step past the
    // end of the reduction range multiplies zeros
    const int all_steps = (k_end - k_begin + KT - 1) / KT;
    const int steps = (all_steps + 1) >> 1;
    const int kfirst = k_begin + team * KT;     // reduction start of this team's step i: kfirst + 2*i*KT
    constexpr int KS = 2 * KT;

    // prologue: step 0 into LDS stage 0; steps 1 and 2 on their way in register sets 1 and 0
    PH_FETCH(0, kfirst);
    PH_FETCH(1, kfirst + KS);
    PH_STORE(0, 0, kfirst);
    PH_FETCH(0, kfirst + 2 * KS);
    __syncthreads();

    // step t multiplies LDS stage t%2; on entry the operands of step t+1 sit in register set (t+1)%2 and
    // are moved to the other LDS stage, whose readers finished before the barrier that ended step t-1
    int t = 0;
    for (; t + 1 < steps; t += 2) {
        PH_STAMP(0);
        PH_STORE(1, 1, kfirst + (t + 1) * KS);
        PH_STAMP(1);
        PH_FETCH(1, kfirst + (t + 3) * KS);
        PH_STAMP(2);
        mfma_tile<KA, KB>(acc, s0a, s0b, wm, wn, lane);
        PH_STAMP(3);
        __syncthreads();
        PH_STAMP(4);
        PH_STORE(0, 0, kfirst + (t + 2) * KS);
        PH_FETCH(0, kfirst + (t + 4) * KS);
        mfma_tile<KA, KB>(acc, s1a, s1b, wm, wn, lane);
        __syncthreads();
    }
    if (t < steps) mfma_tile<KA, KB>(acc, s0a, s0b, wm, wn, lane);
    __syncthreads();
#undef PH_FETCH
#undef PH_STORE

    // the two teams hold partial sums of the same tile: swap halves through LDS (2 x 32 KB of floats)
    float *xch = (float *)smem_raw;
    {
        float *mine = xch + (team ? 0 : 256 * 32) + tid;      // team 1 gives its upper rows, team 0 its lower rows
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int e = 0; e < 16; ++e)
                mine[(j * 16 + e) * 256] = team ? acc[0][j][e] : acc[1][j][e];
    }
    __syncthreads();
    {
        const float *theirs = xch + (team ? 256 * 32 : 0) + tid;
        if (team == 0) {
#pragma unroll
            for (int j = 0; j < 2; ++j)
#pragma unroll
                for (int e = 0; e < 16; ++e) acc[0][j][e] += theirs[(j * 16 + e) * 256];
            epilogue_rows<TOut, ATOMIC>(P, g, acc[0], m0 + wm, n0 + wn, lane);
        } else {
#pragma unroll
            for (int j = 0; j < 2; ++j)
#pragma unroll
                for (int e = 0; e < 16; ++e) acc[1][j][e] += theirs[(j * 16 + e) * 256];
            epilogue_rows<TOut, ATOMIC>(P, g, acc[1], m0 + wm + 32, n0 + wn, lane);
        }
    }
}

}  // namespace phantom

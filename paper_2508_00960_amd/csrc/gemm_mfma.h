// bf16 x bf16 -> fp32 tiled product on the CDNA4 matrix cores:
//   C(m, n) = sum_c A(m, c) * B(n, c),   A, B and C given as Views (views.h).
//
// One workgroup (256 threads = 4 wavefronts of 64) owns a 128 x 128 tile of C and walks the
// reduction index in steps of 64.  Each wavefront owns a 64 x 64 quadrant = 2 x 2 MFMA tiles of
// v_mfma_f32_32x32x16_bf16, accumulators in registers (64 floats per lane).
//
// Operand staging: global -> registers (next tile, issued before the MFMAs of the current tile)
// -> LDS (two stages).  Two loader kinds, chosen per operand:
//   LD_KC  the reduction index is contiguous in memory (X, G, L, D in the forward; delta in dX).
//          LDS tile [128 rows][64 + 8]; a lane's MFMA operand is one 16-byte LDS read.
//   LD_KM  the free index is contiguous, the reduction index strides (L, C, D in dX and error
//          compression; delta, X, G in the weight gradients).  LDS tile [64][128 + 16]; the MFMA
//          operand is built by two ds_read_b64_tr_b16 (the gfx950 transposing LDS read: within 16
//          lanes, lanes 4j..4j+3 supply row j of a 4 x 16 block, lane i receives column i).
// The peers' segments (G_i, D_i) are addressed in place through the View; VEC (8, 4 or 2
// elements) is the widest vector that never straddles a segment boundary.
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
constexpr int MFMA_LDS_BYTES = 2 /*stages*/ * 2 /*operands*/ * TILE_ELEMS * 2;

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

template <int VEC> struct VecOf;
template <> struct VecOf<8> { typedef uint4 type; };
template <> struct VecOf<4> { typedef uint2 type; };
template <> struct VecOf<2> { typedef uint32_t type; };

template <int VEC> __device__ __forceinline__ typename VecOf<VEC>::type vec_zero();
template <> __device__ __forceinline__ uint4 vec_zero<8>() { return make_uint4(0, 0, 0, 0); }
template <> __device__ __forceinline__ uint2 vec_zero<4>() { return make_uint2(0, 0); }
template <> __device__ __forceinline__ uint32_t vec_zero<2>() { return 0u; }

// ---- staging one operand tile ---------------------------------------------------------
// KIND == LD_KC: tile rows = free index r in [r0, r0+128), columns = reduction index c in [c0, c0+64)
// KIND == LD_KM: tile rows = reduction index c in [c0, c0+64), columns = free index r in [r0, r0+128)
template <int KIND, int VEC>
struct Stager {
    typedef typename VecOf<VEC>::type V;
    static constexpr int PER_ROW = (KIND == LD_KC ? KT : MT) / VEC;   // vectors per LDS row
    static constexpr int ROWS = KIND == LD_KC ? MT : KT;
    static constexpr int NV = ROWS * PER_ROW / 256;                   // vectors per thread
    static constexpr int ROW_STEP = 256 / PER_ROW;
    static constexpr int PITCH = KIND == LD_KC ? KC_PITCH : KM_PITCH;

    const __bf16 *p0, *p1;
    Axis ax_c;          // the axis that changes from step to step
    int skip;
    int col;            // this thread's vector column inside the tile (elements)
    int row0;           // this thread's first tile row
    int r_lim, c_lim;   // extents of the free and the reduction index
    // LD_KC: r does not decide; row offsets are multiples of mult0/mult1
    int64_t r_mult0, r_mult1;
    int rbase;          // r0 (LD_KC) ; unused (LD_KM)
    // LD_KM: the thread's r is fixed for the whole kernel
    Loc lr;
    bool r_ok;
    V regs[NV];

    __device__ __forceinline__ void init(const View &v, int g, int r0, int r_limit, int c_limit, int tid)
    {
        p0 = (const __bf16 *)v.p0 + g * v.g0;
        p1 = (const __bf16 *)v.p1 + g * v.g1;
        ax_c = v.c;
        skip = v.skip0 + g * v.skip_g;
        col = (tid % PER_ROW) * VEC;
        row0 = tid / PER_ROW;
        r_lim = r_limit; c_lim = c_limit;
        if (KIND == LD_KC) {
            r_mult0 = v.r.mult0; r_mult1 = v.r.mult1; rbase = r0;
            lr = Loc{0, 0, -1}; r_ok = true;
        } else {
            const int r = r0 + col;
            r_ok = r < r_limit;
            lr = locate(v.r, r_ok ? r : 0, skip);
            r_mult0 = r_mult1 = 0; rbase = 0;
        }
    }

    // issue the global loads of the tile whose reduction index starts at c0
    __device__ __forceinline__ void fetch(int c0)
    {
        if (KIND == LD_KC) {
            const int c = c0 + col;
            const bool c_ok = c < c_lim;
            const Loc lc = locate(ax_c, c_ok ? c : 0, skip);
            const int region = lc.region > 0 ? 1 : 0;
            const __bf16 *base = (region ? p1 + lc.off1 : p0 + lc.off0);
            const int64_t rm = region ? r_mult1 : r_mult0;
#pragma unroll
            for (int j = 0; j < NV; ++j) {
                const int r = rbase + row0 + j * ROW_STEP;
                regs[j] = (c_ok && r < r_lim) ? *(const V *)(base + (int64_t)r * rm) : vec_zero<VEC>();
            }
        } else {
#pragma unroll
            for (int j = 0; j < NV; ++j) {
                const int c = c0 + row0 + j * ROW_STEP;
                const bool ok = r_ok && c < c_lim;
                const Loc lc = locate(ax_c, ok ? c : 0, skip);
                int region;
                const int64_t off = join(lr, lc, region);
                regs[j] = ok ? *(const V *)((region ? p1 : p0) + off) : vec_zero<VEC>();
            }
        }
    }

    __device__ __forceinline__ void store(__bf16 *tile) const
    {
#pragma unroll
        for (int j = 0; j < NV; ++j)
            *(V *)(tile + (row0 + j * ROW_STEP) * PITCH + col) = regs[j];
    }
};

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
    View a, b, o;
    Epilogue ep;
    int M, N, K;
    int tiles_m, tiles_n;
    int ksplit;          // > 1: the reduction range is cut into ksplit pieces, results added atomically
    int k_per_split;     // multiple of KT
    int total_wg;
};

template <int KA, int KB, int VA, int VB, typename TOut, bool ATOMIC>
__global__ __launch_bounds__(256) void gemm_mfma_kernel(MfmaParams P)
{
    extern __shared__ __attribute__((aligned(16))) unsigned char smem_raw[];
    __bf16 *smem = (__bf16 *)smem_raw;

    // XCD-aware id: hardware deals workgroup ids round-robin over 8 XCDs
    int wg = blockIdx.x;
    {
        const int per = P.total_wg >> 3;
        if (wg < per * 8) wg = (wg & 7) * per + (wg >> 3);
    }
    const int tiles = P.tiles_m * P.tiles_n;
    const int g = wg / (tiles * P.ksplit);
    int rem = wg - g * tiles * P.ksplit;
    const int ks = rem / tiles;
    rem -= ks * tiles;
    const int tm = rem / P.tiles_n, tn = rem - tm * P.tiles_n;
    const int m0 = tm * MT, n0 = tn * MT;
    const int k_begin = ks * P.k_per_split;
    const int k_end = min(P.K, k_begin + P.k_per_split);

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = (wave >> 1) * 64, wn = (wave & 1) * 64;

    Stager<KA, VA> sa;
    Stager<KB, VB> sb;
    sa.init(P.a, g, m0, P.M, k_end, tid);
    sb.init(P.b, g, n0, P.N, k_end, tid);

    f32x16 acc[2][2];
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;

    const int steps = (k_end - k_begin + KT - 1) / KT;
    if (steps > 0) {
        sa.fetch(k_begin);
        sb.fetch(k_begin);
        sa.store(smem);
        sb.store(smem + TILE_ELEMS);
    }
    __syncthreads();

    for (int t = 0; t < steps; ++t) {
        const __bf16 *ta = smem + (t & 1) * 2 * TILE_ELEMS;
        const __bf16 *tb = ta + TILE_ELEMS;
        const bool more = t + 1 < steps;
        if (more) {
            sa.fetch(k_begin + (t + 1) * KT);
            sb.fetch(k_begin + (t + 1) * KT);
        }
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
        if (more) {
            __bf16 *na = smem + ((t + 1) & 1) * 2 * TILE_ELEMS;
            sa.store(na);
            sb.store(na + TILE_ELEMS);
        }
        __syncthreads();
    }

    // epilogue: lane holds, for each 32x32 block, column (lane & 31) and rows 8*(e/4) + 4*(lane>>5) + e%4
    TOut *o0 = (TOut *)P.o.p0 + g * P.o.g0, *o1 = (TOut *)P.o.p1 + g * P.o.g1;
    const int skip_o = P.o.skip0 + g * P.o.skip_g;
    const Epilogue &ep = P.ep;
#pragma unroll
    for (int j = 0; j < 2; ++j) {
        const int n = n0 + wn + j * 32 + (lane & 31);
        if (n >= P.N) continue;
        const Loc ln = locate(P.o.c, n, skip_o);
        float bias = 0.f;
        if (ep.mode == EPI_BIAS_ACT) bias = (float)((const __bf16 *)ep.bias + g * ep.bias_g)[n];
#pragma unroll
        for (int i = 0; i < 2; ++i) {
#pragma unroll
            for (int e = 0; e < 16; ++e) {
                const int m = m0 + wm + i * 32 + (e >> 2) * 8 + (lane >> 5) * 4 + (e & 3);
                if (m >= P.M) continue;
                const Loc lm = locate(P.o.r, m, skip_o);
                int region;
                const int64_t off = join(lm, ln, region);
                float v = acc[i][j][e];
                if (ep.mode == EPI_BIAS_ACT) {
                    v += bias;
                    if (ep.aux) {
                        const int64_t at = g * ep.aux_g + (int64_t)m * ep.aux_ld + n;
                        if (ep.aux_f32) ((float *)ep.aux)[at] = v; else ((__bf16 *)ep.aux)[at] = (__bf16)v;
                    }
                    v = act_apply(ep.act, v);
                } else if (ep.mode == EPI_DACT) {
                    const int64_t at = g * ep.aux_g + (int64_t)m * ep.aux_ld + n;
                    const float a = ep.aux_f32 ? ((const float *)ep.aux)[at] : (float)((const __bf16 *)ep.aux)[at];
                    v *= act_deriv(ep.act, a);
                }
                TOut *dst = (region ? o1 : o0) + off;
                if constexpr (ATOMIC) unsafeAtomicAdd((float *)dst, v); else *dst = from_f32<TOut>(v);
            }
        }
    }
}

}  // namespace phantom

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
//          compression; delta, X, G in the weight gradients).  LDS tile [64][128 + 32]; the MFMA
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
//
// An operand's tail block may also be a sum that is formed on read (SumOnRead, fetch_summed): the in-memory
// reduce-scatter of the backward pass as part of the input gradient's loader.
//
// Kernels in this file, all built on mfma_workgroup (one workgroup's work on one product):
//   gemm_mfma_kernel       one product, or two of the same operand layout and output type
//   gemm_mfma_table_kernel one rank: the weight + compressor gradients of all layers, parameter blocks in device memory
//   gemm_mfma_tail_kernel  weight + compressor gradients with riders of other layouts (the error compression of
//                          the layer below, the SGD update of the layer above)
//   gemm_mfma_fwd_kernel   a rank's layer update with the thin compression shared out over its workgroups
#pragma once
#include "common.h"
#include "elementwise.h"    // SgdBatch, sgd_rider
#include "gemm_generic.h"   // Epilogue, EPI_*
#include "thin_product.h"   // thin_workgroup
#include "views.h"

namespace phantom {

enum { LD_KC = 0, LD_KM = 1 };

constexpr int MT = 128;               // tile rows (m) and columns (n)
constexpr int KT = 64;                // reduction step
constexpr int KC_PITCH = KT + 8;      // elements per LDS row, K-contiguous tile [128][72]
#ifndef PH_KM_PITCH
#define PH_KM_PITCH (MT + 32)
#endif
// elements per LDS row, K-major tile [64][160]: 80 words = 16 mod 64, so the four rows that 16 lanes of a
// transposing read touch start 16 banks apart and the next 16 lanes (16 columns = 8 banks further) fall between
// them; with 144 the two half-groups met on the same banks (SQ_LDS_BANK_CONFLICT: a quarter of the LDS cycles)
constexpr int KM_PITCH = PH_KM_PITCH;
constexpr int TILE_ELEMS = (MT * KC_PITCH > KT * KM_PITCH) ? MT * KC_PITCH : KT * KM_PITCH;   // one operand stage
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

// The epilogues' loads and stores, likewise: their pointers come out of parameter blocks, so the compiler would
// take them for generic ones and use flat instructions (which also count as LDS operations: every wait for an LDS
// read then waits for all of them).  _nt: streaming (read or written once).
template <typename V> __device__ __forceinline__ V gload(const void *p) { return *(const __attribute__((address_space(1))) V *)(uintptr_t)p; }
template <typename V> __device__ __forceinline__ V gload_nt(const void *p)
{
    return __builtin_nontemporal_load((const __attribute__((address_space(1))) V *)(uintptr_t)p);
}
template <typename V> __device__ __forceinline__ void gstore(void *p, const V &v) { *(__attribute__((address_space(1))) V *)(uintptr_t)p = v; }
template <typename V> __device__ __forceinline__ void gstore_nt(void *p, const V &v)
{
    __builtin_nontemporal_store(v, (__attribute__((address_space(1))) V *)(uintptr_t)p);
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
// PART = 2: the 256 threads of a team stage only half of the tile's rows (the other team stages the
// other half of an operand tile that both teams read; see the DUAL mode of gemm_mfma_kernel)
template <int KIND, int VEC, int PART = 1>
struct StageCfg {
    typedef typename VecOf<VEC>::type V;
    static constexpr int PER_ROW = (KIND == LD_KC ? KT : MT) / VEC;   // vectors per LDS row
    static constexpr int ROWS = KIND == LD_KC ? MT : KT;
    static constexpr int NV = ROWS * PER_ROW / 256 / PART;            // vectors per thread
    static_assert(NV >= 1 && NV * 256 * PART == ROWS * PER_ROW, "the team's threads tile its share of the rows");
    static constexpr int ROW_STEP = 256 / PER_ROW;
    static constexpr int PITCH = KIND == LD_KC ? KC_PITCH : KM_PITCH;
};

struct StageState {          // scalars only, so that it lives in registers
    const __bf16 *base0, *base1;
    int col, row0;           // this thread's vector column (elements) and first row inside the tile
    int c_lim;
    int c_decides, c_split, c_seg, c_skip;
    unsigned c_magic;        // ceil(2^32 / c_seg)
    int c_mult0, c_mult1, c_seg_stride;
    int r_region;            // LD_KM: region of the thread's fixed free index (-1: the reduction index decides)
    // "regular" shapes: a 64-wide step of the reduction index never straddles the head / tail boundary,
    // and a peer segment either holds whole steps or a whole number of segments fills a step
    // (n/p a multiple of 64; k a divisor or a multiple of 64).  Then the region is the same for the
    // whole workgroup in every step and the addressing of a full tile is almost free.
    int regular;
    int col_seg, col_in_seg; // LD_KC regular, k < 64: segment and position of the thread's column inside a step
};

// off0[j], off1[j]: element offsets of the thread's j-th vector that do not depend on the step, in
// region 0 and region 1.  LD_KC: row * row stride.  LD_KM: fixed free-index offset + (row0 + j*ROW_STEP) * c stride.
template <int KIND, int VEC, int PART = 1>
__device__ __forceinline__ StageState stage_init(const View &v, int g, int r0, int r_limit, int c_limit, int tid,
                                                 int (&off0)[StageCfg<KIND, VEC, PART>::NV],
                                                 int (&off1)[StageCfg<KIND, VEC, PART>::NV], int row_shift = 0)
{
    typedef StageCfg<KIND, VEC, PART> C;
    StageState s;
    s.base0 = (const __bf16 *)v.p0 + g * v.g0;
    s.base1 = (const __bf16 *)v.p1 + g * v.g1;
    const int skip = v.skip0 + g * v.skip_g;
    s.col = (tid % C::PER_ROW) * VEC;
    s.row0 = tid / C::PER_ROW + row_shift;           // row_shift: first row of this team's share (PART = 2)
    s.c_lim = c_limit;
    s.c_decides = v.c.decides;
    s.c_split = v.c.decides ? v.c.split : 0x7fffffff;
    s.c_seg = v.c.seg; s.c_skip = skip;
    s.c_magic = v.c.magic;                           // the MFMA path never sees seg == 1 (VEC >= 2 divides seg)
    s.c_mult0 = (int)v.c.mult0; s.c_mult1 = (int)v.c.mult1; s.c_seg_stride = (int)v.c.seg_stride;
    s.r_region = -1;
    s.col_seg = 0; s.col_in_seg = s.col;
    if (KIND == LD_KC) {
        s.regular = !v.c.decides || (v.c.split % KT == 0 && (KT % v.c.seg == 0 || v.c.seg % KT == 0));
        if (s.regular && v.c.decides && v.c.seg < KT) {
            s.col_seg = (int)__umulhi((unsigned)s.col, v.c.magic);
            s.col_in_seg = s.col - s.col_seg * v.c.seg;
        }
#pragma unroll
        for (int j = 0; j < C::NV; ++j) {
            const int r = min(r0 + s.row0 + j * C::ROW_STEP, r_limit - 1);
            off0[j] = r * (int)v.r.mult0;
            off1[j] = r * (int)v.r.mult1;
        }
    } else {
        // the region of the free index is the same for the whole tile unless the tile straddles the split
        const bool r_uniform = !v.r.decides || r0 + MT <= v.r.split || r0 >= v.r.split;
        s.regular = r_uniform && (!v.c.decides || v.c.split % KT == 0);
        const int r = min(r0 + s.col, r_limit - VEC);
        const Loc lr = locate(v.r, r, skip);
        s.r_region = lr.region;
        // one region for the whole kernel (the usual case): fold the choice into base0 / off0 / c_mult0
        const bool fold = s.regular && !v.c.decides && __builtin_amdgcn_readfirstlane(lr.region) > 0;
        if (fold) { s.base0 = s.base1; s.c_mult0 = s.c_mult1; }
#pragma unroll
        for (int j = 0; j < C::NV; ++j) {
            const int cj = s.row0 + j * C::ROW_STEP;
            off1[j] = (int)lr.off1 + (v.c.decides ? cj - s.c_split : cj) * s.c_mult1;
            off0[j] = fold ? off1[j] : (int)lr.off0 + cj * s.c_mult0;
        }
    }
    return s;
}

// issue the global loads of vectors J0 .. J1-1 of the tile whose reduction index starts at c0 (any shape).
// CAREFUL = false: the caller guarantees c0 + KT <= c_lim (a full interior tile).
template <int KIND, int VEC, bool CAREFUL, int PART = 1, int J0 = 0, int J1 = StageCfg<KIND, VEC, PART>::NV>
__device__ __forceinline__ void stage_fetch(const StageState &s, const int (&off0)[StageCfg<KIND, VEC, PART>::NV],
                                            const int (&off1)[StageCfg<KIND, VEC, PART>::NV],
                                            typename VecOf<VEC>::type (&regs)[StageCfg<KIND, VEC, PART>::NV], int c0)
{
    typedef StageCfg<KIND, VEC, PART> C;
    typedef typename C::V V;
    const bool interior = !CAREFUL || c0 + KT <= s.c_lim;   // uniform
    if (KIND == LD_KC) {
        const int c = interior ? c0 + s.col : max(0, min(c0 + s.col, s.c_lim - VEC));
        if (!s.c_decides) {                            // uniform: a plain operand
            const __bf16 *base = s.base0 + c;
#pragma unroll
            for (int j = J0; j < J1; ++j) regs[j] = load_global<V>(base + off0[j]);
        } else {
            const bool reg1 = c >= s.c_split;
            const unsigned t = reg1 ? (unsigned)(c - s.c_split) : 0u;
            const unsigned i = __umulhi(t, s.c_magic);
            const int w = (int)(t - i * (unsigned)s.c_seg);
            const int slot = (int)i + ((int)i >= s.c_skip ? 1 : 0);
            const int coff = reg1 ? slot * s.c_seg_stride + w : c;
            const __bf16 *base = (reg1 ? s.base1 : s.base0) + coff;
#pragma unroll
            for (int j = J0; j < J1; ++j) {
                const int o0 = off0[j], o1 = off1[j];
                regs[j] = load_global<V>(base + (reg1 ? o1 : o0));
            }
        }
    } else {
#pragma unroll
        for (int j = J0; j < J1; ++j) {
            const int cj = s.row0 + j * C::ROW_STEP;
            const int c = interior ? c0 + cj : max(0, min(c0 + cj, s.c_lim - 1));
            const bool reg1 = s.c_decides ? (c >= s.c_split) : (s.r_region > 0);
            const int o0 = off0[j], o1 = off1[j];
            const int off = reg1 ? o1 + (c - cj) * s.c_mult1 : o0 + (c - cj) * s.c_mult0;
            regs[j] = load_global<V>((reg1 ? s.base1 : s.base0) + off);
        }
    }
}

// whether stage_init would call the tile whose free index starts at r0 regular (same predicate, no state)
template <int KIND>
__device__ __forceinline__ bool tile_is_regular(const View &v, int r0)
{
    if (KIND == LD_KC) return !v.c.decides || (v.c.split % KT == 0 && (KT % v.c.seg == 0 || v.c.seg % KT == 0));
    const bool r_uniform = !v.r.decides || r0 + MT <= v.r.split || r0 >= v.r.split;
    return r_uniform && (!v.c.decides || v.c.split % KT == 0);
}

// ---- the fast path: regular shapes, full interior tiles ----------------------------------
// What a step's loads share: a base pointer that is the same for the whole workgroup (it lives in
// scalar registers and the load takes it as its scalar base), which of the two offset arrays
// applies, and one 32-bit term added to every offset.  No branch, no clamp, no 64-bit vector math.
struct FastStep {
    const __bf16 *base;
    bool tail;          // uniform: offsets come from off1
    unsigned add;
};

template <int KIND, int VEC>
__device__ __forceinline__ FastStep fast_step_addr(const StageState &s, int c0 /* uniform, multiple of KT */)
{
    FastStep f;
    const bool head = c0 < s.c_split;                  // c_split = INT_MAX when c does not decide
    if (KIND == LD_KC) {
        const unsigned t0 = head ? 0u : (unsigned)(c0 - s.c_split);
        const unsigned i0 = __umulhi(t0, s.c_magic);   // first segment the step touches (scalar unit)
        const int rem = (int)(t0 - i0 * (unsigned)s.c_seg);   // 0 unless a segment holds several steps
        const int i = (int)i0 + s.col_seg;
        const int slot = i + (i >= s.c_skip ? 1 : 0);
        const int coff = slot * s.c_seg_stride + rem + s.col_in_seg;
        f.base = head ? s.base0 : s.base1;
        f.tail = !head;
        f.add = (unsigned)(head ? c0 + s.col : coff);
    } else {
        // stage_init left the free index's region folded into base0 / off0 / c_mult0 when c does not decide
        f.base = head ? s.base0 + (int64_t)c0 * s.c_mult0 : s.base1 + (int64_t)(c0 - s.c_split) * s.c_mult1;
        f.tail = !head;
        f.add = head ? 0u : (unsigned)(s.c_split * s.c_mult1);   // off1 holds (row - split) * stride: make it non-negative
    }
    return f;
}

template <int KIND, int VEC, int PART, int J0, int J1>
__device__ __forceinline__ void fast_fetch(const FastStep &f, const int (&off0)[StageCfg<KIND, VEC, PART>::NV],
                                           const int (&off1)[StageCfg<KIND, VEC, PART>::NV],
                                           typename VecOf<VEC>::type (&regs)[StageCfg<KIND, VEC, PART>::NV])
{
    typedef typename StageCfg<KIND, VEC, PART>::V V;
#pragma unroll
    for (int j = J0; j < J1; ++j) {
        const int o0 = off0[j], o1 = off1[j];          // values first: a conditional on the array elements themselves
        const unsigned off = (unsigned)(f.tail ? o1 : o0) + f.add;   // would select an address and force the arrays into memory
        regs[j] = *(const __attribute__((address_space(1))) V *)((uintptr_t)f.base + (uint64_t)off * 2u);
    }
}

// move vectors J0 .. J1-1 of the tile fetched for reduction start c0 into LDS; CAREFUL zeroes reduction indices >= c_lim
template <int KIND, int VEC, bool CAREFUL, int PART = 1, int J0 = 0, int J1 = StageCfg<KIND, VEC, PART>::NV>
__device__ __forceinline__ void stage_store(const StageState &s, const typename VecOf<VEC>::type (&regs)[StageCfg<KIND, VEC, PART>::NV],
                                            __bf16 *tile, int c0)
{
    typedef StageCfg<KIND, VEC, PART> C;
    typedef typename C::V V;
    __bf16 *dst = tile + s.row0 * C::PITCH + s.col;
#pragma unroll
    for (int j = J0; j < J1; ++j) {
        if (CAREFUL) {
            const int c = KIND == LD_KC ? c0 + s.col : c0 + s.row0 + j * C::ROW_STEP;
            const uint32_t keep = c < s.c_lim ? 0xffffffffu : 0u;
            *(V *)(dst + j * C::ROW_STEP * C::PITCH) = regs[j] & keep;
        } else {
            *(V *)(dst + j * C::ROW_STEP * C::PITCH) = regs[j];
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

// Reduce-scatter as a sum on read (all ranks on the device; Algorithm 1, backward): the tail block of operand A
// (the k columns behind a.c.split, dg_own in the input-gradient product) is not read from memory but summed
// from what the other ranks sent, dg_own[g] = sum_{j != g} src[j][slot of g on j], src = dG_send [p, p-1, per_slot],
// per_slot = rows * k.  The workgroups of tile column 0 also write the sums to out [p, per_slot] for later kernels.
// src == nullptr: operand A is read as its View says.
struct SumOnRead {
    const __bf16 *src;
    __bf16 *out;
    int64_t per_slot;
    int p, k;
};

// SGD inside the epilogue that finishes a weight gradient (float output with 8-element vectors, whole or cut into
// pieces): the parameters that the gradient belongs to, laid out like the output View's two regions.
// master0 == nullptr: none.
struct SgdInPlace {
    float *master0, *master1;    // fp32 master copies: master -= lr * gradient
    __bf16 *w0, *w1;             // bf16 compute copies: w = bf16(master)
    float lr;
    int keep_grad;               // also store the gradient (the caller wants to see it)
    float *bias_master;          // weight gradients only: the layer's bias [M], its bf16 copy and its finished gradient
    __bf16 *bias_w;              //   (Eq. (bpb): column sums of delta, left by earlier launches); the tiles of the
    const float *bias_grad;      //   first tile column update the rows they cover.  NULL: none
};

struct MfmaParams {
    View a, b, o;        // o: the row index must not decide the region (true for every output here)
    Epilogue ep;
    SumOnRead rs;
    int M, N, K;
    int tiles_m, tiles_n;
    int ksplit;          // > 1: the reduction range is cut into ksplit pieces; their results are added atomically
                         //   (ATOMIC kernels) or by the piece that finishes last (parts)
    int k_per_split;     // multiple of KT
    int total_wg;
    float *parts;        // ksplit > 1 without atomics (float output, 8-element vectors, one group): room for ksplit
    unsigned *arrived;   //   tiles of 128 x 128 floats per output tile, and one word per output tile, zero on entry
                         //   and left zero (see epilogue_pieces_from_lds)
    SgdInPlace sgd;      // what the epilogue that finishes a float output tile does besides storing it
};

// The vectors of a K-contiguous A tile (reduction start c0) that lie in the summed block: replaces what the loader
// fetched for them.  A thread holds NV vectors of the same columns in rows row0 + j * ROW_STEP; the loads of seven
// senders are in flight together (with fewer senders the last one is read again and not added).  Sums in fp32 in
// the order of the senders, one rounding to bf16.
template <int VEC>
__device__ __forceinline__ void fetch_summed(const SumOnRead &rs, int g, int r0, int r_limit, const StageState &s, int c0,
                                             typename VecOf<VEC>::type (&regs)[StageCfg<LD_KC, VEC>::NV], bool write_out)
{
    typedef StageCfg<LD_KC, VEC> C;
    typedef typename C::V V;
    const int c = c0 + s.col;
    if (c < s.c_split || c + VEC > s.c_lim) return;
    const int w = c - s.c_split;
    int64_t row_off[C::NV];
#pragma unroll
    for (int j = 0; j < C::NV; ++j) row_off[j] = (int64_t)min(r0 + s.row0 + j * C::ROW_STEP, r_limit - 1) * rs.k + w;
    float acc[C::NV][VEC];
#pragma unroll
    for (int j = 0; j < C::NV; ++j)
#pragma unroll
        for (int u = 0; u < VEC; ++u) acc[j][u] = 0.f;
    constexpr int AHEAD = 7;                 // the host allows at most 8 ranks: all senders in one batch
    const int senders = rs.p - 1;
    for (int a0 = 0; a0 < senders; a0 += AHEAD) {
        V v[AHEAD][C::NV];
#pragma unroll
        for (int a = 0; a < AHEAD; ++a) {
            const int i = min(a0 + a, senders - 1);            // the i-th sender other than g
            const int from = i < g ? i : i + 1;
            const int slot = g < from ? g : g - 1;
            const __bf16 *base = rs.src + ((int64_t)from * (rs.p - 1) + slot) * rs.per_slot;
#pragma unroll
            for (int j = 0; j < C::NV; ++j) v[a][j] = load_global<V>(base + row_off[j]);
        }
#pragma unroll
        for (int a = 0; a < AHEAD; ++a) {
            const float take = a0 + a < senders ? 1.f : 0.f;
#pragma unroll
            for (int j = 0; j < C::NV; ++j) {
                union { V v; __bf16 e[VEC]; } x;
                x.v = v[a][j];
#pragma unroll
                for (int u = 0; u < VEC; ++u) acc[j][u] = fmaf(take, (float)x.e[u], acc[j][u]);
            }
        }
    }
#pragma unroll
    for (int j = 0; j < C::NV; ++j) {
        union { V v; __bf16 e[VEC]; } x;
#pragma unroll
        for (int u = 0; u < VEC; ++u) x.e[u] = (__bf16)acc[j][u];
        regs[j] = x.v;
        if (write_out) *(V *)(rs.out + (int64_t)g * rs.per_slot + row_off[j]) = x.v;
    }
}

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
                acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(bv[j], av[i], acc[i][j], 0, 0, 0);   // B first: see acc_to_lds
    }
}

// One reduction step with everything interleaved: a quarter (16 of 64 reduction indices) of the
// MFMAs on the current LDS stage, then a quarter of the NEXT tile moved from registers to the other
// LDS stage, then a quarter of the loads of the tile after that into the registers just freed.  In
// this order the LDS writes (128 B/clk) and the global loads (64 B/clk through the vector L1, which
// for a 128 x 128 tile is as many cycles as the MFMAs themselves) run under the MFMAs instead of
// before them.
template <int KA, int KB, int VA, int VB, bool CAREFUL, int Q, int BP>
__device__ __forceinline__ void fused_quarter(f32x16 (&acc)[2][2], const __bf16 *ta, const __bf16 *tb, int wm, int wn, int lane,
                                              const StageState &sa, const int (&a_off0)[StageCfg<KA, VA>::NV],
                                              const int (&a_off1)[StageCfg<KA, VA>::NV],
                                              typename VecOf<VA>::type (&ra)[StageCfg<KA, VA>::NV], __bf16 *na,
                                              const StageState &sb, const int (&b_off0)[StageCfg<KB, VB, BP>::NV],
                                              const int (&b_off1)[StageCfg<KB, VB, BP>::NV],
                                              typename VecOf<VB>::type (&rb)[StageCfg<KB, VB, BP>::NV], __bf16 *nb,
                                              int c_store, int c_fetch)
{
    constexpr int NA = StageCfg<KA, VA>::NV, NB = StageCfg<KB, VB, BP>::NV;
    constexpr int A0 = Q * NA / 4, A1 = (Q + 1) * NA / 4, B0 = Q * NB / 4, B1 = (Q + 1) * NB / 4;   // this quarter's vectors
    bf16x8 av[2], bv[2];
    av[0] = lds_operand<KA>(ta, wm, Q, lane);
    av[1] = lds_operand<KA>(ta, wm + 32, Q, lane);
    bv[0] = lds_operand<KB>(tb, wn, Q, lane);
    bv[1] = lds_operand<KB>(tb, wn + 32, Q, lane);
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
            acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(bv[j], av[i], acc[i][j], 0, 0, 0);   // B first: see acc_to_lds
    stage_store<KA, VA, CAREFUL, 1, A0, A1>(sa, ra, na, c_store);
    stage_store<KB, VB, CAREFUL, BP, B0, B1>(sb, rb, nb, c_store);
    stage_fetch<KA, VA, CAREFUL, 1, A0, A1>(sa, a_off0, a_off1, ra, c_fetch);
    stage_fetch<KB, VB, CAREFUL, BP, B0, B1>(sb, b_off0, b_off1, rb, c_fetch);
}

// One reduction step of the fast path.  Per quarter kk (16 of the 64 reduction indices):
//   - the LDS reads of the NEXT quarter's MFMA operands are issued first (two operand buffers), so
//     their latency runs under this quarter's MFMAs;
//   - the four MFMAs alternate with the other traffic of the quarter, which therefore issues while
//     the matrix pipe is busy: quarters 0..2 move the next tile from registers to the other LDS
//     stage, quarters 1..3 issue the global loads of the tile after that into the registers just
//     freed.
// The workgroup's barrier sits before quarter 3: by then every wavefront has finished reading the
// current stage (its last operands are in registers) and writing the next one, so quarter 3
// already reads the first operands of the next step and no barrier is needed at the step's end.
// On entry fr[0] holds the operands of quarter 0; on exit it holds those of the next step.
template <int KIND_A, int KIND_B>
__device__ __forceinline__ void read_operands(bf16x8 (&f)[4], const __bf16 *ta, const __bf16 *tb, int wm, int wn, int kk, int lane)
{
    f[0] = lds_operand<KIND_A>(ta, wm, kk, lane);
    f[1] = lds_operand<KIND_A>(ta, wm + 32, kk, lane);
    f[2] = lds_operand<KIND_B>(tb, wn, kk, lane);
    f[3] = lds_operand<KIND_B>(tb, wn + 32, kk, lane);
}

constexpr int part_lo(int n, int q) { return n * q / 3; }       // the q-th third of n vectors

// ---- the compression inside the update's reduction loop (one rank's forward) ----------------------------
// g = X C^T shares its A operand with the update: the rows of X that a workgroup stages for its tile are the rows the
// compression needs, over the first part [0, K) of the update's reduction range.  The 128 rows of a tile row and the
// N <= 64 phantom neurons make 4 x ceil(N / 32) blocks of 32 x 32; the workgroup of tile column tn takes block tn:
// it stages the block's 32 rows of C beside its B tile (4 KB per step, one more 16-byte vector per thread), and the
// one wavefront whose A fragment covers the block's rows issues one more MFMA per quarter step with the fragment it
// has read anyway.  No second pass over X, no partial sums between workgroups, and the work rides under a loop that
// the memory side bounds.  Conditions (host): 8-element vectors, regular shapes (fast path only), a tile row has at
// least as many workgroups as blocks, one tile per workgroup (the two-tile loop has no registers left for it).
// Configuration 4's forward launch: 36.1 us, against 37.6 with the compression as a share of rows behind the epilogue
// and 33.9 without any compression.
struct FoldParams {
    const __bf16 *C;     // [N, K] per group
    __bf16 *G;           // [M, N] per group, M = the update's
    int64_t c_g, o_g;    // element offsets per group
    int N, K;
    int ncb;             // blocks per row of blocks = ceil(N / 32)
    int nblocks;         // 4 * ncb; 0: no folding
};

constexpr int E_SLOT_OFF = MT * KC_PITCH;      // a K-contiguous tile leaves the last 1024 elements of its slot unused:
static_assert(TILE_ELEMS - E_SLOT_OFF >= 16 * KT, "room for 16 unpadded rows of the block's C tile behind a K-contiguous tile");

struct FoldState {
    bool on;             // the workgroup has a block (uniform)
    bool owner;          // this wavefront multiplies it (uniform per wavefront)
    bool own_hi;         // ... with the second of its two 32-row A fragments
    int limit;           // reduction indices below it belong to X (uniform)
    const __bf16 *base;  // row 0 of the block's C rows, reduction index 0 (uniform)
    int src_off;         // this thread's 16-byte vector of those rows: element offset from base
    int st_off;          // where that vector goes inside a stage's C tile (element offset)
    int rd_off;          // owner: element offset of the lane's row inside a stage's C tile, and
    int rd_swz;          //        the XOR of its 16-byte slot index
    f32x16 acc;
    bf16x8 fe;
};

// The C tile of a stage: two halves of 16 rows, HALF elements apart (the halves sit behind two different operand tiles
// when two teams share an output tile); rows of 64 elements without padding; the 16-byte slots of row r sit at
// slot ^ ((r >> 1) & 7), which spreads the 16 rows that the lanes of an operand read touch over all banks.
__device__ __forceinline__ bf16x8 fold_read(const FoldState &fs, const __bf16 *tile, int kk, int lane)
{
    const int slot = (2 * kk + (lane >> 5)) ^ fs.rd_swz;
    return *(const bf16x8 *)(tile + fs.rd_off + slot * 8);
}

// FOLD: the step also carries the compression's block: fs; re: the register that holds the next tile's vector of C
// rows (stored, then refilled with the tile's at c_fetch); e_cur, e_nxt: the C tile in the current and in the next
// stage; c_cur, c_next: where this step's and the next step's tiles start in the reduction range.
template <int KA, int KB, int VA, int VB, int BP, bool DRAIN, bool FOLD = false>
__device__ __forceinline__ void fast_step(f32x16 (&acc)[2][2], bf16x8 (&fr)[2][4], const __bf16 *ta, const __bf16 *tb,
                                          int wm, int wn, int lane,
                                          const StageState &sa, const int (&a_off0)[StageCfg<KA, VA>::NV],
                                          const int (&a_off1)[StageCfg<KA, VA>::NV],
                                          typename VecOf<VA>::type (&ra)[StageCfg<KA, VA>::NV], __bf16 *na,
                                          const StageState &sb, const int (&b_off0)[StageCfg<KB, VB, BP>::NV],
                                          const int (&b_off1)[StageCfg<KB, VB, BP>::NV],
                                          typename VecOf<VB>::type (&rb)[StageCfg<KB, VB, BP>::NV], __bf16 *nb, int c_fetch,
                                          bool do_mfma, bool do_store, bool do_fetch,
                                          FoldState &fs, u32x4 &re, const __bf16 *e_cur, __bf16 *e_nxt, int c_cur, int c_next)
{
    constexpr int NA = StageCfg<KA, VA>::NV, NB = StageCfg<KB, VB, BP>::NV;
    // all uniform (per workgroup, or per wavefront for the owner's)
    const bool e_mul = FOLD && fs.owner && (!DRAIN || do_mfma) && c_cur < fs.limit;
    const bool e_next = FOLD && fs.on && (!DRAIN || do_store) && c_next < fs.limit;
    const bool e_fetch = FOLD && fs.on && (!DRAIN || do_fetch) && c_fetch < fs.limit;
    // the block's operand of a quarter is read at the quarter's start and used behind its four MFMAs (one register set)
#define PH_E_READ(kk) do { if (FOLD && e_mul) fs.fe = fold_read(fs, e_cur, kk, lane); } while (0)
    // (a branch, not a select between the two fragments: a select of array elements would move the array to memory)
#define PH_E_MFMA(buf) do { if (FOLD && e_mul) { \
        if (fs.own_hi) fs.acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fs.fe, fr[buf][1], fs.acc, 0, 0, 0); \
        else fs.acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fs.fe, fr[buf][0], fs.acc, 0, 0, 0); } } while (0)
    // a tile that does not exist has no valid address: its step start is replaced by one that does
    const int c_safe = (DRAIN && !do_fetch) ? sa.c_lim - KT : c_fetch;
    const FastStep fa = fast_step_addr<KA, VA>(sa, c_safe), fb = fast_step_addr<KB, VB>(sb, c_safe);
#define PH_MFMA(buf, i, j) do { if (!DRAIN || do_mfma) acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fr[buf][2 + j], fr[buf][i], acc[i][j], 0, 0, 0); } while (0)
#define PH_STORE_A(q) do { if (!DRAIN || do_store) stage_store<KA, VA, false, 1, part_lo(NA, q), part_lo(NA, q + 1)>(sa, ra, na, 0); } while (0)
#define PH_STORE_B(q) do { if (!DRAIN || do_store) stage_store<KB, VB, false, BP, part_lo(NB, q), part_lo(NB, q + 1)>(sb, rb, nb, 0); } while (0)
#define PH_FETCH_A(q) do { if (!DRAIN || do_fetch) fast_fetch<KA, VA, 1, part_lo(NA, q), part_lo(NA, q + 1)>(fa, a_off0, a_off1, ra); } while (0)
#define PH_FETCH_B(q) do { if (!DRAIN || do_fetch) fast_fetch<KB, VB, BP, part_lo(NB, q), part_lo(NB, q + 1)>(fb, b_off0, b_off1, rb); } while (0)
#define PH_PIN __builtin_amdgcn_sched_barrier(0)   /* the compiler's scheduler would regroup the sequence */
    // quarter 0
    PH_PIN; read_operands<KA, KB>(fr[1], ta, tb, wm, wn, 1, lane); PH_E_READ(0); PH_PIN;
    PH_MFMA(0, 0, 0); PH_STORE_A(0); PH_PIN;
    PH_MFMA(0, 0, 1); PH_STORE_B(0); PH_PIN;
    PH_MFMA(0, 1, 0);
    if (FOLD && e_next) *(u32x4 *)(e_nxt + fs.st_off) = re;
    PH_MFMA(0, 1, 1); PH_E_MFMA(0); PH_PIN;
    // quarter 1
    read_operands<KA, KB>(fr[0], ta, tb, wm, wn, 2, lane); PH_E_READ(1); PH_PIN;
    PH_MFMA(1, 0, 0); PH_STORE_A(1); PH_PIN;
    PH_MFMA(1, 0, 1); PH_STORE_B(1); PH_PIN;
    PH_MFMA(1, 1, 0); PH_FETCH_A(0); PH_PIN;
    PH_MFMA(1, 1, 1); PH_FETCH_B(0); PH_E_MFMA(1); PH_PIN;
    // quarter 2
    read_operands<KA, KB>(fr[1], ta, tb, wm, wn, 3, lane); PH_E_READ(2); PH_PIN;
    PH_MFMA(0, 0, 0); PH_STORE_A(2); PH_PIN;
    PH_MFMA(0, 0, 1); PH_STORE_B(2); PH_PIN;
    PH_MFMA(0, 1, 0); PH_FETCH_A(1); PH_PIN;
    PH_MFMA(0, 1, 1); PH_FETCH_B(1); PH_E_MFMA(0); PH_PIN;
    PH_E_READ(3); PH_PIN;          // before the barrier, like every read of the current stage
    __syncthreads();
    // quarter 3
    PH_PIN; read_operands<KA, KB>(fr[0], na, nb, wm, wn, 0, lane); PH_PIN;
    PH_MFMA(1, 0, 0); PH_FETCH_A(2); PH_PIN;
    PH_MFMA(1, 0, 1); PH_FETCH_B(2); PH_PIN;
    PH_MFMA(1, 1, 0);
    if (FOLD && e_fetch) re = load_global<u32x4>(fs.base + (fs.src_off + c_fetch));
    PH_MFMA(1, 1, 1); PH_E_MFMA(1); PH_PIN;
#undef PH_E_READ
#undef PH_E_MFMA
#undef PH_PIN
#undef PH_MFMA
#undef PH_STORE_A
#undef PH_STORE_B
#undef PH_FETCH_A
#undef PH_FETCH_B
}

// ---- epilogue ---------------------------------------------------------------------------
// The MFMA accumulator layout gives a lane one column and scattered rows: stored from registers,
// every store instruction would write two 64-byte pieces of 2-byte elements (measured: 12 us for
// the 8 MB of a 4096 x 1024 bf16 output, a third of the kernel).  Instead the finished fp32 tile
// goes to LDS and all 512 threads walk it row by row, VEC consecutive columns per thread: bias,
// activation (or its derivative) and every global access are then 16-byte vectors on full lines.
constexpr int CT_PITCH = MT + 4;                       // floats per row of an fp32 tile in LDS (132 = 4 mod 64: the 16-byte
                                                       // writes of 16 lanes in 16 different rows fall on 64 different banks)
constexpr int CT_ELEMS = MT * CT_PITCH;                // one tile per team
static_assert((2 * CT_ELEMS + MFMA_THREADS / 64) * 4 <= MFMA_LDS_BYTES, "both teams' fp32 tiles and one float per wavefront fit in the staging space");

// A wavefront's 64 x 64 block of accumulators -> its team's fp32 tile in LDS.
// The MFMAs are issued with the B operand first, i.e. they compute the transpose of each 32 x 32 block:
// a lane then holds, of block (i, j), row (lane & 31) and the columns 8*(e/4) + 4*(lane>>5) + e%4, so
// every group of four accumulators is 16 contiguous bytes of a row-major tile (one ds_write_b128;
// in the untransposed layout the same data would take four 4-byte writes).
__device__ __forceinline__ void acc_to_lds(float *ctile, const f32x16 (&acc)[2][2], int wm, int wn, int lane)
{
    typedef float f32x4 __attribute__((ext_vector_type(4)));
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                f32x4 v = {acc[i][j][4 * q], acc[i][j][4 * q + 1], acc[i][j][4 * q + 2], acc[i][j][4 * q + 3]};
                *(f32x4 *)(ctile + (wm + 32 * i + (lane & 31)) * CT_PITCH + wn + 32 * j + 8 * q + 4 * (lane >> 5)) = v;
            }
}

template <typename T, int VEC> struct PackOf { typedef T type __attribute__((ext_vector_type(VEC))); };

// rows [m0, m0+128) x columns [n0, n0+128) of the output = sum of the two teams' fp32 tiles in LDS, walked by
// all 512 threads; SOLO: the tile at ctile alone, walked by the 256 threads of one team (thread = 0..255)
// EPI: the only mode other than EPI_STORE that the kernel is built for (the first product's; the second
// product of a pair always stores plainly).  Building every mode into every kernel made the epilogue, which
// every workgroup runs exactly once and so fetches cold, long enough to cost each launch about 1 us.
template <int VEC, typename TOut, bool SOLO, int EPI>
__device__ __forceinline__ void epilogue_from_lds(const MfmaParams &P, int g, const float *ctile, int m0, int n0, int thread,
                                                  float *wave_sums)
{
    constexpr int THREADS = SOLO ? 256 : MFMA_THREADS;
    typedef typename PackOf<TOut, VEC>::type OutV;
    typedef typename PackOf<__bf16, VEC>::type BfV;
    typedef typename PackOf<float, VEC>::type FlV;
    TOut *o0 = (TOut *)P.o.p0 + g * P.o.g0, *o1 = (TOut *)P.o.p1 + g * P.o.g1;
    const int skip_o = P.o.skip0 + g * P.o.skip_g;
    const Epilogue &ep = P.ep;
    constexpr int PER_ROW = MT / VEC;                  // vectors per tile row
    constexpr int PASSES = MT * PER_ROW / THREADS;
    static_assert(THREADS % PER_ROW == 0, "a thread keeps its columns from pass to pass");
    float csum[VEC];                                   // this thread's share of the column sums (ep.colsum)
#pragma unroll
    for (int u = 0; u < VEC; ++u) csum[u] = 0.f;
    float sq_sum = 0.f;                                // ... and of the squared output error (ep.mse_target)
    // What the epilogue reads from memory besides the tile is requested before anything else, for all passes at once:
    // read inside the loop, every pass waited a memory latency for it (the float sigma' of a two-tile workgroup's
    // input gradient: 7.2 us of epilogue against 1.0 us with a plain store; the bias: 2 us).
    BfV bias_v;
#pragma unroll
    for (int u = 0; u < VEC; ++u) bias_v[u] = (__bf16)0.f;
    if (EPI == EPI_BIAS_ACT && ep.mode == EPI_BIAS_ACT) {
        const int n = n0 + (thread % PER_ROW) * VEC;   // a thread keeps its columns from pass to pass
        if (n < P.N) bias_v = gload<BfV>((const __bf16 *)ep.bias + g * ep.bias_g + n);
    }
    union AuxU { FlV f; BfV h; unsigned bits; __device__ AuxU() {} };
    constexpr int AUX_PASSES = EPI == EPI_DACT ? PASSES : 1;
    AuxU aux_v[AUX_PASSES];
    if (EPI == EPI_DACT && ep.mode == EPI_DACT && ep.aux) {
        // One straight run of loads per kind of aux, addresses clamped into the tile's valid part instead of skipped:
        // with the choice of kind and the bounds test inside the loop every pass was a basic block of its own and
        // the compiler waited for each pass's load before it issued the next one's (eight memory latencies in a row).
        int64_t at[AUX_PASSES];
#pragma unroll
        for (int i = 0; i < AUX_PASSES; ++i) {
            const int v = thread + i * THREADS;
            const int m = min(m0 + v / PER_ROW, P.M - 1), n = min(n0 + (v % PER_ROW) * VEC, P.N - VEC);
            at[i] = g * ep.aux_g + (int64_t)m * ep.aux_ld + n;
        }
        if (ep.aux_bits) {                             // uniform
#pragma unroll
            for (int i = 0; i < AUX_PASSES; ++i) aux_v[i].bits = gload<uint8_t>((const uint8_t *)ep.aux + (at[i] >> 3));
        } else if (ep.aux_deriv) {
#pragma unroll
            for (int i = 0; i < AUX_PASSES; ++i) aux_v[i].f = gload_nt<FlV>((const float *)ep.aux + at[i]);   // read once
        } else if (ep.aux_f32) {
#pragma unroll
            for (int i = 0; i < AUX_PASSES; ++i) aux_v[i].f = gload<FlV>((const float *)ep.aux + at[i]);
        } else {
#pragma unroll
            for (int i = 0; i < AUX_PASSES; ++i) aux_v[i].h = gload<BfV>((const __bf16 *)ep.aux + at[i]);
        }
    }
    constexpr int EPI_UNROLL = EPI == EPI_DACT ? PASSES : 2;     // EPI_DACT: unrolled, the prefetched vectors stay in registers
#pragma unroll EPI_UNROLL
    for (int i = 0; i < PASSES; ++i) {
        const int v = thread + i * THREADS;
        const int row = v / PER_ROW, col = (v % PER_ROW) * VEC;
        const int m = m0 + row, n = n0 + col;
        if (m >= P.M || n >= P.N) continue;
        float x[VEC];
        {
            const FlV c0 = *(const FlV *)(ctile + row * CT_PITCH + col);
            if constexpr (SOLO) {
#pragma unroll
                for (int u = 0; u < VEC; ++u) x[u] = c0[u];
            } else {
                const FlV c1 = *(const FlV *)(ctile + CT_ELEMS + row * CT_PITCH + col);
#pragma unroll
                for (int u = 0; u < VEC; ++u) x[u] = c0[u] + c1[u];
            }
        }
        const int64_t aux_at = g * ep.aux_g + (int64_t)m * ep.aux_ld + n;
        float deriv[VEC];                              // EPI_BIAS_ACT: sigma'(pre-activation), for the output error
        if (EPI == EPI_BIAS_ACT && ep.mode == EPI_BIAS_ACT) {
#pragma unroll
            for (int u = 0; u < VEC; ++u) x[u] += (float)bias_v[u];
            if (ep.act == ACT_GELU) {                  // uniform
                float pre[VEC];
#pragma unroll
                for (int u = 0; u < VEC; ++u) {
                    pre[u] = x[u];
                    gelu_both(pre[u], x[u], deriv[u]);
                }
                if (ep.aux) {
                    if (ep.aux_deriv) {
                        // written once, read once by the backward pass much later: a streaming store keeps it from
                        // pushing the operand panels that other workgroups still share out of L2
                        FlV a;
#pragma unroll
                        for (int u = 0; u < VEC; ++u) a[u] = deriv[u];
                        gstore_nt<FlV>((float *)ep.aux + aux_at, a);
                    } else if (ep.aux_f32) {
                        FlV a;
#pragma unroll
                        for (int u = 0; u < VEC; ++u) a[u] = pre[u];
                        gstore<FlV>((float *)ep.aux + aux_at, a);
                    } else {
                        BfV a;
#pragma unroll
                        for (int u = 0; u < VEC; ++u) a[u] = (__bf16)pre[u];
                        gstore<BfV>((__bf16 *)ep.aux + aux_at, a);
                    }
                }
            } else {
                if (ep.aux && !ep.aux_bits) {
                    if (ep.aux_deriv) {
                        FlV a;
#pragma unroll
                        for (int u = 0; u < VEC; ++u) a[u] = act_deriv(ep.act, x[u]);
                        gstore<FlV>((float *)ep.aux + aux_at, a);
                    } else if (ep.aux_f32) {
                        FlV a;
#pragma unroll
                        for (int u = 0; u < VEC; ++u) a[u] = x[u];
                        gstore<FlV>((float *)ep.aux + aux_at, a);
                    } else {
                        BfV a;
#pragma unroll
                        for (int u = 0; u < VEC; ++u) a[u] = (__bf16)x[u];
                        gstore<BfV>((__bf16 *)ep.aux + aux_at, a);
                    }
                }
#pragma unroll
                for (int u = 0; u < VEC; ++u) {
                    deriv[u] = act_deriv(ep.act, x[u]);
                    x[u] = act_apply(ep.act, x[u]);
                }
            }
        } else if (EPI == EPI_DACT && ep.mode == EPI_DACT && ep.aux) {      // no aux: sigma' = 1, column sums only
            const AuxU &av = aux_v[EPI == EPI_DACT ? i : 0];
            if (ep.aux_bits) {                         // one bit per element: ReLU' of the stored output
                if constexpr (VEC == 8) {
#pragma unroll
                    for (int u = 0; u < VEC; ++u) x[u] = (av.bits >> u) & 1u ? x[u] : 0.f;
                }
            } else if (ep.aux_deriv) {                 // sigma' itself, float
#pragma unroll
                for (int u = 0; u < VEC; ++u) x[u] *= av.f[u];
            } else if (ep.aux_f32) {
#pragma unroll
                for (int u = 0; u < VEC; ++u) x[u] *= act_deriv(ep.act, av.f[u]);
            } else {                                   // the pre-activation (or ReLU output) in bf16
#pragma unroll
                for (int u = 0; u < VEC; ++u) x[u] *= act_deriv(ep.act, (float)av.h[u]);
            }
        }
        const Loc ln = locate(P.o.c, n, skip_o);
        const int region = ln.region > 0 ? 1 : 0;
        TOut *dst = (region ? o1 + ln.off1 : o0 + ln.off0) + (int64_t)m * (region ? P.o.r.mult1 : P.o.r.mult0);
        OutV o;
#pragma unroll
        for (int u = 0; u < VEC; ++u) o[u] = from_f32<TOut>(x[u]);
        if constexpr (EPI == EPI_STORE && sizeof(TOut) == 4 && VEC == 8) {
            if (P.sgd.master0) {                       // uniform: Section VI's plain SGD on the finished gradient
                const int64_t at = dst - (region ? o1 : o0);
                float *master = (region ? P.sgd.master1 : P.sgd.master0) + g * (region ? P.o.g1 : P.o.g0) + at;
                __bf16 *w = (region ? P.sgd.w1 : P.sgd.w0) + g * (region ? P.o.g1 : P.o.g0) + at;
                const FlV before = gload<FlV>(master);     // (requested ahead of the loop like sigma', the launch got 4 % slower)
                FlV after;
                BfV rounded;
#pragma unroll
                for (int u = 0; u < VEC; ++u) {
                    after[u] = before[u] - P.sgd.lr * x[u];
                    rounded[u] = (__bf16)after[u];
                }
                // (the master is next read a step later, by this epilogue; the bf16 copy by the next forward pass, which
                // found it in the last-level cache before a streaming store put it out of there: 1.8 us per forward launch)
                gstore_nt<FlV>(master, after);
                gstore<BfV>(w, rounded);
                if (!P.sgd.keep_grad) continue;
            }
        }
        // (outputs are written once and read by a later launch at the earliest: a streaming store leaves less for the
        // write-back at the end of the kernel; 0.4 % of configuration 4's step, 2-4 % of the forward-only and small ones)
        gstore_nt<OutV>(dst, o);
        if constexpr (EPI == EPI_BIAS_ACT && VEC == 8) {
            if (ep.mode == EPI_BIAS_ACT && ep.aux && ep.aux_bits) {     // uniform
                unsigned bits = 0;
#pragma unroll
                for (int u = 0; u < VEC; ++u) bits |= ((float)o[u] > 0.f ? 1u : 0u) << u;
                gstore<uint8_t>((uint8_t *)ep.aux + (aux_at >> 3), (uint8_t)bits);
            }
        }
        if (EPI == EPI_BIAS_ACT && sizeof(TOut) == 2 && ep.mode == EPI_BIAS_ACT && ep.mse_target) {      // uniform
            // the MSE output error of Eq. (deltaL) from the output as stored, rounded once
            const BfV t = gload<BfV>((const __bf16 *)ep.mse_target + aux_at);
            BfV dl;
#pragma unroll
            for (int u = 0; u < VEC; ++u) {
                const float diff = (float)o[u] - (float)t[u];
                sq_sum += diff * diff;
                float e = diff * ep.mse_inv_b;
                if (ep.act != ACT_IDENTITY) e *= deriv[u];
                dl[u] = (__bf16)e;
                csum[u] += (float)dl[u];
            }
            gstore<BfV>((__bf16 *)ep.mse_delta + aux_at, dl);
        } else {
#pragma unroll
            for (int u = 0; u < VEC; ++u) csum[u] += (float)o[u];
        }
    }
    if constexpr (EPI == EPI_STORE && sizeof(TOut) == 4 && VEC == 8) {
        if (P.sgd.bias_master && n0 == 0 && thread < MT && m0 + thread < P.M) {
            const int64_t at = g * (int64_t)P.M + m0 + thread;
            const float nb = gload<float>(P.sgd.bias_master + at) - P.sgd.lr * gload<float>(P.sgd.bias_grad + at);
            gstore<float>(P.sgd.bias_master + at, nb);
            gstore<__bf16>(P.sgd.bias_w + at, (__bf16)nb);
        }
    }
    if (EPI == EPI_BIAS_ACT && sizeof(TOut) == 2 && ep.mode == EPI_BIAS_ACT && ep.mse_target) {          // uniform
        // the tile's share of sum (y - t)^2: wavefront sums, then one thread adds those of the tile's wavefronts
        // (wave_sums lies behind the fp32 tiles; nothing else uses it)
#pragma unroll
        for (int off = 32; off > 0; off >>= 1) sq_sum += __shfl_down(sq_sum, off);
        const int wave_in_wg = (int)(threadIdx.x >> 6);
        if ((threadIdx.x & 63) == 0) wave_sums[wave_in_wg] = sq_sum;
        __syncthreads();
        if (thread == 0 && m0 < P.M) {
            constexpr int WAVES = THREADS / 64;
            const int first = SOLO ? (int)(threadIdx.x >> 6) : 0;
            float total = 0.f;
#pragma unroll
            for (int w = 0; w < WAVES; ++w) total += wave_sums[first + w];
            const int tiles_m = (P.M + MT - 1) / MT, tiles_n = (P.N + MT - 1) / MT;
            ep.mse_partial[(g * tiles_m + m0 / MT) * tiles_n + n0 / MT] = total;
        }
    }
    if (EPI != EPI_STORE && ep.colsum) {               // uniform
        // threads tid, tid + PER_ROW, ... hold partial sums of the same VEC columns: add them up through
        // LDS (over the fp32 tiles, once every thread has read its share), one atomic per column
        constexpr int SHARERS = THREADS / PER_ROW;
        float *red = const_cast<float *>(ctile);       // SOLO: each team reduces over its own tile
        __syncthreads();
#pragma unroll
        for (int u = 0; u < VEC; ++u) red[(thread / PER_ROW) * MT + (thread % PER_ROW) * VEC + u] = csum[u];
        __syncthreads();
        if (thread < MT && n0 + thread < P.N) {
            float t = 0.f;
#pragma unroll 8
            for (int r = 0; r < SHARERS; ++r) t += red[r * MT + thread];
            unsafeAtomicAdd(ep.colsum + g * ep.colsum_g + n0 + thread, t);
        }
    }
}

// Split reductions: the sum of the two teams' fp32 tiles is ADDED to a float output, element by element
// (plain store semantics only: no bias, activation or column sums).  Device-wide float atomics that
// fall into one 64-byte line are served together, so the 16 lanes that share a tile row take 16
// consecutive columns per instruction (thread: row t / 16 of each group of 32 rows, columns
// t % 16 + 16 u), four full lines per wavefront instruction; eight consecutive columns per lane touch 32
// half-used lines per instruction (measured on a 1024 x 1984 x 4096 product cut into 390 partial tiles:
// 186 us against 47 us for the whole launch).  What remains is about one add per clock and memory
// channel, 15-20 us for those 6.4 M adds, which is why a split reduction is a last resort.
__device__ __forceinline__ void epilogue_atomic_from_lds(const MfmaParams &P, int g, const float *ctile, int m0, int n0, int thread)
{
    constexpr int LANES = 16;                          // lanes per tile row
    constexpr int COLS = MT / LANES;                   // columns per thread
    constexpr int ROWS_PER_PASS = MFMA_THREADS / LANES;
    float *o0 = (float *)P.o.p0 + g * P.o.g0, *o1 = (float *)P.o.p1 + g * P.o.g1;
    const int skip_o = P.o.skip0 + g * P.o.skip_g;
    const int cl = thread % LANES, r0 = thread / LANES;
    // a thread keeps its columns from pass to pass: their places in the output, once
    int64_t col_off[COLS];
    bool col_tail[COLS];
#pragma unroll
    for (int u = 0; u < COLS; ++u) {
        const int n = min(n0 + cl + LANES * u, P.N - 1);
        const Loc ln = locate(P.o.c, n, skip_o);
        col_tail[u] = ln.region > 0;
        col_off[u] = col_tail[u] ? ln.off1 : ln.off0;
    }
#pragma unroll 2
    for (int i = 0; i < MT / ROWS_PER_PASS; ++i) {
        const int row = r0 + i * ROWS_PER_PASS;
        const int m = m0 + row;
        if (m >= P.M) continue;
#pragma unroll
        for (int u = 0; u < COLS; ++u) {
            const int col = cl + LANES * u;
            if (n0 + col >= P.N) continue;
            const float x = ctile[row * CT_PITCH + col] + ctile[CT_ELEMS + row * CT_PITCH + col];
            float *dst = (col_tail[u] ? o1 + (int64_t)m * P.o.r.mult1 : o0 + (int64_t)m * P.o.r.mult0) + col_off[u];
            unsafeAtomicAdd(dst, x);
        }
    }
}

// The epilogue of one piece of a reduction that is cut into ksplit pieces without atomics (float output, plain store
// semantics, 8 columns per thread, all 512 threads).  Every piece writes its 128 x 128 result to its own slot of
// P.parts and then counts itself in P.arrived[tile]; the piece that finds all others counted adds the slots up in the
// order of the pieces (its own from registers), writes the output and leaves the word zero for the next launch.  The
// sum does not depend on which piece comes last, and no workgroup ever waits for another.
// The pieces may run on different XCDs, whose L2 caches do not see each other's lines.  What goes from one to the
// other therefore uses device-scope atomic stores and loads (8 bytes each; the cache policy writes them through to
// memory and reads them from there), as the counter does, so no cache has to be written back or invalidated as a whole:
// with such fences, one per wavefront, the launch took 130 us against 44 us for the uncut product.  Within a slot,
// thread t holds the 8-byte words t, t + 512, ...: every store and load instruction covers 4 KB without gaps.
__device__ __forceinline__ void epilogue_pieces_from_lds(const MfmaParams &P, int tile, int ks, const float *ctile, unsigned *lds_word,
                                                         int m0, int n0, int thread)
{
    typedef unsigned long long u64;
    typedef float f32x4 __attribute__((ext_vector_type(4)));
    constexpr int VEC = 8, PER_ROW = MT / VEC, PASSES = MT * PER_ROW / MFMA_THREADS, WORDS = VEC / 2;
    constexpr int ROWS_PER_PASS = MFMA_THREADS / PER_ROW;
    constexpr int64_t SLOT = MT * MT / 2;              // 8-byte words per slot
    constexpr int GROUP = 2;                           // other pieces whose loads are in flight together
    union Two { u64 w; float f[2]; __device__ Two() {} };
    // passes whose rows all lie below the output's last row (the compressor gradient has k <= 64 rows) move nothing
    const int passes = min(PASSES, (P.M - m0 + ROWS_PER_PASS - 1) / ROWS_PER_PASS);      // uniform
    float x[PASSES][VEC];
#pragma unroll
    for (int i = 0; i < PASSES; ++i) {
        const int v = thread + i * MFMA_THREADS;
        const int row = v / PER_ROW, col = (v % PER_ROW) * VEC;
#pragma unroll
        for (int h = 0; h < 2; ++h) {
            const f32x4 c0 = *(const f32x4 *)(ctile + row * CT_PITCH + col + 4 * h);
            const f32x4 c1 = *(const f32x4 *)(ctile + CT_ELEMS + row * CT_PITCH + col + 4 * h);
#pragma unroll
            for (int u = 0; u < 4; ++u) x[i][4 * h + u] = c0[u] + c1[u];
        }
    }
    u64 *slots = (u64 *)P.parts + (int64_t)tile * P.ksplit * SLOT;
    u64 *mine = slots + ks * SLOT + thread;
#pragma unroll
    for (int i = 0; i < PASSES; ++i) {
        if (i >= passes) break;
#pragma unroll
        for (int c = 0; c < WORDS; ++c) {
            Two t;
            t.f[0] = x[i][2 * c]; t.f[1] = x[i][2 * c + 1];
            __hip_atomic_store(mine + (i * WORDS + c) * MFMA_THREADS, t.w, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
    }
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");   // written through before this piece counts itself
    __syncthreads();
    if (thread == 0) *lds_word = __hip_atomic_fetch_add(P.arrived + tile, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    __syncthreads();
    if (*lds_word + 1 != (unsigned)P.ksplit) return;   // uniform: another piece will finish the tile
    float t[PASSES][VEC];
#pragma unroll
    for (int i = 0; i < PASSES; ++i)
#pragma unroll
        for (int u = 0; u < VEC; ++u) t[i][u] = 0.f;
    for (int j0 = 0; j0 < P.ksplit; j0 += GROUP) {     // uniform
        Two got[GROUP][PASSES][WORDS];
#pragma unroll
        for (int jj = 0; jj < GROUP; ++jj) {
            const int j = j0 + jj;
            if (j >= P.ksplit || j == ks) continue;
            const u64 *theirs = slots + j * SLOT + thread;
#pragma unroll
            for (int i = 0; i < PASSES; ++i) {
                if (i >= passes) break;
#pragma unroll
                for (int c = 0; c < WORDS; ++c)
                    got[jj][i][c].w = __hip_atomic_load(theirs + (i * WORDS + c) * MFMA_THREADS, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            }
        }
#pragma unroll
        for (int jj = 0; jj < GROUP; ++jj) {
            const int j = j0 + jj;
            if (j >= P.ksplit) break;
#pragma unroll
            for (int i = 0; i < PASSES; ++i) {
                if (i >= passes) break;
#pragma unroll
                for (int c = 0; c < WORDS; ++c) {
                    t[i][2 * c] += j == ks ? x[i][2 * c] : got[jj][i][c].f[0];
                    t[i][2 * c + 1] += j == ks ? x[i][2 * c + 1] : got[jj][i][c].f[1];
                }
            }
        }
    }
    float *o0 = (float *)P.o.p0, *o1 = (float *)P.o.p1;
#pragma unroll
    for (int i = 0; i < PASSES; ++i) {
        const int v = thread + i * MFMA_THREADS;
        const int m = m0 + v / PER_ROW, n = n0 + (v % PER_ROW) * VEC;
        if (m >= P.M || n >= P.N) continue;
        const Loc ln = locate(P.o.c, n, P.o.skip0);
        const int region = ln.region > 0 ? 1 : 0;
        const int64_t at = (region ? ln.off1 : ln.off0) + (int64_t)m * (region ? P.o.r.mult1 : P.o.r.mult0);
        float *dst = (region ? o1 : o0) + at;
        if (P.sgd.master0) {                           // uniform: Section VI's plain SGD on the finished gradient
            float *master = (region ? P.sgd.master1 : P.sgd.master0) + at;
            __bf16 *w = (region ? P.sgd.w1 : P.sgd.w0) + at;
            const f32x4 m_lo = gload<f32x4>(master), m_hi = gload<f32x4>(master + 4);
            float nm[VEC];
            bf16x8 nw;
#pragma unroll
            for (int u = 0; u < VEC; ++u) {
                nm[u] = (u < 4 ? m_lo[u] : m_hi[u - 4]) - P.sgd.lr * t[i][u];
                nw[u] = (__bf16)nm[u];
            }
            gstore_nt<f32x4>(master, f32x4{nm[0], nm[1], nm[2], nm[3]});
            gstore_nt<f32x4>(master + 4, f32x4{nm[4], nm[5], nm[6], nm[7]});
            gstore<bf16x8>(w, nw);
            if (!P.sgd.keep_grad) continue;
        }
        gstore_nt<f32x4>(dst, f32x4{t[i][0], t[i][1], t[i][2], t[i][3]});
        gstore_nt<f32x4>(dst + 4, f32x4{t[i][4], t[i][5], t[i][6], t[i][7]});
    }
    if (thread == 0) __hip_atomic_store(P.arrived + tile, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

#ifdef PHANTOM_TIMELINE   // cycle stamps for the development micro-benchmark, never built into the library
// per workgroup 16 words at P.rs.out: slots 0..7 the core clock, 8..15 the 100 MHz wall clock at the same points
#define PH_PHASE(slot) do { __builtin_amdgcn_sched_barrier(0); if (threadIdx.x == 0 && P.rs.out) { \
        ((long long *)P.rs.out)[blockIdx.x * 16 + (slot)] = clock64(); ((long long *)P.rs.out)[blockIdx.x * 16 + 8 + (slot)] = wall_clock64(); } \
        __builtin_amdgcn_sched_barrier(0); } while (0)
#else
#define PH_PHASE(slot) do { } while (0)
#endif

// 512 threads = two teams of 4 wavefronts.  Both teams work on the SAME 128 x 128 tile of C; team q
// takes the reduction steps q, q+2, q+4, ... with its own pair of LDS stages, so every SIMD holds two
// wavefronts whose loads, LDS traffic and MFMAs interleave, without reading any operand twice.  At
// the end each team writes its partial fp32 tile to LDS and the epilogue adds the two.
// One launch may carry two independent products of the same operand layout and output type (the
// layer update with the compression, the error compression with the input gradient, the weight
// gradients with the compressor gradient): their workgroups run side by side instead of one thin
// launch waiting for the other.
struct MfmaBatch {
    MfmaParams p[2];
    int count;
    int total_wg;
    int first_wg;        // = p[0].total_wg
};


// The parameter block of one product, read from the kernel-argument segment at a byte offset that the compiler
// cannot see through.  With several blocks as ordinary arguments (or a word-by-word selection between two of
// them) it moves the loads of all of them to the top of the kernel and, out of scalar registers, spills each one
// before loading the next: a chain of load-wait-spill rounds in front of the first product (four blocks: some
// fifty rounds, 3 us; two blocks: 1.7 us).  This way a block is read where the product starts, with loads that
// do not wait for each other.  The batch structure is the kernel's only argument, so it starts at offset 0.
__device__ __forceinline__ MfmaParams params_at(size_t offset)
{
    constexpr int WORDS = sizeof(MfmaParams) / 4;
    union Words { MfmaParams p; uint32_t w[WORDS]; __device__ Words() {} };
    Words out;
#if defined(__HIP_DEVICE_COMPILE__)
    asm volatile("" : "+s"(offset) :: "memory");
    typedef const uint32_t __attribute__((address_space(4))) *ArgWords;
    const ArgWords in = (ArgWords)((const char __attribute__((address_space(4))) *)__builtin_amdgcn_kernarg_segment_ptr() + offset);
#pragma unroll
    for (int i = 0; i < WORDS; ++i) out.w[i] = in[i];
#endif
    return out.p;
}

// DUAL: the two teams take two tiles that lie one above the other (rows m0 .. m0+127 and m0+128 .. m0+255)
// instead of alternate reduction steps of one tile.  They share the B tile (each team stages half of its
// rows), so per FLOP a quarter less goes through the vector-memory return path and into LDS, which is
// what bounds the loop; the price is half as many workgroups, so this is for launches with more tiles
// than compute units (the host decides).  Each team finishes its own tile: no sum in the epilogue.
// XCD-aware id: hardware deals workgroup ids round-robin over 8 XCDs; `first` (a multiple of 8) is the id of the
// first of `count` consecutive workgroups that share a list of tiles.  Workgroups of one XCD get neighbouring tiles.
__device__ __forceinline__ int xcd_order(int id, int first, int count)
{
    const int i = id - first, per = count >> 3;
    return i < per * 8 ? (i & 7) * per + (i >> 3) : i;
}

// One workgroup's work: workgroup number wg (of P.total_wg, in tile order) of the product P.
// FOLD (the forward layout with 8-element vectors, regular shapes only): the workgroup also computes its block of
// the compression F (FoldParams).
template <int KA, int KB, int VA, int VB, typename TOut, bool ATOMIC, bool DUAL, int EPI, bool FOLD = false>
__device__ __forceinline__ void mfma_workgroup(const MfmaParams &P, int wg, const FoldParams *Fp = nullptr)
{
    static_assert(!FOLD || (KA == LD_KC && KB == LD_KC && VA == 8 && !ATOMIC), "the compression rides with the forward product only");
    extern __shared__ __attribute__((aligned(16))) unsigned char smem_raw[];
    static_assert(!(DUAL && ATOMIC), "a split reduction keeps the two-teams-per-tile form");
    static_assert(!ATOMIC || EPI == EPI_STORE, "partial sums are added as they are");
    constexpr int BP = DUAL ? 2 : 1;                   // share of the B tile one team stages
    PH_PHASE(0);
    const int tiles = P.tiles_m * P.tiles_n;           // DUAL: tiles_m counts pairs of tile rows
    const int g = wg / (tiles * P.ksplit);
    int rem = wg - g * tiles * P.ksplit;
    const int ks = rem / tiles;
    rem -= ks * tiles;
    // tiles are walked in bands of RASTER_M tile rows, down the band first: the workgroups that run
    // together on one XCD then cover a near-square patch of C and share both operand panels in L2
    constexpr int RASTER_M = DUAL ? 4 : 8;
    const int band = rem / (RASTER_M * P.tiles_n);
    const int in_band = rem - band * (RASTER_M * P.tiles_n);
    const int band_rows = min(P.tiles_m - band * RASTER_M, RASTER_M);
    const int tn = in_band / band_rows;
    const int tm = band * RASTER_M + (in_band - tn * band_rows);
    const int team = threadIdx.x >> 8;
    const int team_u = __builtin_amdgcn_readfirstlane(team);
    const int m0 = DUAL ? (tm * 2 + team_u) * MT : tm * MT, n0 = tn * MT;
    const int k_begin = ks * P.k_per_split;
    const int k_end = min(P.K, k_begin + P.k_per_split);
    PH_PHASE(6);

    const int tid = threadIdx.x & 255, lane = tid & 63, wave = tid >> 6;
    const int wm = (wave >> 1) * 64, wn = (wave & 1) * 64;

    typedef StageCfg<KA, VA> SA;
    typedef StageCfg<KB, VB, BP> SB;
    int a_off0[SA::NV], a_off1[SA::NV], b_off0[SB::NV], b_off1[SB::NV];
    // a DUAL team whose tile lies below the last row still stages its half of B and keeps the barriers:
    // its loaders read the last valid row, its epilogue writes nothing
    const StageState sa = stage_init<KA, VA>(P.a, g, min(m0, (P.M - 1) / MT * MT), P.M, k_end, tid, a_off0, a_off1);
    const StageState sb = stage_init<KB, VB, BP>(P.b, g, n0, P.N, k_end, tid, b_off0, b_off1,
                                                 DUAL ? team_u * (SB::ROWS / 2) : 0);
    PH_PHASE(7);
    typename SA::V ra0[SA::NV], ra1[SA::NV];
    typename SB::V rb0[SB::NV], rb1[SB::NV];
    // the compression's block of this workgroup: block tn of its tile row (block = 32 rows x 32 phantom neurons)
    FoldState fs;
    u32x4 re0 = {0, 0, 0, 0}, re1 = {0, 0, 0, 0};
    int e_rb = 0, e_cb = 0;
    fs.on = false; fs.owner = false;
    // the two halves (16 rows each) of a stage's C tile lie this many elements apart
    constexpr int E_HALF = DUAL ? 16 * KT : TILE_ELEMS;
    if constexpr (FOLD) {
        const FoldParams &F = *Fp;
        fs.on = tn < F.nblocks;
        e_rb = tn / F.ncb; e_cb = tn - e_rb * F.ncb;
        fs.owner = fs.on && __builtin_amdgcn_readfirstlane(wave) == (e_rb >> 1) * 2;   // the wavefront with wm = 64 (rb / 2), wn = 0
        fs.own_hi = e_rb & 1;
        fs.limit = F.K;
        const int erow = tid >> 3, eslot = tid & 7;              // 256 threads of a team: 32 rows x 8 vectors
        fs.base = F.C + g * F.c_g + (int64_t)(e_cb * 32) * F.K;
        fs.src_off = min(erow, F.N - 1 - e_cb * 32) * F.K + eslot * 8;
        fs.st_off = (erow >> 4) * E_HALF + (erow & 15) * KT + ((eslot ^ ((erow >> 1) & 7)) * 8);
        const int rrow = lane & 31;
        fs.rd_off = (rrow >> 4) * E_HALF + (rrow & 15) * KT;
        fs.rd_swz = (rrow >> 1) & 7;
#pragma unroll
        for (int e = 0; e < 16; ++e) fs.acc[e] = 0.f;
    }
#define PH_FETCH(set, c0) do { stage_fetch<KA, VA, true>(sa, a_off0, a_off1, ra##set, (c0)); \
                               stage_fetch<KB, VB, true, BP>(sb, b_off0, b_off1, rb##set, (c0)); } while (0)
#define PH_STORE(set, stage, c0) do { stage_store<KA, VA, true>(sa, ra##set, s##stage##a, (c0)); \
                                      stage_store<KB, VB, true, BP>(sb, rb##set, s##stage##b, (c0)); } while (0)

    f32x16 acc[2][2];
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;
    PH_PHASE(1);

    // LDS: two stages per operand tile.  Two teams on one tile: each team has its own A and B stages
    // (8 tiles).  DUAL: own A stages, the B stages are common (6 tiles).
    __bf16 *smem = (__bf16 *)smem_raw;
    __bf16 *s0a, *s0b, *s1a, *s1b;
    if (DUAL) {
        s0a = smem + team * 2 * TILE_ELEMS; s1a = s0a + TILE_ELEMS;
        s0b = smem + 4 * TILE_ELEMS; s1b = s0b + TILE_ELEMS;
    } else {
        s0a = smem + team * 4 * TILE_ELEMS; s0b = s0a + TILE_ELEMS; s1a = s0a + 2 * TILE_ELEMS; s1b = s0a + 3 * TILE_ELEMS;
    }
    // the C tile of the compression's block, per stage.  Two teams on one tile: its halves behind the team's own A and
    // B tiles; DUAL (B stages shared by the teams): in the space behind the six operand tiles.
    __bf16 *e0 = nullptr, *e1 = nullptr;
    if constexpr (FOLD) {
        if (DUAL) { e0 = smem + 6 * TILE_ELEMS + team * 4 * 16 * KT; e1 = e0 + 2 * 16 * KT; }
        else { e0 = s0a + E_SLOT_OFF; e1 = s1a + E_SLOT_OFF; }
    }
    // The reduction range is cut into tiles of KT.  Two teams on one tile: team q takes the tiles q, q+2, ...;
    // DUAL: every team takes every tile.  Both teams pass the same number of barriers (`steps`).
    const int all_steps = (k_end - k_begin + KT - 1) / KT;
    const int steps = DUAL ? all_steps : (all_steps + 1) >> 1;
    const int my_steps = DUAL ? all_steps : (all_steps - team_u + 1) >> 1;      // tiles this team really has
    constexpr int KS = DUAL ? KT : 2 * KT;
    const int kfirst = DUAL ? k_begin : k_begin + team_u * KT;     // start of this team's first tile
    // Regular shapes walk their tiles from the LAST one down: the only tile that can be ragged (the end of the
    // reduction range) then comes first and is staged by the careful prologue; every later tile is a full
    // one and every step takes the fast path.  Other shapes walk upwards through the general loop.
    const bool regular = sa.regular && sb.regular &&
                         (!DUAL || tile_is_regular<KA>(P.a, min((tm * 2 + (1 - team_u)) * MT, (P.M - 1) / MT * MT)));
    int t = 0;
    if (regular) {                                                  // uniform (in DUAL for both teams alike)
        const int c_last = kfirst + (my_steps - 1) * KS;            // start of the tile processed first
        auto c_of = [c_last](int i) { return c_last - i * KS; };    // tile processed in step i (i < my_steps)
        // only that first tile needs the careful loader (clamped indices, zeroed tail: some 30 vector instructions
        // per fetch and operand); a full one and the two tiles behind it take the loop's own addressing
#define PH_FETCH_FAST(set, c0) do { \
        const FastStep fa_ = fast_step_addr<KA, VA>(sa, (c0)), fb_ = fast_step_addr<KB, VB>(sb, (c0)); \
        fast_fetch<KA, VA, 1, 0, SA::NV>(fa_, a_off0, a_off1, ra##set); \
        fast_fetch<KB, VB, BP, 0, SB::NV>(fb_, b_off0, b_off1, rb##set); } while (0)
        const bool ragged_first = my_steps > 0 && c_of(0) + KT > k_end;     // the same for the whole team
        if (ragged_first) PH_FETCH(0, c_of(0));
        else if (my_steps > 0) PH_FETCH_FAST(0, c_of(0));
        if (my_steps > 1) PH_FETCH_FAST(1, c_of(1));
        if constexpr (KA == LD_KC && KB == LD_KM && VA == 8) {    // the input gradient's layout, 16-byte vectors
            // the summed block lies in the tile processed first (the host sees to it: it starts at a tile boundary
            // and is at most one tile long)
            if (P.rs.src && my_steps > 0 && c_of(0) + KT > sa.c_split)
                fetch_summed<VA>(P.rs, g, min(m0, (P.M - 1) / MT * MT), P.M, sa, c_of(0), ra0, tn == 0);
        }
        if (ragged_first) {
            PH_STORE(0, 0, c_of(0));
        } else if (my_steps > 0) {
            stage_store<KA, VA, false>(sa, ra0, s0a, 0);
            stage_store<KB, VB, false, BP>(sb, rb0, s0b, 0);
        }
        if (my_steps > 2) PH_FETCH_FAST(0, c_of(2));
#undef PH_FETCH_FAST
        if constexpr (FOLD) {
            // the C tile of the block for the first three tiles, as far as they lie in X's part of the reduction range
            if (fs.on) {                                             // uniform
                if (my_steps > 1 && c_of(1) < fs.limit) re1 = load_global<u32x4>(fs.base + (fs.src_off + c_of(1)));
                if (my_steps > 0 && c_of(0) < fs.limit)
                    *(u32x4 *)(e0 + fs.st_off) = load_global<u32x4>(fs.base + (fs.src_off + c_of(0)));
                if (my_steps > 2 && c_of(2) < fs.limit) re0 = load_global<u32x4>(fs.base + (fs.src_off + c_of(2)));
            }
        }
        __syncthreads();
        PH_PHASE(2);
        // step i multiplies LDS stage i%2; on entry tile i+1 sits in register set (i+1)%2 and is moved to the other
        // stage (whose readers finished before the barrier inside step i-1), tile i+2 in the other set
        bf16x8 fr[2][4];
        read_operands<KA, KB>(fr[0], s0a, s0b, wm, wn, 0, lane);
#define PH_ES(cur, nxt, i) e##cur, e##nxt, c_of(i), c_of((i) + 1)
        for (; t + 1 < steps && t + 4 < my_steps; t += 2) {          // everything these two steps touch exists
            fast_step<KA, KB, VA, VB, BP, false, FOLD>(acc, fr, s0a, s0b, wm, wn, lane, sa, a_off0, a_off1, ra1, s1a, sb, b_off0, b_off1,
                                                       rb1, s1b, c_of(t + 3), true, true, true, fs, re1, PH_ES(0, 1, t));
            fast_step<KA, KB, VA, VB, BP, false, FOLD>(acc, fr, s1a, s1b, wm, wn, lane, sa, a_off0, a_off1, ra0, s0a, sb, b_off0, b_off1,
                                                       rb0, s0b, c_of(t + 4), true, true, true, fs, re0, PH_ES(1, 0, t + 1));
        }
        for (; t + 1 < steps; t += 2) {                              // the last steps: the pipeline runs empty
            fast_step<KA, KB, VA, VB, BP, true, FOLD>(acc, fr, s0a, s0b, wm, wn, lane, sa, a_off0, a_off1, ra1, s1a, sb, b_off0, b_off1,
                                                      rb1, s1b, c_of(t + 3), t < my_steps, t + 1 < my_steps, t + 3 < my_steps, fs, re1,
                                                      PH_ES(0, 1, t));
            fast_step<KA, KB, VA, VB, BP, true, FOLD>(acc, fr, s1a, s1b, wm, wn, lane, sa, a_off0, a_off1, ra0, s0a, sb, b_off0, b_off1,
                                                      rb0, s0b, c_of(t + 4), t + 1 < my_steps, t + 2 < my_steps, t + 4 < my_steps, fs, re0,
                                                      PH_ES(1, 0, t + 1));
        }
        if (t < steps)
            fast_step<KA, KB, VA, VB, BP, true, FOLD>(acc, fr, s0a, s0b, wm, wn, lane, sa, a_off0, a_off1, ra1, s1a, sb, b_off0, b_off1,
                                                      rb1, s1b, 0, t < my_steps, false, false, fs, re1, PH_ES(0, 1, t));
#undef PH_ES
    } else {
        // prologue: tile 0 into LDS stage 0; tiles 1 and 2 on their way in register sets 1 and 0.  A tile past the
        // end of the range (the shorter team's last step) is stored as zeros.
        PH_FETCH(0, kfirst);
        PH_FETCH(1, kfirst + KS);
        PH_STORE(0, 0, kfirst);
        PH_FETCH(0, kfirst + 2 * KS);
        __syncthreads();
        PH_PHASE(2);
#define PH_STEP(set, cur, nxt, c_store, c_fetch) do { \
        fused_quarter<KA, KB, VA, VB, true, 0, BP>(acc, s##cur##a, s##cur##b, wm, wn, lane, sa, a_off0, a_off1, ra##set, s##nxt##a, sb, b_off0, b_off1, rb##set, s##nxt##b, (c_store), (c_fetch)); \
        fused_quarter<KA, KB, VA, VB, true, 1, BP>(acc, s##cur##a, s##cur##b, wm, wn, lane, sa, a_off0, a_off1, ra##set, s##nxt##a, sb, b_off0, b_off1, rb##set, s##nxt##b, (c_store), (c_fetch)); \
        fused_quarter<KA, KB, VA, VB, true, 2, BP>(acc, s##cur##a, s##cur##b, wm, wn, lane, sa, a_off0, a_off1, ra##set, s##nxt##a, sb, b_off0, b_off1, rb##set, s##nxt##b, (c_store), (c_fetch)); \
        fused_quarter<KA, KB, VA, VB, true, 3, BP>(acc, s##cur##a, s##cur##b, wm, wn, lane, sa, a_off0, a_off1, ra##set, s##nxt##a, sb, b_off0, b_off1, rb##set, s##nxt##b, (c_store), (c_fetch)); \
    } while (0)
        for (; t + 1 < steps; t += 2) {
            PH_STEP(1, 0, 1, kfirst + (t + 1) * KS, kfirst + (t + 3) * KS);
            __syncthreads();
            PH_STEP(0, 1, 0, kfirst + (t + 2) * KS, kfirst + (t + 4) * KS);
            __syncthreads();
        }
#undef PH_STEP
        if (t < steps) mfma_tile<KA, KB>(acc, s0a, s0b, wm, wn, lane);
    }
    __syncthreads();
    PH_PHASE(3);
#undef PH_FETCH
#undef PH_STORE

    // each team writes its fp32 tile over the staging space (free after the barrier above).  Two teams
    // on one tile hold partial sums of it: the epilogue adds the two while reading.
    float *ctile = (float *)smem_raw;
    constexpr bool PIECES = !ATOMIC && !DUAL && !FOLD && EPI == EPI_STORE && sizeof(TOut) == 4 && VA == 8;
    acc_to_lds(ctile + team * CT_ELEMS, acc, wm, wn, lane);
    __syncthreads();
    PH_PHASE(4);
    if constexpr (ATOMIC) epilogue_atomic_from_lds(P, g, ctile, m0, n0, (int)threadIdx.x);
    else if constexpr (DUAL) epilogue_from_lds<VA, TOut, true, EPI>(P, g, ctile + team * CT_ELEMS, m0, n0, tid, ctile + 2 * CT_ELEMS);
    else if constexpr (PIECES) {
        if (P.parts && P.ksplit > 1)                                 // uniform (one group: the host sees to that)
            epilogue_pieces_from_lds(P, rem, ks, ctile, (unsigned *)(ctile + 2 * CT_ELEMS), m0, n0, (int)threadIdx.x);
        else epilogue_from_lds<VA, TOut, false, EPI>(P, g, ctile, m0, n0, (int)threadIdx.x, ctile + 2 * CT_ELEMS);
    } else epilogue_from_lds<VA, TOut, false, EPI>(P, g, ctile, m0, n0, (int)threadIdx.x, ctile + 2 * CT_ELEMS);
    PH_PHASE(5);
    if constexpr (FOLD) {
        if (fs.on) {                                                 // uniform
            // the block of g: two teams on one tile hold partial sums of it (alternate reduction steps): team 1's goes
            // through LDS to team 0's owner.  A lane holds row (lane & 31) of the block and the columns
            // 8 * (e / 4) + 4 * (lane >> 5) + e % 4 (B operand first, as in acc_to_lds).
            const FoldParams &F = *Fp;
            float *ex = (float *)smem_raw;
            if (!DUAL) {
                __syncthreads();                                     // the tile's epilogue is done with LDS
                if (fs.owner && team == 1) {
#pragma unroll
                    for (int e = 0; e < 16; ++e) ex[e * 64 + lane] = fs.acc[e];
                }
                __syncthreads();
                if (fs.owner && team == 0) {
#pragma unroll
                    for (int e = 0; e < 16; ++e) fs.acc[e] += ex[e * 64 + lane];
                }
            }
            if (fs.owner && (DUAL || team == 0)) {
                const int m = m0 + 32 * e_rb + (lane & 31);
                if (m < P.M) {
                    __bf16 *row = F.G + g * F.o_g + (int64_t)m * F.N;
                    typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
#pragma unroll
                    for (int q = 0; q < 4; ++q) {
                        const int c = 32 * e_cb + 8 * q + 4 * (lane >> 5);
                        if (c < F.N) {                               // N is a multiple of 8: four columns at a time stay inside
                            bf16x4 v = {(__bf16)fs.acc[4 * q], (__bf16)fs.acc[4 * q + 1], (__bf16)fs.acc[4 * q + 2], (__bf16)fs.acc[4 * q + 3]};
                            *(bf16x4 *)(row + c) = v;
                        }
                    }
                }
            }
        }
    }
}

template <int KA, int KB, int VA, int VB, typename TOut, bool ATOMIC, bool PAIR, bool DUAL, int EPI>
__global__ __launch_bounds__(512, 1) void gemm_mfma_kernel(MfmaBatch batch)
{
    int wg = xcd_order(blockIdx.x, 0, batch.total_wg);
    const bool second = PAIR && wg >= batch.first_wg;
    if (second) wg -= batch.first_wg;
    const MfmaParams P = params_at(second ? offsetof(MfmaBatch, p[1]) : offsetof(MfmaBatch, p[0]));
    mfma_workgroup<KA, KB, VA, VB, TOut, ATOMIC, DUAL, EPI>(P, wg);
}

// The last launch of a layer's backward pass, the weight + compressor gradients (tail[0], tail[1]: weight-gradient
// layout, float out; tail[1] may be empty: total_wg = 0), with up to two riders that need nothing it produces:
//  - head, all ranks on the device: the error compression of the layer below (input-gradient layout, storage
//    type out), which fills half of the device or less for a short while.  It runs in the workgroups
//    [0, head_wg) so that it is dispatched first and frees its compute units early.
//    One rank, first layer (no input gradient to share a launch with): the layer's own error compression.  Nothing
//    waits for it, so with more workgroups than compute units it goes out last (rotate) and fills in behind the
//    longer weight-gradient workgroups.
//  - the SGD update of the layer above (sgd_wg workgroups from sgd_first on) on compute units that the
//    products leave idle; its gradients sit in other buffers than the ones tail[] writes.
// tail_first and sgd_first are multiples of 8; workgroups in the gaps do nothing.
struct MfmaTailBatch {
    MfmaParams head;
    MfmaParams tail[2];
    SgdBatch sgd;
    float lr;
    int head_wg;         // = head.total_wg (0: no head)
    int tail_first;
    int tail_wg;         // = tail[0].total_wg + tail[1].total_wg
    int tail0_wg;        // = tail[0].total_wg
    int sgd_first;
    int sgd_wg;          // 0: no update
    int rotate;          // workgroup b does the work of number (b + rotate) mod the grid size: rotate = tail_first
                         //   sends the head's workgroups out last instead of first
    int dual;            // every product of the launch in two-tile workgroups (DUAL of mfma_workgroup): for a launch
                         //   that would otherwise not fit one workgroup per compute unit
};

template <int VEC>
__global__ __launch_bounds__(512, 1) void gemm_mfma_tail_kernel(MfmaTailBatch tb)
{
    int id = (int)blockIdx.x + tb.rotate;
    if (id >= (int)gridDim.x) id -= (int)gridDim.x;
    if (id < tb.tail_first) {                          // uniform, like every branch here
        if (id >= tb.head_wg) return;
        const MfmaParams P = params_at(offsetof(MfmaTailBatch, head));
        if (tb.dual) mfma_workgroup<LD_KC, LD_KM, VEC, VEC, __bf16, false, true, EPI_STORE>(P, xcd_order(id, 0, tb.head_wg));
        else mfma_workgroup<LD_KC, LD_KM, VEC, VEC, __bf16, false, false, EPI_STORE>(P, xcd_order(id, 0, tb.head_wg));
    } else if (id < tb.sgd_first) {
        if (id >= tb.tail_first + tb.tail_wg) return;
        // The XCD-aware order within each product, and within each slab of pieces of a product whose reduction is cut
        // (all first pieces, then all second ones, ...: a piece waits for the one before it, which must not sit
        // behind it in the dispatch order)
        int wg = id - tb.tail_first;
        const bool second = wg >= tb.tail0_wg;
        if (second) wg -= tb.tail0_wg;
        wg = xcd_order(wg, 0, second ? tb.tail_wg - tb.tail0_wg : tb.tail0_wg);
        const MfmaParams P = params_at(second ? offsetof(MfmaTailBatch, tail[1]) : offsetof(MfmaTailBatch, tail[0]));
        if (tb.dual) mfma_workgroup<LD_KM, LD_KM, VEC, VEC, float, false, true, EPI_STORE>(P, wg);
        else mfma_workgroup<LD_KM, LD_KM, VEC, VEC, float, false, false, EPI_STORE>(P, wg);
    } else {
        extern __shared__ __attribute__((aligned(16))) unsigned char smem_raw[];
        sgd_rider<__bf16>(tb.sgd, tb.lr, id - tb.sgd_first, tb.sgd_wg, MFMA_THREADS, (float *)smem_raw);
    }
}

// One rank's weight and compressor gradients of ALL layers in one launch, at the end of the backward pass.
// They depend on nothing but each layer's delta and input, one layer's cover few of the 256 compute units with
// narrow shards (configuration 4: 128 + 8 tiles of 64 reduction steps), and a launch per layer ends when its
// slowest tile does; together they are 1088 tiles that the hardware deals out as compute units come free
// (8 launches of 41 us against one of 170 us).  The SGD update runs in the epilogues (SgdInPlace): every
// launch that reads the weights has finished by then.
// The products' parameter blocks do not fit the 4 KB of kernel arguments (16 blocks of some 600 bytes), so they sit in
// a table in device memory that small launches fill beforehand (table_upload_kernel).  Product j has the
// workgroups [first_wg[j], first_wg[j + 1]) (starts are multiples of 8; workgroups beyond a product's own do nothing).
constexpr int TABLE_PRODUCTS = 32;
constexpr int CHUNK_PRODUCTS = 6;          // parameter blocks per upload launch: kernel arguments hold 4 KB

struct ProductTable {
    int count;
    int first_wg[TABLE_PRODUCTS + 1];
    int wgs[TABLE_PRODUCTS];               // = p[j].total_wg
    int dual[TABLE_PRODUCTS];              // product j in two-tile workgroups (DUAL of mfma_workgroup)
    LossTail tail;                         // workgroup 0 finishes the loss first (partial == NULL: nothing to do)
    MfmaParams p[TABLE_PRODUCTS];
};

struct TableChunk {
    int at, n;                             // blocks p[0 .. n) go to the table's entries at .. at + n
    int count;                             // the table's count once every chunk is there
    int first_wg[CHUNK_PRODUCTS + 1];      // first_wg[at .. at + n]
    int wgs[CHUNK_PRODUCTS];
    int dual[CHUNK_PRODUCTS];
    LossTail tail;
    float *clear_at;                       // the upload also clears clear_count floats there (the step's buffers that
    int clear_count;                       //   are added into: one launch less)
    MfmaParams p[CHUNK_PRODUCTS];
};
static_assert(sizeof(TableChunk) + sizeof(void *) <= 3840, "a chunk travels as kernel arguments (4 KB with the hidden ones)");

// one workgroup of 256 threads copies a chunk from the kernel arguments into the table
__global__ __launch_bounds__(256) void table_upload_kernel(TableChunk c, ProductTable *table)
{
#if defined(__HIP_DEVICE_COMPILE__)
    typedef const uint32_t __attribute__((address_space(4))) *ArgWords;
    const ArgWords in = (ArgWords)((const char __attribute__((address_space(4))) *)__builtin_amdgcn_kernarg_segment_ptr() + offsetof(TableChunk, p));
    uint32_t *out = (uint32_t *)(table->p + c.at);
    const int words = c.n * (int)(sizeof(MfmaParams) / 4);
    for (int i = (int)threadIdx.x; i < words; i += 256) out[i] = in[i];
#endif
    if ((int)threadIdx.x <= c.n) table->first_wg[c.at + threadIdx.x] = c.first_wg[threadIdx.x];
    if ((int)threadIdx.x < c.n) { table->wgs[c.at + threadIdx.x] = c.wgs[threadIdx.x]; table->dual[c.at + threadIdx.x] = c.dual[threadIdx.x]; }
    if (threadIdx.x == 0) { table->count = c.count; table->tail = c.tail; }
    for (int i = (int)threadIdx.x; i < c.clear_count; i += 256) c.clear_at[i] = 0.f;
}

template <int VEC>
__global__ __launch_bounds__(512, 1) void gemm_mfma_table_kernel(const ProductTable *table)
{
#if defined(__HIP_DEVICE_COMPILE__)
    // read through the constant address space: the table is not written during this launch, and its entries are
    // the same for every lane (scalar loads)
    typedef const ProductTable __attribute__((address_space(4))) *TablePtr;
    const TablePtr t = (TablePtr)(uintptr_t)table;
    const int id = (int)blockIdx.x;
    if (id == 0 && t->tail.partial) {                           // uniform
        extern __shared__ __attribute__((aligned(16))) unsigned char smem_raw[];
        LossTail tail;
        tail.partial = t->tail.partial; tail.n = t->tail.n; tail.scale = t->tail.scale; tail.loss = t->tail.loss;
        finish_loss(tail, (float *)smem_raw);
        __syncthreads();
    }
    const int count = t->count;
    int j = 0;
    while (j + 1 < count && id >= t->first_wg[j + 1]) ++j;      // uniform
    const int local = id - t->first_wg[j], wgs = t->wgs[j];
    if (local >= wgs) return;
    constexpr int WORDS = sizeof(MfmaParams) / 4;
    union Words { MfmaParams p; uint32_t w[WORDS]; __device__ Words() {} };
    Words blk;
    typedef const uint32_t __attribute__((address_space(4))) *ArgWords;
    const ArgWords in = (ArgWords)&t->p[j];
#pragma unroll
    for (int i = 0; i < WORDS; ++i) blk.w[i] = in[i];
    if (t->dual[j]) mfma_workgroup<LD_KM, LD_KM, VEC, VEC, float, false, true, EPI_STORE>(blk.p, xcd_order(local, 0, wgs));
    else mfma_workgroup<LD_KM, LD_KM, VEC, VEC, float, false, false, EPI_STORE>(blk.p, xcd_order(local, 0, wgs));
#endif
}

// One rank's forward of a layer in one launch: the layer update, and the thin compression g = C y (see
// thin_product.h), which in one-rank mode do not depend on each other (the peers' g are inputs).  Every
// workgroup takes one tile (or pair of tiles) of the update and then its share of the compression's rows:
// thin_rows consecutive rows (a multiple of 16), all 8 wavefronts splitting the reduction range.  The rows are
// read again right after the update streamed them through the same XCD's L2 (workgroup w's rows lie in the
// band of tile rows that its XCD works on), and no compute unit waits for a compression workgroup: as
// workgroups of their own in front of the update's, the compression's kept half of the device from the
// update for 9 us of a 38 us launch (configuration 5, k = 64: 40.9 -> 38.4 us per launch; at configuration 4,
// where each workgroup's share is 16 rows, the two arrangements take the same time: a share costs a chain of
// latencies, load -> multiply -> exchange -> store, about 5 us however short it is, and starting its loads
// ahead of the update's epilogue changed nothing).
struct MfmaFwdBatch {
    MfmaParams update;
    const __bf16 *X, *C;     // compression operands: X [M, K] per group, C [N, K] per group
    __bf16 *G;               // [M, N] per group
    int M, N, K;
    int64_t x_g, c_g, o_g;
    int update_wg;           // = update.total_wg
    int wg_per_group;        // workgroups of the update per group
    int thin_rows;           // rows of the compression per workgroup: wg_per_group * thin_rows >= M
    FoldParams fold;         // FOLD kernels: the compression inside the update's loop instead (the fields above unused)
};

template <int VEC, bool DUAL, bool FOLD>
__global__ __launch_bounds__(512, 1) void gemm_mfma_fwd_kernel(MfmaFwdBatch fb)
{
    extern __shared__ __attribute__((aligned(16))) unsigned char smem_raw[];
    const int wg = xcd_order((int)blockIdx.x, 0, fb.update_wg);
    const MfmaParams update = params_at(offsetof(MfmaFwdBatch, update));
    if constexpr (FOLD) {
        // the compression rides inside the update's reduction loop (FoldParams)
        mfma_workgroup<LD_KC, LD_KC, VEC, VEC, __bf16, false, DUAL, EPI_BIAS_ACT, true>(update, wg, &fb.fold);
    } else {
        mfma_workgroup<LD_KC, LD_KC, VEC, VEC, __bf16, false, DUAL, EPI_BIAS_ACT>(update, wg);
        const int grp = wg / fb.wg_per_group;
        const int first = (wg - grp * fb.wg_per_group) * fb.thin_rows;
        const int last = min(first + fb.thin_rows, fb.M);
        for (int m0 = first; m0 < last; m0 += THIN_ROWS) {           // uniform
            __syncthreads();                                         // the epilogue, or the block before, is done with LDS
            if (fb.N <= 32) thin_workgroup<1, 8>(fb.X, fb.C, fb.G, last, fb.N, fb.K, fb.x_g, fb.c_g, fb.o_g, m0, grp, (float *)smem_raw);
            else thin_workgroup<2, 8>(fb.X, fb.C, fb.G, last, fb.N, fb.K, fb.x_g, fb.c_g, fb.o_g, m0, grp, (float *)smem_raw);
        }
    }
}

}  // namespace phantom

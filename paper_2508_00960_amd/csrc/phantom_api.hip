// C ABI of libphantom.so: argument checks, workspace layout, and the sequence of
// kernel launches that makes up each operator of the phantom layer.
// Declarations and the meaning of every argument: include/phantom.h.
#include "../../include/phantom.h"

#include <hip/hip_runtime.h>

#include <cstdarg>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <algorithm>
#include <mutex>
#include <string>
#include <type_traits>
#include <vector>

#include "common.h"
#include "elementwise.h"
#include "gemm_generic.h"
#include "gemm_mfma.h"
#include "thin_product.h"
#include "views.h"

using namespace phantom;

namespace {

thread_local std::string g_err;

ph_status fail(ph_status st, const char *fmt, ...)
{
    char buf[512];
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(buf, sizeof buf, fmt, ap);
    va_end(ap);
    g_err = buf;
    return st;
}

#define PH_TRY(expr) do { ph_status st__ = (expr); if (st__ != PH_OK) return st__; } while (0)

// Measurement switches (force one of two launch schedules that the library otherwise chooses between by
// its own model) exist only in a library built with -DPHANTOM_TUNING_ENV; a production build reads no
// environment variable.
inline const char *tuning_env(const char *name)
{
#ifdef PHANTOM_TUNING_ENV
    return getenv(name);
#else
    (void)name;
    return nullptr;
#endif
}

// One layer's shapes on this GPU.  si / so: inputs / outputs of the layer held by one rank (equal unless
// the problem gives per-layer widths).
struct Geo {
    int64_t p, k, B, si, so, q, Kc;
    int groups;       // ranks held on this GPU: 1 or p
    bool all;         // all-ranks mode
    int act, dtype, rank, layers;
    size_t esz;       // bytes per element of the storage type
    int vec;          // bf16: widest vector (8, 4, 2 elements) dividing si, so and k; 0: shape-agnostic kernels only
};

// Checks the problem and fills in the shapes of layer `layer` (0-based).
ph_status make_geo(const ph_problem *pr, Geo &g, int layer = 0)
{
    if (!pr) return fail(PH_ERR_INVALID_ARG, "problem is NULL");
    if (pr->p < 1) return fail(PH_ERR_INVALID_ARG, "p = %lld must be >= 1", (long long)pr->p);
    if (pr->batch < 1) return fail(PH_ERR_INVALID_ARG, "batch = %lld must be >= 1", (long long)pr->batch);
    if (pr->act < PH_ACT_IDENTITY || pr->act > PH_ACT_GELU) return fail(PH_ERR_INVALID_ARG, "unknown activation %d", pr->act);
    if (pr->dtype != PH_F32 && pr->dtype != PH_BF16) return fail(PH_ERR_INVALID_ARG, "unknown dtype %d", pr->dtype);
    if (pr->rank < -1 || pr->rank >= pr->p) return fail(PH_ERR_INVALID_ARG, "rank = %d must lie in [-1, p)", pr->rank);
    if (pr->layers < 1) return fail(PH_ERR_INVALID_ARG, "layers = %d must be >= 1", pr->layers);
    if (layer < 0 || layer >= pr->layers) return fail(PH_ERR_INVALID_ARG, "layer %d of %d", layer, pr->layers);
    int64_t n_in = pr->n, n_out = pr->n, k = pr->k;
    if (pr->widths) {
        if (pr->p > 1 && !pr->ks) return fail(PH_ERR_INVALID_ARG, "widths without ks");
        n_in = pr->widths[layer]; n_out = pr->widths[layer + 1];
        if (pr->ks) k = pr->ks[layer];
    } else if (pr->ks) {
        return fail(PH_ERR_INVALID_ARG, "ks without widths");
    }
    if (n_in < 1 || n_in % pr->p || n_out < 1 || n_out % pr->p)
        return fail(PH_ERR_INVALID_ARG, "layer %d: widths %lld -> %lld must be positive multiples of p = %lld", layer,
                    (long long)n_in, (long long)n_out, (long long)pr->p);
    const int64_t si = n_in / pr->p, so = n_out / pr->p;
    if (pr->p > 1 && (k < 1 || k > std::max(si, so)))
        return fail(PH_ERR_INVALID_ARG, "layer %d: k = %lld must lie in [1, n/p = %lld]", layer, (long long)k,
                    (long long)std::max(si, so));
    g.p = pr->p; g.B = pr->batch; g.si = si; g.so = so; g.q = pr->p - 1;
    g.k = g.q > 0 ? k : 0;
    g.Kc = si + g.q * g.k;
    g.all = pr->rank < 0;
    g.groups = g.all ? (int)pr->p : 1;
    g.act = pr->act; g.dtype = pr->dtype; g.rank = pr->rank; g.layers = pr->layers;
    g.esz = pr->dtype == PH_BF16 ? 2 : 4;
    g.vec = 0;
    if (pr->dtype == PH_BF16) {
        for (int v = 8; v >= 2 && !g.vec; v >>= 1)
            if (si % v == 0 && so % v == 0 && (g.q == 0 || g.k % v == 0)) g.vec = v;
    }
    // The matrix-core kernels address an operand with 32-bit element offsets inside one rank's share of a tensor:
    // a problem with a larger tensor goes through the shape-agnostic kernels (64-bit offsets) like one whose widths
    // allow no vector loads.
    {
        const int64_t wide = std::max(si, so), slots = g.all ? g.p : g.q;
        const int64_t largest = std::max({g.B * wide, slots * g.B * g.k, so * si, slots * so * g.k, g.k * si});
        if (largest > 0x7fffffff) g.vec = 0;
        // they also divide a position among the peers' segments by k with a multiply (Axis::magic), exact while
        // position * k < 2^32
        if (g.q * g.k * g.k >= (int64_t)1 << 32) g.vec = 0;
    }
    // index arithmetic inside the kernels uses 32-bit row/column numbers and a 3-D grid
    if (g.B > (1 << 22) || si > (1 << 22) || so > (1 << 22) || g.Kc > (1 << 24) || so + g.q * g.k > (1 << 24) || g.p > 65535)
        return fail(PH_ERR_UNSUPPORTED, "problem too large for 32-bit tile indices (batch, n/p <= 2^22, n/p+(p-1)k <= 2^24)");
    // ... and numbers its 128 x 128 output tiles with 32 bits, over all ranks held: the largest product of the layer
    {
        auto t = [](int64_t x) { return (x + 127) / 128; };
        const int64_t tiles = std::max({t(g.B) * t(so), t(g.B) * t(si), t(g.B) * t(std::max<int64_t>(g.q * g.k, 1)),
                                        t(so) * t(g.Kc), t(std::max<int64_t>(g.k, 1)) * t(si)}) * g.groups;
        if (tiles * 8 > 0x7fffffff)
            return fail(PH_ERR_UNSUPPORTED, "layer %d: %lld output tiles in one product, more than the kernels number", layer,
                        (long long)tiles);
    }
    return PH_OK;
}

// every layer's shapes (a uniform problem: `layers` copies of the same)
ph_status make_geos(const ph_problem *pr, std::vector<Geo> &geos)
{
    Geo first;
    PH_TRY(make_geo(pr, first, 0));
    geos.assign((size_t)pr->layers, first);
    for (int l = 1; l < pr->layers; ++l) PH_TRY(make_geo(pr, geos[(size_t)l], l));
    return PH_OK;
}

ph_status need(const void *p, const char *name)
{
    if (!p) return fail(PH_ERR_INVALID_ARG, "%s is NULL", name);
    if ((uintptr_t)p & 15) return fail(PH_ERR_INVALID_ARG, "%s is not 16-byte aligned", name);
    return PH_OK;
}
ph_status optional(const void *p, const char *name)
{
    if (p && ((uintptr_t)p & 15)) return fail(PH_ERR_INVALID_ARG, "%s is not 16-byte aligned", name);
    return PH_OK;
}

ph_status check_launch(const char *what)
{
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return fail(PH_ERR_LAUNCH, "%s: %s", what, hipGetErrorString(e));
    return PH_OK;
}

// ---- optional per-launch timing (phantom_profile_begin / _end) ----------------------------
struct ProfRec {
    const char *name;
    int64_t M, N, K;
    int groups;
    int64_t M2, N2, K2;   // second to fourth product of a launch that carries several (0 if none)
    int64_t M3, N3, K3;
    int64_t M4, N4, K4;
};
struct Profiler {
    bool on = false;
    std::vector<hipEvent_t> ev;      // 2 per record: start, stop
    std::vector<ProfRec> recs;
    size_t cap = 0;
    bool calibrated = false;
};
thread_local Profiler g_prof;
constexpr int PROF_CALIBRATION_LAUNCHES = 32;
const char *const PROF_EMPTY_NAME = "(empty launch)";

// Brackets one kernel launch with a pair of events on its stream while profiling is on.
struct ProfScope {
    hipStream_t st;
    long idx = -1;
    ProfScope(const char *name, int64_t M, int64_t N, int64_t K, int groups, hipStream_t s, int64_t M2 = 0,
              int64_t N2 = 0, int64_t K2 = 0, int64_t M3 = 0, int64_t N3 = 0, int64_t K3 = 0, int64_t M4 = 0, int64_t N4 = 0,
              int64_t K4 = 0) : st(s)
    {
        if (!g_prof.on) return;
        if (!g_prof.calibrated) {
            // What an event pair reads around a kernel that does nothing: the part of every figure
            // below that is launch and time-stamp latency rather than execution.  Reported as an
            // entry of its own so that the caller can subtract it.
            g_prof.calibrated = true;
            for (int i = 0; i < PROF_CALIBRATION_LAUNCHES && g_prof.recs.size() < g_prof.cap; ++i) {
                const long at = (long)g_prof.recs.size();
                g_prof.recs.push_back(ProfRec{PROF_EMPTY_NAME, 0, 0, 0, 1, 0, 0, 0, 0, 0, 0, 0, 0, 0});
                (void)hipEventRecord(g_prof.ev[2 * at], st);
                hipLaunchKernelGGL(fill_zero_kernel, dim3(256), dim3(256), 0, st, (float *)nullptr, (int64_t)0);
                (void)hipEventRecord(g_prof.ev[2 * at + 1], st);
            }
        }
        if (g_prof.recs.size() >= g_prof.cap) return;
        idx = (long)g_prof.recs.size();
        g_prof.recs.push_back(ProfRec{name, M, N, K, groups, M2, N2, K2, M3, N3, K3, M4, N4, K4});
        (void)hipEventRecord(g_prof.ev[2 * idx], st);
    }
    ~ProfScope()
    {
        if (idx >= 0) (void)hipEventRecord(g_prof.ev[2 * idx + 1], st);
    }
};

// ---- workspace ---------------------------------------------------------------
struct Arena {
    char *base;
    size_t used;
    void *take(size_t bytes)
    {
        size_t at = (used + 255) & ~(size_t)255;
        used = at + bytes;
        return base ? base + at : nullptr;
    }
};

constexpr int MSE_BLOCKS = 1024;
constexpr int PIECE_WORDS = 512;      // output tiles of the products of one launch whose reduction may be cut into pieces (MfmaParams::arrived)

struct BwdWs {
    void *delta;        // [groups, B, so] storage type
};

BwdWs carve_bwd(Arena &a, const Geo &g)
{
    BwdWs w;
    w.delta = a.take((size_t)g.groups * g.B * g.so * g.esz);
    return w;
}

struct StepWs {
    std::vector<void *> Y, A, G;
    std::vector<void *> relu_bits;                  // per layer, or NULL: one bit per element of y_l (y_l > 0), see relu_bits_ok
    void *dYa, *dYb, *dG_send, *dg_own;
    float *dLw[2], *dCw[2], *dDw[2];                // two sets, used by alternate layers: a layer's update may still read
                                                    //   its gradients while the layer below writes its own
    float *dbias, *mse_partial;                     // dbias: one block, layer l's [groups, so_l] at dbias_at[l]
    std::vector<int64_t> dbias_at;                  // float offsets into dbias; dbias_at[layers] = the block's length
    unsigned *arrived;                              // PIECE_WORDS words right behind the dbias block: cleared with it at the
                                                    //   start of a step, left zero by every launch that uses them
    float *parts;                                   // deferred weight gradients (one rank): the pieces' results of the cut
    ProductTable *table;                            //   compressor gradients, the launch's parameter table, and every
    std::vector<void *> delta_of;                   //   layer's delta [B, so_l]
    BwdWs bwd;
};

// ReLU in bf16 storage: what the backward pass needs of layer l is the sign of its stored output alone.  Where the
// update of layer l and the input gradient of layer l + 1 (whose epilogue multiplies by sigma'_l) both run on the
// matrix cores with 8-element vectors, the update leaves one bit per element and the input gradient reads
// that instead of the bf16 output: an eighth of the bytes (configuration 2: 8.4 MB -> 0.5 MB per launch).
bool relu_bits_ok(const std::vector<Geo> &geos, size_t l)
{
    return l + 1 < geos.size() && geos[l].act == PH_ACT_RELU && geos[l].dtype == PH_BF16 && geos[l].vec == 8 &&
           geos[l + 1].vec == 8;
}

inline int64_t tiles_of(int64_t M, int64_t N) { return ((M + MT - 1) / MT) * ((N + MT - 1) / MT); }

// One rank's backward pass over two or more layers keeps every layer's delta and runs all weight + compressor
// gradients in one launch at its end (gemm_mfma_table_kernel) where a layer's own would leave compute units idle:
// bf16 with 8-element vectors and at most 256 weight-gradient tiles in every layer.  (All ranks on the device:
// the weight gradients' launches carry the next error compression and the update on the compute units they leave
// idle, and putting them off made configuration 2 slower, 0.272 against 0.260 ms; a single layer has nothing to gain.)
bool deferred_weight_gradients(const std::vector<Geo> &geos)
{
    if (geos.size() < 2 || 2 * geos.size() > (size_t)TABLE_PRODUCTS) return false;
    for (const Geo &g : geos)
        if (g.all || g.dtype != PH_BF16 || g.vec != 8 || tiles_of(g.so, g.Kc) > 256) return false;
    return true;
}

// The compressor gradient [k, si] of a layer has few tiles with a long reduction (configuration 4: 8 tiles of 64
// steps, half of their rows empty).  In that launch they are cut along the batch into pieces of at least 16 steps,
// at most 4, which go out first and add up without atomics (MfmaParams::parts).
int compressor_gradient_pieces(const Geo &g)
{
    const int64_t ksteps = (g.B + KT - 1) / KT;
    return (int)std::max<int64_t>(1, std::min<int64_t>(ksteps / 16, 4));
}

// geos: every layer's shapes.  Buffers that are reused from layer to layer take the largest layer's size.
StepWs carve_step(Arena &a, const std::vector<Geo> &geos)
{
    StepWs w;
    for (size_t l = 0; l < geos.size(); ++l)
        w.relu_bits.push_back(relu_bits_ok(geos, l) ? a.take((size_t)geos[l].groups * geos[l].B * geos[l].so / 8) : nullptr);
    const Geo &g0 = geos[0];
    size_t act_max = 0, k_max = 0, lw_max = 0, cw_max = 0, dw_max = 0;
    int64_t dbias_total = 0;
    for (const Geo &g : geos) {
        const size_t act_bytes = (size_t)g.groups * g.B * g.so * g.esz;
        w.Y.push_back(a.take(act_bytes));
        // GELU keeps per layer, in float: fp32 storage, the pre-activation; bf16 storage, sigma'(pre-activation)
        w.A.push_back(g.act == PH_ACT_GELU ? a.take((size_t)g.groups * g.B * g.so * sizeof(float)) : nullptr);
        w.G.push_back(g.q > 0 ? a.take((size_t)g.groups * g.B * g.k * g.esz) : nullptr);   // all-ranks: [p,B,k]; one-rank: [B,k]
        act_max = std::max(act_max, (size_t)std::max(g.si, g.so));
        k_max = std::max(k_max, (size_t)g.k);
        lw_max = std::max(lw_max, (size_t)(g.so * g.si));
        cw_max = std::max(cw_max, (size_t)(g.k * g.si));
        dw_max = std::max(dw_max, (size_t)(g.q * g.so * g.k));
        w.dbias_at.push_back(dbias_total);
        dbias_total += ((int64_t)g.groups * g.so + 3) & ~(int64_t)3;   // every layer's block starts 16-byte aligned
    }
    w.dbias_at.push_back(dbias_total);
    const size_t groups = (size_t)g0.groups, B = (size_t)g0.B;
    w.dYa = a.take(groups * B * act_max * g0.esz);
    w.dYb = a.take(groups * B * act_max * g0.esz);
    w.dG_send = g0.q > 0 ? a.take(groups * g0.q * B * k_max * g0.esz) : nullptr;
    w.dg_own = g0.q > 0 ? a.take(groups * B * k_max * g0.esz) : nullptr;
    for (int set = 0; set < 2; ++set) {
        w.dLw[set] = (float *)a.take(groups * lw_max * 4);
        w.dCw[set] = (float *)a.take(groups * cw_max * 4 + 16);
        w.dDw[set] = (float *)a.take(groups * dw_max * 4 + 16);
    }
    w.dbias = (float *)a.take((size_t)(dbias_total + PIECE_WORDS) * 4);
    w.arrived = w.dbias ? (unsigned *)(w.dbias + dbias_total) : nullptr;
    if (deferred_weight_gradients(geos)) {
        size_t slots = 0;
        for (const Geo &g : geos) {
            w.delta_of.push_back(a.take((size_t)g.B * g.so * g.esz));
            if (g.q > 0) slots += (size_t)tiles_of(g.k, g.si) * compressor_gradient_pieces(g);
        }
        w.parts = (float *)a.take(std::max<size_t>(slots, 1) * MT * MT * sizeof(float));
        w.table = (ProductTable *)a.take(sizeof(ProductTable));
    } else {
        w.parts = nullptr;
        w.table = nullptr;
    }
    w.mse_partial = (float *)a.take(MSE_BLOCKS * sizeof(float));
    w.bwd.delta = a.take(groups * B * act_max * g0.esz);
    return w;
}

// ---- one product ---------------------------------------------------------------
inline unsigned blocks_for(int64_t count, int per_block = 256, int cap = 8192)
{
    int64_t b = (count + per_block - 1) / per_block;
    if (b < 1) b = 1;
    if (b > cap) b = cap;
    return (unsigned)b;
}

// How a product is to be run: loader kinds of the two operands for the MFMA kernel, the vector
// width the problem allows (0: use the shape-agnostic kernel), and whether the reduction may be
// split over workgroups (float outputs only; the output is cleared first and added to atomically).
struct GemmPlan {
    int ka, kb;
    int vec;
    bool may_split;
};

struct Product {
    View a, b, o;
    Epilogue ep;
    int64_t M, N, K;
    SumOnRead rs;        // matrix-core path only: the tail block of a is summed on read (src != nullptr)
};

template <int KA, int KB, int VEC, typename TOut, bool ATOMIC, bool PAIR, bool DUAL, int EPI>
ph_status launch_mfma_kernel(const MfmaBatch &batch, hipStream_t st, const char *what)
{
    auto kern = gemm_mfma_kernel<KA, KB, VEC, VEC, TOut, ATOMIC, PAIR, DUAL, EPI>;
    static thread_local bool configured = false;
    if (!configured) {
        hipError_t e = hipFuncSetAttribute((const void *)kern, hipFuncAttributeMaxDynamicSharedMemorySize, MFMA_LDS_BYTES);
        if (e != hipSuccess) return fail(PH_ERR_LAUNCH, "%s: cannot reserve %d bytes of LDS: %s", what, MFMA_LDS_BYTES,
                                         hipGetErrorString(e));
        configured = true;
    }
    hipLaunchKernelGGL(kern, dim3((unsigned)batch.total_wg), dim3(MFMA_THREADS), MFMA_LDS_BYTES, st, batch);
    return check_launch(what);
}

template <int KA, int KB, int VEC, typename TOut, bool ATOMIC, int EPI>
ph_status launch_mfma_inst(const MfmaBatch &batch, bool dual, hipStream_t st, const char *what)
{
    if constexpr (!ATOMIC) {
        if (dual) {
            if (batch.count == 2) return launch_mfma_kernel<KA, KB, VEC, TOut, false, true, true, EPI>(batch, st, what);
            return launch_mfma_kernel<KA, KB, VEC, TOut, false, false, true, EPI>(batch, st, what);
        }
    }
    if (batch.count == 2) return launch_mfma_kernel<KA, KB, VEC, TOut, ATOMIC, true, false, EPI>(batch, st, what);
    return launch_mfma_kernel<KA, KB, VEC, TOut, ATOMIC, false, false, EPI>(batch, st, what);
}

// EPI: the epilogue mode the kernel is built for besides the plain store (see epilogue_from_lds)
template <int KA, int KB, typename TOut, bool ATOMIC, int EPI>
ph_status launch_mfma_vec(const MfmaBatch &batch, int vec, bool dual, hipStream_t st, const char *what)
{
    switch (vec) {
    case 8: return launch_mfma_inst<KA, KB, 8, TOut, ATOMIC, EPI>(batch, dual, st, what);
    case 4: return launch_mfma_inst<KA, KB, 4, TOut, ATOMIC, EPI>(batch, dual, st, what);
    default: return launch_mfma_inst<KA, KB, 2, TOut, ATOMIC, EPI>(batch, dual, st, what);
    }
}

MfmaParams mfma_params(const Product &pr, int groups, int ksplit, bool dual)
{
    MfmaParams P{};
    P.a = pr.a; P.b = pr.b; P.o = pr.o; P.ep = pr.ep; P.rs = pr.rs;
    P.M = (int)pr.M; P.N = (int)pr.N; P.K = (int)pr.K;
    const int mt = dual ? 2 * MT : MT;               // rows of C per workgroup
    P.tiles_m = (int)((pr.M + mt - 1) / mt);
    P.tiles_n = (int)((pr.N + MT - 1) / MT);
    const int ksteps = (int)((pr.K + KT - 1) / KT);
    const int steps_per = (ksteps + ksplit - 1) / ksplit;
    P.ksplit = (ksteps + steps_per - 1) / steps_per;
    P.k_per_split = steps_per * KT;
    P.total_wg = P.tiles_m * P.tiles_n * groups * P.ksplit;
    return P;
}

// bf16 operands on the matrix cores: one product, or two of the same layout side by side in one launch
template <typename TOut>
ph_status launch_mfma(const GemmPlan &plan, const Product *prods, int count, int groups, hipStream_t st, const char *what)
{
    int ksplit = 1;
    const Product &first = prods[0];
    const int64_t tiles = ((first.M + MT - 1) / MT) * ((first.N + MT - 1) / MT) * groups;
    if (tiles * 8 > 0x7fffffff) return fail(PH_ERR_LAUNCH, "%s: internal error, too many tiles (make_geo admits none such)", what);
    if (count == 1 && plan.may_split && std::is_same<TOut, float>::value && first.ep.mode == EPI_STORE) {
        // Splitting pays only when the tiles cover a small part of the 256 compute units: the atomic
        // adds of a split cost about as much as the product itself (measured: 512 x 736 x 1024 x 8
        // takes 34 us unsplit, 64 us in 3 pieces).  Then aim at one workgroup per compute unit and
        // keep at least 8 reduction steps per piece.
        const int ksteps = (int)((first.K + KT - 1) / KT);
        // A short reduction is not worth a split either (32 x 512 x 1024 x 16: 13 us whole, 27 us + a clear in pieces).
        if (tiles < 96 && ksteps >= 32)
            ksplit = (int)std::max<int64_t>(1, std::min<int64_t>((256 + tiles - 1) / tiles, ksteps / 8));
    }
    // More tiles than compute units: the launch would run in rounds.  Then two tiles, one above the other,
    // go to one workgroup (its teams share the B tile): fewer bytes staged per FLOP and half the rounds.
    // PHANTOM_DUAL=0 / 1 forces the choice (for measurements).
    bool dual = false;
    if (ksplit == 1) {
        int64_t all_tiles = tiles;
        if (count == 2) all_tiles += ((prods[1].M + MT - 1) / MT) * ((prods[1].N + MT - 1) / MT) * groups;
        dual = all_tiles > 256;
        static const char *force = tuning_env("PHANTOM_DUAL");
        if (force) dual = force[0] == '1';
    }
    MfmaBatch batch{};
    batch.count = count;
    batch.p[0] = mfma_params(first, groups, ksplit, dual);
    batch.total_wg = batch.p[0].total_wg;
    batch.first_wg = batch.p[0].total_wg;
    if (count == 2) {
        batch.p[1] = mfma_params(prods[1], groups, 1, dual);
        batch.total_wg += batch.p[1].total_wg;
    }
    const Product &second = prods[count - 1];
    if (batch.p[0].ksplit > 1) {
        if constexpr (std::is_same<TOut, float>::value) {
            // clear what the split pieces add into (both regions of the output view)
            for (int region = 0; region < 2; ++region) {
                float *base = (float *)(region ? first.o.p1 : first.o.p0);
                const int64_t per_group = region ? first.o.g1 : first.o.g0;
                if (!base || per_group <= 0) continue;
                const int64_t n = per_group * groups;
                ProfScope prof("clear split-K output", 0, n, 0, 1, st);
                hipLaunchKernelGGL(fill_zero_kernel, dim3(blocks_for(n, 1024)), dim3(256), 0, st, base, n);
                PH_TRY(check_launch("clear split-K output"));
            }
            ProfScope prof(what, first.M, first.N, first.K, groups, st);
            if (plan.ka == LD_KM && plan.kb == LD_KM) return launch_mfma_vec<LD_KM, LD_KM, float, true, EPI_STORE>(batch, plan.vec, false, st, what);
        }
        return fail(PH_ERR_LAUNCH, "%s: internal error, split reduction asked for an operand layout that has none", what);
    }
    ProfScope prof(what, first.M, first.N, first.K, groups, st, count == 2 ? second.M : 0, count == 2 ? second.N : 0,
                   count == 2 ? second.K : 0);
    // The kernels that exist: the forward layout (both operands read along the reduction index) with the
    // bias + activation epilogue, the input-gradient layout with the sigma' epilogue, each also with the plain
    // store alone, in the storage type; the weight-gradient layout with the plain store in float.  The
    // second product of a pair always stores plainly.
    const int mode = first.ep.mode;
    if (count == 2 && second.ep.mode != EPI_STORE) return fail(PH_ERR_LAUNCH, "%s: internal error, the second product of a pair must store plainly", what);
    if constexpr (std::is_same<TOut, float>::value) {
        if (plan.ka == LD_KM && plan.kb == LD_KM && mode == EPI_STORE)
            return launch_mfma_vec<LD_KM, LD_KM, float, false, EPI_STORE>(batch, plan.vec, dual, st, what);
    } else {
        if (plan.ka == LD_KC && plan.kb == LD_KC) {
            if (mode == EPI_BIAS_ACT) return launch_mfma_vec<LD_KC, LD_KC, TOut, false, EPI_BIAS_ACT>(batch, plan.vec, dual, st, what);
            if (mode == EPI_STORE) return launch_mfma_vec<LD_KC, LD_KC, TOut, false, EPI_STORE>(batch, plan.vec, dual, st, what);
        }
        if (plan.ka == LD_KC && plan.kb == LD_KM) {
            if (mode == EPI_DACT) return launch_mfma_vec<LD_KC, LD_KM, TOut, false, EPI_DACT>(batch, plan.vec, dual, st, what);
            if (mode == EPI_STORE) return launch_mfma_vec<LD_KC, LD_KM, TOut, false, EPI_STORE>(batch, plan.vec, dual, st, what);
        }
    }
    return fail(PH_ERR_LAUNCH, "%s: internal error, no kernel for this operand layout, output type and epilogue", what);
}

// The weight + compressor gradients (tail0, tail1; tail1 may be empty) with their riders in one launch: the
// error compression of the layer below (head, may be NULL) and the SGD update of the layer above (sgd, may be
// NULL, on sgd_wg workgroups): see MfmaTailBatch.
template <int VEC>
ph_status launch_tail_kernel(const MfmaTailBatch &tb, unsigned total_wg, hipStream_t st, const char *what)
{
    auto kern = gemm_mfma_tail_kernel<VEC>;
    static thread_local bool configured = false;
    if (!configured) {
        hipError_t e = hipFuncSetAttribute((const void *)kern, hipFuncAttributeMaxDynamicSharedMemorySize, MFMA_LDS_BYTES);
        if (e != hipSuccess) return fail(PH_ERR_LAUNCH, "%s: cannot reserve %d bytes of LDS: %s", what, MFMA_LDS_BYTES,
                                         hipGetErrorString(e));
        configured = true;
    }
    hipLaunchKernelGGL(kern, dim3(total_wg), dim3(MFMA_THREADS), MFMA_LDS_BYTES, st, tb);
    return check_launch(what);
}

ph_status launch_tail(const Product *head, const Product &tail0, const Product &tail1, const SgdBatch *sgd, float lr,
                      int sgd_wg, int groups, int vec, hipStream_t st, const char *what, bool head_last = false)
{
    MfmaTailBatch tb{};
    const bool two = tail1.M > 0 && tail1.N > 0;
    // More tiles than compute units with the head's: in two-tile workgroups if the launch then fits one round
    // (PHANTOM_TAIL_DUAL=0 / 1 forces the choice, for measurements)
    auto wgs = [&](bool dual) {
        int64_t n = (head ? (int64_t)mfma_params(*head, groups, 1, dual).total_wg : 0) + mfma_params(tail0, groups, 1, dual).total_wg;
        if (two) n += mfma_params(tail1, groups, 1, dual).total_wg;
        return n;
    };
    bool dual = head && !head_last && wgs(false) > 256 && wgs(true) <= 256;
    static const char *dual_force = tuning_env("PHANTOM_TAIL_DUAL");
    if (dual_force) dual = dual_force[0] == '1';
    tb.dual = dual;
    if (head) tb.head = mfma_params(*head, groups, 1, dual);
    tb.head_wg = head ? tb.head.total_wg : 0;
    tb.tail_first = (tb.head_wg + 7) & ~7;
    tb.tail[0] = mfma_params(tail0, groups, 1, dual);
    tb.tail_wg = tb.tail[0].total_wg;
    tb.tail0_wg = tb.tail[0].total_wg;
    if (two) {
        tb.tail[1] = mfma_params(tail1, groups, 1, dual);
        tb.tail_wg += tb.tail[1].total_wg;
    }
    tb.sgd_first = (tb.tail_first + tb.tail_wg + 7) & ~7;
    tb.sgd_wg = sgd ? sgd_wg : 0;
    if (sgd) { tb.sgd = *sgd; tb.lr = lr; }
    ProfScope prof(what, tail0.M, tail0.N, tail0.K, groups, st, two ? tail1.M : 0, two ? tail1.N : 0, two ? tail1.K : 0,
                   head ? head->M : 0, head ? head->N : 0, head ? head->K : 0);
    const unsigned total = (unsigned)(tb.sgd_first + tb.sgd_wg);
    tb.rotate = (head && head_last) ? tb.tail_first : 0;
    switch (vec) {
    case 8: return launch_tail_kernel<8>(tb, total, st, what);
    case 4: return launch_tail_kernel<4>(tb, total, st, what);
    default: return launch_tail_kernel<2>(tb, total, st, what);
    }
}

// The weight-gradient-layout products `prods` (float out, 8-element vectors, one group each; at most TABLE_PRODUCTS)
// in one launch through a parameter table in device memory: see gemm_mfma_table_kernel.  upload_product_table
// fills the table (small launches, any time before); launch_product_table runs the products.
// splits[j] > 1 cuts product j's reduction into pieces (parts, arrived: room for all of them, see MfmaParams);
// sgd[j].master0 != NULL puts the SGD update into product j's epilogue.  tail: the launch's first workgroup finishes
// the loss.  clear_at, clear_count: floats that the first upload launch clears on its way.  *grid: the launch's size.
ph_status upload_product_table(const std::vector<Product> &prods, const std::vector<int> &splits, const std::vector<SgdInPlace> &sgd,
                               ProductTable *table, float *parts, unsigned *arrived, const LossTail &tail, float *clear_at,
                               int64_t clear_count, hipStream_t st, int *grid)
{
    const char *what = "parameter table";
    if (prods.size() > (size_t)TABLE_PRODUCTS) return fail(PH_ERR_LAUNCH, "%s: internal error, more products than the table holds", what);
    size_t slot = 0, word = 0;
    std::vector<MfmaParams> blocks;
    std::vector<int> first, duals;
    int64_t all_tiles = 0;
    for (const Product &pr : prods) all_tiles += tiles_of(pr.M, pr.N);
    const bool many_tiles = all_tiles > 256;
    int next = 0;
    for (size_t j = 0; j < prods.size(); ++j) {
        const Product &pr = prods[j];
        if (tiles_of(pr.M, pr.N) * 8 > 0x7fffffff) return fail(PH_ERR_LAUNCH, "%s: internal error, too many tiles (make_geo admits none such)", what);
        // with more than 256 tiles in the launch, the uncut products run in two-tile workgroups like a launch of their own
        const bool dual = splits[j] == 1 && many_tiles;
        MfmaParams P = mfma_params(pr, 1, splits[j], dual);
        duals.push_back(dual ? 1 : 0);
        const int64_t tiles = tiles_of(pr.M, pr.N);
        if (P.ksplit > 1) {
            P.parts = parts + slot * MT * MT; P.arrived = arrived + word;
            slot += (size_t)tiles * splits[j]; word += (size_t)tiles;
        }
        P.sgd = sgd[j];
        first.push_back(next);
        next += (P.total_wg + 7) & ~7;
        blocks.push_back(P);
    }
    first.push_back(next);
    if (word > (size_t)PIECE_WORDS) return fail(PH_ERR_LAUNCH, "%s: internal error, more cut tiles than words to count them", what);
    const int count = (int)blocks.size();
    for (int at = 0; at < count; at += CHUNK_PRODUCTS) {
        TableChunk c{};
        c.at = at; c.n = std::min(CHUNK_PRODUCTS, count - at); c.count = count; c.tail = tail;
        if (at == 0) { c.clear_at = clear_at; c.clear_count = (int)clear_count; }
        for (int i = 0; i < c.n; ++i) { c.p[i] = blocks[(size_t)(at + i)]; c.wgs[i] = blocks[(size_t)(at + i)].total_wg; c.dual[i] = duals[(size_t)(at + i)]; }
        for (int i = 0; i <= c.n; ++i) c.first_wg[i] = first[(size_t)(at + i)];
        ProfScope prof(what, 0, (int64_t)c.n * (int64_t)(sizeof(MfmaParams) / 4) + c.clear_count, 0, 1, st);
        hipLaunchKernelGGL(table_upload_kernel, dim3(1), dim3(256), 0, st, c, table);
        PH_TRY(check_launch(what));
    }
    *grid = next;
    return PH_OK;
}

// prof_a, prof_b, prof_groups: the profile entry's two shapes and how many products of each the table holds (exact
// when all layers have the same shapes)
ph_status launch_product_table(const ProductTable *table, int grid, hipStream_t st, const char *what, const Product &prof_a,
                               const Product &prof_b, int prof_groups)
{
    auto kern = gemm_mfma_table_kernel<8>;
    static thread_local bool configured = false;
    if (!configured) {
        hipError_t e = hipFuncSetAttribute((const void *)kern, hipFuncAttributeMaxDynamicSharedMemorySize, MFMA_LDS_BYTES);
        if (e != hipSuccess) return fail(PH_ERR_LAUNCH, "%s: cannot reserve %d bytes of LDS: %s", what, MFMA_LDS_BYTES,
                                         hipGetErrorString(e));
        configured = true;
    }
    ProfScope prof(what, prof_a.M, prof_a.N, prof_a.K, prof_groups, st, prof_b.M, prof_b.N, prof_b.K);
    hipLaunchKernelGGL(kern, dim3((unsigned)grid), dim3(MFMA_THREADS), MFMA_LDS_BYTES, st, table);
    return check_launch(what);
}

// One rank's thin compression and layer update in one launch: see MfmaFwdBatch.
template <int VEC, bool DUAL, bool FOLD = false>
ph_status launch_fwd_kernel(const MfmaFwdBatch &fb, unsigned total_wg, hipStream_t st, const char *what)
{
    auto kern = gemm_mfma_fwd_kernel<VEC, DUAL, FOLD>;
    static thread_local bool configured = false;
    if (!configured) {
        hipError_t e = hipFuncSetAttribute((const void *)kern, hipFuncAttributeMaxDynamicSharedMemorySize, MFMA_LDS_BYTES);
        if (e != hipSuccess) return fail(PH_ERR_LAUNCH, "%s: cannot reserve %d bytes of LDS: %s", what, MFMA_LDS_BYTES,
                                         hipGetErrorString(e));
        configured = true;
    }
    hipLaunchKernelGGL(kern, dim3(total_wg), dim3(MFMA_THREADS), MFMA_LDS_BYTES, st, fb);
    return check_launch(what);
}

ph_status launch_fwd_pair(const Product &update, const Product &compress, int groups, int vec, hipStream_t st, const char *what)
{
    const int64_t tiles = tiles_of(update.M, update.N) * groups;
    if (tiles * 8 > 0x7fffffff) return fail(PH_ERR_LAUNCH, "%s: internal error, too many tiles (make_geo admits none such)", what);
    const bool dual = tiles > 256;                     // as for a launch of the update alone
    MfmaFwdBatch fb{};
    fb.update = mfma_params(update, groups, 1, dual);
    fb.X = (const __bf16 *)compress.a.p0; fb.C = (const __bf16 *)compress.b.p0; fb.G = (__bf16 *)compress.o.p0;
    fb.M = (int)compress.M; fb.N = (int)compress.N; fb.K = (int)compress.K;
    fb.x_g = compress.a.g0; fb.c_g = compress.b.g0; fb.o_g = compress.o.g0;
    fb.update_wg = fb.update.total_wg;
    fb.wg_per_group = fb.update.total_wg / groups;
    fb.thin_rows = (int)(((compress.M + fb.wg_per_group - 1) / fb.wg_per_group + 15) / 16 * 16);
    const unsigned total = (unsigned)fb.update.total_wg;
    ProfScope prof(what, update.M, update.N, update.K, groups, st, compress.M, compress.N, compress.K);
    // The compression inside the update's reduction loop (FoldParams): 16-byte vectors, shapes that take the loop's
    // fast path (widths multiples of 64; the phantom width a divisor of 64), and a tile row with at least as many
    // workgroups as the compression has 32 x 32 blocks per 128 rows.
    const int64_t si = compress.K, k = compress.N;
    const int ncb = (int)((k + 31) / 32);
    // One tile per workgroup only: with two tiles per workgroup (more than 256 tiles) the loop has no registers to
    // spare, and the share behind the epilogue measured as fast or faster (configuration 5, k = 16: 0.195 against 0.221 ms).
    if (!dual && vec == 8 && si % KT == 0 && KT % k == 0 && 4 * ncb <= fb.update.tiles_n && update.a.c.decides && update.a.c.split == si) {
        fb.fold.C = fb.C; fb.fold.G = fb.G; fb.fold.c_g = fb.c_g; fb.fold.o_g = fb.o_g;
        fb.fold.N = (int)k; fb.fold.K = (int)si; fb.fold.ncb = ncb; fb.fold.nblocks = 4 * ncb;
        return launch_fwd_kernel<8, false, true>(fb, total, st, what);
    }
    switch (vec) {
    case 8: return dual ? launch_fwd_kernel<8, true>(fb, total, st, what) : launch_fwd_kernel<8, false>(fb, total, st, what);
    case 4: return dual ? launch_fwd_kernel<4, true>(fb, total, st, what) : launch_fwd_kernel<4, false>(fb, total, st, what);
    default: return dual ? launch_fwd_kernel<2, true>(fb, total, st, what) : launch_fwd_kernel<2, false>(fb, total, st, what);
    }
}

// Runs one product, or two independent ones of the same kind (names: `what` for the pair on the
// matrix cores, `what` / `what2` when they run as separate launches of the shape-agnostic kernel).
template <typename TIn, typename TOut>
ph_status launch_products(const GemmPlan &plan, const Product *prods_in, int count_in, int groups, hipStream_t st,
                          const char *what, const char *what_first = nullptr, const char *what_second = nullptr)
{
    Product prods[2];
    const char *names[2];
    int count = 0;
    for (int i = 0; i < count_in; ++i)
        if (prods_in[i].M > 0 && prods_in[i].N > 0) {
            names[count] = i == 0 ? (what_first ? what_first : what) : (what_second ? what_second : what);
            prods[count++] = prods_in[i];
        }
    if (count == 0 || groups <= 0) return PH_OK;
    if constexpr (std::is_same<TIn, bf16_t>::value) {
        if (plan.vec > 0) {
            // Two products share a launch when the launch-time model below says the pair is faster.  A
            // workgroup occupies a whole compute unit, so up to 256 tiles run at once (fixed cost ~8.6 us +
            // 0.5 us per 64 of the reduction length); above that, workgroups take two tiles each (~9.5 us +
            // 0.76 us per 64) and run in rounds of 256.  Separate launches pay ~2.5 us for the extra launch.
            // PHANTOM_PAIR=0 / 1 forces the choice (for measurements).
            bool pair = count == 2;
            if (pair) {
                auto tiles_of = [&](const Product &pr) { return ((pr.M + MT - 1) / MT) * ((pr.N + MT - 1) / MT) * groups; };
                auto launch_us = [](int64_t tiles, int64_t K) {
                    const double steps = (double)((K + KT - 1) / KT);
                    if (tiles <= 256) return 8.6 + 0.5 * steps;
                    return (double)(((tiles + 1) / 2 + 255) / 256) * (9.5 + 0.76 * steps);
                };
                const int64_t t0 = tiles_of(prods[0]), t1 = tiles_of(prods[1]);
                const double together = launch_us(t0 + t1, std::max(prods[0].K, prods[1].K));
                const double apart = launch_us(t0, prods[0].K) + launch_us(t1, prods[1].K) + 2.5;
                pair = together < apart;
                static const char *force = tuning_env("PHANTOM_PAIR");
                if (force) pair = force[0] == '1';
            }
            if (pair || count == 1) return launch_mfma<TOut>(plan, prods, count, groups, st, count == 2 ? what : names[0]);
            GemmPlan single = plan;
            PH_TRY(launch_mfma<TOut>(single, &prods[0], 1, groups, st, names[0]));
            return launch_mfma<TOut>(single, &prods[1], 1, groups, st, names[1]);
        }
    }
    for (int i = 0; i < count; ++i) {
        const Product &pr = prods[i];
        ProfScope prof(names[i], pr.M, pr.N, pr.K, groups, st);
        dim3 grid((unsigned)((pr.N + GT - 1) / GT), (unsigned)((pr.M + GT - 1) / GT), (unsigned)groups);
        hipLaunchKernelGGL((gemm_generic_kernel<TIn, TOut>), grid, dim3(256), 0, st, pr.a, pr.b, pr.o, pr.ep, (int)pr.M,
                           (int)pr.N, (int)pr.K);
        PH_TRY(check_launch(names[i]));
    }
    return PH_OK;
}

template <typename TIn, typename TOut>
ph_status launch_gemm(const GemmPlan &plan, const View &a, const View &b, const View &o, const Epilogue &ep,
                      int64_t M, int64_t N, int64_t K, int groups, hipStream_t st, const char *what)
{
    Product pr{a, b, o, ep, M, N, K};
    return launch_products<TIn, TOut>(plan, &pr, 1, groups, st, what);
}

Epilogue epi_store()
{
    Epilogue e{};
    e.mode = EPI_STORE;
    return e;
}

// ---- forward of one layer (Eq. (ylq)) ------------------------------------------------
struct FwdArgs {
    const void *X, *Lw, *Cw, *Dw, *bias, *G;
    void *Y, *g_own, *A_save;
    bool a_f32;   // step only: A_save is float
    bool a_deriv; // step only: A_save receives sigma'(A), in float, instead of A
    bool a_bits;  // step only, ReLU: A_save receives one bit per element (stored output > 0)
    const struct OutputError *mse;   // step only, last layer: form the MSE output error in the update's epilogue
};

// What the last layer's update needs to leave the output error of the MSE loss behind (Epilogue::mse_*), and
// the buffers a thin compression launch before it clears on its way (they are added into from then on;
// clear_count = 0: the caller has cleared them).
struct OutputError {
    const void *target;      // [groups, B, s] storage type
    void *delta;             // [groups, B, s] storage type
    float *partial;          // one partial sum of squares per tile of the update
    float inv_b;
    float *dbias;            // [groups, s], receives the column sums of delta (zero on entry)
    float *clear_at;         // cleared by the compression launch: clear_count floats
    int64_t clear_count;
};

// Does the forward of this geometry run its compression as the thin kernel in a launch of its own before the
// update?  (All ranks on the device, and the conditions of the thin kernel as in fwd_impl.)
bool thin_launch_before_update(const Geo &g)
{
    return g.all && g.dtype == PH_BF16 && g.q > 0 && g.k <= THIN_MAX_N && g.si % 16 == 0 && g.vec > 0;
}

template <typename T>
ph_status fwd_impl(const Geo &g, const FwdArgs &f, hipStream_t st)
{
    const int64_t B = g.B, si = g.si, so = g.so, k = g.k, q = g.q;
    const GemmPlan plan{LD_KC, LD_KC, g.vec, false};
    // compression g = C y: [B, si] x [k, si]^T -> [B, k]
    Product compress{view_plain(f.X, si, B * si), view_plain(f.Cw, si, k * si), view_plain(f.g_own, k, B * k), epi_store(),
                     q > 0 ? B : 0, k, si};
    // local update + decompression + remote update + bias + activation: one product over the
    // concatenated reduction index [y | g_1 .. g_{p-1}] . [L | D_1 .. D_{p-1}]^T
    const void *gathered = g.all ? f.g_own : f.G;
    Product update{};
    update.a = q > 0 ? view_rowseg(f.X, si, (int)si, B * si, gathered, (int)k, B * k, 0, g.all ? 0 : NO_SKIP, g.all ? 1 : 0)
                     : view_plain(f.X, si, B * si);
    update.b = q > 0 ? view_rowseg(f.Lw, si, (int)si, so * si, f.Dw, (int)k, so * k, q * so * k) : view_plain(f.Lw, si, so * si);
    update.o = view_plain(f.Y, so, B * so);
    update.ep.mode = EPI_BIAS_ACT; update.ep.act = g.act; update.ep.bias = f.bias; update.ep.bias_g = so;
    update.ep.aux = f.A_save; update.ep.aux_ld = so; update.ep.aux_g = B * so; update.ep.aux_f32 = f.a_f32; update.ep.aux_deriv = f.a_deriv; update.ep.aux_bits = f.a_bits;
    update.M = B; update.N = so; update.K = g.Kc;
    float *clear_at = nullptr;
    int64_t clear_count = 0;
    if (f.mse) {
        update.ep.mse_target = f.mse->target; update.ep.mse_delta = f.mse->delta; update.ep.mse_partial = f.mse->partial;
        update.ep.mse_inv_b = f.mse->inv_b;
        update.ep.colsum = f.mse->dbias; update.ep.colsum_g = so;
        clear_at = f.mse->clear_at; clear_count = f.mse->clear_count;
    }
    // A compression with few phantom neurons has a kernel of its own (32 rows per workgroup instead of 128)
    bool thin = false;
    if constexpr (std::is_same<T, bf16_t>::value) thin = q > 0 && k <= THIN_MAX_N && si % 16 == 0 && g.vec > 0;
    auto launch_thin = [&]() -> ph_status {
        if constexpr (std::is_same<T, bf16_t>::value) {
            ProfScope prof("compression", B, k, si, g.groups, st);
            dim3 grid((unsigned)((B + THIN_ROWS - 1) / THIN_ROWS), (unsigned)g.groups);
            if (k <= 32)
                hipLaunchKernelGGL((thin_product_kernel<1>), grid, dim3(THIN_WAVES * 64), 0, st, (const __bf16 *)f.X, (const __bf16 *)f.Cw,
                                   (__bf16 *)f.g_own, (int)B, (int)k, (int)si, B * si, k * si, B * k, clear_at, clear_count);
            else
                hipLaunchKernelGGL((thin_product_kernel<2>), grid, dim3(THIN_WAVES * 64), 0, st, (const __bf16 *)f.X, (const __bf16 *)f.Cw,
                                   (__bf16 *)f.g_own, (int)B, (int)k, (int)si, B * si, k * si, B * k, clear_at, clear_count);
            return check_launch("compression");
        }
        return PH_OK;
    };
    if (g.all) {
        // every rank reads the other ranks' g: the compression of all ranks has to finish first
        if (thin) PH_TRY(launch_thin());
        else PH_TRY((launch_products<T, T>(plan, &compress, 1, g.groups, st, "compression")));
        return launch_products<T, T>(plan, &update, 1, g.groups, st, "layer update");
    }
    // one rank: the peers' g are inputs, so the rank's own compression runs beside the update when the two
    // fit the device together
    const int64_t tiles_both = (tiles_of(B, so) + tiles_of(B, k)) * g.groups;
    if (thin && tiles_both > 256) {
        if constexpr (std::is_same<T, bf16_t>::value) {
            static const char *force = tuning_env("PHANTOM_FWD_PAIR");     // =0: two launches (for measurements)
            if (!(force && force[0] == '0'))
                return launch_fwd_pair(update, compress, g.groups, g.vec, st, "layer update + thin compression");
        }
        PH_TRY(launch_thin());
        return launch_products<T, T>(plan, &update, 1, g.groups, st, "layer update");
    }
    Product both[2] = {update, compress};
    return launch_products<T, T>(plan, both, 2, g.groups, st, "layer update + compression", "layer update", "compression");
}

// ---- backward of one layer (Eq. (deltaL), (backprop), (bpb)-(bpD)) ---------------------------
struct BwdArgs {
    const void *dY, *X, *S, *Lw, *Cw, *Dw, *G;
    void *dg_own;
    void *dX;
    float *dLw, *dCw, *dDw, *dbias;
    void *dG_send;
    const void *delta_ready;   // step only: delta already formed (dY, S unused)
    bool dx_S_f32;             // step only: dx_S holds float
    bool dx_S_deriv;           // step only: dx_S holds sigma' itself, in float
    bool dx_S_bits;            // step only, ReLU: dx_S holds one bit per element (the layer below's stored output > 0)
    const void *dx_S;          // step only: multiply dX by sigma'(dx_S) on the way out, which makes it the
                               //   previous layer's delta with a single rounding (Eq. (backprop))
    float *dx_colsum;          // step only: zeroed [groups, s]; the input-gradient product adds the column sums
                               //   of what it stores, i.e. the layer below's bias gradient (Eq. (bpb))
    bool dbias_ready;          // step only: dbias already holds the column sums of delta
    bool dbias_zeroed;         // step only: dbias is zero on entry
    bool send_done;            // step only: this layer's error compression was launched by the layer above (below)
    const void *below_Dw;      // step only, all ranks: D of the layer below; its error compression (dX -> dG_send)
    const Geo *below_g;        //   (that layer's shapes)
    bool *below_done;          //   may then ride with this layer's weight gradients; *below_done says whether it did
    const SgdBatch *ride_sgd;  // step only: the update of the layer above, not launched yet; it may ride with this
    float ride_lr;             //   layer's weight gradients on compute units they leave idle; *ride_sgd_done says
    bool *ride_sgd_done;       //   whether it did
    LossTail *loss_tail;       // step only, last layer: the first memory-bound kernel of this backward finishes
                               //   the loss as a rider and clears loss_tail->partial; left alone if there is none
    void *tap_dG_send;         // step only, optional: copies of this layer's dG_send / (all ranks) dg_own, taken right
    void *tap_dg_own;          //   after the launch that finishes each
    bool defer;                // step only: the weight + compressor gradients are not launched here (the step runs all
                               //   layers' in one launch at the end of the backward pass)
};

// copy of a tensor for a tap of the step (count elements of the storage type)
template <typename T>
ph_status tap_copy(void *dst, const void *src, int64_t count, hipStream_t st)
{
    if (!dst || !src || count <= 0) return PH_OK;
    hipLaunchKernelGGL((copy_kernel<T>), dim3(blocks_for(count)), dim3(256), 0, st, (const T *)src, (T *)dst, count);
    return check_launch("tap copy");
}

// error compression: dG_send[i] = delta . D_i   ([B, so] x [so, k] for every peer, one product over N = q*k);
// w_out, kk: the output width and phantom width of the layer whose delta (dl) and D these are
Product error_compression_product(int64_t B, int64_t q, void *dG_send, const void *dl, const void *Dw, int64_t w_out, int64_t kk)
{
    Product send{};
    send.a = view_plain(dl, w_out, B * w_out);
    send.b.p0 = nullptr; send.b.p1 = const_cast<void *>(Dw); send.b.g0 = 0; send.b.g1 = q * w_out * kk;
    send.b.r = axis_seg(0, (int)kk, 0, 1, w_out * kk); send.b.c = axis_plain(0, kk);
    send.b.skip0 = NO_SKIP; send.b.skip_g = 0;
    send.o.p0 = nullptr; send.o.p1 = dG_send; send.o.g0 = 0; send.o.g1 = q * B * kk;
    send.o.r = axis_plain(0, kk); send.o.c = axis_seg(0, (int)kk, 0, 1, B * kk);
    send.o.skip0 = NO_SKIP; send.o.skip_g = 0;
    send.ep = epi_store();
    send.M = q > 0 ? B : 0; send.N = q * kk; send.K = w_out;
    return send;
}

// The four products of a layer's backward pass (Eq. (backprop), (bpL)-(bpD)) from its local error delta.
struct BwdProducts {
    Product send, dx, dw, dc;
};

BwdProducts make_bwd_products(const Geo &g, const BwdArgs &b, const void *delta)
{
    const int64_t B = g.B, si = g.si, so = g.so, k = g.k, q = g.q;
    BwdProducts pr{};
    pr.send = error_compression_product(B, q, b.dG_send, delta, b.Dw, so, k);

    // dX = delta . L + dg_own . C: reduction index = [delta | dg_own] against [L ; C]
    Product &dx = pr.dx;
    dx.a = q > 0 ? view_rowseg(delta, so, (int)so, B * so, b.dg_own, (int)k, 0, B * k) : view_plain(delta, so, B * so);
    dx.b = q > 0 ? view_colstack(b.Lw, si, (int)so, so * si, b.Cw, si, (int)k, k * si) : view_plain_t(b.Lw, si, so * si);
    dx.o = view_plain(b.dX, si, B * si);
    dx.ep = epi_store();
    if (b.dx_S && g.act != PH_ACT_IDENTITY) {
        dx.ep.mode = EPI_DACT; dx.ep.act = g.act; dx.ep.aux = const_cast<void *>(b.dx_S); dx.ep.aux_ld = si;
        dx.ep.aux_g = B * si; dx.ep.aux_f32 = b.dx_S_f32; dx.ep.aux_deriv = b.dx_S_deriv; dx.ep.aux_bits = b.dx_S_bits;
    } else if (b.dx_colsum) {
        dx.ep.mode = EPI_DACT; dx.ep.act = g.act; dx.ep.aux = nullptr;      // identity: column sums only
    }
    dx.ep.colsum = b.dx_colsum; dx.ep.colsum_g = si;
    dx.M = b.dX ? B : 0; dx.N = si; dx.K = so + k;

    // weight gradients: [dL | dD_1 .. dD_{p-1}] = delta^T . [X | G_1 .. G_{p-1}], and dC = dg_own^T . X beside it
    Product &dw = pr.dw;
    dw.a = view_plain_t(delta, so, B * so);
    dw.b = q > 0 ? view_rowseg_t(b.X, si, (int)si, B * si, b.G, (int)k, B * k, 0, g.all ? 0 : NO_SKIP, g.all ? 1 : 0)
                 : view_plain_t(b.X, si, B * si);
    dw.o.p0 = b.dLw; dw.o.p1 = b.dDw; dw.o.g0 = so * si; dw.o.g1 = q * so * k;
    dw.o.r = axis_plain(si, k);
    dw.o.c = q > 0 ? axis_seg((int)si, (int)k, 1, 1, so * k) : axis_plain(1, 0);
    dw.o.skip0 = NO_SKIP; dw.o.skip_g = 0;
    dw.ep = epi_store();
    dw.M = so; dw.N = g.Kc; dw.K = B;
    pr.dc = Product{view_plain_t(b.dg_own, k, B * k), view_plain_t(b.X, si, B * si), view_plain(b.dCw, si, k * si), epi_store(),
                    q > 0 ? k : 0, si, B};
    return pr;
}

template <typename T>
ph_status bwd_impl(const Geo &g, const BwdArgs &b, const BwdWs &w, hipStream_t st)
{
    const int64_t B = g.B, so = g.so, k = g.k, q = g.q;
    const int64_t act_count = (int64_t)g.groups * B * so;

    // local error delta = dY * sigma'
    const void *delta = b.delta_ready;
    if (!delta) {
        ProfScope prof("local error", 0, act_count, 0, 1, st);
        hipLaunchKernelGGL((delta_kernel<T>), dim3(blocks_for(act_count)), dim3(256), 0, st,
                           (const T *)b.dY, (const T *)b.S, (T *)w.delta, act_count, g.act);
        PH_TRY(check_launch("local error"));
        delta = w.delta;
    }

    // the loss rider goes to the first launch that can carry it
    auto take_tail = [&]() {
        LossTail t{};
        if (b.loss_tail) { t = *b.loss_tail; b.loss_tail->partial = nullptr; }
        return t;
    };

    // bias gradient: column sums of delta
    {
        const int strips = (int)((so + CSUM_COLS - 1) / CSUM_COLS);
        // enough workgroups to pull the whole tensor at memory speed: split the rows when the strips are few
        int chunks = (int)std::max<int64_t>(1, std::min<int64_t>(256 / ((int64_t)strips * g.groups), B / 128));
        if (g.dtype == PH_F32) chunks = 1;      // the fp32 path keeps a fixed summation order
        const int rows_per_chunk = (int)((B + chunks - 1) / chunks);
        chunks = (int)((B + rows_per_chunk - 1) / rows_per_chunk);
        if (chunks > 1 && !b.dbias_zeroed && !b.dbias_ready) {
            ProfScope prof("clear bias gradient", 0, (int64_t)g.groups * so, 0, 1, st);
            hipLaunchKernelGGL(fill_zero_kernel, dim3(blocks_for((int64_t)g.groups * so)), dim3(256), 0, st, b.dbias,
                               (int64_t)g.groups * so);
            PH_TRY(check_launch("clear bias gradient"));
        }
        if (!b.dbias_ready) {
            dim3 grid((unsigned)strips, (unsigned)g.groups, (unsigned)chunks);
            ProfScope prof("bias gradient", 0, act_count, 0, 1, st);
            hipLaunchKernelGGL((colsum_kernel<T>), grid, dim3(256), 0, st, (const T *)delta, b.dbias, (int)B, (int)so,
                               rows_per_chunk, take_tail());
            PH_TRY(check_launch("bias gradient"));
        }
    }

    BwdProducts pr = make_bwd_products(g, b, delta);
    const Product &send = pr.send, &dw = pr.dw, &dc = pr.dc;
    Product &dx = pr.dx;
    auto error_compression = [&](const void *dl, const void *Dw, int64_t w_out, int64_t kk) {
        return error_compression_product(B, q, b.dG_send, dl, Dw, w_out, kk);
    };
    // Riders of the weight-gradient launch (MfmaTailBatch) exist on the matrix-core path for launches of at most one
    // tile per compute unit.  PHANTOM_TAIL=0 switches them off (for measurements).
    const int64_t tail_tiles = (tiles_of(dw.M, dw.N) + tiles_of(dc.M, dc.N)) * g.groups;
    static const char *tail_force = tuning_env("PHANTOM_TAIL");
    const bool riders = std::is_same<T, bf16_t>::value && g.vec > 0 && tail_tiles <= 256 && !(tail_force && tail_force[0] == '0');
    // One rank, no input gradient wanted (the first layer): this layer's error compression has no launch to share
    // with the input gradient and nothing waits for it, so it rides with the weight gradients.
    const bool send_rides = riders && !g.all && !b.dX && q > 0 && !b.defer;

    const GemmPlan plan_x{LD_KC, LD_KM, g.vec, false};
    const int64_t send_count = (int64_t)g.groups * q * B * k;
    if (g.all) {
        // the input gradient needs dg_own, which is the sum of what all ranks send: three launches
        if (!b.send_done) PH_TRY((launch_products<T, T>(plan_x, &send, 1, g.groups, st, "error compression")));
        PH_TRY(tap_copy<T>(b.tap_dG_send, b.dG_send, send_count, st));
        // Reduce-scatter as a sum on read: the input gradient's loader sums the p-1 senders' slices while it stages
        // the one reduction tile that holds dg_own, and writes dg_own out for the compressor gradient.  Conditions:
        // the block starts on a tile boundary of the reduction index and fits one tile (so a multiple of 64,
        // k a divisor of 64), 16-byte vectors, and at most 8 ranks: a thread has the loads of seven senders
        // in flight at a time, and with 16 ranks the step got 0.4 % slower instead of 1.8 % faster.  PHANTOM_RS_ON_READ=0 keeps the kernel of its own (for measurements).
        static const char *rs_force = tuning_env("PHANTOM_RS_ON_READ");
        const bool sum_on_read = std::is_same<T, bf16_t>::value && g.vec == 8 && q > 0 && b.dX && g.p <= 8 && k <= KT &&
                                 KT % k == 0 && so % KT == 0 && !(rs_force && rs_force[0] == '0');
        if (sum_on_read) {
            dx.rs.src = (const __bf16 *)b.dG_send; dx.rs.out = (__bf16 *)b.dg_own;
            dx.rs.per_slot = B * k; dx.rs.p = (int)g.p; dx.rs.k = (int)k;
        } else if (q > 0) {
            const int64_t per_slot = B * k;
            constexpr int RS_VEC = 16 / (int)sizeof(T);
            const bool wide = per_slot % RS_VEC == 0 && (((uintptr_t)b.dG_send | (uintptr_t)b.dg_own) & 15) == 0;
            const int64_t per_wg = 32 * (wide ? RS_VEC : 1);
            dim3 grid((unsigned)((per_slot + per_wg - 1) / per_wg), (unsigned)g.p);
            ProfScope prof("reduce-scatter", 0, per_slot * g.p * (g.p - 1), 0, 1, st);
            if (wide)
                hipLaunchKernelGGL((reduce_scatter_kernel<T, RS_VEC>), grid, dim3(256), 0, st, (const T *)b.dG_send,
                                   (T *)b.dg_own, (int)g.p, per_slot, take_tail());
            else
                hipLaunchKernelGGL((reduce_scatter_kernel<T, 1>), grid, dim3(256), 0, st, (const T *)b.dG_send,
                                   (T *)b.dg_own, (int)g.p, per_slot, take_tail());
            PH_TRY(check_launch("reduce-scatter"));
        }
        PH_TRY((launch_products<T, T>(plan_x, &dx, 1, g.groups, st, "input gradient")));
        PH_TRY(tap_copy<T>(b.tap_dg_own, b.dg_own, (int64_t)g.groups * B * k, st));
    } else if (!send_rides) {
        Product both[2] = {dx, send};
        PH_TRY((launch_products<T, T>(plan_x, both, 2, g.groups, st, "input gradient + error compression",
                                      "input gradient", "error compression")));
        PH_TRY(tap_copy<T>(b.tap_dG_send, b.dG_send, send_count, st));
    }

    Product grads[2] = {dw, dc};
    if (b.below_done) *b.below_done = false;
    if (b.ride_sgd_done) *b.ride_sgd_done = false;
    if (b.defer) return PH_OK;
    if constexpr (std::is_same<T, bf16_t>::value) {
        if (riders) {
            // The layer below starts its backward with an error compression that fills half of the device or less
            // for a short while: it comes along when it leaves at least half of the compute units to the weight
            // gradients from the start (they take over the rest as it finishes).  The update of the layer above
            // comes along when at least a quarter of the compute units would otherwise be idle.
            Product below{};
            bool with_head = false;
            int64_t used = tail_tiles;
            int vec = g.vec;
            if (send_rides) {
                below = send;
                with_head = true;
                used += (tiles_of(below.M, below.N) * g.groups + 7) & ~(int64_t)7;
            } else if (b.below_Dw && b.below_g && b.below_g->vec > 0 && b.dX && g.all && q > 0) {
                below = error_compression(b.dX, b.below_Dw, b.below_g->so, b.below_g->k);
                vec = std::min(vec, b.below_g->vec);
                const int64_t head_tiles = tiles_of(below.M, below.N) * g.groups;
                with_head = head_tiles <= 128;
                if (with_head) used += (head_tiles + 7) & ~(int64_t)7;
            }
            const int64_t idle = 256 - ((used + 7) & ~(int64_t)7);      // negative: the launch runs in rounds
            // (a launch that runs in rounds anyway takes the update along on a quarter of the compute units: its
            // workgroups go out before the error compression, which fills in as compute units come free)
            const bool rounds = send_rides && used > 256;
            const bool with_sgd = b.ride_sgd && (idle >= 64 || rounds);
            // a loss that no kernel has finished yet (and no update to carry it): one more workgroup does it
            const bool with_loss = !with_sgd && !b.ride_sgd && b.loss_tail && b.loss_tail->partial;
            if (with_head || with_sgd || with_loss) {
                SgdBatch loss_only{};
                if (with_loss) loss_only.tail = take_tail();
                PH_TRY(launch_tail(with_head ? &below : nullptr, dw, dc, with_sgd ? b.ride_sgd : with_loss ? &loss_only : nullptr,
                                   b.ride_lr, with_sgd ? (int)std::max<int64_t>(idle, 64) : 1, g.groups, vec, st,
                                   send_rides ? (with_sgd ? "weight + compressor gradients | error compression | SGD above"
                                                          : "weight + compressor gradients | error compression")
                                   : with_head ? (with_sgd ? "weight + compressor gradients | error compr. below | SGD above"
                                                           : "weight + compressor gradients | error compression below")
                                               : with_sgd ? "weight + compressor gradients | SGD above"
                                                          : "weight + compressor gradients | loss",
                                   rounds));
                if (b.below_done) *b.below_done = with_head && !send_rides;
                if (b.ride_sgd_done) *b.ride_sgd_done = with_sgd;
                if (send_rides) PH_TRY(tap_copy<T>(b.tap_dG_send, b.dG_send, send_count, st));
                return PH_OK;
            }
        }
    }
    // a lone weight-gradient product with few tiles may split its reduction; a pair never does
    // (send_rides never gets here: its launch above carries the error compression)
    return launch_products<T, float>(GemmPlan{LD_KM, LD_KM, g.vec, true}, grads, q > 0 ? 2 : 1, g.groups, st,
                                     "weight + compressor gradients", "weight gradients", "compressor gradient");
}

ph_status check_fwd_args(const Geo &g, const FwdArgs &f)
{
    PH_TRY(need(f.X, "X")); PH_TRY(need(f.Lw, "Lw")); PH_TRY(need(f.bias, "bias")); PH_TRY(need(f.Y, "Y"));
    PH_TRY(optional(f.A_save, "A_save"));
    if (g.q > 0) {
        PH_TRY(need(f.Cw, "Cw")); PH_TRY(need(f.Dw, "Dw")); PH_TRY(need(f.g_own, "g_own"));
        if (!g.all) PH_TRY(need(f.G, "G"));
    }
    return PH_OK;
}

ph_status check_bwd_args(const Geo &g, const BwdArgs &b)
{
    PH_TRY(need(b.dY, "dY")); PH_TRY(need(b.X, "X")); PH_TRY(need(b.Lw, "Lw"));
    if (g.act != PH_ACT_IDENTITY) PH_TRY(need(b.S, "A_or_Y"));
    PH_TRY(optional(b.dX, "dX"));
    PH_TRY(need(b.dLw, "dLw")); PH_TRY(need(b.dbias, "dbias"));
    if (g.q > 0) {
        PH_TRY(need(b.Cw, "Cw")); PH_TRY(need(b.Dw, "Dw")); PH_TRY(need(b.G, "G")); PH_TRY(need(b.dg_own, "dg_own"));
        PH_TRY(need(b.dCw, "dCw")); PH_TRY(need(b.dDw, "dDw")); PH_TRY(need(b.dG_send, "dG_send"));
    }
    return PH_OK;
}

ph_status check_ws(void *ws, size_t have, size_t want)
{
    if (want == 0) return PH_OK;
    if (!ws) return fail(PH_ERR_WORKSPACE, "workspace is NULL, %zu bytes needed", want);
    if ((uintptr_t)ws & 255) return fail(PH_ERR_WORKSPACE, "workspace is not 256-byte aligned");
    if (have < want) return fail(PH_ERR_WORKSPACE, "workspace has %zu bytes, %zu needed", have, want);
    return PH_OK;
}

template <typename T>
ph_status step_impl(const std::vector<Geo> &geos, const ph_step_args &a, const StepWs &w, hipStream_t st)
{
    const Geo &g = geos.back();       // the last layer; what does not depend on the layer is read from it
    const int L = g.layers;
    const int64_t B = g.B, q = g.q;
    const int64_t act_count = (int64_t)g.groups * B * g.so;      // elements of the network output

    // What the backward pass needs of a layer's pre-activation A is sigma'(A) alone.  ReLU reads it off the
    // layer's output.  GELU in bf16 storage has the forward epilogue, which evaluates erf and exp for
    // sigma(A) anyway, store sigma'(A) in float: the bytes of an fp32 A and no second evaluation in the
    // input-gradient epilogue.  (Any coarser grid for that factor moves delta across bf16 rounding
    // boundaries often enough to show after a few layers.)  fp32 storage keeps A itself.
    const bool gelu = g.act == PH_ACT_GELU;
    const bool save_deriv = gelu && std::is_same<T, bf16_t>::value;

    // Bias gradients (Eq. (bpb)) are column sums of delta.  On the MFMA path the product that writes a
    // layer's delta (the input gradient of the layer above; for the last layer its own update, see below)
    // adds them up on its way out, so every layer's bias gradient has a buffer of its own that is zeroed once
    // for the whole step: the caller's buffers by launches of their own, the workspace's (one block) by a
    // kernel that runs anyway.
    const bool train = a.mode != PH_STEP_FORWARD;
    auto on_mfma = [&](int l) { return std::is_same<T, bf16_t>::value && geos[(size_t)l].vec > 0; };
    auto dbias_of = [&](int l) { return a.dbias ? a.dbias[l] : w.dbias + w.dbias_at[(size_t)l]; };
    if (train && a.dbias) {
        for (int l = 0; l < L; ++l) {
            const int64_t bias_count = (int64_t)g.groups * geos[(size_t)l].so;
            hipLaunchKernelGGL(fill_zero_kernel, dim3(blocks_for(bias_count)), dim3(256), 0, st, a.dbias[l], bias_count);
            PH_TRY(check_launch("clear bias gradients"));
        }
    }
    // (the words for cut reductions lie right behind the workspace's block and are cleared with it)
    float *clear_at = a.dbias ? (float *)w.arrived : w.dbias;
    const int64_t clear_count = a.dbias ? PIECE_WORDS : w.dbias_at[(size_t)L] + PIECE_WORDS;

    // The output error of the MSE loss (Eq. (deltaL)) is elementwise in the last layer's output, so on the MFMA
    // path that layer's update forms it in its epilogue, together with the last bias gradient and one partial
    // sum of the loss per tile: two launches less than a kernel for the error and one for the column sums.
    // The buffers it adds into have to be clear by then: the thin compression launch right before it does that
    // on its way where there is one, else a launch of its own at the start of the step.
    const int64_t out_tiles = tiles_of(B, g.so) * g.groups;
    const bool mse_in_update = train && on_mfma(L - 1) && out_tiles <= MSE_BLOCKS;
    const bool clear_in_compression = mse_in_update && thin_launch_before_update(g);
    // (one rank with deferred weight gradients keeps every layer's delta: the last layer's goes to its own buffer)
    bool deferred = false;
    if constexpr (std::is_same<T, bf16_t>::value) deferred = mse_in_update && w.table && deferred_weight_gradients(geos);
    if (mse_in_update && !clear_in_compression && !deferred && clear_count > 0) {
        ProfScope prof("clear bias gradients", 0, clear_count, 0, 1, st);
        hipLaunchKernelGGL(fill_zero_kernel, dim3(blocks_for(clear_count)), dim3(256), 0, st, clear_at, clear_count);
        PH_TRY(check_launch("clear bias gradients"));
    }
    void *delta_top = deferred ? w.delta_of[(size_t)L - 1] : w.dYa;
    OutputError oe{a.T, delta_top, w.mse_partial, 1.0f / (float)B, dbias_of(L - 1), clear_in_compression ? clear_at : nullptr,
                   clear_in_compression ? clear_count : 0};

    // Deferred weight gradients: the products of all layers are known from the buffers alone.  Their parameter table
    // goes up now, ahead of the forward pass (the first of those small launches also clears what the step adds
    // into), and the launch itself comes at the end of the backward pass: the compressor gradients first (few
    // tiles with half of their rows empty, cut into pieces), then the weight gradients' tiles, which fill the compute
    // units as those come free; the SGD update of L, C, D and the bias in the epilogues, the loss by the first workgroup.
    int table_grid = 0;
    Product table_dw{}, table_dc{};
    if (deferred) {
        const bool update = a.mode != PH_STEP_NO_UPDATE;
        std::vector<Product> later;
        std::vector<int> splits;
        std::vector<SgdInPlace> inside;
        for (int pass = 0; pass < 2; ++pass)
            for (int l = L - 1; l >= 0; --l) {
                const Geo &gl = geos[(size_t)l];
                BwdArgs b{};
                b.X = l > 0 ? w.Y[l - 1] : a.X0;
                b.G = q ? a.G[l] : nullptr;
                b.dg_own = q ? const_cast<void *>(a.dg_own[l]) : nullptr;
                // (gradients that the caller does not want: a training step has the update in the epilogues and stores
                // none; a step without update stores every layer's in the same place, where nobody reads them)
                b.dLw = a.dLw ? a.dLw[l] : w.dLw[0];
                b.dCw = q ? (a.dCw ? a.dCw[l] : w.dCw[0]) : nullptr;
                b.dDw = q ? (a.dDw ? a.dDw[l] : w.dDw[0]) : nullptr;
                const BwdProducts all = make_bwd_products(gl, b, w.delta_of[(size_t)l]);
                const Product &pr = pass ? all.dw : all.dc;
                if (l == L - 1) (pass ? table_dw : table_dc) = pr;
                if (pr.M <= 0 || pr.N <= 0) continue;
                SgdInPlace in{};
                if (update && pass)
                    in = SgdInPlace{a.Lw_master[l], q ? a.Dw_master[l] : nullptr, (__bf16 *)a.Lw[l], q ? (__bf16 *)a.Dw[l] : nullptr, a.lr,
                                    (a.dLw || a.dDw) ? 1 : 0, a.bias_master[l], (__bf16 *)a.bias[l], dbias_of(l)};
                if (update && !pass)
                    in = SgdInPlace{a.Cw_master[l], nullptr, (__bf16 *)a.Cw[l], nullptr, a.lr, a.dCw ? 1 : 0, nullptr, nullptr, nullptr};
                later.push_back(pr);
                splits.push_back(pass ? 1 : compressor_gradient_pieces(gl));
                inside.push_back(in);
            }
        const LossTail tail{w.mse_partial, (int)out_tiles, 0.5f / (float)B, a.loss};
        PH_TRY(upload_product_table(later, splits, inside, w.table, w.parts, w.arrived, tail, clear_at, clear_count, st, &table_grid));
    }

    // forward through every layer; y_l stays in the storage type between layers
    const void *in = a.X0;
    std::vector<const void *> inputs(L);
    for (int l = 0; l < L; ++l) {
        inputs[l] = in;
        const bool bits = train && w.relu_bits[(size_t)l] != nullptr;
        FwdArgs f{in, a.Lw[l], q ? a.Cw[l] : nullptr, q ? a.Dw[l] : nullptr, a.bias[l],
                  (q && !g.all) ? a.G[l] : nullptr, w.Y[l], w.G[l], bits ? w.relu_bits[(size_t)l] : w.A[l],
                  !save_deriv && !bits, save_deriv, bits, (mse_in_update && l == L - 1) ? &oe : nullptr};
        PH_TRY(fwd_impl<T>(geos[(size_t)l], f, st));
        in = w.Y[l];
        if (a.taps) {
            const Geo &gl = geos[(size_t)l];
            if (a.taps->Y) PH_TRY(tap_copy<T>(a.taps->Y[l], w.Y[l], (int64_t)gl.groups * B * gl.so, st));
            if (a.taps->g_own && q) PH_TRY(tap_copy<T>(a.taps->g_own[l], w.G[l], (int64_t)gl.groups * B * gl.k, st));
        }
    }
    if (a.Y_out) {
        hipLaunchKernelGGL((copy_kernel<T>), dim3(blocks_for(act_count)), dim3(256), 0, st, (const T *)w.Y[L - 1],
                           (T *)a.Y_out, act_count);
        PH_TRY(check_launch("output copy"));
    }
    if (!train) return PH_OK;

    // The loss is the sum of partial sums that the output-error computation leaves; the first memory-bound
    // kernel after it adds them up as a rider (LossTail), a kernel of its own if there is none.
    LossTail loss_tail{w.mse_partial, (int)out_tiles, 0.5f / (float)B, a.loss};
    if (!mse_in_update) {
        // output error as a kernel of its own; it also clears the workspace's bias-gradient block
        const void *S = gelu ? w.A[L - 1] : w.Y[L - 1];
        const int s_kind = save_deriv ? 2 : (gelu ? 1 : 0);
        const bool wide = act_count % 8 == 0 && (((uintptr_t)a.T | (uintptr_t)w.Y[L - 1] | (uintptr_t)S | (uintptr_t)w.dYa) & 31) == 0;
        const unsigned mse_blocks = blocks_for(wide ? act_count / 8 : act_count, 256, MSE_BLOCKS);
        loss_tail.n = (int)mse_blocks;
        ProfScope prof("output error", 0, act_count, 0, 1, st);
        if (wide)
            hipLaunchKernelGGL((mse_delta_kernel<T, 8>), dim3(mse_blocks), dim3(256), 0, st, (const T *)w.Y[L - 1],
                               (const T *)a.T, S, s_kind, (T *)w.dYa, act_count, 1.0f / (float)B, g.act,
                               w.mse_partial, clear_at, clear_count);
        else
            hipLaunchKernelGGL((mse_delta_kernel<T, 1>), dim3(mse_blocks), dim3(256), 0, st, (const T *)w.Y[L - 1],
                               (const T *)a.T, S, s_kind, (T *)w.dYa, act_count, 1.0f / (float)B, g.act,
                               w.mse_partial, clear_at, clear_count);
        PH_TRY(check_launch("output error"));
    }

    if (a.taps && a.taps->delta) PH_TRY(tap_copy<T>(a.taps->delta[L - 1], delta_top, act_count, st));   // delta_L, Eq. (deltaL)

    void *dY = w.dYa, *dX = w.dYb;    // delta of the current layer / of the layer below
    bool send_done = false;           // the current layer's error compression went out with the layer above
    SgdBatch pending{};               // the update of the layer above, if it has not been launched yet
    int64_t pending_elems = 0, pending_largest = 0;
    bool have_pending = false;
    auto launch_sgd = [&](const SgdBatch &batch, int tensors, int64_t largest, int64_t total) -> ph_status {
        ProfScope prof("SGD update", 0, total, 0, 1, st);
        hipLaunchKernelGGL((sgd_kernel<T>), dim3(blocks_for(largest, 256, 2048), (unsigned)tensors), dim3(256), 0, st, batch, a.lr);
        return check_launch("SGD update");
    };
    for (int l = L - 1; l >= 0; --l) {
        BwdArgs b{};
        b.send_done = send_done;
        b.below_Dw = (g.all && q > 0 && l > 0) ? a.Dw[l - 1] : nullptr;
        b.below_g = l > 0 ? &geos[(size_t)l - 1] : nullptr;
        b.below_done = &send_done;
        b.dbias_zeroed = true;
        b.loss_tail = &loss_tail;
        // the layer's bias gradient is there already if the product that wrote its delta took the column sums
        b.dbias_ready = l < L - 1 ? on_mfma(l + 1) : mse_in_update;
        b.dx_colsum = (on_mfma(l) && l > 0) ? dbias_of(l - 1) : nullptr;
        if (deferred) { dY = w.delta_of[(size_t)l]; dX = l > 0 ? w.delta_of[(size_t)l - 1] : nullptr; b.defer = true; b.loss_tail = nullptr; }
        b.delta_ready = dY; b.X = inputs[l];
        b.dx_S_bits = l > 0 && w.relu_bits[(size_t)l - 1] != nullptr;
        b.dx_S = l > 0 ? (b.dx_S_bits ? w.relu_bits[(size_t)l - 1] : g.act == PH_ACT_GELU ? w.A[l - 1] : w.Y[l - 1]) : nullptr;
        b.dx_S_f32 = gelu && !save_deriv;
        b.dx_S_deriv = save_deriv;
        b.Lw = a.Lw[l]; b.Cw = q ? a.Cw[l] : nullptr; b.Dw = q ? a.Dw[l] : nullptr;
        b.G = q ? (g.all ? w.G[l] : a.G[l]) : nullptr;
        b.dg_own = q ? (g.all ? w.dg_own : const_cast<void *>(a.dg_own[l])) : nullptr;
        b.dX = l > 0 ? dX : nullptr;
        b.dLw = a.dLw ? a.dLw[l] : w.dLw[l & 1];
        b.dCw = q ? (a.dCw ? a.dCw[l] : w.dCw[l & 1]) : nullptr;
        b.dDw = q ? (a.dDw ? a.dDw[l] : w.dDw[l & 1]) : nullptr;
        b.dbias = dbias_of(l);
        b.dG_send = w.dG_send;
        bool sgd_rode = false;
        b.ride_sgd = have_pending ? &pending : nullptr;
        b.ride_lr = a.lr;
        b.ride_sgd_done = &sgd_rode;
        const Geo &gl = geos[(size_t)l];
        const int64_t si = gl.si, so = gl.so, k = gl.k;
        if (a.taps) {
            b.tap_dG_send = (a.taps->dG_send && q) ? a.taps->dG_send[l] : nullptr;
            b.tap_dg_own = (a.taps->dg_own && q && g.all) ? a.taps->dg_own[l] : nullptr;
        }
        PH_TRY(bwd_impl<T>(gl, b, w.bwd, st));
        // what the input gradient's epilogue left in dX is delta_{l-1} (Eq. (backprop), sigma' applied)
        if (a.taps && a.taps->delta && l > 0) PH_TRY(tap_copy<T>(a.taps->delta[l - 1], dX, (int64_t)g.groups * B * si, st));
        if (have_pending && !sgd_rode) PH_TRY(launch_sgd(pending, 4, pending_largest, pending_elems));
        have_pending = false;
        if (deferred) continue;

        if (a.mode == PH_STEP_NO_UPDATE) {
            if (loss_tail.partial) {                   // no kernel of this layer's backward could carry the rider
                ProfScope prof("loss", 0, loss_tail.n, 0, 1, st);
                hipLaunchKernelGGL(loss_kernel, dim3(1), dim3(256), 0, st, loss_tail);
                PH_TRY(check_launch("loss"));
                loss_tail.partial = nullptr;
            }
            void *t = dY; dY = dX; dX = t;
            continue;
        }
        // SGD on this layer: nothing later in the backward pass reads its weights
        struct Upd { void *w; float *master; const float *grad; int64_t count; };
        Upd upd[4] = {
            {a.Lw[l], a.Lw_master ? a.Lw_master[l] : nullptr, b.dLw, (int64_t)g.groups * so * si},
            {a.bias[l], a.bias_master ? a.bias_master[l] : nullptr, b.dbias, (int64_t)g.groups * so},
            {q ? a.Cw[l] : nullptr, (q && a.Cw_master) ? a.Cw_master[l] : nullptr, b.dCw, (int64_t)g.groups * k * si},
            {q ? a.Dw[l] : nullptr, (q && a.Dw_master) ? a.Dw_master[l] : nullptr, b.dDw, (int64_t)g.groups * q * so * k},
        };
        SgdBatch batch{};
        int tensors = 0;
        int64_t largest = 0, total = 0;
        for (const Upd &u : upd) {
            if (!u.w || u.count == 0) continue;
            batch.t[tensors++] = SgdTensor{u.w, u.master, u.grad, u.count};
            largest = std::max(largest, u.count);
            total += u.count;
        }
        if (tensors > 0) {
            batch.tail = loss_tail;                    // still set: no kernel of this layer's backward carried the rider
            loss_tail.partial = nullptr;
            // The update may wait for the weight-gradient launch of the layer below and use the compute units
            // that launch leaves idle (bwd_impl decides); the first layer's has nothing to wait for.
            if (l > 0 && on_mfma(l - 1)) {
                pending = batch;
                pending_elems = total;
                pending_largest = largest;
                have_pending = true;
            } else {
                PH_TRY(launch_sgd(batch, tensors, largest, total));
            }
        }
        void *t = dY; dY = dX; dX = t;
    }
    if (deferred)
        PH_TRY(launch_product_table(w.table, table_grid, st,
                                    a.mode != PH_STEP_NO_UPDATE ? "weight + compressor gradients of all layers + SGD | loss"
                                                                : "weight + compressor gradients of all layers | loss",
                                    table_dw, table_dc, L));
    return PH_OK;
}

ph_status check_ptr_array(const void *const *arr, int L, const char *name)
{
    if (!arr) return fail(PH_ERR_INVALID_ARG, "%s (host array of device pointers) is NULL", name);
    for (int l = 0; l < L; ++l) {
        char nm[64];
        snprintf(nm, sizeof nm, "%s[%d]", name, l);
        PH_TRY(need(arr[l], nm));
    }
    return PH_OK;
}

}  // namespace

extern "C" {

int32_t phantom_abi_version(void) { return 4; }

ph_status phantom_profile_begin(int32_t max_launches)
{
    if (max_launches < 1) return fail(PH_ERR_INVALID_ARG, "max_launches = %d must be >= 1", max_launches);
    if (g_prof.on) return fail(PH_ERR_INVALID_ARG, "profiling is already on");
    max_launches += PROF_CALIBRATION_LAUNCHES;
    while (g_prof.ev.size() < (size_t)max_launches * 2) {
        hipEvent_t e;
        hipError_t err = hipEventCreate(&e);
        if (err != hipSuccess) return fail(PH_ERR_LAUNCH, "hipEventCreate: %s", hipGetErrorString(err));
        g_prof.ev.push_back(e);
    }
    g_prof.recs.clear();
    g_prof.cap = (size_t)max_launches;
    g_prof.calibrated = false;
    g_prof.on = true;
    return PH_OK;
}

ph_status phantom_profile_end(ph_profile_entry *entries, int32_t capacity, int32_t *count)
{
    if (!g_prof.on) return fail(PH_ERR_INVALID_ARG, "profiling is not on");
    g_prof.on = false;
    if (!count || (capacity > 0 && !entries)) return fail(PH_ERR_INVALID_ARG, "entries / count is NULL");
    int32_t used = 0;
    for (size_t i = 0; i < g_prof.recs.size(); ++i) {
        const ProfRec &r = g_prof.recs[i];
        hipError_t err = hipEventSynchronize(g_prof.ev[2 * i + 1]);
        float ms = 0.f;
        if (err == hipSuccess) err = hipEventElapsedTime(&ms, g_prof.ev[2 * i], g_prof.ev[2 * i + 1]);
        if (err != hipSuccess) return fail(PH_ERR_LAUNCH, "profile event %zu: %s", i, hipGetErrorString(err));
        int32_t at = -1;
        for (int32_t j = 0; j < used && at < 0; ++j)
            if (!strncmp(entries[j].name, r.name, sizeof entries[j].name - 1) && entries[j].M == r.M &&
                entries[j].N == r.N && entries[j].K == r.K && entries[j].groups == r.groups && entries[j].M2 == r.M2 &&
                entries[j].N2 == r.N2 && entries[j].K2 == r.K2 && entries[j].M3 == r.M3 && entries[j].N3 == r.N3 &&
                entries[j].K3 == r.K3 && entries[j].M4 == r.M4 && entries[j].N4 == r.N4 && entries[j].K4 == r.K4)
                at = j;
        if (at < 0) {
            if (used >= capacity) continue;
            at = used++;
            memset(&entries[at], 0, sizeof entries[at]);
            strncpy(entries[at].name, r.name, sizeof entries[at].name - 1);
            entries[at].M = r.M; entries[at].N = r.N; entries[at].K = r.K; entries[at].groups = r.groups;
            entries[at].M2 = r.M2; entries[at].N2 = r.N2; entries[at].K2 = r.K2;
            entries[at].M3 = r.M3; entries[at].N3 = r.N3; entries[at].K3 = r.K3;
            entries[at].M4 = r.M4; entries[at].N4 = r.N4; entries[at].K4 = r.K4;
        }
        entries[at].calls += 1;
        entries[at].total_ms += ms;
    }
    *count = used;
    return PH_OK;
}

const char *phantom_last_error(void) { return g_err.c_str(); }

ph_status phantom_workspace_bytes(const ph_problem *prob, size_t *bytes)
{
    std::vector<Geo> geos;
    PH_TRY(make_geos(prob, geos));
    if (!bytes) return fail(PH_ERR_INVALID_ARG, "bytes is NULL");
    Arena a{nullptr, 0};
    carve_step(a, geos);       // the step's layout contains the backward's; the forward needs none
    *bytes = a.used + 256;
    return PH_OK;
}

ph_status phantom_layer_fwd(const ph_problem *prob, const void *X, const void *Lw, const void *Cw, const void *Dw,
                            const void *bias, const void *G, void *Y, void *g_own, void *A_save,
                            void *workspace, size_t workspace_bytes, void *hip_stream)
{
    (void)workspace; (void)workspace_bytes;
    Geo g;
    PH_TRY(make_geo(prob, g));
    FwdArgs f{};
    f.X = X; f.Lw = Lw; f.Cw = Cw; f.Dw = Dw; f.bias = bias; f.G = G; f.Y = Y; f.g_own = g_own; f.A_save = A_save;
    PH_TRY(check_fwd_args(g, f));
    hipStream_t st = (hipStream_t)hip_stream;
    return g.dtype == PH_F32 ? fwd_impl<float>(g, f, st) : fwd_impl<bf16_t>(g, f, st);
}

ph_status phantom_layer_bwd(const ph_problem *prob, const void *dY, const void *X, const void *A_or_Y,
                            const void *Lw, const void *Cw, const void *Dw, const void *G, void *dg_own,
                            void *dX, float *dLw, float *dCw, float *dDw, float *dbias, void *dG_send,
                            void *workspace, size_t workspace_bytes, void *hip_stream)
{
    Geo g;
    PH_TRY(make_geo(prob, g));
    BwdArgs b{};
    b.dY = dY; b.X = X; b.S = A_or_Y; b.Lw = Lw; b.Cw = Cw; b.Dw = Dw; b.G = G; b.dg_own = dg_own; b.dX = dX;
    b.dLw = dLw; b.dCw = dCw; b.dDw = dDw; b.dbias = dbias; b.dG_send = dG_send;
    PH_TRY(check_bwd_args(g, b));
    Arena sizing{nullptr, 0};
    carve_bwd(sizing, g);
    PH_TRY(check_ws(workspace, workspace_bytes, sizing.used));
    Arena a{(char *)workspace, 0};
    BwdWs w = carve_bwd(a, g);
    hipStream_t st = (hipStream_t)hip_stream;
    return g.dtype == PH_F32 ? bwd_impl<float>(g, b, w, st) : bwd_impl<bf16_t>(g, b, w, st);
}

}  // extern "C"

namespace {

// The argument checks of a step, all made before any GPU call; `ws_need`: the bytes of workspace it takes.
ph_status check_step_args(const ph_problem *prob, const ph_step_args *args, std::vector<Geo> &geos, size_t &ws_need)
{
    PH_TRY(make_geos(prob, geos));
    const Geo &g = geos[0];
    if (!args) return fail(PH_ERR_INVALID_ARG, "args is NULL");
    const int L = g.layers;
    if (args->mode < PH_STEP_TRAIN || args->mode > PH_STEP_NO_UPDATE) return fail(PH_ERR_INVALID_ARG, "unknown step mode %d", args->mode);
    const bool train = args->mode != PH_STEP_FORWARD;
    const bool update = args->mode == PH_STEP_TRAIN;
    PH_TRY(need(args->X0, "X0"));
    PH_TRY(check_ptr_array((const void *const *)args->Lw, L, "Lw"));
    PH_TRY(check_ptr_array((const void *const *)args->bias, L, "bias"));
    if (g.q > 0) {
        PH_TRY(check_ptr_array((const void *const *)args->Cw, L, "Cw"));
        PH_TRY(check_ptr_array((const void *const *)args->Dw, L, "Dw"));
        if (!g.all) {
            PH_TRY(check_ptr_array(args->G, L, "G"));
            if (train) PH_TRY(check_ptr_array(args->dg_own, L, "dg_own"));
        }
    }
    PH_TRY(optional(args->Y_out, "Y_out"));
    if (train) {
        PH_TRY(need(args->T, "T"));
        if (!args->loss) return fail(PH_ERR_INVALID_ARG, "loss is NULL");
        if (g.dtype == PH_BF16 && update) {
            PH_TRY(check_ptr_array((const void *const *)args->Lw_master, L, "Lw_master"));
            PH_TRY(check_ptr_array((const void *const *)args->bias_master, L, "bias_master"));
            if (g.q > 0) {
                PH_TRY(check_ptr_array((const void *const *)args->Cw_master, L, "Cw_master"));
                PH_TRY(check_ptr_array((const void *const *)args->Dw_master, L, "Dw_master"));
            }
        }
        if (args->dLw) PH_TRY(check_ptr_array((const void *const *)args->dLw, L, "dLw"));
        if (args->dbias) PH_TRY(check_ptr_array((const void *const *)args->dbias, L, "dbias"));
        if (g.q > 0 && args->dCw) PH_TRY(check_ptr_array((const void *const *)args->dCw, L, "dCw"));
        if (g.q > 0 && args->dDw) PH_TRY(check_ptr_array((const void *const *)args->dDw, L, "dDw"));
    }
    if (args->taps) {
        const ph_step_taps &t = *args->taps;
        const struct { void *const *arr; const char *name; } taps[] = {
            {t.Y, "taps.Y"}, {t.g_own, "taps.g_own"}, {t.delta, "taps.delta"}, {t.dG_send, "taps.dG_send"}, {t.dg_own, "taps.dg_own"}};
        for (const auto &tp : taps)
            for (int l = 0; tp.arr && l < L; ++l) {
                char nm[64];
                snprintf(nm, sizeof nm, "%s[%d]", tp.name, l);
                PH_TRY(optional(tp.arr[l], nm));
            }
    }
    Arena sizing{nullptr, 0};
    carve_step(sizing, geos);
    ws_need = sizing.used;
    return PH_OK;
}

ph_status run_step(const std::vector<Geo> &geos, const ph_step_args *args, void *workspace, void *hip_stream)
{
    Arena a{(char *)workspace, 0};
    StepWs w = carve_step(a, geos);
    hipStream_t st = (hipStream_t)hip_stream;
    return geos[0].dtype == PH_F32 ? step_impl<float>(geos, *args, w, st) : step_impl<bf16_t>(geos, *args, w, st);
}

// ---- the step for callers that cannot allocate -------------------------------------------------
// Its workspace is this array: device memory that every GPU the library runs on holds from the moment the
// code object is loaded there until the process ends.  In host code the array's name is only a handle:
// the address a kernel can use comes from hipGetSymbolAddress, once per device, with that device current.
constexpr size_t STATIC_WS_BYTES = (size_t)64 << 20;
static __device__ __align__(256) unsigned char scratch[STATIC_WS_BYTES];

constexpr int MAX_DEVICES = 64;
void *g_scratch_ptr[MAX_DEVICES];      // per device; written once under g_scratch_lock
std::mutex g_scratch_lock;

ph_status scratch_of_current_device(void **out)
{
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return fail(PH_ERR_LAUNCH, "hipGetDevice: %s", hipGetErrorString(e));
    if (dev < 0 || dev >= MAX_DEVICES) return fail(PH_ERR_UNSUPPORTED, "device index %d beyond %d", dev, MAX_DEVICES);
    std::lock_guard<std::mutex> hold(g_scratch_lock);
    if (!g_scratch_ptr[dev]) {
        void *ptr = nullptr;
        e = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch));
        if (e != hipSuccess || !ptr) return fail(PH_ERR_LAUNCH, "hipGetSymbolAddress(scratch): %s", hipGetErrorString(e));
        g_scratch_ptr[dev] = ptr;
    }
    *out = g_scratch_ptr[dev];
    return PH_OK;
}

}  // namespace

extern "C" {

ph_status phantom_ffn_step(const ph_problem *prob, const ph_step_args *args, void *workspace, size_t workspace_bytes,
                           void *hip_stream)
{
    std::vector<Geo> geos;
    size_t ws_need = 0;
    PH_TRY(check_step_args(prob, args, geos, ws_need));
    PH_TRY(check_ws(workspace, workspace_bytes, ws_need));
    return run_step(geos, args, workspace, hip_stream);
}

size_t phantom_static_workspace_bytes(void) { return STATIC_WS_BYTES; }

ph_status phantom_ffn_step_static(const ph_problem *prob, const ph_step_args *args, void *hip_stream)
{
    std::vector<Geo> geos;
    size_t ws_need = 0;
    PH_TRY(check_step_args(prob, args, geos, ws_need));
    if (ws_need > STATIC_WS_BYTES)
        return fail(PH_ERR_WORKSPACE, "the step needs %zu bytes of workspace, the library's own scratch array holds %zu: "
                                      "use phantom_ffn_step with a workspace of the caller's", ws_need, STATIC_WS_BYTES);
    void *ws = nullptr;
    PH_TRY(scratch_of_current_device(&ws));
    return run_step(geos, args, ws, hip_stream);
}

}  // extern "C"

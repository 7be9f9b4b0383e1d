/*
 * phantom.h -- C ABI of the MI355X phantom-layer library (libphantom.so).
 *
 * The library computes, on ONE GPU, the per-rank operators of phantom
 * parallelism for feed-forward networks (paper: Section IV, "Phantom Parallel
 * Operations").  A layer of width n is split over p ranks; each rank owns
 * s = n/p neurons and stores (Section IV-A)
 *     L   [s, s]        local matrix              L_l^(j)
 *     C   [k, s]        compressor                C_l^(j)
 *     D   [p-1, s, k]   decompressors             D_l^(i,j), i != j, in increasing i
 *     b   [s]           bias                      b_l^(j)
 * and computes   y^(j) = sigma(b + L y^(j) + sum_{i!=j} D^(i,j) g^(i)),  g^(i) = C^(i) y^(i)   (Eq. (ylq)).
 * The phantom layers g^(i) of the other ranks reach rank j by an All-Gather,
 * their gradients go back by a Reduce-Scatter (Algorithm 1).  No collective
 * runs here: in one-rank mode the peers' buffers are arguments, in all-ranks
 * mode all p ranks live on this GPU and the exchange is done in memory.
 *
 * Layout: row-major, batch-major; activations [batch, features], weights
 * [out, in].  In all-ranks mode (rank == -1) every tensor below gains a leading
 * [p] axis (X is [p, B, s]: rank j's columns of the full-width activation).
 *
 * Storage types:
 *   PH_F32  : every tensor is float; fp32 arithmetic.
 *   PH_BF16 : activations, errors, phantom layers and the compute copy of the
 *             weights are bfloat16; products accumulate in fp32; weight
 *             gradients, the loss and the master weights are float.
 *
 * Ownership: the caller owns every buffer, including the workspace.  The
 * library never allocates or frees device memory, never synchronises, and
 * enqueues work only on the HIP stream it is given.  Every pointer is a DEVICE
 * pointer, 16-byte aligned, unless stated otherwise ("host").  Inputs are not
 * modified.
 *
 * Errors: every entry point returns a ph_status; phantom_last_error() gives
 * the message of the calling thread's last failure.  PH_ERR_INVALID_ARG,
 * PH_ERR_UNSUPPORTED and PH_ERR_WORKSPACE are decided from the arguments alone,
 * before any GPU call (so they can be exercised on a host without a GPU): a call
 * that returns one of them has launched nothing and touched no buffer.
 * PH_ERR_LAUNCH is reported where it happens: launches that the same call
 * made before it stay enqueued, and the call's outputs are then undefined.
 */
#ifndef PHANTOM_H
#define PHANTOM_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    PH_OK = 0,
    PH_ERR_INVALID_ARG = -1,   /* bad shape, enum, null or misaligned pointer */
    PH_ERR_UNSUPPORTED = -2,   /* valid request this build cannot run */
    PH_ERR_WORKSPACE = -3,     /* workspace missing or too small */
    PH_ERR_LAUNCH = -4         /* the HIP runtime refused a launch in mid-call, or an internal inconsistency */
} ph_status;

typedef enum { PH_ACT_IDENTITY = 0, PH_ACT_RELU = 1, PH_ACT_GELU = 2 /* x*Phi(x), erf form */ } ph_act;
typedef enum { PH_F32 = 0, PH_BF16 = 1 } ph_dtype;

/*
 * The problem as the paper states it: (n, p, k, batch, layers, activation).
 *
 * Layers of different widths (Section IV, first paragraph: widths n_l and phantom widths k_l; the paper then
 * writes one n and one k for brevity): `widths` and `ks`, HOST arrays read during each call, or both NULL for
 * the uniform network.  widths[0 .. layers] = n_0 .. n_L (n_0 the network input, n_l the output of layer l,
 * each a multiple of p); ks[0 .. layers-1] = k_1 .. k_L.  Layer l then has, per rank, si = n_{l-1}/p inputs
 * and so = n_l/p outputs: Lw [so, si], Cw [k_l, si] (it compresses the layer's input), Dw [p-1, so, k_l],
 * bias [so]; wherever a shape below says s, read si for the layer's input side (X, dX, columns of Lw and
 * Cw) and so for its output side (Y, A, dY, bias, rows of Lw and Dw).  n and k are ignored when widths
 * is given.  The single-layer calls use widths[0], widths[1], ks[0].
 *
 * Size limits (PH_ERR_UNSUPPORTED beyond them): batch and every n_l/p at most 2^22, n_l/p + (p-1) k_l at most
 * 2^24, p at most 65535.  A bf16 problem in which one rank's share of a tensor ([B, n_l/p] activations, the
 * [p-1 or p, B, k] gathered buffer, a weight block) has more than 2^31 - 1 elements runs on the slower
 * shape-agnostic kernels (as one whose n_l/p or k_l is odd does); results are the same.
 */
typedef struct {
    int64_t n;        /* layer width; n % p == 0 */
    int64_t p;        /* ranks; p >= 1.  p == 1: a plain dense layer, no C, D, G */
    int64_t k;        /* ghost neurons per phantom layer; 1 <= k <= n/p when p > 1 */
    int64_t batch;    /* B >= 1 */
    int32_t layers;   /* L >= 1; used by phantom_ffn_step only */
    int32_t act;      /* ph_act, same for every layer incl. the last (sigma_L in Eq. (deltaL)) */
    int32_t dtype;    /* ph_dtype */
    int32_t rank;     /* j in [0, p): one-rank mode.  -1: all p ranks on this GPU */
    const int64_t *widths;   /* host, layers + 1 entries, or NULL */
    const int64_t *ks;       /* host, layers entries, or NULL (required with widths when p > 1) */
} ph_problem;

/* Bytes of workspace that any of the three calls below needs for this problem (host pointer out). */
ph_status phantom_workspace_bytes(const ph_problem *prob, size_t *bytes);

/*
 * Forward of one phantom layer, Eq. (ylq) (Section IV-A: local update,
 * compression, decompression, remote update, bias and activation).
 *
 *   X     in   [B, s]        y_{l-1}^(j)
 *   Lw, Cw, Dw, bias         the rank's weights (Cw, Dw ignored when p == 1)
 *   G     in   one-rank: [p-1, B, k], the gathered g^(i) of the peers in increasing i.
 *              all-ranks: ignored (may be NULL); the gathered buffer is g_own.
 *   Y     out  [B, s]        y_l^(j)
 *   g_own out  [B, k]        g_l^(j) = C y_{l-1}^(j): the rank's All-Gather contribution.
 *              all-ranks: [p, B, k]; written first, then read as every rank's gathered buffer
 *              (rank j skips slot j).  Ignored when p == 1.
 *   A_save out [B, s] or NULL  pre-activation b + z, needed by phantom_layer_bwd for GELU
 *              (for ReLU the backward accepts Y instead; for identity nothing).
 */
ph_status phantom_layer_fwd(const ph_problem *prob,
                            const void *X, const void *Lw, const void *Cw, const void *Dw,
                            const void *bias, const void *G,
                            void *Y, void *g_own, void *A_save,
                            void *workspace, size_t workspace_bytes, void *hip_stream);

/*
 * Backward of one phantom layer (Section IV-B):
 *   delta   = dY * sigma'(A)                           Eq. (deltaL) / the sigma' factor of Eq. (backprop)
 *   dG_send = (D^(i,j))^T delta for each peer i        "error compression", h of Eq. (backprop)
 *   dX      = L^T delta + C^T dg_own                   braces of Eq. (backprop)
 *   dbias, dLw, dCw, dDw                               Eq. (bpb), (bpL), (bpC), (bpD); dDw in D's own [s, k] shape
 *
 *   dY      in   [B, s]   dLoss/dy_l^(j)
 *   X       in   [B, s]   the layer's input
 *   A_or_Y  in   [B, s]   GELU: the saved pre-activation.  ReLU: pre-activation or output (only the
 *                         sign is used; ReLU'(0) = 0).  Identity: ignored, may be NULL.
 *   G       in   one-rank: [p-1, B, k] as in the forward.  all-ranks: [p, B, k], the forward's g_own.
 *   dg_own  one-rank: in  [B, k], dLoss/dg^(j) = the Reduce-Scatter result from the peers.
 *           all-ranks: out [p, B, k], computed here from dG_send (sum over holders).
 *   dX      out  [B, s] or NULL (first layer)
 *   dLw [s,s], dCw [k,s], dDw [p-1,s,k], dbias [s]   out, ALWAYS float (also with PH_BF16)
 *   dG_send out  [p-1, B, k] storage type: what the rank returns to peer i (Reduce-Scatter input).
 *   Ignored when p == 1: Cw, Dw, G, dg_own, dCw, dDw, dG_send.
 */
ph_status phantom_layer_bwd(const ph_problem *prob,
                            const void *dY, const void *X, const void *A_or_Y,
                            const void *Lw, const void *Cw, const void *Dw,
                            const void *G, void *dg_own,
                            void *dX, float *dLw, float *dCw, float *dDw, float *dbias,
                            void *dG_send,
                            void *workspace, size_t workspace_bytes, void *hip_stream);

typedef enum {
    PH_STEP_TRAIN = 0,      /* forward, loss, backward, SGD update */
    PH_STEP_FORWARD = 1,    /* inference: forward only; T, loss, masters, G-gradients unused */
    PH_STEP_NO_UPDATE = 2   /* forward, loss, backward; gradients are produced, weights are left alone */
} ph_step_mode;

/*
 * Optional taps of phantom_ffn_step, for checking every stage of the step on its own (NULL in production):
 * copies of the tensors that pass from one stage of Eq. (ylq) / Eq. (backprop) to the next, taken right after
 * the launch that finishes each of them (one small copy launch per tap; the step's own launches are the same
 * with and without taps).  HOST arrays of prob->layers DEVICE pointers, each array and each entry may be NULL;
 * storage type, shapes per layer l as in phantom_layer_fwd / _bwd (all ranks: the leading [p] axis):
 *   Y[l]       [B, so]       y_l as stored (the next layer's operand)
 *   g_own[l]   [B, k]        g_l^(j) = C y_{l-1}^(j)          (all ranks: [p, B, k], the gathered buffer)
 *   delta[l]   [B, so]       delta_l = dLoss/dz_l: Eq. (deltaL) for the last layer, Eq. (backprop) below it
 *   dG_send[l] [p-1, B, k]   (D^(i,j))^T delta_l^(j), the Reduce-Scatter input
 *   dg_own[l]  [p, B, k]     all-ranks mode only: the Reduce-Scatter result the step computed
 * Ignored with PH_STEP_FORWARD: delta, dG_send, dg_own.
 */
typedef struct {
    void *const *Y;
    void *const *g_own;
    void *const *delta;
    void *const *dG_send;
    void *const *dg_own;
} ph_step_taps;

/*
 * Arguments of phantom_ffn_step.  The arrays are HOST arrays of prob->layers
 * DEVICE pointers, read during the call.
 */
typedef struct {
    const void *X0;            /* [B, s] network input (the rank's columns) */
    const void *T;             /* [B, s] target; may be NULL with PH_STEP_FORWARD */
    void *const *Lw;           /* compute weights in storage type, updated in place */
    void *const *Cw;
    void *const *Dw;
    void *const *bias;
    float *const *Lw_master;   /* PH_BF16 only: fp32 master weights, updated in place, then rounded into */
    float *const *Cw_master;   /*   the bfloat16 compute copy.  NULL arrays with PH_F32. */
    float *const *Dw_master;
    float *const *bias_master;
    const void *const *G;      /* one-rank mode: per-layer gathered peer buffers [p-1, B, k]; else NULL */
    const void *const *dg_own; /* one-rank mode: per-layer Reduce-Scatter results [B, k]; else NULL */
    float *const *dLw;         /* optional (array may be NULL): gradients are also written here */
    float *const *dCw;
    float *const *dDw;
    float *const *dbias;
    void *Y_out;               /* optional: network output [B, s], storage type */
    float *loss;               /* device scalar: 1/(2B) sum (y_L - t)^2 over batch, features and ranks held */
    float lr;                  /* SGD: w <- w - lr * dLoss/dw, all gradients taken before the update */
    int32_t mode;              /* ph_step_mode */
    const ph_step_taps *taps;  /* host; NULL: none */
} ph_step_args;

/*
 * One training step of an L-layer phantom FFN on this GPU's share: forward
 * through every layer (Eq. (ylq)), MSE output error dLoss/dy_L = (y_L - t)/B
 * (Section IV-B, "Local error at the output", averaged over the batch),
 * backward through every layer (Eq. (backprop), (bpb)-(bpD)) and a plain SGD
 * update.  Between layers, y_l and delta_l = dLoss/dz_l are kept in the storage
 * type; delta_l is formed as (L^T delta + C^T dg_own) * sigma_l' and rounded once,
 * as Eq. (backprop) writes it (dLoss/dy_l itself is never stored).  For GELU the
 * workspace keeps, between forward and backward, sigma_l'(b + z) in float (PH_BF16) or
 * the pre-activation in float (PH_F32); ReLU's derivative is read off the stored y_l.
 * The workspace need not be cleared by the caller and holds nothing between calls.
 */
ph_status phantom_ffn_step(const ph_problem *prob, const ph_step_args *args,
                           void *workspace, size_t workspace_bytes, void *hip_stream);

/*
 * phantom_ffn_step for callers that cannot allocate device memory: code under HIP graph capture, serving
 * loops that must not call hipMalloc, harnesses that forbid it.  Same arguments, same kernels and same
 * results as phantom_ffn_step, but the workspace is the library's own: a file-scope device array of
 * phantom_static_workspace_bytes() = 64 MiB that every GPU the library runs on holds until the process
 * ends.  The call allocates and frees nothing (no hipMalloc, hipFree or allocating library routine); its
 * first call on a device looks the array's address up there (hipGetSymbolAddress), later calls reuse it.
 * A problem whose step needs more than that (phantom_workspace_bytes) is refused with PH_ERR_WORKSPACE
 * before any GPU call: use phantom_ffn_step with a workspace of the caller's.
 * All calls on one GPU share that one array, which keeps the last call's contents; the step clears what it
 * needs cleared itself.  Two calls that overlap on one GPU (different streams, or threads) race: serialise them.
 */
ph_status phantom_ffn_step_static(const ph_problem *prob, const ph_step_args *args, void *hip_stream);
size_t phantom_static_workspace_bytes(void);

/* Message of the calling thread's last error ("" if none).  Host string owned by the library. */
const char *phantom_last_error(void);

/*
 * Per-kernel timing for benchmarks (measurement of the operators above, Section VI reports times
 * per epoch only).  Between phantom_profile_begin and phantom_profile_end every kernel launch this
 * library makes from the calling thread is bracketed by a pair of HIP events on its stream.
 * phantom_profile_end waits for those events (the only call here that blocks), and returns one
 * entry per distinct (kernel, shape): how often it ran and the summed time between its events.
 * For products, M x N is the output and K the reduction length per group; for elementwise kernels
 * N is the element count.  `entries` is a HOST array of `capacity` entries.
 * The time between two events around a launch includes launch and time-stamp latency (a few
 * microseconds); to let the caller subtract it, the first profiled launch is preceded by 32
 * launches of a kernel that does nothing, reported as the entry named "(empty launch)".
 */
typedef struct {
    char name[64];
    int64_t M, N, K;
    int32_t groups;
    int32_t calls;
    double total_ms;
    int64_t M2, N2, K2;   /* a launch that carries several products: the second one's shape, */
    int64_t M3, N3, K3;   /*   the third one's */
    int64_t M4, N4, K4;   /*   and the fourth one's, else 0 */
} ph_profile_entry;

ph_status phantom_profile_begin(int32_t max_launches);
ph_status phantom_profile_end(ph_profile_entry *entries, int32_t capacity, int32_t *count);

/* Library version, for the binding's sanity check. */
int32_t phantom_abi_version(void);

#ifdef __cplusplus
}
#endif
#endif /* PHANTOM_H */

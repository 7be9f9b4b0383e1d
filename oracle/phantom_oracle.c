/*
 * CPU oracle for the phantom layer -- TEST INFRASTRUCTURE, not part of the product.
 *
 * Plain fp64 loops that follow the paper's definitions term by term:
 *   forward   : Section IV-A, Eq. (ylq)       y = sigma(b + L y + sum_{i!=j} D^(i,j) g^(i)),  g = C y
 *   backward  : Section IV-B, Eq. (deltaL), Eq. (backprop), Eq. (bpb)-(bpD)
 * for ONE rank j and ONE layer.  Several ranks, several layers, the loss and
 * the update are put together from these calls by oracle/oracle.py.
 *
 * Layer widths may differ (Section IV, first paragraph: widths n_l and phantom widths k_l per layer; the
 * equations are then written for one width to keep them short).  Reading taken here: layer l maps
 * n_{l-1} to n_l, rank j holds si = n_{l-1}/p inputs and so = n_l/p outputs of it, so L is [so, si], C is
 * [k, si] (it compresses the layer's input), D^(i,j) is [so, k], b is [so].  Below, "s" in a shape
 * stands for so where the tensor lives on the output side (A, Y, dY, delta, bias, rows of L and D) and
 * for si on the input side (X, dX, columns of L and C).
 *
 * Conventions (row-major, batch-major):
 *   X   [B, s]      y_{l-1}^(j)                 Lw  [s, s]      L_l^(j)
 *   Cw  [k, s]      C_l^(j)                     Dw  [q, s, k]   D_l^(i,j) for the q = p-1 peers i != j,
 *   bias[s]         b_l^(j)                                      in increasing order of i
 *   G   [q, B, k]   g_l^(i), same peer order    A   [B, s]      b + z (pre-activation)
 *   dY  [B, s]      dLoss/dy_l^(j)              delta [B, s]    dLoss/dz_l^(j)
 *   dg_own [B, k]   dLoss/dg_l^(j) = sum over the other ranks of what they send back
 *   dG_send [q,B,k] dLoss/dg_l^(i,j) = (D^(i,j))^T delta^(j): what rank j sends back to peer i
 *
 * Readings of the paper taken here:
 *   - D^(i,j) is stored on rank j and applied to the phantom layer that came from
 *     rank i (Eq. (ylq)); its gradient is kept in D's own [s, k] shape,
 *     delta^(j) (g^(i))^T, i.e. the transpose of what Eq. (bpD) prints.
 *   - no bias and no activation on the phantom layer (Eq. (ylq) has neither).
 *   - ReLU'(0) = 0.  GELU is x*Phi(x), its derivative Phi(x) + x*phi(x).
 *   - when the storage type is bfloat16, a tensor that is the operand of a
 *     later matrix product (here: delta) is rounded to bfloat16 once it is
 *     formed; sums and elementwise functions are exact (fp64).
 *   - the sigma' factor of Eq. (deltaL) / Eq. (backprop) is sigma'(A) itself, in fp64, whatever the
 *     storage type: the paper rounds nothing there.
 *
 * Parallelism: OpenMP over independent output rows only; no blocking, no
 * reordering of a sum other than the loop order written below.
 *
 * Pins: tests/test_oracle_pins.py (dense special cases, finite differences,
 * Table 1 parameter counts, brute-force Python loops on tiny inputs).
 */
#include <math.h>
#include <stdint.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

enum { ACT_IDENTITY = 0, ACT_RELU = 1, ACT_GELU = 2 };

static double act_f(int act, double a) {
    switch (act) {
    case ACT_RELU: return a > 0.0 ? a : 0.0;
    case ACT_GELU: return a * 0.5 * (1.0 + erf(a * M_SQRT1_2));
    default: return a;
    }
}

static double act_df(int act, double a) {
    switch (act) {
    case ACT_RELU: return a > 0.0 ? 1.0 : 0.0;
    case ACT_GELU: {
        double Phi = 0.5 * (1.0 + erf(a * M_SQRT1_2));
        double phi = exp(-0.5 * a * a) * 0.3989422804014326779; /* 1/sqrt(2 pi) */
        return Phi + a * phi;
    }
    default: return 1.0;
    }
}

/* Nearest-even rounding of a double to the bfloat16 grid (8 significant bits).
 * Exponent range is not clamped: the values met here are far from bfloat16's limits. */
double pho_round_bf16(double v) {
    uint64_t u;
    memcpy(&u, &v, sizeof u);
    if (((u >> 52) & 0x7FF) == 0x7FF || v == 0.0) return v;
    const int drop = 52 - 7;
    uint64_t lsb = (u >> drop) & 1u;
    u += ((UINT64_C(1) << (drop - 1)) - 1) + lsb;
    u &= ~((UINT64_C(1) << drop) - 1);
    memcpy(&v, &u, sizeof v);
    return v;
}

void pho_round_bf16_array(double *a, int64_t count) {
    for (int64_t i = 0; i < count; ++i) a[i] = pho_round_bf16(a[i]);
}

int pho_num_threads(void) {
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/* Forward of one layer on one rank, Eq. (ylq), in the two pieces the method has
 * (Section IV-A, "Parallel Complexity"); pho_layer_fwd below runs them in order.
 *
 * (1) compression: g^(j) = C^(j) y^(j).  The result is what the rank contributes to the All-Gather. */
void pho_compress(int64_t B, int64_t s, int64_t k,
                  const double *X, const double *Cw, double *g_own)
{
#pragma omp parallel for schedule(static)
    for (int64_t b = 0; b < B; ++b) {
        const double *x = X + b * s;
        for (int64_t c = 0; c < k; ++c) {
            double acc = 0.0;
            for (int64_t m = 0; m < s; ++m) acc += Cw[c * s + m] * x[m];
            g_own[b * k + c] = acc;
        }
    }
}

/* (2) local update, decompression, remote update, bias and activation:
 *     A = b + L y + sum_{i != j} D^(i,j) g^(i),  Y = sigma(A).   q = 0 means p = 1: Dw, G unused. */
void pho_layer_update(int64_t B, int64_t si, int64_t so, int64_t k, int64_t q, int act,
                      const double *X, const double *Lw, const double *Dw,
                      const double *bias, const double *G,
                      double *A, double *Y)
{
#pragma omp parallel for schedule(static)
    for (int64_t b = 0; b < B; ++b) {
        const double *x = X + b * si;
        for (int64_t o = 0; o < so; ++o) {
            double z = 0.0;
            /* local update L^(j) y^(j) */
            for (int64_t m = 0; m < si; ++m) z += Lw[o * si + m] * x[m];
            /* decompression and remote update: sum_i D^(i,j) g^(i) */
            for (int64_t i = 0; i < q; ++i) {
                const double *d = Dw + (i * so + o) * k;
                const double *g = G + (i * B + b) * k;
                double t = 0.0;
                for (int64_t c = 0; c < k; ++c) t += d[c] * g[c];
                z += t;
            }
            double a = bias[o] + z;
            A[b * so + o] = a;
            Y[b * so + o] = act_f(act, a);
        }
    }
}

void pho_layer_fwd(int64_t B, int64_t si, int64_t so, int64_t k, int64_t q, int act,
                   const double *X, const double *Lw, const double *Cw, const double *Dw,
                   const double *bias, const double *G,
                   double *A, double *Y, double *g_own)
{
    if (q > 0) pho_compress(B, si, k, X, Cw, g_own);
    pho_layer_update(B, si, so, k, q, act, X, Lw, Dw, bias, G, A, Y);
}

/* Backward of one layer on one rank, in the three pieces the method has
 * (Section IV-B, "Parallel Complexity"); pho_layer_bwd below runs them in order.
 *
 * (1) local error:        delta = dY * sigma'(A)            Eq. (deltaL); the sigma' factor of Eq. (backprop)
 *     round_operands != 0: delta is rounded to bfloat16 when formed (see header).
 */
void pho_delta(int64_t B, int64_t s, int act, int round_operands,
               const double *dY, const double *A, double *delta)
{
#pragma omp parallel for schedule(static)
    for (int64_t b = 0; b < B; ++b) {
        for (int64_t o = 0; o < s; ++o) {
            double d = dY[b * s + o] * act_df(act, A[b * s + o]);
            delta[b * s + o] = round_operands ? pho_round_bf16(d) : d;
        }
    }
}

/* (2) error compression:  dG_send[i] = (D^(i,j))^T delta^(j)   h of Eq. (backprop); what rank j
 *     returns to peer i for the reduce-scatter. */
void pho_error_compress(int64_t B, int64_t s, int64_t k, int64_t q,
                        const double *Dw, const double *delta, double *dG_send)
{
#pragma omp parallel for schedule(static)
    for (int64_t b = 0; b < B; ++b) {
        const double *dl = delta + b * s;
        for (int64_t i = 0; i < q; ++i) {
            for (int64_t c = 0; c < k; ++c) {
                double acc = 0.0;
                for (int64_t o = 0; o < s; ++o) acc += Dw[(i * s + o) * k + c] * dl[o];
                dG_send[(i * B + b) * k + c] = acc;
            }
        }
    }
}

/* (3) local errors and individual gradients, once dg_own (the reduce-scatter result) is known:
 *     dX      = L^T delta + C^T dg_own                        braces of Eq. (backprop)
 *     dbias   = sum_b delta                                   Eq. (bpb)
 *     dLw     = sum_b delta x^T                               Eq. (bpL)
 *     dDw[i]  = sum_b delta (g^(i))^T                         Eq. (bpD), in D's own shape
 *     dCw     = sum_b dg_own x^T                              Eq. (bpC), its sum over ranks already in dg_own
 *     dX may be NULL.  q = 0: Cw, G, dg_own, dCw, dDw unused.
 */
void pho_layer_grads(int64_t B, int64_t si, int64_t so, int64_t k, int64_t q,
                     const double *delta, const double *X,
                     const double *Lw, const double *Cw,
                     const double *G, const double *dg_own,
                     double *dX, double *dLw, double *dCw, double *dDw, double *dbias)
{
    if (dX) {
#pragma omp parallel for schedule(static)
        for (int64_t b = 0; b < B; ++b) {
            const double *dl = delta + b * so;
            double *dx = dX + b * si;
            for (int64_t m = 0; m < si; ++m) dx[m] = 0.0;
            for (int64_t o = 0; o < so; ++o) {
                double d = dl[o];
                for (int64_t m = 0; m < si; ++m) dx[m] += Lw[o * si + m] * d;
            }
            for (int64_t c = 0; c < (q > 0 ? k : 0); ++c) {
                double h = dg_own[b * k + c];
                for (int64_t m = 0; m < si; ++m) dx[m] += Cw[c * si + m] * h;
            }
        }
    }

#pragma omp parallel for schedule(static)
    for (int64_t o = 0; o < so; ++o) {
        double sb = 0.0;
        double *gl = dLw + o * si;
        for (int64_t m = 0; m < si; ++m) gl[m] = 0.0;
        for (int64_t i = 0; i < q; ++i)
            for (int64_t c = 0; c < k; ++c) dDw[(i * so + o) * k + c] = 0.0;
        for (int64_t b = 0; b < B; ++b) {
            double d = delta[b * so + o];
            sb += d;
            const double *x = X + b * si;
            for (int64_t m = 0; m < si; ++m) gl[m] += d * x[m];
            for (int64_t i = 0; i < q; ++i) {
                const double *g = G + (i * B + b) * k;
                double *gd = dDw + (i * so + o) * k;
                for (int64_t c = 0; c < k; ++c) gd[c] += d * g[c];
            }
        }
        dbias[o] = sb;
    }

    if (q > 0) {
#pragma omp parallel for schedule(static)
        for (int64_t c = 0; c < k; ++c) {
            double *gc = dCw + c * si;
            for (int64_t m = 0; m < si; ++m) gc[m] = 0.0;
            for (int64_t b = 0; b < B; ++b) {
                double h = dg_own[b * k + c];
                const double *x = X + b * si;
                for (int64_t m = 0; m < si; ++m) gc[m] += h * x[m];
            }
        }
    }
}

void pho_layer_bwd(int64_t B, int64_t si, int64_t so, int64_t k, int64_t q, int act, int round_operands,
                   const double *dY, const double *X, const double *A,
                   const double *Lw, const double *Cw, const double *Dw,
                   const double *G, const double *dg_own,
                   double *delta, double *dX, double *dLw, double *dCw, double *dDw,
                   double *dbias, double *dG_send)
{
    pho_delta(B, so, act, round_operands, dY, A, delta);
    if (q > 0) pho_error_compress(B, so, k, q, Dw, delta, dG_send);
    pho_layer_grads(B, si, so, k, q, delta, X, Lw, Cw, G, dg_own, dX, dLw, dCw, dDw, dbias);
}

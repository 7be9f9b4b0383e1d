// Shape-agnostic tiled product C(m, n) = sum_c A(m, c) * B(n, c) with fp32 FMAs.
//
// Serves the fp32 storage type (true fp32 arithmetic, as the 1e-5 parity bound
// needs) and every bf16 shape the MFMA kernels do not take (k not a multiple
// of the vector width, tiny shards).  Operands and the output are Views, so the
// same kernel runs every product of the forward and backward operators.
#pragma once
#include "common.h"
#include "views.h"

namespace phantom {

enum { EPI_STORE = 0, EPI_BIAS_ACT = 1, EPI_DACT = 2 };

struct Epilogue {
    int32_t mode;
    int32_t act;
    const void *bias;    // EPI_BIAS_ACT: [N] per group, storage type
    int64_t bias_g;
    void *aux;           // EPI_BIAS_ACT: optional pre-activation out; EPI_DACT: pre-activation (or ReLU output) in
                         //   (MFMA kernel: NULL = multiply by nothing, for the column sums alone)
    int64_t aux_ld;      //   plain row-major [M x N]
    int64_t aux_g;
    int32_t aux_f32;     // aux holds float instead of the storage type
    int32_t aux_deriv;   // aux holds sigma'(pre-activation), in float, instead of the pre-activation:
                         //   EPI_BIAS_ACT writes it, EPI_DACT multiplies by it as it stands
    float *colsum;       // MFMA kernel only, optional: the column sums of the stored output (as rounded to
    int64_t colsum_g;    //   the output type) are ADDED to colsum[N] per group; the caller zeroes it first
    // MFMA kernel only, EPI_BIAS_ACT, optional (mse_target != NULL): the layer is the last one and the MSE output
    // error is formed on the way out (Eq. (deltaL)): with y the output as stored and t = mse_target (laid out
    // like aux: aux_ld, aux_g, storage type), mse_delta <- ((y - t) * mse_inv_b) * sigma'(pre-activation)
    // (sigma' of the pre-activation in float for GELU, from y for ReLU), colsum
    // then receives the column sums of mse_delta instead of y's, and mse_partial[tile] <- sum over the
    // tile of (y - t)^2, tile = (group * ceil(M/128) + tile row) * ceil(N/128) + tile column.
    const void *mse_target;
    void *mse_delta;
    float *mse_partial;
    float mse_inv_b;
    int32_t aux_bits;    // MFMA kernel, 8-element vectors, ReLU only: aux holds ONE BIT per element, (stored output > 0), i.e.
                         //   ReLU' as the backward pass reads it off the stored output, in an eighth of the bytes:
                         //   EPI_BIAS_ACT writes it (bit u of byte (g*aux_g + m*aux_ld + n) / 8 = column n + u),
                         //   EPI_DACT keeps or zeroes each element by it
};

constexpr int GT = 64;   // tile edge
constexpr int GK = 16;   // reduction step

template <typename TIn, typename TOut>
__global__ __launch_bounds__(256) void gemm_generic_kernel(View va, View vb, View vo, Epilogue ep,
                                                          int M, int N, int K)
{
    __shared__ float As[GK][GT + 4];
    __shared__ float Bs[GK][GT + 4];

    const int g = blockIdx.z;
    const int m0 = blockIdx.y * GT, n0 = blockIdx.x * GT;
    const int tid = threadIdx.x;
    const int tx = tid & 15, ty = tid >> 4;

    const TIn *a0 = (const TIn *)va.p0 + g * va.g0, *a1 = (const TIn *)va.p1 + g * va.g1;
    const TIn *b0 = (const TIn *)vb.p0 + g * vb.g0, *b1 = (const TIn *)vb.p1 + g * vb.g1;
    const int skip_a = va.skip0 + g * va.skip_g, skip_b = vb.skip0 + g * vb.skip_g;

    // this thread stages rows lr + 16*i (i = 0..3) at reduction offset lk of every step
    const int lk = tid & 15, lr = tid >> 4;
    Loc ra[4], rb[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        int m = m0 + lr + 16 * i, n = n0 + lr + 16 * i;
        ra[i] = locate(va.r, m < M ? m : 0, skip_a);
        rb[i] = locate(vb.r, n < N ? n : 0, skip_b);
    }

    // Three levels of partial sums (16 terms, 16 of those, the rest): a single running fp32 sum over a reduction
    // range of several thousand (a weight gradient over the batch) drifts past 1e-5 of the result.
    float acc[4][4] = {}, mid[4][4] = {};
    int steps_in_mid = 0;
    for (int k0 = 0; k0 < K; k0 += GK) {
        const int kk = k0 + lk;
        const bool kin = kk < K;
        Loc ca = locate(va.c, kin ? kk : 0, skip_a);
        Loc cb = locate(vb.c, kin ? kk : 0, skip_b);
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            float av = 0.f, bv = 0.f;
            if (kin && m0 + lr + 16 * i < M) {
                int reg; int64_t off = join(ra[i], ca, reg);
                av = to_f32((reg ? a1 : a0)[off]);
            }
            if (kin && n0 + lr + 16 * i < N) {
                int reg; int64_t off = join(rb[i], cb, reg);
                bv = to_f32((reg ? b1 : b0)[off]);
            }
            As[lk][lr + 16 * i] = av;
            Bs[lk][lr + 16 * i] = bv;
        }
        __syncthreads();
        float part[4][4] = {};
#pragma unroll
        for (int q = 0; q < GK; ++q) {
            float av[4], bv[4];
#pragma unroll
            for (int i = 0; i < 4; ++i) { av[i] = As[q][ty * 4 + i]; bv[i] = Bs[q][tx * 4 + i]; }
#pragma unroll
            for (int i = 0; i < 4; ++i)
#pragma unroll
                for (int j = 0; j < 4; ++j) part[i][j] = fmaf(av[i], bv[j], part[i][j]);
        }
        const bool flush = ++steps_in_mid == 16;       // uniform
#pragma unroll
        for (int i = 0; i < 4; ++i)
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                mid[i][j] += part[i][j];
                if (flush) { acc[i][j] += mid[i][j]; mid[i][j] = 0.f; }
            }
        if (flush) steps_in_mid = 0;
        __syncthreads();
    }
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) acc[i][j] += mid[i][j];

    TOut *o0 = (TOut *)vo.p0 + g * vo.g0, *o1 = (TOut *)vo.p1 + g * vo.g1;
    const int skip_o = vo.skip0 + g * vo.skip_g;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int m = m0 + ty * 4 + i;
        if (m >= M) continue;
        Loc lm = locate(vo.r, m, skip_o);
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int n = n0 + tx * 4 + j;
            if (n >= N) continue;
            Loc ln = locate(vo.c, n, skip_o);
            int reg; int64_t off = join(lm, ln, reg);
            float v = acc[i][j];
            if (ep.mode == EPI_BIAS_ACT) {
                v += to_f32(((const TIn *)ep.bias)[g * ep.bias_g + n]);
                if (ep.aux) {
                    const int64_t at = g * ep.aux_g + (int64_t)m * ep.aux_ld + n;
                    if (ep.aux_deriv) ((float *)ep.aux)[at] = act_deriv(ep.act, v);
                    else if (ep.aux_f32) ((float *)ep.aux)[at] = v;
                    else ((TIn *)ep.aux)[at] = from_f32<TIn>(v);
                }
                v = act_apply(ep.act, v);
            } else if (ep.mode == EPI_DACT) {
                const int64_t at = g * ep.aux_g + (int64_t)m * ep.aux_ld + n;
                if (ep.aux_deriv) {
                    v *= ((const float *)ep.aux)[at];
                } else {
                    const float a = ep.aux_f32 ? ((const float *)ep.aux)[at] : to_f32(((const TIn *)ep.aux)[at]);
                    v *= act_deriv(ep.act, a);
                }
            }
            (reg ? o1 : o0)[off] = from_f32<TOut>(v);
        }
    }
}

}  // namespace phantom

// The compression g = C y of Eq. (ylq) as a kernel of its own: G[m, n] = sum_c X[m, c] * C[n, c] with a
// short n range (k <= 64 phantom neurons), bf16 in, fp32 accumulate, bf16 out.
//
// As a tile of the general product it has few workgroups (one per 128 rows: 64 for an 8192-row batch)
// and every one of them walks the whole reduction range, so three quarters of the device wait for
// 14 us.  Here a workgroup owns 32 rows and all n; its eight wavefronts split the reduction range and
// feed the MFMAs straight from global memory (a lane's operand is 16 contiguous bytes of one row; the
// four 16-byte pieces of a 128-byte line are used by consecutive steps of the same wavefront, from L1),
// then add their partial sums through LDS.  C (k x s, at most 128 KB) is read by every workgroup, from L2.
#pragma once
#include "common.h"

namespace phantom {

constexpr int THIN_ROWS = 32;       // rows of X per workgroup
constexpr int THIN_MAX_N = 64;
constexpr int THIN_WAVES = 8;       // wavefronts per workgroup of the stand-alone kernel

typedef __bf16 thin_bf16x8 __attribute__((ext_vector_type(8)));
typedef float thin_f32x16 __attribute__((ext_vector_type(16)));

// One workgroup's share: rows [m0, m0 + 32) of group grp.  NF = number of 32-wide column blocks (1: N <= 32,
// 2: N <= 64); WAVES wavefronts split the K / 16 reduction chunks (K is a multiple of 16); part: WAVES * NF * 1024
// floats of LDS.  x_g, c_g, o_g: element offsets per group.
// M: end of the rows this call may read and store (the matrix's row count, or the end of a shorter share of a
// 32-row block: the MFMA rows beyond it repeat the last one and are dropped).
template <int NF, int WAVES>
__device__ __forceinline__ void thin_workgroup(const __bf16 *__restrict__ X, const __bf16 *__restrict__ C,
                                               __bf16 *__restrict__ G, int M, int N, int K, int64_t x_g, int64_t c_g,
                                               int64_t o_g, int m0, int grp, float *part)
{
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const __bf16 *x = X + grp * x_g, *c = C + grp * c_g;
    __bf16 *out = G + grp * o_g;
    auto part_at = [part](int w, int f, int e, int l) -> float & { return part[((w * NF + f) * 16 + e) * 64 + l]; };

    // this wavefront's share of the K / 16 reduction chunks
    const int chunks = K >> 4;
    const int c_lo = (int)((int64_t)chunks * wave / WAVES), c_hi = (int)((int64_t)chunks * (wave + 1) / WAVES);
    // MFMA operand of a lane: row (lane & 31), 8 consecutive reduction indices starting at 8 * (lane >> 5).
    // Rows past the end read the last row; what they produce is never stored.
    const int half = (lane >> 5) * 8;
    const __bf16 *xrow = x + (int64_t)min(m0 + (lane & 31), M - 1) * K + half;
    const __bf16 *crow[NF];
#pragma unroll
    for (int f = 0; f < NF; ++f) crow[f] = c + (int64_t)min(f * 32 + (lane & 31), N - 1) * K + half;

    thin_f32x16 acc[NF];
#pragma unroll
    for (int f = 0; f < NF; ++f)
#pragma unroll
        for (int e = 0; e < 16; ++e) acc[f][e] = 0.f;
    int ch = c_lo;
    for (; ch + 4 <= c_hi; ch += 4) {                  // four chunks' loads in flight together
        thin_bf16x8 a[4], b[NF][4];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            a[u] = *(const thin_bf16x8 *)(xrow + (ch + u) * 16);
#pragma unroll
            for (int f = 0; f < NF; ++f) b[f][u] = *(const thin_bf16x8 *)(crow[f] + (ch + u) * 16);
        }
#pragma unroll
        for (int u = 0; u < 4; ++u)
#pragma unroll
            for (int f = 0; f < NF; ++f) acc[f] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[u], b[f][u], acc[f], 0, 0, 0);
    }
    for (; ch < c_hi; ++ch) {
        const thin_bf16x8 a = *(const thin_bf16x8 *)(xrow + ch * 16);
#pragma unroll
        for (int f = 0; f < NF; ++f) {
            const thin_bf16x8 b = *(const thin_bf16x8 *)(crow[f] + ch * 16);
            acc[f] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, acc[f], 0, 0, 0);
        }
    }
#pragma unroll
    for (int f = 0; f < NF; ++f)
#pragma unroll
        for (int e = 0; e < 16; ++e) part_at(wave, f, e, lane) = acc[f][e];
    __syncthreads();

    // accumulator e of lane l in column block f is element (row 8*(e/4) + 4*(l>>5) + e%4, column 32*f + (l&31))
    for (int o = threadIdx.x; o < THIN_ROWS * NF * 32; o += WAVES * 64) {
        const int row = o / (NF * 32), col = o - row * (NF * 32);
        const int m = m0 + row;
        if (m >= M || col >= N) continue;
        const int f = col >> 5, e = (row >> 3) * 4 + (row & 3), l = (col & 31) + 32 * ((row >> 2) & 1);
        float sum = 0.f;
#pragma unroll
        for (int w = 0; w < WAVES; ++w) sum += part_at(w, f, e, l);
        out[(int64_t)m * N + col] = (__bf16)sum;
    }
}

// The kernel: workgroup (x, y) = rows [32 x, 32 x + 32) of group y, THIN_WAVES wavefronts.
// Rider: the kernel also clears zero_count floats at `zero` (buffers that later launches of a training step
// add into; the compression is the launch before the first of them).
template <int NF>
__global__ __launch_bounds__(THIN_WAVES * 64) void thin_product_kernel(const __bf16 *__restrict__ X, const __bf16 *__restrict__ C,
                                                          __bf16 *__restrict__ G, int M, int N, int K,
                                                          int64_t x_g, int64_t c_g, int64_t o_g,
                                                          float *__restrict__ zero, int64_t zero_count)
{
    constexpr int THREADS = THIN_WAVES * 64;
    for (int64_t z = ((int64_t)blockIdx.y * gridDim.x + blockIdx.x) * THREADS + threadIdx.x; z < zero_count;
         z += (int64_t)gridDim.x * gridDim.y * THREADS)
        zero[z] = 0.f;
    __shared__ float part[THIN_WAVES * NF * 16 * 64];  // [wavefront][column block][accumulator][lane]
    thin_workgroup<NF, THIN_WAVES>(X, C, G, M, N, K, x_g, c_g, o_g, blockIdx.x * THIN_ROWS, blockIdx.y, part);
}

}  // namespace phantom

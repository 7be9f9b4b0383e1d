// Memory-bound helpers of the phantom layer: local error, bias gradient,
// in-memory reduce-scatter, MSE output error, SGD update.
#pragma once
#include "common.h"

namespace phantom {

// delta = dY * sigma'(S)   (Eq. (deltaL); the sigma' factor of Eq. (backprop)).
// S is the pre-activation (any activation) or, for ReLU, the layer output.
template <typename T>
__global__ __launch_bounds__(256) void delta_kernel(const T *__restrict__ dY, const T *__restrict__ S,
                                                   T *__restrict__ delta, int64_t count, int act)
{
    int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    for (; i < count; i += stride) {
        float d = to_f32(dY[i]);
        if (act != ACT_IDENTITY) d *= act_deriv(act, to_f32(S[i]));
        delta[i] = from_f32<T>(d);
    }
}

// The loss of a step is left as partial sums (one per workgroup of the output-error kernel, or one per tile of
// the last layer's product); a launch of its own for adding up to 1024 of them costs 4 us, so the first
// memory-bound kernel that follows in the stream carries the sum as a rider: one of its workgroups (all
// 256 threads) calls finish_loss, which adds the partial sums in a fixed order into loss = scale * sum.
struct LossTail {
    const float *partial;    // NULL: nothing to do
    int n;
    float scale;
    float *loss;
};

// lred: 256 floats of LDS that nothing else uses meanwhile
__device__ __forceinline__ void finish_loss(const LossTail &t, float *lred)
{
    // 256 threads do the work; a larger workgroup's other threads only keep the barriers company
    const int me = threadIdx.x;
    if (me < 256) {
        float acc = 0.f;
        for (int i = me; i < t.n; i += 256) acc += t.partial[i];
        lred[me] = acc;
    }
    __syncthreads();
    for (int w = 128; w > 0; w >>= 1) {
        if (me < w) lred[me] += lred[me + w];
        __syncthreads();
    }
    if (me == 0) *t.loss = lred[0] * t.scale;
}

__global__ __launch_bounds__(256) void loss_kernel(LossTail t)
{
    __shared__ float lred[256];
    finish_loss(t, lred);
}

// Column sums of delta [rows x cols] (Eq. (bpb): dLoss/db = sum over the batch of delta).  One workgroup
// owns CSUM_COLS columns of one group and rows [chunk*rows_per_chunk, ...): 16-byte loads, row lanes x
// column lanes, one LDS reduction at the end.  With one chunk the result is stored (deterministic);
// with several chunks (few columns, many rows) each adds its part atomically into the cleared output.
// Rider (step only): workgroup (0,0,0) also finishes the loss (see LossTail).
constexpr int CSUM_COLS = 128;
template <typename T>
__global__ __launch_bounds__(256) void colsum_kernel(const T *__restrict__ delta, float *__restrict__ out, int rows, int cols,
                                                    int rows_per_chunk, LossTail tail)
{
    constexpr int VEC = 16 / (int)sizeof(T);            // elements per 16-byte load
    constexpr int CL = CSUM_COLS / VEC;                 // column lanes
    constexpr int RL = 256 / CL;                        // row lanes
    __shared__ float red[RL][CSUM_COLS + 1];
    const int g = blockIdx.y;
    const int cl = threadIdx.x % CL, rl = threadIdx.x / CL;
    const int col = blockIdx.x * CSUM_COLS + cl * VEC;
    const T *d = delta + (int64_t)g * rows * cols;
    const int r_begin = blockIdx.z * rows_per_chunk;
    const int r_end = min(rows, r_begin + rows_per_chunk);
    float acc[VEC];
#pragma unroll
    for (int v = 0; v < VEC; ++v) acc[v] = 0.f;
    if (col + VEC <= cols && (cols % VEC) == 0) {
        for (int r = r_begin + rl; r < r_end; r += RL) {
            const uint4 raw = *(const uint4 *)(d + (int64_t)r * cols + col);
            const T *e = (const T *)&raw;
#pragma unroll
            for (int v = 0; v < VEC; ++v) acc[v] += to_f32(e[v]);
        }
    } else {
        for (int r = r_begin + rl; r < r_end; r += RL)
#pragma unroll
            for (int v = 0; v < VEC; ++v)
                if (col + v < cols) acc[v] += to_f32(d[(int64_t)r * cols + col + v]);
    }
#pragma unroll
    for (int v = 0; v < VEC; ++v) red[rl][cl * VEC + v] = acc[v];
    __syncthreads();
    if (threadIdx.x < CSUM_COLS) {
        const int c = blockIdx.x * CSUM_COLS + threadIdx.x;
        float sum = 0.f;
#pragma unroll
        for (int r = 0; r < RL; ++r) sum += red[r][threadIdx.x];
        if (c < cols) {
            if (gridDim.z == 1) out[(int64_t)g * cols + c] = sum;
            else unsafeAtomicAdd(out + (int64_t)g * cols + c, sum);
        }
    }
    __shared__ float lred[256];
    if (tail.partial && blockIdx.x == 0 && blockIdx.y == 0 && blockIdx.z == 0) finish_loss(tail, lred);      // uniform
}

// In-memory Reduce-Scatter of Algorithm 1's backward: dg_own[i] = sum_{j != i} dG_send[j][slot of i on j].
// dG_send [p, p-1, B*k], dg_own [p, B*k]; on holder j, source i sits in slot i (i < j) or i-1 (i > j).
// A workgroup owns 32 * VEC consecutive elements of one receiver: thread = (element vector, sender lane);
// sender lane g adds the senders g, g + 8, g + 16, ... in fp32, the eight partial sums are added in lane
// order through LDS (a fixed order, whatever p is).  With one thread walking all p-1 senders the kernel
// was bound by the latency of its own loads (33 MB in 24 us at p = 64).  Workgroup (0,0) may carry the
// loss rider (LossTail).
constexpr int RS_LANES = 8;
template <typename T, int VEC>
__global__ __launch_bounds__(256) void reduce_scatter_kernel(const T *__restrict__ dG_send, T *__restrict__ dg_own,
                                                            int p, int64_t per_slot, LossTail tail)
{
    typedef T TV __attribute__((ext_vector_type(VEC)));
    // part[lane][u * 40 + ev]: element u of vector ev.  A wavefront writes 32 consecutive words per sender lane, its
    // two sender lanes 32 banks apart; the 64 threads of a wavefront read 8 u-rows x 8 vectors, and the rows start
    // 40 words = 8 banks mod 64 apart in a permuted order (with rows of 32 * VEC + 1 words indexed [ev * VEC + u]
    // the writes met each bank four times: SQ_LDS_BANK_CONFLICT 448 cycles per workgroup, now 64)
    constexpr int RS_U_PITCH = 40, RS_LANE_PITCH = VEC * RS_U_PITCH + 32;
    __shared__ float part[RS_LANES * RS_LANE_PITCH];
    const int ev = threadIdx.x & 31, lane = threadIdx.x >> 5;
    const int64_t e = ((int64_t)blockIdx.x * 32 + ev) * VEC;
    const int i = blockIdx.y;
    float acc[VEC];
#pragma unroll
    for (int u = 0; u < VEC; ++u) acc[u] = 0.f;
    if (e < per_slot) {
        for (int j = lane; j < p; j += RS_LANES) {
            if (j == i) continue;
            const int slot = i < j ? i : i - 1;
            const T *src = dG_send + ((int64_t)j * (p - 1) + slot) * per_slot + e;
            if constexpr (VEC > 1) {
                const TV v = *(const TV *)src;
#pragma unroll
                for (int u = 0; u < VEC; ++u) acc[u] += to_f32((T)v[u]);
            } else {
                acc[0] += to_f32(src[0]);
            }
        }
    }
#pragma unroll
    for (int u = 0; u < VEC; ++u) part[lane * RS_LANE_PITCH + u * RS_U_PITCH + ev] = acc[u];
    __syncthreads();
    // 256 threads, 32 * VEC elements: thread t finishes elements t, t + 256, ...
    for (int c = threadIdx.x; c < 32 * VEC; c += 256) {
        const int64_t at = (int64_t)blockIdx.x * 32 * VEC + c;
        if (at >= per_slot) continue;
        float sum = 0.f;
#pragma unroll
        for (int g = 0; g < RS_LANES; ++g) sum += part[g * RS_LANE_PITCH + (c % VEC) * RS_U_PITCH + c / VEC];
        dg_own[(int64_t)i * per_slot + at] = from_f32<T>(sum);
    }
    __shared__ float lred[256];
    if (tail.partial && blockIdx.x == 0 && blockIdx.y == 0) finish_loss(tail, lred);      // uniform; rider, see LossTail
}

// MSE output error (Section IV-B, "Local error at the output", Eq. (deltaL)):
// delta_L = ((Y - T) / B) * sigma'(S) with one rounding (Eq. (deltaL) for the MSE loss), and one partial
// sum of (Y - T)^2 per workgroup (added up by the rider of colsum_kernel).  S: pre-activation, or the
// output for ReLU (s_kind 0: storage type, 1: float), or sigma'(pre-activation) itself in float
// (s_kind 2).  VEC elements per thread and iteration (VEC > 1: count is a multiple of VEC and
// every pointer is VEC-element aligned).
// Rider: the kernel also clears `zero_count` floats at `zero` (the step's bias-gradient buffers, which later
// launches add into), a launch of its own otherwise.
template <typename T, int VEC>
__global__ __launch_bounds__(256) void mse_delta_kernel(const T *__restrict__ Y, const T *__restrict__ Tg,
                                                       const void *__restrict__ S, int s_kind, T *__restrict__ delta,
                                                       int64_t count, float inv_b, int act,
                                                       float *__restrict__ partial, float *__restrict__ zero,
                                                       int64_t zero_count)
{
    for (int64_t z = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; z < zero_count; z += (int64_t)gridDim.x * blockDim.x)
        zero[z] = 0.f;
    typedef T TV __attribute__((ext_vector_type(VEC)));
    typedef float FV __attribute__((ext_vector_type(VEC)));
    __shared__ float red[256];
    int64_t i = ((int64_t)blockIdx.x * blockDim.x + threadIdx.x) * VEC;
    const int64_t stride = (int64_t)gridDim.x * blockDim.x * VEC;
    float acc = 0.f;
    for (; i < count; i += stride) {
        TV y, t, o;
        FV sv;
        if constexpr (VEC > 1) {
            y = *(const TV *)(Y + i);
            t = *(const TV *)(Tg + i);
            if (act != ACT_IDENTITY) {
                if (s_kind == 1 || s_kind == 2) {
                    sv = *(const FV *)((const float *)S + i);
                } else {
                    const TV sraw = *(const TV *)((const T *)S + i);
#pragma unroll
                    for (int u = 0; u < VEC; ++u) sv[u] = to_f32((T)sraw[u]);
                }
            }
        } else {
            y[0] = Y[i]; t[0] = Tg[i];
            if (act != ACT_IDENTITY)
                sv[0] = s_kind != 0 ? ((const float *)S)[i] : to_f32(((const T *)S)[i]);
        }
#pragma unroll
        for (int u = 0; u < VEC; ++u) {
            const float d = to_f32((T)y[u]) - to_f32((T)t[u]);
            acc += d * d;
            float e = d * inv_b;
            if (act != ACT_IDENTITY) e *= s_kind == 2 ? sv[u] : act_deriv(act, sv[u]);
            o[u] = from_f32<T>(e);
        }
        if constexpr (VEC > 1) *(TV *)(delta + i) = o;
        else delta[i] = o[0];
    }
    red[threadIdx.x] = acc;
    __syncthreads();
    for (int w = 128; w > 0; w >>= 1) {
        if ((int)threadIdx.x < w) red[threadIdx.x] += red[threadIdx.x + w];
        __syncthreads();
    }
    if (threadIdx.x == 0) partial[blockIdx.x] = red[0];
}

// SGD on the (up to four) parameter tensors of one layer in one launch; blockIdx.y picks the tensor.
// fp32 storage: w -= lr * g.  bf16 storage: master -= lr * g, w = bf16(master).
// Four elements per thread and iteration where the count allows (every pointer is 16-byte aligned).
struct SgdTensor {
    void *w;             // storage-type weights
    float *master;       // bf16 storage: fp32 master copy
    const float *grad;
    int64_t count;
};
struct SgdBatch {
    SgdTensor t[4];
    LossTail tail;       // rider for workgroup (0,0), see LossTail
};

// one tensor's update by workgroup `job` of `jobs` (all of the workgroup's `threads` threads)
template <typename T>
__device__ __forceinline__ void sgd_tensor(const SgdTensor &t, float lr, int job, int jobs, int threads)
{
    typedef float F4 __attribute__((ext_vector_type(4)));
    typedef T T4 __attribute__((ext_vector_type(4)));
    int64_t i = (int64_t)job * threads + threadIdx.x;
    const int64_t stride = (int64_t)jobs * threads;
    if ((t.count & 3) == 0) {                          // uniform
        for (const int64_t quads = t.count >> 2; i < quads; i += stride) {
            const F4 gr = ((const F4 *)t.grad)[i];
            if constexpr (sizeof(T) == 4) {
                F4 *w = (F4 *)t.w;
                w[i] = w[i] - lr * gr;
            } else {
                const F4 m = ((const F4 *)t.master)[i] - lr * gr;
                ((F4 *)t.master)[i] = m;
                T4 o;
#pragma unroll
                for (int u = 0; u < 4; ++u) o[u] = from_f32<T>(m[u]);
                ((T4 *)t.w)[i] = o;
            }
        }
        return;
    }
    for (; i < t.count; i += stride) {
        const float gr = t.grad[i];
        if constexpr (sizeof(T) == 4) {
            float *w = (float *)t.w;
            w[i] = w[i] - lr * gr;
        } else {
            const float m = t.master[i] - lr * gr;
            t.master[i] = m;
            ((T *)t.w)[i] = from_f32<T>(m);
        }
    }
}

template <typename T>
__global__ __launch_bounds__(256) void sgd_kernel(SgdBatch batch, float lr)
{
    // fixed-index copies selected by value: indexing the argument block with blockIdx.y would make
    // every access a dependent load
    SgdTensor t = batch.t[0];
    if (blockIdx.y == 1) t = batch.t[1];
    if (blockIdx.y == 2) t = batch.t[2];
    if (blockIdx.y == 3) t = batch.t[3];
    __shared__ float lred[256];
    if (batch.tail.partial && blockIdx.x == 0 && blockIdx.y == 0) finish_loss(batch.tail, lred);      // uniform
    sgd_tensor<T>(t, lr, blockIdx.x, gridDim.x, 256);
}

// The same update as a few workgroups of another launch (workgroup `job` of `jobs`): every tensor in turn.
template <typename T>
__device__ __forceinline__ void sgd_rider(const SgdBatch &batch, float lr, int job, int jobs, int threads, float *lred)
{
    if (batch.tail.partial && job == 0) finish_loss(batch.tail, lred);      // uniform
#pragma unroll
    for (int i = 0; i < 4; ++i)
        if (batch.t[i].count > 0) sgd_tensor<T>(batch.t[i], lr, job, jobs, threads);
}

__global__ __launch_bounds__(256) void fill_zero_kernel(float *__restrict__ dst, int64_t count)
{
    int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    for (; i < count; i += stride) dst[i] = 0.f;
}

template <typename T>
__global__ __launch_bounds__(256) void copy_kernel(const T *__restrict__ src, T *__restrict__ dst, int64_t count)
{
    int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    for (; i < count; i += stride) dst[i] = src[i];
}

}  // namespace phantom

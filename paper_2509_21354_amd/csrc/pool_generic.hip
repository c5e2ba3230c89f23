// Chunk aggregation, Eq. 2 of the paper: mean of the chunk's C rows, then the
// d -> d_sum -> d MLP with exact GELU, for keys and values with their own
// weights.  Generic fp32-arithmetic kernel for any storage dtype and any d_sum:
// one workgroup per (sequence, chunk).  The bf16 fast path lives in
// pool_mfma.hip; this one serves fp32 storage and shapes the MFMA tiling does
// not cover.
#include "common.hpp"
#include "kernels.hpp"

namespace kvev {

template <typename T, int D>
__global__ __launch_bounds__(256) void pool_generic_kernel(PoolArgs a)
{
    constexpr int EPL = D / 16;
    extern __shared__ float smem[];
    float *red = smem;                    // [16][2][D] per-group partial sums
    float *mean = red + 16 * 2 * D;       // [2][D]
    float *act = mean + 2 * D;            // [2][d_sum]

    const int tid = threadIdx.x, grp = tid >> 4, cl = tid & 15;
    const int nchunks = a.c1 - a.c0;
    const int s = blockIdx.x / nchunks;
    const int c = a.c0 + blockIdx.x % nchunks;
    const int l = s / a.BH;

    const T *Kp = static_cast<const T *>(a.K) + ((size_t)s * a.T_cap + (size_t)c * a.C) * D;
    const T *Vp = static_cast<const T *>(a.V) + ((size_t)s * a.T_cap + (size_t)c * a.C) * D;
    const bool is_max = a.mode == KVEV_POOL_MAX;     // element-wise maximum instead of the mean
    T *Kb = static_cast<T *>(a.Kbar) + ((size_t)s * a.N_cap + c) * D;
    T *Vb = static_cast<T *>(a.Vbar) + ((size_t)s * a.N_cap + c) * D;
    const int ds = a.d_sum;
    if (a.mode == KVEV_POOL_TOKEN_MLP) {
        // the MLP on every token, outputs averaged; layer 2 is linear, so the average is taken over the
        // hidden activations: a 16-lane group keeps one W1 row in registers and walks the chunk's tokens
        for (int o = grp; o < 2 * ds; o += 16) {
            const int kv = o / ds, u = o % ds;
            const T *W1 = static_cast<const T *>(kv ? a.W1V : a.W1K) + ((size_t)l * ds + u) * D;
            const float b1 = Storage<T>::load(static_cast<const T *>(kv ? a.b1V : a.b1K) + (size_t)l * ds + u);
            float w[EPL];
#pragma unroll
            for (int e = 0; e < EPL; ++e) w[e] = Storage<T>::load(W1 + cl + 16 * e);
            const T *X = kv ? Vp : Kp;
            float total = 0.f;
            for (int j = 0; j < a.C; ++j) {
                float acc = 0.f;
#pragma unroll
                for (int e = 0; e < EPL; ++e) acc = fmaf(w[e], Storage<T>::load(X + (size_t)j * D + cl + 16 * e), acc);
                total += gelu_erf(group16_sum(acc) + b1);
            }
            if (cl == 0) act[kv * ds + u] = total / (float)a.C;
        }
        __syncthreads();
    } else {
    float ak[EPL], av[EPL];
#pragma unroll
    for (int e = 0; e < EPL; ++e) ak[e] = av[e] = is_max ? -INFINITY : 0.f;
    for (int j = grp; j < a.C; j += 16) {
        float x[EPL], y[EPL];
        VecLoad<T, EPL>::run(Kp + (size_t)j * D + cl * EPL, x);
        VecLoad<T, EPL>::run(Vp + (size_t)j * D + cl * EPL, y);
#pragma unroll
        for (int e = 0; e < EPL; ++e) {
            ak[e] = is_max ? fmaxf(ak[e], x[e]) : ak[e] + x[e];
            av[e] = is_max ? fmaxf(av[e], y[e]) : av[e] + y[e];
        }
    }
#pragma unroll
    for (int e = 0; e < EPL; ++e) {
        red[(grp * 2 + 0) * D + cl * EPL + e] = ak[e];
        red[(grp * 2 + 1) * D + cl * EPL + e] = av[e];
    }
    __syncthreads();
    for (int i = tid; i < 2 * D; i += 256) {
        const int kv = i / D, e = i % D;
        float sum = is_max ? -INFINITY : 0.f;
#pragma unroll
        for (int g = 0; g < 16; ++g) sum = is_max ? fmaxf(sum, red[(g * 2 + kv) * D + e]) : sum + red[(g * 2 + kv) * D + e];
        mean[i] = is_max ? sum : sum / (float)a.C;
    }
    __syncthreads();

    if (a.mode != KVEV_POOL_MLP) {
        for (int i = tid; i < 2 * D; i += 256) Storage<T>::store((i < D ? Kb : Vb) + (i % D), mean[i]);
        return;
    }

    // layer 1: 2*d_sum dot products of length D, one per 16-lane group at a time
    for (int o = grp; o < 2 * ds; o += 16) {
        const int kv = o / ds, u = o % ds;
        const T *W1 = static_cast<const T *>(kv ? a.W1V : a.W1K) + ((size_t)l * ds + u) * D;
        float acc = 0.f;
        for (int e = cl; e < D; e += 16) acc = fmaf(Storage<T>::load(W1 + e), mean[kv * D + e], acc);
        acc = group16_sum(acc);
        if (cl == 0) {
            const T *b1 = static_cast<const T *>(kv ? a.b1V : a.b1K) + (size_t)l * ds;
            act[kv * ds + u] = gelu_erf(acc + Storage<T>::load(b1 + u));
        }
    }
    __syncthreads();
    }
    // layer 2: 2*D dot products of length d_sum
    for (int o = grp; o < 2 * D; o += 16) {
        const int kv = o / D, e = o % D;
        const T *W2 = static_cast<const T *>(kv ? a.W2V : a.W2K) + ((size_t)l * D + e) * ds;
        float acc = 0.f;
        for (int u = cl; u < ds; u += 16) acc = fmaf(Storage<T>::load(W2 + u), act[kv * ds + u], acc);
        acc = group16_sum(acc);
        if (cl == 0) {
            const T *b2 = static_cast<const T *>(kv ? a.b2V : a.b2K) + (size_t)l * D;
            Storage<T>::store((kv ? Vb : Kb) + e, acc + Storage<T>::load(b2 + e));
        }
    }
}

template <typename T, int D>
static hipError_t launch_t(const PoolArgs &a, hipStream_t st)
{
    const size_t blocks = (size_t)a.L * a.BH * (a.c1 - a.c0);
    if (blocks == 0) return hipSuccess;
    const size_t lds = sizeof(float) * (16 * 2 * D + 2 * D + 2 * (size_t)a.d_sum);
    hipLaunchKernelGGL((pool_generic_kernel<T, D>), dim3((unsigned)blocks), dim3(256), lds, st, a);
    return hipGetLastError();
}

hipError_t launch_pool_generic(const PoolArgs &a, int dtype, hipStream_t st)
{
    if (dtype == KVEV_F32) return a.d == 64 ? launch_t<float, 64>(a, st) : launch_t<float, 128>(a, st);
    return a.d == 64 ? launch_t<bf16_t, 64>(a, st) : launch_t<bf16_t, 128>(a, st);
}

}  // namespace kvev

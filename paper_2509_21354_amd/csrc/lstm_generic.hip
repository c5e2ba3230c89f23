// Recurrent gate, Eq. 3 of the paper: a standard LSTM cell (gate rows i,f,g,o)
// over the chunk summaries [Kbar_t ; Vbar_t] with a scalar utility head on h_t.
// Generic fp32-arithmetic kernel for any storage dtype and any d_g: one
// workgroup walks one sequence through its steps; the input projection is
// fused, so no workspace is used.  The bf16 fast path lives in lstm_mfma.hip.
#include "common.hpp"
#include "kernels.hpp"

namespace kvev {

template <typename T, int D>
__global__ __launch_bounds__(256) void lstm_generic_kernel(LstmArgs a)
{
    extern __shared__ float smem[];
    const int dg = a.d_g, G = 4 * dg;
    float *x = smem;            // [2D]
    float *h = x + 2 * D;       // [d_g]
    float *c = h + dg;          // [d_g]
    float *pre = c + dg;        // [4 d_g]

    const int tid = threadIdx.x, grp = tid >> 4, cl = tid & 15;
    const int s = blockIdx.x, l = s / a.BH;
    const T *W_ih = static_cast<const T *>(a.W_ih) + (size_t)l * G * 2 * D;
    const T *W_hh = static_cast<const T *>(a.W_hh) + (size_t)l * G * dg;
    const T *b_ih = static_cast<const T *>(a.b_ih) + (size_t)l * G;
    const T *b_hh = static_cast<const T *>(a.b_hh) + (size_t)l * G;
    const T *w_s = static_cast<const T *>(a.w_s) + (size_t)l * dg;
    const float b_s = Storage<T>::load(static_cast<const T *>(a.b_s) + l);

    const bool fresh = a.c0 == 0;        // the recurrence starts from a zero state at chunk 0, whatever the buffers hold
    for (int j = tid; j < dg; j += 256) {
        h[j] = fresh ? 0.f : a.h[(size_t)s * dg + j];
        c[j] = fresh ? 0.f : a.c[(size_t)s * dg + j];
    }
    for (int t = a.c0; t < a.c1; ++t) {
        const size_t row = ((size_t)s * a.N_cap + t) * D;
        for (int e = tid; e < 2 * D; e += 256)
            x[e] = Storage<T>::load((e < D ? static_cast<const T *>(a.Kbar) : static_cast<const T *>(a.Vbar)) + row + (e % D));
        __syncthreads();
        for (int r = grp; r < G; r += 16) {
            float acc = 0.f;
            const T *wi = W_ih + (size_t)r * 2 * D;
            for (int e = cl; e < 2 * D; e += 16) acc = fmaf(Storage<T>::load(wi + e), x[e], acc);
            const T *wh = W_hh + (size_t)r * dg;
            for (int j = cl; j < dg; j += 16) acc = fmaf(Storage<T>::load(wh + j), h[j], acc);
            acc = group16_sum(acc);
            if (cl == 0) pre[r] = acc + Storage<T>::load(b_ih + r) + Storage<T>::load(b_hh + r);
        }
        __syncthreads();
        for (int j = tid; j < dg; j += 256) {
            const float ig = 1.f / (1.f + expf(-pre[j]));
            const float fg = 1.f / (1.f + expf(-pre[dg + j]));
            const float gg = tanhf(pre[2 * dg + j]);
            const float og = 1.f / (1.f + expf(-pre[3 * dg + j]));
            const float cn = fg * c[j] + ig * gg;
            c[j] = cn;
            h[j] = og * tanhf(cn);
        }
        __syncthreads();
        if (tid < kWave) {
            float u = 0.f;
            for (int j = tid; j < dg; j += kWave) u = fmaf(Storage<T>::load(w_s + j), h[j], u);
#pragma unroll
            for (int off = 32; off >= 1; off >>= 1) u += __shfl_xor(u, off);
            if (tid == 0) {
                u += b_s;
                a.util[(size_t)s * a.N_cap + t] = u;
                a.gate[(size_t)s * a.N_cap + t] = 1.f / (1.f + expf(-u));
            }
        }
    }
    __syncthreads();
    for (int j = tid; j < dg; j += 256) {
        a.h[(size_t)s * dg + j] = h[j];
        a.c[(size_t)s * dg + j] = c[j];
    }
}

template <typename T, int D>
static hipError_t launch_t(const LstmArgs &a, hipStream_t st)
{
    const size_t S = (size_t)a.L * a.BH;
    if (S == 0 || a.c1 == a.c0) return hipSuccess;
    const size_t lds = sizeof(float) * (2 * D + 6 * (size_t)a.d_g);
    hipLaunchKernelGGL((lstm_generic_kernel<T, D>), dim3((unsigned)S), dim3(256), lds, st, a);
    return hipGetLastError();
}

hipError_t launch_lstm_generic(const LstmArgs &a, int dtype, hipStream_t st)
{
    if (dtype == KVEV_F32) return a.d == 64 ? launch_t<float, 64>(a, st) : launch_t<float, 128>(a, st);
    return a.d == 64 ? launch_t<bf16_t, 64>(a, st) : launch_t<bf16_t, 128>(a, st);
}

}  // namespace kvev

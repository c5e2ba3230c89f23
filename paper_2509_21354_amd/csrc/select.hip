// Retention: top-k by utility (or the threshold rule of section 3.2) over the
// candidate chunks of one sequence.  One workgroup of four wavefronts per
// sequence: the scores sit in LDS, every lane ranks its own candidate by
// counting the candidates that beat it under the strict order (utility
// descending, index ascending), and the kept indices are compacted in
// ascending order with a ballot per wave and a prefix over the wave counts.
// Integer output, exact by construction.
#include "common.hpp"
#include "kernels.hpp"

namespace kvev {

__global__ __launch_bounds__(256) void select_kernel(SelectArgs a)
{
    extern __shared__ float s_key[];
    __shared__ int s_cnt[4];
    const int s = blockIdx.x, tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const float *src = (a.mode == KVEV_SELECT_TOPK ? a.util : a.gate) + (size_t)s * a.N_cap;
    for (int c = tid; c < a.n_cand; c += 256) {
        float u = src[c];
        if (a.mode == KVEV_SELECT_TOPK && u != u) u = -INFINITY;   // NaN ranks last
        s_key[c] = u;
    }
    __syncthreads();
    int32_t *out = a.idx + (size_t)s * a.k_cap;
    int base = 0;
    for (int c0 = 0; c0 < a.n_cand; c0 += 256) {
        const int c = c0 + tid;
        bool keep = false;
        if (c < a.n_cand) {
            const float u = s_key[c];
            if (a.mode == KVEV_SELECT_TOPK) {
                // rank = candidates that beat this one; 4 independent LDS reads per trip
                int rank = 0, j = 0;
                for (; j + 4 <= a.n_cand; j += 4) {
                    const float u0 = s_key[j], u1 = s_key[j + 1], u2 = s_key[j + 2], u3 = s_key[j + 3];
                    rank += (u0 > u || (u0 == u && j < c)) ? 1 : 0;
                    rank += (u1 > u || (u1 == u && j + 1 < c)) ? 1 : 0;
                    rank += (u2 > u || (u2 == u && j + 2 < c)) ? 1 : 0;
                    rank += (u3 > u || (u3 == u && j + 3 < c)) ? 1 : 0;
                }
                for (; j < a.n_cand; ++j) {
                    const float uj = s_key[j];
                    rank += (uj > u || (uj == u && j < c)) ? 1 : 0;
                }
                keep = rank < a.k;
            } else {
                keep = u >= a.tau;
            }
        }
        const unsigned long long mask = __ballot(keep);
        if (lane == 0) s_cnt[wave] = __popcll(mask);
        __syncthreads();
        int before = base;
        for (int w = 0; w < wave; ++w) before += s_cnt[w];
        if (keep) {
            const int pos = before + __popcll(mask & ((1ull << lane) - 1ull));
            if (pos < a.k_cap) out[pos] = c;
        }
        base += s_cnt[0] + s_cnt[1] + s_cnt[2] + s_cnt[3];
        __syncthreads();
    }
    if (tid == 0) a.count[s] = min(base, a.k_cap);
}

hipError_t launch_select(const SelectArgs &a, hipStream_t st)
{
    if (a.S == 0) return hipSuccess;
    const size_t lds = (size_t)(a.n_cand > 0 ? a.n_cand : 1) * sizeof(float);
    hipLaunchKernelGGL(select_kernel, dim3(a.S), dim3(256), lds, st, a);
    return hipGetLastError();
}

}  // namespace kvev

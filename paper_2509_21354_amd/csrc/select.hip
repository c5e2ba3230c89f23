// Retention: top-k by utility (or the threshold rule of section 3.2) over the
// candidate chunks of one sequence.  One wavefront per sequence: the scores sit
// in LDS, every lane ranks its own candidate by counting the candidates that
// beat it under the strict order (utility descending, index ascending), and the
// kept indices are compacted in ascending order with a ballot and a prefix
// popcount.  Integer output, exact by construction.
#include "common.hpp"
#include "kernels.hpp"

namespace kvev {

__global__ __launch_bounds__(64) void select_kernel(SelectArgs a)
{
    extern __shared__ float s_key[];
    const int s = blockIdx.x, lane = threadIdx.x;
    const float *src = (a.mode == KVEV_SELECT_TOPK ? a.util : a.gate) + (size_t)s * a.N_cap;
    for (int c = lane; c < a.n_cand; c += kWave) {
        float u = src[c];
        if (a.mode == KVEV_SELECT_TOPK && u != u) u = -INFINITY;   // NaN ranks last
        s_key[c] = u;
    }
    __syncthreads();
    int32_t *out = a.idx + (size_t)s * a.k_cap;
    int base = 0;
    for (int c0 = 0; c0 < a.n_cand; c0 += kWave) {
        const int c = c0 + lane;
        bool keep = false;
        if (c < a.n_cand) {
            const float u = s_key[c];
            if (a.mode == KVEV_SELECT_TOPK) {
                int rank = 0;
                for (int j = 0; j < a.n_cand; ++j) {
                    const float uj = s_key[j];
                    rank += (uj > u || (uj == u && j < c)) ? 1 : 0;
                }
                keep = rank < a.k;
            } else {
                keep = u >= a.tau;
            }
        }
        const unsigned long long mask = __ballot(keep);
        if (keep) {
            const int pos = base + __popcll(mask & ((1ull << lane) - 1ull));
            if (pos < a.k_cap) out[pos] = c;
        }
        base += __popcll(mask);
    }
    if (lane == 0) a.count[s] = min(base, a.k_cap);
}

hipError_t launch_select(const SelectArgs &a, hipStream_t st)
{
    if (a.S == 0) return hipSuccess;
    const size_t lds = (size_t)(a.n_cand > 0 ? a.n_cand : 1) * sizeof(float);
    hipLaunchKernelGGL(select_kernel, dim3(a.S), dim3(kWave), lds, st, a);
    return hipGetLastError();
}

}  // namespace kvev

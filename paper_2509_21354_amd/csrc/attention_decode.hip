// Decode attention (few queries per sequence): Eq. 1 of the paper evaluated
// over a row list that is either the whole cache (dense baseline) or the kept
// chunk summaries followed by the raw recent window (section 3.3, n' = W + M).
//
// The op moves 2*n*d elements per query and does 4*n*d flops: it is bound by
// HBM, so the kernel is a pure streaming design.  A 16-lane group owns one row
// at a time (one 16-byte load per lane covers a 128-wide bf16 row), a wave
// covers 4 consecutive rows per load instruction and a workgroup 16, so every
// wave-level load is one contiguous 1 KiB piece of the cache.  Each lane group
// keeps its own online-softmax state (m, l, o); the groups are merged by
// shuffles, the waves through LDS, and the splits of one sequence by a second,
// deterministic kernel (no float atomics).
#include "common.hpp"
#include "kernels.hpp"

namespace kvev {

constexpr float kNegBig = -1.0e30f;   // finite stand-in for -inf: exp2(kNegBig - x) == 0, no NaN

template <typename T, int D, int U>
__global__ __launch_bounds__(256) void attn_decode_kernel(AttnArgs a)
{
    constexpr int EPL = D / 16;
    const int tid = threadIdx.x;
    const int wave = tid >> 6;
    const int grp = tid >> 4;      // row group within the workgroup, 0..15
    const int cl = tid & 15;       // column lane within the group
    const int split = blockIdx.x % a.nsplit;
    const int sq = blockIdx.x / a.nsplit;
    const int s = sq / a.Tq;

    const T *K = static_cast<const T *>(a.K), *V = static_cast<const T *>(a.V);
    const T *Kbar = static_cast<const T *>(a.Kbar), *Vbar = static_cast<const T *>(a.Vbar);

    int cnt = 0;
    if (a.gated) cnt = min(max(a.count[s], 0), a.k_cap);
    const int n = cnt + (a.T - a.win0);
    const int j0 = split * a.rows_per_split;
    const int j1 = min(n, j0 + a.rows_per_split);

    float qv[EPL];
    {
        Raw<T, EPL> r;
        r.load(static_cast<const T *>(a.Q) + (size_t)sq * D + cl * EPL);
        r.get(qv);
#pragma unroll
        for (int e = 0; e < EPL; ++e) qv[e] *= a.scale_log2e;
    }

    float m = kNegBig, l = 0.f, o[EPL];
#pragma unroll
    for (int e = 0; e < EPL; ++e) o[e] = 0.f;

    const size_t seq_raw = (size_t)s * a.T_cap;
    const size_t seq_sum = (size_t)s * a.N_cap;
    const int32_t *idx = a.idx ? a.idx + (size_t)s * a.k_cap : nullptr;   // null: the store is compact, row j is entry j

    for (int base = j0; base < j1; base += 16 * U) {
        Raw<T, EPL> kr[U], vr[U];
        bool valid[U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            int j = base + grp + 16 * u;
            valid[u] = j < j1;
            j = valid[u] ? j : j1 - 1;
            size_t off;
            const T *kb, *vb;
            if (j < cnt) {
                int c = min(max(idx ? idx[j] : j, 0), a.N_cap - 1);
                off = (seq_sum + c) * D;
                kb = Kbar; vb = Vbar;
            } else {
                off = (seq_raw + a.win0 + (j - cnt)) * D;
                kb = K; vb = V;
            }
            kr[u].load(kb + off + cl * EPL);
            vr[u].load(vb + off + cl * EPL);
        }
        float sc[U];
        float mx = kNegBig;
#pragma unroll
        for (int u = 0; u < U; ++u) {
            float kv[EPL];
            kr[u].get(kv);
            float d = 0.f;
#pragma unroll
            for (int e = 0; e < EPL; ++e) d = fmaf(qv[e], kv[e], d);
            d = group16_sum(d);
            sc[u] = valid[u] ? d : kNegBig;
            mx = fmaxf(mx, sc[u]);
        }
        const float m_new = fmaxf(m, mx);
        const float alpha = exp2f(m - m_new);
        l *= alpha;
#pragma unroll
        for (int e = 0; e < EPL; ++e) o[e] *= alpha;
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const float p = valid[u] ? exp2f(sc[u] - m_new) : 0.f;
            float vv[EPL];
            vr[u].get(vv);
            l += p;
#pragma unroll
            for (int e = 0; e < EPL; ++e) o[e] = fmaf(p, vv[e], o[e]);
        }
        m = m_new;
    }

    // merge the 4 lane groups of the wave
#pragma unroll
    for (int off = 16; off <= 32; off <<= 1) {
        const float m2 = __shfl_xor(m, off), l2 = __shfl_xor(l, off);
        const float M = fmaxf(m, m2);
        const float a1 = exp2f(m - M), a2 = exp2f(m2 - M);
        l = l * a1 + l2 * a2;
#pragma unroll
        for (int e = 0; e < EPL; ++e) o[e] = o[e] * a1 + __shfl_xor(o[e], off) * a2;
        m = M;
    }

    __shared__ float s_m[4], s_l[4], s_o[4][D];
    if ((tid & 63) < 16) {
        if (cl == 0) { s_m[wave] = m; s_l[wave] = l; }
#pragma unroll
        for (int e = 0; e < EPL; ++e) s_o[wave][cl * EPL + e] = o[e];
    }
    __syncthreads();
    if (tid < D) {
        float M = fmaxf(fmaxf(s_m[0], s_m[1]), fmaxf(s_m[2], s_m[3]));
        float L = 0.f, acc = 0.f;
#pragma unroll
        for (int w = 0; w < 4; ++w) {
            const float f = exp2f(s_m[w] - M);
            L += s_l[w] * f;
            acc += s_o[w][tid] * f;
        }
        if (a.nsplit == 1) {
            Storage<T>::store(static_cast<T *>(a.O) + (size_t)sq * D + tid, L > 0.f ? acc / L : 0.f);
        } else {
            float *p = a.part + ((size_t)sq * a.nsplit + split) * (D + 2);
            p[tid] = acc;
            if (tid == 0) { p[D] = M; p[D + 1] = L; }
        }
    }
}

// Merge of the split partials (o[D], m, l) of one (sequence, query): a
// log-sum-exp combination in a fixed order (tree over lanes, then waves).  The
// splits' maxima and sums are reduced across the workgroup first, so that the
// D-wide accumulation only issues independent loads.
template <typename T, int D>
__global__ __launch_bounds__(D) void attn_combine_kernel(const float *part, int nsplit, T *O)
{
    extern __shared__ float s_w[];                 // [nsplit] weights exp2(m_i - M)
    __shared__ float s_red[2][D / 64];
    const int sq = blockIdx.x, t = threadIdx.x, wave = t >> 6;
    const float *p = part + (size_t)sq * nsplit * (D + 2);
    float mloc = kNegBig;
    for (int i = t; i < nsplit; i += D) mloc = fmaxf(mloc, p[(size_t)i * (D + 2) + D]);
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) mloc = fmaxf(mloc, __shfl_xor(mloc, off));
    if ((t & 63) == 0) s_red[0][wave] = mloc;
    __syncthreads();
    float M = s_red[0][0];
#pragma unroll
    for (int w = 1; w < D / 64; ++w) M = fmaxf(M, s_red[0][w]);
    float lloc = 0.f;
    for (int i = t; i < nsplit; i += D) {
        const float *pi = p + (size_t)i * (D + 2);
        const float f = exp2f(pi[D] - M);
        s_w[i] = f;
        lloc += pi[D + 1] * f;
    }
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) lloc += __shfl_xor(lloc, off);
    if ((t & 63) == 0) s_red[1][wave] = lloc;
    __syncthreads();
    float L = s_red[1][0];
#pragma unroll
    for (int w = 1; w < D / 64; ++w) L += s_red[1][w];
    float acc = 0.f;
    int i = 0;
    for (; i + 8 <= nsplit; i += 8) {
        float v[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) v[u] = p[(size_t)(i + u) * (D + 2) + t];
#pragma unroll
        for (int u = 0; u < 8; ++u) acc = fmaf(v[u], s_w[i + u], acc);
    }
    for (; i < nsplit; ++i) acc = fmaf(p[(size_t)i * (D + 2) + t], s_w[i], acc);
    Storage<T>::store(O + (size_t)sq * D + t, L > 0.f ? acc / L : 0.f);
}

template <typename T, int D>
static hipError_t launch_decode_t(const AttnArgs &a, hipStream_t st)
{
    constexpr int U = 4;
    const unsigned blocks = (unsigned)((size_t)a.S * a.Tq * a.nsplit);
    if (blocks == 0) return hipSuccess;
    hipLaunchKernelGGL((attn_decode_kernel<T, D, U>), dim3(blocks), dim3(256), 0, st, a);
    if (a.nsplit > 1)
        hipLaunchKernelGGL((attn_combine_kernel<T, D>), dim3((unsigned)((size_t)a.S * a.Tq)), dim3(D),
                           (size_t)a.nsplit * sizeof(float), st, a.part, a.nsplit, static_cast<T *>(a.O));
    return hipGetLastError();
}

hipError_t launch_attn_decode(const AttnArgs &a, int dtype, hipStream_t st)
{
    if (dtype == KVEV_F32) return a.d == 64 ? launch_decode_t<float, 64>(a, st) : launch_decode_t<float, 128>(a, st);
    return a.d == 64 ? launch_decode_t<bf16_t, 64>(a, st) : launch_decode_t<bf16_t, 128>(a, st);
}

}  // namespace kvev

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
// shuffles, the waves through LDS, and the splits of one sequence inside the
// same launch: every split leaves its partial (o, m, l) in scratch and draws an
// integer ticket; the workgroup that draws the last one merges all partials in
// split order (so the result does not depend on who arrives when, and no float
// atomics are involved) and puts the ticket back to zero.  A workgroup serves up
// to 4 queries that share the rows (the heads of a grouped-query group, a short
// frame).
#include "common.hpp"
#include "kernels.hpp"
#include <type_traits>

namespace kvev {

constexpr float kNegBig = -1.0e30f;   // finite stand-in for -inf: exp2(kNegBig - x) == 0, no NaN
constexpr int kMaxSplit = KVEV_ATTN_MAX_SPLIT;   // most splits per query (the host plans within it)

// Device-scope accesses for what workgroups on different XCDs hand each other: the store writes through the
// XCD's L2, the load reads past the caches that are not coherent across XCDs.
__device__ __forceinline__ void store_device(float *p, float v)
{
    __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ float load_device(const float *p)
{
    return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// Queries that share a key-value sequence: the Tq queries of each of the G query
// heads of its group (grouped-query attention), numbered r = g * Tq + tq.  Row of
// query r in Q / O [L,B,H,Tq,d] for key-value sequence s of [L,B,H_kv].
__device__ __forceinline__ size_t query_row(const AttnArgs &a, int s, int r)
{
    const int g = r / a.Tq, tq = r - g * a.Tq;
    const size_t head = (size_t)(s / a.Hkv) * ((size_t)a.Hkv * a.G) + (size_t)(s % a.Hkv) * a.G + g;
    return head * a.Tq + tq;
}

// NQ queries of one key-value sequence per workgroup: every row that is loaded
// serves all of them (what grouped-query heads and short query frames are for).
// NW waves per workgroup: 4 normally; 16 when the launch has no more workgroups than the chip has compute units
// (a short cache and few sequences: the rows of a sequence are then spread over four times the lanes).
template <typename T, int D, int U, int NQ, int NW>
__global__ __launch_bounds__(64 * NW) void attn_decode_kernel(AttnArgs a)
{
    constexpr int EPL = D / 16, GROUPS = 4 * NW;     // 16-lane row groups per workgroup
    const int tid = threadIdx.x;
    const int wave = tid >> 6;
    const int grp = tid >> 4;      // row group within the workgroup, 0 .. GROUPS-1
    const int cl = tid & 15;       // column lane within the group
    const int R = a.G * a.Tq;
    const int qgroups = (R + NQ - 1) / NQ;
    int blk = blockIdx.x;
    const int split = blk % a.nsplit; blk /= a.nsplit;
    const int qg = blk % qgroups;
    const int s = blk / qgroups;

    const T *K = static_cast<const T *>(a.K), *V = static_cast<const T *>(a.V);
    const T *Kbar = static_cast<const T *>(a.Kbar), *Vbar = static_cast<const T *>(a.Vbar);

    // The raw rows are cut into nsplit runs of rows_per_split; the kept summaries go with the first run.  The cut thus
    // depends on the raw rows alone, and the compact form (same raw rows, another capacity for the summaries) walks
    // and merges exactly as the indexed form does.  A workgroup takes its raw rows first: their addresses need
    // nothing from memory, so their loads leave together with those of the queries, the kept count and the first
    // chunk indices, and the summaries (whose addresses come out of the index list) follow one round trip later
    // instead of two.
    const int wlen = a.T - a.win0;
    const int w0 = split * a.rows_per_split;
    const int w1 = min(wlen, w0 + a.rows_per_split);
    const int32_t *idx = a.idx ? a.idx + (size_t)s * a.k_cap : nullptr;   // null: the store is compact, row j is entry j
    int cnt_raw = 0;
    if (a.gated && split == 0) cnt_raw = a.count[s];
    int idx0[U];                  // the chunk indices of this lane group's first batch of summaries, asked for early
#pragma unroll
    for (int u = 0; u < U; ++u) {
        const int j = grp + GROUPS * u;
        idx0[u] = a.gated && split == 0 && idx && a.k_cap > 0 ? idx[min(j, a.k_cap - 1)] : j;
    }

    // per query: its row in Q / O and the first raw row it must not see (causal frame: the queries are the
    // last Tq cached tokens and see nothing after their own position; a summary is older than every raw row)
    float qv[NQ][EPL];
    size_t qrow[NQ];
    int lim[NQ];
    bool qok[NQ];
#pragma unroll
    for (int i = 0; i < NQ; ++i) {
        const int r = qg * NQ + i;
        qok[i] = r < R;
        const int rc = qok[i] ? r : R - 1;
        qrow[i] = query_row(a, s, rc);
        lim[i] = qok[i] ? (a.causal ? wlen - (a.Tq - 1 - rc % a.Tq) : wlen) : -1;
        Raw<T, EPL> raw;
        raw.load(static_cast<const T *>(a.Q) + qrow[i] * D + cl * EPL);
        raw.get(qv[i]);
#pragma unroll
        for (int e = 0; e < EPL; ++e) qv[i][e] *= a.scale_log2e;
    }

    float m[NQ], l[NQ], o[NQ][EPL];
#pragma unroll
    for (int i = 0; i < NQ; ++i) {
        m[i] = kNegBig; l[i] = 0.f;
#pragma unroll
        for (int e = 0; e < EPL; ++e) o[i][e] = 0.f;
    }

    const size_t seq_raw = (size_t)s * a.T_cap;
    const size_t seq_sum = (size_t)s * a.N_cap;

    // One batch: U rows per lane group are loaded, scored against the NQ queries and folded into the running
    // softmax.  pos[u] is the row's position for the causal test: its raw index, -1 for a summary (visible to every
    // query), a huge value for a slot past the end.
    auto fold = [&](const Raw<T, EPL> (&kr)[U], const Raw<T, EPL> (&vr)[U], const int (&pos)[U]) {
        float sc[NQ][U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            float kv[EPL];
            kr[u].get(kv);
#pragma unroll
            for (int i = 0; i < NQ; ++i) {
                float d = 0.f;
#pragma unroll
                for (int e = 0; e < EPL; ++e) d = fmaf(qv[i][e], kv[e], d);
                d = group16_sum(d);
                sc[i][u] = pos[u] < lim[i] ? d : kNegBig;
            }
        }
        float alpha[NQ], p[NQ][U];
#pragma unroll
        for (int i = 0; i < NQ; ++i) {
            float mx = kNegBig;
#pragma unroll
            for (int u = 0; u < U; ++u) mx = fmaxf(mx, sc[i][u]);
            const float m_new = fmaxf(m[i], mx);
            alpha[i] = exp2f(m[i] - m_new);
            l[i] *= alpha[i];
#pragma unroll
            for (int u = 0; u < U; ++u) {
                p[i][u] = pos[u] < lim[i] ? exp2f(sc[i][u] - m_new) : 0.f;
                l[i] += p[i][u];
            }
            m[i] = m_new;
#pragma unroll
            for (int e = 0; e < EPL; ++e) o[i][e] *= alpha[i];
        }
#pragma unroll
        for (int u = 0; u < U; ++u) {
            float vv[EPL];
            vr[u].get(vv);
#pragma unroll
            for (int i = 0; i < NQ; ++i)
#pragma unroll
                for (int e = 0; e < EPL; ++e) o[i][e] = fmaf(p[i][u], vv[e], o[i][e]);
        }
    };
    constexpr int kPast = 0x3fffffff;

    // Rows are read once per launch.  When a launch reads more than the memory-side cache holds (a.stream), the loads
    // carry the non-temporal hint: nothing of it can be kept anyway, and the read stream runs 13 % faster without
    // the allocations.  Smaller launches keep plain loads, so that the next decode step finds its rows in cache.
    auto walk = [&](auto stream_tag) __attribute__((always_inline)) {
        constexpr bool STREAM = decltype(stream_tag)::value;
        // ---- raw rows w0 .. w1-1 of the window (of the whole cache for the dense baseline) ----
        for (int base = w0; base < w1; base += GROUPS * U) {
            Raw<T, EPL> kr[U], vr[U];
            int pos[U];
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const int w = base + grp + GROUPS * u;
                pos[u] = w < w1 ? w : kPast;
                int r = a.win0 + min(w, w1 - 1) + a.ring_first;       // (ring_first is 0 unless the raw buffer is a ring)
                r = r >= a.T_cap ? r - a.T_cap : r;
                const size_t off = (seq_raw + r) * D + cl * EPL;
                if (STREAM) { kr[u].load_stream(K + off); vr[u].load_stream(V + off); }
                else { kr[u].load(K + off); vr[u].load(V + off); }
            }
            fold(kr, vr, pos);
        }
        // ---- the kept summaries (first run only) ----
        const int cnt = min(max(cnt_raw, 0), a.k_cap);
        for (int base = 0; base < cnt; base += GROUPS * U) {
            Raw<T, EPL> kr[U], vr[U];
            int pos[U];
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const int j = base + grp + GROUPS * u;
                pos[u] = j < cnt ? -1 : kPast;
                const int jc = min(j, cnt - 1);
                // (idx0[u] is entry min(j, k_cap - 1) of the list: the right one whenever row j exists)
                int c = idx ? (base == 0 ? idx0[u] : idx[jc]) : jc;
                c = min(max(c, 0), a.N_cap - 1);
                const size_t off = (seq_sum + c) * D + cl * EPL;
                if (STREAM) { kr[u].load_stream(Kbar + off); vr[u].load_stream(Vbar + off); }
                else { kr[u].load(Kbar + off); vr[u].load(Vbar + off); }
            }
            fold(kr, vr, pos);
        }
    };
    if (a.stream) walk(std::true_type{}); else walk(std::false_type{});

    __shared__ float s_m[NQ][NW], s_l[NQ][NW], s_o[NQ][NW][D];
#pragma unroll
    for (int i = 0; i < NQ; ++i) {
        // merge the 4 lane groups of the wave
        float mi = m[i], li = l[i];
#pragma unroll
        for (int off = 16; off <= 32; off <<= 1) {
            const float m2 = __shfl_xor(mi, off), l2 = __shfl_xor(li, off);
            const float M = fmaxf(mi, m2);
            const float a1 = exp2f(mi - M), a2 = exp2f(m2 - M);
            li = li * a1 + l2 * a2;
#pragma unroll
            for (int e = 0; e < EPL; ++e) o[i][e] = o[i][e] * a1 + __shfl_xor(o[i][e], off) * a2;
            mi = M;
        }
        if ((tid & 63) < 16) {
            if (cl == 0) { s_m[i][wave] = mi; s_l[i][wave] = li; }
#pragma unroll
            for (int e = 0; e < EPL; ++e) s_o[i][wave][cl * EPL + e] = o[i][e];
        }
    }
    __syncthreads();
    if (tid < D) {
#pragma unroll
        for (int i = 0; i < NQ; ++i) {
            if (!qok[i]) continue;
            float M = s_m[i][0];
#pragma unroll
            for (int w = 1; w < NW; ++w) M = fmaxf(M, s_m[i][w]);
            float L = 0.f, acc = 0.f;
#pragma unroll
            for (int w = 0; w < NW; ++w) {
                const float f = exp2f(s_m[i][w] - M);
                L += s_l[i][w] * f;
                acc += s_o[i][w][tid] * f;
            }
            if (a.nsplit == 1) {
                Storage<T>::store(static_cast<T *>(a.O) + qrow[i] * D + tid, L > 0.f ? acc / L : 0.f);
            } else {
                float *pp = a.part + (((size_t)s * R + (qg * NQ + i)) * a.nsplit + split) * (D + 2);
                store_device(pp + tid, acc);
                if (tid == 0) { store_device(pp + D, M); store_device(pp + D + 1, L); }
            }
        }
    }
    if (a.nsplit == 1) return;

    // ---- the splits of these queries meet here: the last one to arrive merges them all ----
    // Partials and tickets travel with device-scope accesses (stores that write through the XCD's L2, loads that
    // read past it), so no cache has to be written back or invalidated as a whole.  A workgroup waits until its
    // partial stores are acknowledged, then draws its ticket; the workgroup that draws number nsplit - 1 therefore
    // knows that all partials are in memory.  The merge walks the splits in their own order, whoever arrived last.
    __shared__ int s_last;
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");       // this thread's stores have completed
    __syncthreads();
    int32_t *ticket = a.tickets + ((size_t)s * qgroups + qg);
    if (tid == 0)
        s_last = __hip_atomic_fetch_add(ticket, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) == a.nsplit - 1;
    __syncthreads();
    if (!s_last) return;
    // the splits' maxima and sums first, one (query, split) per thread: a single round trip for all of them
    __shared__ float s_pm[NQ][kMaxSplit], s_pl[NQ][kMaxSplit];
    for (int e = tid; e < NQ * a.nsplit; e += 64 * NW) {
        const int i = e / a.nsplit, sp = e - i * a.nsplit;
        const int r = qg * NQ + i;
        if (r < R) {
            const float *ps = a.part + (((size_t)s * R + r) * a.nsplit + sp) * (D + 2);
            s_pm[i][sp] = load_device(ps + D);
            s_pl[i][sp] = load_device(ps + D + 1);
        }
    }
    __syncthreads();
    const int t = tid % D;
    for (int i = tid / D; i < NQ; i += 64 * NW / D) {
        const int r = qg * NQ + i;
        if (r >= R) break;
        const float *p = a.part + ((size_t)s * R + r) * a.nsplit * (D + 2) + t;
        float M = kNegBig;
        for (int sp = 0; sp < a.nsplit; ++sp) M = fmaxf(M, s_pm[i][sp]);
        float L = 0.f, acc = 0.f;
        for (int sp0 = 0; sp0 < a.nsplit; sp0 += 8) {
            float v[8];
#pragma unroll
            for (int u = 0; u < 8; ++u) v[u] = load_device(p + (size_t)min(sp0 + u, a.nsplit - 1) * (D + 2));
#pragma unroll
            for (int u = 0; u < 8; ++u) {
                if (sp0 + u < a.nsplit) {
                    const float f = exp2f(s_pm[i][sp0 + u] - M);
                    L = fmaf(s_pl[i][sp0 + u], f, L);
                    acc = fmaf(v[u], f, acc);
                }
            }
        }
        Storage<T>::store(static_cast<T *>(a.O) + query_row(a, s, r) * D + t, L > 0.f ? acc / L : 0.f);
    }
    if (tid == 0) __hip_atomic_store(ticket, 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);   // ready for the next call
}

template <typename T, int D, int NQ>
static hipError_t launch_decode_q(const AttnArgs &a, hipStream_t st)
{
    constexpr int U = NQ >= 4 ? 2 : 4;       // rows in flight per lane group: fewer when more queries hold registers
    const int R = a.G * a.Tq;
    const size_t blocks = (size_t)a.S * ((R + NQ - 1) / NQ) * a.nsplit;
    if (blocks == 0) return hipSuccess;
    if (blocks <= 256 && a.rows_per_split > 64)
        hipLaunchKernelGGL((attn_decode_kernel<T, D, U, NQ, 16>), dim3((unsigned)blocks), dim3(1024), 0, st, a);
    else
        hipLaunchKernelGGL((attn_decode_kernel<T, D, U, NQ, 4>), dim3((unsigned)blocks), dim3(256), 0, st, a);
    return hipGetLastError();
}

template <typename T, int D>
static hipError_t launch_decode_t(const AttnArgs &a, hipStream_t st)
{
    const int R = a.G * a.Tq;
    if (R >= 4) return launch_decode_q<T, D, 4>(a, st);
    if (R >= 2) return launch_decode_q<T, D, 2>(a, st);
    return launch_decode_q<T, D, 1>(a, st);
}

hipError_t launch_attn_decode(const AttnArgs &a, int dtype, hipStream_t st)
{
    if (dtype == KVEV_F32) return a.d == 64 ? launch_decode_t<float, 64>(a, st) : launch_decode_t<float, 128>(a, st);
    return a.d == 64 ? launch_decode_t<bf16_t, 64>(a, st) : launch_decode_t<bf16_t, 128>(a, st);
}

}  // namespace kvev

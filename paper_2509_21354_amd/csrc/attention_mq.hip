// Multi-query attention (a new frame of Tq query tokens per sequence), bf16
// storage: Eq. 1 of the paper over the kept summaries + raw window (or the whole
// cache for the dense baseline), on the matrix cores.
//
// With Tq queries sharing every key/value row the op does 4*Tq flop per 2 bytes
// of cache read, which puts it near the machine's ridge: the cache must still be
// read only once per sequence, and the contractions must run on MFMA.
//
// A workgroup owns 16*QS queries per wave (4 waves, or 8 for frames above 128 queries) of one sequence and walks the
// rows in tiles of 64.  A tile's K and V rows are copied once, coalesced, into
// LDS (a kept summary is reached through its chunk index); the copy of tile t+1
// is in flight in registers while tile t is computed.  Both products are taken
// transposed, so that the softmax weights never change lanes between the MFMAs:
//   S^T = K Q^T   A = 16 key rows from LDS, B = 16 queries (registers, loaded once);
//                 C puts query l%16 in the lane and 4 keys in its registers;
//   O^T = V^T P^T B = those same registers, rounded to bf16; A = V^T, read from the
//                 row-major LDS tile with the transposing LDS load of gfx950
//                 (ds_read_b64_tr_b16): 16 lanes that each point at 4 consecutive
//                 d of one key receive, per lane, one d of 4 keys.  Two such loads
//                 give a lane its 8 keys in the order the C layout holds them (the
//                 contraction index may be permuted freely as long as A and B agree).
// Online softmax state (m, l) is per query = per lane, shared by 4 lanes through
// two shuffles; the running output is rescaled only when some maximum moved.
// Query tiles of one sequence sit in neighbouring workgroups of the same XCD, so
// the second one finds the cache rows in that XCD's L2.
#include "common.hpp"
#include "kernels.hpp"

namespace kvev {

constexpr float kNegBigMq = -1.0e30f;
typedef short v4i16_t __attribute__((ext_vector_type(4)));
typedef v4i16_t __attribute__((address_space(3))) lds_v4i16_t;

template <int D, int QS, int NWV = 4>
__global__ __launch_bounds__(64 * NWV, NWV == 4 ? 2 : 1) void attn_mq_kernel(AttnArgs a, int qtiles, int nblocks)
{
    constexpr int BN = 64, RP = D + 8, KS = D / 32, DT = D / 16, BM = 16 * NWV * QS, NT = 64 * NWV;
    // V rows are padded by 32 bytes: the transposing load has 16 lanes read 8 bytes each from 4 consecutive
    // rows, and a row pitch of 8 banks (mod 64) puts those 16 pieces in 16 different bank pairs; the 16-byte
    // row reads of K want the 16-byte padding instead
    constexpr int RPV = D + 16;
    constexpr int CPT = BN * (D / 8) / NT;          // 16-byte chunks per thread per tile, for K and for V
    __shared__ __align__(16) bf16_t s_k[BN * RP];    // row-major, padded rows
    __shared__ __align__(16) bf16_t s_v[BN * RPV];

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int n = lane & 15, g = lane >> 4;
    // XCD-aware order: consecutive hardware workgroup ids go round-robin over the 8
    // XCDs; give each XCD a contiguous run of logical ids
    int b = blockIdx.x;
    if (nblocks % 8 == 0) b = (b % 8) * (nblocks / 8) + b / 8;
    const int s = b / qtiles, qt = b % qtiles;

    const bf16_t *K = static_cast<const bf16_t *>(a.K), *V = static_cast<const bf16_t *>(a.V);
    const bf16_t *Kbar = static_cast<const bf16_t *>(a.Kbar), *Vbar = static_cast<const bf16_t *>(a.Vbar);
    int cnt = 0;
    if (a.gated) cnt = min(max(a.count[s], 0), a.k_cap);
    const int nrows = cnt + (a.T - a.win0);
    const int32_t *idx = a.idx ? a.idx + (size_t)s * a.k_cap : nullptr;   // null: compact store, row j is entry j
    const size_t seq_raw = (size_t)s * a.T_cap, seq_sum = (size_t)s * a.N_cap;

    // staging role of this thread: column chunk dc of rows sr, sr + 256/(D/8), ...
    const int dc = tid % (D / 8), sr = tid / (D / 8);
    constexpr int RSTEP = NT / (D / 8);
    u32x4_t kreg[CPT], vreg[CPT];
    // branch-free so that the copies stay in registers while the tile before is computed
#define KVEV_MQ_FETCH(J0)                                                                              \
    _Pragma("unroll") for (int i = 0; i < CPT; ++i)                                                    \
    {                                                                                                  \
        const int j = min((J0) + sr + RSTEP * i, nrows - 1);                                           \
        const bool sm = j < cnt;                                                                       \
        const int c_ = sm ? min(max(idx ? idx[j] : j, 0), a.N_cap - 1) : 0;                            \
        int r_ = a.win0 + (j - cnt) + a.ring_first;                                                    \
        r_ = r_ >= a.T_cap ? r_ - a.T_cap : r_;                                                        \
        const size_t off = (sm ? (seq_sum + c_) : (seq_raw + r_)) * D + dc * 8;                        \
        kreg[i] = *reinterpret_cast<const u32x4_t *>((sm ? Kbar : K) + off);                             \
        vreg[i] = *reinterpret_cast<const u32x4_t *>((sm ? Vbar : V) + off);                             \
    }

    // Tiles that hold raw rows only (all of them for the dense baseline, all but the first one or two
    // otherwise) are fetched through buffer descriptors: one lane offset for all loads, the tile and row
    // step in a scalar register; rows past the end read as zeros (they are masked in the softmax).
    const size_t raw_rows = (size_t)(a.T - a.win0);
    const bool fast = raw_rows * D * sizeof(bf16_t) < ((size_t)1 << 32) && a.ring_first == 0;   // (a ring wraps: no linear tile addresses)
    const __amdgpu_buffer_rsrc_t rk = make_rsrc(K + (seq_raw + a.win0) * D, (uint32_t)(raw_rows * D * sizeof(bf16_t)));
    const __amdgpu_buffer_rsrc_t rv = make_rsrc(V + (seq_raw + a.win0) * D, (uint32_t)(raw_rows * D * sizeof(bf16_t)));
    const uint32_t voff = (uint32_t)((sr * D + dc * 8) * sizeof(bf16_t));
#define KVEV_MQ_FETCH_RAW(J0)                                                                          \
    _Pragma("unroll") for (int i = 0; i < CPT; ++i)                                                    \
    {                                                                                                  \
        const uint32_t soff = (uint32_t)(((J0) - cnt + RSTEP * i) * D * (int)sizeof(bf16_t));          \
        kreg[i] = buffer_load16<u32x4_t>(rk, voff, soff);                                              \
        vreg[i] = buffer_load16<u32x4_t>(rv, voff, soff);                                              \
    }
#define KVEV_MQ_FETCH_ANY(J0)                                                                          \
    if (fast && (J0) >= cnt) { KVEV_MQ_FETCH_RAW(J0) } else { KVEV_MQ_FETCH(J0) }

    // queries of this wave: sub-tile u holds query qt*BM + wave*16*QS + u*16 + n
    // (queries that share the sequence: the Tq queries of each of the G heads of its group, r = g*Tq + tq)
    bf16x8_t qf[QS][KS];
    int qrow[QS], lim[QS];
    size_t orow[QS];
    const int R = a.G * a.Tq;
#pragma unroll
    for (int u = 0; u < QS; ++u) {
        qrow[u] = qt * BM + (wave * QS + u) * 16 + n;
        const int rc = min(qrow[u], R - 1);
        const int gq = rc / a.Tq, tq = rc - gq * a.Tq;
        orow[u] = ((size_t)(s / a.Hkv) * ((size_t)a.Hkv * a.G) + (size_t)(s % a.Hkv) * a.G + gq) * a.Tq + tq;
        // causal frame: the queries are the last Tq cached tokens; rows after a query's own token are hidden
        lim[u] = a.causal ? nrows - (a.Tq - 1 - tq) : nrows;
        const bf16_t *Qp = static_cast<const bf16_t *>(a.Q) + orow[u] * D + g * 8;
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) qf[u][ks] = *reinterpret_cast<const bf16x8_t *>(Qp + ks * 32);
    }

    float m[QS], lsum[QS];
    f32x4_t o[QS][DT];
#pragma unroll
    for (int u = 0; u < QS; ++u) {
        m[u] = kNegBigMq;
        lsum[u] = 0.f;
#pragma unroll
        for (int dt = 0; dt < DT; ++dt) o[u][dt] = f32x4_t{0.f, 0.f, 0.f, 0.f};
    }
    const float c = a.scale_log2e;

    if (nrows > 0) { KVEV_MQ_FETCH_ANY(0) }
    for (int j0 = 0; j0 < nrows; j0 += BN) {
#pragma unroll
        for (int i = 0; i < CPT; ++i) {
            *reinterpret_cast<u32x4_t *>(s_k + (size_t)(sr + RSTEP * i) * RP + dc * 8) = kreg[i];
            *reinterpret_cast<u32x4_t *>(s_v + (size_t)(sr + RSTEP * i) * RPV + dc * 8) = vreg[i];
        }
        __syncthreads();
        if (j0 + BN < nrows) { KVEV_MQ_FETCH_ANY(j0 + BN) }   // next tile's copy rides under this tile's math
        const bool full = j0 + BN <= nrows - (a.causal ? a.Tq - 1 : 0);    // no row of the tile is hidden from any query

        // ---- S^T = K Q^T: every K fragment read from LDS serves all QS query sub-tiles of the wave ----
        f32x4_t st[QS][4];
#pragma unroll
        for (int u = 0; u < QS; ++u)
#pragma unroll
            for (int kt = 0; kt < 4; ++kt) st[u][kt] = f32x4_t{0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int ks = 0; ks < KS; ++ks)
#pragma unroll
            for (int kt = 0; kt < 4; ++kt) {
                const bf16x8_t kf = *reinterpret_cast<const bf16x8_t *>(s_k + (size_t)(kt * 16 + n) * RP + ks * 32 + g * 8);
#pragma unroll
                for (int u = 0; u < QS; ++u)
                    st[u][kt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(kf, qf[u][ks], st[u][kt], 0, 0, 0);
            }
        // ---- online softmax for this lane's queries (raw scores; scale folded into exp2) ----
        bf16x8_t pb[QS][2];
#pragma unroll
        for (int u = 0; u < QS; ++u) {
            if (!full) {
#pragma unroll
                for (int kt = 0; kt < 4; ++kt)
#pragma unroll
                    for (int r = 0; r < 4; ++r)
                        if (j0 + kt * 16 + 4 * g + r >= lim[u]) st[u][kt][r] = kNegBigMq;
            }
            float mx = kNegBigMq;
#pragma unroll
            for (int kt = 0; kt < 4; ++kt)
#pragma unroll
                for (int r = 0; r < 4; ++r) mx = fmaxf(mx, st[u][kt][r]);
            mx = fmaxf(mx, __shfl_xor(mx, 16));
            mx = fmaxf(mx, __shfl_xor(mx, 32));
            const float m_new = fmaxf(m[u], mx);
            if (__any(m_new > m[u])) {
                const float alpha = __builtin_amdgcn_exp2f((m[u] - m_new) * c);
                lsum[u] *= alpha;
#pragma unroll
                for (int dt = 0; dt < DT; ++dt)
#pragma unroll
                    for (int r = 0; r < 4; ++r) o[u][dt][r] *= alpha;
                m[u] = m_new;
            }
            const float mc = -m_new * c;
#pragma unroll
            for (int h2 = 0; h2 < 2; ++h2) {
                float p[8];
#pragma unroll
                for (int e = 0; e < 8; ++e) {
                    p[e] = __builtin_amdgcn_exp2f(fmaf(st[u][2 * h2 + (e >> 2)][e & 3], c, mc));   // masked: exp2(-huge) = 0
                    lsum[u] += p[e];
                }
                pb[u][h2] = __builtin_bit_cast(bf16x8_t, make_uint4(pack_bf16x2(p[0], p[1]), pack_bf16x2(p[2], p[3]),
                                                                     pack_bf16x2(p[4], p[5]), pack_bf16x2(p[6], p[7])));
            }
        }
        // ---- O^T += V^T P^T: every V^T fragment serves all QS sub-tiles ----------------
        // transposing load: source lane i of a 16-lane block points at key 4g + i/4,
        // d = 16 dt + 4 (i%4) .. +3; destination lane i receives d = 16 dt + i of keys
        // 4g .. 4g+3.  The second load does the same 16 keys further (registers e >= 4).
#pragma unroll
        for (int h2 = 0; h2 < 2; ++h2)
#pragma unroll
            for (int dt = 0; dt < DT; ++dt) {
                const bf16_t *src = s_v + (size_t)(h2 * 32 + 4 * g + (n >> 2)) * RPV + dt * 16 + 4 * (n & 3);
                const v4i16_t lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_v4i16_t *)src);
                const v4i16_t hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_v4i16_t *)(src + 16 * RPV));
                const bf16x8_t vf = __builtin_bit_cast(bf16x8_t, __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7));
#pragma unroll
                for (int u = 0; u < QS; ++u)
                    o[u][dt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(vf, pb[u][h2], o[u][dt], 0, 0, 0);
            }
        __syncthreads();
    }

#pragma unroll
    for (int u = 0; u < QS; ++u) {
        float l = lsum[u];
        l += __shfl_xor(l, 16);
        l += __shfl_xor(l, 32);
        if (qrow[u] < R) {
            const float inv = l > 0.f ? 1.0f / l : 0.f;
            bf16_t *Op = static_cast<bf16_t *>(a.O) + orow[u] * D + 4 * g;
#pragma unroll
            for (int dt = 0; dt < DT; ++dt) {
                uint2 w;
                w.x = pack_bf16x2(o[u][dt][0] * inv, o[u][dt][1] * inv);
                w.y = pack_bf16x2(o[u][dt][2] * inv, o[u][dt][3] * inv);
                *reinterpret_cast<uint2 *>(Op + dt * 16) = w;
            }
        }
    }
}

#undef KVEV_MQ_FETCH
#undef KVEV_MQ_FETCH_RAW
#undef KVEV_MQ_FETCH_ANY

template <int D, int QS, int NWV = 4>
static hipError_t launch_mq_t(const AttnArgs &a, hipStream_t st)
{
    const int qtiles = (a.G * a.Tq + 16 * NWV * QS - 1) / (16 * NWV * QS);
    const size_t blocks = (size_t)a.S * qtiles;
    if (blocks == 0) return hipSuccess;
    hipLaunchKernelGGL((attn_mq_kernel<D, QS, NWV>), dim3((unsigned)blocks), dim3(64 * NWV), 0, st, a, qtiles, (int)blocks);
    return hipGetLastError();
}

hipError_t launch_attn_mq(const AttnArgs &a, hipStream_t st)
{
    // 128 queries per workgroup halve the LDS traffic per flop; frames shorter than
    // that would leave half the waves idle.  Frames of more than 128 queries take workgroups of 8 waves (256 queries):
    // a tile of K and V is then fetched and staged once for all of them, instead of by two workgroups that meet in L2
    // (dense launch at 256 queries and 32768 rows: 11.0 -> 10.0 ms; 10 tiles per workgroup: 290 -> 287 us).
    const bool wide = a.G * a.Tq > 64;
    if (a.G * a.Tq > 128) return a.d == 64 ? launch_mq_t<64, 2, 8>(a, st) : launch_mq_t<128, 2, 8>(a, st);
    if (a.d == 64) return wide ? launch_mq_t<64, 2>(a, st) : launch_mq_t<64, 1>(a, st);
    return wide ? launch_mq_t<128, 2>(a, st) : launch_mq_t<128, 1>(a, st);
}

}  // namespace kvev

// Multi-query attention (a new frame of Tq query tokens per sequence), bf16
// storage: Eq. 1 of the paper over the kept summaries + raw window (or the whole
// cache for the dense baseline), on the matrix cores.
//
// With Tq queries sharing every key/value row the op does 4*Tq flop per 2 bytes
// of cache read, which puts it near the machine's ridge: the cache must still be
// read only once per sequence, and the contractions must run on MFMA.
//
// A workgroup owns 64 queries of one sequence (16 per wave) and walks the rows in
// tiles of 64.  Both products are taken transposed, so that the softmax weights
// never change lanes between the two MFMAs:
//   S^T = K Q^T   A = 16 key rows (16-byte pieces straight from global memory; a
//                 kept summary is reached through its chunk index), B = the wave's
//                 16 queries (held in registers for the whole kernel);
//                 C puts query l%16 in the lane and 4 keys in its registers;
//   O^T = V^T P^T B = those same registers, rounded to bf16; A = V^T, which the
//                 workgroup stages row-major in LDS (coalesced 16-byte copies) and
//                 reads back with the transposing LDS load of gfx950
//                 (ds_read_b64_tr_b16): 16 lanes that each point at 4 consecutive
//                 d of one key receive, per lane, one d of 4 keys.  Two such loads
//                 give a lane its 8 keys in the order the C layout holds them (the
//                 contraction index may be permuted freely as long as A and B agree).
// Online softmax state (m, l) is per query = per lane, shared by 4 lanes through
// two shuffles.  Queries of the same sequence sit in neighbouring workgroups of
// the same XCD, so the other three read the cache rows from that XCD's L2.
#include "common.hpp"
#include "kernels.hpp"

namespace kvev {

constexpr float kNegBigMq = -1.0e30f;
typedef short v4i16_t __attribute__((ext_vector_type(4)));
typedef v4i16_t __attribute__((address_space(3))) lds_v4i16_t;

template <int D>
__global__ __launch_bounds__(256) void attn_mq_kernel(AttnArgs a, int qtiles, int nblocks)
{
    constexpr int BN = 64, VP = D + 8, KS = D / 32, DT = D / 16;
    __shared__ __align__(16) bf16_t s_v[BN * VP];      // V tile, row-major, padded rows

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int n = lane & 15, g = lane >> 4;
    // XCD-aware order: consecutive hardware workgroup ids go round-robin over the 8
    // XCDs; give each XCD a contiguous run of logical ids so the query tiles of one
    // sequence share an L2
    int b = blockIdx.x;
    if (nblocks % 8 == 0) b = (b % 8) * (nblocks / 8) + b / 8;
    const int s = b / qtiles, qt = b % qtiles;

    const bf16_t *K = static_cast<const bf16_t *>(a.K), *V = static_cast<const bf16_t *>(a.V);
    const bf16_t *Kbar = static_cast<const bf16_t *>(a.Kbar), *Vbar = static_cast<const bf16_t *>(a.Vbar);
    int cnt = 0;
    if (a.gated) cnt = min(max(a.count[s], 0), a.k_cap);
    const int nrows = cnt + (a.T - a.win0);
    const int32_t *idx = a.idx + (size_t)s * a.k_cap;
    const size_t seq_raw = (size_t)s * a.T_cap, seq_sum = (size_t)s * a.N_cap;

    auto row_off = [&](int j, bool &summary) -> size_t {
        summary = j < cnt;
        if (summary) return (seq_sum + min(max(idx[j], 0), a.N_cap - 1)) * D;
        return (seq_raw + a.win0 + (j - cnt)) * D;
    };

    const int q = qt * 64 + wave * 16 + n;
    const bool q_live = q < a.Tq;
    const bf16_t *Qp = static_cast<const bf16_t *>(a.Q) + ((size_t)s * a.Tq + min(q, a.Tq - 1)) * D + g * 8;
    bf16x8_t qf[KS];
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) qf[ks] = *reinterpret_cast<const bf16x8_t *>(Qp + ks * 32);

    float m = kNegBigMq, lsum = 0.f;
    f32x4_t o[DT];
#pragma unroll
    for (int dt = 0; dt < DT; ++dt) o[dt] = f32x4_t{0.f, 0.f, 0.f, 0.f};

    for (int j0 = 0; j0 < nrows; j0 += BN) {
        // ---- V tile into LDS (row-major) --------------------------------------
#pragma unroll
        for (int i = 0; i < BN * (D / 8) / 256; ++i) {
            const int chunk = tid + 256 * i;
            const int row = chunk / (D / 8), dc = chunk % (D / 8);
            bool sm;
            const size_t off = row_off(min(j0 + row, nrows - 1), sm);
            *reinterpret_cast<uint4 *>(s_v + (size_t)row * VP + dc * 8) =
                *reinterpret_cast<const uint4 *>((sm ? Vbar : V) + off + dc * 8);
        }

        // ---- S^T = K Q^T ------------------------------------------------------
        f32x4_t st[4];
#pragma unroll
        for (int kt = 0; kt < 4; ++kt) {
            bool sm;
            const size_t off = row_off(min(j0 + kt * 16 + n, nrows - 1), sm);
            const bf16_t *kp = (sm ? Kbar : K) + off + g * 8;
            f32x4_t acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int ks = 0; ks < KS; ++ks)
                acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(*reinterpret_cast<const bf16x8_t *>(kp + ks * 32), qf[ks],
                                                              acc, 0, 0, 0);
            st[kt] = acc;
        }

        // ---- online softmax for this lane's query ----------------------------
        float mx = kNegBigMq;
#pragma unroll
        for (int kt = 0; kt < 4; ++kt)
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                const bool ok = j0 + kt * 16 + 4 * g + r < nrows;
                st[kt][r] = ok ? st[kt][r] * a.scale_log2e : kNegBigMq;
                mx = fmaxf(mx, st[kt][r]);
            }
        mx = fmaxf(mx, __shfl_xor(mx, 16));
        mx = fmaxf(mx, __shfl_xor(mx, 32));
        const float m_new = fmaxf(m, mx);
        const float alpha = __builtin_amdgcn_exp2f(m - m_new);
        m = m_new;
        lsum *= alpha;
#pragma unroll
        for (int dt = 0; dt < DT; ++dt)
#pragma unroll
            for (int r = 0; r < 4; ++r) o[dt][r] *= alpha;
        bf16x8_t pb[2];
#pragma unroll
        for (int h2 = 0; h2 < 2; ++h2) {
            float p[8];
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                const int kt = 2 * h2 + (e >> 2), r = e & 3;
                const bool ok = j0 + kt * 16 + 4 * g + r < nrows;
                p[e] = ok ? __builtin_amdgcn_exp2f(st[kt][r] - m_new) : 0.f;
                lsum += p[e];
            }
            pb[h2] = __builtin_bit_cast(bf16x8_t, make_uint4(pack_bf16x2(p[0], p[1]), pack_bf16x2(p[2], p[3]),
                                                              pack_bf16x2(p[4], p[5]), pack_bf16x2(p[6], p[7])));
        }
        __syncthreads();

        // ---- O^T += V^T P^T ---------------------------------------------------
        // transposing load: source lane i of a 16-lane block points at key 4g + i/4,
        // d = 16 dt + 4 (i%4) .. +3; destination lane i receives d = 16 dt + i of keys
        // 4g .. 4g+3.  The second load does the same 16 keys further (registers e >= 4).
#pragma unroll
        for (int h2 = 0; h2 < 2; ++h2)
#pragma unroll
            for (int dt = 0; dt < DT; ++dt) {
                const bf16_t *src = s_v + (size_t)(h2 * 32 + 4 * g + (n >> 2)) * VP + dt * 16 + 4 * (n & 3);
                const v4i16_t lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_v4i16_t *)src);
                const v4i16_t hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_v4i16_t *)(src + 16 * VP));
                const bf16x8_t vf = __builtin_bit_cast(bf16x8_t, __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7));
                o[dt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(vf, pb[h2], o[dt], 0, 0, 0);
            }
        __syncthreads();
    }

    lsum += __shfl_xor(lsum, 16);
    lsum += __shfl_xor(lsum, 32);
    if (q_live) {
        const float inv = lsum > 0.f ? 1.0f / lsum : 0.f;
        bf16_t *Op = static_cast<bf16_t *>(a.O) + ((size_t)s * a.Tq + q) * D + 4 * g;
#pragma unroll
        for (int dt = 0; dt < DT; ++dt) {
            uint2 w;
            w.x = pack_bf16x2(o[dt][0] * inv, o[dt][1] * inv);
            w.y = pack_bf16x2(o[dt][2] * inv, o[dt][3] * inv);
            *reinterpret_cast<uint2 *>(Op + dt * 16) = w;
        }
    }
}

hipError_t launch_attn_mq(const AttnArgs &a, hipStream_t st)
{
    const int qtiles = (a.Tq + 63) / 64;
    const size_t blocks = (size_t)a.S * qtiles;
    if (blocks == 0) return hipSuccess;
    if (a.d == 64)
        hipLaunchKernelGGL((attn_mq_kernel<64>), dim3((unsigned)blocks), dim3(256), 0, st, a, qtiles, (int)blocks);
    else
        hipLaunchKernelGGL((attn_mq_kernel<128>), dim3((unsigned)blocks), dim3(256), 0, st, a, qtiles, (int)blocks);
    return hipGetLastError();
}

}  // namespace kvev

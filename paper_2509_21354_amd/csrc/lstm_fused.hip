// Recurrent gate, Eq. 3 of the paper, bf16 storage, d_g = 256, for launches that fill the chip: one kernel that
// takes the chunk summaries and leaves the scores, with no intermediate in memory.
//
// The two-kernel form (lstm_mfma.hip) writes the input projections W_ih [Kbar_t ; Vbar_t] of a block of steps to
// scratch as fp32 and reads them back in the recurrence: 16 KiB out and 16 KiB back per sequence and step against
// 512 bytes of summaries, which at 8192 sequences x 256 steps is most of the gate's time.  Here a workgroup owns 32
// sequences of one layer and, every step, contracts [x_t ; h_{t-1}] against [W_ih | W_hh] on the matrix cores:
//   * W_ih x_t with bf16 operands (exact products), W_hh h_{t-1} with fp16 operands as in the two-kernel form
//     (W_hh scaled by a power of two s, h as hi + lo terms); the x part is accumulated first, multiplied by s
//     (exact), then the h part joins the same accumulators and the sum is scaled back once: fp32-grade throughout;
//   * the weights of a step are 1 MiB per workgroup (W_ih bf16 + W_hh fp16), far more than a compute unit can
//     hold, and a unit pulls 64 bytes per clock out of L2; two blocks of 16 sequences share every weight fragment,
//     which makes the step's matrix time (2 x 768 MFMAs per wave) as long as its weight stream, and makes 8192
//     sequences exactly one workgroup per compute unit.  A few weight items stay in registers and LDS, the rest
//     runs through a ring of register buffers a few items ahead, across step boundaries;
//   * the part of a step that does not depend on h_{t-1} (W_ih x_t for the first unit tile) is placed before the
//     step's only barrier, so a wave that is ahead has work while the others finish the step before;
//   * the summaries of step t + 3 are in flight from HBM while step t is computed (registers -> a three-deep ring
//     in LDS): the kernel's memory traffic is the summaries in and the scores out.
// Geometry as in the two-kernel form: 8 waves, wave w owns hidden units 32 w .. 32 w + 31 as two tiles of 16, all
// four gates of a unit meet in one lane, so the packed weight layouts of lstm_prep_kernel / pack_whh are shared.
#include "common.hpp"
#include "kernels.hpp"
#include "lstm_common.hpp"
#include <utility>

namespace kvev {

template <int D> struct Fus {
    static constexpr int DG = 256, NW = 8, UT = 2, SB = 2, SEQ = 16 * SB;
    static constexpr int KS = DG / 32, KX = 2 * D / 32, PER = KX + KS, ITEMS = UT * PER;
    static constexpr int HP = DG + 8, XP = 2 * D + 8;
    // the cyclic walk of a step: [x items of tile 0 | h items of tile 0 | x items of tile 1 | h items of tile 1];
    // the step's barrier sits in front of the first h item
    static constexpr int ut_of(int i) { return i / PER; }
    static constexpr bool is_x(int i) { return i % PER < KX; }
    static constexpr int ks_of(int i) { return is_x(i) ? i % PER : i % PER - KX; }
    // where an item's weights live: 0 LDS, 1 registers, 2 streamed from L2 every step
    static constexpr int cls(int i)
    {
        if (i == PER + KX / 2) return 0;
        if (i == KX + 2 || i == PER + KX + 4 || i == KX / 2) return 1;
        return 2;
    }
    static constexpr int count(int c) { int k = 0; for (int i = 0; i < ITEMS; ++i) k += cls(i) == c; return k; }
    static constexpr int idx(int i) { int k = 0; for (int j = 0; j < i; ++j) k += cls(j) == cls(i); return k; }
    static constexpr int pos(int c, int k) { for (int i = 0; i < ITEMS; ++i) if (cls(i) == c && idx(i) == k) return i; return 0; }
    static constexpr int LRES = count(0), RRES = count(1), NS = count(2);
    static constexpr int NSLOT = 4, PF = NSLOT - 1;
    static_assert(NS % NSLOT == 0, "slot rotation must line up with the item loop");
    static_assert(LRES == 1, "one LDS item per wave, read one item ahead into a single buffer");
    static_assert(ITEMS % 2 == 0, "operand buffer parity must survive the wrap into the next step");
    static constexpr size_t lds_h = (size_t)2 * 2 * SEQ * HP * sizeof(f16_t);      // [buffer][hi, lo][sequence][unit]
    static constexpr size_t lds_x = (size_t)3 * SEQ * XP * sizeof(bf16_t);         // [ring of 3 steps][sequence][2d]
    static constexpr size_t lds_up = (size_t)2 * NW * SEQ * sizeof(float);         // shares of the utility logit
    static constexpr size_t lds_b = (size_t)4 * DG * sizeof(float);                // b_ih + b_hh
    static constexpr size_t lds_w = (size_t)NW * LRES * 4096;
    static constexpr size_t lds_ub = (size_t)16 * SEQ * sizeof(float);             // utility logits of 16 steps, written out together
    static constexpr size_t lds = lds_h + lds_x + lds_up + lds_b + lds_w + lds_ub;
    static_assert(lds <= 160 * 1024, "LDS budget of a CU");
};

template <int D>
__global__ __launch_bounds__(512) void lstm_fused_kernel(LstmArgs a, int t0, int nb)
{
    using F = Fus<D>;
    constexpr int DG = F::DG, NW = F::NW, UT = F::UT, SB = F::SB, SEQ = F::SEQ, KS = F::KS, KX = F::KX, ITEMS = F::ITEMS;
    constexpr int HP = F::HP, XP = F::XP, RRES = F::RRES, NS = F::NS, NSLOT = F::NSLOT, PF = F::PF;
    typedef _Float16 f16x4_t __attribute__((ext_vector_type(4)));
    extern __shared__ __align__(16) unsigned char smem_f[];
    f16_t *s_h = reinterpret_cast<f16_t *>(smem_f);
    bf16_t *s_x = reinterpret_cast<bf16_t *>(smem_f + F::lds_h);
    float *s_up = reinterpret_cast<float *>(smem_f + F::lds_h + F::lds_x);           // [2][NW][SEQ]
    float *s_bias = reinterpret_cast<float *>(smem_f + F::lds_h + F::lds_x + F::lds_up);
    unsigned char *s_w = smem_f + F::lds_h + F::lds_x + F::lds_up + F::lds_b;
    float *s_ubuf = reinterpret_cast<float *>(smem_f + F::lds_h + F::lds_x + F::lds_up + F::lds_b + F::lds_w);   // [16][SEQ]

    const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int n = lane & 15, g4 = lane >> 4;
    const int gpl = (a.BH + SEQ - 1) / SEQ;
    const int gid = xcd_order(blockIdx.x, gridDim.x);
    const int l = gid / gpl, grp = gid % gpl;
    bool live[SB];
    size_t sq[SB];
#pragma unroll
    for (int sb = 0; sb < SB; ++sb) {
        live[sb] = grp * SEQ + sb * 16 + n < a.BH;
        sq[sb] = (size_t)l * a.BH + min(grp * SEQ + sb * 16 + n, a.BH - 1);
    }

    const bf16_t *w_s = static_cast<const bf16_t *>(a.w_s) + (size_t)l * DG;
    const float b_s = bf16_to_f32(static_cast<const bf16_t *>(a.b_s)[l]);
    const int sexp = whh_scale_exp(whh_layer_max(a.whh_max_bits, l));
    const float scale = ldexpf(1.f, sexp), inv_scale = ldexpf(1.f, -sexp);
    for (int i = tid; i < 4 * DG; i += 512)
        s_bias[i] = bf16_to_f32(static_cast<const bf16_t *>(a.b_ih)[(size_t)l * 4 * DG + i]) +
                    bf16_to_f32(static_cast<const bf16_t *>(a.b_hh)[(size_t)l * 4 * DG + i]);

    // state of (sequence sb*16 + n, units 32 wave + 16 ut + 4 g4 + r) lives in this lane
    float c_reg[UT][SB][4], ws_reg[UT][4];
    f16_t *h_wr = s_h + (size_t)n * HP + wave * 32 + 4 * g4;       // + ((buf*2 + plane)*SEQ + sb*16)*HP + ut*16
    const f16_t *h_rd = s_h + (size_t)n * HP + g4 * 8;             // + ((buf*2 + plane)*SEQ + sb*16)*HP + ks*32
    const bf16_t *x_rd = s_x + (size_t)n * XP + g4 * 8;            // + (ring*SEQ + sb*16)*XP + ks*32
    auto publish_h = [&](int buf, int ut, int sb, const float (&hv)[4]) {
        f16x4_t hi, lo;
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            hi[r] = (f16_t)hv[r];
            lo[r] = (f16_t)(hv[r] - (float)hi[r]);
        }
        *reinterpret_cast<f16x4_t *>(h_wr + ((size_t)(buf * 2 + 0) * SEQ + sb * 16) * HP + ut * 16) = hi;
        *reinterpret_cast<f16x4_t *>(h_wr + ((size_t)(buf * 2 + 1) * SEQ + sb * 16) * HP + ut * 16) = lo;
    };
#pragma unroll
    for (int ut = 0; ut < UT; ++ut) {
#pragma unroll
        for (int r = 0; r < 4; ++r) ws_reg[ut][r] = bf16_to_f32(w_s[wave * 32 + ut * 16 + 4 * g4 + r]);
#pragma unroll
        for (int sb = 0; sb < SB; ++sb) {
            float hv[4];
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                const int unit = wave * 32 + ut * 16 + 4 * g4 + r;
                // (chunk 0 starts the recurrence from a zero state, whatever the buffers hold)
                c_reg[ut][sb][r] = live[sb] && t0 > 0 ? a.c[sq[sb] * DG + unit] : 0.f;
                hv[r] = live[sb] && t0 > 0 ? a.h[sq[sb] * DG + unit] : 0.f;
            }
            publish_h(0, ut, sb, hv);
        }
    }

    // ---- the summaries: 16-byte pieces, SEQ rows of 2d/8 pieces per step, NP pieces per thread ----
    constexpr int PPR = 2 * D / 8, NP = SEQ * PPR / 512;
    static_assert(SEQ * PPR % 512 == 0, "pieces divide over the threads");
    const bf16_t *xsrc[NP];
    bf16_t *xdst[NP];
#pragma unroll
    for (int k = 0; k < NP; ++k) {
        const int p = tid + 512 * k, row = p / PPR, e = (p % PPR) * 8;
        const size_t s = (size_t)l * a.BH + min(grp * SEQ + row, a.BH - 1);
        xsrc[k] = (e < D ? static_cast<const bf16_t *>(a.Kbar) + e : static_cast<const bf16_t *>(a.Vbar) + (e - D)) +
                  (s * a.N_cap + t0) * D;
        xdst[k] = s_x + (size_t)row * XP + e;                       // + ring * SEQ * XP
    }
    u32x4_t xreg[NP];
    auto fetch_x = [&](int tt) {                // step tt of this launch (clamped: the last steps fetch a valid row again)
        const size_t off = (size_t)min(tt, nb - 1) * D;
#pragma unroll
        for (int k = 0; k < NP; ++k)      // read once: the hint keeps the stream from pushing the weights out of L2
            xreg[k] = __builtin_nontemporal_load(reinterpret_cast<const u32x4_t *>(xsrc[k] + off));
    };
    auto stash_x = [&](int ring) {
#pragma unroll
        for (int k = 0; k < NP; ++k) *reinterpret_cast<u32x4_t *>(xdst[k] + (size_t)ring * SEQ * XP) = xreg[k];
    };
    fetch_x(0); stash_x(0);
    fetch_x(1); stash_x(1);
    fetch_x(2);

    // ---- weights: buffer descriptors over this wave's packed fragments ----
    // W_hh: fragment q of item (ut, ks) at (ut*KS + ks)*4096 + q*1024 + lane*16; W_ih: fragment (ut, q, ks) at
    // ((ut*4 + q)*KX + ks)*1024 + lane*16
    const uint32_t lane16 = lane * 16;
    const __amdgpu_buffer_rsrc_t wh_rsrc =
        make_rsrc(reinterpret_cast<const unsigned char *>(a.whh_packed + ((size_t)l * NW + wave) * UT * KS * 4 * 64), UT * KS * 4096);
    const __amdgpu_buffer_rsrc_t wx_rsrc =
        make_rsrc(reinterpret_cast<const unsigned char *>(a.wih_packed + ((size_t)l * NW + wave) * UT * 4 * KX * 64), UT * KX * 4096);
    auto load_item = [&](auto ic, u32x4_t (&dst)[4]) __attribute__((always_inline)) {
        constexpr int i = decltype(ic)::value, ut = F::ut_of(i), ks = F::ks_of(i);
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            if constexpr (F::is_x(i)) dst[q] = buffer_load16<u32x4_t>(wx_rsrc, lane16, ((ut * 4 + q) * KX + ks) * 1024);
            else dst[q] = buffer_load16<u32x4_t>(wh_rsrc, lane16 + q * 1024, (ut * KS + ks) * 4096);
        }
    };
    unsigned char *w_lds = s_w + (size_t)wave * 4096 + lane16;     // + q*1024: the wave's LDS item
    {
        u32x4_t tmp[4];
        load_item(std::integral_constant<int, F::pos(0, 0)>{}, tmp);
#pragma unroll
        for (int q = 0; q < 4; ++q) *reinterpret_cast<u32x4_t *>(w_lds + q * 1024) = tmp[q];
    }
    u32x4_t wres[RRES][4];
    static_for<RRES>([&](auto kc) { load_item(std::integral_constant<int, F::pos(1, decltype(kc)::value)>{}, wres[decltype(kc)::value]); });
    u32x4_t wbuf[NSLOT][4];
    auto load_w = [&](auto jc) __attribute__((always_inline)) {     // jc: index within the streamed items
        constexpr int j = decltype(jc)::value;
        load_item(std::integral_constant<int, F::pos(2, j)>{}, wbuf[j % NSLOT]);
    };
    static_for<PF>(load_w);
    u32x4_t wl[4];
    auto read_wl = [&]() __attribute__((always_inline)) {
#pragma unroll
        for (int q = 0; q < 4; ++q) wl[q] = *reinterpret_cast<const u32x4_t *>(w_lds + q * 1024);
    };

    // B operands of an item: an h item takes (lo, hi) x 2 sequence blocks, an x item 2 sequence blocks
    u32x4_t bop[2][4];
    auto read_ops = [&](auto ic, int hbuf, int ring) __attribute__((always_inline)) {
        constexpr int i = decltype(ic)::value, ks = F::ks_of(i);
        if constexpr (F::is_x(i)) {
#pragma unroll
            for (int sb = 0; sb < SB; ++sb)
                bop[i & 1][sb] = *reinterpret_cast<const u32x4_t *>(x_rd + ((size_t)ring * SEQ + sb * 16) * XP + ks * 32);
        } else {
#pragma unroll
            for (int p = 0; p < 2; ++p)
#pragma unroll
                for (int sb = 0; sb < SB; ++sb)
                    bop[i & 1][p * 2 + sb] = *reinterpret_cast<const u32x4_t *>(h_rd + ((size_t)(hbuf * 2 + p) * SEQ + sb * 16) * HP + ks * 32);
        }
    };

    __syncthreads();             // h of step t0 - 1, the first two steps' summaries, the bias and the LDS items are in place
    read_ops(std::integral_constant<int, 0>{}, 0, 0);
    if constexpr (F::cls(0) == 0) read_wl();

    // The utility logit of chunk c, from the waves' shares in s_up[ub], by wave 0.  Scores are held back in LDS and
    // leave in runs of 16 chunks (64 bytes per sequence at a time), so that a cache line of the score arrays is written
    // while it is still in L2 instead of 4 bytes at a time across hundreds of microseconds.
    auto emit_score = [&](int c, int ub, bool last) {
        if (lane < SEQ) {
            float u = 0.f;
#pragma unroll
            for (int w = 0; w < NW; ++w) u += s_up[(ub * NW + w) * SEQ + lane];
            s_ubuf[(c & 15) * SEQ + lane] = u + b_s;
        }
        if ((c & 15) == 15 || last) {
            const int c_lo = max(t0, c & ~15), sq2 = lane >> 1, half = lane & 1;
            if (grp * SEQ + sq2 < a.BH) {
                const size_t s = (size_t)l * a.BH + grp * SEQ + sq2;
#pragma unroll
                for (int j = 0; j < 8; ++j) {
                    const int cj = (c & ~15) + half * 8 + j;
                    if (cj >= c_lo && cj <= c) {
                        const float u = s_ubuf[(cj & 15) * SEQ + sq2];
                        a.util[s * a.N_cap + cj] = u;
                        a.gate[s * a.N_cap + cj] = sigmoid_hw(u);
                    }
                }
            }
        }
    };

    f32x4_t acc[SB][4];
    float upart[SB] = {0.f, 0.f};
    int ring = 0;                // tt % 3
    for (int tt = 0; tt < nb; ++tt) {
        const int cur = tt & 1, nxt = cur ^ 1;
        const int ring_next = ring == 2 ? 0 : ring + 1;
        auto cell_update = [&](auto utc) __attribute__((always_inline)) {
            constexpr int ut = decltype(utc)::value;
            f32x4_t bias[4];
#pragma unroll
            for (int q = 0; q < 4; ++q)
                bias[q] = *reinterpret_cast<const f32x4_t *>(s_bias + q * DG + wave * 32 + ut * 16 + 4 * g4);
#pragma unroll
            for (int sb = 0; sb < SB; ++sb) {
                float hv[4];
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                    const float ig = sigmoid_hw(fmaf(acc[sb][0][r], inv_scale, bias[0][r]));
                    const float fg = sigmoid_hw(fmaf(acc[sb][1][r], inv_scale, bias[1][r]));
                    const float gg = tanh_hw(fmaf(acc[sb][2][r], inv_scale, bias[2][r]));
                    const float og = sigmoid_hw(fmaf(acc[sb][3][r], inv_scale, bias[3][r]));
                    const float cn = fmaf(fg, c_reg[ut][sb][r], ig * gg);
                    c_reg[ut][sb][r] = cn;
                    float hn = og * tanh_hw(cn);
                    asm volatile("" : "+v"(hn));     // opaque to the optimiser: hn is the rounded product from here on
                    hv[r] = hn;
                    upart[sb] = fmaf(ws_reg[ut][r], hn, upart[sb]);
                }
                publish_h(nxt, ut, sb, hv);
                if (tt == nb - 1 && live[sb])        // the state leaves the kernel as fp32
                    *reinterpret_cast<float4 *>(a.h + sq[sb] * DG + wave * 32 + ut * 16 + 4 * g4) = make_float4(hv[0], hv[1], hv[2], hv[3]);
            }
        };
        static_for<ITEMS>([&](auto ic) {
            constexpr int i = decltype(ic)::value, ut = F::ut_of(i), ks = F::ks_of(i);
            constexpr bool isx = F::is_x(i);
            constexpr int c = F::cls(i), k = F::idx(i), inext = (i + 1) % ITEMS;
            if constexpr (i == KX) {
                // ---- the step's barrier: every wave has published its part of h_{t-1} ----
                __syncthreads();
                if (tt > 0 && wave == 0) emit_score(t0 + tt - 1, nxt, false);       // the logit of the step before
                read_ops(ic, cur, ring);
            }
            // operands of what comes next are asked for before this item's MFMAs (h of this step only after the barrier)
            if constexpr (inext != KX) read_ops(std::integral_constant<int, inext>{}, cur, inext == 0 ? ring_next : ring);
            if constexpr (F::cls(inext) == 0) read_wl();
            if constexpr (c == 2) load_w(std::integral_constant<int, (k + PF) % NS>{});
            if constexpr (!isx && ks == 0) {     // the x part is complete: bring it to the scale of the packed W_hh
#pragma unroll
                for (int sb = 0; sb < SB; ++sb)
#pragma unroll
                    for (int q = 0; q < 4; ++q) acc[sb][q] *= scale;
            }
            auto chain = [&](const u32x4_t (&wf)[4]) __attribute__((always_inline)) {
                if constexpr (isx) {
#pragma unroll
                    for (int q = 0; q < 4; ++q)
#pragma unroll
                        for (int sb = 0; sb < SB; ++sb) {
                            const f32x4_t zero = {0.f, 0.f, 0.f, 0.f};
                            acc[sb][q] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8_t, wf[q]),
                                                                                 __builtin_bit_cast(bf16x8_t, bop[i & 1][sb]),
                                                                                 ks == 0 ? zero : acc[sb][q], 0, 0, 0);
                        }
                } else {
#pragma unroll
                    for (int p = 1; p >= 0; --p)          // the small term first
#pragma unroll
                        for (int q = 0; q < 4; ++q)
#pragma unroll
                            for (int sb = 0; sb < SB; ++sb)
                                acc[sb][q] = __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(f16x8_t, wf[q]),
                                                                                    __builtin_bit_cast(f16x8_t, bop[i & 1][p * 2 + sb]),
                                                                                    acc[sb][q], 0, 0, 0);
                }
            };
            if constexpr (c == 0) chain(wl);
            else if constexpr (c == 1) chain(wres[k]);
            else chain(wbuf[k % NSLOT]);
            // the prefetch depths are the ones written here, not whatever the scheduler can hoist
            __builtin_amdgcn_sched_barrier(0);
            if constexpr (!isx && ks == KS - 1) cell_update(std::integral_constant<int, ut>{});
        });
        // the summaries of step tt + 2 go from registers to the ring, those of step tt + 3 leave HBM
        stash_x(ring == 0 ? 2 : ring - 1);
        fetch_x(tt + 3);
#pragma unroll
        for (int sb = 0; sb < SB; ++sb) {
            float u = upart[sb];
            u += __shfl_xor(u, 16);
            u += __shfl_xor(u, 32);
            if (g4 == 0) s_up[(cur * NW + wave) * SEQ + sb * 16 + n] = u;
            upart[sb] = 0.f;
        }
        ring = ring_next;
    }
    __syncthreads();
    if (wave == 0) emit_score(t0 + nb - 1, (nb - 1) & 1, true);       // the last step's logit, and whatever is still held back
#pragma unroll
    for (int ut = 0; ut < UT; ++ut)
#pragma unroll
        for (int sb = 0; sb < SB; ++sb)
            if (live[sb])
                *reinterpret_cast<float4 *>(a.c + sq[sb] * DG + wave * 32 + ut * 16 + 4 * g4) =
                    make_float4(c_reg[ut][sb][0], c_reg[ut][sb][1], c_reg[ut][sb][2], c_reg[ut][sb][3]);
}

size_t lstm_fused_lds(int d) { return d == 64 ? Fus<64>::lds : Fus<128>::lds; }

// One launch for the whole range of steps: groups of 32 sequences, never across layers.
hipError_t launch_lstm_fused(const LstmArgs &a, hipStream_t st)
{
    const unsigned groups = (unsigned)(a.L * ((a.BH + 31) / 32));
    const int nb = a.c1 - a.c0;
    hipError_t e;
    if (a.d == 64) {
        e = hipFuncSetAttribute(reinterpret_cast<const void *>(lstm_fused_kernel<64>), hipFuncAttributeMaxDynamicSharedMemorySize, (int)Fus<64>::lds);
        if (e != hipSuccess) return e;
        hipLaunchKernelGGL((lstm_fused_kernel<64>), dim3(groups), dim3(512), Fus<64>::lds, st, a, a.c0, nb);
    } else {
        e = hipFuncSetAttribute(reinterpret_cast<const void *>(lstm_fused_kernel<128>), hipFuncAttributeMaxDynamicSharedMemorySize, (int)Fus<128>::lds);
        if (e != hipSuccess) return e;
        hipLaunchKernelGGL((lstm_fused_kernel<128>), dim3(groups), dim3(512), Fus<128>::lds, st, a, a.c0, nb);
    }
    return hipGetLastError();
}

}  // namespace kvev

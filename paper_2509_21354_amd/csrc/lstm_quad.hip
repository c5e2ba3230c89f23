// Recurrent gate, Eq. 3 of the paper, bf16 storage, d_g = 512: 32 sequences on four compute units, one kernel for the
// input projection and the recurrence.
//
// At d_g = 512 the recurrent matrix is 2 MiB as fp16 and a compute unit pulls 64 bytes per clock out of L2: one
// workgroup per 16 sequences spends 14 us per step on that stream, a pair of workgroups (lstm_rec_pair_kernel) 7 us
// each for their halves.  Here four workgroups share a group of 32 sequences: each owns a quarter of the hidden units
// (8 waves x 16 units, all four gates) and, every step, contracts [x_t ; h_{t-1}] against its rows of [W_ih | W_hh]:
//   * W_ih x_t with bf16 operands (exact products), W_hh h_{t-1} with fp16 operands as in the other kernels (W_hh
//     scaled by a power of two s, h as hi + lo terms); the x part is accumulated first, multiplied by s (exact), then
//     the h part joins the same accumulators and the sum is scaled back once: fp32-grade throughout.  No projection
//     goes through memory (the two-kernel form writes and reads 8 KiB per sequence and step for them);
//   * a step streams 768 KiB of weights per compute unit, and every fragment that arrives serves two blocks of 16
//     sequences: 4.5 us of matrix work per step and unit against 5.5 us of stream.  A launch of 64 such groups (2048
//     sequences) is one workgroup per compute unit;
//   * the summaries of step t + 3 are in flight from HBM while step t is computed (registers -> a three-deep ring in
//     LDS), and the x part of step t + 1 is multiplied right after the cell of step t, before the step's last
//     barrier: it needs nothing from the other waves, and it covers the exchange below.
//
// What the members owe each other every step is the new h of their quarters (32 x 128 values as hi + lo fp16 terms).
// A wave publishes its unit tile with one 16-byte device-scope store per lane and block of sequences, into a slot of
// its own: two 8-byte words {hi, hi, lo, lo}, each of which a store writes and a load reads as one.  |h| <= 1, so bit
// 14 of an fp16 hi term (set from 2.0 on) is free: the first hi of each word carries a flag there that says which use
// of the slot the word belongs to, and the same wave of each other member polls the slot until every word carries
// the flag of the step it waits for; no separate flag, fence or ordering between addresses is involved.  Two slots
// by step parity: a slot is rewritten two steps later, which its writer reaches only after all three readers have
// consumed it (it needs their next h, published after that read); so a reader finds either the step it waits for or
// the use before it (or the zeros that a small launch leaves in all slots first), and one bit, flipped from use to
// use and set on the first one, tells them apart.  (A NaN in h has bit 14 set in its hi term: the reader recognises
// the exponent that no |h| <= 1 can have once the flag is masked off and puts the NaN back.)
//
// A step:  products over the own quarter of h (no exchange needed) | take the partners' quarters, stage them in LDS |
// barrier | products over the other three quarters | cell, publish, own h to LDS | x part of the next step | barrier.
// One copy of h in LDS is enough: the own quarter's columns are read before the first barrier only and written after
// it, the partners' columns are written before the first barrier and read after it.  The utility logit
// w_s . h_t + b_s is completed one step later by one wave of member 0.
//
// Every wait is bounded (a.pair_spin_limit polls); on expiry the workgroup leaves the loop together, marks the launch's
// scores and cell state NaN and sets the status word at the head of the caller's scratch.  The members of a group are
// neighbours in the launch order, workgroups are started in that order, and the host takes this kernel only while the
// launch has at most one workgroup per compute unit of the device: a running member's partners are next in line for
// the first unit that frees up.
#include "common.hpp"
#include "kernels.hpp"
#include "lstm_common.hpp"
#include <atomic>
#include <utility>

namespace kvev {

template <int D> struct QuadGeo {
    static constexpr int DG = 512, NW = 8, NM = 4, SB = 2, SEQ = 16 * SB;
    static constexpr int KS = DG / 32, KQ = KS / NM, KX = 2 * D / 32, WALK = KS + KX, HP = DG + 8, XP = 2 * D + 8;
    // The cyclic walk of a wave over its weight items (4 KiB each): positions [0, KS) are the k-steps of W_hh (own
    // quarter first), [KS, WALK) those of W_ih for the step after.  All items stream from L2 through a ring of NSLOT
    // register buffers that runs PF items ahead.
    static constexpr int NSLOT = 4, PF = NSLOT - 1;
    static_assert(WALK % NSLOT == 0, "slot rotation must line up with the walk");
    static_assert(WALK % 2 == 0, "operand buffer parity must survive the wrap into the next step");
    static constexpr uint32_t slot_bytes = SB * 1024;                        // one wave's publication: a line of 1 KiB per block of 16 sequences
    static constexpr uint32_t exch_bytes = 2 * NM * NW * slot_bytes;         // [parity][member][wave] per group of 32 sequences
    static constexpr size_t lds_h = (size_t)2 * SEQ * HP * sizeof(f16_t);       // [hi, lo][sequence][unit]
    static constexpr size_t lds_x = (size_t)3 * SEQ * XP * sizeof(bf16_t);      // [ring of 3 steps][sequence][2d]
    static constexpr size_t lds_up = (size_t)2 * NW * SB * 64 * sizeof(float);  // own shares of the utility logit, by step parity
    static constexpr size_t lds_up2 = (size_t)NW * SB * 64 * sizeof(float);     // the partners' shares
    static constexpr size_t lds_b = (size_t)4 * (DG / NM) * sizeof(float);      // b_ih + b_hh of the own quarter
    static constexpr size_t lds_ws = (size_t)DG * sizeof(float);                // w_s
    static constexpr size_t lds = lds_h + lds_x + lds_up + lds_up2 + lds_b + lds_ws + 16;
    static_assert(lds <= 160 * 1024, "LDS budget of a CU");
};
static_assert(QuadGeo<128>::exch_bytes == kLstmQuadExchBytes, "the scratch planner's figure");

__global__ __launch_bounds__(256) void lstm_quad_clear_kernel(uint4 *p, size_t n16)
{
    for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n16; i += (size_t)gridDim.x * 256) p[i] = make_uint4(0u, 0u, 0u, 0u);
}

// g0, ng: the launch takes groups g0 .. g0 + ng - 1 of the call (four workgroups each)
template <int D>
__global__ __launch_bounds__(512) void lstm_quad_kernel(LstmArgs a, int t0, int nb, int g0, int ng)
{
    using G = Geo<512>;                    // the packed operands keep the single-workgroup kernel's geometry
    using Q = QuadGeo<D>;
    constexpr int NW = Q::NW, NM = Q::NM, SB = Q::SB, SEQ = Q::SEQ, KS = Q::KS, KQ = Q::KQ, KX = Q::KX, WALK = Q::WALK;
    constexpr int HP = Q::HP, XP = Q::XP, DG = Q::DG, NSLOT = Q::NSLOT, PF = Q::PF;
    typedef _Float16 f16x4_t __attribute__((ext_vector_type(4)));
    extern __shared__ __align__(16) unsigned char smem_quad[];
    f16_t *s_h = reinterpret_cast<f16_t *>(smem_quad);
    bf16_t *s_x = reinterpret_cast<bf16_t *>(smem_quad + Q::lds_h);
    float *s_up = reinterpret_cast<float *>(smem_quad + Q::lds_h + Q::lds_x);                       // [2][NW][SB][64]
    float *s_up2 = reinterpret_cast<float *>(smem_quad + Q::lds_h + Q::lds_x + Q::lds_up);          // [NW][SB][64]
    float *s_bias = reinterpret_cast<float *>(smem_quad + Q::lds_h + Q::lds_x + Q::lds_up + Q::lds_up2);   // [4][DG / NM]
    float *s_ws = reinterpret_cast<float *>(smem_quad + Q::lds_h + Q::lds_x + Q::lds_up + Q::lds_up2 + Q::lds_b);
    int &s_fail = *reinterpret_cast<int *>(smem_quad + Q::lds_h + Q::lds_x + Q::lds_up + Q::lds_up2 + Q::lds_b + Q::lds_ws);

    const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int n = lane & 15, g4 = lane >> 4;
    const int gpl = (a.BH + SEQ - 1) / SEQ;
    // Members of a group are neighbours in the launch order, and hardware workgroup ids go round-robin over the 8
    // XCDs: XCD x runs member x % 4 of the groups of the parity of x / 4.  The groups of one parity are given a
    // contiguous run of (layer, group) pairs, so that an XCD's L2 serves one member's weights of half the layers, and
    // the groups of a layer find them there together, instead of every layer's weights once.
    const int member = blockIdx.x & 3;
    const int slot = blockIdx.x >> 2;          // the group's place in this launch: its exchange slots
    if (slot >= ng) return;
    const int gid = g0 + (ng % 2 == 0 ? (slot & 1) * (ng / 2) + (slot >> 1) : slot);
    const int l = gid / gpl, grp = gid % gpl;
    bool live[SB];
    size_t sq[SB];
#pragma unroll
    for (int sb = 0; sb < SB; ++sb) {
        live[sb] = grp * SEQ + sb * 16 + n < a.BH;
        sq[sb] = (size_t)l * a.BH + min(grp * SEQ + sb * 16 + n, a.BH - 1);
    }
    // unit tiles (16 units) by quarter: quarter 0 is this workgroup's own, 1..3 the partners' in ring order
    int tile_q[NM];
#pragma unroll
    for (int qd = 0; qd < NM; ++qd) tile_q[qd] = ((member + qd) & 3) * NW + wave;
    const int tile = tile_q[0];

    const float b_s = bf16_to_f32(static_cast<const bf16_t *>(a.b_s)[l]);
    const int sexp = whh_scale_exp(whh_layer_max(a.whh_max_bits, l));
    const float scale = ldexpf(1.f, sexp), inv_scale = ldexpf(1.f, -sexp);
    if (tid == 0) s_fail = 0;
    s_ws[tid] = bf16_to_f32(static_cast<const bf16_t *>(a.w_s)[(size_t)l * DG + tid]);
    {
        const int q = tid / (DG / NM), u = member * (DG / NM) + tid % (DG / NM);       // 512 threads: 4 gates x 128 units
        s_bias[tid] = bf16_to_f32(static_cast<const bf16_t *>(a.b_ih)[(size_t)l * 4 * DG + q * DG + u]) +
                      bf16_to_f32(static_cast<const bf16_t *>(a.b_hh)[(size_t)l * 4 * DG + q * DG + u]);
    }

    const uint32_t lane16 = lane * 16;
    // the wave's weights.  W_hh: the item of k-step ks at ks * 4096 from the tile's place in the packed order, fragment
    // q at q * 1024; W_ih: fragment (q, ks) at (q * KX + ks) * 1024
    const __amdgpu_buffer_rsrc_t wh_rsrc = make_rsrc(
        reinterpret_cast<const unsigned char *>(a.whh_packed + (((size_t)l * G::NW + tile / G::UT) * G::ITEMS + (tile % G::UT) * G::KS) * 4 * 64),
        KS * 4096);
    const __amdgpu_buffer_rsrc_t wx_rsrc = make_rsrc(
        reinterpret_cast<const unsigned char *>(a.wih_packed + (((size_t)l * G::NW + tile / G::UT) * G::UT + tile % G::UT) * 4 * KX * 64),
        KX * 4096);
    u32x4_t wbuf[NSLOT][4];
    auto load_w = [&](auto cc) __attribute__((always_inline)) {        // cc: position in the walk
        constexpr int c = decltype(cc)::value;
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            if constexpr (c < KS)       // quarter c / KQ (own first), k-step c % KQ within it
                wbuf[c % NSLOT][q] = buffer_load16<u32x4_t>(wh_rsrc, lane16 + q * 1024, (uint32_t)(((((member + c / KQ) & 3) * KQ) + c % KQ) * 4096));
            else
                wbuf[c % NSLOT][q] = buffer_load16<u32x4_t>(wx_rsrc, lane16, (q * KX + (c - KS)) * 1024);
        }
    };
    static_for<PF>([&](auto ic) { load_w(std::integral_constant<int, KS + decltype(ic)::value>{}); });

    const __amdgpu_buffer_rsrc_t e_rsrc = make_rsrc(a.exch + (size_t)slot * Q::exch_bytes, Q::exch_bytes);

    float c_reg[SB][4];
    f16_t *h_wr[NM];             // + (plane*SEQ + sb*16)*HP
    const f16_t *h_rd[NM];       // + (plane*SEQ + sb*16)*HP + j*32
#pragma unroll
    for (int qd = 0; qd < NM; ++qd) {
        h_wr[qd] = s_h + (size_t)n * HP + tile_q[qd] * 16 + 4 * g4;
        h_rd[qd] = s_h + (size_t)n * HP + ((member + qd) & 3) * KQ * 32 + g4 * 8;
    }
    const bf16_t *x_rd = s_x + (size_t)n * XP + g4 * 8;            // + (ring*SEQ + sb*16)*XP + ks*32
    auto split = [](const float (&hv)[4], f16x4_t &hi, f16x4_t &lo) {
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            hi[r] = (f16_t)hv[r];
            lo[r] = (f16_t)(hv[r] - (float)hi[r]);
        }
    };
    auto put_h = [&](int qd, int sb, f16x4_t hi, f16x4_t lo) __attribute__((always_inline)) {
        *reinterpret_cast<f16x4_t *>(h_wr[qd] + ((size_t)0 * SEQ + sb * 16) * HP) = hi;
        *reinterpret_cast<f16x4_t *>(h_wr[qd] + ((size_t)1 * SEQ + sb * 16) * HP) = lo;
    };
#pragma unroll
    for (int qd = 0; qd < NM; ++qd) {       // h of step t0 - 1, all quarters, from the fp32 state
#pragma unroll
        for (int sb = 0; sb < SB; ++sb) {
            float hv[4];
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                const int u = tile_q[qd] * 16 + 4 * g4 + r;
                // (chunk 0 starts the recurrence from a zero state, whatever the buffers hold)
                hv[r] = live[sb] && t0 > 0 ? a.h[sq[sb] * DG + u] : 0.f;
                if (qd == 0) c_reg[sb][r] = live[sb] && t0 > 0 ? a.c[sq[sb] * DG + u] : 0.f;
            }
            f16x4_t hi, lo;
            split(hv, hi, lo);
            put_h(qd, sb, hi, lo);
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

    // one look at the same wave's slots of the three partners, parity `par` (device-scope loads, examined later)
    struct Look { u32x4_t v[NM - 1][SB]; };
    auto ask = [&](int par, Look &k) __attribute__((always_inline)) {
#pragma unroll
        for (int qd = 1; qd < NM; ++qd) {
            const uint32_t off = (uint32_t)((par * NM + ((member + qd) & 3)) * NW + wave) * Q::slot_bytes;
#pragma unroll
            for (int sb = 0; sb < SB; ++sb)
                k.v[qd - 1][sb] = __builtin_amdgcn_raw_buffer_load_b128(e_rsrc, (int)lane16, (int)(off + sb * 1024), 16);
        }
    };
    // the flag of the publication of step tt (within the launch): flipped from one use of a slot to the next, set on the first
    auto flag_of = [](int tt) { return (uint32_t)(((tt >> 1) + 1) & 1) << 14; };
    // The partners' h of step tt, from slots of parity `par`: staged in LDS, their share of the utility logit left in
    // s_up2.  k: a look asked for earlier; more looks follow until every word carries the step's flag.
    auto receive = [&](int par, int tt, Look &k) __attribute__((always_inline)) {
        const uint32_t flag = flag_of(tt);
        auto all_in = [&](const Look &x) __attribute__((always_inline)) {
            bool ok = true;
#pragma unroll
            for (int qd = 0; qd < NM - 1; ++qd)
#pragma unroll
                for (int sb = 0; sb < SB; ++sb) ok = ok && (x.v[qd][sb][0] & 0x4000u) == flag && (x.v[qd][sb][2] & 0x4000u) == flag;
            return __all(ok) != 0;
        };
        bool got = all_in(k);
        for (int spin = 0; !got && spin < a.pair_spin_limit; ++spin) {
            if ((spin & 255) == 255 && s_fail) break;
            ask(par, k);
            asm volatile("" ::: "memory");
            got = all_in(k);
        }
        if (!got) s_fail = 1;
        float up[SB] = {0.f, 0.f};
#pragma unroll
        for (int qd = 1; qd < NM; ++qd) {
            const f32x4_t ws = *reinterpret_cast<const f32x4_t *>(s_ws + tile_q[qd] * 16 + 4 * g4);
#pragma unroll
            for (int sb = 0; sb < SB; ++sb) {
                const u32x4_t v = k.v[qd - 1][sb];
                // the flag off; an exponent of 15 with a mantissa is what that leaves of a NaN
                uint32_t h0 = v[0] & ~0x4000u, h2 = v[2] & ~0x4000u;
                if ((h0 & 0x7FFFu) > 0x3C00u) h0 |= 0x4000u;
                if ((h2 & 0x7FFFu) > 0x3C00u) h2 |= 0x4000u;
                const f16x4_t hi = __builtin_bit_cast(f16x4_t, make_uint2(h0, h2)), lo = __builtin_bit_cast(f16x4_t, make_uint2(v[1], v[3]));
                put_h(qd, sb, hi, lo);
#pragma unroll
                for (int r = 0; r < 4; ++r) up[sb] = fmaf(ws[r], (float)hi[r] + (float)lo[r], up[sb]);
            }
        }
#pragma unroll
        for (int sb = 0; sb < SB; ++sb) s_up2[(wave * SB + sb) * 64 + lane] = up[sb];
    };
    // Member 0 completes the logit of a step once all quarters are in: own shares (parity `ub`), then the partners'.
    auto write_util = [&](int ub, int step) __attribute__((always_inline)) {
        if (member == 0 && wave == 0) {
#pragma unroll
            for (int sb = 0; sb < SB; ++sb) {
                float u = 0.f;
#pragma unroll
                for (int w = 0; w < NW; ++w) u += s_up[((ub * NW + w) * SB + sb) * 64 + lane];
#pragma unroll
                for (int w = 0; w < NW; ++w) u += s_up2[(w * SB + sb) * 64 + lane];
                u += __shfl_xor(u, 16);
                u += __shfl_xor(u, 32);
                u += b_s;
                if (live[sb] && g4 == 0) {
                    a.util[sq[sb] * a.N_cap + t0 + step] = u;
                    a.gate[sq[sb] * a.N_cap + t0 + step] = sigmoid_hw(u);
                }
            }
        }
    };
    // B operands of the item at walk position c: an h item takes (lo, hi) x 2 sequence blocks, an x item 2 blocks
    u32x4_t bop[2][4];
    auto read_ops = [&](auto cc, int ring) __attribute__((always_inline)) {
        constexpr int c = decltype(cc)::value;
        if constexpr (c < KS) {
#pragma unroll
            for (int pl = 0; pl < 2; ++pl)
#pragma unroll
                for (int sb = 0; sb < SB; ++sb)
                    bop[c & 1][pl * 2 + sb] = *reinterpret_cast<const u32x4_t *>(h_rd[c / KQ] + ((size_t)pl * SEQ + sb * 16) * HP + (c % KQ) * 32);
        } else {
#pragma unroll
            for (int sb = 0; sb < SB; ++sb)
                bop[c & 1][sb] = *reinterpret_cast<const u32x4_t *>(x_rd + ((size_t)ring * SEQ + sb * 16) * XP + (c - KS) * 32);
        }
    };
    using std::integral_constant;

    f32x4_t acc[SB][4];
    // walk positions [C0, C1): the operands of an item are read while the item before it is multiplied (ring: the
    // slot of the summaries that x items take)
    auto run = [&](auto c0c, auto c1c, int ring) __attribute__((always_inline)) {
        constexpr int C0 = decltype(c0c)::value, C1 = decltype(c1c)::value;
        read_ops(c0c, ring);
        static_for<C1 - C0>([&](auto ic) {
            constexpr int c = C0 + decltype(ic)::value;
            if constexpr (c + 1 < C1) read_ops(integral_constant<int, c + 1>{}, ring);
            load_w(integral_constant<int, (c + PF) % WALK>{});
            const u32x4_t (&wf)[4] = wbuf[c % NSLOT];
            if constexpr (c >= KS) {
#pragma unroll
                for (int q = 0; q < 4; ++q)
#pragma unroll
                    for (int sb = 0; sb < SB; ++sb) {
                        const f32x4_t zero = {0.f, 0.f, 0.f, 0.f};
                        acc[sb][q] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8_t, wf[q]),
                                                                             __builtin_bit_cast(bf16x8_t, bop[c & 1][sb]),
                                                                             c == KS ? zero : acc[sb][q], 0, 0, 0);
                    }
            } else {
#pragma unroll
                for (int pl = 1; pl >= 0; --pl)          // the small term first
#pragma unroll
                    for (int q = 0; q < 4; ++q)
#pragma unroll
                        for (int sb = 0; sb < SB; ++sb)
                            acc[sb][q] = __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(f16x8_t, wf[q]),
                                                                                __builtin_bit_cast(f16x8_t, bop[c & 1][pl * 2 + sb]),
                                                                                acc[sb][q], 0, 0, 0);
            }
            __builtin_amdgcn_sched_barrier(0);      // the ring's depth is the one written here
        });
    };
    // the x part of a step: W_ih x on the summaries in ring slot `ring`, brought to the scale of the packed W_hh
    auto x_part = [&](int ring) __attribute__((always_inline)) {
        run(integral_constant<int, KS>{}, integral_constant<int, WALK>{}, ring);
#pragma unroll
        for (int sb = 0; sb < SB; ++sb)
#pragma unroll
            for (int q = 0; q < 4; ++q) acc[sb][q] *= scale;
    };

    __syncthreads();             // h of step t0 - 1, the first two steps' summaries, bias and w_s are in place
    x_part(0);

    bool failed = false;
    int ring = 0;                // tt % 3
    for (int tt = 0; tt < nb; ++tt) {
        const int cur = tt & 1, nxt = cur ^ 1;
        const int ring_next = ring == 2 ? 0 : ring + 1;
        // the summaries of step tt + 2 go from registers to the ring, those of step tt + 3 leave HBM
        stash_x(ring == 0 ? 2 : ring - 1);
        fetch_x(tt + 3);
        // the partners published h of step tt - 1 at the end of that step (slots of parity nxt)
        Look k;
        if (tt > 0) ask(nxt, k);
        __builtin_amdgcn_sched_barrier(0);
        run(integral_constant<int, 0>{}, integral_constant<int, KQ>{}, 0);
        if (tt > 0) receive(nxt, tt - 1, k);
        lds_barrier();
        if (s_fail) { failed = true; break; }
        run(integral_constant<int, KQ>{}, integral_constant<int, KS>{}, 0);

        f32x4_t bias[4];
#pragma unroll
        for (int q = 0; q < 4; ++q) bias[q] = *reinterpret_cast<const f32x4_t *>(s_bias + q * (DG / NM) + wave * 16 + 4 * g4);
        const f32x4_t ws = *reinterpret_cast<const f32x4_t *>(s_ws + tile * 16 + 4 * g4);
#pragma unroll
        for (int sb = 0; sb < SB; ++sb) {
            float hv[4], upart = 0.f;
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                const float ig = sigmoid_hw(fmaf(acc[sb][0][r], inv_scale, bias[0][r]));
                const float fg = sigmoid_hw(fmaf(acc[sb][1][r], inv_scale, bias[1][r]));
                const float gg = tanh_hw(fmaf(acc[sb][2][r], inv_scale, bias[2][r]));
                const float og = sigmoid_hw(fmaf(acc[sb][3][r], inv_scale, bias[3][r]));
                const float cn = fmaf(fg, c_reg[sb][r], ig * gg);
                c_reg[sb][r] = cn;
                float hn = og * tanh_hw(cn);
                asm volatile("" : "+v"(hn));     // opaque to the optimiser: hn is the rounded product from here on
                hv[r] = hn;
                upart = fmaf(ws[r], hn, upart);
            }
            f16x4_t hi, lo;
            split(hv, hi, lo);
            // to the partners first (the long way), then to this workgroup's own waves
            const uint2 hi2 = __builtin_bit_cast(uint2, hi), lo2 = __builtin_bit_cast(uint2, lo);
            const uint32_t flag = flag_of(tt);
            const uint32_t off = (uint32_t)((cur * NM + member) * NW + wave) * Q::slot_bytes + sb * 1024;
            const u32x4_t line = {(hi2.x & ~0x4000u) | flag, lo2.x, (hi2.y & ~0x4000u) | flag, lo2.y};
            if (member != a.pair_mute)         // device scope: the store writes through to where the partners' loads look
                __builtin_amdgcn_raw_buffer_store_b128(line, e_rsrc, (int)lane16, (int)off, 16);
            put_h(0, sb, hi, lo);
            if (tt == nb - 1 && live[sb])        // the state leaves the kernel as fp32
                *reinterpret_cast<float4 *>(a.h + sq[sb] * DG + tile * 16 + 4 * g4) = make_float4(hv[0], hv[1], hv[2], hv[3]);
            s_up[((cur * NW + wave) * SB + sb) * 64 + lane] = upart;
        }
        if (tt > 0) write_util(nxt, tt - 1);       // all quarters of step tt - 1 have been in LDS since this step's first barrier
        x_part(ring_next);                         // of step tt + 1: nothing in it depends on the other waves
        lds_barrier();
        ring = ring_next;
    }
    if (!failed) {      // the last step's logit needs the partners' last h
        Look k;
        ask((nb - 1) & 1, k);
        receive((nb - 1) & 1, nb - 1, k);
        lds_barrier();
        failed = s_fail != 0;
        if (!failed) write_util((nb - 1) & 1, nb - 1);
    }
#pragma unroll
    for (int sb = 0; sb < SB; ++sb)
        if (live[sb]) {
#pragma unroll
            for (int r = 0; r < 4; ++r) a.c[sq[sb] * DG + tile * 16 + 4 * g4 + r] = failed ? __builtin_nanf("") : c_reg[sb][r];
        }
    if (failed && tid == 0) __hip_atomic_store(a.status, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);   // sticky: the caller's to clear
    if (failed && tid < SEQ && grp * SEQ + tid < a.BH) {
        const size_t s = (size_t)l * a.BH + grp * SEQ + tid;
        for (int t = 0; t < nb; ++t) {
            a.util[s * a.N_cap + t0 + t] = __builtin_nanf("");
            a.gate[s * a.N_cap + t0 + t] = __builtin_nanf("");
        }
    }
}

template <int D>
static hipError_t launch_quad_d(const LstmArgs &a, hipStream_t st)
{
    static std::atomic<uint64_t> done{0};
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    const uint64_t bit = (uint64_t)1 << (dev & 63);
    if (!(done.load(std::memory_order_acquire) & bit)) {
        e = hipFuncSetAttribute(reinterpret_cast<const void *>(lstm_quad_kernel<D>), hipFuncAttributeMaxDynamicSharedMemorySize, (int)QuadGeo<D>::lds);
        if (e != hipSuccess) return e;
        done.fetch_or(bit, std::memory_order_release);
    }
    const int groups = a.L * ((a.BH + QuadGeo<D>::SEQ - 1) / QuadGeo<D>::SEQ);
    const int per_launch = a.quad_groups > 0 ? a.quad_groups : 1;
    // at most one workgroup per compute unit at a time: a call with more groups takes several launches, one after
    // the other on the stream, each with cleared exchange slots
    for (int g0 = 0; g0 < groups; g0 += per_launch) {
        const int ng = groups - g0 < per_launch ? groups - g0 : per_launch;
        const size_t n16 = (size_t)ng * QuadGeo<D>::exch_bytes / 16;
        hipLaunchKernelGGL(lstm_quad_clear_kernel, dim3((unsigned)((n16 + 1023) / 1024)), dim3(256), 0, st, reinterpret_cast<uint4 *>(a.exch), n16);
        hipLaunchKernelGGL(lstm_quad_kernel<D>, dim3((unsigned)(QuadGeo<D>::NM * ng)), dim3(512), QuadGeo<D>::lds, st, a, a.c0, a.c1 - a.c0, g0, ng);
    }
    return hipGetLastError();
}

// The whole range of steps in one launch per quad_groups groups (weights already packed), each after a small launch
// that clears the exchange slots.
hipError_t launch_lstm_quad(const LstmArgs &a, hipStream_t st)
{
    return a.d == 64 ? launch_quad_d<64>(a, st) : launch_quad_d<128>(a, st);
}

}  // namespace kvev

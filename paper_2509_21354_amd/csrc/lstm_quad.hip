// Recurrent gate, Eq. 3 of the paper, bf16 storage, d_g = 512: the recurrence of 32 sequences on four compute units.
//
// At d_g = 512 the recurrent matrix is 2 MiB as fp16, and a compute unit pulls 64 bytes per clock out of L2: one
// workgroup per 16 sequences spends 14 us per step on that stream, a pair of workgroups (lstm_rec_pair_kernel) 7 us
// each for their halves, against 1.8 us of matrix work.  Here four workgroups share a group of 32 sequences: each
// owns a quarter of the hidden units (8 waves x 16 units, all four gates), so a step streams 512 KiB per compute unit,
// and every weight fragment that arrives serves two blocks of 16 sequences: 3.6 us of matrix work per step and unit,
// about as long as its weight stream.  A launch of 64 such groups (2048 sequences) is one workgroup per compute unit.
//
// What the members owe each other every step is the new h of their quarters (32 x 128 values as hi + lo fp16 terms).
// The exchange is the paired kernel's: a wave publishes its unit tile as 16-byte stores of the form
// {payload, stamp, payload, stamp} (stamp = step + 1 within the launch) with device scope into a slot of its own, and
// the same wave of each other member polls that slot until every stamp carries the step it waits for.  Data and stamp
// share an aligned 8-byte word, so no flag, fence or ordering between addresses is involved.  Two slots by step
// parity: a slot is rewritten two steps later, which its writer reaches only after all three readers have consumed it
// (it needs their next h, published after that read).  The input projection's launch clears the slots.
//
// A step:  products over the own quarter of h (no exchange needed; the looks at the partners' slots are in flight
// behind them) | take the partners' quarters, stage them in LDS | barrier | products over the other three quarters |
// cell, publish | barrier.  The utility logit w_s . h_t + b_s is completed one step later by one wave of member 0.
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

struct QuadGeo {
    static constexpr int DG = 512, NW = 8, NM = 4, SB = 2, SEQ = 16 * SB;
    static constexpr int KS = DG / 32, KQ = KS / NM, ITEMS = KS, HP = DG + 8;
    // weight items of a wave (one per k-step, 4 KiB): RRES stay in registers, the rest streams from L2 through a ring
    // of NSLOT register buffers that runs PF items ahead, across the phases of a step and into the next step
    static constexpr int RRES = 0, NS = ITEMS - RRES, NSLOT = 4, PF = NSLOT - 1;
    static_assert(NS % NSLOT == 0, "slot rotation must line up with the item loop");
    static constexpr uint32_t slot_bytes = SB * 2 * 1024;                    // one wave's publication: SB blocks x (hi, lo) lines of 1 KiB
    static constexpr uint32_t exch_bytes = 2 * NM * NW * slot_bytes;         // [parity][member][wave] per group of 32 sequences
    static constexpr size_t lds_h = (size_t)2 * 2 * SEQ * HP * sizeof(f16_t);   // [buffer][hi, lo][sequence][unit]
    static constexpr size_t lds_up = (size_t)2 * NW * SB * 64 * sizeof(float);  // own shares of the utility logit, by step parity
    static constexpr size_t lds_up2 = (size_t)NW * SB * 64 * sizeof(float);     // the partners' shares
    static constexpr size_t lds = lds_h + lds_up + lds_up2 + 16;
    static_assert(lds <= 160 * 1024, "LDS budget of a CU");
};
static_assert(QuadGeo::exch_bytes == kLstmQuadExchBytes, "the scratch planner's figure");

__global__ __launch_bounds__(512) void lstm_rec_quad_kernel(LstmArgs a, int t0, int nb)
{
    using G = Geo<512>;                    // the packed operands keep the single-workgroup kernel's geometry
    using Q = QuadGeo;
    constexpr int NW = Q::NW, NM = Q::NM, SB = Q::SB, SEQ = Q::SEQ, KQ = Q::KQ, ITEMS = Q::ITEMS, HP = Q::HP, DG = Q::DG;
    constexpr int RRES = Q::RRES, NS = Q::NS, NSLOT = Q::NSLOT, PF = Q::PF;
    typedef _Float16 f16x4_t __attribute__((ext_vector_type(4)));
    extern __shared__ __align__(16) unsigned char smem_quad[];
    f16_t *s_h = reinterpret_cast<f16_t *>(smem_quad);
    float *s_up = reinterpret_cast<float *>(smem_quad + Q::lds_h);                       // [2][NW][SB][64]
    float *s_up2 = reinterpret_cast<float *>(smem_quad + Q::lds_h + Q::lds_up);          // [NW][SB][64]
    int &s_fail = *reinterpret_cast<int *>(smem_quad + Q::lds_h + Q::lds_up + Q::lds_up2);

    const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int n = lane & 15, g4 = lane >> 4;
    const int member = blockIdx.x & 3, gid = blockIdx.x >> 2;
    const int gpl = (a.BH + SEQ - 1) / SEQ, gpl16 = (a.BH + 15) / 16;
    if (gid >= a.L * gpl) return;
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

    const bf16_t *w_s = static_cast<const bf16_t *>(a.w_s) + (size_t)l * DG;
    const float b_s = bf16_to_f32(static_cast<const bf16_t *>(a.b_s)[l]);
    const float inv_scale = ldexpf(1.f, -whh_scale_exp(whh_layer_max(a.whh_max_bits, l)));
    if (tid == 0) s_fail = 0;

    const uint32_t lane16 = lane * 16;
    // the wave's weights: the item of k-step ks at ks * 4096 from the tile's place in the packed order
    const unsigned char *wbase = reinterpret_cast<const unsigned char *>(
        a.whh_packed + (((size_t)l * G::NW + tile / G::UT) * G::ITEMS + (tile % G::UT) * G::KS) * 4 * 64);
    const __amdgpu_buffer_rsrc_t w_rsrc = make_rsrc(wbase, ITEMS * 4096);
    // item p of the walk: quarter p / KQ (own first), k-step p % KQ within it
    auto item_off = [&](int p) { return (uint32_t)(((((member + p / KQ) & 3) * KQ) + p % KQ) * 4096); };
    f16x8_t wres[RRES > 0 ? RRES : 1][4];
    static_for<RRES>([&](auto pc) {
        constexpr int p = decltype(pc)::value;
#pragma unroll
        for (int q = 0; q < 4; ++q) wres[p][q] = buffer_load16<f16x8_t>(w_rsrc, lane16 + q * 1024, item_off(p));
    });
    f16x8_t wbuf[NSLOT][4];
    auto load_w = [&](auto sc) __attribute__((always_inline)) {        // sc: index within the streamed items
        constexpr int si = decltype(sc)::value, p = RRES + si;
#pragma unroll
        for (int q = 0; q < 4; ++q) wbuf[si % NSLOT][q] = buffer_load16<f16x8_t>(w_rsrc, lane16 + q * 1024, item_off(p));
    };
    static_for<PF>(load_w);

    // the input projections of the two blocks of 16 sequences (written per group of 16 by the projection kernel)
    __amdgpu_buffer_rsrc_t x_rsrc[SB];
#pragma unroll
    for (int sb = 0; sb < SB; ++sb) {
        const int g16 = l * gpl16 + min(grp * SB + sb, gpl16 - 1);      // (a block past the layer's end reads the last one; it is not live)
        const unsigned char *xbase = reinterpret_cast<const unsigned char *>(
            reinterpret_cast<const f32x4_t *>(a.xproj) + xp_block<DG>(g16, a.tb, 0, tile / G::UT, tile % G::UT, 0) * 64);
        x_rsrc[sb] = make_rsrc(xbase, (uint32_t)nb * G::NW * G::UT * 4096 - (uint32_t)tile * 4096);
    }
    const __amdgpu_buffer_rsrc_t e_rsrc = make_rsrc(a.exch + (size_t)gid * Q::exch_bytes, Q::exch_bytes);

    float c_reg[SB][4], ws_q[NM][4];
    f16_t *h_wr[NM];             // + ((buf*2 + plane)*SEQ + sb*16)*HP
    const f16_t *h_rd[NM];       // + ((buf*2 + plane)*SEQ + sb*16)*HP + j*32
#pragma unroll
    for (int qd = 0; qd < NM; ++qd) {
        h_wr[qd] = s_h + (size_t)n * HP + tile_q[qd] * 16 + 4 * g4;
        h_rd[qd] = s_h + (size_t)n * HP + ((member + qd) & 3) * KQ * 32 + g4 * 8;
    }
    auto split = [](const float (&hv)[4], f16x4_t &hi, f16x4_t &lo) {
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            hi[r] = (f16_t)hv[r];
            lo[r] = (f16_t)(hv[r] - (float)hi[r]);
        }
    };
    auto put_h = [&](int qd, int buf, int sb, f16x4_t hi, f16x4_t lo) __attribute__((always_inline)) {
        *reinterpret_cast<f16x4_t *>(h_wr[qd] + ((size_t)(buf * 2 + 0) * SEQ + sb * 16) * HP) = hi;
        *reinterpret_cast<f16x4_t *>(h_wr[qd] + ((size_t)(buf * 2 + 1) * SEQ + sb * 16) * HP) = lo;
    };
#pragma unroll
    for (int qd = 0; qd < NM; ++qd) {       // h of step t0 - 1, all quarters, from the fp32 state
#pragma unroll
        for (int r = 0; r < 4; ++r) ws_q[qd][r] = bf16_to_f32(w_s[tile_q[qd] * 16 + 4 * g4 + r]);
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
            put_h(qd, 0, sb, hi, lo);
        }
    }
    __syncthreads();

    // one look at the same wave's slots of the three partners, parity `par` (device-scope loads, examined later)
    struct Look { u32x4_t v[NM - 1][SB][2]; };
    auto ask = [&](int par, Look &k) __attribute__((always_inline)) {
#pragma unroll
        for (int qd = 1; qd < NM; ++qd) {
            const uint32_t off = (uint32_t)((par * NM + ((member + qd) & 3)) * NW + wave) * Q::slot_bytes;
#pragma unroll
            for (int sb = 0; sb < SB; ++sb)
#pragma unroll
                for (int pl = 0; pl < 2; ++pl)
                    k.v[qd - 1][sb][pl] = __builtin_amdgcn_raw_buffer_load_b128(e_rsrc, (int)lane16, (int)(off + (sb * 2 + pl) * 1024), 16);
        }
    };
    // The partners' h of the step stamped `stamp`, from slots of parity `par`: staged in LDS buffer `buf`, their share
    // of the utility logit left in s_up2.  k: a look asked for earlier; more looks follow until all stamps match.
    auto receive = [&](int par, uint32_t stamp, int buf, Look &k) __attribute__((always_inline)) {
        auto all_in = [&](const Look &x) __attribute__((always_inline)) {
            bool ok = true;
#pragma unroll
            for (int qd = 0; qd < NM - 1; ++qd)
#pragma unroll
                for (int sb = 0; sb < SB; ++sb)
#pragma unroll
                    for (int pl = 0; pl < 2; ++pl) ok = ok && x.v[qd][sb][pl][1] == stamp && x.v[qd][sb][pl][3] == stamp;
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
        for (int qd = 1; qd < NM; ++qd)
#pragma unroll
            for (int sb = 0; sb < SB; ++sb) {
                const u32x4_t vh = k.v[qd - 1][sb][0], vl = k.v[qd - 1][sb][1];
                const f16x4_t hi = __builtin_bit_cast(f16x4_t, make_uint2(vh[0], vh[2])), lo = __builtin_bit_cast(f16x4_t, make_uint2(vl[0], vl[2]));
                put_h(qd, buf, sb, hi, lo);
#pragma unroll
                for (int r = 0; r < 4; ++r) up[sb] = fmaf(ws_q[qd][r], (float)hi[r] + (float)lo[r], up[sb]);
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
    // the B operands of one k-step: (hi, lo) x the two blocks of sequences
    auto read_h = [&](f16x8_t (&dst)[2][SB], int buf, int qd, int j) __attribute__((always_inline)) {
#pragma unroll
        for (int pl = 0; pl < 2; ++pl)
#pragma unroll
            for (int sb = 0; sb < SB; ++sb)
                dst[pl][sb] = *reinterpret_cast<const f16x8_t *>(h_rd[qd] + ((size_t)(buf * 2 + pl) * SEQ + sb * 16) * HP + j * 32);
    };
    using std::integral_constant;

    bool failed = false;
    for (int tt = 0; tt < nb; ++tt) {
        const int cur = tt & 1, nxt = cur ^ 1;
        f32x4_t acc[SB][4], xin[SB][4];
#pragma unroll
        for (int sb = 0; sb < SB; ++sb)
#pragma unroll
            for (int q = 0; q < 4; ++q) acc[sb][q] = f32x4_t{0.f, 0.f, 0.f, 0.f};
        // the partners published h of step tt - 1 at the end of that step (slots of parity nxt, stamp tt)
        Look k;
        if (tt > 0) ask(nxt, k);
        __builtin_amdgcn_sched_barrier(0);

        f16x8_t hb[2][2][SB];
        // items [P0, P1) of the walk; the operands of an item are read while the item before it is multiplied
        auto run = [&](auto p0c, auto p1c) __attribute__((always_inline)) {
            constexpr int P0 = decltype(p0c)::value, P1 = decltype(p1c)::value;
            read_h(hb[P0 & 1], cur, P0 / KQ, P0 % KQ);
            static_for<P1 - P0>([&](auto ic) {
                constexpr int p = P0 + decltype(ic)::value;
                if constexpr (p + 1 < P1) read_h(hb[(p + 1) & 1], cur, (p + 1) / KQ, (p + 1) % KQ);
                if constexpr (p >= RRES) load_w(integral_constant<int, (p - RRES + PF) % NS>{});
                if constexpr (p == ITEMS - 2) {
                    // the input projections of this step, asked for one item before they are used
#pragma unroll
                    for (int sb = 0; sb < SB; ++sb)
#pragma unroll
                        for (int q = 0; q < 4; ++q)
                            xin[sb][q] = buffer_load16_nt<f32x4_t>(x_rsrc[sb], lane16 + q * 1024, (uint32_t)(tt * G::NW * G::UT) * 4096);
                }
                auto chain = [&](const f16x8_t (&wf)[4]) __attribute__((always_inline)) {
#pragma unroll
                    for (int pl = 1; pl >= 0; --pl)          // the small term first
#pragma unroll
                        for (int q = 0; q < 4; ++q)
#pragma unroll
                            for (int sb = 0; sb < SB; ++sb)
                                acc[sb][q] = __builtin_amdgcn_mfma_f32_16x16x32_f16(wf[q], hb[p & 1][pl][sb], acc[sb][q], 0, 0, 0);
                };
                if constexpr (p < RRES) chain(wres[p]);
                else chain(wbuf[(p - RRES) % NSLOT]);
                __builtin_amdgcn_sched_barrier(0);      // the ring's depth is the one written here
            });
        };
        run(integral_constant<int, 0>{}, integral_constant<int, KQ>{});
        if (tt > 0) {
            receive(nxt, (uint32_t)tt, cur, k);
            lds_barrier();
            if (s_fail) { failed = true; break; }
        }
        run(integral_constant<int, KQ>{}, integral_constant<int, ITEMS>{});

        float upart[SB];
#pragma unroll
        for (int sb = 0; sb < SB; ++sb) {
            float hv[4];
            upart[sb] = 0.f;
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                const float ig = sigmoid_hw(fmaf(acc[sb][0][r], inv_scale, xin[sb][0][r]));
                const float fg = sigmoid_hw(fmaf(acc[sb][1][r], inv_scale, xin[sb][1][r]));
                const float gg = tanh_hw(fmaf(acc[sb][2][r], inv_scale, xin[sb][2][r]));
                const float og = sigmoid_hw(fmaf(acc[sb][3][r], inv_scale, xin[sb][3][r]));
                const float cn = fmaf(fg, c_reg[sb][r], ig * gg);
                c_reg[sb][r] = cn;
                float hn = og * tanh_hw(cn);
                asm volatile("" : "+v"(hn));     // opaque to the optimiser: hn is the rounded product from here on
                hv[r] = hn;
                upart[sb] = fmaf(ws_q[0][r], hn, upart[sb]);
            }
            f16x4_t hi, lo;
            split(hv, hi, lo);
            // to the partners first (the long way), then to this workgroup's own waves
            const uint2 hi2 = __builtin_bit_cast(uint2, hi), lo2 = __builtin_bit_cast(uint2, lo);
            const uint32_t stamp = (uint32_t)tt + 1;
            const uint32_t off = (uint32_t)((cur * NM + member) * NW + wave) * Q::slot_bytes + sb * 2048;
            const u32x4_t l0 = {hi2.x, stamp, hi2.y, stamp}, l1 = {lo2.x, stamp, lo2.y, stamp};
            if (member != a.pair_mute) {       // device scope: the stores write through to where the partners' loads look
                __builtin_amdgcn_raw_buffer_store_b128(l0, e_rsrc, (int)lane16, (int)off, 16);
                __builtin_amdgcn_raw_buffer_store_b128(l1, e_rsrc, (int)lane16, (int)(off + 1024), 16);
            }
            put_h(0, nxt, sb, hi, lo);
            if (tt == nb - 1 && live[sb])
                *reinterpret_cast<float4 *>(a.h + sq[sb] * DG + tile * 16 + 4 * g4) = make_float4(hv[0], hv[1], hv[2], hv[3]);
            s_up[((cur * NW + wave) * SB + sb) * 64 + lane] = upart[sb];
        }
        if (tt > 0) write_util(nxt, tt - 1);       // all quarters of step tt - 1 have been in LDS since this step's first barrier
        lds_barrier();
    }
    if (!failed) {      // the last step's logit needs the partners' last h
        Look k;
        ask((nb - 1) & 1, k);
        receive((nb - 1) & 1, (uint32_t)nb, nb & 1, k);
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

// One launch per block of steps, after that block's input projection (which also clears the exchange slots).
hipError_t launch_lstm_rec_quad(const LstmArgs &a, int t0, int nb, hipStream_t st)
{
    static std::atomic<uint64_t> done{0};
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    const uint64_t bit = (uint64_t)1 << (dev & 63);
    if (!(done.load(std::memory_order_acquire) & bit)) {
        e = hipFuncSetAttribute(reinterpret_cast<const void *>(lstm_rec_quad_kernel), hipFuncAttributeMaxDynamicSharedMemorySize, (int)QuadGeo::lds);
        if (e != hipSuccess) return e;
        done.fetch_or(bit, std::memory_order_release);
    }
    const unsigned groups = (unsigned)(a.L * ((a.BH + QuadGeo::SEQ - 1) / QuadGeo::SEQ));
    hipLaunchKernelGGL(lstm_rec_quad_kernel, dim3(QuadGeo::NM * groups), dim3(512), QuadGeo::lds, st, a, t0, nb);
    return hipGetLastError();
}

}  // namespace kvev

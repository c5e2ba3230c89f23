// Recurrent gate, Eq. 3 of the paper, bf16 storage, on the matrix cores.
//
// Two kernels per block of steps:
//   lstm_inproj_kernel  the time-parallel half  W_ih [Kbar_t ; Vbar_t] + b_ih + b_hh
//                       for every step of the block (bf16 x bf16 products are
//                       exact in the fp32 accumulator), written to scratch in
//                       the exact register layout the recurrence reads back;
//   lstm_rec_kernel     the sequential half: one workgroup owns 16 sequences
//                       of one layer and walks them through the block's steps;
//   lstm_rec_pair_kernel  the same on two workgroups per 16 sequences, each
//                       with half of the hidden units, for launches small enough
//                       to be resident at once (further down).
// Before them, once per set of weights: lstm_prep_kernel (W_ih into fragment
// order, per-layer scale of W_hh) and lstm_pack_whh_kernel.  Launches with more
// sequence groups than compute units take one kernel for both halves instead
// (lstm_fused.hip), and so do launches at d_g = 512 that put 32 sequences on
// four workgroups (lstm_quad.hip); both share the preparation and the packed
// layouts of this file.
//
// Tiling (both kernels): v_mfma_f32_16x16x32_bf16 with the gate rows as the M
// side (A operand = weight rows, read straight from global memory / L2 in
// 16-byte pieces) and the 16 sequences as the N side (B operand = h or x).
// A wave owns UT tiles of 16 hidden units for all four gates, so i, f, g, o of a
// unit meet in the same lane and the cell update needs no data movement; with
// UT = 2 a workgroup has two waves per SIMD and one wave's weight loads hide
// behind the other's MFMAs.  Within a wave the unit tiles are walked one after the
// other (4 live accumulators), which leaves the registers to a deep ring of
// prefetched weight fragments.
//
// The state h is fp32 and the weights are bf16.  To feed the product W_hh h to the
// matrix cores without losing the state's precision, both go to fp16 operands:
//   * W_hh times a per-layer power of two s that lifts its largest magnitude to
//     [2^14, 2^15): a bf16 value has 8 significant bits, fp16 holds 11 and keeps
//     subnormals (checked on the device), so s*w is exact for every weight down to
//     2^-31 of the largest one (below that the rounding error is < 2^-39 of the
//     largest weight: far under the fp32 accumulation's own);
//   * h = hi + lo with hi = fp16(h), lo = fp16(h - hi): 22 significant bits (|h| < 1,
//     absolute error <= max(2^-22 |h|, 2^-25)).
// An fp16 x fp16 product has 22 bits and is exact in the fp32 accumulator, so two
// MFMAs per weight fragment give an fp32-grade W_hh h (three would be needed with
// bf16 terms); the result is scaled back by 1/s, exactly.
#include "common.hpp"
#include "kernels.hpp"
#include "lstm_common.hpp"
#include <atomic>
#include <utility>


namespace kvev {

constexpr int kTT = 8;   // steps per workgroup of the input projection (2 when that leaves compute units idle)

// Where the weight items of the recurrence live.  A CU pulls at most 64 bytes per
// clock out of L2, which for d_g = 256 (512 KiB of W_hh per step) is longer than
// the step's MFMA time, so part of the stream stays on chip: class 0 items sit in
// LDS, class 1 items in registers, and only class 2 items are streamed from L2
// every step, through a ring of NSLOT register buffers.  d_g <= 128 keeps the
// whole matrix in LDS; d_g = 512 has room for neither.  Resident items are spread
// over the step so that the streamed ones arrive at an even pace.
template <int DG> struct Res {
    using G = Geo<DG>;
    static constexpr int ITEMS = G::ITEMS;
    static constexpr int cls(int i)
    {
        if (DG <= 128) return 0;
        if (DG == 256) {                       // of 16: 3 in LDS, 7 in registers, 6 streamed
            constexpr int t[16] = {0, 1, 2, 1, 1, 2, 0, 1, 2, 1, 1, 2, 0, 1, 2, 2};
            return t[i];
        }
        return 2;
    }
    static constexpr int count(int c) { int k = 0; for (int i = 0; i < ITEMS; ++i) k += cls(i) == c; return k; }
    static constexpr int idx(int i) { int k = 0; for (int j = 0; j < i; ++j) k += cls(j) == cls(i); return k; }   // rank within its class
    static constexpr int pos(int c, int k) { for (int i = 0; i < ITEMS; ++i) if (cls(i) == c && idx(i) == k) return i; return 0; }
    static constexpr int LRES = count(0), RRES = count(1), NS = count(2);
    static constexpr int NSLOT = NS == 0 ? 1 : DG == 256 ? 3 : 8;
    static constexpr int PF = NSLOT - 1;
    static_assert(NS % NSLOT == 0, "slot rotation must line up with the item loop");
    // register buffers for LDS items, read one item ahead: two when LDS items follow each other
    static constexpr bool lds_adjacent() { for (int i = 0; i < ITEMS; ++i) if (cls(i) == 0 && cls((i + 1) % ITEMS) == 0) return true; return false; }
    static constexpr int NWL = lds_adjacent() ? 2 : 1;
    static_assert(NWL == 1 || LRES % 2 == 0, "buffer parity must survive the wrap into the next step");
    static constexpr size_t lds_h = (size_t)2 * 2 * 16 * (DG + 8) * sizeof(f16_t);      // 2 buffers x (hi, lo) planes
    static constexpr size_t lds_up = (size_t)2 * G::NW * 16 * sizeof(float);
    static constexpr size_t lds_w = (size_t)G::NW * LRES * 4096;
    static constexpr size_t lds = lds_h + lds_up + lds_w;
    static_assert(lds <= 160 * 1024, "LDS budget of a CU");
};

// The 16 sequences x TT steps of input rows [Kbar_t ; Vbar_t] that a workgroup projects are staged once in
// LDS (every wave needs all of them as the B operand); a wave keeps the 2d-long weight rows of one (unit tile,
// gate) in registers and walks the TT steps with them.  Its output is the bulk of the traffic (4*d_g floats per
// sequence and step), written as 1 KiB per wave-level store in the fragment layout the recurrence reads back.
template <int DG> __device__ void pack_whh_blocks(const LstmArgs &a, int block, int nblocks);

template <int DG, int D, int TT>
__global__ __launch_bounds__(Geo<DG>::THREADS) void lstm_inproj_kernel(LstmArgs a, int t0, int nb)
{
    constexpr int KS = 2 * D / 32, UT = Geo<DG>::UT, XP = 2 * D + 8, THREADS = Geo<DG>::THREADS;
    if (a.exch_bytes) {      // the paired recurrence that follows starts from cleared exchange slots
        const size_t nthreads = (size_t)gridDim.x * gridDim.y * THREADS;
        for (size_t i = ((size_t)blockIdx.y * gridDim.x + blockIdx.x) * THREADS + threadIdx.x; i * 16 < a.exch_bytes; i += nthreads)
            reinterpret_cast<uint4 *>(a.exch)[i] = make_uint4(0u, 0u, 0u, 0u);
    }
    extern __shared__ __align__(16) unsigned char smem_in[];
    bf16_t *s_x = reinterpret_cast<bf16_t *>(smem_in);           // [TT][16][XP]
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int n = lane & 15, g4 = lane >> 4;
    const int gpl = (a.BH + 15) / 16;
    const int gid = xcd_order(blockIdx.x, gridDim.x);
    const int l = gid / gpl, grp = gid % gpl;
    const int tt0 = blockIdx.y * TT;

    // stage the rows: 16-byte pieces, 2D/8 per row (the first D/8 from Kbar, the rest from Vbar)
    const bf16_t *Kbar = static_cast<const bf16_t *>(a.Kbar), *Vbar = static_cast<const bf16_t *>(a.Vbar);
    constexpr int PPR = 2 * D / 8;
    for (int p = tid; p < TT * 16 * PPR; p += THREADS) {
        const int piece = p % PPR, row = p / PPR, sq = row % 16, j = row / 16;
        const size_t s = (size_t)l * a.BH + min(grp * 16 + sq, a.BH - 1);
        const int t = t0 + min(tt0 + j, nb - 1);
        const int e = piece * 8;
        const bf16_t *src = e < D ? Kbar + (s * a.N_cap + t) * D + e : Vbar + (s * a.N_cap + t) * D + (e - D);
        *reinterpret_cast<bf16x8_t *>(s_x + (size_t)row * XP + e) = *reinterpret_cast<const bf16x8_t *>(src);
    }
    __syncthreads();

    const bf16x8_t *Wp = a.wih_packed + ((size_t)l * Geo<DG>::NW + wave) * UT * 4 * KS * 64 + lane;
    const bf16_t *b_ih = static_cast<const bf16_t *>(a.b_ih) + (size_t)l * 4 * DG;
    const bf16_t *b_hh = static_cast<const bf16_t *>(a.b_hh) + (size_t)l * 4 * DG;
    const bf16_t *xrd = s_x + (size_t)n * XP + g4 * 8;           // + j*16*XP + ks*32
    bf16x8_t wf[2][KS];
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) wf[0][ks] = Wp[(size_t)ks * 64];
#pragma unroll
    for (int it = 0; it < UT * 4; ++it) {
        const int ut = it / 4, q = it % 4;
        const int row0 = q * DG + wave * 16 * UT + ut * 16;
        // the next (unit tile, gate)'s weight rows travel while this one is used
        if (it + 1 < UT * 4) {
#pragma unroll
            for (int ks = 0; ks < KS; ++ks) wf[(it + 1) & 1][ks] = Wp[((size_t)(it + 1) * KS + ks) * 64];
        }
        float bias[4];
#pragma unroll
        for (int r = 0; r < 4; ++r)
            bias[r] = bf16_to_f32(b_ih[row0 + 4 * g4 + r]) + bf16_to_f32(b_hh[row0 + 4 * g4 + r]);
        // (a real loop for the long tiles: unrolled, the rows' fragments fill the register file, and by two it measured
        // 4 % slower; the two-step tiles of small launches are faster unrolled)
#pragma unroll TT <= 2 ? 2 : 1
        for (int j = 0; j < TT; ++j) {
            f32x4_t acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int ks = 0; ks < KS; ++ks) {
                const bf16x8_t xb = *reinterpret_cast<const bf16x8_t *>(xrd + (size_t)j * 16 * XP + ks * 32);
                acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(wf[it & 1][ks], xb, acc, 0, 0, 0);
            }
            if (tt0 + j < nb) {
                const f32x4_t o = {acc[0] + bias[0], acc[1] + bias[1], acc[2] + bias[2], acc[3] + bias[3]};
                float *dst = a.xproj + xp_block<DG>(gid, a.tb, tt0 + j, wave, ut, q) * 256 + lane * 4;
                *reinterpret_cast<f32x4_t *>(dst) = o;
            }
        }
    }
}

// Weight preparation, one launch: blocks [0, nb_wih) re-lay W_ih in A-fragment order for the input projection
// ([layer][wave][unit tile][gate][k-step][lane][8]); the kScaleBlocks blocks per layer after them each write the
// largest finite |W_hh| of their share of the layer as a bit pattern (non-negative floats order like unsigned
// integers) into a slot of their own: no atomics, nothing to clear between calls.
template <int DG, int D>
__global__ __launch_bounds__(256) void lstm_prep_kernel(const bf16_t *W_ih, bf16x8_t *wih_packed, const bf16_t *W_hh,
                                                        uint32_t *max_bits, int L, int nb_wih)
{
    const int t = threadIdx.x;
    if ((int)blockIdx.x < nb_wih) {
        constexpr int NW = Geo<DG>::NW, UT = Geo<DG>::UT, KS = 2 * D / 32;
        const size_t frag = (size_t)blockIdx.x * 256 + t;
        const size_t total = (size_t)L * NW * UT * 4 * KS * 64;
        if (frag >= total) return;
        const int lane = frag % 64;
        size_t r = frag / 64;
        const int ks = r % KS; r /= KS;
        const int q = r % 4; r /= 4;
        const int ut = r % UT; r /= UT;
        const int wave = r % NW;
        const int l = (int)(r / NW);
        const int n = lane & 15, g4 = lane >> 4;
        const bf16_t *src = W_ih + ((size_t)l * 4 * DG + q * DG + wave * 16 * UT + ut * 16 + n) * 2 * D + ks * 32 + g4 * 8;
        wih_packed[frag] = *reinterpret_cast<const bf16x8_t *>(src);
        return;
    }
    __shared__ float s_max[4];
    const int b = (int)blockIdx.x - nb_wih, l = b / kScaleBlocks, part = b % kScaleBlocks;
    constexpr size_t per_layer = (size_t)4 * DG * DG;
    const bf16_t *W = W_hh + (size_t)l * per_layer;
    float m = 0.f;
    for (size_t i = ((size_t)part * 256 + t) * 8; i < per_layer; i += (size_t)kScaleBlocks * 256 * 8) {
        const uint4 v = *reinterpret_cast<const uint4 *>(W + i);
        const uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const float lo = fabsf(__uint_as_float(w[j] << 16)), hi = fabsf(__uint_as_float(w[j] & 0xFFFF0000u));
            m = fmaxf(m, (lo == lo && lo < INFINITY) ? lo : 0.f);       // a NaN or infinite weight takes no part
            m = fmaxf(m, (hi == hi && hi < INFINITY) ? hi : 0.f);
        }
    }
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) m = fmaxf(m, __shfl_xor(m, off));
    if ((t & 63) == 0) s_max[t >> 6] = m;
    __syncthreads();
    if (t == 0) max_bits[b] = __float_as_uint(fmaxf(fmaxf(s_max[0], s_max[1]), fmaxf(s_max[2], s_max[3])));
}

// W_hh scaled, converted to fp16 and re-laid in A-fragment order so that every
// wave-level load of the recurrence is one contiguous 1 KiB piece (the row-major
// matrix would give 16 half-used cache lines per load):
// [layer][wave][item][gate][lane][8], items in the order the wave walks them.
// Run by `nblocks` workgroups of the input projection's first launch; one 16-byte fragment per thread and turn.
template <int DG> __device__ void pack_whh_blocks(const LstmArgs &a, int block, int nblocks)
{
    using G = Geo<DG>;
    constexpr int NW = G::NW, UT = G::UT, THREADS = G::THREADS;
    const bf16_t *W_hh = static_cast<const bf16_t *>(a.W_hh);
    f16x8_t *packed = reinterpret_cast<f16x8_t *>(const_cast<bf16x8_t *>(a.whh_packed));
    const size_t total = (size_t)a.L * NW * G::ITEMS * 4 * 64;
    for (size_t frag = (size_t)block * THREADS + threadIdx.x; frag < total; frag += (size_t)nblocks * THREADS) {
        const int lane = frag % 64;
        size_t r = frag / 64;
        const int q = r % 4; r /= 4;
        const int item = r % G::ITEMS; r /= G::ITEMS;
        const int ut = G::ut_of(item), ks = G::ks_of(item);
        const int wave = r % NW;
        const int l = (int)(r / NW);
        const int n = lane & 15, g4 = lane >> 4;
        const bf16_t *src = W_hh + ((size_t)l * 4 * DG + q * DG + wave * 16 * UT + ut * 16 + n) * DG + ks * 32 + g4 * 8;
        const uint4 v = *reinterpret_cast<const uint4 *>(src);
        const uint32_t w[4] = {v.x, v.y, v.z, v.w};
        const float sc = ldexpf(1.f, whh_scale_exp(whh_layer_max(a.whh_max_bits, l)));
        f16x8_t o;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            o[2 * j] = (f16_t)(__uint_as_float(w[j] << 16) * sc);
            o[2 * j + 1] = (f16_t)(__uint_as_float(w[j] & 0xFFFF0000u) * sc);
        }
        packed[frag] = o;
    }
}

// The re-layout of W_hh (fp16, scaled, fragment order) as a launch of its own: part of the weight preparation, which
// runs once per set of weights (kvev_lstm_prepare) or at the head of a gate call that was handed plain weights.
template <int DG>
__global__ __launch_bounds__(Geo<DG>::THREADS) void lstm_pack_whh_kernel(LstmArgs a)
{
    pack_whh_blocks<DG>(a, (int)blockIdx.x, (int)gridDim.x);
}

template <int DG>
__global__ __launch_bounds__(Geo<DG>::THREADS) void lstm_rec_kernel(LstmArgs a, int t0, int nb)
{
    using G = Geo<DG>;
    using R = Res<DG>;
    constexpr int NW = G::NW, KS = G::KS, UT = G::UT, ITEMS = G::ITEMS, HP = DG + 8;
    constexpr int LRES = R::LRES, RRES = R::RRES, NS = R::NS, NSLOT = R::NSLOT, PF = R::PF, NWL = R::NWL;
    extern __shared__ __align__(16) unsigned char smem_raw[];
    f16_t *s_h = reinterpret_cast<f16_t *>(smem_raw);                                     // [2][2][16][HP]: buffer, (hi, lo)
    float *s_up = reinterpret_cast<float *>(smem_raw + R::lds_h);                         // [2][NW][16]
    unsigned char *s_w = smem_raw + R::lds_h + R::lds_up;                                 // [NW][LRES] items of 4 KiB

    // wave index as a scalar, so that per-wave base addresses live in SGPRs and every
    // fragment load is (scalar base) + (one lane-offset VGPR) + (immediate)
    const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int n = lane & 15, g4 = lane >> 4;
    const int gpl = (a.BH + 15) / 16;
    const int gid = xcd_order(blockIdx.x, gridDim.x);
    const int l = gid / gpl, grp = gid % gpl;
    const bool live = grp * 16 + n < a.BH;
    const size_t s = (size_t)l * a.BH + min(grp * 16 + n, a.BH - 1);

    const bf16_t *w_s = static_cast<const bf16_t *>(a.w_s) + (size_t)l * DG;
    const float b_s = bf16_to_f32(static_cast<const bf16_t *>(a.b_s)[l]);
    const float inv_scale = ldexpf(1.f, -whh_scale_exp(whh_layer_max(a.whh_max_bits, l)));   // undoes the power-of-two scaling of the packed W_hh

    // state of (sequence n, units 16*UT*wave + 16*ut + 4*g4 + r) lives in this lane
    float c_reg[UT][4], h_reg[UT][4], ws_reg[UT][4];
#pragma unroll
    for (int ut = 0; ut < UT; ++ut)
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            const int unit = wave * 16 * UT + ut * 16 + 4 * g4 + r;
            // (chunk 0 starts the recurrence from a zero state, whatever the buffers hold)
            c_reg[ut][r] = live && t0 > 0 ? a.c[s * DG + unit] : 0.f;
            h_reg[ut][r] = live && t0 > 0 ? a.h[s * DG + unit] : 0.f;
            ws_reg[ut][r] = bf16_to_f32(w_s[unit]);
        }

    // this wave's packed A fragments: fragment q of item i of this lane sits at wbase + i*4096 + q*1024 + lane*16
    const unsigned char *wbase = reinterpret_cast<const unsigned char *>(a.whh_packed + ((size_t)l * NW + wave) * ITEMS * 4 * 64);
    const unsigned char *xbase = reinterpret_cast<const unsigned char *>(
        reinterpret_cast<const f32x4_t *>(a.xproj) + xp_block<DG>(gid, a.tb, 0, wave, 0, 0) * 64);
    const uint32_t lane16 = lane * 16;
    const __amdgpu_buffer_rsrc_t w_rsrc = make_rsrc(wbase, ITEMS * 4096);
    const __amdgpu_buffer_rsrc_t x_rsrc = make_rsrc(xbase, (uint32_t)nb * NW * UT * 4096 - (uint32_t)wave * UT * 4096);
    f16_t *h_wr = s_h + (size_t)n * HP + wave * 16 * UT + 4 * g4;           // + (buf*2+p)*16*HP + ut*16
    const f16_t *h_rd = s_h + (size_t)n * HP + g4 * 8;                 // + (buf*2+p)*16*HP + ks*32
    unsigned char *w_lds = s_w + (size_t)wave * LRES * 4096 + lane16;  // + k*4096 + q*1024 for the wave's k-th LDS item

    // h leaves the registers as two fp16 terms (hi + lo = h to 22 bits)
    auto publish_h = [&](int buf, int ut, const float (&hv)[4]) {
        typedef _Float16 f16x4_t __attribute__((ext_vector_type(4)));
        f16x4_t hi, lo;
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            hi[r] = (f16_t)hv[r];
            lo[r] = (f16_t)(hv[r] - (float)hi[r]);
        }
        *reinterpret_cast<f16x4_t *>(h_wr + (size_t)(buf * 2 + 0) * 16 * HP + ut * 16) = hi;
        *reinterpret_cast<f16x4_t *>(h_wr + (size_t)(buf * 2 + 1) * 16 * HP + ut * 16) = lo;
    };

    // ---- resident items: LDS and registers, filled once ------------------------
    static_for<LRES>([&](auto kc) {
        constexpr int k = decltype(kc)::value, i = R::pos(0, k);
#pragma unroll
        for (int q = 0; q < 4; ++q)
            *reinterpret_cast<f16x8_t *>(w_lds + k * 4096 + q * 1024) = buffer_load16<f16x8_t>(w_rsrc, lane16 + q * 1024, i * 4096);
    });
    f16x8_t wres[RRES > 0 ? RRES : 1][4];
    static_for<RRES>([&](auto kc) {
        constexpr int k = decltype(kc)::value, i = R::pos(1, k);
#pragma unroll
        for (int q = 0; q < 4; ++q)
            wres[k][q] = buffer_load16<f16x8_t>(w_rsrc, lane16 + q * 1024, i * 4096);
    });
    // ---- streamed items: the ring runs PF items ahead and wraps into the next step,
    // so the cell update and the barrier overlap with loads already in flight ----
    f16x8_t wbuf[NSLOT][4];
    auto load_w = [&](auto jc) {               // jc: index within the streamed items
        constexpr int j = decltype(jc)::value, i = R::pos(2, j);
#pragma unroll
        for (int q = 0; q < 4; ++q)
            wbuf[j % NSLOT][q] = buffer_load16<f16x8_t>(w_rsrc, lane16 + q * 1024, i * 4096);
    };
    if constexpr (NS > 0) static_for<PF>(load_w);
    // LDS items pass through a register buffer that is read one item ahead
    f16x8_t wl[NWL][4];
    auto read_wl = [&](auto kc) {              // kc: index within the LDS items
        constexpr int k = decltype(kc)::value;
#pragma unroll
        for (int q = 0; q < 4; ++q) wl[k % NWL][q] = *reinterpret_cast<const f16x8_t *>(w_lds + k * 4096 + q * 1024);
    };
    // the two fp16 terms of h for one k-step, read one item ahead
    f16x8_t hb[2][2];
    auto read_h = [&](f16x8_t (&dst)[2], int buf, int ks) {
#pragma unroll
        for (int p = 0; p < 2; ++p)
            dst[p] = *reinterpret_cast<const f16x8_t *>(h_rd + (size_t)(buf * 2 + p) * 16 * HP + ks * 32);
    };

#pragma unroll
    for (int ut = 0; ut < UT; ++ut) publish_h(0, ut, h_reg[ut]);
    __syncthreads();             // h of step t0 - 1 and the LDS items are in place
    if constexpr (R::cls(0) == 0) read_wl(std::integral_constant<int, 0>{});

    for (int tt = 0; tt < nb; ++tt) {
        const int cur = tt & 1, nxt = cur ^ 1;
        float upart = 0.f;
        read_h(hb[0], cur, 0);
        // The step's input projection (read back in the C-fragment layout it was written
        // in) is asked for now and added after the MFMA chain, which hides its latency.
        f32x4_t acc[4], xin[4];
        auto cell_update = [&](auto utc) {
            constexpr int ut = decltype(utc)::value;
            float hv[4];
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                const float ig = sigmoid_hw(fmaf(acc[0][r], inv_scale, xin[0][r]));
                const float fg = sigmoid_hw(fmaf(acc[1][r], inv_scale, xin[1][r]));
                const float gg = tanh_hw(fmaf(acc[2][r], inv_scale, xin[2][r]));
                const float og = sigmoid_hw(fmaf(acc[3][r], inv_scale, xin[3][r]));
                const float cn = fmaf(fg, c_reg[ut][r], ig * gg);
                c_reg[ut][r] = cn;
                float hn = og * tanh_hw(cn);
                asm volatile("" : "+v"(hn));     // opaque to the optimiser: hn is the rounded product from here on
                hv[r] = hn;
                upart = fmaf(ws_reg[ut][r], hn, upart);
            }
            publish_h(nxt, ut, hv);
            if (tt == nb - 1 && live) {          // the state leaves the kernel as fp32
                const int unit = wave * 16 * UT + ut * 16 + 4 * g4;
                *reinterpret_cast<float4 *>(a.h + s * DG + unit) = make_float4(hv[0], hv[1], hv[2], hv[3]);
            }
        };
        static_for<ITEMS>([&](auto ic) {
            constexpr int i = decltype(ic)::value, ut = G::ut_of(i), ks = G::ks_of(i);
            constexpr int c = R::cls(i), k = R::idx(i);
            if constexpr (ks == 0) {
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    xin[q] = buffer_load16_nt<f32x4_t>(x_rsrc, lane16 + q * 1024, (uint32_t)(tt * NW * UT + ut) * 4096);
                    acc[q] = f32x4_t{0.f, 0.f, 0.f, 0.f};
                }
            }
            // operands of what comes next are asked for before this item's MFMAs
            if constexpr (i + 1 < ITEMS) read_h(hb[(i + 1) & 1], cur, G::ks_of(i + 1));
            if constexpr (R::cls((i + 1) % ITEMS) == 0) read_wl(std::integral_constant<int, R::idx((i + 1) % ITEMS)>{});
            if constexpr (c == 2) load_w(std::integral_constant<int, (k + PF) % NS>{});
            auto chain = [&](const f16x8_t (&wf)[4]) {
#pragma unroll
                for (int p = 1; p >= 0; --p)          // the small term first
#pragma unroll
                    for (int q = 0; q < 4; ++q)
                        acc[q] = __builtin_amdgcn_mfma_f32_16x16x32_f16(wf[q], hb[i & 1][p], acc[q], 0, 0, 0);
            };
            if constexpr (c == 0) chain(wl[k % NWL]);
            else if constexpr (c == 1) chain(wres[k]);
            else chain(wbuf[k % NSLOT]);
            // the prefetch depths are the ones written here, not whatever the scheduler can hoist
            __builtin_amdgcn_sched_barrier(0);
            if constexpr (ks == KS - 1) cell_update(std::integral_constant<int, ut>{});
        });
        upart += __shfl_xor(upart, 16);
        upart += __shfl_xor(upart, 32);
        if (g4 == 0) s_up[(cur * NW + wave) * 16 + n] = upart;
        __syncthreads();
        if (tid < 16) {
            float u = 0.f;
#pragma unroll
            for (int w = 0; w < NW; ++w) u += s_up[(cur * NW + w) * 16 + tid];
            u += b_s;
            if (live) {
                a.util[s * a.N_cap + t0 + tt] = u;
                a.gate[s * a.N_cap + t0 + tt] = sigmoid_hw(u);
            }
        }
    }

    if (live) {
#pragma unroll
        for (int ut = 0; ut < UT; ++ut)
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                const int unit = wave * 16 * UT + ut * 16 + 4 * g4 + r;
                a.c[s * DG + unit] = c_reg[ut][r];
            }
    }
}

// ---- the recurrence of a 16-sequence group on a pair of compute units ----------------------------------------
// With few sequences (config 2: 32) the chip is empty and the step time of the kernel above is what one CU can do:
// at d_g = 256, 1.7 us of MFMA and a weight stream out of L2 on top; at d_g = 512
// 13.7 us for the 2 MiB of W_hh that a CU pulls out of L2 every step.  Here two workgroups share a group: each owns
// half of the hidden units (8 waves x 16 or 32 units, all four gates), so a step is half the matrix work, half the
// gate nonlinearities and half the weight bytes per CU; at d_g = 256 its half of W_hh (256 KiB as fp16) sits in
// registers for the whole launch.  What the halves owe each other every step is the new h of the other half,
// 16 x d_g/2 values as (hi, lo) fp16 terms.
//
// Exchange: a wave publishes each of its unit tiles (16 units x 16 sequences) as two 16-byte stores per lane of the
// form {payload, stamp, payload, stamp} (stamp = step + 1 within the launch) with device scope, into a slot of its own;
// the same wave of the partner polls that slot until all stamps of its loads carry the step it waits for.
// Data and stamp share an aligned 8-byte word, which a store writes and a load reads as one, so no flag, fence or
// ordering between different addresses is involved.  Two slots by step parity: a slot is rewritten two steps
// later, which the writer can only reach after the partner has consumed it (it needs the partner's next h, published
// after that read).  The input projection's launch clears the slots before every launch of this kernel, so a stamp
// can only come from the current one.
//
// The products over the workgroup's own half of h do not need the exchange and run while it is in flight:
//   own-half MFMAs | take partner's h, stage in LDS | barrier | partner-half MFMAs | cell, publish | barrier.
// The utility logit w_s . h_t + b_s is completed one step later, when the partner's half has arrived (as hi + lo,
// 22 bits); one wave of member 0 writes it while it would otherwise wait at the step's last barrier.
// Measured at config 2 (32 sequences, 4 workgroups): 2.1 us per step against 3.1 us for one workgroup per group;
// the exchange is mostly hidden (the first look finds the data 60-90 % of the time), and what is left is a SIMD's
// own serial work: 0.87 us of MFMA and 0.7 us of gate nonlinearities (quarter-rate exp2 and rcp) for its two
// waves, plus two barriers and the LDS latency in front of each run of MFMAs.  At d_g = 512 with 256 workgroups: 13 us
// per step against 20 us (launches with more than 16 sequences per layer go to four workgroups per 32 sequences instead:
// lstm_quad.hip).
//
// Every wait is bounded: a wave that does not see its partner's data within a.pair_spin_limit polls raises a flag in
// LDS, the workgroup leaves the step loop together after the next barrier, marks the launch's scores as NaN and sets
// the status word at the head of the caller's scratch (it stays set until the caller clears it).
// Members of a pair are neighbours in the launch order; workgroups are started in that order here, so a launch that
// does not fit the chip at once still completes pair by pair (the bound covers any other case).  The host takes this
// kernel only while the launch has at most one workgroup per compute unit of the device.
// Geometry of the paired kernel: 8 waves, each with UT unit tiles of the workgroup's half of the hidden units; a
// weight item is the 4 gate fragments of one tile at one k-step (4 KiB per wave), walked k-step by k-step (the B
// operand of a k-step serves all tiles), own half of the k range first.  d_g = 256 keeps all 8 items of a wave in
// registers; d_g = 512 (32 items, 128 KiB per wave) keeps RRES of them and streams the rest out of L2 through a ring
// of NSLOT register buffers that runs PF items ahead, across the halves of a step and into the next step.
template <int DG> struct PairGeo {
    static constexpr int NW = 8, UT = DG / 256, KS = DG / 32, KH = KS / 2, ITEMS = UT * KS, HP = DG + 8;
    static constexpr int RRES = DG == 256 ? ITEMS : 2, NS = ITEMS - RRES;
    static constexpr int NSLOT = NS == 0 ? 1 : 5, PF = NSLOT - 1;   // (3 or 6 slots measured within 4 % of 5: the stream is not what the step waits for)
    static_assert(NS % NSLOT == 0, "slot rotation must line up with the item loop");
    // item p of the walk: half (0 own, 1 partner's), k-step within the half, unit tile
    static constexpr int half_of(int p) { return p / (UT * KH); }
    static constexpr int j_of(int p) { return (p % (UT * KH)) / UT; }
    static constexpr int ut_of(int p) { return p % UT; }
    static constexpr uint32_t slot_bytes = UT * 2 * 64 * 16;                 // one wave's publication: UT tiles x (hi, lo) lines of 1 KiB
    static constexpr uint32_t exch_bytes = 2 * 2 * NW * slot_bytes;          // [parity][member][wave] per sequence group
    static constexpr size_t lds_h = (size_t)2 * 2 * 16 * HP * sizeof(f16_t); // [buffer][hi, lo][sequence][unit]
    static constexpr size_t lds_up = (size_t)3 * NW * 64 * sizeof(float);    // shares of the utility logit: own (2 parities), partner's
    static constexpr size_t lds = lds_h + lds_up + 16;
};

template <int DG>
__global__ __launch_bounds__(512) void lstm_rec_pair_kernel(LstmArgs a, int t0, int nb)
{
    using G = Geo<DG>;                     // the packed operands keep the single-workgroup kernel's geometry
    using P = PairGeo<DG>;
    constexpr int NW = P::NW, UT = P::UT, KS = P::KS, KH = P::KH, HP = P::HP;
    constexpr int RRES = P::RRES, NS = P::NS, NSLOT = P::NSLOT, PF = P::PF;
    typedef _Float16 f16x4_t __attribute__((ext_vector_type(4)));
    extern __shared__ __align__(16) unsigned char smem_pair[];
    f16_t *s_h = reinterpret_cast<f16_t *>(smem_pair);
    float (*s_up)[NW][64] = reinterpret_cast<float (*)[NW][64]>(smem_pair + P::lds_h);           // [2]
    float (*s_up2)[64] = reinterpret_cast<float (*)[64]>(smem_pair + P::lds_h + 2 * NW * 64 * sizeof(float));
    int &s_fail = *reinterpret_cast<int *>(smem_pair + P::lds_h + P::lds_up);

    const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int n = lane & 15, g4 = lane >> 4;
    // The members of a pair are neighbours in the launch order.  Workgroups are started in that order, so whatever
    // else holds compute units, a member that is running finds its partner next in line for the first unit that
    // frees up: a launch that does not fit the chip at once still completes pair by pair.  (Neighbouring ids sit
    // on different XCDs, so the exchange always takes the write-through path below; at d_g = 512 this also means
    // that an XCD's L2 serves one half of W_hh only.)
    const int member = blockIdx.x & 1, gid = blockIdx.x >> 1;
    const int gpl = (a.BH + 15) / 16;
    if (gid >= a.L * gpl) return;
    const int l = gid / gpl, grp = gid % gpl;
    const bool live = grp * 16 + n < a.BH;
    const size_t s = (size_t)l * a.BH + min(grp * 16 + n, a.BH - 1);
    // unit tiles (16 units each) of this wave and of its partner wave: tile0 + ut, ptile0 + ut
    const int tile0 = (member * NW + wave) * UT, ptile0 = ((1 - member) * NW + wave) * UT;
    const int ks_own = member * KH, ks_par = (1 - member) * KH;

    const bf16_t *w_s = static_cast<const bf16_t *>(a.w_s) + (size_t)l * DG;
    const float b_s = bf16_to_f32(static_cast<const bf16_t *>(a.b_s)[l]);
    const float inv_scale = ldexpf(1.f, -whh_scale_exp(whh_layer_max(a.whh_max_bits, l)));
    if (tid == 0) s_fail = 0;

    const uint32_t lane16 = lane * 16;
    // the wave's weights: item (ut, ks) at wbase + (ut*KS + ks) * 4096 (its tiles are neighbours in the packed order)
    const unsigned char *wbase = reinterpret_cast<const unsigned char *>(
        a.whh_packed + (((size_t)l * G::NW + tile0 / G::UT) * G::ITEMS + (tile0 % G::UT) * KS) * 4 * 64);
    const __amdgpu_buffer_rsrc_t w_rsrc = make_rsrc(wbase, UT * KS * 4096);
    auto item_off = [&](int p) { return (uint32_t)((P::ut_of(p) * KS + (P::half_of(p) == 0 ? ks_own : ks_par) + P::j_of(p)) * 4096); };
    f16x8_t wres[RRES][4];
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
    if constexpr (NS > 0) static_for<PF>(load_w);

    const unsigned char *xbase = reinterpret_cast<const unsigned char *>(
        reinterpret_cast<const f32x4_t *>(a.xproj) + xp_block<DG>(gid, a.tb, 0, tile0 / G::UT, tile0 % G::UT, 0) * 64);
    const __amdgpu_buffer_rsrc_t x_rsrc = make_rsrc(xbase, (uint32_t)nb * G::NW * G::UT * 4096 - (uint32_t)tile0 * 4096);
    const __amdgpu_buffer_rsrc_t e_rsrc = make_rsrc(a.exch + (size_t)gid * P::exch_bytes, P::exch_bytes);

    float c_reg[UT][4], ws_own[UT][4], ws_par[UT][4];
    f16_t *h_own = s_h + (size_t)n * HP + tile0 * 16 + 4 * g4;       // + (buf*2 + plane)*16*HP + ut*16
    f16_t *h_par = s_h + (size_t)n * HP + ptile0 * 16 + 4 * g4;
    const f16_t *h_rd = s_h + (size_t)n * HP + g4 * 8;               // + (buf*2 + plane)*16*HP + ks*32
    auto split = [](const float (&hv)[4], f16x4_t &hi, f16x4_t &lo) {
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            hi[r] = (f16_t)hv[r];
            lo[r] = (f16_t)(hv[r] - (float)hi[r]);
        }
    };
#pragma unroll
    for (int ut = 0; ut < UT; ++ut) {   // h of step t0 - 1, both halves, from the fp32 state
        float ho[4], hp[4];
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            const int uo = (tile0 + ut) * 16 + 4 * g4 + r, up = (ptile0 + ut) * 16 + 4 * g4 + r;
            // (chunk 0 starts the recurrence from a zero state, whatever the buffers hold)
            c_reg[ut][r] = live && t0 > 0 ? a.c[s * DG + uo] : 0.f;
            ho[r] = live && t0 > 0 ? a.h[s * DG + uo] : 0.f;
            hp[r] = live && t0 > 0 ? a.h[s * DG + up] : 0.f;
            ws_own[ut][r] = bf16_to_f32(w_s[uo]);
            ws_par[ut][r] = bf16_to_f32(w_s[up]);
        }
        f16x4_t hi, lo;
        split(ho, hi, lo);
        *reinterpret_cast<f16x4_t *>(h_own + ut * 16) = hi;
        *reinterpret_cast<f16x4_t *>(h_own + 16 * HP + ut * 16) = lo;
        split(hp, hi, lo);
        *reinterpret_cast<f16x4_t *>(h_par + ut * 16) = hi;
        *reinterpret_cast<f16x4_t *>(h_par + 16 * HP + ut * 16) = lo;
    }
    __syncthreads();

    // one look at the partner wave's slot `par` (device-scope loads; their results are examined later)
    struct Look { u32x4_t v[UT][2]; };
    auto ask = [&](int par, Look &k) __attribute__((always_inline)) {
        const uint32_t off = (uint32_t)((par * 2 + (1 - member)) * NW + wave) * P::slot_bytes;
#pragma unroll
        for (int ut = 0; ut < UT; ++ut)
#pragma unroll
            for (int pl = 0; pl < 2; ++pl)
                k.v[ut][pl] = __builtin_amdgcn_raw_buffer_load_b128(e_rsrc, (int)lane16, (int)(off + (ut * 2 + pl) * 1024), 16);
    };
    // The partner wave's h of the step stamped `stamp`, from slot `par`: staged in LDS buffer `buf`, and its share of
    // the utility logit left in s_up2.  (ka, k: looks at the slot asked for earlier, so that their round trips,
    // about 1 us behind the stores of the publication, run behind the own-half MFMAs; more looks follow if neither
    // carries the stamp yet.)
    auto receive = [&](int par, uint32_t stamp, int buf, const Look &ka, Look &k) __attribute__((always_inline)) {
        auto all_in = [&](const Look &x) __attribute__((always_inline)) {
            bool ok = true;
#pragma unroll
            for (int ut = 0; ut < UT; ++ut)
#pragma unroll
                for (int pl = 0; pl < 2; ++pl) ok = ok && x.v[ut][pl][1] == stamp && x.v[ut][pl][3] == stamp;
            return __all(ok) != 0;
        };
        auto stage = [&](const Look &x) __attribute__((always_inline)) {
            float up = 0.f;
#pragma unroll
            for (int ut = 0; ut < UT; ++ut) {
                const uint2 hi2 = make_uint2(x.v[ut][0][0], x.v[ut][0][2]), lo2 = make_uint2(x.v[ut][1][0], x.v[ut][1][2]);
                const f16x4_t hi = __builtin_bit_cast(f16x4_t, hi2), lo = __builtin_bit_cast(f16x4_t, lo2);
                *reinterpret_cast<f16x4_t *>(h_par + (size_t)(buf * 2 + 0) * 16 * HP + ut * 16) = hi;
                *reinterpret_cast<f16x4_t *>(h_par + (size_t)(buf * 2 + 1) * 16 * HP + ut * 16) = lo;
#pragma unroll
                for (int r = 0; r < 4; ++r) up = fmaf(ws_par[ut][r], (float)hi[r] + (float)lo[r], up);
            }
            s_up2[wave][lane] = up;
        };
        if (all_in(ka)) {
            stage(ka);
            return;
        }
        bool got = false;
        for (int spin = 0; spin < a.pair_spin_limit; ++spin) {
            asm volatile("" ::: "memory");
            if (all_in(k)) { got = true; break; }
            if ((spin & 255) == 255 && s_fail) break;
            ask(par, k);
        }
        if (!got) s_fail = 1;
        stage(k);
    };
    // Member 0 completes the logit of a step once both halves are in: own shares (buffer `ub`), then the partner's.
    // One wave does it, at a point where it would otherwise wait at the barrier for the slower ones.
    auto write_util = [&](int ub, int step) __attribute__((always_inline)) {
        if (member == 0 && wave == 0) {
            float u = 0.f;
#pragma unroll
            for (int w = 0; w < NW; ++w) u += s_up[ub][w][lane];
#pragma unroll
            for (int w = 0; w < NW; ++w) u += s_up2[w][lane];
            u += __shfl_xor(u, 16);
            u += __shfl_xor(u, 32);
            u += b_s;
            if (live && g4 == 0) {
                a.util[s * a.N_cap + t0 + step] = u;
                a.gate[s * a.N_cap + t0 + step] = sigmoid_hw(u);
            }
        }
    };
    // the two fp16 terms of h for one k-step
    auto read_h = [&](f16x8_t (&dst)[2], int buf, int ks) __attribute__((always_inline)) {
#pragma unroll
        for (int pl = 0; pl < 2; ++pl)
            dst[pl] = *reinterpret_cast<const f16x8_t *>(h_rd + (size_t)(buf * 2 + pl) * 16 * HP + ks * 32);
    };
    using std::integral_constant;

    bool failed = false;
    Look ka;
#pragma unroll
    for (int ut = 0; ut < UT; ++ut) ka.v[ut][0] = ka.v[ut][1] = u32x4_t{0, 0, 0, 0};
    for (int tt = 0; tt < nb; ++tt) {
        const int cur = tt & 1, nxt = cur ^ 1;
        f32x4_t acc[UT][4], xin[UT][4];
#pragma unroll
        for (int ut = 0; ut < UT; ++ut)
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                if (UT == 1) xin[ut][q] = buffer_load16_nt<f32x4_t>(x_rsrc, lane16 + q * 1024, (uint32_t)(tt * G::NW * G::UT + ut) * 4096);
                acc[ut][q] = f32x4_t{0.f, 0.f, 0.f, 0.f};
            }
        // the partner published h of step tt - 1 at the end of that step (slot nxt, stamp tt); a first look at the slot
        // went out right after this workgroup's own publication, a second one goes now (one tile per wave only:
        // with two, the own half is long enough for the first)
        Look kb;
        if constexpr (UT == 1) {
            if (tt > 0) ask(nxt, kb);
        }
        __builtin_amdgcn_sched_barrier(0);

        // one half of the step's products: items [half * UT*KH, (half + 1) * UT*KH) of the walk
        auto run_half = [&](auto halfc) __attribute__((always_inline)) {
            constexpr int half = decltype(halfc)::value, p0 = half * UT * KH;
            const int ks0 = half == 0 ? ks_own : ks_par;
            // B operands: all k-steps of the half at once where the registers allow it, else one k-step ahead
            constexpr int NHB = UT == 1 ? KH : 2;
            f16x8_t hb[NHB][2];
            if constexpr (UT == 1) {
#pragma unroll
                for (int j = 0; j < KH; ++j) read_h(hb[j], cur, ks0 + j);
            } else {
                read_h(hb[0], cur, ks0);
            }
            static_for<UT * KH>([&](auto ic) {
                constexpr int p = p0 + decltype(ic)::value, j = P::j_of(p), ut = P::ut_of(p);
                if constexpr (UT > 1 && ut == 0 && j + 1 < KH) read_h(hb[(j + 1) % NHB], cur, ks0 + j + 1);
                if constexpr (p >= RRES) load_w(integral_constant<int, (p - RRES + PF) % (NS > 0 ? NS : 1)>{});
                if constexpr (UT > 1 && half == 1 && j == KH - 2 && ut == 0) {
                    // the input projections of this step, asked for one k-step before they are used
#pragma unroll
                    for (int u2 = 0; u2 < UT; ++u2)
#pragma unroll
                        for (int q = 0; q < 4; ++q)
                            xin[u2][q] = buffer_load16_nt<f32x4_t>(x_rsrc, lane16 + q * 1024, (uint32_t)(tt * G::NW * G::UT + u2) * 4096);
                }
                auto chain = [&](const f16x8_t (&wf)[4]) __attribute__((always_inline)) {
#pragma unroll
                    for (int pl = 1; pl >= 0; --pl)          // the small term first
#pragma unroll
                        for (int q = 0; q < 4; ++q)
                            acc[ut][q] = __builtin_amdgcn_mfma_f32_16x16x32_f16(wf[q], hb[j % NHB][pl], acc[ut][q], 0, 0, 0);
                };
                if constexpr (p < RRES) chain(wres[p]);
                else chain(wbuf[(p - RRES) % NSLOT]);
                if constexpr (NS > 0) __builtin_amdgcn_sched_barrier(0);      // the ring's depth is the one written here
            });
        };
        run_half(integral_constant<int, 0>{});
        if (tt > 0) {
            if constexpr (UT == 1) receive(nxt, (uint32_t)tt, cur, ka, kb);
            else receive(nxt, (uint32_t)tt, cur, ka, ka);         // (further looks may overwrite the first)
            lds_barrier();
            if (s_fail) { failed = true; break; }
        }
        run_half(integral_constant<int, 1>{});

        float upart = 0.f;
        f16x4_t hi[UT], lo[UT];
        float hv[UT][4];
#pragma unroll
        for (int ut = 0; ut < UT; ++ut) {
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                const float ig = sigmoid_hw(fmaf(acc[ut][0][r], inv_scale, xin[ut][0][r]));
                const float fg = sigmoid_hw(fmaf(acc[ut][1][r], inv_scale, xin[ut][1][r]));
                const float gg = tanh_hw(fmaf(acc[ut][2][r], inv_scale, xin[ut][2][r]));
                const float og = sigmoid_hw(fmaf(acc[ut][3][r], inv_scale, xin[ut][3][r]));
                const float cn = fmaf(fg, c_reg[ut][r], ig * gg);
                c_reg[ut][r] = cn;
                float hn = og * tanh_hw(cn);
                asm volatile("" : "+v"(hn));
                hv[ut][r] = hn;
                upart = fmaf(ws_own[ut][r], hn, upart);
            }
            split(hv[ut], hi[ut], lo[ut]);
            // to the partner first (the long way), then to this workgroup's own waves
            const uint2 hi2 = __builtin_bit_cast(uint2, hi[ut]), lo2 = __builtin_bit_cast(uint2, lo[ut]);
            const uint32_t stamp = (uint32_t)tt + 1;
            const uint32_t off = (uint32_t)((cur * 2 + member) * NW + wave) * P::slot_bytes + ut * 2048;
            const u32x4_t l0 = {hi2.x, stamp, hi2.y, stamp}, l1 = {lo2.x, stamp, lo2.y, stamp};
            if (member != a.pair_mute) {       // device scope: the stores write through to where the partner's loads look
                __builtin_amdgcn_raw_buffer_store_b128(l0, e_rsrc, (int)lane16, (int)off, 16);
                __builtin_amdgcn_raw_buffer_store_b128(l1, e_rsrc, (int)lane16, (int)(off + 1024), 16);
            }
        }
        ask(cur, ka);                // the partner is about to publish the same step
#pragma unroll
        for (int ut = 0; ut < UT; ++ut) {
            *reinterpret_cast<f16x4_t *>(h_own + (size_t)(nxt * 2 + 0) * 16 * HP + ut * 16) = hi[ut];
            *reinterpret_cast<f16x4_t *>(h_own + (size_t)(nxt * 2 + 1) * 16 * HP + ut * 16) = lo[ut];
            if (tt == nb - 1 && live)
                *reinterpret_cast<float4 *>(a.h + s * DG + (tile0 + ut) * 16 + 4 * g4) = make_float4(hv[ut][0], hv[ut][1], hv[ut][2], hv[ut][3]);
        }
        s_up[cur][wave][lane] = upart;
        if (tt > 0) write_util(nxt, tt - 1);       // both halves of step tt - 1 have been in LDS since this step's first barrier
        lds_barrier();
    }
    if (!failed) {      // the last step's logit needs the partner's last h
        Look k;
        ask((nb - 1) & 1, k);
        receive((nb - 1) & 1, (uint32_t)nb, nb & 1, ka, k);
        lds_barrier();
        failed = s_fail != 0;
        if (!failed) write_util((nb - 1) & 1, nb - 1);
    }
    if (live) {
#pragma unroll
        for (int ut = 0; ut < UT; ++ut)
#pragma unroll
            for (int r = 0; r < 4; ++r) a.c[s * DG + (tile0 + ut) * 16 + 4 * g4 + r] = failed ? __builtin_nanf("") : c_reg[ut][r];
    }
    if (failed && tid == 0) __hip_atomic_store(a.status, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);   // sticky: the caller's to clear
    if (failed && tid < 16 && live) {
        for (int t = 0; t < nb; ++t) {
            a.util[s * a.N_cap + t0 + t] = __builtin_nanf("");
            a.gate[s * a.N_cap + t0 + t] = __builtin_nanf("");
        }
    }
}

// One-time launch attributes (LDS beyond 64 KiB), per kernel instance and device: a bit per device id.
template <int DG>
static hipError_t set_attributes_once()
{
    static std::atomic<uint64_t> done{0};
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    const uint64_t bit = (uint64_t)1 << (dev & 63);
    if (done.load(std::memory_order_acquire) & bit) return hipSuccess;
    e = hipFuncSetAttribute(reinterpret_cast<const void *>(lstm_rec_kernel<DG>), hipFuncAttributeMaxDynamicSharedMemorySize,
                            (int)Res<DG>::lds);
    if (e != hipSuccess) return e;
    // (the in-projection's staged rows pass 64 KiB at d = 128)
    e = hipFuncSetAttribute(reinterpret_cast<const void *>(lstm_inproj_kernel<DG, 128, kTT>),
                            hipFuncAttributeMaxDynamicSharedMemorySize, (int)(kTT * 16 * (2 * 128 + 8) * sizeof(bf16_t)));
    if (e != hipSuccess) return e;
    if constexpr (DG == 256 || DG == 512) {
        static_assert(PairGeo<DG>::exch_bytes == (DG / 256) * kLstmPairExchBytes256, "the scratch planner's figure");
        e = hipFuncSetAttribute(reinterpret_cast<const void *>(lstm_rec_pair_kernel<DG>),
                                hipFuncAttributeMaxDynamicSharedMemorySize, (int)PairGeo<DG>::lds);
        if (e != hipSuccess) return e;
    }
    done.fetch_or(bit, std::memory_order_release);
    return hipSuccess;
}

// Weight preparation: W_ih into fragment order and the partial maxima of |W_hh| (one launch), then W_hh scaled,
// converted and re-laid (a second one, which needs the maxima).  What it leaves depends on the weights alone.
template <int DG>
static hipError_t prepare_dg(const LstmArgs &a, hipStream_t st)
{
    const size_t frags_i = (size_t)a.L * 4 * DG * 2 * a.d / 8;
    const int nb_wih = (int)((frags_i + 255) / 256);
    const dim3 grid_p((unsigned)(nb_wih + a.L * kScaleBlocks));
    if (a.d == 64)
        hipLaunchKernelGGL((lstm_prep_kernel<DG, 64>), grid_p, dim3(256), 0, st, static_cast<const bf16_t *>(a.W_ih),
                           const_cast<bf16x8_t *>(a.wih_packed), static_cast<const bf16_t *>(a.W_hh), a.whh_max_bits, a.L, nb_wih);
    else
        hipLaunchKernelGGL((lstm_prep_kernel<DG, 128>), grid_p, dim3(256), 0, st, static_cast<const bf16_t *>(a.W_ih),
                           const_cast<bf16x8_t *>(a.wih_packed), static_cast<const bf16_t *>(a.W_hh), a.whh_max_bits, a.L, nb_wih);
    // W_hh fragments: 16 bytes per thread and turn, about 4 turns per packing workgroup
    const size_t frags_h = (size_t)a.L * 4 * DG * DG / 8;
    const size_t want = (frags_h + (size_t)4 * Geo<DG>::THREADS - 1) / ((size_t)4 * Geo<DG>::THREADS);
    hipLaunchKernelGGL((lstm_pack_whh_kernel<DG>), dim3((unsigned)(want > 4096 ? 4096 : want)), dim3(Geo<DG>::THREADS), 0, st, a);
    return hipGetLastError();
}

template <int DG>
static hipError_t launch_dg(const LstmArgs &a, hipStream_t st)
{
    const int gpl = (a.BH + 15) / 16;
    const unsigned groups = (unsigned)(a.L * gpl);
    const size_t lds = Res<DG>::lds;
    hipError_t e = set_attributes_once<DG>();
    if (e != hipSuccess) return e;
    if (!a.prepared) {
        e = prepare_dg<DG>(a, st);
        if (e != hipSuccess) return e;
    }
    if constexpr (DG == 256) {
        if (a.fused) return launch_lstm_fused(a, st);
    }
    if constexpr (DG == 512) {
        if (a.split == 4) return launch_lstm_quad(a, st);
    }
    for (int t0 = a.c0; t0 < a.c1; t0 += a.tb) {
        const int nb = a.c1 - t0 < a.tb ? a.c1 - t0 : a.tb;
        // few sequences: shorter runs of steps per workgroup so that the launch still covers the chip
        const bool small = (size_t)groups * ((nb + kTT - 1) / kTT) < 256;
        const int tt = small ? 2 : kTT;
        const int ny_proj = (nb + tt - 1) / tt;
        const dim3 grid_in(groups, (unsigned)ny_proj);
        const size_t lds_in = (size_t)tt * 16 * (2 * a.d + 8) * sizeof(bf16_t);
        if (a.d == 64) {
            if (small) hipLaunchKernelGGL((lstm_inproj_kernel<DG, 64, 2>), grid_in, dim3(Geo<DG>::THREADS), lds_in, st, a, t0, nb);
            else hipLaunchKernelGGL((lstm_inproj_kernel<DG, 64, kTT>), grid_in, dim3(Geo<DG>::THREADS), lds_in, st, a, t0, nb);
        } else {
            if (small) hipLaunchKernelGGL((lstm_inproj_kernel<DG, 128, 2>), grid_in, dim3(Geo<DG>::THREADS), lds_in, st, a, t0, nb);
            else hipLaunchKernelGGL((lstm_inproj_kernel<DG, 128, kTT>), grid_in, dim3(Geo<DG>::THREADS), lds_in, st, a, t0, nb);
        }
        if constexpr (DG == 256 || DG == 512) {
            if (a.split == 2) {
                hipLaunchKernelGGL((lstm_rec_pair_kernel<DG>), dim3(2 * groups), dim3(512), PairGeo<DG>::lds, st, a, t0, nb);
                continue;
            }
        }
        hipLaunchKernelGGL((lstm_rec_kernel<DG>), dim3(groups), dim3(Geo<DG>::THREADS), lds, st, a, t0, nb);
    }
    return hipGetLastError();
}

hipError_t launch_lstm_mfma(const LstmArgs &a, hipStream_t st)
{
    switch (a.d_g) {
    case 64: return launch_dg<64>(a, st);
    case 128: return launch_dg<128>(a, st);
    case 256: return launch_dg<256>(a, st);
    case 512: return launch_dg<512>(a, st);
    default: return hipErrorInvalidValue;
    }
}

hipError_t launch_lstm_prepare(const LstmArgs &a, hipStream_t st)
{
    switch (a.d_g) {
    case 64: return prepare_dg<64>(a, st);
    case 128: return prepare_dg<128>(a, st);
    case 256: return prepare_dg<256>(a, st);
    case 512: return prepare_dg<512>(a, st);
    default: return hipErrorInvalidValue;
    }
}

}  // namespace kvev

// Chunk aggregation, Eq. 2 of the paper, bf16 storage.
//
// The op reads every raw key and value once (2*C*d elements per chunk) and
// writes one summary pair: about 8 flop per byte, far below the machine's
// ridge, so the kernel is a streaming reader with the MLP as a side dish.  A
// workgroup owns a tile of 16 (sequence, chunk) rows of one layer:
//   1. each wave streams 4 of the rows: a 16-lane group owns a token at a time
//      (one 16-byte load per lane, 1 KiB contiguous per wave-level load), sums
//      in fp32, and the chunk means land in LDS as fp32;
//   2. layer 1 and 3. layer 2 run on v_mfma_f32_16x16x32_bf16 with the weight
//      rows as the A operand (read from global memory; the four weight
//      matrices total 128 KiB and stay in cache) and the 16 tile rows as B.
// The fp32 means and activations are fed to the bf16 matrix cores as three
// bf16 terms each (x = hi + mid + lo, exact to 24 bits; cut once, when the value
// is written to LDS, into three bf16 planes): weights are bf16, so
// every partial product is exact and the fp32 accumulation gives fp32-grade
// results, which is what keeps the stored summaries equal to a double
// precision evaluation except for rare last-bit flips.
#include "common.hpp"
#include "kernels.hpp"
#include <algorithm>
#include <atomic>
#include <type_traits>

namespace kvev {

// two fp32 -> three packed bf16 pairs whose sums are the inputs (to 24 bits)
__device__ __forceinline__ void split3_pair(float x0, float x1, uint32_t &hi, uint32_t &mid, uint32_t &lo)
{
    hi = pack_bf16x2(x0, x1);
    const float r0 = x0 - __uint_as_float(hi << 16), r1 = x1 - __uint_as_float(hi & 0xFFFF0000u);
    mid = pack_bf16x2(r0, r1);
    lo = pack_bf16x2(r0 - __uint_as_float(mid << 16), r1 - __uint_as_float(mid & 0xFFFF0000u));
}

// NW waves per workgroup: 4 when the launch fills the chip several times over, 16 (one tile row per wave) when
// there are few tiles, so that a compute unit still has enough loads in flight.
//
// The NW = 4 form is persistent (a workgroup walks tiles blockIdx.x, blockIdx.x + gridDim.x, ...) and does not write a
// tile's summaries when they are ready: a thread keeps its 16-byte pieces of up to NS tiles in registers, and every
// wave writes what it holds when the chip-wide real-time counter enters a new slot of 2^flush_shift ticks (100 MHz),
// i.e. all waves of the chip within a few microseconds of each other.  Summaries are 3 % of the bytes the kernel
// moves, but trickling out between the reads they cost a streaming kernel a fifth of its read rate on this chip (a
// plain reader: 7.3 TB/s alone, 5.7 TB/s with 3 % written back tile by tile, 6.6 TB/s with the same bytes written in
// such synchronised bursts): the memory controllers turn the bus around for a handful of writes at a time unless the
// writes arrive together.
//
// PK: the MLP weights come from a.wpack, re-laid by pool_pack_kernel so that a wave-level load of a weight fragment is
// 1 KiB of consecutive bytes.  As the caller gives them (row-major) such a load touches 16 rows, half a cache line of
// each; a tile asks L2 for 128 KiB of weights next to its 256 KiB of raw rows, and at scale those requests cost the
// kernel 3 % (the loads themselves 7 %: measured with the weights read from one cached fragment).
template <int D, int NW, bool PK>
__global__ __launch_bounds__(64 * NW, NW == 4 ? 3 : 1) void pool_mfma_kernel(PoolArgs a)
{
    constexpr int RPW = 16 / NW;         // tile rows per wave
    constexpr int EPL = D / 16;          // elements per lane of a 16-lane row group
    constexpr int XP = D + 8;            // padded bf16 row of a mean plane
    constexpr int PIECES = 2 * 16 * (D / 8);                 // 16-byte pieces of a tile's output
    constexpr bool STAGED = NW == 4;
    constexpr int PPT = STAGED ? PIECES / (64 * NW) : 1;     // pieces per thread and tile
    constexpr int NS = 2;                                    // tiles a thread can hold back
    extern __shared__ __align__(16) bf16_t smem[];
    bf16_t *xm = smem;                   // [3 terms][2 (K,V)][16 rows][XP]   chunk means
    const int AP = a.d_sum + 8;
    bf16_t *act = smem + 3 * 2 * 16 * XP;   // [3][2][16][AP]   hidden activations

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int n = lane & 15, g4 = lane >> 4;
    const int nch = a.c1 - a.c0;
    const int rows_per_layer = a.BH * nch;
    const int tiles_per_layer = (rows_per_layer + 15) / 16;
    const int ntiles = a.L * tiles_per_layer;

    const bf16_t *K = static_cast<const bf16_t *>(a.K), *V = static_cast<const bf16_t *>(a.V);
    bf16_t *Kb = static_cast<bf16_t *>(a.Kbar), *Vb = static_cast<bf16_t *>(a.Vbar);
    const bool is_max = a.mode == KVEV_POOL_MAX;

    // Summaries leave as whole 256-byte rows, 16 bytes per lane (a wave-level store is 1 KiB of consecutive chunks of
    // one sequence): 8-byte pieces straight out of the MFMA layout would touch every line four times.  Launches that
    // fill the chip many times over (NW = 4) stream, so their stores carry the non-temporal hint like their loads.
    // output row of piece i of a tile (-1: past the end), and the store of one piece into such a row
    auto out_row = [&](int tile, int i) __attribute__((always_inline)) {
        const int rt = (i / (D / 8)) % 16;
        const int l = tile / tiles_per_layer;
        const int r = (tile % tiles_per_layer) * 16 + rt;
        return r < rows_per_layer ? (int)((l * a.BH + r / nch) * a.N_cap + (a.c0 + r % nch)) : -1;
    };
    auto store_piece = [&](int row, int i, u32x4_t w) __attribute__((always_inline)) {
        const int kv = i / (16 * (D / 8)), piece = i % (D / 8);
        if (row >= 0) {
            bf16_t *dst = (kv ? Vb : Kb) + (size_t)row * D + piece * 8;
            if (NW == 4) __builtin_nontemporal_store(w, reinterpret_cast<u32x4_t *>(dst));
            else *reinterpret_cast<u32x4_t *>(dst) = w;
        }
    };
    // held-back pieces of this thread: slot q holds PPT pieces of one tile (all in output row held_row[q]: a thread's
    // pieces of a tile differ in K / V only) while bit q of held is set (wave-uniform)
    static_assert(!STAGED || (64 * NW) % (16 * (D / 8)) == 0, "a thread's pieces of a tile share the tile row");
    u32x4_t held_w[NS][PPT];
    int held_row[NS];
    unsigned held = 0;
    long long slot = 0;
    if constexpr (STAGED) slot = wall_clock64() >> a.flush_shift;
    auto flush = [&]() __attribute__((always_inline)) {
        if constexpr (STAGED) {
#pragma unroll
            for (int q = 0; q < NS; ++q)
                if (held >> q & 1u) {
#pragma unroll
                    for (int k = 0; k < PPT; ++k) store_piece(held_row[q], tid + k * 64 * NW, held_w[q][k]);
                }
            held = 0;
        }
    };
    auto flush_if_new_slot = [&]() __attribute__((always_inline)) {
        if constexpr (STAGED) {
            const long long now = wall_clock64() >> a.flush_shift;
            if (now != slot) { flush(); slot = now; }
        }
    };
    // a finished tile's pieces: held back (NW = 4) or written at once
    auto emit = [&](int tile, auto piece_of) __attribute__((always_inline)) {
        if constexpr (STAGED) {
            if (held == (1u << NS) - 1u) flush();            // no room (a slot is shorter than NS tiles normally)
            const int q = (held & 1u) == 0 ? 0 : 1;
            const int row = out_row(tile, tid);
#pragma unroll
            for (int qq = 0; qq < NS; ++qq)
                if (qq == q) {
#pragma unroll
                    for (int k = 0; k < PPT; ++k) held_w[qq][k] = piece_of(tid + k * 64 * NW);
                    held_row[qq] = row;
                }
            held |= 1u << q;
        } else {
            for (int i = tid; i < PIECES; i += 64 * NW) store_piece(out_row(tile, i), i, piece_of(i));
        }
    };
    static_assert(NS == 2, "emit() picks the first free of two slots");

    // One batch = 32 tokens of a tile row (16 loads of 16 bytes per lane: 8 tokens x {K, V}).
    // first element this lane reads of row i (of this wave) of a tile
    auto row_base = [&](int tl, int i) __attribute__((always_inline)) {
        const int r = min((tl % tiles_per_layer) * 16 + wave * RPW + i, rows_per_layer - 1);   // clamped: a tail row repeats the last one
        const size_t s = (size_t)(tl / tiles_per_layer) * a.BH + r / nch;
        const int c = a.c0 + r % nch;
        return (s * a.T_cap + (size_t)c * a.C) * D + n * EPL;
    };
    Raw<bf16_t, EPL> xk[8], xv[8];
    // tokens j0 + g4 + 4u, u in [U0, U1): branch-free tail, a token past the chunk is loaded from the last one and gets
    // weight 0 (x * 1 + s rounds as x + s; the maximum needs no weight: the repeated token changes nothing), so every
    // load of a batch is in flight before the first use
    auto issue = [&](size_t tok0, int j0, auto u0_tag, auto u1_tag) __attribute__((always_inline)) {
#pragma unroll
        for (int u = decltype(u0_tag)::value; u < decltype(u1_tag)::value; ++u) {
            const int j = j0 + g4 + 4 * u;
            const size_t off = tok0 + (size_t)(j < a.C ? j : a.C - 1) * D;
            xk[u].load_stream(K + off);
            xv[u].load_stream(V + off);
        }
    };
    float sk[EPL], sv[EPL];
    auto consume = [&](int j0, auto u0_tag, auto u1_tag) __attribute__((always_inline)) {
#pragma unroll
        for (int u = decltype(u0_tag)::value; u < decltype(u1_tag)::value; ++u) {
            const float wgt = j0 + g4 + 4 * u < a.C ? 1.f : 0.f;
            float fk[EPL], fv[EPL];
            xk[u].get(fk);
            xv[u].get(fv);
            if (is_max) {
#pragma unroll
                for (int e = 0; e < EPL; ++e) { sk[e] = fmaxf(sk[e], fk[e]); sv[e] = fmaxf(sv[e], fv[e]); }
            } else {
#pragma unroll
                for (int e = 0; e < EPL; ++e) { sk[e] = fmaf(fk[e], wgt, sk[e]); sv[e] = fmaf(fv[e], wgt, sv[e]); }
            }
        }
    };
    using I0 = std::integral_constant<int, 0>;
    using I4 = std::integral_constant<int, 4>;
    using I8 = std::integral_constant<int, 8>;

    int tile = blockIdx.x;           // (one tile per workgroup unless the form is persistent)
    // The persistent form keeps half a batch ahead of itself at all times: the first 4 tokens of the next batch are
    // requested before the last 4 of this one are used, across rows, tiles and the MLP phase, so that a workgroup has
    // loads in flight while its waves are at the barriers and in the matrix work.
    size_t tok0 = row_base(tile, 0);
    if constexpr (STAGED) issue(tok0, 0, I0{}, I4{});
    do {
        const int l = tile / tiles_per_layer;

        // ---- 1. stream the chunks, fp32 means to LDS ------------------------------
        for (int i = 0; i < RPW; ++i) {
            const int rt = wave * RPW + i;                       // row within the tile
            if constexpr (!STAGED) tok0 = row_base(tile, i);
#pragma unroll
            for (int e = 0; e < EPL; ++e) sk[e] = sv[e] = is_max ? -INFINITY : 0.f;
            for (int j0 = 0; j0 < a.C; j0 += 32) {
                if constexpr (STAGED) {
                    flush_if_new_slot();
                    issue(tok0, j0, I4{}, I8{});
                    consume(j0, I0{}, I4{});
                    // the batch after this one: same row, next row, first row of the next tile; after the last batch of
                    // all, this one again (its values are never used)
                    int jn = j0 + 32, in = i, tn = tile;
                    if (jn >= a.C) {
                        jn = 0; in = i + 1;
                        if (in == RPW) {
                            in = 0; tn = tile + (int)gridDim.x;
                            if (tn >= ntiles) { tn = tile; in = i; jn = j0; }
                        }
                    }
                    const size_t tok0n = row_base(tn, in);
                    issue(tok0n, jn, I0{}, I4{});
                    consume(j0, I4{}, I8{});
                    tok0 = tok0n;
                } else {
                    issue(tok0, j0, I0{}, I8{});
                    consume(j0, I0{}, I8{});
                }
            }
            const float cf = is_max ? 1.f : (float)a.C;
#pragma unroll
            for (int e = 0; e < EPL; ++e) {
                if (is_max) {
                    sk[e] = fmaxf(sk[e], __shfl_xor(sk[e], 16)); sk[e] = fmaxf(sk[e], __shfl_xor(sk[e], 32));
                    sv[e] = fmaxf(sv[e], __shfl_xor(sv[e], 16)); sv[e] = fmaxf(sv[e], __shfl_xor(sv[e], 32));
                } else {
                    sk[e] += __shfl_xor(sk[e], 16); sk[e] += __shfl_xor(sk[e], 32);
                    sv[e] += __shfl_xor(sv[e], 16); sv[e] += __shfl_xor(sv[e], 32);
                }
            }
            if (g4 == 0) {
#pragma unroll
                for (int e = 0; e < EPL; e += 2) {
                    uint32_t hi, mid, lo;
                    split3_pair(sk[e] / cf, sk[e + 1] / cf, hi, mid, lo);
                    *reinterpret_cast<uint32_t *>(xm + ((0 * 2 + 0) * 16 + rt) * XP + n * EPL + e) = hi;
                    *reinterpret_cast<uint32_t *>(xm + ((1 * 2 + 0) * 16 + rt) * XP + n * EPL + e) = mid;
                    *reinterpret_cast<uint32_t *>(xm + ((2 * 2 + 0) * 16 + rt) * XP + n * EPL + e) = lo;
                    split3_pair(sv[e] / cf, sv[e + 1] / cf, hi, mid, lo);
                    *reinterpret_cast<uint32_t *>(xm + ((0 * 2 + 1) * 16 + rt) * XP + n * EPL + e) = hi;
                    *reinterpret_cast<uint32_t *>(xm + ((1 * 2 + 1) * 16 + rt) * XP + n * EPL + e) = mid;
                    *reinterpret_cast<uint32_t *>(xm + ((2 * 2 + 1) * 16 + rt) * XP + n * EPL + e) = lo;
                }
            }
        }
        __syncthreads();

        if (a.mode != KVEV_POOL_MLP) {      // mean or maximum: the tile rows are the output (a bf16 maximum is its own hi term)
            emit(tile, [&](int i) __attribute__((always_inline)) {
                const int kv = i / (16 * (D / 8)), rt = (i / (D / 8)) % 16, piece = i % (D / 8);
                float m[8];
#pragma unroll
                for (int e = 0; e < 8; ++e) m[e] = 0.f;      // lo + mid + hi is exact: each partial sum is a prefix of the fp32 mean
#pragma unroll
                for (int p = 2; p >= 0; --p) {
                    const u32x4_t w = *reinterpret_cast<const u32x4_t *>(xm + ((p * 2 + kv) * 16 + rt) * XP + piece * 8);
#pragma unroll
                    for (int q = 0; q < 4; ++q) {
                        m[2 * q] += __uint_as_float(w[q] << 16);
                        m[2 * q + 1] += __uint_as_float(w[q] & 0xFFFF0000u);
                    }
                }
                return u32x4_t{pack_bf16x2(m[0], m[1]), pack_bf16x2(m[2], m[3]), pack_bf16x2(m[4], m[5]), pack_bf16x2(m[6], m[7])};
            });
            __syncthreads();                // the planes are read: the next tile may overwrite them
            continue;
        }

        // ---- 2. layer 1: act = GELU(W1 xbar + b1), tiles of 16 hidden units ------
        const int ds = a.d_sum;
        const int tiles1 = ds / 16;
        // this layer's packed weights: [W1: side, unit tile, k-step][W2: side, output tile, k-step][b1: side][b2: side]
        const unsigned char *wpl = static_cast<const unsigned char *>(a.wpack) + (size_t)l * ((size_t)8 * ds * D + (size_t)8 * (ds + D));
        for (int t = wave; t < 2 * tiles1; t += NW) {
            const int kv = t / tiles1, u0 = (t % tiles1) * 16;
            const bf16_t *W1 = static_cast<const bf16_t *>(kv ? a.W1V : a.W1K) + ((size_t)l * ds + u0 + n) * D + g4 * 8;
            const bf16_t *b1 = static_cast<const bf16_t *>(kv ? a.b1V : a.b1K) + (size_t)l * ds + u0 + 4 * g4;
            const bf16x8_t *W1p = reinterpret_cast<const bf16x8_t *>(wpl) + (size_t)t * (D / 32) * 64 + lane;
            f32x4_t acc;
            if constexpr (PK) {
                acc = *reinterpret_cast<const f32x4_t *>(wpl + (size_t)8 * ds * D + ((size_t)kv * ds + u0 + 4 * g4) * 4);
            } else {
#pragma unroll
                for (int r = 0; r < 4; ++r) acc[r] = bf16_to_f32(b1[r]);
            }
#pragma unroll
            for (int ks = 0; ks < D / 32; ++ks) {
                const bf16x8_t w = PK ? W1p[ks * 64] : *reinterpret_cast<const bf16x8_t *>(W1 + ks * 32);
#pragma unroll
                for (int p = 2; p >= 0; --p) {
                    const bf16x8_t x = *reinterpret_cast<const bf16x8_t *>(xm + ((p * 2 + kv) * 16 + n) * XP + ks * 32 + g4 * 8);
                    acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(w, x, acc, 0, 0, 0);
                }
            }
            uint32_t hi[2], mid[2], lo[2];
            split3_pair(gelu_erf(acc[0]), gelu_erf(acc[1]), hi[0], mid[0], lo[0]);
            split3_pair(gelu_erf(acc[2]), gelu_erf(acc[3]), hi[1], mid[1], lo[1]);
            bf16_t *ap = act + (size_t)(kv * 16 + n) * AP + u0 + 4 * g4;
            *reinterpret_cast<uint2 *>(ap + (size_t)0 * 2 * 16 * AP) = make_uint2(hi[0], hi[1]);
            *reinterpret_cast<uint2 *>(ap + (size_t)1 * 2 * 16 * AP) = make_uint2(mid[0], mid[1]);
            *reinterpret_cast<uint2 *>(ap + (size_t)2 * 2 * 16 * AP) = make_uint2(lo[0], lo[1]);
        }
        __syncthreads();

        // ---- 3. layer 2: summary = W2 act + b2, tiles of 16 output elements ------
        constexpr int tiles2 = D / 16;
        for (int t = wave; t < 2 * tiles2; t += NW) {
            const int kv = t / tiles2, e0 = (t % tiles2) * 16;
            const bf16_t *W2 = static_cast<const bf16_t *>(kv ? a.W2V : a.W2K) + ((size_t)l * D + e0 + n) * ds + g4 * 8;
            const bf16_t *b2 = static_cast<const bf16_t *>(kv ? a.b2V : a.b2K) + (size_t)l * D + e0 + 4 * g4;
            const bf16x8_t *W2p = reinterpret_cast<const bf16x8_t *>(wpl + (size_t)4 * ds * D) + (size_t)t * (ds / 32) * 64 + lane;
            f32x4_t acc;
            if constexpr (PK) {
                acc = *reinterpret_cast<const f32x4_t *>(wpl + (size_t)8 * ds * D + ((size_t)2 * ds + kv * D + e0 + 4 * g4) * 4);
            } else {
#pragma unroll
                for (int r = 0; r < 4; ++r) acc[r] = bf16_to_f32(b2[r]);
            }
            for (int ks = 0; ks < ds / 32; ++ks) {
                const bf16x8_t w = PK ? W2p[ks * 64] : *reinterpret_cast<const bf16x8_t *>(W2 + ks * 32);
#pragma unroll
                for (int p = 2; p >= 0; --p) {
                    const bf16x8_t x = *reinterpret_cast<const bf16x8_t *>(act + ((size_t)(p * 2 + kv) * 16 + n) * AP + ks * 32 + g4 * 8);
                    acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(w, x, acc, 0, 0, 0);
                }
            }
            // (the mean planes are free since the barrier before this layer: the output tile takes their place)
            uint2 o;
            o.x = pack_bf16x2(acc[0], acc[1]);
            o.y = pack_bf16x2(acc[2], acc[3]);
            *reinterpret_cast<uint2 *>(xm + (size_t)(kv * 16 + n) * XP + e0 + 4 * g4) = o;
        }
        __syncthreads();
        emit(tile, [&](int i) __attribute__((always_inline)) {
            const int kv = i / (16 * (D / 8)), rt = (i / (D / 8)) % 16, piece = i % (D / 8);
            return *reinterpret_cast<const u32x4_t *>(xm + (size_t)(kv * 16 + rt) * XP + piece * 8);
        });
        __syncthreads();                    // the output tile is read: the next tile may overwrite it
    } while (STAGED && (tile += gridDim.x) < ntiles);
    flush();
}

// One 16-byte piece per thread: the weight fragments in the order pool_mfma_kernel<D, NW, true> reads them, then the
// biases as fp32 (four per thread).
template <int D>
__global__ __launch_bounds__(256) void pool_pack_kernel(PoolArgs a)
{
    const int ds = a.d_sum;
    const size_t nw = (size_t)2 * ds * D / 8;                 // pieces of W1 (both sides) per layer; W2 has as many
    const size_t nb = (size_t)2 * (ds + D) / 4;               // bias pieces per layer
    const size_t per_layer = 2 * nw + nb;
    const size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
    if (i >= per_layer * a.L) return;
    const int l = (int)(i / per_layer);
    size_t r = i % per_layer;
    unsigned char *dst = static_cast<unsigned char *>(a.wpack) + (size_t)l * pool_pack_layer_bytes(D, ds) + r * 16;
    if (r < 2 * nw) {
        const bool second = r >= nw;                           // W2: rows are output elements, columns hidden units
        if (second) r -= nw;
        const int rows = second ? D : ds, cols = second ? ds : D, ksn = cols / 32;
        const int lane = (int)(r % 64);
        size_t q = r / 64;
        const int ks = (int)(q % ksn); q /= ksn;
        const int t = (int)(q % (rows / 16)), kv = (int)(q / (rows / 16));
        const bf16_t *W = static_cast<const bf16_t *>(second ? (kv ? a.W2V : a.W2K) : (kv ? a.W1V : a.W1K));
        const bf16_t *src = W + ((size_t)l * rows + t * 16 + (lane & 15)) * cols + ks * 32 + (lane >> 4) * 8;
        *reinterpret_cast<uint4 *>(dst) = *reinterpret_cast<const uint4 *>(src);
    } else {
        r -= 2 * nw;                                           // four biases: b1 of K, b1 of V, b2 of K, b2 of V
        const int e = (int)r * 4;
        const bf16_t *b;
        if (e < 2 * ds) b = static_cast<const bf16_t *>(e < ds ? a.b1K : a.b1V) + (size_t)l * ds + e % ds;
        else b = static_cast<const bf16_t *>(e - 2 * ds < D ? a.b2K : a.b2V) + (size_t)l * D + (e - 2 * ds) % D;
        *reinterpret_cast<float4 *>(dst) = make_float4(bf16_to_f32(b[0]), bf16_to_f32(b[1]), bf16_to_f32(b[2]), bf16_to_f32(b[3]));
    }
}

// Workgroups of the persistent form: as many as stay resident at once (by LDS and registers), per compute unit.  The
// answer for the last LDS size asked about is kept (one word: size and answer together), so that a serving loop does not
// query the runtime on every launch.
template <int D> static int persistent_grid(size_t lds, int compute_units)
{
    static std::atomic<uint64_t> last{0};
    const uint64_t seen = last.load(std::memory_order_relaxed);
    int per_cu = 0;
    if (seen != 0 && (seen >> 8) == lds) per_cu = (int)(seen & 0xff);
    else {
        if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, pool_mfma_kernel<D, 4, true>, 256, lds) != hipSuccess || per_cu < 1) per_cu = 1;
        per_cu = std::min(per_cu, 255);
        last.store(((uint64_t)lds << 8) | (uint64_t)per_cu, std::memory_order_relaxed);
    }
    return per_cu * compute_units;
}

hipError_t launch_pool_mfma(const PoolArgs &a, hipStream_t st)
{
    const int nch = a.c1 - a.c0;
    const size_t rows_per_layer = (size_t)a.BH * nch;
    const size_t blocks = (size_t)a.L * ((rows_per_layer + 15) / 16);
    if (blocks == 0) return hipSuccess;
    const size_t lds = sizeof(bf16_t) * 3 * 2 * 16 * (((size_t)a.d + 8) + ((size_t)a.d_sum + 8));
    const bool few = blocks < 2048;          // fewer than 8 tiles per compute unit
    // launches that fill the chip many times over read the MLP weights in fragment order when the caller gave room for them
    const bool pk = !few && a.mode == KVEV_POOL_MLP && a.wpack != nullptr;
    if (pk) {
        const size_t pieces = pool_pack_bytes(a.L, a.d, a.d_sum) / 16;
        const dim3 pgrid((unsigned)((pieces + 255) / 256));
        if (a.d == 64) hipLaunchKernelGGL((pool_pack_kernel<64>), pgrid, dim3(256), 0, st, a);
        else hipLaunchKernelGGL((pool_pack_kernel<128>), pgrid, dim3(256), 0, st, a);
    }
    if (a.d == 64) {
        const dim3 pgrid((unsigned)std::min<size_t>(blocks, persistent_grid<64>(lds, a.compute_units)));
        if (few) hipLaunchKernelGGL((pool_mfma_kernel<64, 16, false>), dim3((unsigned)blocks), dim3(1024), lds, st, a);
        else if (pk) hipLaunchKernelGGL((pool_mfma_kernel<64, 4, true>), pgrid, dim3(256), lds, st, a);
        else hipLaunchKernelGGL((pool_mfma_kernel<64, 4, false>), pgrid, dim3(256), lds, st, a);
    } else {
        const dim3 pgrid((unsigned)std::min<size_t>(blocks, persistent_grid<128>(lds, a.compute_units)));
        if (few) hipLaunchKernelGGL((pool_mfma_kernel<128, 16, false>), dim3((unsigned)blocks), dim3(1024), lds, st, a);
        else if (pk) hipLaunchKernelGGL((pool_mfma_kernel<128, 4, true>), pgrid, dim3(256), lds, st, a);
        else hipLaunchKernelGGL((pool_mfma_kernel<128, 4, false>), pgrid, dim3(256), lds, st, a);
    }
    return hipGetLastError();
}

}  // namespace kvev

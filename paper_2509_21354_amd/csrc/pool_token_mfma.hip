// Chunk aggregation with the MLP applied to every token (section 3 of the paper
// lists a multi-layer perceptron among the aggregators; Eq. 2 feeds it the set of
// the chunk's C vectors): summary = (1/C) sum_j [ W2 GELU(W1 x_j + b1) + b2 ],
// bf16 storage.
//
// The second layer is linear, so it commutes with the average:
//   summary = W2 * ( (1/C) sum_j GELU(W1 x_j + b1) ) + b2.
// What is left per token is one d -> d_sum layer, a real dense contraction
// (2*C*d*d_sum flop per chunk and side), and C*d_sum GELUs, which are what the
// kernel's time goes into: one exp2 (quarter rate) and 11 vector operations each
// against 1/8 of an MFMA.
//
// A workgroup (16 waves) holds W1 of both sides of one layer in LDS and walks
// tiles of 16 (sequence, chunk) rows of that layer.  A wave takes one row of the
// tile, 16 tokens at a time:
//   A = the tokens' rows, straight from global memory (lane = token, 16 bytes of
//       the row per k-step; the next 16 tokens are in flight meanwhile),
//   B = 16 hidden units' rows of W1 from LDS,
//   C = 4 tokens x 1 hidden unit per lane, bias already in the accumulator:
//       GELU, summed over the lane's tokens into one register per 16 hidden units.
// After the chunk's last token the sums of the 4 lane groups are added, divided
// by C and cut into three bf16 terms (exact to 24 bits) for the second layer, which
// runs for the 16 rows together as in pool_mfma.hip.
#include "common.hpp"
#include "kernels.hpp"

namespace kvev {

// GELU(z) = z Phi(z) = max(z, 0) - |z| E(|z|) = z/2 + |z| (1/2 - E(|z|)), E(u) = erfc(u / sqrt 2) / 2 = exp2(u P(u) - 1) with u clamped
// to 4 sqrt 2 (E there is 7.7e-9): P is a 7-coefficient fit (fit_gelu_poly.py beside this file derives the
// constants; |E_poly - E| < 9e-8 in fp32, i.e. the exact-erf GELU to fp32 accuracy).  Returns acc + GELU(z):
// 11 vector operations and one exp2.
__device__ __forceinline__ float add_gelu_poly(float acc, float z)
{
    const float u = __builtin_amdgcn_fmed3f(fabsf(z), 0.f, 5.656854f);      // = min(|z|, 4 sqrt 2) in one operation
    float q = 8.858236e-06f;
    q = fmaf(q, u, -5.7695375e-05f);
    q = fmaf(q, u, -0.0004069862f);
    q = fmaf(q, u, 0.007363135f);
    q = fmaf(q, u, -0.052666616f);
    q = fmaf(q, u, -0.45916432f);
    q = fmaf(q, u, -1.1511089f);
    q = fmaf(q, u, -1.0f);
    const float e = __builtin_amdgcn_exp2f(q);
    return fmaf(fabsf(z), 0.5f - e, fmaf(0.5f, z, acc));                    // max(z, 0) = (z + |z|) / 2
}

// two fp32 -> three bf16 terms each (sum exact to 24 bits), one value at a time
__device__ __forceinline__ void split3_one(float x, bf16_t &hi, bf16_t &mid, bf16_t &lo)
{
    const uint32_t h = pack_bf16x2(x, 0.f) & 0xFFFFu;
    const float r = x - __uint_as_float(h << 16);
    const uint32_t m = pack_bf16x2(r, 0.f) & 0xFFFFu;
    const uint32_t l = pack_bf16x2(r - __uint_as_float(m << 16), 0.f) & 0xFFFFu;
    hi = (bf16_t)h; mid = (bf16_t)m; lo = (bf16_t)l;
}

constexpr int kTokWaves = 16;            // waves per workgroup = rows of a tile: one row each
constexpr int kTokMaxCT = 16;            // hidden-unit tiles a lane can accumulate: d_sum <= 256

// One token tile of one side: for each of the NCT tiles of 16 hidden units, layer 1 on the matrix cores and the
// GELUs of the lane's 4 tokens added to the tile's running sum.  PARTIAL: the chunk ends inside this token tile;
// a row past its end enters as z = 0 (GELU(0) = 0).
// Software pipeline over the hidden tiles, in program order and pinned there: while the four GELUs of tile ct
// are evaluated, the MFMAs of tile ct+1 are issued between them (the matrix pipe works under the vector
// instructions of the same wave) and the W1 fragments of tile ct+2 travel from LDS.  The accumulator starts
// from the bias, read as one 16-byte LDS load from a table that holds every bias four times.
template <int D, int NCT, bool PARTIAL>
__device__ __forceinline__ void token_tile(const bf16x8_t (&xa)[D / 32], const bf16_t *wrow, const f32x4_t *brow,
                                           int live_tokens, float (&sum)[NCT])
{
    constexpr int KS = D / 32, XP = D + 8;
    bf16x8_t wb[2][KS];
    f32x4_t acc[2];
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) wb[0][ks] = *reinterpret_cast<const bf16x8_t *>(wrow + ks * 32);
    acc[0] = brow[0];
    if (NCT > 1) {
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) wb[1][ks] = *reinterpret_cast<const bf16x8_t *>(wrow + (size_t)16 * XP + ks * 32);
        acc[1] = brow[16];
    }
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) acc[0] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(xa[ks], wb[0][ks], acc[0], 0, 0, 0);
    static_for<NCT>([&](auto ct_) {
        constexpr int ct = decltype(ct_)::value, cur = ct & 1, nxt = cur ^ 1;
        f32x4_t z = acc[cur];
        if (PARTIAL) {
#pragma unroll
            for (int r = 0; r < 4; ++r) z[r] = r < live_tokens ? z[r] : 0.f;
        }
        if (ct + 2 < NCT) {      // wb[cur] and acc[cur] are free again: tile ct+2 starts its way
#pragma unroll
            for (int ks = 0; ks < KS; ++ks)
                wb[cur][ks] = *reinterpret_cast<const bf16x8_t *>(wrow + (size_t)(ct + 2) * 16 * XP + ks * 32);
            acc[cur] = brow[(ct + 2) * 16];
        }
        __builtin_amdgcn_sched_barrier(0);
        // (two partial sums: the chain through one register would serialise the four GELUs)
        // The empty asm statements are ordered among themselves and carry the values through: they pin each
        // MFMA before, and each GELU after, its place in the sequence (pure arithmetic would otherwise float).
        float s0 = sum[ct], s1 = 0.f;
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            float ze = z[e];
            if (ct + 1 < NCT && (e + 1) * KS / 4 > e * KS / 4) {
#pragma unroll
                for (int ks = e * KS / 4; ks < (e + 1) * KS / 4; ++ks)
                    acc[nxt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(xa[ks], wb[nxt][ks], acc[nxt], 0, 0, 0);
                asm volatile("" : "+v"(acc[nxt]), "+v"(ze));
            } else {
                asm volatile("" : "+v"(ze));
            }
            if (e & 1) { s1 = add_gelu_poly(s1, ze); asm volatile("" : "+v"(s1)); }
            else { s0 = add_gelu_poly(s0, ze); asm volatile("" : "+v"(s0)); }
        }
        sum[ct] = s0 + s1;
    });
}

template <int D, int NCT>
__global__ __launch_bounds__(64 * kTokWaves) void pool_token_mfma_kernel(PoolArgs a)
{
    constexpr int KS = D / 32, XP = D + 8, THREADS = 64 * kTokWaves;
    extern __shared__ __align__(16) bf16_t smem_tok[];
    constexpr int ds = NCT * 16, AP = ds + 8;
    bf16_t *w1s = smem_tok;                                   // [2 (K,V)][d_sum][XP]
    bf16_t *act = w1s + (size_t)2 * ds * XP;                  // [3 terms][2][16 rows][AP]   mean activations
    f32x4_t *b1s = reinterpret_cast<f32x4_t *>(act + (size_t)3 * 2 * 16 * AP);   // [2][d_sum], every bias four times

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int n = lane & 15, g4 = lane >> 4;
    const int nch = a.c1 - a.c0;
    const int rows_per_layer = a.BH * nch;
    const int tiles_per_layer = (rows_per_layer + 15) / 16;
    const int l = blockIdx.y;

    // ---- 0. this layer's first-layer weights and biases into LDS -----------------
    for (int p = tid; p < 2 * ds * (D / 8); p += THREADS) {
        const int piece = p % (D / 8), u = (p / (D / 8)) % ds, kv = p / ((D / 8) * ds);
        const bf16_t *W1 = static_cast<const bf16_t *>(kv ? a.W1V : a.W1K) + ((size_t)l * ds + u) * D + piece * 8;
        *reinterpret_cast<bf16x8_t *>(w1s + ((size_t)kv * ds + u) * XP + piece * 8) = *reinterpret_cast<const bf16x8_t *>(W1);
    }
    for (int p = tid; p < 2 * ds; p += THREADS) {
        const int kv = p / ds, u = p % ds;
        const float b = bf16_to_f32(static_cast<const bf16_t *>(kv ? a.b1V : a.b1K)[(size_t)l * ds + u]);
        b1s[p] = f32x4_t{b, b, b, b};
    }
    __syncthreads();

    const bf16_t *K = static_cast<const bf16_t *>(a.K), *V = static_cast<const bf16_t *>(a.V);
    bf16_t *Kb = static_cast<bf16_t *>(a.Kbar), *Vb = static_cast<bf16_t *>(a.Vbar);
    const int ntt = (a.C + 15) / 16;                    // token tiles per chunk
    const int nsteps = 2 * ntt;                         // (side, token tile)
    for (int tile = blockIdx.x; tile < tiles_per_layer; tile += gridDim.x) {
    const int row0 = tile * 16;
    // ---- 1. per token: layer 1 + GELU, summed over the chunk ---------------------
    // the A fragments of step q: token tile tt of side kv (a token past the chunk repeats the last one)
    auto fetch = [&](int q, bf16x8_t (&x)[KS]) {
        const int tt = q % ntt, kv = q / ntt;
        const int r = min(row0 + wave, rows_per_layer - 1);              // a tail row repeats the last one
        const size_t s = (size_t)l * a.BH + r / nch;
        const int c = a.c0 + r % nch;
        const int j = min(tt * 16 + n, a.C - 1);
        const bf16_t *src = (kv ? V : K) + (s * a.T_cap + (size_t)c * a.C + j) * D + g4 * 8;
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) x[ks] = *reinterpret_cast<const bf16x8_t *>(src + ks * 32);
    };
    bf16x8_t xa[KS], xn[KS];
    float sum[NCT];
    fetch(0, xn);
    for (int q = 0; q < nsteps; ++q) {
        const int tt = q % ntt, kv = q / ntt;
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) xa[ks] = xn[ks];
        if (q + 1 < nsteps) fetch(q + 1, xn);
        if (tt == 0) {
#pragma unroll
            for (int ct = 0; ct < NCT; ++ct) sum[ct] = 0.f;
        }
        const int live_tokens = a.C - tt * 16 - 4 * g4;     // rows 4*g4 + r of this tile with r < live_tokens exist
        const bf16_t *wrow = w1s + ((size_t)kv * ds + n) * XP + g4 * 8;
        const f32x4_t *brow = b1s + kv * ds + n;
        if (tt * 16 + 16 <= a.C)
            token_tile<D, NCT, false>(xa, wrow, brow, live_tokens, sum);
        else
            token_tile<D, NCT, true>(xa, wrow, brow, live_tokens, sum);
        if (tt == ntt - 1) {
            const int rt = wave;
            const float inv_c = 1.0f / (float)a.C;
#pragma unroll
            for (int ct = 0; ct < NCT; ++ct) {
                float v = sum[ct];
                v += __shfl_xor(v, 16);
                v += __shfl_xor(v, 32);
                if (g4 == 0) {
                    bf16_t hi, mid, lo;
                    split3_one(v * inv_c, hi, mid, lo);
                    bf16_t *ap = act + (size_t)(kv * 16 + rt) * AP + ct * 16 + n;
                    ap[(size_t)0 * 2 * 16 * AP] = hi;
                    ap[(size_t)1 * 2 * 16 * AP] = mid;
                    ap[(size_t)2 * 2 * 16 * AP] = lo;
                }
            }
        }
    }
    __syncthreads();

    // ---- 2. layer 2 for the 16 rows: summary = W2 act + b2, tiles of 16 output elements ----
    const int r_out = row0 + n;
    const bool live = r_out < rows_per_layer;
    const int r_c = min(r_out, rows_per_layer - 1);
    const size_t out_row = (((size_t)l * a.BH + r_c / nch) * a.N_cap + (a.c0 + r_c % nch)) * D;
    constexpr int tiles2 = D / 16;
    for (int t = wave; t < 2 * tiles2; t += kTokWaves) {
        const int kv = t / tiles2, e0 = (t % tiles2) * 16;
        const bf16_t *W2 = static_cast<const bf16_t *>(kv ? a.W2V : a.W2K) + ((size_t)l * D + e0 + n) * ds + g4 * 8;
        const bf16_t *b2 = static_cast<const bf16_t *>(kv ? a.b2V : a.b2K) + (size_t)l * D + e0 + 4 * g4;
        f32x4_t acc;
#pragma unroll
        for (int r = 0; r < 4; ++r) acc[r] = bf16_to_f32(b2[r]);
        for (int ks = 0; ks < ds / 32; ++ks) {
            const bf16x8_t w = *reinterpret_cast<const bf16x8_t *>(W2 + ks * 32);
#pragma unroll
            for (int p = 2; p >= 0; --p) {
                const bf16x8_t x = *reinterpret_cast<const bf16x8_t *>(act + ((size_t)(p * 2 + kv) * 16 + n) * AP + ks * 32 + g4 * 8);
                acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(w, x, acc, 0, 0, 0);
            }
        }
        if (live) {
            uint2 o;
            o.x = pack_bf16x2(acc[0], acc[1]);
            o.y = pack_bf16x2(acc[2], acc[3]);
            *reinterpret_cast<uint2 *>((kv ? Vb : Kb) + out_row + e0 + 4 * g4) = o;
        }
    }
    __syncthreads();        // the next tile overwrites the activations
    }
}

constexpr size_t pool_token_lds_c(int d, int d_sum)
{
    return sizeof(bf16_t) * ((size_t)2 * d_sum * (d + 8) + (size_t)3 * 2 * 16 * (d_sum + 8)) + sizeof(float) * 4 * 2 * (size_t)d_sum;
}

size_t pool_token_mfma_lds(int d, int d_sum) { return pool_token_lds_c(d, d_sum); }

template <int D, int NCT>
static hipError_t launch_tok(const PoolArgs &a, dim3 grid, size_t lds, hipStream_t st)
{
    if constexpr (pool_token_lds_c(D, NCT * 16) > 160 * 1024) return hipErrorInvalidValue;   // does not fit: never built
    else {
    if (lds > 64 * 1024) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(pool_token_mfma_kernel<D, NCT>),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        if (e != hipSuccess) return e;
    }
    hipLaunchKernelGGL((pool_token_mfma_kernel<D, NCT>), grid, dim3(64 * kTokWaves), lds, st, a);
    return hipGetLastError();
    }
}

template <int D>
static hipError_t launch_tok_d(const PoolArgs &a, dim3 grid, size_t lds, hipStream_t st)
{
    switch (a.d_sum / 32) {
    case 1: return launch_tok<D, 2>(a, grid, lds, st);
    case 2: return launch_tok<D, 4>(a, grid, lds, st);
    case 3: return launch_tok<D, 6>(a, grid, lds, st);
    case 4: return launch_tok<D, 8>(a, grid, lds, st);
    case 5: return launch_tok<D, 10>(a, grid, lds, st);
    case 6: return launch_tok<D, 12>(a, grid, lds, st);
    case 7: return launch_tok<D, 14>(a, grid, lds, st);
    case 8: return launch_tok<D, 16>(a, grid, lds, st);
    default: return hipErrorInvalidValue;
    }
}

// needs bf16 storage, d in {64, 128}, d_sum a multiple of 32 up to 256, and pool_token_mfma_lds() of LDS
hipError_t launch_pool_token_mfma(const PoolArgs &a, hipStream_t st)
{
    if (a.d_sum % 32 != 0 || a.d_sum < 32 || a.d_sum > 16 * kTokMaxCT) return hipErrorInvalidValue;
    const int nch = a.c1 - a.c0;
    const size_t rows_per_layer = (size_t)a.BH * nch;
    const size_t tiles = (rows_per_layer + 15) / 16;
    if (tiles == 0) return hipSuccess;
    // one workgroup per compute unit and layer share is enough: each stages W1 once and loops over its tiles
    const size_t per_layer = (256 + a.L - 1) / a.L;
    const dim3 grid((unsigned)(tiles < per_layer ? tiles : per_layer), (unsigned)a.L);
    const size_t lds = pool_token_mfma_lds(a.d, a.d_sum);
    return a.d == 64 ? launch_tok_d<64>(a, grid, lds, st) : launch_tok_d<128>(a, grid, lds, st);
}

}  // namespace kvev

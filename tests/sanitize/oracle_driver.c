/*
 * Runs every function of the CPU oracle on small seeded inputs held in heap
 * buffers of exactly the size each call is entitled to touch, so that a build
 * with -fsanitize=address,undefined stops on any access outside them and on
 * undefined arithmetic.  Prints one checksum line per output; the test builds
 * this file twice (with and without the sanitizers) and compares the lines.
 * Test code: it includes the oracle's source, nothing of the GPU library.
 */
#include "../../oracle/kvev_oracle.c"
#include <stdio.h>

static uint32_t g_state = 1u;
static uint32_t lcg(void) { g_state = g_state * 1664525u + 1013904223u; return g_state; }
static float unif(void) { return (float)(lcg() >> 8) / 8388608.0f - 1.0f; }       /* [-1, 1) */

static void *buf(int dtype, size_t n, float scale)
{
    size_t es = dtype == KVO_F32 ? 4 : 2;
    void *p = malloc(n * es + (n == 0));
    for (size_t i = 0; i < n; ++i) st(p, dtype, i, (double)(unif() * scale));
    return p;
}

static uint64_t fnv(const void *p, size_t bytes)
{
    const unsigned char *b = p;
    uint64_t h = 1469598103934665603ull;
    for (size_t i = 0; i < bytes; ++i) { h ^= b[i]; h *= 1099511628211ull; }
    return h;
}

static void line(const char *what, int id, const void *p, size_t bytes)
{
    printf("%s %d %016llx\n", what, id, (unsigned long long)fnv(p, bytes));
}

static int run_case(int id, int dtype, int L, int B, int H, int H_kv, int d, int T, int T_pad, int C, int W, int k,
                    int d_sum, int d_g, int Tq, int mode)
{
    const int T_cap = T + T_pad, N = T / C, N_cap = N + 1, S = L * B * H_kv, k_cap = k + 1;
    const size_t es = dtype == KVO_F32 ? 4 : 2;
    int rc = 0;
    g_state = 977u * (uint32_t)id + 13u;
    void *K = buf(dtype, (size_t)S * T_cap * d, 1.f), *V = buf(dtype, (size_t)S * T_cap * d, 1.f);
    void *Q = buf(dtype, (size_t)L * B * H * Tq * d, 1.f);
    void *W1K = buf(dtype, (size_t)L * d_sum * d, 0.1f), *b1K = buf(dtype, (size_t)L * d_sum, 0.1f);
    void *W2K = buf(dtype, (size_t)L * d * d_sum, 0.1f), *b2K = buf(dtype, (size_t)L * d, 0.1f);
    void *W1V = buf(dtype, (size_t)L * d_sum * d, 0.1f), *b1V = buf(dtype, (size_t)L * d_sum, 0.1f);
    void *W2V = buf(dtype, (size_t)L * d * d_sum, 0.1f), *b2V = buf(dtype, (size_t)L * d, 0.1f);
    void *W_ih = buf(dtype, (size_t)L * 4 * d_g * 2 * d, 0.1f), *W_hh = buf(dtype, (size_t)L * 4 * d_g * d_g, 0.1f);
    void *b_ih = buf(dtype, (size_t)L * 4 * d_g, 0.1f), *b_hh = buf(dtype, (size_t)L * 4 * d_g, 0.1f);
    void *w_s = buf(dtype, (size_t)L * d_g, 0.3f), *b_s = buf(dtype, (size_t)L, 0.3f);
    void *Kbar = calloc((size_t)S * N_cap * d + 1, es), *Vbar = calloc((size_t)S * N_cap * d + 1, es);
    float *h = calloc((size_t)S * d_g + 1, 4), *c = calloc((size_t)S * d_g + 1, 4);
    float *util = calloc((size_t)S * N_cap + 1, 4), *gate = calloc((size_t)S * N_cap + 1, 4);
    int32_t *idx = calloc((size_t)S * k_cap + 1, 4), *count = calloc((size_t)S + 1, 4);
    int32_t *idx_t = calloc((size_t)S * N_cap + 1, 4), *count_t = calloc((size_t)S + 1, 4);
    void *O = calloc((size_t)L * B * H * Tq * d + 1, es), *D = calloc((size_t)L * B * H * Tq * d + 1, es);
    void *E = calloc((size_t)L * B * H * Tq * d + 1, es);

    /* pool in two ranges, gate in two calls that carry the state */
    rc |= kvo_chunk_pool(dtype, L, B, H_kv, d, T, T_cap, C, N_cap, d_sum, mode, K, V, W1K, b1K, W2K, b2K, W1V, b1V, W2V, b2V,
                         0, N / 2, Kbar, Vbar);
    rc |= kvo_chunk_pool(dtype, L, B, H_kv, d, T, T_cap, C, N_cap, d_sum, mode, K, V, W1K, b1K, W2K, b2K, W1V, b1V, W2V, b2V,
                         N / 2, N, Kbar, Vbar);
    rc |= kvo_lstm_gate(dtype, L, B, H_kv, d, N_cap, d_g, Kbar, Vbar, W_ih, W_hh, b_ih, b_hh, w_s, b_s, 0, N / 3, h, c, util, gate);
    rc |= kvo_lstm_gate(dtype, L, B, H_kv, d, N_cap, d_g, Kbar, Vbar, W_ih, W_hh, b_ih, b_hh, w_s, b_s, N / 3, N, h, c, util, gate);
    rc |= kvo_select_topk(S, T, C, W, N_cap, util, k, k_cap, idx, count);
    rc |= kvo_select_threshold(S, T, C, W, N_cap, gate, 0.5f, N_cap, idx_t, count_t);
    line("Kbar", id, Kbar, (size_t)S * N_cap * d * es);
    line("Vbar", id, Vbar, (size_t)S * N_cap * d * es);
    line("h", id, h, (size_t)S * d_g * 4);
    line("c", id, c, (size_t)S * d_g * 4);
    line("util", id, util, (size_t)S * N_cap * 4);
    line("idx", id, idx, (size_t)S * k_cap * 4);
    line("count", id, count, (size_t)S * 4);
    line("count_threshold", id, count_t, (size_t)S * 4);
    if (H_kv == H) {
        rc |= kvo_gated_attention(dtype, L, B, H, d, T, T_cap, C, N_cap, W, Q, Tq, K, V, Kbar, Vbar, idx, count, k_cap, O, NULL, 0);
        rc |= kvo_dense_attention(dtype, L, B, H, d, T, T_cap, Q, Tq, K, V, D, NULL, 0);
        line("O_gated", id, O, (size_t)L * B * H * Tq * d * es);
        line("O_dense", id, D, (size_t)L * B * H * Tq * d * es);
    }
    const int n_cand = (T > W ? T - W : 0) / C, win0 = n_cand * C;
    for (int causal = 0; causal <= (Tq <= T - win0 ? 1 : 0); ++causal) {
        rc |= kvo_attention_ext(dtype, L, B, H, H_kv, d, T, T_cap, C, N_cap, W, 1, causal, Q, Tq, K, V, Kbar, Vbar, idx, count,
                                k_cap, E);
        line(causal ? "O_ext_causal" : "O_ext", id, E, (size_t)L * B * H * Tq * d * es);
    }
    /* eviction: the store fed in two batches, then attention over store + the window kept in a ring */
    {
        void *Kc = calloc((size_t)S * k_cap * d + 1, es), *Vc = calloc((size_t)S * k_cap * d + 1, es);
        int32_t *ids = calloc((size_t)S * k_cap + 1, 4), *cnt = calloc((size_t)S + 1, 4);
        float *uc = calloc((size_t)S * k_cap + 1, 4);
        const int half = n_cand / 2;
        /* (summaries and scores of chunk c live in row c of the per-sequence arrays: pass the arrays whole) */
        rc |= kvo_retain(dtype, S, d, k, k_cap, Kbar, Vbar, util, N_cap, 0, half, Kc, Vc, ids, uc, cnt);
        if (n_cand > half) {
            /* the later chunks' rows, repacked per sequence (the call takes its own row capacity) */
            void *Kn = calloc((size_t)S * (n_cand - half) * d + 1, es), *Vn = calloc((size_t)S * (n_cand - half) * d + 1, es);
            float *un = calloc((size_t)S * (n_cand - half) + 1, 4);
            for (int s = 0; s < S; ++s) {
                memcpy((char *)Kn + (size_t)s * (n_cand - half) * d * es, (const char *)Kbar + ((size_t)s * N_cap + half) * d * es,
                       (size_t)(n_cand - half) * d * es);
                memcpy((char *)Vn + (size_t)s * (n_cand - half) * d * es, (const char *)Vbar + ((size_t)s * N_cap + half) * d * es,
                       (size_t)(n_cand - half) * d * es);
                memcpy(un + (size_t)s * (n_cand - half), util + (size_t)s * N_cap + half, (size_t)(n_cand - half) * 4);
            }
            rc |= kvo_retain(dtype, S, d, k, k_cap, Kn, Vn, un, n_cand - half, half, n_cand - half, Kc, Vc, ids, uc, cnt);
            free(Kn); free(Vn); free(un);
        }
        line("store_ids", id, ids, (size_t)S * k_cap * 4);
        line("store_count", id, cnt, (size_t)S * 4);
        const int wl = T - win0, W_cap = wl + 3, first = wl > 0 ? 2 : 0;
        void *Kr = calloc((size_t)S * W_cap * d + 1, es), *Vr = calloc((size_t)S * W_cap * d + 1, es);
        for (int s = 0; s < S; ++s)
            for (int t = 0; t < wl; ++t) {
                const int row = (first + t) % W_cap;
                memcpy((char *)Kr + ((size_t)s * W_cap + row) * d * es, (const char *)K + ((size_t)s * T_cap + win0 + t) * d * es, d * es);
                memcpy((char *)Vr + ((size_t)s * W_cap + row) * d * es, (const char *)V + ((size_t)s * T_cap + win0 + t) * d * es, d * es);
            }
        rc |= kvo_compact_attention(dtype, L, B, H, H_kv, d, wl, W_cap, first, Q, Tq, Kr, Vr, Kc, Vc, cnt, k_cap, 0, E);
        line("O_compact", id, E, (size_t)L * B * H * Tq * d * es);
        free(Kc); free(Vc); free(ids); free(cnt); free(uc); free(Kr); free(Vr);
    }
    free(K); free(V); free(Q); free(W1K); free(b1K); free(W2K); free(b2K); free(W1V); free(b1V); free(W2V); free(b2V);
    free(W_ih); free(W_hh); free(b_ih); free(b_hh); free(w_s); free(b_s); free(Kbar); free(Vbar); free(h); free(c);
    free(util); free(gate); free(idx); free(count); free(idx_t); free(count_t); free(O); free(D); free(E);
    return rc;
}

int main(void)
{
    int rc = 0;
    /*             id dtype     L  B  H  Hkv d   T    pad C   W    k  d_sum d_g Tq mode */
    rc |= run_case(1, KVO_F32,  1, 1, 2, 2, 16, 200,  0,  8,  24,  5, 12,  10, 1, KVO_POOL_MLP);
    rc |= run_case(2, KVO_BF16, 2, 1, 3, 3, 32, 333,  7, 16,  40,  6, 16,   8, 3, KVO_POOL_MLP);      /* ragged T */
    rc |= run_case(3, KVO_BF16, 1, 2, 2, 2, 16,  20,  0,  8,  64,  4,  8,   8, 1, KVO_POOL_MEAN);     /* T < W: no candidates */
    rc |= run_case(4, KVO_F32,  1, 1, 1, 1,  8,  96,  2,  4,   8,  0,  4,   4, 2, KVO_POOL_MAX);      /* k = 0 */
    rc |= run_case(5, KVO_BF16, 1, 1, 4, 2, 16, 160,  0,  8,  16, 99, 16,  12, 2, KVO_POOL_TOKEN_MLP); /* k > N_cand, grouped heads */
    rc |= run_case(6, KVO_F32,  1, 1, 1, 1,  8,   0,  4,  4,   8,  2,  4,   4, 1, KVO_POOL_MLP);      /* empty cache */
    rc |= run_case(7, KVO_BF16, 1, 1, 6, 3, 32, 128,  0, 32,  32,  2,  8,  16, 4, KVO_POOL_MLP);      /* a frame of queries, grouped */
    printf("bf16 %04x %04x %04x\n", kvo_bf16_round(1.00390625), kvo_bf16_round(-3.0e38), kvo_bf16_round(1e-45));
    printf("gelu %.17g %.17g\n", kvo_gelu(0.5), kvo_gelu(-3.0));
    printf("status %d\n", rc);
    return rc;
}

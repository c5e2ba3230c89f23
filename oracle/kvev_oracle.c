/*
 * CPU oracle for the RNN-gated chunked KV-cache decode step of KV-Efficient VLA.
 *
 * TEST INFRASTRUCTURE ONLY.  This file defines what the GPU library must
 * compute; it is slow on purpose (one thread, double arithmetic, no blocking,
 * no fusion) so that it can be checked against the paper by eye.  It shares
 * no code with the GPU library and must never be linked into, or called
 * from, the product path: only the tests, the smoke check and the bench's
 * CPU-baseline leg may use it.
 *
 * Every step follows the paper's own statement of the method:
 *   partition  section 3.2 (non-overlapping fixed-length chunks, temporal
 *              order) and section 3.3 (only chunks that are complete are aggregated)
 *   pool       Eq. 2, MLP_K / MLP_V; section 3.3 (the aggregator is a two-layer MLP); Eq. 6's
 *              term 4*d_sum*d per chunk fixes "once per chunk"
 *   gate       Eq. 3, an LSTM over [Kbar_t, Vbar_t] carrying h_t and emitting
 *              a score s_t in [0,1]
 *   select     retention of the most useful chunks, recent window excluded
 *              (section 3.2 last paragraph, section 3.3)
 *   attend     Eq. 1 over the union of kept summaries and the raw window
 *              (section 3.3, n' = W + M)
 *   dense      Eq. 1 over the whole cache
 *
 * Readings taken where the paper is silent are listed next to each function.
 *
 * Storage types: 0 = IEEE fp32, 1 = bfloat16 (top 16 bits of fp32).  Stored
 * values are up-cast exactly; all arithmetic is double; a result is rounded
 * to its storage type exactly once (round-to-nearest-even).
 *
 * Pinned by tests/test_oracle_pins.py (no function here is unpinned; the
 * readings themselves cannot be pinned, they are choices).
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

enum { KVO_F32 = 0, KVO_BF16 = 1 };
enum { KVO_OK = 0, KVO_BAD_ARG = 1 };
enum { KVO_POOL_MEAN = 0, KVO_POOL_MLP = 1, KVO_POOL_MAX = 2, KVO_POOL_TOKEN_MLP = 3 };

/* ---------- storage <-> double ------------------------------------------- */

static double ld(const void *p, int dtype, size_t i)
{
    if (dtype == KVO_F32)
        return (double)((const float *)p)[i];
    uint32_t bits = (uint32_t)((const uint16_t *)p)[i] << 16;
    float f;
    memcpy(&f, &bits, sizeof f);
    return (double)f;
}

/* double -> bfloat16, round to nearest even, done on the double itself so
 * that the value is rounded once and not twice (double->float->bf16). */
static uint16_t bf16_from_double(double x)
{
    if (isnan(x))
        return 0x7FC0u;
    double a = fabs(x);
    double r;
    if (isinf(a) || a == 0.0) {
        r = a;
    } else {
        int e;
        (void)frexp(a, &e);           /* a = m * 2^e, m in [0.5, 1) */
        int q = e - 8;                /* 8 significant bits: quantum 2^(e-8) */
        if (q < -133)
            q = -133;                 /* subnormal quantum of bfloat16 */
        r = ldexp(nearbyint(ldexp(a, -q)), q);   /* default mode: ties to even */
    }
    float f = (float)r;               /* exact, or +inf on overflow */
    if (signbit(x))
        f = -f;
    uint32_t bits;
    memcpy(&bits, &f, sizeof bits);
    return (uint16_t)(bits >> 16);
}

static void st(void *p, int dtype, size_t i, double x)
{
    if (dtype == KVO_F32)
        ((float *)p)[i] = (float)x;
    else
        ((uint16_t *)p)[i] = bf16_from_double(x);
}

/* exported so that a test can pin the rounding itself */
uint16_t kvo_bf16_round(double x) { return bf16_from_double(x); }

static double sigmoid(double x) { return 1.0 / (1.0 + exp(-x)); }

/* exact GELU (reading: the aggregator's activation is the erf form) */
static double gelu(double x) { return 0.5 * x * (1.0 + erf(x / sqrt(2.0))); }

double kvo_gelu(double x) { return gelu(x); }

/* ---------- pool: Eq. 2 ---------------------------------------------------
 * Reading: a chunk (a set of C vectors) enters the d -> d_sum -> d MLP through
 * its arithmetic mean; MLP_K and MLP_V have separate weights; weights are per
 * layer, shared by batch rows and heads.  Mode MEAN stops after the mean;
 * mode MAX (one of the alternative aggregators section 3 names, "pooling")
 * takes the element-wise maximum of the chunk instead, no weights.  Mode
 * TOKEN_MLP is the other way a set can enter an MLP of width d: the same
 * d -> d_sum -> d MLP is applied to every token of the chunk and the C outputs
 * are averaged (the "multi-layer perceptron" aggregator of section 3 read as a
 * per-element network followed by a symmetric reduction).
 *   K, V        [L,B,H,T_cap,d]       Kbar, Vbar [L,B,H,N_cap,d]
 *   W1 [L,d_sum,d] b1 [L,d_sum] W2 [L,d,d_sum] b2 [L,d]     (row-major out x in)
 * Writes summary rows [c0, c1); needs 0 <= c0 <= c1 <= floor(T/C) <= N_cap.
 */
static void pool_one(int dtype, int d, int C, int d_sum, int mode,
                     const void *X, size_t x_off,       /* first token of the chunk */
                     const void *W1, size_t w1_off, const void *b1, size_t b1_off,
                     const void *W2, size_t w2_off, const void *b2, size_t b2_off,
                     void *Y, size_t y_off, double *mean, double *act)
{
    if (mode == KVO_POOL_MAX) {             /* the "pooling" alternative of section 3: element-wise maximum */
        for (int e = 0; e < d; ++e) {
            double m = ld(X, dtype, x_off + e);
            for (int j = 1; j < C; ++j) {
                double x = ld(X, dtype, x_off + (size_t)j * d + e);
                if (x > m) m = x;
            }
            st(Y, dtype, y_off + e, m);
        }
        return;
    }
    if (mode == KVO_POOL_TOKEN_MLP) {       /* y = (1/C) sum_j MLP(x_j); mean[] holds the running sum of outputs */
        for (int e = 0; e < d; ++e)
            mean[e] = 0.0;
        for (int j = 0; j < C; ++j) {
            for (int u = 0; u < d_sum; ++u) {
                double z = ld(b1, dtype, b1_off + u);
                for (int e = 0; e < d; ++e)
                    z += ld(W1, dtype, w1_off + (size_t)u * d + e) * ld(X, dtype, x_off + (size_t)j * d + e);
                act[u] = gelu(z);
            }
            for (int e = 0; e < d; ++e) {
                double y = ld(b2, dtype, b2_off + e);
                for (int u = 0; u < d_sum; ++u)
                    y += ld(W2, dtype, w2_off + (size_t)e * d_sum + u) * act[u];
                mean[e] += y;
            }
        }
        for (int e = 0; e < d; ++e)
            st(Y, dtype, y_off + e, mean[e] / (double)C);
        return;
    }
    for (int e = 0; e < d; ++e) {
        double s = 0.0;
        for (int j = 0; j < C; ++j)
            s += ld(X, dtype, x_off + (size_t)j * d + e);
        mean[e] = s / (double)C;
    }
    if (mode == KVO_POOL_MEAN) {
        for (int e = 0; e < d; ++e)
            st(Y, dtype, y_off + e, mean[e]);
        return;
    }
    for (int u = 0; u < d_sum; ++u) {
        double z = ld(b1, dtype, b1_off + u);
        for (int e = 0; e < d; ++e)
            z += ld(W1, dtype, w1_off + (size_t)u * d + e) * mean[e];
        act[u] = gelu(z);
    }
    for (int e = 0; e < d; ++e) {
        double y = ld(b2, dtype, b2_off + e);
        for (int u = 0; u < d_sum; ++u)
            y += ld(W2, dtype, w2_off + (size_t)e * d_sum + u) * act[u];
        st(Y, dtype, y_off + e, y);
    }
}

int kvo_chunk_pool(int dtype, int L, int B, int H, int d, int T, int T_cap, int C, int N_cap,
                   int d_sum, int mode, const void *K, const void *V,
                   const void *W1K, const void *b1K, const void *W2K, const void *b2K,
                   const void *W1V, const void *b1V, const void *W2V, const void *b2V,
                   int c0, int c1, void *Kbar, void *Vbar)
{
    if (L < 1 || B < 1 || H < 1 || d < 1 || C < 1 || T < 0 || T > T_cap || d_sum < 1)
        return KVO_BAD_ARG;
    if (c0 < 0 || c0 > c1 || c1 > T / C || T / C > N_cap)
        return KVO_BAD_ARG;
    if (mode < KVO_POOL_MEAN || mode > KVO_POOL_TOKEN_MLP)
        return KVO_BAD_ARG;
    double *mean = malloc(sizeof(double) * (size_t)d);
    double *act = malloc(sizeof(double) * (size_t)d_sum);
    for (int l = 0; l < L; ++l)
        for (int b = 0; b < B; ++b)
            for (int h = 0; h < H; ++h) {
                size_t s = ((size_t)l * B + b) * H + h;
                for (int c = c0; c < c1; ++c) {
                    size_t x_off = (s * T_cap + (size_t)c * C) * d;
                    size_t y_off = (s * N_cap + c) * d;
                    pool_one(dtype, d, C, d_sum, mode, K, x_off,
                             W1K, (size_t)l * d_sum * d, b1K, (size_t)l * d_sum,
                             W2K, (size_t)l * d * d_sum, b2K, (size_t)l * d,
                             Kbar, y_off, mean, act);
                    pool_one(dtype, d, C, d_sum, mode, V, x_off,
                             W1V, (size_t)l * d_sum * d, b1V, (size_t)l * d_sum,
                             W2V, (size_t)l * d * d_sum, b2V, (size_t)l * d,
                             Vbar, y_off, mean, act);
                }
            }
    free(mean);
    free(act);
    return KVO_OK;
}

/* ---------- gate: Eq. 3 ---------------------------------------------------
 * Readings: the LSTM input is the concatenation [Kbar_t ; Vbar_t] (K first,
 * width 2d); the cell is the standard one with gate row blocks i, f, g, o and
 * two bias vectors; the score comes from a scalar linear head on h_t: the
 * utility u_t = w_s . h_t + b_s and the gate s_t = sigmoid(u_t) in [0,1].
 * One independent sequence per (layer, batch row, head), in chunk order.
 * The carried state (h, c) is fp32: it is rounded to fp32 after every step, so
 * that a run cut into several calls gives the same bits as one call.
 *   W_ih [L,4d_g,2d] W_hh [L,4d_g,d_g] b_ih,b_hh [L,4d_g] w_s [L,d_g] b_s [L]
 *   h, c [L,B,H,d_g] fp32 in/out;  util, gate [L,B,H,N_cap] fp32, [c0,c1) written
 */
int kvo_lstm_gate(int dtype, int L, int B, int H, int d, int N_cap, int d_g,
                  const void *Kbar, const void *Vbar,
                  const void *W_ih, const void *W_hh, const void *b_ih, const void *b_hh,
                  const void *w_s, const void *b_s, int c0, int c1,
                  float *h, float *c, float *util, float *gate)
{
    if (L < 1 || B < 1 || H < 1 || d < 1 || d_g < 1 || c0 < 0 || c0 > c1 || c1 > N_cap)
        return KVO_BAD_ARG;
    const int G = 4 * d_g;
    double *pre = malloc(sizeof(double) * (size_t)G);
    double *hn = malloc(sizeof(double) * (size_t)d_g);
    for (int l = 0; l < L; ++l)
        for (int b = 0; b < B; ++b)
            for (int hd = 0; hd < H; ++hd) {
                size_t s = ((size_t)l * B + b) * H + hd;
                float *hs = h + s * d_g, *cs = c + s * d_g;
                for (int t = c0; t < c1; ++t) {
                    size_t x_off = (s * N_cap + t) * d;
                    for (int r = 0; r < G; ++r) {
                        size_t wr = (size_t)l * G + r;
                        double a = ld(b_ih, dtype, wr) + ld(b_hh, dtype, wr);
                        for (int e = 0; e < d; ++e)
                            a += ld(W_ih, dtype, wr * 2 * d + e) * ld(Kbar, dtype, x_off + e);
                        for (int e = 0; e < d; ++e)
                            a += ld(W_ih, dtype, wr * 2 * d + d + e) * ld(Vbar, dtype, x_off + e);
                        for (int j = 0; j < d_g; ++j)
                            a += ld(W_hh, dtype, wr * d_g + j) * (double)hs[j];
                        pre[r] = a;
                    }
                    for (int j = 0; j < d_g; ++j) {
                        double ig = sigmoid(pre[j]);
                        double fg = sigmoid(pre[d_g + j]);
                        double gg = tanh(pre[2 * d_g + j]);
                        double og = sigmoid(pre[3 * d_g + j]);
                        double cn = fg * (double)cs[j] + ig * gg;
                        cs[j] = (float)cn;
                        /* h_t is formed from the stored (fp32) cell state */
                        hn[j] = og * tanh((double)cs[j]);
                    }
                    for (int j = 0; j < d_g; ++j)
                        hs[j] = (float)hn[j];
                    double u = ld(b_s, dtype, (size_t)l);
                    for (int j = 0; j < d_g; ++j)
                        u += ld(w_s, dtype, (size_t)l * d_g + j) * (double)hs[j];
                    util[s * N_cap + t] = (float)u;
                    gate[s * N_cap + t] = (float)sigmoid(u);
                }
            }
    free(pre);
    free(hn);
    return KVO_OK;
}

/* ---------- select ---------------------------------------------------------
 * Candidates are the chunks that lie wholly outside the raw recent window:
 * c < N_cand = floor(max(0, T - W) / C).  Order them by (utility descending,
 * index ascending); keep the first min(k, N_cand); emit ascending.  A NaN
 * utility counts as minus infinity.
 *   util [S,N_cap] fp32;  idx [S,k_cap] int32 (entries >= count untouched);
 *   count [S] int32.   S = L*B*H.
 * Threshold mode (the paper's literal rule, section 3.2): keep candidate c iff
 * gate[c] >= tau, at most k_cap of them (lowest indices first on overflow is
 * NOT applied: overflow is an argument error reported by the return value).
 */
typedef struct { float u; int c; } cand_t;

static float key_of(float u) { return isnan(u) ? -INFINITY : u; }

static int cand_cmp(const void *pa, const void *pb)
{
    const cand_t *a = pa, *b = pb;
    if (a->u > b->u) return -1;
    if (a->u < b->u) return 1;
    return (a->c > b->c) - (a->c < b->c);
}

static int int_cmp(const void *pa, const void *pb)
{
    int a = *(const int *)pa, b = *(const int *)pb;
    return (a > b) - (a < b);
}

int kvo_select_topk(int S, int T, int C, int W, int N_cap, const float *util, int k, int k_cap,
                    int32_t *idx, int32_t *count)
{
    if (S < 1 || C < 1 || T < 0 || W < 0 || k < 0 || k_cap < 0)
        return KVO_BAD_ARG;
    int n_cand = (T > W ? T - W : 0) / C;
    if (n_cand > N_cap)
        return KVO_BAD_ARG;
    int keep = k < n_cand ? k : n_cand;
    if (keep > k_cap)
        return KVO_BAD_ARG;
    cand_t *cand = malloc(sizeof(cand_t) * (size_t)(n_cand > 0 ? n_cand : 1));
    int *kept = malloc(sizeof(int) * (size_t)(keep > 0 ? keep : 1));
    for (int s = 0; s < S; ++s) {
        for (int c = 0; c < n_cand; ++c) {
            cand[c].u = key_of(util[(size_t)s * N_cap + c]);
            cand[c].c = c;
        }
        qsort(cand, (size_t)n_cand, sizeof(cand_t), cand_cmp);
        for (int i = 0; i < keep; ++i)
            kept[i] = cand[i].c;
        qsort(kept, (size_t)keep, sizeof(int), int_cmp);
        for (int i = 0; i < keep; ++i)
            idx[(size_t)s * k_cap + i] = kept[i];
        count[s] = keep;
    }
    free(cand);
    free(kept);
    return KVO_OK;
}

int kvo_select_threshold(int S, int T, int C, int W, int N_cap, const float *gate, float tau,
                         int k_cap, int32_t *idx, int32_t *count)
{
    if (S < 1 || C < 1 || T < 0 || W < 0 || k_cap < 0)
        return KVO_BAD_ARG;
    int n_cand = (T > W ? T - W : 0) / C;
    if (n_cand > N_cap)
        return KVO_BAD_ARG;
    int rc = KVO_OK;
    for (int s = 0; s < S; ++s) {
        int m = 0;
        for (int c = 0; c < n_cand; ++c)
            if (gate[(size_t)s * N_cap + c] >= tau) {   /* false for NaN */
                if (m < k_cap)
                    idx[(size_t)s * k_cap + m] = c;
                ++m;
            }
        if (m > k_cap) {
            rc = KVO_BAD_ARG;
            m = k_cap;
        }
        count[s] = m;
    }
    return rc;
}

/* ---------- attend: Eq. 1 over a list of rows --------------------------------
 * logits l_j = (q . key_j) / sqrt(d); p = softmax(l) (max subtracted);
 * o = sum_j p_j value_j; rounded once to the storage type.
 * `probs`, if not NULL, receives the n softmax weights (double).
 */
static void attend_rows(int dtype, int d, const void *Q, size_t q_off,
                        const void *const *key_base, const void *const *val_base,
                        const size_t *row_off, int n, void *O, size_t o_off,
                        double *logit, double *acc, double *probs)
{
    if (n == 0) {                         /* nothing to attend to: define o = 0 */
        for (int e = 0; e < d; ++e)
            st(O, dtype, o_off + e, 0.0);
        return;
    }
    double scale = 1.0 / sqrt((double)d);
    double m = -INFINITY;
    for (int j = 0; j < n; ++j) {
        double s = 0.0;
        for (int e = 0; e < d; ++e)
            s += ld(Q, dtype, q_off + e) * ld(key_base[j], dtype, row_off[j] + e);
        logit[j] = s * scale;
        if (logit[j] > m)
            m = logit[j];
    }
    double z = 0.0;
    for (int j = 0; j < n; ++j) {
        logit[j] = exp(logit[j] - m);
        z += logit[j];
    }
    for (int e = 0; e < d; ++e)
        acc[e] = 0.0;
    for (int j = 0; j < n; ++j) {
        double p = logit[j] / z;
        if (probs)
            probs[j] = p;
        for (int e = 0; e < d; ++e)
            acc[e] += p * ld(val_base[j], dtype, row_off[j] + e);
    }
    for (int e = 0; e < d; ++e)
        st(O, dtype, o_off + e, acc[e]);
}

/* Gated attention (section 3.3): per (l,b,h) the attended rows are the kept
 * summaries Kbar[idx[0..count)] in ascending chunk order, then the raw tokens
 * win0 .. T-1 with win0 = N_cand * C (readings: a chunk touching the window is
 * never a candidate, so no token is attended twice; the window grows back to
 * the chunk boundary when T-W is not a multiple of C; a summary is one plain
 * softmax position; all T cached tokens are visible to each of the Tq queries
 * and the queries do not attend to each other).
 *   Q, O [L,B,H,Tq,d];  idx [S,k_cap];  count [S]
 *   probs (nullable)    [S,Tq,probs_stride] double
 */
int kvo_gated_attention(int dtype, int L, int B, int H, int d, int T, int T_cap, int C,
                        int N_cap, int W, const void *Q, int Tq, const void *K, const void *V,
                        const void *Kbar, const void *Vbar, const int32_t *idx,
                        const int32_t *count, int k_cap, void *O, double *probs,
                        int probs_stride)
{
    if (L < 1 || B < 1 || H < 1 || d < 1 || C < 1 || T < 0 || T > T_cap || W < 0 || Tq < 0 ||
        k_cap < 0)
        return KVO_BAD_ARG;
    int n_cand = (T > W ? T - W : 0) / C;
    int win0 = n_cand * C;
    int n_max = k_cap + (T - win0);
    const void **kb = malloc(sizeof(void *) * (size_t)(n_max + 1));
    const void **vb = malloc(sizeof(void *) * (size_t)(n_max + 1));
    size_t *off = malloc(sizeof(size_t) * (size_t)(n_max + 1));
    double *logit = malloc(sizeof(double) * (size_t)(n_max + 1));
    double *acc = malloc(sizeof(double) * (size_t)d);
    int rc = KVO_OK;
    size_t S = (size_t)L * B * H;
    for (size_t s = 0; s < S && rc == KVO_OK; ++s) {
        int m = count[s];
        if (m < 0 || m > k_cap) {
            rc = KVO_BAD_ARG;
            break;
        }
        int n = 0;
        for (int i = 0; i < m; ++i) {
            int c = idx[s * k_cap + i];
            if (c < 0 || c >= n_cand || c >= N_cap) {
                rc = KVO_BAD_ARG;
                break;
            }
            kb[n] = Kbar;
            vb[n] = Vbar;
            off[n] = (s * N_cap + (size_t)c) * d;
            ++n;
        }
        if (rc != KVO_OK)
            break;
        for (int t = win0; t < T; ++t) {
            kb[n] = K;
            vb[n] = V;
            off[n] = (s * T_cap + (size_t)t) * d;
            ++n;
        }
        for (int i = 0; i < Tq; ++i) {
            size_t qo = (s * Tq + i) * d;
            attend_rows(dtype, d, Q, qo, kb, vb, off, n, O, qo, logit, acc,
                        probs ? probs + (s * Tq + i) * (size_t)probs_stride : NULL);
        }
    }
    free(kb);
    free(vb);
    free(off);
    free(logit);
    free(acc);
    return rc;
}

/* ---------- physical eviction (sections 3.2-3.3; the memory ratio closes section 3.3) ----
 * Chunks that are not kept are discarded, so what stays resident per sequence is
 * a compact store of at most k summaries plus the raw window.  The store holds,
 * ascending by chunk id: chunk_id [S,k_cap], util_c [S,k_cap], Kc, Vc [S,k_cap,d],
 * count [S].  retain merges n_new freshly scored chunks (ids first_chunk ..
 * first_chunk+n_new-1, all larger than every id in the store; summaries in rows
 * 0..n_new-1 of Kbar_new/Vbar_new [S,n_new_cap,d], scores util_new [S,n_new_cap])
 * and keeps the min(k, count+n_new) best under the order of kvo_select_topk
 * (utility descending, NaN as minus infinity, ties to the lower id).  Because a
 * chunk that drops out of the best k can never come back (scores of old chunks do
 * not change), the store always equals the top-k over every chunk seen so far.
 */
typedef struct { float u; int id; int src; } keep_t;      /* src < 0: new row -src-1, else store slot */

static int keep_cmp(const void *pa, const void *pb)
{
    const keep_t *a = pa, *b = pb;
    if (a->u > b->u) return -1;
    if (a->u < b->u) return 1;
    return (a->id > b->id) - (a->id < b->id);
}

static int keep_id_cmp(const void *pa, const void *pb)
{
    const keep_t *a = pa, *b = pb;
    return (a->id > b->id) - (a->id < b->id);
}

int kvo_retain(int dtype, int S, int d, int k, int k_cap, const void *Kbar_new, const void *Vbar_new,
               const float *util_new, int n_new_cap, int first_chunk, int n_new,
               void *Kc, void *Vc, int32_t *chunk_id, float *util_c, int32_t *count)
{
    if (S < 1 || d < 1 || k < 0 || k > k_cap || n_new < 0 || n_new > n_new_cap || first_chunk < 0)
        return KVO_BAD_ARG;
    size_t es = dtype == KVO_F32 ? 4 : 2, row = (size_t)d * es;
    keep_t *all = malloc(sizeof(keep_t) * (size_t)(k_cap + n_new + 1));
    unsigned char *tk = malloc(row * (size_t)(k_cap + 1)), *tv = malloc(row * (size_t)(k_cap + 1));
    int rc = KVO_OK;
    for (int s = 0; s < S && rc == KVO_OK; ++s) {
        int m = count[s], n = 0;
        if (m < 0 || m > k_cap) { rc = KVO_BAD_ARG; break; }
        for (int j = 0; j < m; ++j) {
            if (chunk_id[(size_t)s * k_cap + j] >= first_chunk) rc = KVO_BAD_ARG;
            all[n].u = key_of(util_c[(size_t)s * k_cap + j]);
            all[n].id = chunk_id[(size_t)s * k_cap + j];
            all[n].src = j;
            ++n;
        }
        for (int i = 0; i < n_new; ++i) {
            all[n].u = key_of(util_new[(size_t)s * n_new_cap + i]);
            all[n].id = first_chunk + i;
            all[n].src = -i - 1;
            ++n;
        }
        if (rc != KVO_OK) break;
        int keep = k < n ? k : n;
        qsort(all, (size_t)n, sizeof(keep_t), keep_cmp);
        qsort(all, (size_t)keep, sizeof(keep_t), keep_id_cmp);
        unsigned char *kc = (unsigned char *)Kc + (size_t)s * k_cap * row;
        unsigned char *vc = (unsigned char *)Vc + (size_t)s * k_cap * row;
        for (int j = 0; j < keep; ++j) {            /* gather into scratch first: slots move */
            const unsigned char *sk, *sv;
            if (all[j].src >= 0) {
                sk = kc + (size_t)all[j].src * row;
                sv = vc + (size_t)all[j].src * row;
            } else {
                size_t r = ((size_t)s * n_new_cap + (size_t)(-all[j].src - 1)) * row;
                sk = (const unsigned char *)Kbar_new + r;
                sv = (const unsigned char *)Vbar_new + r;
            }
            memcpy(tk + (size_t)j * row, sk, row);
            memcpy(tv + (size_t)j * row, sv, row);
        }
        float *uc = util_c + (size_t)s * k_cap;
        int32_t *ic = chunk_id + (size_t)s * k_cap;
        float ut[4096];
        if (keep > 4096) { rc = KVO_BAD_ARG; break; }
        for (int j = 0; j < keep; ++j)              /* the stored score is the raw one (a NaN stays a NaN) */
            ut[j] = all[j].src >= 0 ? uc[all[j].src] : util_new[(size_t)s * n_new_cap + (size_t)(-all[j].src - 1)];
        memcpy(kc, tk, row * (size_t)keep);
        memcpy(vc, tv, row * (size_t)keep);
        for (int j = 0; j < keep; ++j) { uc[j] = ut[j]; ic[j] = all[j].id; }
        count[s] = keep;
    }
    free(all);
    free(tk);
    free(tv);
    return rc;
}

/* Eq. 1 over a compact store: rows 0..count-1 of Kc/Vc [S,k_cap,d] (the kept
 * summaries, ascending chunk id) followed by rows 0..win_len-1 of the resident
 * raw window Kw/Vw [S,W_cap,d], a ring buffer that starts at row win_first
 * (section 3.3: only the recent window stays uncompressed; a ring lets it advance
 * without moving rows).  Same arithmetic as kvo_gated_attention.
 * causal != 0 (strict causality, section 3.2): the Tq queries are the window's
 * last Tq tokens, and query i sees the store and the window rows up to its own,
 * i.e. all rows but the last Tq - 1 - i. */
int kvo_compact_attention(int dtype, int L, int B, int H, int H_kv, int d, int win_len, int W_cap, int win_first,
                          const void *Q, int Tq, const void *Kw, const void *Vw, const void *Kc, const void *Vc,
                          const int32_t *count, int k_cap, int causal, void *O)
{
    /* the window buffer is a ring: its t-th token sits in row (win_first + t) mod W_cap */
    if (win_first < 0 || (win_first > 0 && win_first >= W_cap))
        return KVO_BAD_ARG;
    /* grouped-query heads as in kvo_attention_ext: Q, O have H heads; store, window and count H_kv */
    if (L < 1 || B < 1 || H < 1 || H_kv < 1 || H % H_kv != 0 || d < 1 || win_len < 0 || win_len > W_cap || Tq < 0 || k_cap < 0)
        return KVO_BAD_ARG;
    if (causal && Tq > win_len)
        return KVO_BAD_ARG;
    int n_max = k_cap + win_len;
    const void **kb = malloc(sizeof(void *) * (size_t)(n_max + 1));
    const void **vb = malloc(sizeof(void *) * (size_t)(n_max + 1));
    size_t *off = malloc(sizeof(size_t) * (size_t)(n_max + 1));
    double *logit = malloc(sizeof(double) * (size_t)(n_max + 1));
    double *acc = malloc(sizeof(double) * (size_t)d);
    int rc = KVO_OK;
    size_t S = (size_t)L * B * H;
    int G = H / H_kv;
    for (size_t sq = 0; sq < S; ++sq) {
        size_t s = (sq / H) * H_kv + (sq % H) / G;       /* the key-value head this query head reads */
        int m = count[s], n = 0;
        if (m < 0 || m > k_cap) { rc = KVO_BAD_ARG; break; }
        for (int j = 0; j < m; ++j) { kb[n] = Kc; vb[n] = Vc; off[n] = (s * k_cap + (size_t)j) * d; ++n; }
        for (int t = 0; t < win_len; ++t) {
            kb[n] = Kw; vb[n] = Vw; off[n] = (s * W_cap + (size_t)((win_first + t) % W_cap)) * d; ++n;
        }
        for (int i = 0; i < Tq; ++i) {
            size_t qo = (sq * Tq + i) * d;
            attend_rows(dtype, d, Q, qo, kb, vb, off, causal ? n - (Tq - 1 - i) : n, O, qo, logit, acc, NULL);
        }
    }
    free(kb);
    free(vb);
    free(off);
    free(logit);
    free(acc);
    return rc;
}

/* Grouped-query heads and causal frames (section 4.1 names grouped-query
 * attention with fewer key-value heads than query heads; section 3.2 states
 * strict causality).  Readings: query head h reads the cache, summaries and kept
 * set of key-value head h / (H / H_kv); with causal != 0 the Tq queries ARE the
 * last Tq cached tokens, query i sitting at position T - Tq + i, and it sees the
 * kept summaries (all older than the window) and raw tokens up to and including
 * its own position only.  gated == 0: the dense baseline over tokens 0 .. (own
 * position or T-1).
 *   Q, O [L,B,H,Tq,d];  K, V [L,B,H_kv,T_cap,d];  Kbar, Vbar [L,B,H_kv,N_cap,d];
 *   idx [L,B,H_kv,k_cap];  count [L,B,H_kv]
 * Needs H % H_kv == 0 and, when causal, Tq <= number of raw rows attended. */
int kvo_attention_ext(int dtype, int L, int B, int H, int H_kv, int d, int T, int T_cap, int C, int N_cap,
                      int W, int gated, int causal, const void *Q, int Tq, const void *K, const void *V,
                      const void *Kbar, const void *Vbar, const int32_t *idx, const int32_t *count,
                      int k_cap, void *O)
{
    if (L < 1 || B < 1 || H < 1 || H_kv < 1 || H % H_kv != 0 || d < 1 || C < 1 || T < 0 || T > T_cap ||
        W < 0 || Tq < 0 || k_cap < 0)
        return KVO_BAD_ARG;
    int n_cand = gated ? (T > W ? T - W : 0) / C : 0;
    int win0 = n_cand * C;
    if (causal && Tq > T - win0)
        return KVO_BAD_ARG;
    int n_max = (gated ? k_cap : 0) + (T - win0);
    const void **kb = malloc(sizeof(void *) * (size_t)(n_max + 1));
    const void **vb = malloc(sizeof(void *) * (size_t)(n_max + 1));
    size_t *off = malloc(sizeof(size_t) * (size_t)(n_max + 1));
    double *logit = malloc(sizeof(double) * (size_t)(n_max + 1));
    double *acc = malloc(sizeof(double) * (size_t)d);
    int rc = KVO_OK, G = H / H_kv;
    for (int l = 0; l < L && rc == KVO_OK; ++l)
        for (int b = 0; b < B && rc == KVO_OK; ++b)
            for (int h = 0; h < H && rc == KVO_OK; ++h) {
                size_t sq = ((size_t)l * B + b) * H + h;
                size_t sk = ((size_t)l * B + b) * H_kv + (size_t)(h / G);
                int n = 0;
                if (gated) {
                    int m = count[sk];
                    if (m < 0 || m > k_cap) { rc = KVO_BAD_ARG; break; }
                    for (int i = 0; i < m; ++i) {
                        int c = idx[sk * k_cap + i];
                        if (c < 0 || c >= n_cand || c >= N_cap) { rc = KVO_BAD_ARG; break; }
                        kb[n] = Kbar; vb[n] = Vbar; off[n] = (sk * N_cap + (size_t)c) * d; ++n;
                    }
                    if (rc != KVO_OK) break;
                }
                for (int t = win0; t < T; ++t) { kb[n] = K; vb[n] = V; off[n] = (sk * T_cap + (size_t)t) * d; ++n; }
                for (int i = 0; i < Tq; ++i) {
                    size_t qo = (sq * Tq + i) * d;
                    int n_i = causal ? n - (Tq - 1 - i) : n;     /* rows after the query's own token are hidden */
                    attend_rows(dtype, d, Q, qo, kb, vb, off, n_i, O, qo, logit, acc, NULL);
                }
            }
    free(kb);
    free(vb);
    free(off);
    free(logit);
    free(acc);
    return rc;
}

/* Dense baseline: Eq. 1 over raw tokens 0 .. T-1 of the full cache. */
int kvo_dense_attention(int dtype, int L, int B, int H, int d, int T, int T_cap, const void *Q,
                        int Tq, const void *K, const void *V, void *O, double *probs,
                        int probs_stride)
{
    if (L < 1 || B < 1 || H < 1 || d < 1 || T < 0 || T > T_cap || Tq < 0)
        return KVO_BAD_ARG;
    const void **kb = malloc(sizeof(void *) * (size_t)(T + 1));
    const void **vb = malloc(sizeof(void *) * (size_t)(T + 1));
    size_t *off = malloc(sizeof(size_t) * (size_t)(T + 1));
    double *logit = malloc(sizeof(double) * (size_t)(T + 1));
    double *acc = malloc(sizeof(double) * (size_t)d);
    size_t S = (size_t)L * B * H;
    for (size_t s = 0; s < S; ++s) {
        for (int t = 0; t < T; ++t) {
            kb[t] = K;
            vb[t] = V;
            off[t] = (s * T_cap + (size_t)t) * d;
        }
        for (int i = 0; i < Tq; ++i) {
            size_t qo = (s * Tq + i) * d;
            attend_rows(dtype, d, Q, qo, kb, vb, off, T, O, qo, logit, acc,
                        probs ? probs + (s * Tq + i) * (size_t)probs_stride : NULL);
        }
    }
    free(kb);
    free(vb);
    free(off);
    free(logit);
    free(acc);
    return KVO_OK;
}

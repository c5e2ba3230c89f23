/*
 * kvev — RNN-gated chunked KV-cache decode attention for AMD MI355X (gfx950).
 *
 * C ABI of the per-layer decode step of KV-Efficient VLA (arXiv 2509.21354):
 * the history KV cache is cut into fixed-length chunks, each chunk is pooled
 * into one summary key/value by a small MLP, an LSTM scores the summaries, the
 * top-k chunks are kept, and the new queries attend over the kept summaries
 * plus the raw recent window.  A full-cache attention entry point serves as
 * the baseline the method is compared with.
 *
 * Conventions (all entry points)
 *   - Every function returns an int status (KVEV_OK = 0) and never throws.
 *   - Arguments are validated on the host before any HIP call; a failed
 *     validation enqueues nothing.
 *   - Work is enqueued asynchronously on `stream` (a hipStream_t passed as
 *     void*, NULL = the default stream).  The library never allocates, frees
 *     or synchronises: the caller owns every buffer, including scratch, whose
 *     size kvev_workspace_bytes() reports.
 *   - `kvev_shape`, `kvev_mlp_w`, `kvev_lstm_w` are HOST structs; every other
 *     pointer is a DEVICE pointer, 16-byte aligned, row-major, contiguous.
 *   - Results are deterministic: same inputs, same bits (no float atomics).
 *
 * Symbols follow the paper: C chunk length, W raw recent window, d_sum
 * aggregator hidden width, d_g gate hidden width, n' = W + M attended rows.
 * Derived: N = floor(T/C) completed chunks, N_cand = floor(max(0,T-W)/C)
 * candidate chunks (those that lie wholly outside the window),
 * win0 = N_cand*C first raw-window token.
 */
#ifndef KVEV_H
#define KVEV_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

enum { KVEV_OK = 0, KVEV_ERR_INVALID_ARG = 1, KVEV_ERR_UNSUPPORTED = 2, KVEV_ERR_WORKSPACE = 3,
       KVEV_ERR_HIP = 4, KVEV_ERR_STATIC_SCRATCH = 5 };
enum { KVEV_F32 = 0, KVEV_BF16 = 1 };           /* storage type of Q/K/V, summaries, weights */
enum { KVEV_POOL_MEAN = 0, KVEV_POOL_MLP = 1, KVEV_POOL_MAX = 2, KVEV_POOL_TOKEN_MLP = 3 };
enum { KVEV_SELECT_TOPK = 0, KVEV_SELECT_THRESHOLD = 1 };
enum { KVEV_OP_CHUNK_POOL = 0, KVEV_OP_LSTM_GATE = 1, KVEV_OP_SELECT = 2,
       KVEV_OP_GATED_ATTENTION = 3, KVEV_OP_DENSE_ATTENTION = 4, KVEV_OP_COMPACT_ATTENTION = 5,
       KVEV_OP_LSTM_PREPARE = 6, KVEV_OP_LSTM_GATE_PREPARED = 7 };

/* Problem shape.  L layers are batched in one call; a "sequence" is one
 * (layer, batch row, head) triple, S = L*B*H of them, each independent.
 * T tokens are valid out of T_cap allocated per sequence; N_cap summary rows
 * are allocated per sequence (N_cap >= floor(T/C)).
 * With H_kv key-value heads (H_kv divides H; section 4.1 names grouped-query
 * attention) the caches, summaries, gate state, scores and kept sets exist per
 * (layer, batch row, KV head), i.e. every [L,B,H,...] below except Q and O reads
 * [L,B,H_kv,...], and query head h attends the cache of KV head h / (H / H_kv).
 * Supported: d in {64, 128}; dtype KVEV_F32 or KVEV_BF16; any C, W, d_sum, d_g
 * >= 1 (bf16 with d_sum % 32 == 0 and d_g % 64 == 0 takes the MFMA kernels). */
typedef struct {
    int32_t L, B, H, d;
    int32_t T, T_cap;
    int32_t C, N_cap;
    int32_t W;
    int32_t d_sum, d_g;
    int32_t dtype;
    int32_t H_kv;      /* key-value heads (grouped-query attention); 0 means H */
} kvev_shape;

/* Aggregator MLP of Eq. 2, one set per layer (shared by batch rows and heads),
 * in the storage dtype, row-major [out][in]:
 * W1 [L,d_sum,d]  b1 [L,d_sum]  W2 [L,d,d_sum]  b2 [L,d]. */
typedef struct { const void *W1, *b1, *W2, *b2; } kvev_mlp_w;

/* LSTM gate of Eq. 3, one set per layer, storage dtype, gate row blocks in
 * the order i, f, g, o:
 * W_ih [L,4d_g,2d] (columns: Kbar first, then Vbar)  W_hh [L,4d_g,d_g]
 * b_ih, b_hh [L,4d_g]   scalar utility head  w_s [L,d_g]  b_s [L]. */
typedef struct { const void *W_ih, *W_hh, *b_ih, *b_hh, *w_s, *b_s; } kvev_lstm_w;

/* Eq. 2 (chunk aggregation; section 3.3: a chunk is aggregated once it is
 * complete, by a two-layer MLP).  For every sequence and every chunk c in
 * [chunk_begin, chunk_end):  xbar = mean of the chunk's C keys;
 * Kbar[c] = W2 * GELU(W1 * xbar + b1) + b2 with the K weights (exact erf GELU),
 * the same for V with the V weights; KVEV_POOL_MEAN stores xbar itself and
 * KVEV_POOL_MAX (the "pooling" alternative section 3 names) the element-wise
 * maximum of the chunk's C rows, exactly (wK, wV may then be NULL; inputs are
 * taken to be free of NaN).  KVEV_POOL_TOKEN_MLP applies the same MLP to every
 * token of the chunk and averages the C outputs (section 3's multi-layer
 * perceptron aggregator read as a per-token network under a symmetric reduction):
 * Kbar[c] = (1/C) sum_j [ W2 * GELU(W1 * k_j + b1) + b2 ].  Mean, both layers and GELU
 * are evaluated in fp32-grade arithmetic; each summary element is rounded once to the
 * storage dtype.
 *   K, V        [L,B,H,T_cap,d]   read: tokens [chunk_begin*C, chunk_end*C)
 *   Kbar, Vbar  [L,B,H,N_cap,d]   written: rows [chunk_begin, chunk_end) only
 * Needs 0 <= chunk_begin <= chunk_end <= floor(T/C) <= N_cap.  Workspace:
 * optional.  With kvev_workspace_bytes(KVEV_OP_CHUNK_POOL, ...) bytes (16-byte
 * aligned) a large KVEV_POOL_MLP call first re-lays the MLP weights there for
 * the matrix cores and is a few percent faster; the results are the same bits.
 * ws may be NULL or smaller: then the weights are read as they are.  The first
 * 256 bytes of ws are never touched.  Errors: INVALID_ARG for null/misaligned pointers, a bad
 * range, more than 2^30 (sequence, chunk) pairs in one call or more than
 * 2^31 - 1 summary rows in Kbar; UNSUPPORTED for d, dtype or pool_mode outside
 * the lists above. */
int kvev_chunk_pool(const kvev_shape *shape, const void *K, const void *V, int pool_mode,
                    const kvev_mlp_w *wK, const kvev_mlp_w *wV, int chunk_begin, int chunk_end,
                    void *Kbar, void *Vbar, void *ws, size_t ws_bytes, void *stream);

/* Eq. 3 (recurrent gate).  For every sequence, for t in [chunk_begin,
 * chunk_end) in order: x_t = [Kbar_t ; Vbar_t]; standard LSTM cell
 *   (i,f,g,o) = W_ih x_t + b_ih + W_hh h_{t-1} + b_hh;  c_t = s(f) c_{t-1} + s(i) tanh(g);
 *   h_t = s(o) tanh(c_t);   util_t = w_s . h_t + b_s;   gate_t = s(util_t) in [0,1].
 * State, pre-activations and scores are fp32.
 *   h, c        [L,B,H,d_g] fp32, in/out: a call with chunk_begin == 0 starts
 *               from the zero state h_0 = c_0 = 0 whatever they hold (nothing
 *               to clear), and leaves the state after chunk_end - 1 in them;
 *               pass them back unchanged to continue the stream
 *               (chunk_begin > 0)
 *   util, gate  [L,B,H,N_cap] fp32, entries [chunk_begin, chunk_end) written
 * Needs 0 <= chunk_begin <= chunk_end <= N_cap; h and c 16-byte aligned.
 * Workspace: see kvev_workspace_bytes: a 256-byte head, the weights re-laid for
 * the matrix cores (written by every call; kvev_lstm_gate_prepared takes them
 * from the caller instead), and for most shapes fp32 input projections of a
 * block of steps: any size from one step's worth up is accepted, smaller blocks
 * mean more launches.  Launches of bf16 storage with d_g = 256 that give every
 * compute unit a group of 32 sequences, and with d_g = 512 and more than 16
 * sequences per layer, run as one kernel (at d_g = 512 once per compute
 * units / 4 groups of 32 sequences) and keep no projections at all.  Calls that share a workspace
 * must not overlap (it also carries what the workgroups of one launch
 * exchange).
 * Status word: the first int32 of the workspace.  Small launches (bf16; d_g =
 * 256 or 512 with at most one group of 16 sequences per 2 compute units of the
 * device, or the groups of 32 at d_g = 512 above) run each group on two or four
 * cooperating workgroups, which wait for each other's data with a bounded
 * number of polls.  Should the bound ever
 * expire (the GPU held by other work for seconds), the launch still ends
 * normally, its util, gate and c entries are NaN, and it stores 1 in the status
 * word.  The library never clears the word: fill the workspace with zeros
 * before its first use and read the word whenever you synchronise; non-zero
 * means that the scores of some call since then are not to be used.
 * Errors: INVALID_ARG, UNSUPPORTED as above; WORKSPACE if ws is too small. */
int kvev_lstm_gate(const kvev_shape *shape, const void *Kbar, const void *Vbar,
                   const kvev_lstm_w *w, int chunk_begin, int chunk_end, float *h, float *c,
                   float *util, float *gate, void *ws, size_t ws_bytes, void *stream);

/* The weights of Eq. 3 in the form the matrix-core kernels of the gate read:
 * W_ih and W_hh in fragment order, W_hh scaled by a per-layer power of two and
 * converted so that its products with the two-term state are exact.  The
 * result depends on the weights alone, so a caller whose weights do not change
 * between decode steps prepares them once and passes `packed` to every
 * kvev_lstm_gate_prepared call, which then skips this work (two launches per
 * call).  `packed` is caller-owned device memory of at least
 * kvev_workspace_bytes(KVEV_OP_LSTM_PREPARE, shape, 0, 0) bytes (0 for shapes
 * the matrix-core kernels do not take: then the call does nothing and `packed`
 * may be NULL), 16-byte aligned; only L, d, d_g and dtype of `shape` are used
 * beyond validation.  Errors: INVALID_ARG, UNSUPPORTED as kvev_lstm_gate;
 * WORKSPACE for a missing, misaligned or short `packed`. */
int kvev_lstm_prepare(const kvev_shape *shape, const kvev_lstm_w *w, void *packed, size_t packed_bytes,
                      void *stream);

/* kvev_lstm_gate (Eq. 3) with weights prepared by kvev_lstm_prepare for the
 * same shape and `w`: same results bit for bit.  `w` is still read (biases and
 * the utility head).  Workspace: kvev_workspace_bytes(KVEV_OP_LSTM_GATE_PREPARED,
 * ...), which lacks the packed weights; status word as kvev_lstm_gate. */
int kvev_lstm_gate_prepared(const kvev_shape *shape, const void *Kbar, const void *Vbar,
                            const kvev_lstm_w *w, const void *packed, size_t packed_bytes,
                            int chunk_begin, int chunk_end, float *h, float *c, float *util, float *gate,
                            void *ws, size_t ws_bytes, void *stream);

/* Retention.  Candidates are chunks 0 .. N_cand-1.
 * KVEV_SELECT_TOPK: keep the min(k, N_cand) candidates of largest util, ties
 * going to the lower index, a NaN counting as minus infinity (`gate`, `tau`
 * ignored; gate may be NULL).  KVEV_SELECT_THRESHOLD (the literal rule of
 * section 3.2): keep candidate c iff gate[c] >= tau (`k` ignored, util may be
 * NULL; needs k_cap >= N_cand).
 *   idx    [L,B,H,k_cap] int32: kept chunk indices, ascending, in entries
 *          [0, count); the rest is left untouched
 *   count  [L,B,H] int32
 * Integer output is exact.  Needs k >= 0, k_cap >= min(k, N_cand),
 * N_cand <= N_cap and N_cand <= 16384.  No workspace. */
int kvev_select(const kvev_shape *shape, const float *util, const float *gate, int mode, int k,
                float tau, int k_cap, int32_t *idx, int32_t *count, void *stream);

/* Eq. 1 over the union of kept summaries and the raw window (section 3.3,
 * n' = W + M).  For every sequence and each of its Tq queries the attended
 * rows are Kbar[idx[0..count)] / Vbar[...] followed by the raw tokens
 * win0 .. T-1 of K / V; O = softmax(q . keys^T / sqrt(d)) . values with fp32
 * scores, softmax and accumulation, rounded once to the storage dtype.  (One
 * more rounding on the matrix-core path, which bf16 storage takes when a
 * key-value sequence has 16 or more queries: the softmax weights enter the
 * product with the values rounded to bf16, 8 significant bits, while the
 * normaliser sums them unrounded; the result stays within the bf16 bar, see the
 * measured figures in the parity report of the tests.)  With
 * causal == 0 the Tq queries see the whole cache and not each other; with
 * causal == 1 (strict causality, section 3.2) they ARE the last Tq cached tokens,
 * query i at position T - Tq + i, and each sees the kept summaries and the raw
 * tokens up to and including its own position (needs Tq <= T - win0).
 * count == 0 (e.g. T <= W) is valid: the raw tokens alone are attended; no
 * rows at all gives O = 0.
 *   Q, O  [L,B,H,Tq,d]    idx [L,B,H,k_cap]   count [L,B,H], 0 <= count <= k_cap,
 *   every idx entry below count in [0, N_cand) (not checked: device data).
 * Workspace: see kvev_workspace_bytes (0 when the launch needs no split).  It
 * begins with one int32 ticket per (sequence, query group), followed by the
 * split partials.  The tickets must be zero when a call starts and every call
 * leaves them zero: fill a fresh workspace with zeros once, and again only
 * after lending it to something else (kvev_lstm_gate writes all over its own).
 * Calls that share a workspace must not overlap. */
int kvev_gated_attention(const kvev_shape *shape, const void *Q, int Tq, const void *K,
                         const void *V, const void *Kbar, const void *Vbar, const int32_t *idx,
                         const int32_t *count, int k_cap, int causal, void *O, void *ws,
                         size_t ws_bytes, void *stream);

/* kvev_gated_attention for callers that cannot allocate device memory or carry a
 * scratch buffer of their own: code recorded into a HIP graph, tight serving
 * loops, harnesses that forbid allocation.  Same arguments, arithmetic and
 * results as kvev_gated_attention, minus the workspace: the split partials and
 * tickets live in an array of KVEV_STATIC_SCRATCH_BYTES that is part of the
 * library's code object (one copy per GPU, held until the process ends).  The
 * call allocates nothing and frees nothing.  Every call on a GPU uses that
 * GPU's one array, whatever its stream: calls that may overlap in time on one
 * GPU race and must be ordered by the caller.  The first call on a device looks
 * up the array's address (not a stream operation: make that first call outside
 * stream capture).  Errors as kvev_gated_attention, and KVEV_ERR_STATIC_SCRATCH
 * when the shape wants more scratch than the array holds
 * (kvev_workspace_bytes(KVEV_OP_GATED_ATTENTION, ...) tells how much). */
#define KVEV_STATIC_SCRATCH_BYTES (4u << 20)
int kvev_gated_attention_static(const kvev_shape *shape, const void *Q, int Tq, const void *K,
                                const void *V, const void *Kbar, const void *Vbar, const int32_t *idx,
                                const int32_t *count, int k_cap, int causal, void *O, void *stream);

/* Eq. 1 over the whole cache, tokens 0 .. T-1: the baseline whose O(n) cost
 * per new token the method removes (section 2, "Transformer Attention").
 * Same layouts, arithmetic and workspace rule as kvev_gated_attention. */
int kvev_dense_attention(const kvev_shape *shape, const void *Q, int Tq, const void *K,
                         const void *V, int causal, void *O, void *ws, size_t ws_bytes,
                         void *stream);

/* Physical eviction (sections 3.2-3.3: a chunk that is not kept is discarded;
 * the end of section 3.3: the cache shrinks by n / (W + M)).  Per sequence a compact store
 * holds at most k kept summaries, ascending by chunk id:
 *   Kc, Vc    [L,B,H,k_cap,d]  storage dtype     chunk_id [L,B,H,k_cap] int32
 *   util_c    [L,B,H,k_cap]    fp32 scores        count    [L,B,H] int32 (in/out;
 *                                                  zero it before the first call)
 * This call merges n_new freshly scored chunks, ids first_chunk .. first_chunk +
 * n_new - 1 (summaries in rows 0 .. n_new-1 of Kbar_new, Vbar_new
 * [L,B,H,n_new_cap,d], utilities util_new [L,B,H,n_new_cap]) and keeps the
 * min(k, count + n_new) best under the order of KVEV_SELECT_TOPK (utility
 * descending, NaN as minus infinity, ties to the lower id), in place.  Because
 * the score of an old chunk never changes, the store always equals the top-k
 * over every chunk merged so far, and everything else (the chunk's raw tokens
 * once it left the window, its summary) can be freed by the caller.  Rows and
 * integers are copied exactly.  first_chunk must exceed every id in the store
 * (ids arrive in temporal order; device data, not checked).  Only L, B, H, d and
 * dtype of `shape` are used.  Needs 0 <= k <= k_cap, 0 <= n_new <= n_new_cap,
 * k_cap + n_new <= 4000.  No workspace. */
int kvev_retain(const kvev_shape *shape, int k, int k_cap, const void *Kbar_new, const void *Vbar_new,
                const float *util_new, int n_new_cap, int first_chunk, int n_new, void *Kc, void *Vc,
                int32_t *chunk_id, float *util_c, int32_t *count, void *stream);

/* Eq. 1 over what is resident after eviction: rows 0 .. count-1 of the compact
 * store Kc / Vc followed by the raw window.  Here `shape` describes the resident
 * raw buffer: Kw, Vw are [L,B,H,T_cap,d], used as a ring: the window's t-th
 * token, t = 0 .. T-1, sits in row (win_first + t) mod T_cap, so a caller appends
 * new tokens behind the last one and advances win_first when chunks leave the
 * window, without moving rows (win_first = 0: rows 0 .. T-1; needs
 * 0 <= win_first < T_cap; C, W, N_cap of the shape are not used).  Same arithmetic, row order
 * and rounding as kvev_gated_attention over the same rows, so the two give the
 * same bits.  causal as in kvev_gated_attention: 1 = the Tq queries are the
 * window's last Tq tokens (needs Tq <= T), each seeing the store and the window
 * rows up to its own.  Workspace: kvev_workspace_bytes(KVEV_OP_COMPACT_ATTENTION,
 * shape, Tq, k_cap). */
int kvev_compact_attention(const kvev_shape *shape, const void *Q, int Tq, const void *Kw, const void *Vw,
                           int win_first, const void *Kc, const void *Vc, const int32_t *count, int k_cap,
                           int causal, void *O, void *ws, size_t ws_bytes, void *stream);

/* Scratch bytes that `op` (a KVEV_OP_* value) wants for this shape
 * (KVEV_OP_LSTM_PREPARE: the size of the packed weights).  `n` is Tq
 * for the attention ops and chunk_end - chunk_begin for pool / gate; k_cap is
 * used by KVEV_OP_GATED_ATTENTION and KVEV_OP_COMPACT_ATTENTION only.  Returns 0 when none is needed or the
 * arguments are invalid. */
size_t kvev_workspace_bytes(int op, const kvev_shape *shape, int n, int k_cap);

/* Static description of a status code. */
const char *kvev_status_string(int status);

/* Last HIP error text seen by this thread's most recent KVEV_ERR_HIP return. */
const char *kvev_last_hip_error(void);

/* Library version, major*10000 + minor*100 + patch. */
int kvev_version(void);

#ifdef __cplusplus
}
#endif
#endif /* KVEV_H */

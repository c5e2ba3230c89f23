// C-ABI layer: argument validation (host only, before any HIP call), launch
// planning (split counts, workspace carving) and dispatch to the kernels.
#include <math.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include <algorithm>
#include <atomic>
#include <mutex>

#include "../../include/kvev_test_hooks.h"
#include "common.hpp"
#include "kernels.hpp"

namespace kvev {

static thread_local char g_hip_err[256] = "";

static int hip_fail(hipError_t e)
{
    snprintf(g_hip_err, sizeof g_hip_err, "%s", hipGetErrorString(e));
    return KVEV_ERR_HIP;
}

static bool aligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

// 0 when the shape itself is usable, else a status.
static int check_shape(const kvev_shape *sh, bool chunked = true)
{
    if (!sh) return KVEV_ERR_INVALID_ARG;
    if (sh->L < 1 || sh->B < 1 || sh->H < 1 || sh->d < 1 || sh->C < 1 || sh->T < 0 || sh->T_cap < 1 ||
        sh->N_cap < 0 || sh->W < 0 || sh->d_sum < 1 || sh->d_g < 1)
        return KVEV_ERR_INVALID_ARG;
    if (sh->T > sh->T_cap || (chunked && sh->T / sh->C > sh->N_cap)) return KVEV_ERR_INVALID_ARG;
    if ((int64_t)sh->L * sh->B * sh->H > (int64_t)1 << 24) return KVEV_ERR_INVALID_ARG;
    if (sh->H_kv < 0 || (sh->H_kv > 0 && sh->H % sh->H_kv != 0)) return KVEV_ERR_INVALID_ARG;
    if (sh->dtype != KVEV_F32 && sh->dtype != KVEV_BF16) return KVEV_ERR_UNSUPPORTED;
    if (sh->d != 64 && sh->d != 128) return KVEV_ERR_UNSUPPORTED;
    return KVEV_OK;
}

// key-value heads: the caches, summaries, gate state and kept sets exist per (layer, batch row, KV head)
static int kv_heads(const kvev_shape *sh) { return sh->H_kv > 0 ? sh->H_kv : sh->H; }

static int n_cand_of(const kvev_shape *sh) { return (sh->T > sh->W ? sh->T - sh->W : 0) / sh->C; }

// ---- attention planning ---------------------------------------------------
// Rows are split across workgroups until the launch has a few workgroups per
// compute unit; the splits of a query are merged inside the same launch (the
// last workgroup to arrive does it), so a split only has to be worth a
// workgroup's own start-up: one or two rounds of row loads.
// Scratch: one ticket (int32) per (key-value sequence, query group), padded to
// 256 bytes, then the split partials.
struct AttnPlan { int nsplit, rows_per_split; size_t ticket_bytes, ws_bytes; };

static int env_int(const char *name, int dflt)
{
    const char *v = getenv(name);
    return v && *v ? atoi(v) : dflt;
}
// Tuning knobs (environment, read once; unset = the rule below): workgroups wanted per launch and the smallest
// run of raw rows worth a workgroup.  The rule: with fewer key-value units than compute units the launch is filled
// with up to one 16-wave workgroup per compute unit and runs down to 64 rows (one batch of a 4-wave workgroup);
// with more, four 4-wave workgroups per compute unit and runs of at least 512 rows.
static const int g_attn_target_blocks = env_int("KVEV_ATTN_TARGET_BLOCKS", -1);
static const int g_attn_min_rows = env_int("KVEV_ATTN_MIN_ROWS", -1);
// large pooling launches write their summaries once per 2^shift ticks of the 100 MHz real-time counter: 8192 ticks
// (82 us) with the MLP, 4096 without (tiles complete faster; a slot should not outlast the two tiles a thread holds back)
static const int g_pool_flush_shift_env = env_int("KVEV_POOL_FLUSH_SHIFT", -1);
static int pool_flush_shift(int pool_mode)
{
    if (g_pool_flush_shift_env >= 0) return std::min(std::max(g_pool_flush_shift_env, 6), 40);
    return pool_mode == KVEV_POOL_MLP ? 13 : 12;
}

static AttnPlan plan_attn(const kvev_shape *sh, int Tq, int n_rows)
{
    AttnPlan p;
    // one workgroup serves up to 4 of the queries that share a key-value sequence
    const int64_t R = (int64_t)(sh->H / kv_heads(sh)) * (Tq > 0 ? Tq : 1);
    const int64_t qgroups = R >= 4 ? (R + 3) / 4 : R >= 2 ? (R + 1) / 2 : 1;
    const int64_t units = (int64_t)sh->L * sh->B * kv_heads(sh) * qgroups;
    const int64_t sq = (int64_t)sh->L * sh->B * sh->H * (Tq > 0 ? Tq : 1);
    const bool few = units < 256;
    const int target = g_attn_target_blocks > 0 ? g_attn_target_blocks : few ? 256 : 1024;
    const int min_rows = g_attn_min_rows > 0 ? g_attn_min_rows : few ? 64 : 512;
    int64_t want = (target + units - 1) / units;
    int64_t most = (n_rows + min_rows - 1) / min_rows;
    if (want > most) want = most;
    if (want > KVEV_ATTN_MAX_SPLIT) want = KVEV_ATTN_MAX_SPLIT;
    if (want < 1) want = 1;
    int rps = (int)((n_rows + want - 1) / want);
    rps = (rps + 15) / 16 * 16;
    if (rps < 16) rps = 16;
    p.rows_per_split = rps;
    p.nsplit = n_rows > 0 ? (n_rows + rps - 1) / rps : 1;
    p.ticket_bytes = ((size_t)units * sizeof(int32_t) + 255) / 256 * 256;
    p.ws_bytes = p.nsplit > 1 ? p.ticket_bytes + (size_t)sq * p.nsplit * (sh->d + 2) * sizeof(float) : 0;
    return p;
}

// single-query launches that read more than this take their rows with the non-temporal hint
constexpr size_t kStreamBytesDefault = (size_t)256 << 20;     // what the memory-side cache holds
static std::atomic<size_t> g_stream_bytes{kStreamBytesDefault};

// a frame of queries per key-value sequence (all heads of a group count) goes to the matrix cores
static bool attn_takes_mq(const kvev_shape *sh, int Tq)
{
    return sh->dtype == KVEV_BF16 && (int64_t)(sh->H / kv_heads(sh)) * Tq >= 16;
}

// ---- scratch that the library holds itself (kvev_gated_attention_static) ----
// One array per GPU, there from the moment the code object is loaded until the process ends.  `scratch` names it for
// the device code only: host code reaches its memory through the address that hipGetSymbolAddress reports for the
// current device, looked up once per device and kept.
constexpr size_t kStaticScratchBytes = KVEV_STATIC_SCRATCH_BYTES;
static __device__ __align__(256) __attribute__((used)) unsigned char scratch[kStaticScratchBytes];
constexpr int kMaxDevices = 64;
static std::mutex g_scratch_mutex;
static void *g_scratch_ptr[kMaxDevices];        // device address of `scratch` on device i, or null: not looked up yet

static int static_scratch(void **out)
{
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return hip_fail(e);
    if (dev < 0 || dev >= kMaxDevices) return KVEV_ERR_UNSUPPORTED;
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[dev]) {
        void *ptr = nullptr;
        e = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch));
        if (e != hipSuccess) return hip_fail(e);
        if (!ptr) return hip_fail(hipErrorInvalidSymbol);
        g_scratch_ptr[dev] = ptr;
    }
    *out = g_scratch_ptr[dev];
    return KVEV_OK;
}

// zeroes n16 16-byte words (a kernel, not hipMemsetAsync: the call may be recorded into a HIP graph)
__global__ __launch_bounds__(256) void fill_zero_kernel(uint4 *p, size_t n16)
{
    const size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
    if (i < n16) p[i] = make_uint4(0u, 0u, 0u, 0u);
}

static int attention_common(const kvev_shape *sh, const void *Q, int Tq, const void *K, const void *V,
                            const void *Kbar, const void *Vbar, const int32_t *idx, const int32_t *count,
                            int k_cap, int gated, int causal, void *O, void *ws, size_t ws_bytes,
                            void *stream, int ring_first = 0, bool static_ws = false)
{
    int rc = check_shape(sh, gated != 2);     // a compact store has no chunk grid over the raw buffer
    if (rc) return rc;
    if (!Q || !K || !V || !O || Tq < 0 || !aligned16(Q) || !aligned16(K) || !aligned16(V) || !aligned16(O))
        return KVEV_ERR_INVALID_ARG;
    // gated == 2: compact store (no index list, N_cap = k_cap rows per sequence, raw rows 0 .. T-1)
    const bool compact = gated == 2;
    if (gated && (!Kbar || !Vbar || (!idx && !compact) || !count || k_cap < 0 || !aligned16(Kbar) || !aligned16(Vbar)))
        return KVEV_ERR_INVALID_ARG;
    if (gated && !compact && k_cap > 0 && sh->N_cap < 1) return KVEV_ERR_INVALID_ARG;
    if (causal != 0 && causal != 1) return KVEV_ERR_INVALID_ARG;
    if (ring_first < 0 || (ring_first > 0 && ring_first >= sh->T_cap)) return KVEV_ERR_INVALID_ARG;
    if (Tq == 0) return KVEV_OK;
    if ((int64_t)sh->L * sh->B * sh->H * Tq > (int64_t)1 << 26) return KVEV_ERR_INVALID_ARG;

    const int ncand = n_cand_of(sh);
    const int win0 = gated == 1 ? ncand * sh->C : 0;
    const int kmax = compact ? k_cap : gated ? (k_cap < ncand ? k_cap : ncand) : 0;
    const int n_rows = kmax + sh->T - win0;
    if (causal && Tq > sh->T - win0) return KVEV_ERR_INVALID_ARG;      // the frame must lie inside the raw rows
    // a frame of queries on bf16 storage goes to the matrix-core kernel (no split, no scratch)
    const bool mq = attn_takes_mq(sh, Tq);
    const AttnPlan p = mq ? AttnPlan{1, n_rows, 0, 0} : plan_attn(sh, Tq, sh->T - win0);     // (split by the raw rows)
    if (static_ws) {
        // the library's own array stands in for the caller's scratch; its tickets are cleared on every call, so
        // nothing is assumed about what the call before left there
        if (p.ws_bytes > kStaticScratchBytes) return KVEV_ERR_STATIC_SCRATCH;
        if (p.ws_bytes > 0) {
            rc = static_scratch(&ws);
            if (rc) return rc;
            ws_bytes = kStaticScratchBytes;
            const size_t n16 = p.ticket_bytes / 16;
            hipLaunchKernelGGL(fill_zero_kernel, dim3((unsigned)((n16 + 255) / 256)), dim3(256), 0,
                               static_cast<hipStream_t>(stream), static_cast<uint4 *>(ws), n16);
        }
    }
    if (p.ws_bytes > 0 && (!ws || ws_bytes < p.ws_bytes || !aligned16(ws))) return KVEV_ERR_WORKSPACE;

    AttnArgs a;
    a.Q = Q; a.K = K; a.V = V; a.Kbar = Kbar; a.Vbar = Vbar; a.idx = idx; a.count = count; a.O = O;
    a.tickets = p.nsplit > 1 ? static_cast<int32_t *>(ws) : nullptr;
    a.part = p.nsplit > 1 ? reinterpret_cast<float *>(static_cast<unsigned char *>(ws) + p.ticket_bytes) : nullptr;
    a.S = sh->L * sh->B * kv_heads(sh); a.Tq = Tq; a.d = sh->d;
    a.G = sh->H / kv_heads(sh); a.Hkv = kv_heads(sh); a.causal = causal;
    a.T = sh->T; a.T_cap = sh->T_cap; a.N_cap = compact ? k_cap : sh->N_cap; a.k_cap = k_cap;
    a.win0 = win0; a.ring_first = ring_first; a.gated = gated ? 1 : 0;
    a.nsplit = p.nsplit; a.rows_per_split = p.rows_per_split;
    // rows that no cache can hold until the next call are read with the streaming hint (256 MB: the memory-side cache)
    a.stream = (size_t)a.S * (size_t)n_rows * sh->d * 2 * (sh->dtype == KVEV_F32 ? 4 : 2) > g_stream_bytes.load(std::memory_order_relaxed) ? 1 : 0;
    a.scale_log2e = (float)(1.4426950408889634 / sqrt((double)sh->d));
    hipError_t e = mq ? launch_attn_mq(a, static_cast<hipStream_t>(stream))
                      : launch_attn_decode(a, sh->dtype, static_cast<hipStream_t>(stream));
    return e == hipSuccess ? KVEV_OK : hip_fail(e);
}

// ---- LSTM planning --------------------------------------------------------
// The matrix-core gate takes bf16 storage with d_g a multiple of 64 up to 512;
// its scratch holds, per step of a block, one fp32 pre-activation per gate row
// for every 16-sequence group (groups are padded and never straddle layers).
static bool lstm_takes_mfma(const kvev_shape *sh)
{
    return sh->dtype == KVEV_BF16 && (sh->d_g == 64 || sh->d_g == 128 || sh->d_g == 256 || sh->d_g == 512);
}

// Bound on the polls of one wait of the paired recurrence (each poll is a round trip to memory, about a
// microsecond: seconds in all), and the member whose publications are withheld; kvev_debug_pair_wait changes them.
static std::atomic<int> g_pair_spin_limit{1 << 22}, g_pair_mute{-1};

// Compute units of the current device (what decides whether the workgroups of a paired launch can all be resident);
// 256 when no device answers (argument checks and scratch queries also run on machines without a GPU).
static int device_compute_units()
{
    static std::atomic<int> cached{0};
    int n = cached.load();
    if (n > 0) return n;
    int dev = 0, v = 0;
    n = 256;
    if (hipGetDevice(&dev) == hipSuccess &&
        hipDeviceGetAttribute(&v, hipDeviceAttributeMultiprocessorCount, dev) == hipSuccess && v > 0)
        n = v;
    else
        (void)hipGetLastError();         // not an error of any launch of ours
    cached.store(n);
    return n;
}

// bf16 storage with a hidden width the 16x16x32 tiling divides: chunk pooling on the matrix cores
static bool pool_takes_mfma(const kvev_shape *sh)
{
    return sh->dtype == KVEV_BF16 && sh->d_sum % 32 == 0 && sh->d_sum <= 512;
}
// Scratch that kvev_chunk_pool can use (it works without): a 256-byte head that it never touches, so that a buffer
// which also serves the gate keeps its status word, then the MLP weights re-laid for the matrix cores.
constexpr size_t kPoolWsHead = 256;
static size_t pool_ws_bytes(const kvev_shape *sh)
{
    return pool_takes_mfma(sh) ? kPoolWsHead + pool_pack_bytes(sh->L, sh->d, sh->d_sum) : 0;
}

static long long lstm_groups(const kvev_shape *sh)
{
    return (long long)sh->L * ((sh->B * kv_heads(sh) + 15) / 16);
}

// Launches that give every compute unit a workgroup of 32 sequences take the single-kernel form at d_g = 256
// (no projections in scratch); smaller ones keep the two-kernel form, whose 16-sequence workgroups (or pairs of
// them) have the shorter step.  KVEV_LSTM_FUSED_MIN_GROUPS (groups of 16 sequences, read once) moves the border.
static const int g_lstm_fused_min_groups_default = env_int("KVEV_LSTM_FUSED_MIN_GROUPS", 257);
static std::atomic<int> g_lstm_fused_min_groups{g_lstm_fused_min_groups_default};
static bool lstm_takes_fused(const kvev_shape *sh)
{
    return lstm_takes_mfma(sh) && sh->d_g == 256 && lstm_groups(sh) >= g_lstm_fused_min_groups.load();
}

// W_hh and W_ih re-laid in MFMA fragment order sit at the front of the scratch:
// packed W_hh and W_ih (2 bytes per element), then 32 words per layer (partial maxima of |W_hh|), padded to 256 bytes
static size_t lstm_ws_weights(const kvev_shape *sh)
{
    return (size_t)sh->L * 4 * sh->d_g * ((size_t)sh->d_g + 2 * sh->d) * 2 + ((size_t)sh->L * 32 * 4 + 255) / 256 * 256;
}

// The gate's scratch: a 256-byte head (its first word is the status word), the packed weights unless the caller
// keeps them (kvev_lstm_prepare), the exchange slots of the paired recurrence where it applies, then the projections.
constexpr size_t kLstmWsHead = 256;
// KVEV_LSTM_QUAD=0 (read once) keeps d_g = 512 on pairs of workgroups where quadruples would be taken.
static const int g_lstm_quad = env_int("KVEV_LSTM_QUAD", 1);
static int lstm_split_of(const kvev_shape *sh)
{
    return lstm_takes_fused(sh) ? 0 : lstm_split(sh->d_g, sh->L, sh->B * kv_heads(sh), device_compute_units(), g_lstm_quad != 0);
}
// groups of 32 sequences that one launch of the four-workgroup kernel takes: a workgroup per compute unit at most
// (kvev_debug_lstm_quad_groups lowers it, so that a small shape walks the several-launches path)
static std::atomic<int> g_lstm_quad_groups{0};
static int lstm_quad_groups()
{
    const int forced = g_lstm_quad_groups.load(), fit = device_compute_units() / 4;
    return forced > 0 && forced < fit ? forced : (fit > 0 ? fit : 1);
}
static size_t lstm_exch_bytes(const kvev_shape *sh)
{
    return lstm_split_exch_bytes(lstm_split_of(sh), sh->d_g, sh->L, sh->B * kv_heads(sh), lstm_quad_groups());
}
static size_t lstm_ws_pack(const kvev_shape *sh, bool prepared)
{
    return lstm_takes_mfma(sh) ? kLstmWsHead + (prepared ? 0 : lstm_ws_weights(sh)) + lstm_exch_bytes(sh) : 0;
}

static size_t lstm_ws_per_step(const kvev_shape *sh)
{
    // (the single-kernel forms, d_g = 256 at scale and d_g = 512 on quadruples, keep no projections in scratch)
    if (!lstm_takes_mfma(sh) || lstm_takes_fused(sh) || lstm_split_of(sh) == 4) return 0;
    return (size_t)lstm_groups(sh) * 16 * 4 * sh->d_g * sizeof(float);
}

}  // namespace kvev

using namespace kvev;

extern "C" {

int kvev_chunk_pool(const kvev_shape *sh, const void *K, const void *V, int pool_mode, const kvev_mlp_w *wK,
                    const kvev_mlp_w *wV, int chunk_begin, int chunk_end, void *Kbar, void *Vbar, void *ws,
                    size_t ws_bytes, void *stream)
{
    int rc = check_shape(sh);
    if (rc) return rc;
    if (pool_mode < KVEV_POOL_MEAN || pool_mode > KVEV_POOL_TOKEN_MLP) return KVEV_ERR_UNSUPPORTED;
    const bool has_mlp = pool_mode == KVEV_POOL_MLP || pool_mode == KVEV_POOL_TOKEN_MLP;
    if (!K || !V || !Kbar || !Vbar || !aligned16(K) || !aligned16(V) || !aligned16(Kbar) || !aligned16(Vbar))
        return KVEV_ERR_INVALID_ARG;
    if (chunk_begin < 0 || chunk_begin > chunk_end || chunk_end > sh->T / sh->C) return KVEV_ERR_INVALID_ARG;
    if (has_mlp) {
        if (!wK || !wV) return KVEV_ERR_INVALID_ARG;
        const void *ptrs[8] = {wK->W1, wK->b1, wK->W2, wK->b2, wV->W1, wV->b1, wV->W2, wV->b2};
        for (const void *p : ptrs)
            if (!p || !aligned16(p)) return KVEV_ERR_INVALID_ARG;
        if (sizeof(float) * (16 * 2 * (size_t)sh->d + 2 * sh->d + 2 * (size_t)sh->d_sum) > 64 * 1024)
            return KVEV_ERR_UNSUPPORTED;
    }
    if (chunk_begin == chunk_end) return KVEV_OK;
    if ((int64_t)sh->L * sh->B * kv_heads(sh) * (chunk_end - chunk_begin) > (int64_t)1 << 30) return KVEV_ERR_INVALID_ARG;
    // (summary rows are indexed with 32 bits in the kernels)
    if ((int64_t)sh->L * sh->B * kv_heads(sh) * sh->N_cap > (int64_t)INT32_MAX) return KVEV_ERR_INVALID_ARG;

    PoolArgs a;
    memset(&a, 0, sizeof a);
    a.K = K; a.V = V; a.Kbar = Kbar; a.Vbar = Vbar;
    if (has_mlp) {
        a.W1K = wK->W1; a.b1K = wK->b1; a.W2K = wK->W2; a.b2K = wK->b2;
        a.W1V = wV->W1; a.b1V = wV->b1; a.W2V = wV->W2; a.b2V = wV->b2;
    }
    a.L = sh->L; a.BH = sh->B * kv_heads(sh); a.d = sh->d; a.T_cap = sh->T_cap; a.C = sh->C; a.N_cap = sh->N_cap;
    a.d_sum = sh->d_sum; a.c0 = chunk_begin; a.c1 = chunk_end; a.mode = pool_mode;
    a.compute_units = device_compute_units(); a.flush_shift = pool_flush_shift(pool_mode);
    // bf16 storage with a hidden width the 16x16x32 tiling divides goes to the matrix cores
    const bool mfma = pool_takes_mfma(sh);
    // optional scratch: room for the MLP weights in fragment order, behind a head that is left alone
    if (mfma && pool_mode == KVEV_POOL_MLP && ws && aligned16(ws) && ws_bytes >= pool_ws_bytes(sh))
        a.wpack = static_cast<unsigned char *>(ws) + kPoolWsHead;
    hipError_t e;
    if (pool_mode == KVEV_POOL_TOKEN_MLP && mfma && sh->d_sum <= 256 && pool_token_mfma_lds(sh->d, sh->d_sum) <= 160 * 1024)
        e = launch_pool_token_mfma(a, static_cast<hipStream_t>(stream));     // W1 of both sides fits in LDS
    else
        e = mfma && pool_mode != KVEV_POOL_TOKEN_MLP ? launch_pool_mfma(a, static_cast<hipStream_t>(stream))
                                                     : launch_pool_generic(a, sh->dtype, static_cast<hipStream_t>(stream));
    return e == hipSuccess ? KVEV_OK : hip_fail(e);
}

static int lstm_check_weights(const kvev_lstm_w *w)
{
    if (!w) return KVEV_ERR_INVALID_ARG;
    const void *ptrs[6] = {w->W_ih, w->W_hh, w->b_ih, w->b_hh, w->w_s, w->b_s};
    for (int i = 0; i < 6; ++i)
        if (!ptrs[i] || (i < 5 && !aligned16(ptrs[i]))) return KVEV_ERR_INVALID_ARG;
    return KVEV_OK;
}

// where the packed weights sit inside a buffer that begins at `base`
static void lstm_packed_pointers(const kvev_shape *sh, void *base, LstmArgs &a)
{
    a.whh_packed = static_cast<const bf16x8_t *>(base);
    a.wih_packed = a.whh_packed + (size_t)sh->L * 4 * sh->d_g * sh->d_g / 8;
    a.whh_max_bits = reinterpret_cast<uint32_t *>(static_cast<unsigned char *>(base) +
                                            (size_t)sh->L * 4 * sh->d_g * ((size_t)sh->d_g + 2 * sh->d) * 2);
}

static int lstm_gate_common(const kvev_shape *sh, const void *Kbar, const void *Vbar, const kvev_lstm_w *w,
                            const void *packed, size_t packed_bytes, bool prepared, int chunk_begin, int chunk_end,
                            float *h, float *c, float *util, float *gate, void *ws, size_t ws_bytes, void *stream)
{
    int rc = check_shape(sh);
    if (rc) return rc;
    if (!Kbar || !Vbar || !h || !c || !util || !gate || !aligned16(Kbar) || !aligned16(Vbar) || !aligned16(h) ||
        !aligned16(c))
        return KVEV_ERR_INVALID_ARG;
    rc = lstm_check_weights(w);
    if (rc) return rc;
    if (chunk_begin < 0 || chunk_begin > chunk_end || chunk_end > sh->N_cap) return KVEV_ERR_INVALID_ARG;
    if (sizeof(float) * (2 * (size_t)sh->d + 6 * (size_t)sh->d_g) > 64 * 1024 && !lstm_takes_mfma(sh))
        return KVEV_ERR_UNSUPPORTED;
    if (prepared && lstm_takes_mfma(sh) && (!packed || !aligned16(packed) || packed_bytes < lstm_ws_weights(sh)))
        return KVEV_ERR_WORKSPACE;
    if (chunk_begin == chunk_end) return KVEV_OK;

    LstmArgs a;
    memset(&a, 0, sizeof a);
    a.Kbar = Kbar; a.Vbar = Vbar;
    a.W_ih = w->W_ih; a.W_hh = w->W_hh; a.b_ih = w->b_ih; a.b_hh = w->b_hh; a.w_s = w->w_s; a.b_s = w->b_s;
    a.h = h; a.c = c; a.util = util; a.gate = gate;
    a.L = sh->L; a.BH = sh->B * kv_heads(sh); a.d = sh->d; a.N_cap = sh->N_cap; a.d_g = sh->d_g;
    a.c0 = chunk_begin; a.c1 = chunk_end;
    hipStream_t st = static_cast<hipStream_t>(stream);
    hipError_t e;
    if (lstm_takes_mfma(sh)) {
        const size_t per = lstm_ws_per_step(sh), pack = lstm_ws_pack(sh, prepared);
        if (!ws || !aligned16(ws) || ws_bytes < pack + per) return KVEV_ERR_WORKSPACE;
        a.fused = lstm_takes_fused(sh) ? 1 : 0;
        a.split = lstm_split_of(sh);
        size_t tb = per == 0 ? (size_t)(chunk_end - chunk_begin) : (ws_bytes - pack) / per;
        if (tb > (size_t)(chunk_end - chunk_begin)) tb = (size_t)(chunk_end - chunk_begin);
        a.tb = (int)tb;
        unsigned char *p = static_cast<unsigned char *>(ws);
        a.status = reinterpret_cast<int32_t *>(p);
        p += kLstmWsHead;
        a.prepared = prepared ? 1 : 0;
        if (prepared) {
            lstm_packed_pointers(sh, const_cast<void *>(packed), a);
        } else {
            lstm_packed_pointers(sh, p, a);
            p += lstm_ws_weights(sh);
        }
        a.exch_bytes = lstm_exch_bytes(sh);
        a.quad_groups = lstm_quad_groups();
        a.exch = a.exch_bytes ? p : nullptr;
        a.xproj = reinterpret_cast<float *>(static_cast<unsigned char *>(ws) + pack);
        a.pair_spin_limit = g_pair_spin_limit.load();
        a.pair_mute = g_pair_mute.load();
        e = launch_lstm_mfma(a, st);
    } else {
        e = launch_lstm_generic(a, sh->dtype, st);
    }
    return e == hipSuccess ? KVEV_OK : hip_fail(e);
}

int kvev_lstm_gate(const kvev_shape *sh, const void *Kbar, const void *Vbar, const kvev_lstm_w *w,
                   int chunk_begin, int chunk_end, float *h, float *c, float *util, float *gate, void *ws,
                   size_t ws_bytes, void *stream)
{
    return lstm_gate_common(sh, Kbar, Vbar, w, nullptr, 0, false, chunk_begin, chunk_end, h, c, util, gate, ws, ws_bytes,
                            stream);
}

int kvev_lstm_prepare(const kvev_shape *sh, const kvev_lstm_w *w, void *packed, size_t packed_bytes, void *stream)
{
    int rc = check_shape(sh);
    if (rc) return rc;
    rc = lstm_check_weights(w);
    if (rc) return rc;
    if (!lstm_takes_mfma(sh)) return KVEV_OK;          // the generic kernels read the weights as they are
    if (!packed || !aligned16(packed) || packed_bytes < lstm_ws_weights(sh)) return KVEV_ERR_WORKSPACE;
    LstmArgs a;
    memset(&a, 0, sizeof a);
    a.W_ih = w->W_ih; a.W_hh = w->W_hh;
    a.L = sh->L; a.d = sh->d; a.d_g = sh->d_g;
    lstm_packed_pointers(sh, packed, a);
    hipError_t e = launch_lstm_prepare(a, static_cast<hipStream_t>(stream));
    return e == hipSuccess ? KVEV_OK : hip_fail(e);
}

int kvev_lstm_gate_prepared(const kvev_shape *sh, const void *Kbar, const void *Vbar, const kvev_lstm_w *w,
                            const void *packed, size_t packed_bytes, int chunk_begin, int chunk_end, float *h, float *c,
                            float *util, float *gate, void *ws, size_t ws_bytes, void *stream)
{
    return lstm_gate_common(sh, Kbar, Vbar, w, packed, packed_bytes, true, chunk_begin, chunk_end, h, c, util, gate, ws,
                            ws_bytes, stream);
}

int kvev_select(const kvev_shape *sh, const float *util, const float *gate, int mode, int k, float tau,
                int k_cap, int32_t *idx, int32_t *count, void *stream)
{
    int rc = check_shape(sh);
    if (rc) return rc;
    if (mode != KVEV_SELECT_TOPK && mode != KVEV_SELECT_THRESHOLD) return KVEV_ERR_UNSUPPORTED;
    if (!idx || !count || k_cap < 0) return KVEV_ERR_INVALID_ARG;
    const int ncand = n_cand_of(sh);
    if (ncand > sh->N_cap) return KVEV_ERR_INVALID_ARG;
    if (ncand > 16384) return KVEV_ERR_UNSUPPORTED;
    if (mode == KVEV_SELECT_TOPK) {
        if (!util || k < 0 || k_cap < (k < ncand ? k : ncand)) return KVEV_ERR_INVALID_ARG;
    } else {
        if (!gate || k_cap < ncand || tau != tau) return KVEV_ERR_INVALID_ARG;
    }
    SelectArgs a;
    a.util = util; a.gate = gate; a.idx = idx; a.count = count;
    a.S = sh->L * sh->B * kv_heads(sh); a.N_cap = sh->N_cap; a.n_cand = ncand; a.k = k; a.k_cap = k_cap;
    a.mode = mode; a.tau = tau;
    hipError_t e = launch_select(a, static_cast<hipStream_t>(stream));
    return e == hipSuccess ? KVEV_OK : hip_fail(e);
}

int kvev_gated_attention(const kvev_shape *sh, const void *Q, int Tq, const void *K, const void *V,
                         const void *Kbar, const void *Vbar, const int32_t *idx, const int32_t *count,
                         int k_cap, int causal, void *O, void *ws, size_t ws_bytes, void *stream)
{
    return attention_common(sh, Q, Tq, K, V, Kbar, Vbar, idx, count, k_cap, 1, causal, O, ws, ws_bytes, stream);
}

int kvev_gated_attention_static(const kvev_shape *sh, const void *Q, int Tq, const void *K, const void *V,
                                const void *Kbar, const void *Vbar, const int32_t *idx, const int32_t *count,
                                int k_cap, int causal, void *O, void *stream)
{
    return attention_common(sh, Q, Tq, K, V, Kbar, Vbar, idx, count, k_cap, 1, causal, O, nullptr, 0, stream, 0, true);
}

int kvev_dense_attention(const kvev_shape *sh, const void *Q, int Tq, const void *K, const void *V, int causal,
                         void *O, void *ws, size_t ws_bytes, void *stream)
{
    return attention_common(sh, Q, Tq, K, V, nullptr, nullptr, nullptr, nullptr, 0, 0, causal, O, ws, ws_bytes,
                            stream);
}

int kvev_compact_attention(const kvev_shape *sh, const void *Q, int Tq, const void *Kw, const void *Vw,
                           int win_first, const void *Kc, const void *Vc, const int32_t *count, int k_cap,
                           int causal, void *O, void *ws, size_t ws_bytes, void *stream)
{
    return attention_common(sh, Q, Tq, Kw, Vw, Kc, Vc, nullptr, count, k_cap, 2, causal, O, ws, ws_bytes, stream,
                            win_first);
}

int kvev_retain(const kvev_shape *sh, int k, int k_cap, const void *Kbar_new, const void *Vbar_new,
                const float *util_new, int n_new_cap, int first_chunk, int n_new, void *Kc, void *Vc,
                int32_t *chunk_id, float *util_c, int32_t *count, void *stream)
{
    int rc = check_shape(sh, false);
    if (rc) return rc;
    if (k < 0 || k > k_cap || n_new < 0 || n_new > n_new_cap || first_chunk < 0) return KVEV_ERR_INVALID_ARG;
    if ((int64_t)k_cap + n_new > 4000) return KVEV_ERR_INVALID_ARG;
    if (!Kc || !Vc || !chunk_id || !util_c || !count || !aligned16(Kc) || !aligned16(Vc)) return KVEV_ERR_INVALID_ARG;
    if (n_new > 0 && (!Kbar_new || !Vbar_new || !util_new || !aligned16(Kbar_new) || !aligned16(Vbar_new)))
        return KVEV_ERR_INVALID_ARG;
    RetainArgs a;
    a.Kn = Kbar_new; a.Vn = Vbar_new; a.un = util_new; a.Kc = Kc; a.Vc = Vc; a.ids = chunk_id; a.uc = util_c;
    a.count = count;
    a.S = sh->L * sh->B * kv_heads(sh);
    a.row_bytes = sh->d * (sh->dtype == KVEV_F32 ? 4 : 2);
    a.k = k; a.k_cap = k_cap; a.n_new_cap = n_new_cap; a.first_chunk = first_chunk; a.n_new = n_new;
    hipError_t e = launch_retain(a, static_cast<hipStream_t>(stream));
    return e == hipSuccess ? KVEV_OK : hip_fail(e);
}

int kvev_debug_pair_wait(int spin_limit, int mute_member)
{
    if (spin_limit < 1 || mute_member < -1 || mute_member > 1) return KVEV_ERR_INVALID_ARG;
    g_pair_spin_limit = spin_limit;
    g_pair_mute = mute_member;
    return KVEV_OK;
}

int kvev_debug_attn_stream_bytes(size_t bytes)
{
    g_stream_bytes = bytes == 0 ? kStreamBytesDefault : bytes;
    return KVEV_OK;
}

int kvev_debug_lstm_quad_groups(int groups)
{
    if (groups < 0) return KVEV_ERR_INVALID_ARG;
    g_lstm_quad_groups = groups;
    return KVEV_OK;
}

int kvev_debug_lstm_fused_min_groups(int min_groups)
{
    if (min_groups < 0) return KVEV_ERR_INVALID_ARG;
    g_lstm_fused_min_groups = min_groups == 0 ? g_lstm_fused_min_groups_default : min_groups;
    return KVEV_OK;
}

int kvev_debug_stream_probe(const void *src, size_t src_bytes, int tile_bytes, void *dst, size_t dst_bytes,
                            int write_bytes_per_tile, int hints, void *stream)
{
    if (!src || !dst || !aligned16(src) || !aligned16(dst)) return KVEV_ERR_INVALID_ARG;
    if (tile_bytes < 4096 || tile_bytes % 4096 != 0 || src_bytes % (size_t)tile_bytes != 0) return KVEV_ERR_INVALID_ARG;
    if (write_bytes_per_tile < 0 || write_bytes_per_tile % 16 != 0 || hints < 0 || hints > 7) return KVEV_ERR_INVALID_ARG;
    if ((hints & 4) && write_bytes_per_tile > 48 * 1024) return KVEV_ERR_INVALID_ARG;
    const size_t tiles = src_bytes / (size_t)tile_bytes;
    if (tiles > ((size_t)1 << 31) - 1) return KVEV_ERR_INVALID_ARG;
    const size_t need = write_bytes_per_tile ? tiles * (size_t)write_bytes_per_tile : 16;
    if (dst_bytes < need) return KVEV_ERR_INVALID_ARG;
    hipError_t e = launch_stream_probe(src, tiles, tile_bytes, dst, write_bytes_per_tile, hints, static_cast<hipStream_t>(stream));
    return e == hipSuccess ? KVEV_OK : hip_fail(e);
}

size_t kvev_workspace_bytes(int op, const kvev_shape *sh, int n, int k_cap)
{
    if (check_shape(sh, op != KVEV_OP_COMPACT_ATTENTION) != KVEV_OK || n < 0) return 0;
    switch (op) {
    case KVEV_OP_CHUNK_POOL:
        return pool_ws_bytes(sh);
    case KVEV_OP_LSTM_GATE:
    case KVEV_OP_LSTM_GATE_PREPARED: {
        const size_t per = lstm_ws_per_step(sh);
        const int tb = n < 128 ? n : 128;
        if (!lstm_takes_mfma(sh)) return 0;
        return lstm_ws_pack(sh, op == KVEV_OP_LSTM_GATE_PREPARED) + per * (size_t)(tb < 1 ? 1 : tb);
    }
    case KVEV_OP_LSTM_PREPARE:
        return lstm_takes_mfma(sh) ? lstm_ws_weights(sh) : 0;
    case KVEV_OP_GATED_ATTENTION: {
        if (k_cap < 0) return 0;
        const int ncand = n_cand_of(sh);
        const int kmax = k_cap < ncand ? k_cap : ncand;
        (void)kmax;
        return attn_takes_mq(sh, n) ? 0 : plan_attn(sh, n, sh->T - ncand * sh->C).ws_bytes;
    }
    case KVEV_OP_DENSE_ATTENTION:
        return attn_takes_mq(sh, n) ? 0 : plan_attn(sh, n, sh->T).ws_bytes;
    case KVEV_OP_COMPACT_ATTENTION:
        if (k_cap < 0) return 0;
        return attn_takes_mq(sh, n) ? 0 : plan_attn(sh, n, sh->T).ws_bytes;
    default:
        return 0;
    }
}

const char *kvev_status_string(int status)
{
    switch (status) {
    case KVEV_OK: return "ok";
    case KVEV_ERR_INVALID_ARG: return "invalid argument";
    case KVEV_ERR_UNSUPPORTED: return "unsupported shape, dtype or mode";
    case KVEV_ERR_WORKSPACE: return "workspace missing, misaligned or too small";
    case KVEV_ERR_HIP: return "HIP runtime error";
    case KVEV_ERR_STATIC_SCRATCH: return "the shape needs more scratch than the library's static array holds";
    default: return "unknown status";
    }
}

const char *kvev_last_hip_error(void) { return g_hip_err; }

int kvev_version(void) { return 200; }

}  // extern "C"

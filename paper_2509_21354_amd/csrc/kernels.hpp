// Host-visible launch interface between the C-ABI layer (api.hip) and the
// kernel files.  Everything here is plain data; shapes were validated by the
// caller.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace kvev {

#define KVEV_ATTN_MAX_SPLIT 256   // decode attention: most splits of one query's rows

struct AttnArgs {
    const void *Q, *K, *V, *Kbar, *Vbar;
    const int32_t *idx, *count;
    void *O;
    float *part;          // split partials [S*Tq][nsplit][d+2] (o, m, l), or null when nsplit == 1
    int32_t *tickets;     // one arrival counter per (key-value sequence, query group), zero between calls; null when nsplit == 1
    int S, Tq, d;          // S: key-value sequences (L*B*H_kv)
    int G, Hkv;           // query heads per key-value head; key-value heads per (layer, batch row)
    int causal;           // 1: the Tq queries are the last Tq cached tokens and see nothing after themselves
    int T, T_cap, N_cap, k_cap;
    int win0;             // first raw token attended (0 for the dense baseline)
    int ring_first;       // compact form: the window buffer is a ring, its token t sits in row (ring_first + t) mod T_cap; else 0
    int gated;            // 1: kept summaries precede the raw rows
    int nsplit, rows_per_split;
    int stream;           // 1: the launch reads more than the memory-side cache holds: single-query loads carry the non-temporal hint
    float scale_log2e;    // log2(e) / sqrt(d)
};

struct PoolArgs {
    const void *K, *V;
    void *Kbar, *Vbar;
    const void *W1K, *b1K, *W2K, *b2K, *W1V, *b1V, *W2V, *b2V;   // per layer
    int L, BH, d, T_cap, C, N_cap, d_sum;
    int c0, c1;
    int mode;
    int compute_units;    // of the device the launch goes to
    int flush_shift;      // the persistent form writes its summaries once per 2^flush_shift ticks of the 100 MHz real-time counter
    void *wpack;          // workspace for the MLP weights in MFMA fragment order (pool_pack_bytes), or null: read as given
};

// The MLP weights of both sides re-laid per layer for the matrix cores: W1 and W2 as 1 KiB fragments (one 16-byte piece
// per lane, in the order the kernel walks them), then the biases as fp32.
constexpr size_t pool_pack_layer_bytes(int d, int d_sum) { return (size_t)8 * d_sum * d + (size_t)8 * (d_sum + d); }
inline size_t pool_pack_bytes(int L, int d, int d_sum) { return (size_t)L * pool_pack_layer_bytes(d, d_sum); }

struct LstmArgs {
    const void *Kbar, *Vbar;
    const void *W_ih, *W_hh, *b_ih, *b_hh, *w_s, *b_s;           // per layer
    float *h, *c, *util, *gate;
    float *xproj;         // workspace: fp32 input projections of a block of steps (fragment layout)
    const __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 *whh_packed;   // workspace: W_hh in fragment order (16-byte pieces; fp16 inside)
    uint32_t *whh_max_bits;   // workspace: 32 partial maxima of |W_hh| per layer as bit patterns (their maximum fixes the power-of-two scale)
    const __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 *wih_packed;   // workspace: W_ih in fragment order
    unsigned char *exch;  // workspace: exchange slots of the split recurrence (lstm_split_exch_bytes), or null
    size_t exch_bytes;    // 0: one workgroup per sequence group
    int split;            // workgroups that share a sequence group in the recurrence: 0 (one), 2 or 4 (lstm_split)
    int quad_groups;      // split == 4: groups of 32 sequences per launch at most (compute units / 4)
    int pair_spin_limit;  // polls a wave of the paired recurrence spends on one wait before it gives up
    int pair_mute;        // member (0, 1) whose publications are withheld, -1: none (failure-path tests only)
    int32_t *status;      // workspace: word that a launch sets to 1 when a bounded wait expired (never cleared by the library)
    int prepared;         // 1: the packed weights are already in place (kvev_lstm_prepare), 0: this call packs them first
    int L, BH, d, N_cap, d_g;
    int c0, c1;
    int tb;               // steps per workspace block
    int fused;            // 1: the single-kernel form (d_g = 256, 32 sequences per workgroup, no projections in scratch)
};

// How the gate spreads a group of sequences over workgroups that exchange h every step (0: one workgroup per 16
// sequences, no exchange).  Pairs: 16 sequences on two workgroups when the launch has at most one workgroup per compute
// unit (at d_g = 512 a single workgroup is bound by the weight stream out of L2 and a pair halves it; at d_g = 256 a
// pair keeps all of W_hh in registers).  Quadruples: at d_g = 512 with more than 16 sequences per layer, 32 sequences
// on four workgroups (a quarter of the stream each, and every fragment serves two blocks of sequences); a launch
// takes at most one workgroup per compute unit, larger calls are cut into several launches.  So all workgroups of a
// launch can be resident together on an idle device (bounded waits in the kernels cover the rest).
constexpr size_t kLstmPairExchBytes256 = 65536;     // scratch per group of 16 sequences and 256 hidden units
constexpr size_t kLstmQuadExchBytes = 131072;       // scratch per group of 32 sequences
inline int lstm_split(int d_g, int L, int BH, int compute_units, bool quad_allowed)
{
    const long long g16 = (long long)L * ((BH + 15) / 16);
    if (d_g == 512 && quad_allowed && BH > 16 && compute_units >= 4) return 4;     // (more groups than fit at once: several launches)
    if ((d_g == 256 || d_g == 512) && 2 * g16 <= compute_units) return 2;
    return 0;
}
inline size_t lstm_split_exch_bytes(int split, int d_g, int L, int BH, int quad_groups)
{
    if (split == 4) {       // the slots of one launch (quad_groups groups at most), used again by the next
        const long long g32 = (long long)L * ((BH + 31) / 32);
        return (size_t)(g32 < quad_groups ? g32 : quad_groups) * kLstmQuadExchBytes;
    }
    if (split == 2) return (size_t)L * ((BH + 15) / 16) * (d_g / 256) * kLstmPairExchBytes256;
    return 0;
}

struct SelectArgs {
    const float *util, *gate;
    int32_t *idx, *count;
    int S, N_cap, n_cand, k, k_cap, mode;
    float tau;
};

struct RetainArgs {
    const void *Kn, *Vn;          // new summaries [S, n_new_cap, d]
    const float *un;              // their scores [S, n_new_cap]
    void *Kc, *Vc;                // compact store [S, k_cap, d]
    int32_t *ids;                 // chunk ids of the store rows [S, k_cap], ascending
    float *uc;                    // their scores [S, k_cap]
    int32_t *count;               // [S]
    int S, row_bytes, k, k_cap, n_new_cap, first_chunk, n_new;
};

hipError_t launch_attn_decode(const AttnArgs &a, int dtype, hipStream_t st);
hipError_t launch_attn_mq(const AttnArgs &a, hipStream_t st);           // bf16 MFMA, many queries
hipError_t launch_select(const SelectArgs &a, hipStream_t st);
hipError_t launch_retain(const RetainArgs &a, hipStream_t st);
hipError_t launch_pool_generic(const PoolArgs &a, int dtype, hipStream_t st);
hipError_t launch_pool_mfma(const PoolArgs &a, hipStream_t st);          // bf16
hipError_t launch_pool_token_mfma(const PoolArgs &a, hipStream_t st);    // bf16, the MLP on every token
size_t pool_token_mfma_lds(int d, int d_sum);                            // its LDS need in bytes
hipError_t launch_lstm_generic(const LstmArgs &a, int dtype, hipStream_t st);
hipError_t launch_lstm_mfma(const LstmArgs &a, hipStream_t st);          // bf16
hipError_t launch_lstm_prepare(const LstmArgs &a, hipStream_t st);       // bf16: the packed weights alone
hipError_t launch_stream_probe(const void *src, size_t tiles, int tile_bytes, void *dst, int write_bytes, int hints, hipStream_t st);   // calibration
hipError_t launch_lstm_quad(const LstmArgs &a, hipStream_t st);          // bf16, d_g = 512: projection and recurrence of 32 sequences on four workgroups (weights already packed)
hipError_t launch_lstm_fused(const LstmArgs &a, hipStream_t st);         // bf16, d_g = 256: the recurrence with the input projection inside (weights already packed)

}  // namespace kvev

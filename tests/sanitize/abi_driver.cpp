// Drives the host side of the C ABI (argument checks, launch planning, scratch sizing) from a program whose host code
// is built with -fsanitize=address,undefined: every call here fails validation or has nothing to do, so no GPU is
// needed and none is touched.  Pointers that validation never dereferences are fake but aligned; host structs that it
// does read are real.  Exit status 0 = every status code as expected and no sanitizer report.
#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <cstring>

#include "../../include/kvev.h"
#include "../../include/kvev_test_hooks.h"

static int g_fail = 0;
#define EXPECT(call, want)                                                                       \
    do {                                                                                         \
        const int got_ = (call);                                                                 \
        if (got_ != (want)) { std::printf("line %d: %s = %d, want %d\n", __LINE__, #call, got_, (int)(want)); ++g_fail; } \
    } while (0)

int main()
{
    void *F = reinterpret_cast<void *>(0x1000), *odd = reinterpret_cast<void *>(0x1004);
    float *Ff = static_cast<float *>(F);
    int32_t *Fi = static_cast<int32_t *>(F);
    kvev_shape *sh = static_cast<kvev_shape *>(std::malloc(sizeof(kvev_shape)));      // heap: any read past it is caught
    const kvev_shape base = {1, 1, 32, 128, 4096, 4096, 32, 128, 256, 128, 256, KVEV_BF16, 0};
    *sh = base;
    kvev_mlp_w *mw = static_cast<kvev_mlp_w *>(std::malloc(sizeof(kvev_mlp_w)));
    *mw = kvev_mlp_w{F, F, F, F};
    kvev_lstm_w *lw = static_cast<kvev_lstm_w *>(std::malloc(sizeof(kvev_lstm_w)));
    *lw = kvev_lstm_w{F, F, F, F, F, F};

    // shapes
    EXPECT(kvev_dense_attention(nullptr, F, 1, F, F, 0, F, nullptr, 0, nullptr), KVEV_ERR_INVALID_ARG);
    const int bad_fields[][2] = {{0, 0}, {3, -1}, {6, 0}, {4, 5000}, {7, 3}, {8, -1}, {10, 0}, {12, 5}};
    for (const auto &bf : bad_fields) {
        *sh = base;
        reinterpret_cast<int32_t *>(sh)[bf[0]] = bf[1];
        EXPECT(kvev_dense_attention(sh, F, 1, F, F, 0, F, nullptr, 0, nullptr), KVEV_ERR_INVALID_ARG);
        EXPECT((int)kvev_workspace_bytes(KVEV_OP_DENSE_ATTENTION, sh, 1, 0), 0);
    }
    *sh = base; sh->d = 96;
    EXPECT(kvev_dense_attention(sh, F, 1, F, F, 0, F, nullptr, 0, nullptr), KVEV_ERR_UNSUPPORTED);
    *sh = base; sh->dtype = 7;
    EXPECT(kvev_chunk_pool(sh, F, F, KVEV_POOL_MEAN, nullptr, nullptr, 0, 1, F, F, nullptr, 0, nullptr), KVEV_ERR_UNSUPPORTED);
    *sh = base;

    // attention
    EXPECT(kvev_dense_attention(sh, odd, 1, F, F, 0, F, nullptr, 0, nullptr), KVEV_ERR_INVALID_ARG);
    EXPECT(kvev_dense_attention(sh, F, -1, F, F, 0, F, nullptr, 0, nullptr), KVEV_ERR_INVALID_ARG);
    EXPECT(kvev_dense_attention(sh, F, 1, F, F, 2, F, nullptr, 0, nullptr), KVEV_ERR_INVALID_ARG);
    EXPECT(kvev_dense_attention(sh, F, 1, F, F, 0, F, nullptr, 0, nullptr), KVEV_ERR_WORKSPACE);
    EXPECT(kvev_dense_attention(sh, F, 1, F, F, 0, F, F, 64, nullptr), KVEV_ERR_WORKSPACE);
    EXPECT(kvev_dense_attention(sh, F, 0, F, F, 0, F, nullptr, 0, nullptr), KVEV_OK);
    EXPECT(kvev_gated_attention(sh, F, 1, F, F, F, F, nullptr, Fi, 32, 0, F, nullptr, 0, nullptr), KVEV_ERR_INVALID_ARG);
    EXPECT(kvev_gated_attention(sh, F, 400, F, F, F, F, Fi, Fi, 32, 1, F, nullptr, 0, nullptr), KVEV_ERR_INVALID_ARG);
    EXPECT(kvev_gated_attention_static(sh, F, 1, F, F, F, F, Fi, Fi, -1, 0, F, nullptr), KVEV_ERR_INVALID_ARG);
    EXPECT(kvev_gated_attention_static(sh, F, 0, F, F, F, F, Fi, Fi, 32, 0, F, nullptr), KVEV_OK);
    EXPECT(kvev_compact_attention(sh, F, 1, F, F, -1, F, F, Fi, 32, 0, F, nullptr, 0, nullptr), KVEV_ERR_INVALID_ARG);
    EXPECT(kvev_compact_attention(sh, F, 1, F, F, 0, F, F, Fi, 32, 0, F, nullptr, 0, nullptr), KVEV_ERR_WORKSPACE);
    // pool
    EXPECT(kvev_chunk_pool(sh, F, F, 5, mw, mw, 0, 1, F, F, nullptr, 0, nullptr), KVEV_ERR_UNSUPPORTED);
    EXPECT(kvev_chunk_pool(sh, F, F, KVEV_POOL_MLP, nullptr, mw, 0, 1, F, F, nullptr, 0, nullptr), KVEV_ERR_INVALID_ARG);
    EXPECT(kvev_chunk_pool(sh, F, F, KVEV_POOL_MLP, mw, mw, 0, 129, F, F, nullptr, 0, nullptr), KVEV_ERR_INVALID_ARG);
    EXPECT(kvev_chunk_pool(sh, F, F, KVEV_POOL_MEAN, nullptr, nullptr, 7, 7, F, F, nullptr, 0, nullptr), KVEV_OK);
    // gate
    EXPECT(kvev_lstm_gate(sh, F, F, nullptr, 0, 1, Ff, Ff, Ff, Ff, nullptr, 0, nullptr), KVEV_ERR_INVALID_ARG);
    EXPECT(kvev_lstm_gate(sh, F, F, lw, 0, 129, Ff, Ff, Ff, Ff, nullptr, 0, nullptr), KVEV_ERR_INVALID_ARG);
    EXPECT(kvev_lstm_gate(sh, F, F, lw, 0, 1, Ff, Ff, Ff, Ff, nullptr, 0, nullptr), KVEV_ERR_WORKSPACE);
    EXPECT(kvev_lstm_gate(sh, F, F, lw, 4, 4, Ff, Ff, Ff, Ff, nullptr, 0, nullptr), KVEV_OK);
    const size_t need = kvev_workspace_bytes(KVEV_OP_LSTM_PREPARE, sh, 0, 0);
    EXPECT(need > 0, 1);
    EXPECT(kvev_lstm_prepare(sh, lw, nullptr, need, nullptr), KVEV_ERR_WORKSPACE);
    EXPECT(kvev_lstm_prepare(sh, lw, F, need - 1, nullptr), KVEV_ERR_WORKSPACE);
    EXPECT(kvev_lstm_gate_prepared(sh, F, F, lw, F, need, 0, 1, Ff, Ff, Ff, Ff, nullptr, 0, nullptr), KVEV_ERR_WORKSPACE);
    EXPECT(kvev_lstm_gate_prepared(sh, F, F, lw, F, need, 2, 2, Ff, Ff, Ff, Ff, nullptr, 0, nullptr), KVEV_OK);
    EXPECT(kvev_workspace_bytes(KVEV_OP_LSTM_GATE, sh, 128, 0) > kvev_workspace_bytes(KVEV_OP_LSTM_GATE_PREPARED, sh, 128, 0), 1);
    // select, retain
    EXPECT(kvev_select(sh, Ff, nullptr, 9, 4, 0.f, 4, Fi, Fi, nullptr), KVEV_ERR_UNSUPPORTED);
    EXPECT(kvev_select(sh, nullptr, nullptr, KVEV_SELECT_TOPK, 4, 0.f, 4, Fi, Fi, nullptr), KVEV_ERR_INVALID_ARG);
    EXPECT(kvev_select(sh, Ff, nullptr, KVEV_SELECT_TOPK, 32, 0.f, 31, Fi, Fi, nullptr), KVEV_ERR_INVALID_ARG);
    EXPECT(kvev_retain(sh, 33, 32, F, F, Ff, 8, 0, 4, F, F, Fi, Ff, Fi, nullptr), KVEV_ERR_INVALID_ARG);
    EXPECT(kvev_retain(sh, 4, 3990, F, F, Ff, 16, 0, 16, F, F, Fi, Ff, Fi, nullptr), KVEV_ERR_INVALID_ARG);
    // hooks and strings
    EXPECT(kvev_debug_pair_wait(0, -1), KVEV_ERR_INVALID_ARG);
    EXPECT(kvev_debug_pair_wait(1 << 22, -1), KVEV_OK);
    EXPECT(kvev_debug_lstm_fused_min_groups(-1), KVEV_ERR_INVALID_ARG);
    EXPECT(kvev_debug_lstm_fused_min_groups(0), KVEV_OK);
    for (int st = -1; st <= 7; ++st) EXPECT(std::strlen(kvev_status_string(st)) > 0, 1);
    EXPECT(kvev_version() >= 200, 1);
    std::free(sh); std::free(mw); std::free(lw);
    std::printf("abi driver: %d unexpected\n", g_fail);
    return g_fail ? 1 : 0;
}

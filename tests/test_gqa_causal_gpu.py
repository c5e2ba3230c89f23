"""Grouped-query heads (H_kv < H) and causal query frames on the GPU against the oracle:
the whole chain runs per key-value head, attention serves every query head of a group from one
read of the rows (decode kernel: up to 4 queries per workgroup; matrix-core kernel: the group's
queries form one frame), and a causal frame hides the rows after each query's own token."""
import numpy as np
import pytest
import torch

from oracle import kvev_oracle as orc
from paper_2509_21354_amd import binding as kb
from paper_2509_21354_amd import synth
from tests.helpers import assert_close_storage, dev

pytestmark = pytest.mark.gpu


def _cfg(number, dtype, **kw):
    base = dict(L=2, B=2, H=4, d=64, T=400, C=16, k=6, W=40, d_sum=48, d_g=40, Tq=1)
    base.update(kw)
    return synth.Config(number, f"gqa{number}", dtype, **base)


CASES = [
    # (config, causal)                                          queries per kv sequence -> kernel
    (_cfg(201, "f32", H=6, H_kv=2), 0),                         # 3 -> decode, pairs (one ragged)
    (_cfg(202, "bf16", d=128, H=8, H_kv=2, T=1500, C=32, W=200, k=9), 0),     # 4 -> decode, one group of 4
    (_cfg(203, "bf16", d=128, H=8, H_kv=1, T=2100, C=32, W=256, k=12, L=1), 0),   # 8 -> decode, two groups of 4
    (_cfg(204, "bf16", d=128, H=8, H_kv=2, Tq=8, T=1200, C=32, W=128, k=8, L=1), 0),   # 32 -> matrix cores
    (_cfg(205, "bf16", d=64, H=4, H_kv=2, Tq=40, T=900, C=16, W=100, k=7, L=1), 0),    # 80 -> matrix cores, wide tile
    (_cfg(206, "f32", H=4, H_kv=4, Tq=3), 1),                   # causal, no grouping, decode
    (_cfg(207, "bf16", d=128, H=4, H_kv=0, Tq=5, T=1300, C=32, W=160, k=8), 1),    # causal decode, 4 + 1 queries
    (_cfg(208, "bf16", d=128, H=2, H_kv=0, Tq=48, T=1100, C=32, W=130, k=8, L=1), 1),   # causal on the matrix cores
    (_cfg(209, "bf16", d=128, H=8, H_kv=2, Tq=16, T=1000, C=32, W=96, k=8, L=1), 1),   # causal + grouped, matrix cores
    (_cfg(210, "f32", d=128, H=6, H_kv=3, Tq=2, T=300, C=8, W=30, k=5), 1),        # causal + grouped, decode
    # more than 128 queries per key-value sequence: workgroups of 8 waves (256 queries), last waves partly or wholly idle
    (_cfg(211, "bf16", d=128, H=2, H_kv=0, Tq=150, T=1100, C=32, W=200, k=9, L=1, B=1), 0),
    (_cfg(212, "bf16", d=64, H=8, H_kv=2, Tq=40, T=700, C=16, W=90, k=6, L=1, B=1), 1),      # 160, causal + grouped
    (_cfg(213, "bf16", d=128, H=2, H_kv=0, Tq=300, T=900, C=32, W=320, k=7, L=1, B=1), 1),   # 300: two tiles, the second ragged
]


@pytest.mark.parametrize("cfg,causal", CASES, ids=[c.name + ("_causal" if z else "") for c, z in CASES])
def test_chain_and_attention_with_grouped_heads_and_causal_frames(cfg, causal):
    t = synth.make_inputs(cfg, "cpu")
    g = dev(t)
    assert t["K"].shape[2] == cfg.kv_heads and t["Q"].shape[2] == cfg.H
    st = kb.DecodeState(cfg)
    sh, N = st.shape, cfg.N
    kb.kvev_chunk_pool(sh, g["K"], g["V"], kb.POOL_MLP, kb.mlp_weights(g, "K"), kb.mlp_weights(g, "V"), 0, N,
                       st.Kbar, st.Vbar, st.ws)
    kb.kvev_lstm_gate(sh, st.Kbar, st.Vbar, kb.lstm_weights(g), 0, N, st.h, st.c, st.util, st.gate, st.ws)
    kb.kvev_select(sh, st.util, st.gate, kb.SELECT_TOPK, cfg.k, 0.0, st.k_cap, st.idx, st.count)
    O = torch.empty_like(g["Q"])
    kb.kvev_gated_attention(sh, g["Q"], cfg.Tq, g["K"], g["V"], st.Kbar, st.Vbar, st.idx, st.count, st.k_cap, O, st.ws_attn,
                            causal=causal)
    Od = torch.empty_like(g["Q"])
    kb.kvev_dense_attention(sh, g["Q"], cfg.Tq, g["K"], g["V"], Od, st.ws_attn, causal=causal)
    torch.cuda.synchronize()
    # the chain per key-value head against the oracle's stages
    rK, rV = orc.chunk_pool(t["K"], t["V"], cfg.T, cfg.C, st.N_cap, cfg.d_sum, orc.POOL_MLP,
                            kb.mlp_weights(t, "K"), kb.mlp_weights(t, "V"), 0, N)
    assert st.Kbar.shape[2] == cfg.kv_heads
    assert_close_storage(st.Kbar, rK, cfg.dtype, "Kbar")
    assert_close_storage(st.Vbar, rV, cfg.dtype, "Vbar")
    _, _, ru, _ = orc.lstm_gate(st.Kbar.cpu(), st.Vbar.cpu(), kb.lstm_weights(t), 0, N)
    assert np.abs(st.util.cpu().numpy()[..., :N] - ru[..., :N]).max() <= 1e-5
    ridx, rcnt = orc.select_topk(st.util.cpu(), cfg.T, cfg.C, cfg.W, cfg.k, st.k_cap)
    assert (orc.to_np(st.idx) == ridx).all() and (orc.to_np(st.count) == rcnt).all()
    # attention, teacher-forced on the GPU's own summaries and kept sets
    ref = orc.attention_ext(t["Q"], t["K"], t["V"], cfg.T, cfg.C, cfg.W, st.Kbar.cpu(), st.Vbar.cpu(), st.idx.cpu(),
                            st.count.cpu(), causal=causal)
    assert_close_storage(O, ref, cfg.dtype, "O gated")
    refd = orc.attention_ext(t["Q"], t["K"], t["V"], cfg.T, causal=causal)
    assert_close_storage(Od, refd, cfg.dtype, "O dense")
    # after eviction (per key-value head): compact store + window buffer give the bits of the indexed form
    n_cand, win0 = cfg.N_cand, cfg.N_cand * cfg.C
    lead = (cfg.L, cfg.B, cfg.kv_heads)
    k_cap = cfg.k + 1
    if n_cand > 0 and k_cap + n_cand <= 4000:
        Kc = torch.zeros(lead + (k_cap, cfg.d), dtype=cfg.torch_dtype, device="cuda")
        Vc = torch.zeros_like(Kc)
        ids = torch.full(lead + (k_cap,), -1, dtype=torch.int32, device="cuda")
        uc = torch.zeros(lead + (k_cap,), dtype=torch.float32, device="cuda")
        cnt = torch.zeros(lead, dtype=torch.int32, device="cuda")
        kb.kvev_retain(sh, cfg.k, k_cap, st.Kbar, st.Vbar, st.util, st.N_cap, 0, n_cand, Kc, Vc, ids, uc, cnt)
        Kw = g["K"][..., win0:cfg.T, :].contiguous()
        Vw = g["V"][..., win0:cfg.T, :].contiguous()
        shw = kb.make_shape(cfg, T=cfg.T - win0, T_cap=cfg.T - win0, N_cap=k_cap)
        wsw = kb.alloc_workspace(kb.workspace_bytes(kb.OP_COMPACT_ATTENTION, shw, cfg.Tq, k_cap))
        Oc = torch.empty_like(O)
        kb.kvev_compact_attention(shw, g["Q"], cfg.Tq, Kw, Vw, Kc, Vc, cnt, k_cap, Oc, wsw, causal=causal)
        torch.cuda.synchronize()
        assert (orc.to_np(Oc) == orc.to_np(O)).all()
        refc = orc.compact_attention(t["Q"], Kw.cpu(), Vw.cpu(), cfg.T - win0, Kc.cpu(), Vc.cpu(), cnt.cpu(), causal=causal)
        assert_close_storage(Oc, refc, cfg.dtype, "O compact store")
    if causal:
        # the last query of a causal frame sees everything: same bits as the frame without the mask
        On = torch.empty_like(O)
        kb.kvev_gated_attention(sh, g["Q"], cfg.Tq, g["K"], g["V"], st.Kbar, st.Vbar, st.idx, st.count, st.k_cap, On,
                                st.ws_attn, causal=0)
        torch.cuda.synchronize()
        assert (orc.to_np(On)[..., -1, :] == orc.to_np(O)[..., -1, :]).all()
        assert not (orc.to_np(On)[..., 0, :] == orc.to_np(O)[..., 0, :]).all()


def test_grouped_heads_read_the_rows_once_per_group():
    """Same inputs as multi-head attention with the key-value heads repeated: the outputs agree to
    rounding (the split plan may differ), which pins the head -> key-value head map on the GPU."""
    cfg = _cfg(211, "bf16", d=128, H=8, H_kv=2, T=3000, C=32, W=256, k=16, L=1, B=1)
    t = synth.make_inputs(cfg, "cpu")
    g = dev(t)
    st = kb.DecodeState(cfg)
    O = torch.empty_like(g["Q"])
    kb.kvev_dense_attention(st.shape, g["Q"], 1, g["K"], g["V"], O, st.ws_attn)
    G = cfg.H // cfg.H_kv
    full = cfg.replace(H_kv=0)
    st2 = kb.DecodeState(full)
    K2, V2 = g["K"].repeat_interleave(G, dim=2).contiguous(), g["V"].repeat_interleave(G, dim=2).contiguous()
    O2 = torch.empty_like(O)
    kb.kvev_dense_attention(st2.shape, g["Q"], 1, K2, V2, O2, st2.ws_attn)
    torch.cuda.synchronize()
    assert_close_storage(O, orc.to_np(O2), cfg.dtype, "grouped vs repeated heads")

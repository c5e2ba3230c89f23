"""Physical eviction on the GPU (sections 3.2-3.3): the compact store kept as the running top-k,
attention over store + resident window, and a stream that never holds more than k + window rows,
checked against the oracle and against the non-evicting path."""
import numpy as np
import pytest
import torch

from oracle import kvev_oracle as orc
from paper_2509_21354_amd import binding as kb
from paper_2509_21354_amd import synth
from tests.helpers import assert_close_storage, dev

pytestmark = pytest.mark.gpu


def _bits(t):
    return orc.to_np(t)


@pytest.mark.parametrize("dtype,d,k,k_cap,frames", [
    ("f32", 64, 5, 7, (3, 0, 1, 8, 6, 2, 20)),
    ("bf16", 128, 32, 32, (8, 8, 8, 8, 8, 8, 8, 8)),
    ("bf16", 128, 128, 130, (300, 40, 0, 257, 3)),          # more candidates than threads, several row batches
    ("f32", 128, 40, 40, (33, 64, 1)),
    ("bf16", 64, 0, 4, (5, 5)),                              # k = 0: nothing is ever kept
    ("bf16", 64, 500, 512, (3488, 100, 3488)),               # the largest store + frame the entry point takes (4000)
])
def test_retain_is_bit_exact(dtype, d, k, k_cap, frames):
    torch.manual_seed(11)
    lead = (2, 2, 3)
    cfg = synth.Config(170, "retain", dtype, L=lead[0], B=lead[1], H=lead[2], d=d, T=64, C=16, k=max(k, 1), W=16,
                       d_sum=32, d_g=64, Tq=1)
    sh = kb.make_shape(cfg)
    tdt = cfg.torch_dtype
    N = sum(frames)
    util = torch.randn(lead + (N,))
    util[0, 0, 0, 1::7] = 0.5                                 # ties
    util[1, 1, 2, 3] = float("nan")
    util[1, 0, 1, :] = -2.0                                   # all equal
    Kbar = torch.randn(lead + (N, d)).to(tdt)
    Vbar = torch.randn(lead + (N, d)).to(tdt)
    g = dict(Kc=torch.zeros(lead + (k_cap, d), dtype=tdt, device="cuda"), Vc=torch.zeros(lead + (k_cap, d), dtype=tdt, device="cuda"),
             ids=torch.full(lead + (k_cap,), -1, dtype=torch.int32, device="cuda"),
             uc=torch.zeros(lead + (k_cap,), dtype=torch.float32, device="cuda"),
             cnt=torch.zeros(lead, dtype=torch.int32, device="cuda"))
    r = dict(Kc=_bits(g["Kc"].cpu()).copy(), Vc=_bits(g["Vc"].cpu()).copy(), ids=g["ids"].cpu().numpy().copy(),
             uc=g["uc"].cpu().numpy().copy(), cnt=g["cnt"].cpu().numpy().copy())
    seen = 0
    for n_new in frames:
        cap = n_new + 3
        Kn = torch.zeros(lead + (cap, d), dtype=tdt); Kn[..., :n_new, :] = Kbar[..., seen:seen + n_new, :]
        Vn = torch.zeros(lead + (cap, d), dtype=tdt); Vn[..., :n_new, :] = Vbar[..., seen:seen + n_new, :]
        un = torch.zeros(lead + (cap,)); un[..., :n_new] = util[..., seen:seen + n_new]
        kb.kvev_retain(sh, k, k_cap, Kn.cuda(), Vn.cuda(), un.cuda(), cap, seen, n_new, g["Kc"], g["Vc"], g["ids"],
                       g["uc"], g["cnt"])
        torch.cuda.synchronize()
        orc.retain(Kn, Vn, un, seen, n_new, k, r["Kc"], r["Vc"], r["ids"], r["uc"], r["cnt"])
        seen += n_new
        cnt = g["cnt"].cpu().numpy()
        assert (cnt == r["cnt"]).all() and (cnt == min(k, seen)).all()
        ids, uc, Kc, Vc = g["ids"].cpu().numpy(), g["uc"].cpu().numpy(), _bits(g["Kc"].cpu()), _bits(g["Vc"].cpu())
        for s_ in np.ndindex(lead):
            m = cnt[s_]
            assert (ids[s_][:m] == r["ids"][s_][:m]).all()
            assert np.array_equal(uc[s_][:m], r["uc"][s_][:m], equal_nan=True)
            assert (Kc[s_][:m] == r["Kc"][s_][:m]).all() and (Vc[s_][:m] == r["Vc"][s_][:m]).all()
    # and the store is the cold top-k over everything that was fed
    if k > 0:
        idx, c = orc.select_topk(util, N, 1, 0, k, k_cap)
        assert (g["ids"].cpu().numpy()[..., :min(k, N)] == idx[..., :min(k, N)]).all()


@pytest.mark.parametrize("number,Tq", [(1, 2), (2, 1), (2, 48)])
def test_compact_attention_gives_the_bits_of_the_indexed_attention(number, Tq):
    """Cold step, then evict: the kept summaries move into the compact store (one retain call over all
    candidates), the window into a buffer of its own; attention over those equals the indexed one bit for bit."""
    cfg = synth.CONFIGS[number].replace(Tq=Tq)
    t = synth.make_inputs(cfg, "cpu")
    g = dev(t)
    st = kb.DecodeState(cfg)
    O = torch.empty_like(g["Q"])
    kb.cold_step(st, g, O)
    n_cand, win0 = cfg.N_cand, cfg.N_cand * cfg.C
    lead = (cfg.L, cfg.B, cfg.H)
    k_cap = cfg.k + 2
    Kc = torch.zeros(lead + (k_cap, cfg.d), dtype=cfg.torch_dtype, device="cuda")
    Vc = torch.zeros_like(Kc)
    ids = torch.full(lead + (k_cap,), -1, dtype=torch.int32, device="cuda")
    uc = torch.zeros(lead + (k_cap,), dtype=torch.float32, device="cuda")
    cnt = torch.zeros(lead, dtype=torch.int32, device="cuda")
    kb.kvev_retain(st.shape, cfg.k, k_cap, st.Kbar, st.Vbar, st.util, st.N_cap, 0, n_cand, Kc, Vc, ids, uc, cnt)
    torch.cuda.synchronize()
    assert (cnt == st.count).all()
    assert (ids[..., :cfg.k] == st.idx[..., :cfg.k]).all()
    W_cap = cfg.T - win0 + 5
    Kw = torch.zeros(lead + (W_cap, cfg.d), dtype=cfg.torch_dtype, device="cuda")
    Vw = torch.zeros_like(Kw)
    Kw[..., :cfg.T - win0, :] = g["K"][..., win0:cfg.T, :]
    Vw[..., :cfg.T - win0, :] = g["V"][..., win0:cfg.T, :]
    shw = kb.make_shape(cfg, T=cfg.T - win0, T_cap=W_cap, N_cap=k_cap)
    ws = kb.alloc_workspace(kb.workspace_bytes(kb.OP_COMPACT_ATTENTION, shw, Tq, k_cap))
    O2 = torch.empty_like(O)
    kb.kvev_compact_attention(shw, g["Q"], Tq, Kw, Vw, Kc, Vc, cnt, k_cap, O2, ws)
    torch.cuda.synchronize()
    assert (_bits(O2) == _bits(O)).all()
    ref = orc.compact_attention(t["Q"], Kw.cpu(), Vw.cpu(), cfg.T - win0, Kc.cpu(), Vc.cpu(), cnt.cpu())
    assert_close_storage(O2, ref, cfg.dtype, "O (compact store)")
    # the window buffer as a ring that wraps: same rows, rotated; same bits
    wl, first = cfg.T - win0, W_cap - 3
    rows = (first + torch.arange(wl, device="cuda")) % W_cap
    Kr, Vr = torch.zeros_like(Kw), torch.zeros_like(Vw)
    Kr[..., rows, :] = Kw[..., :wl, :]
    Vr[..., rows, :] = Vw[..., :wl, :]
    O5 = torch.empty_like(O)
    kb.kvev_compact_attention(shw, g["Q"], Tq, Kr, Vr, Kc, Vc, cnt, k_cap, O5, ws, win_first=first)
    torch.cuda.synchronize()
    assert (_bits(O5) == _bits(O2)).all()
    if Tq > 1:
        kb.kvev_compact_attention(shw, g["Q"], Tq, Kr, Vr, Kc, Vc, cnt, k_cap, O5, ws, causal=1, win_first=first)
        torch.cuda.synchronize()
        ref_r = orc.compact_attention(t["Q"], Kr.cpu(), Vr.cpu(), wl, Kc.cpu(), Vc.cpu(), cnt.cpu(), causal=1, win_first=first)
        assert_close_storage(O5, ref_r, cfg.dtype, "O (compact store, ring window, causal frame)")
    # a causal frame (the queries are the window's last Tq tokens): same bits as the indexed causal form, and the oracle's values
    if Tq > 1:
        O3, O4 = torch.empty_like(O), torch.empty_like(O)
        kb.kvev_gated_attention(st.shape, g["Q"], Tq, g["K"], g["V"], st.Kbar, st.Vbar, st.idx, st.count, st.k_cap, O3, st.ws_attn, causal=1)
        kb.kvev_compact_attention(shw, g["Q"], Tq, Kw, Vw, Kc, Vc, cnt, k_cap, O4, ws, causal=1)
        torch.cuda.synchronize()
        assert (_bits(O4) == _bits(O3)).all() and not (_bits(O4) == _bits(O2)).all()
        ref_c = orc.compact_attention(t["Q"], Kw.cpu(), Vw.cpu(), cfg.T - win0, Kc.cpu(), Vc.cpu(), cnt.cpu(), causal=1)
        assert_close_storage(O4, ref_c, cfg.dtype, "O (compact store, causal frame)")


def test_evicting_stream_equals_the_full_cache_stream():
    """Frames arrive; what is resident is only the compact store (k rows), a window buffer (W + one frame)
    and a short staging area for chunks that are pooled but still inside the window.  After every frame the
    attention output equals, bit for bit, the one of the path that keeps the whole cache and re-selects."""
    cfg = synth.Config(171, "evict_stream", "bf16", L=1, B=2, H=3, d=128, T=2048, C=32, k=6, W=256,
                       d_sum=128, d_g=64, Tq=1, steps=8, frame=256, decode_per_step=1)
    t = synth.make_inputs(cfg, "cpu")
    g = dev(t)
    lead = (cfg.L, cfg.B, cfg.H)
    full = kb.DecodeState(cfg, T_cap=cfg.T)                     # the non-evicting reference path (whole cache)
    k_cap = cfg.k
    Kc = torch.zeros(lead + (k_cap, cfg.d), dtype=cfg.torch_dtype, device="cuda")
    Vc = torch.zeros_like(Kc)
    ids = torch.full(lead + (k_cap,), -1, dtype=torch.int32, device="cuda")
    uc = torch.zeros(lead + (k_cap,), dtype=torch.float32, device="cuda")
    cnt = torch.zeros(lead, dtype=torch.int32, device="cuda")
    W_cap = cfg.W + cfg.frame + cfg.C
    Kw = torch.zeros(lead + (W_cap, cfg.d), dtype=cfg.torch_dtype, device="cuda")
    Vw = torch.zeros_like(Kw)
    O1, O2 = torch.empty_like(g["Q"]), torch.empty_like(g["Q"])
    n_old, ncand_old = 0, 0
    resident_max = 0
    wrapped = False
    for step in range(cfg.steps):
        T = (step + 1) * cfg.frame
        N, n_cand = T // cfg.C, max(0, T - cfg.W) // cfg.C
        # ---- reference path: whole cache, pool + gate the new chunks, select over all candidates, indexed attention
        sh = full.shape
        sh.T = T
        kb.kvev_chunk_pool(sh, g["K"], g["V"], kb.POOL_MLP, kb.mlp_weights(g, "K"), kb.mlp_weights(g, "V"), n_old, N,
                           full.Kbar, full.Vbar, full.ws)
        kb.kvev_lstm_gate(sh, full.Kbar, full.Vbar, kb.lstm_weights(g), n_old, N, full.h, full.c, full.util, full.gate,
                          full.ws)
        kb.kvev_select(sh, full.util, full.gate, kb.SELECT_TOPK, cfg.k, 0.0, full.k_cap, full.idx, full.count)
        kb.kvev_gated_attention(sh, g["Q"], 1, g["K"], g["V"], full.Kbar, full.Vbar, full.idx, full.count, full.k_cap,
                                O1, full.ws_attn)
        # ---- evicting path: chunks that left the window this frame enter the store, the window is rebased
        n_in = n_cand - ncand_old
        if n_in > 0:
            Kn = full.Kbar[..., ncand_old:n_cand, :].contiguous()      # staging: pooled earlier, candidates only now
            Vn = full.Vbar[..., ncand_old:n_cand, :].contiguous()
            un = full.util[..., ncand_old:n_cand].contiguous()
            kb.kvev_retain(sh, cfg.k, k_cap, Kn, Vn, un, n_in, ncand_old, n_in, Kc, Vc, ids, uc, cnt)
        win0 = n_cand * cfg.C
        # what a caller keeps of the raw cache: a ring in which token p sits in row p mod W_cap; the frame is
        # appended behind the last token, the window start just advances (no row moves)
        rows = torch.arange(T - cfg.frame, T, device="cuda") % W_cap
        Kw[..., rows, :] = g["K"][..., T - cfg.frame:T, :]
        Vw[..., rows, :] = g["V"][..., T - cfg.frame:T, :]
        wrapped = wrapped or (win0 % W_cap) + (T - win0) > W_cap
        shw = kb.make_shape(cfg, T=T - win0, T_cap=W_cap, N_cap=k_cap)
        ws = kb.alloc_workspace(kb.workspace_bytes(kb.OP_COMPACT_ATTENTION, shw, 1, k_cap))
        kb.kvev_compact_attention(shw, g["Q"], 1, Kw, Vw, Kc, Vc, cnt, k_cap, O2, ws, win_first=win0 % W_cap)
        torch.cuda.synchronize()
        assert (cnt == full.count).all(), step
        m = int(cnt.max())
        assert (ids[..., :m] == full.idx[..., :m]).all(), step
        assert (_bits(O2) == _bits(O1)).all(), step
        resident_max = max(resident_max, k_cap + T - win0)
        n_old, ncand_old = N, n_cand
    ratio = cfg.T / (cfg.k + cfg.T - (max(0, cfg.T - cfg.W) // cfg.C) * cfg.C)
    print(f"\n[evicting stream] resident rows <= {resident_max} of {cfg.T} cached tokens; n/(W+M) = {ratio:.1f}")
    assert resident_max <= cfg.k + cfg.W + cfg.C
    assert wrapped                      # the window did run across the end of its ring buffer

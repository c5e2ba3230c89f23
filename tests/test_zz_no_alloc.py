"""kvev_gated_attention_static: the entry point for callers that cannot allocate (its split scratch is an
array inside the library).  Checked through the C ABI against kvev_gated_attention on two calls in a row, the
second with a smaller input, both of which split their rows over several workgroups and so use the scratch."""
import numpy as np
import pytest
import torch

from oracle import kvev_oracle as orc
from paper_2509_21354_amd import binding as kb
from paper_2509_21354_amd import synth
from tests.helpers import assert_close_storage, dev

pytestmark = pytest.mark.gpu


def _case(number, T, W, k, H, Tq, dtype="bf16", d=128):
    cfg = synth.Config(number, f"static{number}", dtype, L=1, B=1, H=H, d=d, T=T, C=32, k=k, W=W,
                       d_sum=32, d_g=64, Tq=Tq)
    t = synth.make_qkv(cfg, "cpu")
    rng = np.random.default_rng(number)
    N_cap = cfg.N
    lead = (cfg.L, cfg.B, cfg.H)
    Kbar = torch.randn(lead + (N_cap, cfg.d), generator=torch.Generator().manual_seed(number)).to(cfg.torch_dtype)
    Vbar = torch.randn(lead + (N_cap, cfg.d), generator=torch.Generator().manual_seed(number + 1)).to(cfg.torch_dtype)
    n_cand = cfg.N_cand
    idx = np.zeros(lead + (k,), dtype=np.int32)
    count = np.zeros(lead, dtype=np.int32)
    for s in np.ndindex(lead):
        c = int(rng.integers(0, min(k, n_cand) + 1))
        count[s] = c
        idx[s][:c] = np.sort(rng.choice(n_cand, size=c, replace=False))
    return cfg, t, Kbar, Vbar, torch.from_numpy(idx), torch.from_numpy(count)


def _run_both(cfg, t, Kbar, Vbar, idx, count):
    g = dev(t)
    sh = kb.make_shape(cfg)
    k_cap = idx.shape[-1]
    need = kb.workspace_bytes(kb.OP_GATED_ATTENTION, sh, cfg.Tq, k_cap)
    assert 0 < need <= kb.STATIC_SCRATCH_BYTES, need          # the launch splits: the scratch is really used
    ws = kb.alloc_workspace(need)
    gK, gV, gi, gc = Kbar.cuda(), Vbar.cuda(), idx.cuda(), count.cuda()
    O_ref = torch.full_like(g["Q"], 7.0)
    O_new = torch.full_like(g["Q"], -7.0)
    kb.kvev_gated_attention(sh, g["Q"], cfg.Tq, g["K"], g["V"], gK, gV, gi, gc, k_cap, O_ref, ws)
    kb.kvev_gated_attention_static(sh, g["Q"], cfg.Tq, g["K"], g["V"], gK, gV, gi, gc, k_cap, O_new)
    torch.cuda.synchronize()
    # the same kernels over the same rows in the same order: the same bits
    assert torch.equal(O_ref.view(torch.int16 if cfg.dtype == "bf16" else torch.int32),
                       O_new.view(torch.int16 if cfg.dtype == "bf16" else torch.int32))
    want = orc.gated_attention(t["Q"], t["K"], t["V"], Kbar, Vbar, idx, count, cfg.T, cfg.C, cfg.W)
    assert_close_storage(O_new, want, cfg.dtype, f"{cfg.name}: static-scratch attention vs oracle")


def test_static_scratch_entry_matches_the_workspace_entry_twice_in_a_row():
    big = _case(301, T=6000, W=4096, k=24, H=3, Tq=1)
    small = _case(302, T=2300, W=1500, k=8, H=2, Tq=2)
    _run_both(*big)
    _run_both(*small)          # smaller input over the same array: whatever the first call left must not matter
    _run_both(*big)

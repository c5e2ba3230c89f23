"""The end-to-end rule for kept indices (tests/helpers.index_protocol) on the CPU: the comparison itself is
checked with stand-ins for the GPU's results that are made from the oracle, so that each of its three outcomes
(tie, traced to a stored summary, failure) is seen to come out where it should."""
import numpy as np
import pytest

from oracle import kvev_oracle as orc
from paper_2509_21354_amd import binding as kb
from paper_2509_21354_amd import synth
from tests.helpers import index_protocol

CFG = synth.Config(170, "index_protocol_small", "bf16", L=1, B=2, H=3, d=64, T=1344, C=16, k=30, W=64,
                   d_sum=32, d_g=32, Tq=1)


def _chain():
    t = synth.make_inputs(CFG, "cpu")
    r = orc.cold_step(t["Q"], t["K"], t["V"], t, CFG.T, CFG.C, CFG.W, CFG.k, CFG.d_sum)
    return t, r


def _protocol(name, idx, cnt, r, Kbar, Vbar, t):
    return index_protocol(name, idx, cnt, r, Kbar, Vbar, kb.lstm_weights(t), CFG.T, CFG.C, CFG.W, CFG.k, CFG.k)


def test_identical_chains_pass_without_remarks():
    t, r = _chain()
    rec = _protocol("identical", r["idx"], r["count"], r, r["Kbar"], r["Vbar"], t)
    assert rec["index_mismatching"] == 0 and not rec["ties"] and not rec["traced_to_stored_summary"]


def test_swap_caused_by_stored_summary_rounding_is_traced():
    """Stand-in for a GPU whose stored summaries differ from the oracle's in the last bit: the oracle's own gate and
    selection on those summaries give its kept set.  Where that set differs from the reference chain's, the rule
    must find the differing stored element and accept the swap as decided upstream."""
    t, r = _chain()
    rng = np.random.default_rng(7)
    N = CFG.N
    for attempt in range(40):
        Kb = r["Kbar"].copy()
        flip = rng.random(Kb.shape) < 0.5
        Kb[flip] = Kb[flip] ^ np.uint16(1 + attempt // 10)     # the last place(s) of the stored bf16 value
        _, _, util, _ = orc.lstm_gate(Kb, r["Vbar"], kb.lstm_weights(t), 0, N)
        idx, cnt = orc.select_topk(util, CFG.T, CFG.C, CFG.W, CFG.k, CFG.k)
        if (idx != r["idx"]).any():
            break
    else:
        pytest.skip("no perturbation changed a kept set")
    rec = _protocol("traced", idx, cnt, r, Kb, r["Vbar"], t)
    assert rec["index_mismatching"] > 0
    assert len(rec["ties"]) + len(rec["traced_to_stored_summary"]) == rec["index_mismatching"]
    for e in rec["traced_to_stored_summary"]:
        assert e["differing_stored_elements"] > 0 and e["oracle_gap"] > 1e-6


def test_swap_with_identical_summaries_fails():
    """Same stored summaries on both sides, yet a different kept set with a clear utility gap: the gate or the
    selection is wrong, and the rule says so."""
    t, r = _chain()
    idx = r["idx"].copy()
    s0 = (0, 0, 0)
    kept = set(idx[s0][:r["count"][s0]].tolist())
    u = r["util"][s0]
    n_cand = CFG.N_cand
    worst_dropped = min((c for c in range(n_cand) if c not in kept), key=lambda c: u[c])
    best_kept = max(kept, key=lambda c: u[c])
    assert u[best_kept] - u[worst_dropped] > 1e-3
    new = sorted((kept - {best_kept}) | {worst_dropped})
    idx[s0][:len(new)] = new
    with pytest.raises(AssertionError):
        _protocol("planted failure", idx, r["count"], r, r["Kbar"], r["Vbar"], t)


def test_tie_within_1e6_is_reported_not_failed():
    t, r = _chain()
    s0 = (0, 0, 0)
    idx = r["idx"].copy()
    kept = idx[s0][:r["count"][s0]].tolist()
    u = r["util"].copy()
    dropped = next(c for c in range(CFG.N_cand) if c not in kept)
    u[s0][dropped] = u[s0][kept[0]] - 5e-7            # the reference's scores say: these two are a tie
    ref = dict(r)
    ref["util"] = u
    new = sorted(set(kept[1:]) | {dropped})
    idx[s0][:len(new)] = new
    rec = _protocol("tie", idx, r["count"], ref, r["Kbar"], r["Vbar"], t)
    assert rec["index_mismatching"] == 1 and len(rec["ties"]) == 1 and not rec["failures"]


def test_count_mismatch_fails():
    t, r = _chain()
    cnt = r["count"].copy()
    cnt[0, 0, 0] -= 1
    with pytest.raises(AssertionError):
        _protocol("count", r["idx"], cnt, r, r["Kbar"], r["Vbar"], t)

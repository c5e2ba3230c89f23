"""Shared pieces of the GPU parity tests: tolerance rules and device staging."""
import json
import os

import numpy as np
import torch

from oracle import kvev_oracle as orc


def dev(t):
    return {k: v.cuda() for k, v in t.items()}


def vals(x):
    """float64 numpy values of a torch tensor / oracle array in either storage form."""
    return orc.from_bits(orc.to_np(x))


def worst_rel_error(got, ref):
    """max over elements of |got - ref| / max(|ref|, rms(ref)): the quantity the bf16 bar (2e-2) bounds."""
    g, r = vals(got), vals(ref)
    if g.size == 0:
        return 0.0
    rms = float(np.sqrt(np.mean(r * r)))
    return float((np.abs(g - r) / np.maximum(np.maximum(np.abs(r), rms), 1e-30)).max())


def assert_close_storage(got, ref, dtype, what=""):
    """The stated bars: fp32 storage max-abs 1e-4; bf16 storage 'relative 2e-2',
    read per tensor as |got-ref| <= 2e-2 * max(|ref|, rms(ref)) element-wise."""
    g, r = vals(got), vals(ref)
    assert g.shape == r.shape, (what, g.shape, r.shape)
    assert np.isfinite(g).all(), what
    if g.size == 0:
        return 0.0
    err = np.abs(g - r)
    if dtype == "f32":
        assert err.max() <= 1e-4, f"{what}: max abs err {err.max():.3e} > 1e-4"
    else:
        rms = float(np.sqrt(np.mean(r * r)))
        bound = 2e-2 * np.maximum(np.abs(r), rms)
        worst = float((err / np.maximum(bound, 1e-30)).max())
        assert (err <= bound).all(), f"{what}: bf16 rel err {worst * 2e-2:.3e} of the 2e-2 bound"
    return float(err.max())


def bf16_ulp_mismatch(got, ref):
    """Stored-bf16 comparison for fp32-grade pipelines: returns the fraction of
    elements whose bits differ and the largest difference in units of one bf16
    ulp of max(|ref|, 1% of rms(ref)) (the floor keeps results that are tiny by
    cancellation from counting many 'ulps' for an absolute error of 1e-8)."""
    g, r = vals(got), vals(ref)
    differs = orc.to_np(got) != orc.to_np(ref)
    if g.size == 0:
        return 0.0, 0.0
    rms = float(np.sqrt(np.mean(r * r)))
    scale = np.maximum(np.abs(r), 0.01 * rms)
    ulp = 2.0 ** (np.floor(np.log2(np.maximum(scale, 1e-30))) - 7)
    return float(differs.mean()), float((np.abs(g - r) / ulp).max())


def index_report(idx_gpu, cnt_gpu, idx_ref, cnt_ref, util_ref):
    """End-to-end index comparison: returns (n_sequences, n_mismatching, worst
    oracle utility gap among swapped chunks, list of details)."""
    idx_gpu, cnt_gpu = orc.to_np(idx_gpu), orc.to_np(cnt_gpu)
    S = int(np.prod(cnt_ref.shape))
    ig = idx_gpu.reshape(S, -1)
    ir = idx_ref.reshape(S, -1)
    cg, cr = cnt_gpu.reshape(S), cnt_ref.reshape(S)
    u = util_ref.reshape(S, -1)
    bad, worst, details = 0, 0.0, []
    for s in range(S):
        a, b = set(ig[s, :cg[s]].tolist()), set(ir[s, :cr[s]].tolist())
        if cg[s] != cr[s]:
            bad += 1
            worst = float("inf")
            details.append((s, "count", int(cg[s]), int(cr[s])))
            continue
        if a != b:
            bad += 1
            only_g, only_r = sorted(a - b), sorted(b - a)
            gap = max(abs(float(u[s, x]) - float(u[s, y])) for x in only_g for y in only_r)
            worst = max(worst, gap)
            details.append((s, only_g, only_r, gap))
    return S, bad, worst, details


# Lines the parity tests want in the test log whatever pytest's verbosity (conftest.py prints them in the
# terminal summary) and in a file next to the other outputs of a GPU run.
REPORTS = []


def report(line, record=None):
    REPORTS.append(line)
    if record is not None:
        root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
        out = os.path.join(root, "gpurun_out")
        try:
            os.makedirs(out, exist_ok=True)
            with open(os.path.join(out, "parity_report.jsonl"), "a") as f:
                f.write(json.dumps(record) + "\n")
        except OSError:
            pass


TIE_GAP = 1e-6


def index_protocol(name, idx_gpu, cnt_gpu, ref, Kbar_gpu, Vbar_gpu, lstm_w, T, C, W, k, k_cap):
    """The end-to-end rule for kept indices (independent chains: each side's own summaries and scores).
    Kept sets must be identical, except that
      * chunks whose utilities differ by at most 1e-6 in the oracle may swap (a tie: reported), and
      * a wider swap passes only if it is traced to the stored summaries: some element of the sequence's stored
        summaries differs between GPU and oracle (a rounding flip of the storage dtype), and the oracle's own gate
        and selection, run on the GPU's stored summaries, reproduce the GPU's kept set (up to ties in those
        scores).  Then the difference was decided upstream by a stored rounding, not in the gate or the selection.
    Anything else fails.  Returns the record that is also written to the report."""
    S, bad, worst, details = index_report(idx_gpu, cnt_gpu, ref["idx"], ref["count"], ref["util"])
    rec = {"test": name, "sequences": S, "index_mismatching": bad, "worst_oracle_gap": worst if bad else 0.0,
           "ties": [], "traced_to_stored_summary": [], "failures": []}
    if bad:
        N = T // C
        kb_np, vb_np = orc.to_np(Kbar_gpu), orc.to_np(Vbar_gpu)
        _, _, util2, _ = orc.lstm_gate(Kbar_gpu, Vbar_gpu, lstm_w, 0, N)
        idx2, cnt2 = orc.select_topk(util2, T, C, W, k, k_cap)
        ig, cg = orc.to_np(idx_gpu).reshape(S, -1), orc.to_np(cnt_gpu).reshape(S)
        i2, c2, u2 = idx2.reshape(S, -1), cnt2.reshape(S), util2.reshape(S, -1)
        kd = (kb_np != ref["Kbar"]).reshape(S, -1)
        vd = (vb_np != ref["Vbar"]).reshape(S, -1)
        for d in details:
            s = d[0]
            if d[1] == "count":
                rec["failures"].append({"sequence": s, "why": "kept count differs", "gpu": d[2], "oracle": d[3]})
                continue
            _, only_g, only_r, gap = d
            if gap <= TIE_GAP:
                rec["ties"].append({"sequence": s, "gpu_only": only_g, "oracle_only": only_r, "oracle_gap": gap})
                continue
            flips = int(kd[s].sum() + vd[s].sum())
            a, b = set(ig[s, :cg[s]].tolist()), set(i2[s, :c2[s]].tolist())
            regap = max([abs(float(u2[s, x]) - float(u2[s, y])) for x in a - b for y in b - a], default=0.0)
            if flips > 0 and (a == b or regap <= TIE_GAP):
                where = int(np.flatnonzero(kd[s] | vd[s])[0])
                rec["traced_to_stored_summary"].append(
                    {"sequence": s, "gpu_only": only_g, "oracle_only": only_r, "oracle_gap": gap,
                     "differing_stored_elements": flips, "first_differing_element": where,
                     "oracle_on_gpu_summaries_reproduces_gpu_set": True})
            else:
                rec["failures"].append({"sequence": s, "gpu_only": only_g, "oracle_only": only_r, "oracle_gap": gap,
                                        "differing_stored_elements": flips, "rescored_gap": regap})
    report(f"[index parity] {name}: {S} sequences, {bad} with a different kept set "
           f"({len(rec['ties'])} ties <= 1e-6, {len(rec['traced_to_stored_summary'])} traced to a stored-summary "
           f"rounding, {len(rec['failures'])} failures), worst oracle gap {rec['worst_oracle_gap']:.3e}", rec)
    assert not rec["failures"], rec["failures"]
    return rec

"""Shared pieces of the GPU parity tests: tolerance rules and device staging."""
import numpy as np
import torch

from oracle import kvev_oracle as orc


def dev(t):
    return {k: v.cuda() for k, v in t.items()}


def vals(x):
    """float64 numpy values of a torch tensor / oracle array in either storage form."""
    return orc.from_bits(orc.to_np(x))


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

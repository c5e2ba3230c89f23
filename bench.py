#!/usr/bin/env python3
"""Benchmark of the gated chunked-KV decode step on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload cfg3]

One "step" is one pass of the whole hot path over one batch of seeded synthetic
input already resident in HBM: pool every completed chunk (Eq. 2), run the LSTM
gate from a zero state (Eq. 3), keep the top-k chunks, attend the new query over
kept summaries + raw window (section 3.3).  The headline workload is the largest
single-GPU configuration: the full 32-layer decode step at Llama-2-7B shapes,
batch 8 (config 3), all layers in one launch per stage.  The headline value is
tokens/s per layer = B*Tq*L / t_step.  Small configurations rotate their input
sets (more than the 256 MB memory-side cache in total) so that the cache is
really read from HBM; config 3's 34 GB of KV need no rotation.

Printed as ONE JSON line: the contract keys plus
  roofline      dominant kernel of the step (largest share) against its roof
  rooflines     the same object for every stage, the steady-state attention and
                the dense baseline
  steady_state  gated attention alone (the step between two re-gating triggers)
  dense         full-cache attention on the same inputs, the speed-ups and the
                break-even (decode steps per re-gating trigger)
  cfg2, cfg5, streaming_cfg4   the other configurations as sub-records
  cpu_baseline  the CPU oracle timed on this host on a sample of the same workload
  paper_context the paper's own whole-model numbers (other hardware; context)
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time
from concurrent.futures import ThreadPoolExecutor

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK_HBM_GBS = 8000.0          # MI355X HBM3E
PEAK_BF16_TFLOPS = 2500.0      # dense bf16 MFMA
PEAK_F32_TFLOPS = 157.3


def costs(cfg, T=None):
    """Algorithmic bytes / flops of each stage for one step (what the method
    must move or compute; re-reads and padding are not counted)."""
    T = cfg.T if T is None else T
    S, d, es = cfg.L * cfg.B * cfg.H, cfg.d, cfg.elem_size
    N = T // cfg.C
    n_cand = max(0, T - cfg.W) // cfg.C
    k_eff = min(cfg.k, n_cand)
    n_att = k_eff + T - n_cand * cfg.C
    return {
        "pool": {"bytes": S * N * (2 * cfg.C * d * es + 2 * d * es),
                 "flops": S * N * (8 * d * cfg.d_sum + 2 * cfg.C * d)},
        "gate": {"bytes": S * N * (2 * d * es + 8), "flops": S * N * (2 * 2 * d * 4 * cfg.d_g + 2 * cfg.d_g * 4 * cfg.d_g),
                 "steps": N},
        "select": {"bytes": S * (4 * n_cand + 4 * k_eff + 4), "flops": 0},
        "attend": {"bytes": S * (2 * n_att * d * es + 2 * cfg.Tq * d * es + 4 * k_eff),
                   "flops": S * cfg.Tq * 4 * n_att * d, "rows": n_att},
        "dense": {"bytes": S * (2 * T * d * es + 2 * cfg.Tq * d * es), "flops": S * cfg.Tq * 4 * T * d},
    }


def measured_traffic(workload, stage):
    """HBM bytes per launch measured with rocprofv3 --pmc (FETCH_SIZE + WRITE_SIZE, scaled by
    the copy-kernel reading) in runs of their own (counters cannot ride in a timed run); the
    figures are kept as data under profiles/ and repeated here, not observed by this run."""
    path = os.path.join(ROOT, "profiles", "hbm_traffic.json")
    try:
        with open(path) as f:
            return json.load(f).get(workload, {}).get(stage)
    except (OSError, ValueError):
        return None


def roof(name, kernel, cost, us, bound, workload=None):
    if bound == "hbm":
        ach, peak, unit = cost["bytes"] / us / 1e3, PEAK_HBM_GBS, "GB/s"
    else:
        ach, peak, unit = cost["flops"] / us / 1e6, PEAK_BF16_TFLOPS, "TFLOP/s"
    r = {"stage": name, "kernel": kernel, "bound": bound, "achieved": round(ach, 3), "peak": peak, "unit": unit,
         "frac": round(ach / peak, 5), "traffic": measured_traffic(workload, name) if workload else None,
         "us_per_launch": round(us, 3), "algorithmic_bytes": cost["bytes"], "algorithmic_flops": cost["flops"]}
    if r["traffic"] is not None:
        r["traffic_source"] = "profiles/hbm_traffic.json (rocprofv3 --pmc, separate runs of this command)"
    return r


def rec_kernel_name(cfg):
    groups = cfg.L * ((cfg.B * cfg.kv_heads + 15) // 16)
    if cfg.d_g == 256 and groups >= 257:
        return f"lstm_fused_kernel<{cfg.d}>"
    bh = cfg.B * cfg.kv_heads
    if cfg.d_g == 512 and bh > 16:      # (more groups than fit at once: several launches of the same kernel)
        return f"lstm_quad_kernel<{cfg.d}>"
    paired = cfg.d_g in (256, 512) and groups <= 128
    return f"lstm_rec_pair_kernel<{cfg.d_g}>" if paired else f"lstm_rec_kernel<{cfg.d_g}>"


def recurrence_occupancy(cfg, gate_us):
    """The recurrence is N dependent steps on the compute units its sequences occupy, so for small launches its
    share of the whole chip's MFMA peak says little.  This is the local figure: clocks the matrix pipe of an
    occupied SIMD needs for one step (two fp16 terms per weight fragment, 16 clocks per 16x16x32 instruction,
    2.4 GHz) over the measured time per step (the whole gate call, so a lower bound on the recurrence kernel's own
    utilisation; profiles/mfma_counters.md has the counter-based figure)."""
    groups = cfg.L * ((cfg.B * cfg.kv_heads + 15) // 16)
    paired = rec_kernel_name(cfg).startswith("lstm_rec_pair")
    fused = rec_kernel_name(cfg).startswith("lstm_fused")
    quad = rec_kernel_name(cfg).startswith("lstm_quad")
    if fused or quad:              # 32 sequences per workgroup (or four of them), the input projection's MFMAs inside the step
        members = 4 if quad else 1
        wgs = members * cfg.L * ((cfg.B * cfg.kv_heads + 31) // 32)
        cus, rounds = min(256, wgs), -(-wgs // 256)
        mfma_per_group_step = 2 * (2 * (4 * cfg.d_g // 16) * (cfg.d_g // 32) + (4 * cfg.d_g // 16) * (2 * cfg.d // 32))
        per_simd = mfma_per_group_step / members / 4 * rounds
    else:
        cus = min(256, groups * (2 if paired else 1))
        rounds = -(-groups * (2 if paired else 1) // 256)
        mfma_per_group_step = 2 * (4 * cfg.d_g // 16) * (cfg.d_g // 32)
        per_simd = mfma_per_group_step / (2 if paired else 1) / 4 * rounds
    us_step = gate_us / cfg.N
    busy_us = per_simd * 16 / 2400.0
    return {"dependent_steps": cfg.N, "us_per_step": round(us_step, 3), "compute_units_occupied": cus,
            "workgroups_per_sequence_group": 4 if quad else 2 if paired else 1, "sequences_per_group": 32 if fused or quad else 16,
            "mfma_pipe_us_per_step_per_simd": round(busy_us, 3), "mfma_pipe_busy_frac_of_occupied_simds": round(busy_us / us_step, 3)}


class Bench:
    """Inputs, caller-owned state and the stage closures of one configuration."""

    def __init__(self, cfg, n_sets=0):
        import torch
        from paper_2509_21354_amd import binding as kb
        from paper_2509_21354_amd import synth
        self.torch, self.kb, self.cfg = torch, kb, cfg
        dev = "cuda"
        S = cfg.L * cfg.B * cfg.H
        kv_bytes = 2 * cfg.L * cfg.B * cfg.kv_heads * cfg.T * cfg.d * cfg.elem_size
        R = n_sets or max(2, min(16, -(-(600 << 20) // kv_bytes)))
        if kv_bytes > (2 << 30):
            R = 1                       # far beyond every cache by itself
        self.S, self.R = S, R
        self.w = synth.make_weights(cfg, dev)
        self.sets = []
        for r in range(R):
            c_r = cfg.replace(number=cfg.number + 10 * r) if r else cfg
            self.sets.append(synth.make_qkv(c_r, dev))
        self.st = kb.DecodeState(cfg)
        self.O = torch.empty_like(self.sets[0]["Q"])
        self.cost = costs(cfg)
        st, w, O = self.st, self.w, self.O
        wK, wV, lw = kb.mlp_weights(w, "K"), kb.mlp_weights(w, "V"), kb.lstm_weights(w)
        self.wK, self.wV, self.lw = wK, wV, lw
        sh, N, Tq = st.shape, cfg.N, cfg.Tq

        def pool(t): kb.kvev_chunk_pool(sh, t["K"], t["V"], kb.POOL_MLP, wK, wV, 0, N, st.Kbar, st.Vbar, st.ws_pool)

        # the gate's weights are static across decode steps: packed once, outside the timed region
        kb.kvev_lstm_prepare(sh, lw, st.packed)

        def gate(t): kb.kvev_lstm_gate_prepared(sh, st.Kbar, st.Vbar, lw, st.packed, 0, N, st.h, st.c, st.util, st.gate, st.ws)

        def select(t): kb.kvev_select(sh, st.util, st.gate, kb.SELECT_TOPK, cfg.k, 0.0, st.k_cap, st.idx, st.count)

        def attend(t): kb.kvev_gated_attention(sh, t["Q"], Tq, t["K"], t["V"], st.Kbar, st.Vbar, st.idx, st.count,
                                               st.k_cap, O, st.ws_attn)

        def dense(t): kb.kvev_dense_attention(sh, t["Q"], Tq, t["K"], t["V"], O, st.ws_attn)

        self.pool, self.gate, self.select, self.attend, self.dense = pool, gate, select, attend, dense
        self.stages = [("pool", pool), ("gate", gate), ("select", select), ("attend", attend)]
        mfma = cfg.dtype == "bf16"
        self.mfma = mfma
        self.kernels = {
            "pool": "pool_mfma_kernel" if mfma and cfg.d_sum % 32 == 0 else "pool_generic_kernel",
            # one kvev_lstm_gate_prepared call (weights packed once, before the timed region) = per scratch block an input
            # projection and a recurrence launch, or the single fused kernel; the HIP events bracket the call
            "gate": (f"{rec_kernel_name(cfg)} (the whole kvev_lstm_gate_prepared call)"
                     if mfma and cfg.d_g in (64, 128, 256, 512) else "lstm_generic_kernel"),
            "select": "select_kernel",
            "attend": "attn_mq_kernel" if mfma and Tq * (cfg.H // cfg.kv_heads) >= 16 else "attn_decode_kernel",
            "dense": "attn_mq_kernel" if mfma and Tq * (cfg.H // cfg.kv_heads) >= 16 else "attn_decode_kernel"}

    def time_alone(self, f, iters):
        torch = self.torch
        for i in range(3):
            f(self.sets[i % self.R])
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for i in range(iters):
            f(self.sets[i % self.R])
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) * 1e3 / iters

    def cold_steps(self, steps, warmup, only=""):
        """W untimed and K timed cold steps; every stage of every step between two HIP events on the stream the
        library enqueues on (torch's current stream).  Returns the timing record."""
        torch, cfg = self.torch, self.cfg
        stages = self.stages
        if only:
            stages = [(n, f) for n, f in self.stages + [("dense", self.dense)] if n == only]
            for n, f in self.stages[:3]:
                f(self.sets[0])                                   # valid state for a later stage run alone

        def run_steps(n, record):
            marks = []
            for i in range(n):
                t = self.sets[i % self.R]
                row = []
                for _, f in stages:
                    if record:
                        e = torch.cuda.Event(enable_timing=True); e.record(); row.append(e)
                    f(t)
                if record:
                    e = torch.cuda.Event(enable_timing=True); e.record(); row.append(e)
                marks.append(row)
            return marks

        run_steps(warmup, False)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        marks = run_steps(steps, True)
        torch.cuda.synchronize()
        wall_ms = (time.perf_counter() - t0) * 1e3 / steps
        stage_us = {n: 0.0 for n, _ in stages}
        for row in marks:
            for j, (n, _) in enumerate(stages):
                stage_us[n] += row[j].elapsed_time(row[j + 1]) * 1e3 / steps
        gpu_ms = marks[0][0].elapsed_time(marks[-1][-1]) / steps
        per_step_us = sorted(row[0].elapsed_time(row[-1]) * 1e3 for row in marks)
        ms_per_step = max(gpu_ms, wall_ms)       # host launch overhead counts when it is the limit
        bounds = {"pool": "hbm", "gate": "mfma", "select": "hbm", "attend": "hbm", "dense": "hbm"}
        rooflines = [roof(n, self.kernels[n], self.cost[n], stage_us[n], bounds[n], cfg.name)
                     for n, _ in stages if stage_us[n] > 0]
        for r in rooflines:
            if r["stage"] == "gate" and self.mfma and cfg.d_g in (64, 128, 256, 512):
                r["recurrence"] = recurrence_occupancy(cfg, r["us_per_launch"])
            if r["stage"] == "attend" and r["kernel"] == "attn_mq_kernel":
                r["mfma"] = {"bound": "mfma", "achieved": round(self.cost["attend"]["flops"] / r["us_per_launch"] / 1e6, 2),
                             "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s",
                             "frac": round(self.cost["attend"]["flops"] / r["us_per_launch"] / 1e6 / PEAK_BF16_TFLOPS, 5)}
        return {"ms_per_step": ms_per_step, "gpu_ms": gpu_ms, "wall_ms": wall_ms, "stage_us": stage_us,
                "per_step_us": per_step_us, "rooflines": rooflines,
                "value": cfg.B * cfg.Tq * cfg.L / (ms_per_step * 1e-3)}

    def steady_and_dense(self, steps, ms_per_step):
        """Gated attention alone (what runs between two re-gating triggers) and the dense baseline, same inputs."""
        cfg, cost = self.cfg, self.cost
        for n, f in self.stages[:3]:
            f(self.sets[0])
        big = cost["dense"]["bytes"] > (8 << 30)
        t_att = self.time_alone(self.attend, max(20 if big else 50, steps))
        t_den = self.time_alone(self.dense, 5 if big else max(20, steps // 2))
        tok = cfg.B * cfg.Tq * cfg.L
        steady = {"us_per_step": round(t_att, 3), "tokens_per_s_per_layer": round(tok / (t_att * 1e-6), 1),
                  "hbm_GBps": round(cost["attend"]["bytes"] / t_att / 1e3, 1),
                  "hbm_frac": round(cost["attend"]["bytes"] / t_att / 1e3 / PEAK_HBM_GBS, 4)}
        # break-even: a re-gating trigger costs one cold step instead of one steady step; it pays for itself after
        # n decode steps with n * (t_dense - t_steady) >= t_cold - t_steady
        t_cold = ms_per_step * 1e3
        gain = t_den - t_att
        dense = {"us_per_step": round(t_den, 3), "tokens_per_s_per_layer": round(tok / (t_den * 1e-6), 1),
                 "hbm_GBps": round(cost["dense"]["bytes"] / t_den / 1e3, 1),
                 "hbm_frac": round(cost["dense"]["bytes"] / t_den / 1e3 / PEAK_HBM_GBS, 4),
                 "speedup_steady_vs_dense": round(t_den / t_att, 2),
                 "speedup_cold_step_vs_dense": round(t_den / t_cold, 4),
                 "break_even_decode_steps_per_regate": round((t_cold - t_att) / gain, 2) if gain > 0 else None}
        r_att = roof("attend_steady_state", self.kernels["attend"], cost["attend"], t_att, "hbm", None)
        r_att["traffic"] = measured_traffic(cfg.name, "attend")
        r_den = roof("dense", self.kernels["dense"], cost["dense"], t_den, "hbm", cfg.name)
        if self.kernels["dense"] == "attn_mq_kernel":
            for r, c in ((r_att, cost["attend"]), (r_den, cost["dense"])):
                r["mfma"] = {"bound": "mfma", "achieved": round(c["flops"] / r["us_per_launch"] / 1e6, 2), "peak": PEAK_BF16_TFLOPS,
                             "unit": "TFLOP/s", "frac": round(c["flops"] / r["us_per_launch"] / 1e6 / PEAK_BF16_TFLOPS, 5)}
        return steady, dense, [r_att, r_den]

    def graph_replays(self, steps, steady):
        """The steady-state step and the whole cold step replayed from HIP graphs (the library neither allocates nor
        synchronises, so a caller can capture it): GPU time without the host launch path.  Every replay of the cold
        step is checked against the eager result.  Reporting extras: never fail the bench on them."""
        torch, cfg, R, st, O = self.torch, self.cfg, self.R, self.st, self.O
        tok = cfg.B * cfg.Tq * cfg.L
        out = {}
        try:
            gr = torch.cuda.CUDAGraph()
            side = torch.cuda.Stream()
            side.wait_stream(torch.cuda.current_stream())
            with torch.cuda.stream(side):
                self.attend(self.sets[0])
                with torch.cuda.graph(gr, stream=side):
                    for i in range(R):
                        self.attend(self.sets[i % R])
            torch.cuda.current_stream().wait_stream(side)
            torch.cuda.synchronize()
            gr.replay()
            torch.cuda.synchronize()
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            reps = max(5, 200 // R)
            e0.record()
            for _ in range(reps):
                gr.replay()
            e1.record()
            torch.cuda.synchronize()
            t_gr = e0.elapsed_time(e1) * 1e3 / (reps * R)
            steady["graph_replay_us_per_step"] = round(t_gr, 3)
            steady["graph_replay_tokens_per_s_per_layer"] = round(tok / (t_gr * 1e-6), 1)
            steady["graph_replay_hbm_GBps"] = round(self.cost["attend"]["bytes"] / t_gr / 1e3, 1)
        except Exception as ex:
            steady["graph_replay_error"] = str(ex)[:200]
        try:
            for n, f in self.stages:
                f(self.sets[0])
            torch.cuda.synchronize()
            ref_O, ref_idx = O.clone(), st.idx.clone()
            grc = torch.cuda.CUDAGraph()
            side = torch.cuda.Stream()
            side.wait_stream(torch.cuda.current_stream())
            with torch.cuda.stream(side):
                for n, f in self.stages:
                    f(self.sets[0])
                with torch.cuda.graph(grc, stream=side):
                    for i in range(R):
                        for n, f in self.stages:
                            f(self.sets[(i + 1) % R])          # the last step of a replay runs on set 0
            torch.cuda.current_stream().wait_stream(side)
            torch.cuda.synchronize()
            ok = True
            for rep in range(3):
                O.zero_(); st.idx.zero_()
                torch.cuda.synchronize()
                grc.replay()
                torch.cuda.synchronize()
                ok = ok and bool((O == ref_O).all()) and bool((st.idx == ref_idx).all())
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            reps = max(3, steps // R)
            e0.record()
            for _ in range(reps):
                grc.replay()
            e1.record()
            torch.cuda.synchronize()
            t_g = e0.elapsed_time(e1) * 1e3 / (reps * R)
            out = {"us_per_step": round(t_g, 3), "tokens_per_s_per_layer": round(tok / (t_g * 1e-6), 1),
                   "replays_equal_eager": ok}
            del grc
        except Exception as ex:
            out = {"error": str(ex)[:200]}
        return out

    def threshold_mode(self, steps, dense_us):
        """The paper's literal retention rule (section 3.2): keep a chunk iff gate >= tau, with tau at the score
        quantile that keeps the paper's average retention ratio (0.687, section 4.1)."""
        torch, kb, cfg, st, O = self.torch, self.kb, self.cfg, self.st, self.O
        sh, Tq, n_cand = st.shape, cfg.Tq, cfg.N_cand
        if n_cand <= 0:
            return None
        for n, f in self.stages[:2]:
            f(self.sets[0])
        torch.cuda.synchronize()
        g_all = st.gate[..., :n_cand].float().flatten()
        stride = max(1, g_all.numel() // (1 << 22))
        tau = float(torch.quantile(g_all[::stride][: 1 << 23], 1.0 - 0.687))
        lead = (cfg.L, cfg.B, cfg.kv_heads)
        idx_t = torch.zeros(lead + (n_cand,), dtype=torch.int32, device="cuda")
        cnt_t = torch.zeros(lead, dtype=torch.int32, device="cuda")
        ws_t = kb.alloc_workspace(kb.workspace_bytes(kb.OP_GATED_ATTENTION, sh, Tq, n_cand), "cuda")
        kb.kvev_select(sh, None, st.gate, kb.SELECT_THRESHOLD, 0, tau, n_cand, idx_t, cnt_t)
        torch.cuda.synchronize()
        M = float(cnt_t.float().mean())
        t_sel = self.time_alone(lambda t: kb.kvev_select(sh, None, st.gate, kb.SELECT_THRESHOLD, 0, tau, n_cand, idx_t, cnt_t), 30)
        t_thr = self.time_alone(lambda t: kb.kvev_gated_attention(sh, t["Q"], Tq, t["K"], t["V"], st.Kbar, st.Vbar, idx_t, cnt_t,
                                                                  n_cand, O, ws_t), max(20, steps))
        n_att = M + cfg.T - n_cand * cfg.C
        out = {"tau": round(tau, 6), "retention": round(M / n_cand, 4), "paper_retention": 0.687,
               "kept_per_sequence_mean": round(M, 2), "attended_rows_mean": round(n_att, 1),
               "select_us": round(t_sel, 3), "attend_us": round(t_thr, 3),
               "kv_rows_ratio_n_over_W_plus_M": round(cfg.T / n_att, 2),
               "speedup_vs_dense": round(dense_us / t_thr, 2)}
        return out

    def eviction(self, steps):
        """Physical eviction (sections 3.2-3.3): compact store + resident window instead of the whole cache."""
        torch, kb, cfg, st, O, R = self.torch, self.kb, self.cfg, self.st, self.O, self.R
        if cfg.N_cand <= 0 or st.k_cap + cfg.N_cand > 4000:
            return None
        sh, Tq = st.shape, cfg.Tq
        for n, f in self.stages[:3]:
            f(self.sets[0])
        lead = (cfg.L, cfg.B, cfg.kv_heads)
        n_cand, win0 = cfg.N_cand, cfg.N_cand * cfg.C
        kc = st.k_cap
        Kc = torch.zeros(lead + (kc, cfg.d), dtype=cfg.torch_dtype, device="cuda"); Vc = torch.zeros_like(Kc)
        ids = torch.full(lead + (kc,), -1, dtype=torch.int32, device="cuda")
        ucs = torch.zeros(lead + (kc,), dtype=torch.float32, device="cuda")
        cn = torch.zeros(lead, dtype=torch.int32, device="cuda")

        def retain_all(t):
            cn.zero_()
            kb.kvev_retain(sh, cfg.k, kc, st.Kbar, st.Vbar, st.util, st.N_cap, 0, n_cand, Kc, Vc, ids, ucs, cn)
        frame_chunks = max(1, min(n_cand, 256 // cfg.C))

        def retain_frame(t):            # one frame's worth of chunks leaving the window
            kb.kvev_retain(sh, cfg.k, kc, st.Kbar, st.Vbar, st.util, st.N_cap, n_cand, frame_chunks, Kc, Vc, ids, ucs, cn)
        t_all = self.time_alone(retain_all, 20)
        retain_all(None)
        t_frame = self.time_alone(retain_frame, 20)
        retain_all(None)
        wlen = cfg.T - win0
        Kw = [t_["K"][..., win0:cfg.T, :].contiguous() for t_ in self.sets]
        Vw = [t_["V"][..., win0:cfg.T, :].contiguous() for t_ in self.sets]
        shw = kb.make_shape(cfg, T=wlen, T_cap=wlen, N_cap=kc)
        wsw = kb.alloc_workspace(kb.workspace_bytes(kb.OP_COMPACT_ATTENTION, shw, Tq, kc), "cuda")
        it = [0]

        def compact_attend(t):
            i = it[0] % R; it[0] += 1
            kb.kvev_compact_attention(shw, self.sets[i]["Q"], Tq, Kw[i], Vw[i], Kc, Vc, cn, kc, O, wsw)
        t_ca = self.time_alone(compact_attend, max(20, steps))
        rows = min(cfg.k, n_cand) + wlen
        es = cfg.elem_size
        S_kv = cfg.L * cfg.B * cfg.kv_heads
        return {"resident_rows_per_sequence": rows, "cached_tokens": cfg.T,
                "memory_ratio_n_over_W_plus_M": round(cfg.T / rows, 2), "paper_memory_reduction": 1.87,
                "resident_kv_bytes": 2 * S_kv * rows * cfg.d * es, "full_kv_bytes": 2 * S_kv * cfg.T * cfg.d * es,
                "retain_all_candidates_us": round(t_all, 3), "retain_one_frame_us": round(t_frame, 3),
                "compact_attention_us": round(t_ca, 3)}

    def aggregators(self, steps):
        """The other aggregators section 3 names (mean, maximum, the MLP on every token), same inputs."""
        kb, cfg, st = self.kb, self.cfg, self.st
        sh = st.shape
        aggs = {}
        S_kv, N_ = cfg.L * cfg.B * cfg.kv_heads, cfg.N
        tokens = S_kv * N_ * cfg.C
        for name, mode in (("mean", kb.POOL_MEAN), ("max", kb.POOL_MAX), ("mlp_of_mean", kb.POOL_MLP),
                           ("mean_of_token_mlp", kb.POOL_TOKEN_MLP)):
            t_a = self.time_alone(lambda t, m=mode: kb.kvev_chunk_pool(sh, t["K"], t["V"], m, self.wK, self.wV, 0, N_,
                                                                       st.Kbar, st.Vbar, st.ws_pool), max(10, steps // 2))
            e = {"us": round(t_a, 3), "hbm_GBps": round(self.cost["pool"]["bytes"] / t_a / 1e3, 1)}
            if mode == kb.POOL_TOKEN_MLP:
                # 2*C*d*d_sum flop per chunk and side on the matrix cores, C*d_sum GELUs per chunk and side on the
                # vector ALUs.  The GELU rate is a diagnostic of this implementation's polynomial (15 issue slots of 4
                # clocks per 64 GELUs), not a roof of the operation.
                gelus = 2 * tokens * cfg.d_sum
                e.update({"layer1_TFLOPs": round(2 * tokens * 2 * cfg.d * cfg.d_sum / t_a / 1e6, 1),
                          "mfma_frac": round(2 * tokens * 2 * cfg.d * cfg.d_sum / t_a / 1e6 / PEAK_BF16_TFLOPS, 4),
                          "G_gelu_per_s": round(gelus / t_a / 1e3, 1)})
            aggs[name] = e
        self.pool(self.sets[0])          # leave the headline aggregator's summaries in place
        return aggs

    def close(self):
        self.sets = None
        self.st = None
        self.O = None
        self.torch.cuda.empty_cache()


def streaming_cfg4(torch, kb, synth):
    """Config 4: a frame of 256 tokens arrives, the 8 chunks it completes are pooled and scored with the carried gate
    state, the kept set is re-selected, 8 action tokens are decoded (section 3.3 trigger); then the same stream with
    physical eviction."""
    dev = "cuda"
    out = {}
    c4 = synth.CONFIGS[4]
    kv4 = synth.make_qkv(c4, dev)
    w4 = synth.make_weights(c4, dev)
    s4 = kb.DecodeState(c4)
    q4 = synth.make_stream_queries(c4, dev)
    O4 = torch.empty_like(kv4["Q"])
    wK4, wV4, lw4 = kb.mlp_weights(w4, "K"), kb.mlp_weights(w4, "V"), kb.lstm_weights(w4)
    sh4 = s4.shape
    kb.kvev_lstm_prepare(sh4, lw4, s4.packed)          # static weights: packed once

    def frame(si, done):
        sh4.T = (si + 1) * c4.frame
        n4 = sh4.T // c4.C
        kb.kvev_chunk_pool(sh4, kv4["K"], kv4["V"], kb.POOL_MLP, wK4, wV4, done, n4, s4.Kbar, s4.Vbar, s4.ws_pool)
        kb.kvev_lstm_gate_prepared(sh4, s4.Kbar, s4.Vbar, lw4, s4.packed, done, n4, s4.h, s4.c, s4.util, s4.gate, s4.ws)
        kb.kvev_select(sh4, s4.util, s4.gate, kb.SELECT_TOPK, c4.k, 0.0, s4.k_cap, s4.idx, s4.count)
        for j in range(c4.decode_per_step):
            kb.kvev_gated_attention(sh4, q4[si, j], 1, kv4["K"], kv4["V"], s4.Kbar, s4.Vbar, s4.idx, s4.count,
                                    s4.k_cap, O4, s4.ws_attn)
        return n4
    for rep in range(2):                      # first pass warms up, second is timed
        s4.hc.zero_()
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        done = 0
        for si in range(c4.steps):
            done = frame(si, done)
        e1.record()
        torch.cuda.synchronize()
    t_frame = e0.elapsed_time(e1) * 1e3 / c4.steps
    O_gated = O4.clone()

    # the same decodes with full-cache attention over everything that has arrived (no pooling, gate or selection)
    def frame_dense(si):
        sh4.T = (si + 1) * c4.frame
        for j in range(c4.decode_per_step):
            kb.kvev_dense_attention(sh4, q4[si, j], 1, kv4["K"], kv4["V"], O4, s4.ws_attn)
    for rep in range(2):
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for si in range(c4.steps):
            frame_dense(si)
        e1.record()
        torch.cuda.synchronize()
    t_fd = e0.elapsed_time(e1) * 1e3 / c4.steps
    O4.copy_(O_gated)
    out["streaming_cfg4"] = {
        "workload": c4.name + f" ({c4.steps} frames of {c4.frame} tokens, {c4.decode_per_step} decoded tokens per frame, "
                              f"cache grows to {c4.T} tokens)",
        "us_per_frame": round(t_frame, 2),
        "decoded_tokens_per_s_per_layer": round(c4.B * c4.decode_per_step / (t_frame * 1e-6), 1),
        "frames_per_s": round(1e6 / t_frame, 1),
        "dense_us_per_frame": round(t_fd, 2),
        "speedup_vs_dense_stream": round(t_fd / t_frame, 2),
        "note": "the gated frame includes pooling, gating and re-selection of the new frame; the dense frame is the "
                "same decodes over the whole cache that has arrived, averaged over the growing stream"}
    # the same stream with physical eviction: resident are the compact store (k rows), a ring of W + 2 frames
    # raw rows and the summaries of chunks still inside the window; chunks that leave the window are merged
    # into the store (no re-selection over all candidates), the decodes read store + ring
    lead4 = (c4.L, c4.B, c4.H)
    ring_cap = ((c4.W + c4.frame + c4.C + c4.frame - 1) // c4.frame + 1) * c4.frame
    kc4 = c4.k
    Kc4 = torch.zeros(lead4 + (kc4, c4.d), dtype=c4.torch_dtype, device=dev); Vc4 = torch.zeros_like(Kc4)
    id4 = torch.full(lead4 + (kc4,), -1, dtype=torch.int32, device=dev)
    uc4 = torch.zeros(lead4 + (kc4,), dtype=torch.float32, device=dev)
    cn4 = torch.zeros(lead4, dtype=torch.int32, device=dev)
    Kr4 = torch.zeros(lead4 + (ring_cap, c4.d), dtype=c4.torch_dtype, device=dev); Vr4 = torch.zeros_like(Kr4)
    shr = kb.make_shape(c4, T=0, T_cap=ring_cap, N_cap=kc4)
    shr.T = min(c4.W + c4.frame + c4.C, ring_cap)
    wsr = kb.alloc_workspace(kb.workspace_bytes(kb.OP_COMPACT_ATTENTION, shr, 1, kc4), dev)

    def frame_evict(si, done, ncand_old):
        T4 = (si + 1) * c4.frame
        sh4.T = T4
        n4 = T4 // c4.C
        r0 = (T4 - c4.frame) % ring_cap          # token p lives in ring row p mod ring_cap: a frame never wraps
        Kr4[..., r0:r0 + c4.frame, :] = kv4["K"][..., T4 - c4.frame:T4, :]     # stands for the model's cache write
        Vr4[..., r0:r0 + c4.frame, :] = kv4["V"][..., T4 - c4.frame:T4, :]
        kb.kvev_chunk_pool(sh4, kv4["K"], kv4["V"], kb.POOL_MLP, wK4, wV4, done, n4, s4.Kbar, s4.Vbar, s4.ws_pool)
        kb.kvev_lstm_gate_prepared(sh4, s4.Kbar, s4.Vbar, lw4, s4.packed, done, n4, s4.h, s4.c, s4.util, s4.gate, s4.ws)
        ncand = max(0, T4 - c4.W) // c4.C
        if ncand > ncand_old:
            kb.kvev_retain(sh4, c4.k, kc4, kb.RowsFrom(s4.Kbar, ncand_old, c4.d), kb.RowsFrom(s4.Vbar, ncand_old, c4.d),
                           kb.RowsFrom(s4.util, ncand_old, 1), s4.N_cap, ncand_old, ncand - ncand_old, Kc4, Vc4, id4, uc4, cn4)
        win0 = ncand * c4.C
        shr.T = T4 - win0
        for j in range(c4.decode_per_step):
            kb.kvev_compact_attention(shr, q4[si, j], 1, Kr4, Vr4, Kc4, Vc4, cn4, kc4, O4, wsr, win_first=win0 % ring_cap)
        return n4, ncand
    O_ref = O4.clone()                           # last decode of the indexed stream (same queries)
    for rep in range(2):
        s4.hc.zero_(); cn4.zero_()
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        done, nc_old = 0, 0
        for si in range(c4.steps):
            done, nc_old = frame_evict(si, done, nc_old)
        e1.record()
        torch.cuda.synchronize()
    t_fe = e0.elapsed_time(e1) * 1e3 / c4.steps
    rows4 = kc4 + ring_cap
    out["streaming_cfg4_evicting"] = {
        "us_per_frame": round(t_fe, 2),
        "decoded_tokens_per_s_per_layer": round(c4.B * c4.decode_per_step / (t_fe * 1e-6), 1),
        "resident_rows_per_sequence": rows4, "cached_tokens_at_the_end": c4.T,
        "memory_ratio": round(c4.T / rows4, 2),
        "last_output_equals_indexed_stream": bool((O4 == O_ref).all()),
        "note": "per frame: the frame's K/V rows copied into the ring (stands for the model's cache write), "
                "pool + gate of its chunks, chunks leaving the window merged into the store, 8 decodes over "
                "store + ring; no re-selection"}
    return out


def sub_record(cfg, steps, warmup, graphs):
    """Cold step, steady state and dense baseline of another configuration, as a sub-record of the JSON line."""
    b = Bench(cfg)
    rec = b.cold_steps(steps, warmup)
    steady, dense, extra = b.steady_and_dense(steps, rec["ms_per_step"])
    out = {"workload": cfg.name, "tokens_per_s_per_layer": round(rec["value"], 2),
           "ms_per_step": round(rec["ms_per_step"], 5), "gpu_ms_per_step": round(rec["gpu_ms"], 5),
           "stage_us": {k: round(v, 3) for k, v in rec["stage_us"].items()},
           "rooflines": rec["rooflines"] + extra, "steady_state": steady, "dense": dense,
           "rotating_input_sets": b.R}
    if graphs:
        out["cold_step_graph_replay"] = b.graph_replays(steps, steady)
    b.close()
    return out


def grouped_query_cfg3(torch, kb, synth, gated_us_32_heads):
    """Config 3's attention with the paper's 8 key-value heads (section 4.1): every row read serves 4 query heads."""
    c3 = synth.CONFIGS[3]
    c3g = c3.replace(H_kv=8)
    co3 = costs(c3)
    kvg = synth.make_qkv(c3g, "cuda")
    s3g = kb.DecodeState(c3g)
    s3g.Kbar.normal_(); s3g.Vbar.normal_()
    u3g = torch.randn(s3g.util.shape, device="cuda")
    kb.kvev_select(s3g.shape, u3g, None, kb.SELECT_TOPK, c3g.k, 0.0, s3g.k_cap, s3g.idx, s3g.count)
    O3g = torch.empty_like(kvg["Q"])

    def t_of(f, iters):
        for _ in range(2):
            f()
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(iters):
            f()
        e1.record(); torch.cuda.synchronize()
        return e0.elapsed_time(e1) * 1e3 / iters
    tgg = t_of(lambda: kb.kvev_gated_attention(s3g.shape, kvg["Q"], 1, kvg["K"], kvg["V"], s3g.Kbar, s3g.Vbar,
                                               s3g.idx, s3g.count, s3g.k_cap, O3g, s3g.ws_attn), 20)
    tdg = t_of(lambda: kb.kvev_dense_attention(s3g.shape, kvg["Q"], 1, kvg["K"], kvg["V"], O3g, s3g.ws_attn), 5)
    kv_frac = c3g.kv_heads / c3g.H
    return {"workload": c3.name + " with 8 key-value heads for 32 query heads (grouped-query attention; random "
                                  "summaries and scores, attention kernels only)",
            "gated_us": round(tgg, 2), "gated_GBps_unique_rows": round(co3["attend"]["bytes"] * kv_frac / tgg / 1e3, 1),
            "dense_us": round(tdg, 2), "dense_GBps_unique_rows": round(co3["dense"]["bytes"] * kv_frac / tdg / 1e3, 1),
            "speedup_vs_dense": round(tdg / tgg, 2),
            "gated_speedup_vs_32_kv_heads": round(gated_us_32_heads / tgg, 2)}


def calibrate_stream(torch, kb):
    """Reference streams for the HBM-bound kernels, on config 3's footprint.  A plain streaming kernel (one workgroup
    per 256 KiB tile, no arithmetic: kvev_debug_stream_probe) reads 17 GB with no writes, then with 1.5 % and 3 % of
    the bytes written back: what the machine gives the memory pattern of chunk pooling (which writes one summary row
    per chunk of 32 rows: 3 %); each with plain accesses and with the non-temporal hint on loads and stores (what the
    library's streaming kernels use), and with the writes held back and issued in chip-wide bursts (what pooling does
    at scale).  Beside them the library's own pure reader (dense decode attention), pooling in mean
    mode (the same read / write mix as the MLP mode, no matrix work) and a plain device copy."""
    from paper_2509_21354_amd import synth
    cfg = synth.CONFIGS[3]
    kv = synth.make_qkv(cfg, "cuda")
    st = kb.DecodeState(cfg)
    out = {}

    def t_of(f, iters):
        for _ in range(2):
            f()
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(iters):
            f()
        e1.record(); torch.cuda.synchronize()
        return e0.elapsed_time(e1) * 1e3 / iters
    nbytes = kv["K"].numel() * 2
    tile = 256 << 10
    dst = torch.empty((nbytes // tile) * 8192 + 16, dtype=torch.uint8, device="cuda")
    for hname, hints in (("plain", 0), ("nontemporal", 3), ("nontemporal_bursts", 7)):
        for name, wb in (("probe_pure_read", 0), ("probe_read_plus_1.5pct_write", 4096), ("probe_read_plus_3pct_write", 8192)):
            if wb == 0 and hints & 4:
                continue                  # (bursts are about the writes)
            t = t_of(lambda: kb.kvev_debug_stream_probe(kv["K"], tile, dst, wb, hints), 5)
            out[f"{name}_{hname}"] = {"bytes_read": nbytes, "bytes_written": (nbytes // tile) * wb, "us": round(t, 1),
                                      "read_GBps": round(nbytes / t / 1e3, 1),
                                      "total_GBps": round((nbytes + (nbytes // tile) * wb) / t / 1e3, 1)}
    del dst
    O = torch.empty_like(kv["Q"])
    t_dense = t_of(lambda: kb.kvev_dense_attention(st.shape, kv["Q"], 1, kv["K"], kv["V"], O, st.ws_attn), 5)
    db = costs(cfg)["dense"]["bytes"]
    out["dense_decode_attention_pure_read"] = {"bytes": db, "us": round(t_dense, 1), "GBps": round(db / t_dense / 1e3, 1)}
    pb = costs(cfg)["pool"]["bytes"]
    for name, mode in (("pool_mean_read_plus_3pct_write", kb.POOL_MEAN),):
        t = t_of(lambda: kb.kvev_chunk_pool(st.shape, kv["K"], kv["V"], mode, None, None, 0, cfg.N, st.Kbar, st.Vbar, st.ws_pool), 5)
        out[name] = {"bytes": pb, "us": round(t, 1), "GBps": round(pb / t / 1e3, 1)}
    src = kv["K"].view(-1)
    dstc = kv["V"].view(-1)
    t_copy = t_of(lambda: dstc.copy_(src), 5)
    out["device_copy_read_equals_write"] = {"bytes": 2 * nbytes, "us": round(t_copy, 1), "GBps": round(2 * nbytes / t_copy / 1e3, 1)}
    return out


def cpu_baseline(cfg, synth):
    """The CPU oracle on this host, same workload: a bounded sample of independent sequences, once on all the cores the
    box gives this job and once on one core."""
    from oracle import kvev_oracle as orc
    S = cfg.L * cfg.B * cfg.H
    all_cores = max(1, min(os.cpu_count() or 1, int(os.environ.get("OMP_NUM_THREADS", "16"))))
    orc.lib()

    def sample(n_seq):
        c_cpu = cfg if S <= n_seq else cfg.replace(L=1, B=1, H=n_seq)
        t = synth.make_inputs(c_cpu, "cpu")
        Sc = c_cpu.L * c_cpu.B * c_cpu.H
        flat = {k: (v.reshape((1, 1, Sc) + v.shape[3:]) if k in ("Q", "K", "V") else v) for k, v in t.items()}
        return c_cpu, t, Sc, flat

    def leg(cores, n_seq, budget_s):
        c_cpu, t, Sc, flat = sample(n_seq)
        cores = max(1, min(cores, Sc))
        multi_layer = c_cpu.L != 1
        if multi_layer:
            cores = 1
        parts = [list(range(i, Sc, cores)) for i in range(cores)]

        def work(ix):
            sub = {k: (v[:, :, ix].contiguous() if k in ("Q", "K", "V") else v) for k, v in flat.items()}
            orc.cold_step(sub["Q"], sub["K"], sub["V"], sub, c_cpu.T, c_cpu.C, c_cpu.W, c_cpu.k, c_cpu.d_sum)

        def one_step():
            t0 = time.perf_counter()
            if multi_layer:
                orc.cold_step(t["Q"], t["K"], t["V"], t, c_cpu.T, c_cpu.C, c_cpu.W, c_cpu.k, c_cpu.d_sum)
            elif cores == 1:
                work(parts[0])
            else:
                with ThreadPoolExecutor(cores) as ex:
                    list(ex.map(work, parts))
            return time.perf_counter() - t0
        times = [one_step()]
        while len(times) < 10 and sum(times) < budget_s:
            times.append(one_step())
        dt = sum(times) / len(times) * (S / Sc)
        note = "whole problem" if Sc == S else (f"{Sc} of {S} sequences (layer 0 weights), extrapolated linearly over "
                                                "independent sequences")
        return {"value": round(cfg.B * cfg.Tq * cfg.L / dt, 4), "unit": "tokens/s/layer", "cores": cores, "kind": "oracle",
                "sample": f"{note}; cold step (pool+gate+select+attend), mean of {len(times)} steps, "
                          f"{sum(times):.2f} s on {cores} thread(s)",
                "seconds_per_step": round(dt, 3)}
    out = leg(all_cores, 64, 8.0)
    out["single_core"] = leg(1, 8, 8.0)
    return out


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default="cfg3", choices=["cfg1", "cfg2", "cfg3", "cfg5"])
    ap.add_argument("--sets", type=int, default=0, help="rotating input sets (0: enough to exceed 512 MB)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-extra", action="store_true", help="skip the sub-records of the other configurations")
    ap.add_argument("--lean", action="store_true", help="profiling aid: the timed cold steps, the steady-state and dense "
                                                        "lines only (no threshold, eviction, aggregator sections)")
    ap.add_argument("--only", default="", help="profiling aid: run only this stage in the timed loop "
                                                 "(pool|gate|select|attend|dense)")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="profiling aid: run 10 plain device copies of 1 GiB and exit (reference reading "
                         "for the FETCH_SIZE / WRITE_SIZE counters)")
    ap.add_argument("--calibrate-stream", action="store_true",
                    help="reference streams on config 3's pooling footprint: pure read, read + 3 %% write, copy")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU (the path has no inter-GPU step); --gpus must be 1",
              file=sys.stderr)
        sys.exit(2)

    import torch
    from paper_2509_21354_amd import binding as kb
    from paper_2509_21354_amd import synth

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(1)
    kb.lib()
    dev = "cuda"
    if args.calibrate_copy:
        src = torch.empty(1 << 30, dtype=torch.uint8, device=dev).random_()
        dst = torch.empty_like(src)
        for _ in range(10):
            dst.copy_(src)
        torch.cuda.synchronize()
        print(json.dumps({"calibrate_copy": {"bytes_read": 1 << 30, "bytes_written": 1 << 30, "launches": 10}}))
        return
    if args.calibrate_stream:
        print(json.dumps({"calibrate_stream": calibrate_stream(torch, kb)}))
        return
    cfg = synth.CONFIGS[int(args.workload[3:])]
    b = Bench(cfg, args.sets)
    rec = b.cold_steps(args.steps, args.warmup, args.only)
    per_step_us = rec["per_step_us"]
    out = {
        "metric": "gated-chunk decode attn tokens/s per layer", "value": round(rec["value"], 2), "unit": "tokens/s/layer",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(rec["ms_per_step"], 5),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": cfg.dtype, "data": "synthetic",
        "config": {"workload": cfg.name, "L": cfg.L, "B": cfg.B, "H": cfg.H, "d": cfg.d, "T": cfg.T, "C": cfg.C,
                   "k": cfg.k, "W": cfg.W, "d_sum": cfg.d_sum, "d_g": cfg.d_g, "Tq": cfg.Tq,
                   "step": "cold: pool + gate + select + attend" if not args.only else args.only,
                   "rotating_input_sets": b.R},
        "stage_us": {k: round(v, 3) for k, v in rec["stage_us"].items()},
        "gpu_ms_per_step": round(rec["gpu_ms"], 5), "host_wall_ms_per_step": round(rec["wall_ms"], 5),
        "step_us_median": round(per_step_us[len(per_step_us) // 2], 3), "step_us_min": round(per_step_us[0], 3),
        "step_us_max": round(per_step_us[-1], 3),
    }
    rooflines = rec["rooflines"]
    if rooflines:
        dom = max(rooflines, key=lambda r: r["us_per_launch"])
        out["roofline"] = {k: dom[k] for k in ("bound", "achieved", "peak", "unit", "frac", "traffic", "traffic_source", "stage",
                                              "kernel", "us_per_launch", "recurrence") if k in dom}
        out["rooflines"] = rooflines

    if not args.only:
        steady, dense, extra = b.steady_and_dense(args.steps, rec["ms_per_step"])
        out["steady_state"], out["dense"] = steady, dense
        out["rooflines"] = rooflines + extra
        if b.cost["dense"]["bytes"] < (1 << 30):
            out["cold_step_graph_replay"] = b.graph_replays(args.steps, steady)
    if not args.only and not args.lean:
        out["threshold_mode"] = b.threshold_mode(args.steps, dense["us_per_step"])
        out["eviction"] = b.eviction(args.steps)
        from paper_2509_21354_amd import cost_model as cm
        k_eff = min(cfg.k, cfg.N_cand)
        dims = cm.ModelDims(d_model=cfg.H * cfg.d, H=cfg.H, d_k=cfg.d)
        rep = cm.report(cfg.B, cfg.T, cfg.T - cfg.N_cand * cfg.C, k_eff, cfg.C, cfg.d_sum, cfg.d_g, dims)
        out["cost_model"] = {"eq7_speed_up_layer": round(rep["speed_up_eq7"], 3),
                             "eq4_over_eq6_attention_flops": round(rep["attention_only_flops_ratio"], 3),
                             "memory_ratio_n_over_W_plus_M": round(rep["memory_ratio"], 2),
                             "note": "per-layer estimate incl. projections and FFN (Eq. 7); the measured speed-ups "
                                     "in `dense` are for the attention over the cache alone"}
        out["aggregators"] = b.aggregators(args.steps)
    gated_us = out.get("steady_state", {}).get("us_per_step")
    b.close()
    del b

    if not args.no_extra and not args.only:
        free, _ = torch.cuda.mem_get_info()
        if free > 100 << 30:
            if cfg.number == 3 and gated_us:
                out["cfg3_grouped_query"] = grouped_query_cfg3(torch, kb, synth, gated_us)
                torch.cuda.empty_cache()
            for number, graphs in ((2, True), (5, False)):
                if number != cfg.number:
                    out[f"cfg{number}"] = sub_record(synth.CONFIGS[number], max(10, args.steps // 2) if number == 5 else max(50, args.steps),
                                                     args.warmup, graphs)
                    torch.cuda.empty_cache()
            out.update(streaming_cfg4(torch, kb, synth))
            torch.cuda.empty_cache()

    if not args.no_cpu_baseline and not args.only:
        out["cpu_baseline"] = cpu_baseline(cfg, synth)

    out["paper_context"] = {"speedup": 1.34, "flops_saving": 0.246, "kv_memory_reduction": 1.87,
                            "hardware": "inference hardware not stated; fine-tuning on 2x NVIDIA H800; bf16; whole-model numbers"}
    print(json.dumps(out))


if __name__ == "__main__":
    main()

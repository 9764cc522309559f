#!/usr/bin/env python3
"""MoE-layer throughput on one MI355X.

A step is one pass of the whole path -- moe_route, moe_expert_ffn (masked), moe_combine -- over one batch of
synthetic input that is already resident in HBM.  The headline workload is the Mixtral-8x7B-shaped layer
(d=4096, 8 experts top-2, SwiGLU inner 14336, 6 of 8 experts on this GPU) at a prefill of 2048 tokens; the
same layer at decode batches of 1 and 16 tokens is timed in the same run and reported under "decode".
The dominant kernel (the gate/up projection of the expert FFN) is bracketed by HIP events in every timed
step; its algorithmic flops (prefill) or bytes (decode) over its mean duration give the roofline fraction.
The CPU oracle is timed beside it on a bounded token sample of the same batch.

Prints ONE JSON line on stdout; progress goes to stderr.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_BF16_MFMA = 2.5e15   # flop/s, MI355X dense bf16 matrix peak
PEAK_HBM = 8.0e12         # B/s, MI355X HBM3E peak
# HBM bytes per launch of the dominant kernels (fetched + written).  STORED counter values, not measured by the run that
# prints them: rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs of this script, scaled by what the same counters read for a
# plain 1 GiB copy; the profile they come from is named beside them in the JSON line.
TRAFFIC_SOURCE = "stored counter value from profiles/bench_mixtral_kernel_stats_and_hbm_counters.md (rocprofv3 --pmc FETCH_SIZE, WRITE_SIZE), not measured in this run"
TRAFFIC_PREFILL = {"up": 2.4432e9 + 87.3e6, "down": 1.3995e9 + 27.2e6}
TRAFFIC_DECODE_UP = {1: 470.0e6 + 0.1e6, 16: 1.1752e9 + 0.7e6}


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def time_steps(torch, B, L, hd, dw, mask_d, steps, warmup):
    """Run warmup + steps passes.  Returns a dict of seconds: wall (all timed steps, host clock around two
    synchronisations), and mean / median over the timed steps of the whole step, the up-projection stage, the
    down-projection stage and the whole expert FFN, from HIP events recorded on the stream the kernels run on."""
    r, s = L.routing, L.shape

    def one(ev=None):
        if ev is not None:
            ev[0].record()
        L.route(hd, dw)
        if ev is not None:
            ev[1].record()
        B.moe_expert_ffn_stage(s, hd, r.perm, r.offsets, r.counts, dw.w1, dw.w3, dw.w2, mask_d, L.y, L.ws, B.STAGE_UP)
        if ev is not None:
            ev[2].record()
        B.moe_expert_ffn_stage(s, hd, r.perm, r.offsets, r.counts, dw.w1, dw.w3, dw.w2, mask_d, L.y, L.ws, B.STAGE_DOWN)
        if ev is not None:
            ev[3].record()
        L.combine(mask_d)
        if ev is not None:
            ev[4].record()

    for _ in range(warmup):
        one()
    evs = [[torch.cuda.Event(enable_timing=True) for _ in range(5)] for _ in range(steps)]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(steps):
        one(evs[i])
    torch.cuda.synchronize()
    out = {"wall": time.perf_counter() - t0}
    for name, a, b in (("step", 0, 4), ("up", 1, 2), ("down", 2, 3), ("ffn", 1, 3)):
        ts = sorted(e[a].elapsed_time(e[b]) * 1e-3 for e in evs)
        out[name + "_mean"], out[name + "_median"] = sum(ts) / steps, ts[steps // 2]
    return out


def median_event_seconds(torch, fn, runs=20, flush=None):
    """Median over `runs` of the HIP-event time of fn(); flush (a device tensor larger than the 256 MB Infinity Cache) is
    read through between runs, outside the timed interval, so that a small working set comes from HBM every time (read,
    not written: dirty lines would have to be written back during the timed call)."""
    for _ in range(3):
        fn()
    ts = []
    for _ in range(runs):
        if flush is not None:
            flush.sum()
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        a.record()
        fn()
        b.record()
        b.synchronize()
        ts.append(a.elapsed_time(b) * 1e-3)
    return sorted(ts)[runs // 2]


def library_gemm_yardstick(torch):
    """Context for the roofline fractions, not part of the path: what the vendor library's dense bf16 GEMM (torch.matmul)
    reaches on this GPU, (a) on one large GEMM, (b) on one GEMM with the prefill workload's row total, (c) as one GEMM per
    expert with the workload's rows per expert (up: [rows,d] x [d,2I], down: [rows,I] x [I,d]).  No gather, no SwiGLU."""
    d, I = 4096, 14336
    rows = [1540, 379, 283, 550, 165, 126]       # the six masked-on experts of the prefill workload
    g = torch.Generator(device="cuda").manual_seed(0)
    rnd = lambda *shape: torch.randn(*shape, device="cuda", dtype=torch.float32, generator=g).mul_(0.02).to(torch.bfloat16)
    w13, w2 = rnd(2 * I, d), rnd(d, I)
    w13s = [w13] + [rnd(2 * I, d) for _ in rows[1:]]
    w2s = [w2] + [rnd(d, I) for _ in rows[1:]]
    xs, acts = [rnd(r, d) for r in rows], [rnd(r, I) for r in rows]
    xb, xc = rnd(sum(rows), d), rnd(8192, d)
    frac = lambda flop, sec: flop / sec / PEAK_BF16_MFMA
    t_big = median_event_seconds(torch, lambda: xc @ w13.t())
    t_one = median_event_seconds(torch, lambda: xb @ w13.t())
    t_up = median_event_seconds(torch, lambda: [x @ w.t() for x, w in zip(xs, w13s)])
    t_dn = median_event_seconds(torch, lambda: [a @ w.t() for a, w in zip(acts, w2s)])
    rec = {"metric": "vendor-library dense bf16 GEMM, fraction of the MFMA peak (context)", "unit": "fraction", "n_gpus": 1,
           "dense_8192x4096x28672": {"us": t_big * 1e6, "frac": frac(8192 * 4.0 * d * I, t_big)},
           "dense_3043x4096x28672": {"us": t_one * 1e6, "frac": frac(sum(rows) * 4.0 * d * I, t_one)},
           "per_expert_up": {"us": t_up * 1e6, "frac": frac(sum(rows) * 4.0 * d * I, t_up)},
           "per_expert_down": {"us": t_dn * 1e6, "frac": frac(sum(rows) * 2.0 * d * I, t_dn)}, "rows": rows}
    log(f"[bench] library GEMM: 8192 rows {rec['dense_8192x4096x28672']['frac']:.3f}, 3043 rows {rec['dense_3043x4096x28672']['frac']:.3f}, "
        f"per expert up {t_up * 1e6:.0f} us {rec['per_expert_up']['frac']:.3f}, down {t_dn * 1e6:.0f} us {rec['per_expert_down']['frac']:.3f}")
    return rec


def cpu_baseline_oracle():
    """The CPU-baseline leg: the only place where this script touches the oracle, and only to time it on the host cores."""
    import oracle
    return oracle


def greedy_assignment_demo(torch, B, Lm, wl, pcie_gbs):
    """Greedy Assignment (Alg. 1) end to end on the Mixtral-shaped layer.  Cost model of Section "Greedy Assignment
    Strategy": gpu_compute(w) = the expert FFN of this library timed on one expert with w rows; cpu_compute(w) = w times
    the oracle's time per (token, expert) row on the host cores; an uncached expert pays its weights over the host link.
    The workload histograms of a prefill and a decode batch then go through moe_expert_times and moe_greedy_assign, the
    resulting G is used as expert_mask, and the makespan max(T_gpu, T_cpu) is compared with everything on one side and
    with the best of all 2^N assignments."""
    import itertools
    cfg = wl.CONFIGS["mixtral"]
    W, b = wl.gate_weights(cfg), wl.gate_bias(cfg)
    w1, w3, w2 = wl.expert_weights(cfg)
    dw = Lm.LayerWeights.upload(W, b, w1, w3, w2)
    wmax = 2048
    # ---- gpu_compute(w): every token sent to experts 0 and 1 by the gate bias, only expert 0 masked on
    force = torch.zeros(cfg.N, dtype=torch.float32, device="cuda")
    force[0], force[1] = 1e4, 5e3
    only0 = torch.zeros(cfg.N, dtype=torch.uint8, device="cuda")
    only0[0] = 1
    pts, secs = [1, 2, 4, 8, 16, 32, 64, 128, 256, 512, 1024, 2048], []
    for w in pts:
        L = Lm.MoeLayer(cfg, w)
        hd = Lm.to_device_bf16(wl.hidden_states(cfg, w, draw=w))
        L.route(hd, dw, bias=force)
        torch.cuda.synchronize()
        assert int(L.routing.counts[0]) == w
        secs.append(median_event_seconds(torch, lambda: L.expert_ffn(hd, dw, only0), 10))
        log(f"[bench] gpu_compute({w:4d} rows) = {secs[-1] * 1e6:8.1f} us")
    gpu_compute = np.interp(np.arange(wmax + 1), [0] + pts, [0.0] + secs).astype(np.float32)
    # ---- cpu_compute(w): the oracle's expert rows, timed on a few rows
    oracle = cpu_baseline_oracle()
    n = 8
    h8 = wl.hidden_states(cfg, n)
    idx8 = np.tile(np.arange(cfg.k, dtype=np.int32), (n, 1))
    t0 = time.perf_counter()
    oracle.expert_rows(h8, idx8, w1, w3, w2)
    row_s = (time.perf_counter() - t0) / (n * cfg.k)
    cpu_compute = (np.arange(wmax + 1) * row_s).astype(np.float32)
    trans = 3.0 * cfg.d * cfg.I * 2 / (pcie_gbs * 1e9)
    log(f"[bench] cpu_compute = {row_s * 1e3:.2f} ms per row on {oracle.num_threads()} threads; transfer of one expert = {trans * 1e3:.2f} ms")

    cached = wl.mask_random(cfg, 6)
    cases = []
    for T in (2048, 16):
        L = Lm.MoeLayer(cfg, T)
        hd = Lm.to_device_bf16(wl.hidden_states(cfg, T, draw=T))
        L.route(hd, dw)
        torch.cuda.synchronize()
        counts = L.routing.counts.cpu().numpy()
        for what, ca in (("6 of 8 experts cached", cached), ("nothing cached", None)):
            t_gpu, t_cpu = B.expert_times(counts, ca, trans, gpu_compute, cpu_compute)
            G, Cc, Tg, Tc = B.greedy_assign(t_gpu, t_cpu)
            act = [e for e in range(cfg.N) if counts[e] > 0]
            span = lambda on_gpu: max(sum(float(t_gpu[e]) for e in act if on_gpu[e]), sum(float(t_cpu[e]) for e in act if not on_gpu[e]))
            best = min(span(dict(zip(act, bits))) for bits in itertools.product((0, 1), repeat=len(act)))
            md = torch.from_numpy(G).cuda()
            step = median_event_seconds(torch, lambda: (L.expert_ffn(hd, dw, md), L.combine(md)), 10)
            rec = {"tokens": T, "cache": what, "counts": counts.tolist(), "G": G.tolist(), "C": Cc.tolist(),
                   "T_gpu_ms": float(Tg) * 1e3, "T_cpu_ms": float(Tc) * 1e3, "makespan_ms": float(max(Tg, Tc)) * 1e3,
                   "all_gpu_ms": float(t_gpu.sum()) * 1e3, "all_cpu_ms": float(t_cpu.sum()) * 1e3, "optimum_ms": float(best) * 1e3,
                   "gpu_share_measured_ms": float(step) * 1e3}
            log(f"[bench] T={T:4d} {what:22s} counts={counts.tolist()} G={G.tolist()} makespan {rec['makespan_ms']:.2f} ms "
                f"(all GPU {rec['all_gpu_ms']:.2f}, all CPU {rec['all_cpu_ms']:.2f}, optimum {rec['optimum_ms']:.2f}); "
                f"GPU share as run: {step * 1e3:.3f} ms")
            cases.append(rec)
    return {"metric": "Greedy Assignment (Alg. 1) makespan", "unit": "ms", "n_gpus": 1, "dtype": "bf16", "data": "synthetic",
            "config": {"workload": "mixtral-8x7b-shaped layer, prefill 2048 and decode 16 tokens", "pcie_GBps": pcie_gbs},
            "gpu_compute_us": dict(zip(map(str, pts), (float(x) * 1e6 for x in secs))), "cpu_row_ms": float(row_s) * 1e3,
            "cpu_threads": oracle.num_threads(), "transfer_ms": float(trans) * 1e3, "cases": cases}


def time_graph_replays(torch, L, hd, dw, mask_d, steps, warmup):
    """The same pass captured once in a HIP graph and replayed: removes the host's per-launch cost, which at
    decode sizes is a large share of an eagerly launched step.  Returns wall seconds for `steps` replays."""
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        for _ in range(2):
            L.forward(hd, dw, mask_d)
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        L.forward(hd, dw, mask_d)
    for _ in range(warmup):
        g.replay()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        g.replay()
    torch.cuda.synchronize()
    return time.perf_counter() - t0


def survey_config(torch, B, Lm, wl, name, Ts, mask_kind, steps=20, merged=True):
    """One JSON-able record per batch size: the whole step (route, masked routed FFN, shared experts, combine) with HIP
    events between the calls, and the FFN's share of the bf16 MFMA / HBM peaks."""
    cfg = wl.CONFIGS[name]
    w1, w3, w2 = wl.expert_weights(cfg)
    dw = Lm.LayerWeights.upload(wl.gate_weights(cfg), wl.gate_bias(cfg), w1, w3, w2, wl.shared_expert_weights(cfg), merge_shared=True)
    out, flush = [], None
    for T in Ts:
        L = Lm.MoeLayer(cfg, T)
        hd = Lm.to_device_bf16(wl.hidden_states(cfg, T, draw=T))
        L.route(hd, dw)
        torch.cuda.synchronize()
        counts = L.routing.counts.cpu().numpy()
        mask = {"all": np.ones(cfg.N, np.uint8), "half": wl.mask_top_by_counts(counts, cfg.N // 2),
                "rand6": wl.mask_random(cfg, 6)}[mask_kind]
        md, on = torch.from_numpy(mask).cuda(), mask.astype(bool)

        def step(ev=None):
            L.route(hd, dw)
            if ev: ev[0].record()
            L.expert_ffn(hd, dw, md)
            if ev: ev[1].record()
            if cfg.n_shared: L.shared_ffn(hd, dw)
            if ev: ev[2].record()
            L.combine(md)
            if ev: ev[3].record()
        for _ in range(3):
            step()
        evs = [[torch.cuda.Event(enable_timing=True) for _ in range(4)] for _ in range(steps)]
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for i in range(steps):
            step(evs[i])
        torch.cuda.synchronize()
        wall = (time.perf_counter() - t0) / steps
        med = lambda a, b: sorted(e[a].elapsed_time(e[b]) for e in evs)[steps // 2] * 1e-3
        ffn, sh = med(0, 1), med(1, 2)
        rows_on, active = int(counts[on].sum()), int(((counts > 0) & on).sum())
        if T <= 16:
            # a decode step touches few hundred MB at most: flush the Infinity Cache between steps so that it is HBM traffic
            if flush is None:
                flush = torch.zeros(1 << 28, dtype=torch.int32, device="cuda")      # 1 GiB
            wall = median_event_seconds(torch, step, steps, flush)
            ffn = median_event_seconds(torch, lambda: L.expert_ffn(hd, dw, md), steps, flush)
            if cfg.n_shared:
                sh = median_event_seconds(torch, lambda: L.shared_ffn(hd, dw), steps, flush)
        # both bounds of the routed FFN (algorithmic flops of the masked-on routed rows; weights of the touched masked-on
        # experts once from HBM) and of the layer's whole expert work, shared experts included (always on: T rows each)
        F_r, B_r = 6.0 * cfg.d * cfg.I * rows_on, 6.0 * cfg.d * cfg.I * active
        F_s, B_s = 6.0 * cfg.d * cfg.I_shared * cfg.n_shared * T, 6.0 * cfg.d * cfg.I_shared * cfg.n_shared
        t_all = ffn + (sh if cfg.n_shared else 0.0)
        rec = {"workload": name, "tokens": T, "mask": mask_kind, "us_per_step": wall * 1e6, "tokens_per_s": T / wall,
               "ffn_us": ffn * 1e6, "ffn_mfma_frac": F_r / ffn / PEAK_BF16_MFMA,
               "ffn_hbm_frac": B_r / ffn / PEAK_HBM, "shared_us": sh * 1e6 if cfg.n_shared else 0.0,
               "experts_mfma_frac": (F_r + F_s) / t_all / PEAK_BF16_MFMA, "experts_hbm_frac": (B_r + B_s) / t_all / PEAK_HBM,
               "active_experts": active, "rows_on": rows_on}
        rec["bound"] = "mfma" if rec["experts_mfma_frac"] >= rec["experts_hbm_frac"] else "hbm"
        rec["bound_frac"] = max(rec["experts_mfma_frac"], rec["experts_hbm_frac"])     # max(F / (t P_mfma), B / (t BW))
        if L.n_merged and merged:
            # the same layer with its shared experts inside the grouped launches (moe_append_shared)
            xm = L.merged_mask(md)
            mstep = lambda: L.forward_merged(hd, dw, xm)
            for _ in range(3):
                mstep()
            wm = median_event_seconds(torch, mstep, steps, flush if T <= 16 else None)
            ws_ = median_event_seconds(torch, step, steps, flush if T <= 16 else None)
            rec["merged_us_per_step"], rec["merged_tokens_per_s"], rec["separate_us_per_step"] = wm * 1e6, T / wm, ws_ * 1e6
            log(f"[bench] {name:9s} T={T:5d} shared experts inside the grouped launches: step {wm * 1e6:8.1f} us "
                f"(separate launches, timed the same way: {ws_ * 1e6:8.1f} us)")
        log(f"[bench] {name:9s} T={T:5d} step {wall * 1e6:8.1f} us | ffn {ffn * 1e6:8.1f} us mfma {rec['ffn_mfma_frac']:.3f} "
            f"hbm {rec['ffn_hbm_frac']:.3f} | shared {rec['shared_us']:7.1f} us | active {active} rows_on {rows_on}")
        out.append(rec)
    del dw, flush
    torch.cuda.empty_cache()
    return out


def survey_mid(torch, B, Lm, wl, name, Ts=(32, 64, 128, 256, 512, 1024), steps=20):
    """Mid-sized batches, no mask: up and down projection separately, as fractions of the HBM peak of the touched
    experts' weights (median of HIP-event timings)."""
    cfg = wl.CONFIGS[name]
    w1, w3, w2 = wl.expert_weights(cfg)
    dw = Lm.LayerWeights.upload(wl.gate_weights(cfg), wl.gate_bias(cfg), w1, w3, w2)
    out = []
    for T in Ts:
        L = Lm.MoeLayer(cfg, T)
        hd = Lm.to_device_bf16(wl.hidden_states(cfg, T, draw=T))
        L.route(hd, dw)
        torch.cuda.synchronize()
        r = L.routing
        active = int((r.counts > 0).sum())
        rec = {"workload": name, "tokens": T, "active_experts": active}
        for stage, sn, per in ((B.STAGE_UP, "up", 4.0), (B.STAGE_DOWN, "down", 2.0)):
            evs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(steps)]
            for i in range(steps + 3):
                if i >= 3: evs[i - 3][0].record()
                B.moe_expert_ffn_stage(L.shape, hd, r.perm, r.offsets, r.counts, dw.w1, dw.w3, dw.w2, None, L.y, L.ws, stage)
                if i >= 3: evs[i - 3][1].record()
            torch.cuda.synchronize()
            t = sorted(a.elapsed_time(b) for a, b in evs)[steps // 2] * 1e-3
            rec[sn + "_us"] = t * 1e6
            rec[sn + "_hbm_frac"] = per * cfg.d * cfg.I * active / t / PEAK_HBM
        log(f"[bench] {name:9s} T={T:5d} active {active:3d} | up {rec['up_us']:7.1f} us {rec['up_hbm_frac']:.3f} | "
            f"down {rec['down_us']:7.1f} us {rec['down_hbm_frac']:.3f}")
        out.append(rec)
    del dw
    torch.cuda.empty_cache()
    return out


def survey_few_experts(torch, B, Lm, wl, Ts=(4, 16, 32, 128, 256), ons=(1, 2, 4, 8), steps=15):
    """Mixtral-shaped layer with only the n most loaded experts masked on (the usual case when most experts live on the
    host): up and down projection separately, as fractions of the HBM peak of the working experts' weights."""
    cfg = wl.CONFIGS["mixtral"]
    w1, w3, w2 = wl.expert_weights(cfg)
    dw = Lm.LayerWeights.upload(wl.gate_weights(cfg), wl.gate_bias(cfg), w1, w3, w2)
    out = []
    for T in Ts:
        L = Lm.MoeLayer(cfg, T)
        hd = Lm.to_device_bf16(wl.hidden_states(cfg, T, draw=T))
        L.route(hd, dw)
        torch.cuda.synchronize()
        counts = L.routing.counts.cpu().numpy()
        order = np.argsort(-counts, kind="stable")
        r = L.routing
        for n_on in ons:
            mask = np.zeros(cfg.N, np.uint8)
            mask[order[:n_on]] = 1
            md = torch.from_numpy(mask).cuda()
            active = int(((counts > 0) & (mask > 0)).sum())
            rec = {"tokens": T, "experts_on": n_on, "active_experts": active}
            for stage, sn, per in ((B.STAGE_UP, "up", 4.0), (B.STAGE_DOWN, "down", 2.0)):
                t = median_event_seconds(torch, lambda: B.moe_expert_ffn_stage(L.shape, hd, r.perm, r.offsets, r.counts, dw.w1, dw.w3,
                                                                                 dw.w2, md, L.y, L.ws, stage), steps)
                rec[sn + "_us"], rec[sn + "_hbm_frac"] = t * 1e6, per * cfg.d * cfg.I * active / t / PEAK_HBM
            log(f"[bench] mixtral   T={T:5d} experts on {n_on} (working {active}) | up {rec['up_us']:7.1f} us {rec['up_hbm_frac']:.3f} | "
                f"down {rec['down_us']:7.1f} us {rec['down_hbm_frac']:.3f}")
            out.append(rec)
    del dw
    torch.cuda.empty_cache()
    return out


def survey_rows_per_expert(torch, B, Lm, wl, steps=20):
    """The Mixtral-shaped prefill batch under three routings that differ only in rows per expert (the gate bias is the
    workload's Zipf bias, zero, or +-20 so that two experts take every token): MFMA fraction of either projection."""
    cfg, T = wl.CONFIGS["mixtral"], 2048
    w1, w3, w2 = wl.expert_weights(cfg)
    out = []
    for kind in ("zipf", "uniform", "two experts"):
        bias = wl.gate_bias(cfg) if kind == "zipf" else np.zeros(cfg.N, np.float32)
        if kind == "two experts":
            bias = np.array([20, 20] + [-20] * (cfg.N - 2), np.float32)
        dw = Lm.LayerWeights.upload(wl.gate_weights(cfg), bias, w1, w3, w2)
        L = Lm.MoeLayer(cfg, T)
        hd = Lm.to_device_bf16(wl.hidden_states(cfg, T))
        L.route(hd, dw)
        torch.cuda.synchronize()
        r = L.routing
        c = r.counts.cpu().numpy()
        rec = {"routing": kind, "counts": c.tolist()}
        for stage, sn, per in ((B.STAGE_UP, "up", 4.0), (B.STAGE_DOWN, "down", 2.0)):
            evs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(steps)]
            for i in range(steps + 3):
                if i >= 3: evs[i - 3][0].record()
                B.moe_expert_ffn_stage(L.shape, hd, r.perm, r.offsets, r.counts, dw.w1, dw.w3, dw.w2, None, L.y, L.ws, stage)
                if i >= 3: evs[i - 3][1].record()
            torch.cuda.synchronize()
            t = sorted(a.elapsed_time(b) for a, b in evs)[steps // 2] * 1e-3
            rec[sn + "_us"] = t * 1e6
            rec[sn + "_mfma_frac"] = per * cfg.d * cfg.I * float(c.sum()) / t / PEAK_BF16_MFMA
        log(f"[bench] mixtral T=2048 {kind:11s} counts={c.tolist()} | up {rec['up_us']:7.1f} us mfma {rec['up_mfma_frac']:.3f} | "
            f"down {rec['down_us']:7.1f} us mfma {rec['down_mfma_frac']:.3f}")
        out.append(rec)
        del dw
        torch.cuda.empty_cache()
    return out


def timeline(torch, B, Lm, wl, spec):
    """Per-block timeline of the two tiled expert-FFN launches of one shape (moe_debug_set_trace): how long blocks of
    each tile height take, how evenly the compute units and the XCDs finish.  spec: SHAPE:TOKENS:MASK with MASK = all,
    half (top half by this batch's workloads), rand6, or onlyE[,E...] (just those experts on)."""
    name, T, mk = spec.split(":")
    T = int(T)
    cfg = wl.CONFIGS[name]
    w1, w3, w2 = wl.expert_weights(cfg)
    dw = Lm.LayerWeights.upload(wl.gate_weights(cfg), wl.gate_bias(cfg), w1, w3, w2)
    L = Lm.MoeLayer(cfg, T, B.FFN_TILED)
    hd = Lm.to_device_bf16(wl.hidden_states(cfg, T, draw=T))
    L.route(hd, dw)
    torch.cuda.synchronize()
    counts = L.routing.counts.cpu().numpy()
    if mk.startswith("only"):
        mask = np.zeros(cfg.N, np.uint8)
        mask[[int(e) for e in mk[4:].split(",")]] = 1
    else:
        mask = {"all": np.ones(cfg.N, np.uint8), "half": wl.mask_top_by_counts(counts, cfg.N // 2), "rand6": wl.mask_random(cfg, 6)}[mk]
    md = torch.from_numpy(mask).cuda()
    records = torch.zeros(2 * B.TRACE_MAX_BLOCKS * 8, dtype=torch.int64, device="cuda")
    for _ in range(3):
        L.expert_ffn(hd, dw, md)
    torch.cuda.synchronize()
    B.moe_debug_set_trace(records)
    L.expert_ffn(hd, dw, md)
    torch.cuda.synchronize()
    B.moe_debug_set_trace(None)
    tr = records.cpu().numpy().reshape(2, B.TRACE_MAX_BLOCKS, 8)
    out = {"metric": "block timeline of the tiled expert FFN", "unit": "us", "n_gpus": 1, "dtype": "bf16", "data": "synthetic",
           "config": {"workload": f"{name}-shaped layer, {T} tokens, mask {mk}"}, "counts_on": counts[mask.astype(bool)].tolist()}
    for mode, nm in ((0, "up"), (1, "down")):
        t = tr[mode]
        t = t[t[:, 7] == 1]
        if len(t) == 0:
            continue
        t0 = t[:, 0].min()
        b, e = (t[:, 0] - t0) / 100.0, (t[:, 1] - t0) / 100.0
        dur, rows, xcd = e - b, t[:, 5], t[:, 3] & 0xF
        cu = xcd * 4096 + ((t[:, 2] >> 8) & 0xFFF)          # XCD, then shader engine / array / compute unit bits of HW_ID
        span = float(e.max())
        last = {}
        for c, ee in zip(cu.tolist(), e.tolist()):
            last[c] = max(last.get(c, 0.0), ee)
        rec = {"blocks": int(len(t)), "compute_units_used": len(last), "span_us": span, "sum_of_block_us": float(dur.sum()),
               "mean_busy_units": float(dur.sum() / span), "last_end_per_unit_us": {"mean": float(np.mean(list(last.values()))),
                                                                                   "min": float(min(last.values())), "max": float(max(last.values()))},
               "by_rows": [], "by_xcd": []}
        for lo, hi in ((1, 16), (17, 32), (33, 64), (65, 96), (97, 128)):
            m = (rows >= lo) & (rows <= hi)
            if m.any():
                rec["by_rows"].append({"rows": f"{lo}-{hi}", "blocks": int(m.sum()), "mean_us": float(dur[m].mean()),
                                       "min_us": float(dur[m].min()), "max_us": float(dur[m].max())})
        for x in range(8):
            m = xcd == x
            if m.any():
                rec["by_xcd"].append({"xcd": x, "blocks": int(m.sum()), "last_end_us": float(e[m].max()), "sum_of_block_us": float(dur[m].sum()),
                                      "mean_rows": float(rows[m].mean())})
        out[nm] = rec
        log(f"[bench] timeline {name} T={T} {nm}: {rec['blocks']} blocks on {rec['compute_units_used']} units, span {span:.1f} us, "
            f"{rec['mean_busy_units']:.1f} units busy on average; units finish at {rec['last_end_per_unit_us']['mean']:.1f} us on average "
            f"({rec['last_end_per_unit_us']['min']:.1f} .. {rec['last_end_per_unit_us']['max']:.1f})")
        for r in rec["by_rows"]:
            log(f"[bench]    tiles of {r['rows']:>7s} rows: {r['blocks']:5d} blocks, {r['mean_us']:6.1f} us each ({r['min_us']:.1f} .. {r['max_us']:.1f})")
        log("[bench]    XCD finish times: " + " ".join(f"{r['last_end_us']:.0f}" for r in rec["by_xcd"]))
    return out


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--decode-steps", type=int, default=50)
    ap.add_argument("--cpu-sample", type=int, default=2048, help="tokens of the prefill batch the oracle is timed on (0 = skip)")
    ap.add_argument("--no-decode", action="store_true")
    ap.add_argument("--no-other-workloads", action="store_true", help="skip the DeepSeek-V2-Lite-, Qwen1.5-MoE- and Qwen3-shaped layers")
    ap.add_argument("--stack", action="store_true",
                    help="run the Qwen3-30B-A3B-shaped decode stack instead (48 layers, 256 steps, batch 16, AR(1) routing) "
                         "and print its own JSON line: per-step workload histograms, prediction accuracy, tokens/s")
    ap.add_argument("--survey", action="store_true",
                    help="time the other layer shapes instead (DeepSeek-V2-Lite, Qwen1.5-MoE, Qwen3-30B-A3B and Mixtral; prefill, "
                         "decode and the mid-sized batches between them) and print one JSON line with all records")
    ap.add_argument("--one", default=None, metavar="SHAPE:TOKENS:MASK",
                    help="time one layer shape at one batch size instead, e.g. deepseek:2048:half, qwen15:1:all, mixtral:2048:rand6 "
                         "(mask: all | half = top half by this batch's workloads | rand6); prints one JSON record; the run to "
                         "profile when per-shape kernel statistics or counters are wanted")
    ap.add_argument("--timeline", default=None, metavar="SHAPE:TOKENS:MASK",
                    help="per-block timeline of the tiled expert-FFN launches of one shape (block durations by tile height, "
                         "finish times per compute unit and per XCD); MASK as for --one, or onlyE[,E...] for just those experts")
    ap.add_argument("--one-merged", action="store_true", help="--one: also time the variant with the shared experts inside the grouped launches")
    ap.add_argument("--stack-layers", type=int, default=48)
    ap.add_argument("--stack-steps", type=int, default=256)
    ap.add_argument("--assign", action="store_true",
                    help="Greedy Assignment (Alg. 1) on the Mixtral-shaped layer: t_gpu(w) timed on this library's kernels, "
                         "t_cpu(w) from the timed oracle, masks for the prefill and decode workloads")
    ap.add_argument("--pcie-gbs", type=float, default=32.0, help="--assign: host-to-device rate behind the transfer time of an uncached expert")
    ap.add_argument("--library-gemm", action="store_true",
                    help="context only: the vendor library's dense bf16 GEMM (torch.matmul) on the prefill workload's shapes")
    ap.add_argument("--calib-copy", action="store_true",
                    help="only run a plain 1 GiB device-to-device copy 5 times (reference for scaling the FETCH_SIZE / WRITE_SIZE counters)")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        log("bench.py: this build runs on one GPU only (no collectives, no sharding); use --gpus 1")
        sys.exit(2)

    import torch
    from paper_2602_03495_amd import binding as B
    from paper_2602_03495_amd import layer as Lm
    from paper_2602_03495_amd import workloads as wl

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    B.load_library()   # raises if the HIP library has not been built
    torch.cuda.set_device(0)

    if args.library_gemm:
        print(json.dumps(library_gemm_yardstick(torch)), flush=True)
        return

    if args.assign:
        print(json.dumps(greedy_assignment_demo(torch, B, Lm, wl, args.pcie_gbs)), flush=True)
        return

    if args.calib_copy:
        src = torch.empty(1 << 30, dtype=torch.uint8, device="cuda").fill_(1)
        dst = torch.empty_like(src)
        for _ in range(5):
            dst.copy_(src)
        torch.cuda.synchronize()
        log("[bench] calibration copy done: 5 x (1 GiB read + 1 GiB written)")
        return

    if args.timeline:
        print(json.dumps(timeline(torch, B, Lm, wl, args.timeline)), flush=True)
        return

    if args.one:
        name, T1, mk = args.one.split(":")
        rec = survey_config(torch, B, Lm, wl, name, [int(T1)], mk, steps=args.steps, merged=args.one_merged)[0]
        print(json.dumps({"metric": "MoE-layer step time, one shape", "unit": "us", "n_gpus": 1, "dtype": "bf16", "data": "synthetic",
                          "config": {"workload": f"{name}-shaped layer, {T1} tokens, mask {mk}"}, **rec}), flush=True)
        return

    if args.survey:
        recs = []
        for name, Ts, mk in (("mixtral", [2048, 4096, 8192, 16384, 16, 1], "rand6"), ("deepseek", [2048, 16], "half"), ("qwen15", [4096, 1], "all"),
                             ("qwen3", [2048, 16], "half")):
            recs += survey_config(torch, B, Lm, wl, name, Ts, mk)
        mid = []
        for name in ("mixtral", "deepseek", "qwen3"):
            mid += survey_mid(torch, B, Lm, wl, name)
        print(json.dumps({"metric": "MoE-layer step time by shape", "unit": "us", "n_gpus": 1, "dtype": "bf16", "data": "synthetic",
                          "config": {"workload": "all layer shapes: prefill, decode and mid-sized batches"},
                          "steps": recs, "mid_sized": mid, "few_experts_on": survey_few_experts(torch, B, Lm, wl),
                          "rows_per_expert": survey_rows_per_expert(torch, B, Lm, wl)}), flush=True)
        return

    if args.stack:
        from bench_stack import DecodeStack
        cfg5 = wl.CONFIGS["qwen3"]
        t0 = time.time()
        st = DecodeStack(cfg5, args.stack_layers, 16)
        log(f"[bench] stack: {args.stack_layers} layers resident ({torch.cuda.memory_allocated() / 2**30:.1f} GiB) after {time.time() - t0:.0f}s")
        bias = st.bias_paths(args.stack_steps)
        st.calibrate(bias)
        res = st.run(args.stack_steps, bias, use_res_vec=True)
        raw = st.run(min(args.stack_steps, 64), bias, use_res_vec=False)
        # cost of the prediction per layer: issued inline, on a second stream next to routing/FFN/combine, or not at all
        n_ov = min(args.stack_steps, 64)
        ov = {mode: st.run(n_ov, bias, predict=mode).seconds / n_ov / args.stack_layers * 1e6 for mode in ("off", "inline", "side", "fused")}
        log(f"[bench] stack us/layer, eager launches: no prediction {ov['off']:.1f}, inline {ov['inline']:.1f}, side stream {ov['side']:.1f}, fused with routing {ov['fused']:.1f}")
        ovg = {mode: st.layer_graph_seconds(bias, predict=mode) * 1e6 for mode in ("off", "inline", "side", "fused")}
        log(f"[bench] one layer as a replayed graph, us: no prediction {ovg['off']:.1f}, inline {ovg['inline']:.1f}, side stream {ovg['side']:.1f}, fused with routing {ovg['fused']:.1f}")
        c = res.counts
        # Workload-Aware Cache Replacement (Alg. 2) replayed over the measured histogram stream, one cache per layer:
        # 64 of 128 experts resident, w_size = 4, u_size = 8; hit rate = share of the routed rows that found their
        # expert resident, against a cache that keeps its initial (lower-half) contents
        tot = hits_static = 0
        hits, loads = {}, {}
        t_sched = time.perf_counter()
        # Alg. 2 as printed (u_size experts change sides at every window end) and the guarded variant (a pair only while
        # the incoming score is larger), which is not the paper's
        for mode_name, mode in (("as_printed", B.CACHE_ALWAYS), ("guarded_variant", B.CACHE_GUARDED)):
            hits[mode_name] = loads[mode_name] = 0
            for l in range(args.stack_layers):
                cache = B.ExpertCache(cfg5.N, range(cfg5.N // 2), 4, 8, mode)
                for t in range(args.stack_steps):
                    w = c[t, l]
                    hits[mode_name] += int(w[cache.on_gpu.astype(bool)].sum())
                    loads[mode_name] += len(cache.step(w))
        t_sched = (time.perf_counter() - t_sched) / 2
        static = np.zeros(cfg5.N, bool)
        static[: cfg5.N // 2] = True
        for l in range(args.stack_layers):
            for t in range(args.stack_steps):
                hits_static += int(c[t, l][static].sum())
                tot += int(c[t, l].sum())
        # the comparison policy of Section "Workload-Aware Cache Replacement": least recently used, same capacity and
        # initial contents; an activated expert that is not resident is loaded at once in place of the one unused longest
        hits_lru = loads_lru = 0
        for l in range(args.stack_layers):
            last = np.full(cfg5.N, -1, np.int64)
            res_ = np.zeros(cfg5.N, bool)
            res_[: cfg5.N // 2] = True
            for t in range(args.stack_steps):
                w = c[t, l]
                hits_lru += int(w[res_].sum())
                used = np.nonzero(w > 0)[0]
                last[used] = t
                for e in used[~res_[used]]:
                    cand = np.nonzero(res_)[0]
                    victim = cand[np.argmin(last[cand])]
                    if last[victim] == t:
                        break                     # everything resident was used in this step
                    res_[victim], res_[e] = False, True
                    loads_lru += 1
        hist = {"shape": list(c.shape), "max_workload": int(c.max()), "mean_active_experts": float((c > 0).sum(-1).mean()),
                "mean_top1_share": float((c.max(-1) / c.sum(-1)).mean()),
                "first_step_first_layer": c[0, 0].tolist()}
        out = {"metric": "decode-stack tokens/sec (48 layers x 256 steps, batch 16)", "value": res.tokens_per_s, "unit": "tokens/s",
               "n_gpus": 1, "steps": args.stack_steps, "layers": args.stack_layers, "ms_per_step": res.seconds / args.stack_steps * 1e3,
               "us_per_layer": res.seconds / args.stack_steps / args.stack_layers * 1e6, "dtype": "bf16", "data": "synthetic",
               "config": {"workload": "qwen3-30b-a3b-shaped decode stack, AR(1) gate bias rho=0.9, mask = top half by previous step"},
               "prediction_accuracy_with_res_vec": res.acc, "prediction_accuracy_without_res_vec": raw.acc,
               "prediction_overlap_us_per_layer": {"eager": {"no_prediction": ov["off"], "inline": ov["inline"], "side_stream": ov["side"], "fused_with_routing": ov["fused"]},
                                                   "graph_replay": {"no_prediction": ovg["off"], "inline": ovg["inline"], "side_stream": ovg["side"], "fused_with_routing": ovg["fused"]}},
               "cache_replacement": {"policy": "workload-aware (Alg. 2), 64 of 128 resident, w_size 4, u_size 8",
                                     "hit_rate": hits["as_printed"] / tot, "hit_rate_static_cache": hits_static / tot,
                                     "expert_loads_per_layer_step": loads["as_printed"] / (args.stack_layers * args.stack_steps),
                                     "guarded_variant_hit_rate": hits["guarded_variant"] / tot,
                                     "guarded_variant_expert_loads_per_layer_step": loads["guarded_variant"] / (args.stack_layers * args.stack_steps),
                                     "lru_hit_rate": hits_lru / tot,
                                     "lru_expert_loads_per_layer_step": loads_lru / (args.stack_layers * args.stack_steps),
                                     "host_us_per_layer_step": t_sched / (args.stack_layers * args.stack_steps) * 1e6},
               "histograms": hist}
        print(json.dumps(out), flush=True)
        return

    cfg = wl.CONFIGS["mixtral"]
    T = 2048
    t0 = time.time()
    W, b = wl.gate_weights(cfg), wl.gate_bias(cfg)
    w1, w3, w2 = wl.expert_weights(cfg)
    mask = wl.mask_random(cfg, 6)
    log(f"[bench] generated {cfg.name} weights in {time.time() - t0:.1f}s; mask={mask.tolist()}")
    dw = Lm.LayerWeights.upload(W, b, w1, w3, w2)
    mask_d = torch.from_numpy(mask).cuda()
    on = mask.astype(bool)

    # ---- prefill ------------------------------------------------------------------------------------
    h = wl.hidden_states(cfg, T)
    hd = Lm.to_device_bf16(h)
    L = Lm.MoeLayer(cfg, T)
    t = time_steps(torch, B, L, hd, dw, mask_d, args.steps, args.warmup)
    counts = L.routing.counts.cpu().numpy()
    rows_on = int(counts[on].sum())
    active = int(((counts > 0) & on).sum())
    up_flops = 4.0 * cfg.d * cfg.I * rows_on           # gate + up products of the masked-on rows
    down_flops = 2.0 * cfg.d * cfg.I * rows_on
    ffn_flops = up_flops + down_flops                   # 6 d I per masked-on routed row
    ffn_bytes = 6.0 * cfg.d * cfg.I * active            # the other bound: weights of the touched masked-on experts once
    # The timed steps proper: the same pass (route, expert FFN, combine) captured once in a HIP graph and replayed, as the
    # decode steps below are, so that the host's launch cost is not in the figure; the eager steps above, with their
    # events between the launches, give the kernel durations of the roofline.
    wall_graph = time_graph_replays(torch, L, hd, dw, mask_d, args.steps, args.warmup)
    ms_per_step = wall_graph / args.steps * 1e3
    eager_ms_per_step = t["wall"] / args.steps * 1e3
    value = T / (wall_graph / args.steps)
    log(f"[bench] prefill T={T}: {ms_per_step:.3f} ms/step as a replayed graph, {eager_ms_per_step:.3f} eager with events (median {t['step_median'] * 1e3:.3f}), up {t['up_mean'] * 1e3:.3f} ms, "
        f"down {t['down_mean'] * 1e3:.3f} ms, ffn {t['ffn_mean'] * 1e3:.3f} ms, counts={counts.tolist()}, rows_on={rows_on}")
    frac = lambda fl, sec: fl / sec / PEAK_BF16_MFMA
    # The dominant work is the expert FFN: two launches (up projection + SwiGLU, down projection).  achieved = its
    # algorithmic flops, 6 d I per masked-on routed row, over the mean time of the two launches per step.
    roofline = {"bound": "mfma", "kernel": "expert FFN: ffn_tiled_kernel<0,...> (gate/up projection + SwiGLU) + ffn_tiled_kernel<1,...> (down projection)",
                "achieved": ffn_flops / t["ffn_mean"] / 1e12, "peak": PEAK_BF16_MFMA / 1e12, "unit": "TFLOP/s",
                "frac": frac(ffn_flops, t["ffn_mean"]), "traffic": TRAFFIC_PREFILL["up"] + TRAFFIC_PREFILL["down"],
                "traffic_source": TRAFFIC_SOURCE,
                "flops_per_launch": ffn_flops, "avg_launch_ms": t["ffn_mean"] * 1e3, "median_launch_ms": t["ffn_median"] * 1e3,
                "frac_of_median": frac(ffn_flops, t["ffn_median"]),
                "per_kernel": {
                    "up": {"flops_per_launch": up_flops, "avg_launch_ms": t["up_mean"] * 1e3, "median_launch_ms": t["up_median"] * 1e3,
                           "frac": frac(up_flops, t["up_mean"]), "traffic": TRAFFIC_PREFILL["up"]},
                    "down": {"flops_per_launch": down_flops, "avg_launch_ms": t["down_mean"] * 1e3, "median_launch_ms": t["down_median"] * 1e3,
                             "frac": frac(down_flops, t["down_mean"]), "traffic": TRAFFIC_PREFILL["down"]}},
                "ffn_frac": frac(ffn_flops, t["ffn_mean"]),
                # the other bound of the same FFN, and the larger of the two (what a perfect kernel would be held to)
                "ffn_hbm_frac": ffn_bytes / t["ffn_mean"] / PEAK_HBM,
                "bound_frac": max(frac(ffn_flops, t["ffn_mean"]), ffn_bytes / t["ffn_mean"] / PEAK_HBM)}
    # the next-layer workload prediction is not part of the step above; alone it costs (next gate = this layer's, a stand-in)
    rv = torch.from_numpy(wl.layer_drift(cfg)).cuda()
    top = torch.empty(1, dtype=torch.int32, device="cuda")
    predict_us = {"prefill_2048": median_event_seconds(torch, lambda: L.predict(hd, rv, dw, 1, top)) * 1e6}

    # ---- decode -------------------------------------------------------------------------------------
    decode = []
    if not args.no_decode:
        for Td in (1, 16):
            hdd = Lm.to_device_bf16(wl.hidden_states(cfg, Td, draw=10 + Td))
            Ld = Lm.MoeLayer(cfg, Td)
            td = time_steps(torch, B, Ld, hdd, dw, mask_d, args.decode_steps, args.warmup)
            wall_d, up_d, ffn_d = td["wall"], td["up_mean"], td["ffn_mean"]
            c = Ld.routing.counts.cpu().numpy()
            active = int(((c > 0) & on).sum())
            up_bytes = 4.0 * cfg.d * cfg.I * active          # W1 and W3 of the touched, masked-on experts, bf16
            ffn_bytes = 6.0 * cfg.d * cfg.I * active
            wall_g = time_graph_replays(torch, Ld, hdd, dw, mask_d, args.decode_steps, args.warmup)
            decode.append({"T": Td, "value": Td / (wall_g / args.decode_steps), "unit": "tokens/s",
                           "ms_per_step": wall_g / args.decode_steps * 1e3, "launch": "hip graph replay",
                           "eager_ms_per_step": wall_d / args.decode_steps * 1e3, "active_experts": active,
                           "roofline": {"bound": "hbm", "kernel": "skinny_up_kernel", "achieved": up_bytes / up_d / 1e9 if active else 0.0,
                                        "peak": PEAK_HBM / 1e9, "unit": "GB/s", "frac": up_bytes / up_d / PEAK_HBM if active else 0.0,
                                        "ffn_frac": ffn_bytes / ffn_d / PEAK_HBM if active else 0.0,
                                        "step_frac": ffn_bytes / (wall_g / args.decode_steps) / PEAK_HBM if active else 0.0,
                                        "bytes_per_launch": up_bytes, "avg_launch_ms": up_d * 1e3, "median_launch_ms": td["up_median"] * 1e3,
                                        "traffic": TRAFFIC_DECODE_UP.get(Td), "traffic_source": TRAFFIC_SOURCE}})
            predict_us[f"decode_{Td}"] = median_event_seconds(torch, lambda: Ld.predict(hdd, rv, dw, 1, top)) * 1e6
            predict_us[f"decode_{Td}_route_alone"] = median_event_seconds(torch, lambda: Ld.route(hdd, dw)) * 1e6
            predict_us[f"decode_{Td}_route_and_predict_fused"] = median_event_seconds(
                torch, lambda: Ld.route_predict(hdd, dw, rv, dw, 1, top)) * 1e6
            log(f"[bench] decode T={Td}: graph {decode[-1]['ms_per_step']:.4f} ms/step, eager {decode[-1]['eager_ms_per_step']:.4f}, "
                f"up {up_d * 1e3:.4f} ms, ffn {ffn_d * 1e3:.4f} ms, active={active}")

    # ---- CPU oracle on a bounded sample -----------------------------------------------------------------
    cpu = None
    if args.cpu_sample > 0:
        oracle = cpu_baseline_oracle()
        n = min(args.cpu_sample, T)
        toks = np.arange(n, dtype=np.int32)
        t0 = time.perf_counter()
        lg, idx, w, _ = oracle.route(h[:n], W, b, cfg.k, cfg.norm_mode)
        oracle.layer(h[:n], idx, w, w1, w3, w2, mask, tokens=toks)
        dt = time.perf_counter() - t0
        cpu = {"value": n / dt, "unit": "tokens/s", "cores": oracle.num_threads(), "kind": "oracle",
               "sample": f"first {n} tokens of the prefill batch, route + masked expert FFN + combine, {dt:.1f} s"}
        log(f"[bench] oracle: {n} tokens in {dt:.1f}s on {cpu['cores']} threads")

    # ---- the other layer shapes, same run (prefill and decode of each; eager launches, HIP events between the calls,
    # medians; decode steps with the Infinity Cache read through between steps) --------------------------------------
    others = []
    if not args.no_other_workloads:
        del dw, L
        torch.cuda.empty_cache()
        for name, Ts, mk in (("deepseek", [2048, 16], "half"), ("qwen15", [4096, 1], "all"), ("qwen3", [2048, 16], "half")):
            others += survey_config(torch, B, Lm, wl, name, Ts, mk)

    out = {"metric": "MoE-layer tokens/sec (prefill 2048 tok)", "value": value, "unit": "tokens/s", "n_gpus": 1,
           "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_per_step, "launch": "hip graph replay of route + expert FFN + combine",
           "eager_ms_per_step": eager_ms_per_step, "median_eager_ms_per_step": t["step_median"] * 1e3,
           "higher_is_better": True,
           "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
           "config": {"workload": "mixtral-8x7b-shaped layer, prefill 2048 tokens", "d": cfg.d, "experts": cfg.N,
                      "top_k": cfg.k, "inner": cfg.I, "experts_on_gpu": int(on.sum()), "tokens": T},
           "roofline": roofline, "cpu_baseline": cpu, "decode": decode, "predict_workload_us": predict_us,
           "other_workloads": others}
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()

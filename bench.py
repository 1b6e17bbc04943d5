#!/usr/bin/env python3
"""Benchmark of the MoE-layer hot path on one MI355X.

One "step" is one pass of the whole path over one batch of synthetic tokens:
predict_topk (next layer's cloned gate) -> route_topk -> permute -> grouped_ffn -> combine,
all through the C ABI of libprobe.so on one stream, inputs resident in HBM, every buffer
pre-allocated.  The default workload is the DeepSeek-V3-shaped shard (configuration 3 of the
benchmark's list, the one its target is quoted on); successive steps rotate over 8 batches whose
hot expert set moves, so no step re-reads the previous step's activations from cache.

Prints ONE JSON line: metric/value/unit, per-stage times, the roofline of the dominant call
(the grouped FFN) and the CPU oracle timed on the host cores as a baseline.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0     # MI355X dense bf16 MFMA
PEAK_HBM_GBPS = 8000.0        # MI355X HBM3E


def measured_ffn_traffic(cid):
    """L2-miss fetch + write bytes of the FFN's two GEMM kernels per call, from the rocprofv3 --pmc summary
    committed for this configuration (FETCH_SIZE / WRITE_SIZE scaled by a plain copy kernel; the figures and
    the commands are in the file).  None if there is no summary for the configuration."""
    import re
    path = os.path.join(ROOT, "profiles", "bench_cfg%d_hbm_traffic.md" % cid)
    try:
        m = re.search(r"FFN_TRAFFIC_BYTES_PER_CALL\s*[:=]\s*([0-9.eE+]+)", open(path).read())
    except OSError:
        return None
    return float(m.group(1)) if m else None


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=40)
    ap.add_argument("--warmup", type=int, default=8)
    ap.add_argument("--config", type=int, default=3, help="benchmark configuration (1-5; 6, 7 = the shapes of the models the paper evaluates)")
    ap.add_argument("--batches", type=int, default=0, help="distinct batches to rotate over (0 = config default)")
    ap.add_argument("--residual-width", type=int, default=0,
                    help="width D of the predictor's residual MLP (Eq. 7); 0 = residual at its zero initialisation, "
                         "i.e. probe_predict_topk")
    ap.add_argument("--fused-route-predict", action="store_true",
                    help="one probe_route_predict_topk call instead of predict_topk + route_topk (the predictor of "
                         "the next layer reads the same hidden states as this layer's router)")
    ap.add_argument("--gather-on-load", action="store_true",
                    help="probe_permute without the row copy + probe_grouped_ffn_gather (no xp is written or read)")
    ap.add_argument("--graph", action="store_true",
                    help="record each batch's step into a HIP graph and time replays (stage times still come from "
                         "an eager pass)")
    ap.add_argument("--unpacked-gate", action="store_true",
                    help="hand the router and the predictor the fp32 gate matrices, which they split into bf16 planes "
                         "on every call (default: planes made once by probe_pack_gate, untimed set-up whose cost is "
                         "reported as gate_pack_us)")
    ap.add_argument("--main-only", action="store_true",
                    help="only the timed step: no measured peaks, predictor overlap, planner, group-limited gate or "
                         "predicted-plan sections and no CPU baseline (for profiler runs, so that a kernel's average "
                         "in the trace is its average over the step's launches)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-sample-tokens", type=int, default=0)
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="after the timed steps, run a plain 1 GiB read + 1 GiB write elementwise kernel three "
                         "times (reference for the FETCH_SIZE / WRITE_SIZE counters of a rocprofv3 --pmc run)")
    args = ap.parse_args()
    if args.gpus != 1:
        log("bench.py: this build is a one-GPU hot path (no collectives); run with --gpus 1")
        sys.exit(2)

    import torch
    from paper_2602_00509_amd import probe, workload as wl

    if not torch.cuda.is_available():
        log("bench.py: no GPU visible")
        sys.exit(3)
    probe.lib()                                   # fail loudly if the HIP library is missing
    cfg = wl.CONFIGS[args.config]
    T, H, E, k, F, S = cfg.T, cfg.H, cfg.E, cfg.k, cfg.F, cfg.S
    nb = args.batches or min(cfg.n_batches, 8)
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    threads = min(16, os.cpu_count() or 8)

    def dev_bf16(bits):
        return torch.from_numpy(np.ascontiguousarray(bits).view(np.int16)).to(dev).view(torch.bfloat16)

    # ------------------------------------------------------------------ inputs
    t0 = time.time()
    wg = wl.gate_weights(cfg, 0)
    wg_next = wl.gate_weights(cfg, 1)
    d_wg, d_wg_next = torch.from_numpy(wg).to(dev), torch.from_numpy(wg_next).to(dev)
    tpg = wl.tokens_per_group(cfg)
    xs, d_xs, d_bias, d_bias_next, biases = [], [], [], [], []
    for b in range(nb):
        x = wl.activations(cfg, b)
        xs.append(x)
        d_xs.append(dev_bf16(x))
        biases.append(wl.zipf_bias(cfg, b, 0))
        d_bias.append(torch.from_numpy(biases[-1]).to(dev))
        d_bias_next.append(torch.from_numpy(wl.zipf_bias(cfg, b, 1)).to(dev))
    log("inputs: %d batches of %dx%d in %.1fs" % (nb, T, H, time.time() - t0))

    # pre-allocated outputs and workspaces (one set, reused by every step)
    N = T * k
    r_out = dict(idx=torch.empty((T, k), dtype=torch.int32, device=dev),
                 w=torch.empty((T, k), dtype=torch.float32, device=dev),
                 counts=torch.empty((E,), dtype=torch.int32, device=dev))
    p_out_pred = dict(idx=torch.empty((T, k), dtype=torch.int32, device=dev),
                      w=torch.empty((T, k), dtype=torch.float32, device=dev),
                      counts=torch.empty((E,), dtype=torch.int32, device=dev))
    ws_route = torch.empty(probe.route_topk_workspace_bytes(T, H, E, k), dtype=torch.uint8, device=dev)
    ws_fused = (torch.empty(probe.route_predict_topk_workspace_bytes(T, H, E, k), dtype=torch.uint8, device=dev)
                if args.fused_route_predict else None)
    # the gates as the calls take them: bf16 planes packed once (the router's weights are frozen while serving),
    # or the fp32 matrices themselves
    g_route, g_pred, g_fused, g_fused_next, pack_us = d_wg, d_wg_next, d_wg, d_wg_next, None
    if not args.unpacked_gate:
        probe.PackedGate(d_wg)                    # first call: module load
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        g_route = probe.PackedGate(d_wg)
        e1.record()
        torch.cuda.synchronize()
        pack_us = e0.elapsed_time(e1) * 1e3
        g_pred = probe.PackedGate(d_wg_next)
        if args.fused_route_predict:
            g_fused, g_fused_next = probe.PackedGate(d_wg, d_wg_next), None
    D = args.residual_width
    if D:
        rng = np.random.default_rng(1000 + cfg.cid)
        d_w1 = dev_bf16(wl.f32_to_bf16_bits(rng.standard_normal((D, H), dtype=np.float32) * np.float32(1.5 / np.sqrt(H))))
        d_w2 = torch.from_numpy((rng.standard_normal((E, D)) * (0.3 / np.sqrt(D))).astype(np.float32)).to(dev)
        ws_pred = torch.empty(probe.predict_topk_residual_workspace_bytes(T, H, E, k, D), dtype=torch.uint8, device=dev)
    ws_perm = torch.empty(max(256, probe.permute_workspace_bytes(T, E, k, S)), dtype=torch.uint8, device=dev)
    ws_ffn = torch.empty(probe.grouped_ffn_workspace_bytes(S, H, F, N), dtype=torch.uint8, device=dev)
    perm_out = dict(slot_counts=torch.empty((S,), dtype=torch.int32, device=dev),
                    slot_offsets=torch.empty((S + 1,), dtype=torch.int32, device=dev),
                    row_pair=torch.empty((N,), dtype=torch.int32, device=dev),
                    pair_row=torch.empty((T, k), dtype=torch.int32, device=dev),
                    xp=torch.empty((N, H), dtype=torch.bfloat16, device=dev),
                    n_local=torch.empty((1,), dtype=torch.int32, device=dev))
    perm_lean = {kk: v for kk, v in perm_out.items() if kk != "xp"}
    y = torch.empty((N, H), dtype=torch.bfloat16, device=dev)
    out = torch.empty((T, H), dtype=torch.bfloat16, device=dev)

    # plans: the host recipe of the workload, from each batch's routed counts (set-up, untimed)
    plans, d_plans, n_locals, slot_experts, active_slots, all_counts = [], [], [], [], [], []
    for b in range(nb):
        probe.route_topk(d_xs[b], d_wg, d_bias[b], tpg, k, True, out=r_out, workspace=ws_route)
        counts = r_out["counts"].cpu().numpy()
        all_counts.append(counts.copy())
        plan = wl.build_plan(cfg, counts)
        plans.append(plan)
        d_plans.append(probe.Plan(plan["rep_off"], plan["rep_slot"], plan["rep_weight"], plan["num_slots"], dev))
        slot_experts.append(plan["slot_expert"])
    # expert weights: one buffer per (expert) used by any batch; a slot table per batch
    t0 = time.time()
    need = sorted({int(e) for se in slot_experts for e in se})
    host_w = dict(zip(need, wl.expert_weights_many(cfg, need, threads=threads)))
    dev_w = {e: (dev_bf16(host_w[e][0]), dev_bf16(host_w[e][1])) for e in need}
    tables = [probe.WeightTable([dev_w[int(e)][0] for e in se], [dev_w[int(e)][1] for e in se])
              for se in slot_experts]
    log("expert weights: %d experts (%.2f GB) in %.1fs" %
        (len(need), len(need) * 3 * H * F * 2 / 1e9, time.time() - t0))

    def step(b, ev=None):
        def mark(i):
            if ev is not None:
                ev[i].record()
        mark(0)
        if args.fused_route_predict:
            probe.route_predict_topk(d_xs[b], g_fused, d_bias[b], g_fused_next, d_bias_next[b], tpg, k, True,
                                     out=r_out, pred_out=p_out_pred, workspace=ws_fused)
            mark(1)
        elif D:
            probe.predict_topk_residual(d_xs[b], d_wg_next, d_bias_next[b], tpg, d_w1, d_w2, k, True, out=p_out_pred,
                                        workspace=ws_pred)
        else:
            probe.predict_topk(d_xs[b], g_pred, d_bias_next[b], tpg, k, True, out=p_out_pred, workspace=ws_route)
        if not args.fused_route_predict:
            mark(1)
            probe.route_topk(d_xs[b], g_route, d_bias[b], tpg, k, True, out=r_out, workspace=ws_route)
        mark(2)
        if args.gather_on_load:
            probe.permute(r_out["idx"], d_plans[b], d_xs[b], out=perm_lean, workspace=ws_perm, copy_rows=False)
            mark(3)
            probe.grouped_ffn_gather(d_xs[b], perm_out["row_pair"], k, perm_out["slot_offsets"], tables[b], out=y,
                                     workspace=ws_ffn)
        else:
            probe.permute(r_out["idx"], d_plans[b], d_xs[b], out=perm_out, workspace=ws_perm)
            mark(3)
            probe.grouped_ffn(perm_out["xp"], perm_out["slot_offsets"], tables[b], out=y, workspace=ws_ffn)
        mark(4)
        probe.combine(y, perm_out["pair_row"], r_out["w"], out=out)
        mark(5)

    for b in range(nb):                           # rows per batch (set-up; also first warm-up)
        step(b)
        n_locals.append(int(perm_out["n_local"].item()))
        active_slots.append(int((perm_out["slot_counts"] > 0).sum().item()))
    for i in range(args.warmup):
        step(i % nb)
    torch.cuda.synchronize()

    events = [[torch.cuda.Event(enable_timing=True) for _ in range(6)] for _ in range(args.steps)]
    torch.cuda.synchronize()
    t_start = time.perf_counter()
    for i in range(args.steps):
        step(i % nb, events[i])
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t_start
    if args.graph:
        # one graph per batch, recorded on a side stream; the timed region replays them
        graphs = []
        cap = torch.cuda.Stream()
        cap.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(cap):
            for b in range(nb):
                g = torch.cuda.CUDAGraph()
                with torch.cuda.graph(g, stream=cap):
                    step(b)
                graphs.append(g)
        torch.cuda.synchronize()
        for i in range(args.warmup):
            graphs[i % nb].replay()
        torch.cuda.synchronize()
        t_start = time.perf_counter()
        for i in range(args.steps):
            graphs[i % nb].replay()
        torch.cuda.synchronize()
        elapsed = time.perf_counter() - t_start

    names = ["predict", "route", "permute", "ffn", "combine"]
    stage_ms = {n: [] for n in names}
    for i in range(args.steps):
        for j, n in enumerate(names):
            stage_ms[n].append(events[i][j].elapsed_time(events[i][j + 1]))
    mean_ms = {n: float(np.mean(v)) for n, v in stage_ms.items()}
    ms_per_step = elapsed * 1e3 / args.steps
    nl_steps = [n_locals[i % nb] for i in range(args.steps)]
    nl_mean = float(np.mean(nl_steps))

    # algorithmic work per step (mean over the batches the timed steps used)
    ffn_flops = 6.0 * nl_mean * H * F
    ffn_tflops = ffn_flops / (mean_ms["ffn"] * 1e-3) / 1e12
    route_bytes = T * H * 2 + E * H * 4 + T * k * 8
    perm_bytes = T * k * 4 + T * H * 2 + nl_mean * H * 2 + 16 * T * k
    comb_bytes = nl_mean * H * 2 + T * H * 2 + T * k * 8
    gbps = {"predict": route_bytes / mean_ms["predict"] / 1e6, "route": route_bytes / mean_ms["route"] / 1e6,
            "permute": perm_bytes / mean_ms["permute"] / 1e6, "combine": comb_bytes / mean_ms["combine"] / 1e6}
    act_mean = float(np.mean([active_slots[i % nb] for i in range(args.steps)]))
    ffn_bytes = act_mean * 3 * H * F * 2 + 2 * nl_mean * H * 2   # weights of non-empty slots once + xp + y

    # gate GEMMs per stage: the fused call runs both gates under "predict"
    gates = {"predict": 2, "route": 0} if args.fused_route_predict else {"predict": 1, "route": 1}
    gate_tflops = {n: g * 3 * 2.0 * T * H * E / (mean_ms[n] * 1e-3) / 1e12 for n, g in gates.items() if g}

    # The dominant call's roofline: the matrix cores bind when the call's algorithmic intensity (flops per byte of
    # weights, xp and y) is above the ridge of the nominal peaks (2500 TFLOP/s / 8 TB/s = 312 flop/B); below it
    # (decode: a few rows per slot) the call is a stream of the active slots' weights and HBM binds.
    traffic = measured_ffn_traffic(cfg.cid) if nb == min(cfg.n_batches, 8) else None
    ffn_kernels = ("probe_grouped_ffn (ffn_gemm1_skinny_kernel + ffn_gemm2_skinny_kernel)" if N <= 64 * S else
                   "probe_grouped_ffn (ffn_gemm1_kernel + ffn_gemm2_kernel)")    # the library's own rule
    if ffn_flops / ffn_bytes >= PEAK_BF16_TFLOPS * 1e12 / (PEAK_HBM_GBPS * 1e9):
        ffn_roofline = {"kernel": ffn_kernels, "bound": "mfma",
                        "achieved": ffn_tflops, "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s",
                        "frac": ffn_tflops / PEAK_BF16_TFLOPS}
    else:
        ffn_gbps = ffn_bytes / mean_ms["ffn"] / 1e6
        ffn_roofline = {"kernel": ffn_kernels, "bound": "hbm", "achieved": ffn_gbps, "peak": PEAK_HBM_GBPS, "unit": "GB/s",
                        "frac": ffn_gbps / PEAK_HBM_GBPS}
    ffn_roofline.update({"traffic": traffic, "algorithmic_flops_per_launch": ffn_flops,
                         "algorithmic_bytes_per_launch": ffn_bytes, "launch_ms": mean_ms["ffn"]})

    result = {
        "metric": "moe_layer_tokens_per_s",
        "value": T * args.steps / elapsed,
        "unit": "tokens/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic", "launch": "hip_graph_replay" if args.graph else "eager",
        "gate": "fp32 matrices, split per call" if args.unpacked_gate else "bf16 planes packed once (probe_pack_gate)",
        "gate_pack_us": pack_us,
        "config": {"workload": "cfg%d %s: T=%d H=%d E=%d top-%d F=%d, %d native + %d replica slots, Zipf s=%.1f, "
                               "%d rotating batches" % (cfg.cid, cfg.name, T, H, E, k, F, cfg.E_loc, cfg.n_rep,
                                                        cfg.zipf_s, nb),
                   "step": ("route_predict_topk (stage time reported under predict, route = 0)"
                            if args.fused_route_predict else
                            ("predict_topk_residual(D=%d)" % D if D else "predict_topk") + " + route_topk") +
                           (" + permute (index outputs only) + grouped_ffn_gather + combine" if args.gather_on_load
                            else " + permute + grouped_ffn + combine"),
                   "rows_per_step_mean": nl_mean, "active_slots_mean": act_mean},
        "stage_ms": mean_ms,
        "stage_ms_min": {n: float(np.min(v)) for n, v in stage_ms.items()},
        "main_track_tokens_per_s": T / ((mean_ms["route"] + mean_ms["permute"] + mean_ms["ffn"] + mean_ms["combine"]) * 1e-3),
        "ffn_tflops": ffn_tflops,
        "ffn_frac_bf16_mfma_peak": ffn_tflops / PEAK_BF16_TFLOPS,
        "ffn_weight_stream_gbps": ffn_bytes / mean_ms["ffn"] / 1e6,
        # algorithmic bytes of a stage over its time: rows just written by the previous stage are partly served by
        # the 256 MB last-level cache, so these can exceed what a streaming copy reaches on the box
        # (roofline.peak_measured) and are rates of algorithmic bytes, not proven HBM traffic
        "stage_algorithmic_gbps": gbps,
        "stage_algorithmic_frac_hbm_peak": {n: v / PEAK_HBM_GBPS for n, v in gbps.items()},
        # the gate is a contraction of 2*T*H*E flops that runs on the matrix cores as three bf16 planes (fp32
        # weights kept exact), so its arithmetic roof is the bf16 MFMA peak over plane-expanded flops; at E >= 128
        # that roof binds, at E = 8 the HBM one does
        "gate_binding_roof": "mfma" if E >= 64 else "hbm",
        "gate_plane_expanded_tflops": gate_tflops,
        "gate_frac_bf16_mfma_peak": {n: v / PEAK_BF16_TFLOPS for n, v in gate_tflops.items()},
        "roofline": ffn_roofline,
    }

    if not args.main_only:
        # what this machine sustains, next to the nominal peaks: MFMA-only loop (no memory instruction) with zero
        # and with random bf16 operands, and a plain streaming copy
        result["roofline"]["peak_measured"] = measure_peaks(torch, dev)
        result["roofline"]["frac_of_measured_mfma_random"] = (
            ffn_tflops / result["roofline"]["peak_measured"]["mfma_only_random_operands_tflops"])

        # the predictor's top-k accuracy: the cloned gate of the next layer on this layer's hidden states against
        # the same gate on the next layer's hidden states (drifted copies of batch 0; two drift levels)
        ov = {}
        for alpha in (0.2, 0.5):
            d_xn = dev_bf16(wl.drifted_activations(cfg, xs[0], alpha, 0))
            pr = probe.predict_topk(d_xs[0], d_wg_next, d_bias_next[0], tpg, k, True)
            tr = probe.route_topk(d_xn, d_wg_next, d_bias_next[0], tpg, k, True)
            hits, _ = probe.predictor_metrics(pr["idx"], tr["idx"])
            ov["drift_%.1f" % alpha] = int(hits.item()) / float(T * k)
            del d_xn
        result["predictor_topk_overlap"] = ov

        # the greedy planner (Algorithm 1) on the device, timed on its own: the batches stand in for the source
        # ranks whose predicted counts an all-gather would deliver; not part of `value`
        ep = cfg.E // cfg.E_loc
        if 2 <= ep <= 16 and cfg.E_loc * ep == E:
            rows = [all_counts[r % nb] for r in range(ep)]
            d_nhat = torch.from_numpy(np.stack(rows).astype(np.int32)).to(dev)
            kw = dict(max_replicas=cfg.n_rep if cfg.n_rep else 3, budget=3, k_max=16, n0=64, g_num=1, g_den=4)
            for _ in range(3):
                pl = probe.plan_greedy(d_nhat, cfg.E_loc, rank=0, **kw)
            torch.cuda.synchronize()
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            for _ in range(20):
                pl = probe.plan_greedy(d_nhat, cfg.E_loc, rank=0, **kw)
            e1.record()
            torch.cuda.synchronize()
            st = pl["stats"].cpu().tolist()
            # Eq. 1 on token loads: before = every expert at home, after = the plan's assignment
            per_expert = np.stack(rows).astype(np.int64).sum(0)
            home_load = per_expert.reshape(ep, cfg.E_loc).sum(1)
            mean_load = float(per_expert.sum()) / ep
            result["planner"] = {"us_per_call": e0.elapsed_time(e1) * 1e3 / 20, "ranks": ep, "experts": E,
                                 "params": kw, "moves": st[3], "bottleneck_latency_before": st[0],
                                 "bottleneck_latency_after": st[1],
                                 "imbalance_ratio_before": float(home_load.max()) / mean_load,
                                 "imbalance_ratio_after": float(st[2]) / mean_load}

        # The same step under a plan that was NOT built with hindsight: the lookahead predictor (this layer's cloned
        # gate, Sec. 4.2) runs on drifted copies of the tokens that stand in for the previous layer's hidden states,
        # its per-expert counts of the batch's eight token chunks (one chunk per virtual source rank, the all-gather
        # of Sec. 4.2) go to the device planner (Algorithm 1), and the true router's pairs are permuted under that
        # plan.  Set-up is untimed (the paper hides predictor and planner under the dispatch); what is timed is the
        # main track, so the cost of a predicted plan shows as rows per step and step time.  Not part of `value`.
        if 2 <= ep <= 16 and cfg.E_loc * ep == E and cfg.n_rep and T % ep == 0:
            alpha = 0.5
            kw = dict(max_replicas=cfg.n_rep, budget=3, k_max=16, n0=64, g_num=1, g_den=4)
            chunk = T // ep
            pl_plans, pl_tables, pl_rows, ir_pred, ir_hind = [], [], [], [], []
            cnt = torch.empty((ep, E), dtype=torch.int32, device=dev)
            for b in range(nb):
                d_hp = dev_bf16(wl.drifted_activations(cfg, xs[b], alpha, b))
                for r in range(ep):
                    sl = slice(r * chunk, (r + 1) * chunk)
                    # chunk r uses the bias rows of its own tokens
                    assert d_bias[b].shape[0] == 1 or (r * chunk) % tpg == 0
                    g0 = min((r * chunk) // tpg, d_bias[b].shape[0] - 1)
                    probe.predict_topk(d_hp[sl], g_route, d_bias[b][g0:], tpg, k, True,
                                       out=dict(idx=p_out_pred["idx"][sl], w=p_out_pred["w"][sl], counts=cnt[r]),
                                       workspace=ws_route)
                pg = probe.plan_greedy(cnt, cfg.E_loc, rank=0, **kw)
                se = pg["slot_expert"].cpu().numpy()
                pl_plans.append(pg["plan"])
                need2 = sorted({int(e) for e in se if e >= 0} - set(dev_w))
                for e, w in zip(need2, wl.expert_weights_many(cfg, need2, threads=threads)):
                    dev_w[e] = (dev_bf16(w[0]), dev_bf16(w[1]))
                pick = [int(e) if e >= 0 else 0 for e in se]          # an unused replica slot gets no rows
                pl_tables.append(probe.WeightTable([dev_w[e][0] for e in pick], [dev_w[e][1] for e in pick]))
                del d_hp
            saved = (d_plans, tables)
            d_plans, tables = pl_plans, pl_tables
            S_pl = cfg.E_loc + cfg.n_rep
            assert S_pl == S
            for b in range(nb):
                step(b)
                pl_rows.append(int(perm_out["n_local"].item()))
            torch.cuda.synchronize()
            ev2 = [[torch.cuda.Event(enable_timing=True) for _ in range(6)] for _ in range(args.steps)]
            t_start = time.perf_counter()
            for i in range(args.steps):
                step(i % nb, ev2[i])
            torch.cuda.synchronize()
            el2 = time.perf_counter() - t_start
            d_plans, tables = saved
            st2 = {n: float(np.mean([ev2[i][j].elapsed_time(ev2[i][j + 1]) for i in range(args.steps)]))
                   for j, n in enumerate(names)}
            rows2 = float(np.mean([pl_rows[i % nb] for i in range(args.steps)]))
            result["predicted_plan"] = {
                "what": "plan = probe_plan_greedy on probe_predict_topk counts of h_prev = drifted tokens (alpha %.1f), "
                        "8 token chunks as source ranks; same step, same batches" % alpha,
                "ms_per_step": el2 * 1e3 / args.steps, "tokens_per_s": T * args.steps / el2, "stage_ms": st2,
                "rows_per_step_mean": rows2, "rows_per_step_mean_hindsight_plan": nl_mean,
                "ffn_tflops": 6.0 * rows2 * H * F / (st2["ffn"] * 1e-3) / 1e12, "planner_params": kw}

        # the group-limited gate (sigmoid scores, E / 32 groups of 32 experts, half of them allowed) on the same
        # inputs, timed on its own next to the plain router; not part of `value`
        if E % 32 == 0 and E >= 64:
            ng = E // 32
            gkw = dict(scoring="sigmoid", n_group=ng, topk_group=max(ng // 2, 1), group_top=2, k=k, renormalize=True,
                       routed_scale=2.5)
            d_sb = torch.zeros((E,), dtype=torch.float32, device=dev)
            times = {}
            for name, fn in (("route_topk", lambda: probe.route_topk(d_xs[0], d_wg, d_bias[0], tpg, k, True, workspace=ws_route)),
                             ("route_grouped", lambda: probe.route_grouped(d_xs[0], d_wg, d_bias[0], tpg, d_sb, workspace=ws_route, **gkw))):
                for _ in range(3):
                    fn()
                torch.cuda.synchronize()
                e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                e0.record()
                for _ in range(20):
                    fn()
                e1.record()
                torch.cuda.synchronize()
                times[name] = e0.elapsed_time(e1) * 1e3 / 20
            result["grouped_gate"] = {"us_per_call": times["route_grouped"], "plain_router_us_per_call": times["route_topk"],
                                      "n_group": ng, "topk_group": gkw["topk_group"], "scoring": "sigmoid"}

    if args.calibrate_copy:
        src = torch.ones((1 << 28,), dtype=torch.float32, device=dev)      # 1 GiB
        dst = torch.empty_like(src)
        for _ in range(3):
            torch.mul(src, 1.0, out=dst)
        torch.cuda.synchronize()
        del src, dst

    if not args.no_cpu_baseline and not args.main_only:
        result["cpu_baseline"] = cpu_baseline(cfg, xs[0], wg, biases[0], tpg, plans[0], host_w, slot_experts[0],
                                              args.cpu_sample_tokens)
    print(json.dumps(result), flush=True)


def measure_peaks(torch, dev):
    import ctypes as C
    peaks = C.CDLL(os.path.join(ROOT, "paper_2602_00509_amd", "libprobe_peaks.so"))   # bench-only aid, not libprobe
    peaks.peaks_mfma_flops_per_launch.restype = C.c_double
    peaks.peaks_mfma_flops_per_launch.argtypes = [C.c_int, C.c_int]
    peaks.peaks_mfma.argtypes = [C.c_void_p, C.c_int, C.c_int, C.c_int, C.c_void_p]

    def timed(fn, reps):
        fn()
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(reps):
            fn()
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) * 1e-3 / reps
    wgs, iters = 256, 20000
    out = torch.empty((wgs * 512,), dtype=torch.float32, device=dev)
    res = {}
    for name, rnd in (("mfma_only_zero_operands_tflops", False), ("mfma_only_random_operands_tflops", True)):
        def run():
            rc = peaks.peaks_mfma(C.c_void_p(out.data_ptr()), wgs, iters, 1 if rnd else 0,
                                  C.c_void_p(torch.cuda.current_stream().cuda_stream))
            assert rc == 0, rc
        t = timed(run, 3)
        res[name] = float(peaks.peaks_mfma_flops_per_launch(wgs, iters)) / t / 1e12
    src = torch.empty((1 << 28,), dtype=torch.float32, device=dev)          # 1 GiB read + 1 GiB write
    dst = torch.empty_like(src)
    src.fill_(1.0)
    t = timed(lambda: dst.copy_(src), 5)
    res["copy_read_plus_write_gbps"] = 2 * src.numel() * 4 / t / 1e9
    del src, dst, out
    # context only: the vendor GEMM library (through torch.matmul) on one plain bf16 GEMM with the FFN's
    # first-GEMM shape and N(0,1) / N(0,0.02) operands; none of the library's code is on the product path
    M, N, K = 16384, 4096, 7168
    a = torch.empty((M, K), device=dev, dtype=torch.float32).normal_(0.0, 1.0).to(torch.bfloat16)
    b = torch.empty((N, K), device=dev, dtype=torch.float32).normal_(0.0, 0.02).to(torch.bfloat16)
    c = torch.empty((M, N), device=dev, dtype=torch.bfloat16)
    t = timed(lambda: torch.matmul(a, b.t(), out=c), 10)
    res["vendor_gemm_16384x4096x7168_tflops"] = 2.0 * M * N * K / t / 1e12
    del a, b, c
    return res


def cpu_baseline(cfg, x, wg, bias, tpg, plan, host_w, slot_expert, sample_tokens):
    """The CPU oracle, as it stands, on batch 0, stage by stage (route, permute, FFN, combine).

    The whole batch when the FFN of its local rows fits the time budget (it does for the default workload);
    otherwise the FFN is timed on the leading rows of the row space until the budget is spent and its time is
    scaled to all rows, which the `sample` string then says."""
    import oracle
    oracle.build()
    budget_s = 40.0
    T = min(sample_tokens or cfg.T, cfg.T)
    xs = np.ascontiguousarray(x[:T])
    w13 = [host_w[int(e)][0] for e in slot_expert]
    w2 = [host_w[int(e)][1] for e in slot_expert]
    clock = time.perf_counter
    t0 = clock()
    r = oracle.route_topk(xs, wg, bias, tpg, cfg.k, True)
    t1 = clock()
    p = oracle.permute(r["idx"], plan["rep_off"], plan["rep_slot"], plan["rep_weight"], plan["num_slots"], xs)
    t2 = clock()
    nl = p["n_local"]
    H = xs.shape[1]
    y = np.zeros((max(nl, 1), H), np.float64)
    done, chunk, t_ffn = 0, 256, 0.0
    while done < nl and t_ffn < budget_s:
        hi = min(nl, done + chunk)
        ta = clock()
        y[done:hi] = oracle.grouped_ffn(p["xp"], p["slot_offsets"], w13, w2, rows=np.arange(done, hi, dtype=np.int32))
        t_ffn += clock() - ta
        done = hi
        chunk = min(chunk * 2, 4096)
    t3 = clock()
    oracle.combine(y, p["pair_row"], r["w"])
    t4 = clock()
    ffn_full = t_ffn * (nl / done) if done else 0.0
    stage_s = {"route": t1 - t0, "permute": t2 - t1, "ffn": ffn_full, "combine": t4 - t3}
    total = sum(stage_s.values())
    what = ("all %d tokens of batch 0, stage by stage: route, permute, FFN of the %d local rows, combine" % (T, nl)
            if done == nl else
            "all %d tokens of batch 0 for route, permute and combine; FFN timed on the first %d of %d local rows "
            "(%.1f s) and scaled to all of them" % (T, done, nl, t_ffn))
    return {"value": T / total, "unit": "tokens/s", "cores": oracle.num_threads(), "kind": "oracle",
            "sample": what + "; %.1f s of CPU work" % (t4 - t0), "stage_s": stage_s}


if __name__ == "__main__":
    main()

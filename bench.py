#!/usr/bin/env python3
"""Benchmark of the replay-guided MoE expert-layer path on one MI355X.

A step = one pass of the whole hot path over one training batch of a workload: histogram of every
micro-batch -> plan (host) -> per micro-batch: permute, expert FFN forward, combine, combine
backward (by default folded into the expert backward: --backward), expert FFN backward, gather
backward -> weight gradients of the batch.  Inputs are seeded synthetic and resident in HBM before
the timed region.  The default workload is the largest one that fits the GPU (the Qwen3-235B-A22B-
shaped stress layer: 32 micro-batches x 16384 tokens, E=128, top-8, h=4096, h'=1536, simulated
EP=16, r=2); the Qwen3-30B-A3B-shaped layer is then timed as well and reported under "config2".

Prints ONE JSON line: metric = expert-layer fwd+bwd TFLOP/s (18*h*h'*N flops per micro-batch over
the whole step time), plus `roofline` for the dominant kernel (HIP events recorded by the library
around each launch, live in the timed region) and `cpu_baseline` (the CPU oracle timed on a bounded
sample of the same workload on this machine's host cores).
"""
import argparse
import concurrent.futures
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0     # MI355X dense bf16 MFMA
PEAK_HBM_GBS = 8000.0

GEMM_FLOP_FACTOR = {"fwd_gate_up": 4, "fwd_down": 2, "bwd_act": 2, "bwd_dx": 4, "wgrad_down": 2,
                    "wgrad_gate_up": 4}          # x h*h'*N per launch (2hh' per row per GEMM, Eq. 4)
TABLES = ("inst_ptr", "inst_rows", "inst_group", "group_offset", "group_expert", "group_dw_slot")


def log(*a):
    print("[bench]", *a, file=sys.stderr, flush=True)


def run_config(args, config_index, steps, warmup, extras_level, cpu_seconds):
    """Time `steps` steps of workload `config_index`; extras_level 0: nothing else, 1: the bandwidth kernels'
    figures, 2: also straggler rank, replica buffer, communication model.  Returns the result dict."""
    import numpy as np
    import torch
    import workloads as wl
    import paper_2605_08639_amd as rl

    dev = "cuda"
    cfg = wl.CONFIGS[config_index]
    E, k, h, hff, T, n_mb, EP, r, G, N = cfg.E, cfg.k, cfg.h, cfg.hff, cfg.T, cfg.n_mb, cfg.EP, cfg.r, cfg.G, cfg.N
    n_slots = E + EP * r

    # ---------------- inputs, resident in HBM
    t0 = time.time()
    routed = [wl.make_routing(cfg, mb) for mb in range(n_mb)]
    ids_h = np.stack([x[0] for x in routed])
    gates_h = np.stack([x[1] for x in routed])
    ids_all = torch.from_numpy(ids_h).to(dev)
    gates_all = torch.from_numpy(gates_h).to(dev)
    tok = [wl.make_tokens_device(cfg, mb, dev) for mb in range(n_mb)]
    Wg, Wu, Wd = wl.make_weights(cfg, dev)
    log(f"inputs for {cfg.name} drawn in {time.time() - t0:.1f}s")

    # ---------------- buffers (allocated once; the library allocates nothing)
    bf = lambda *s: torch.empty(s, dtype=torch.bfloat16, device=dev)
    i32 = lambda *s: torch.empty(s, dtype=torch.int32, device=dev)
    counts_d = i32(n_mb, E)
    err = rl.new_err_flag(dev)
    row_of, src_of = i32(N), i32(N)
    batched = args.wgrad == "batched"
    assert not batched or n_mb <= rl.MAX_WGRAD_MB
    n_keep = n_mb if batched else 1          # batched weight gradients keep every micro-batch's rows resident
    fused_gather = batched and not args.gathered_copy
    gate_fused = fused_gather and (args.backward == "gate-fused" or (args.backward == "auto" and hff < 4096))
    Xrows_k = [bf(N, h) for _ in range(1 if fused_gather else n_keep)]
    row_tok_k = [i32(N) for _ in range(n_keep)] if fused_gather else []
    dYrows_k = [] if gate_fused else [bf(N, h) for _ in range(n_keep)]   # gate-fused: the upstream rows are never materialised
    row_gate = torch.empty(N, dtype=torch.float32, device=dev)
    dgate_scratch = torch.empty(max(rl.workspace_bytes(rl.WS_DGATE, N, k, E, G, h, hff), 1), dtype=torch.uint8, device=dev)
    A_k = [bf(N, hff) for _ in range(n_keep)]            # gate-fused: holds gate * A (see layer())
    Ag_k = A_k if gate_fused else []
    Yrows, dXrows = bf(N, h), bf(N, h)
    Gt, U = bf(N, hff), bf(N, hff)
    Out, dX = bf(T, h), bf(T, h)
    dgate = torch.empty((T, k), dtype=torch.float32, device=dev)
    dWg = torch.empty((n_slots, hff, h), dtype=torch.float32, device=dev)
    dWu = torch.empty_like(dWg)
    dWd = torch.empty((n_slots, h, hff), dtype=torch.float32, device=dev)
    ws_perm = torch.empty(rl.workspace_bytes(rl.WS_PERMUTE, T, k, E, G, h, hff), dtype=torch.uint8, device=dev)
    ws_ffn_k = [torch.empty(rl.workspace_bytes(rl.WS_FFN_BWD, T, k, E, G, h, hff), dtype=torch.uint8, device=dev)
                for _ in range(n_keep)]
    ws_wgrad = torch.empty(rl.workspace_bytes(rl.WS_WGRAD_BATCHED, T, k, E, G, h, hff), dtype=torch.uint8, device=dev)
    Xrows, A, ws_ffn = Xrows_k[0], A_k[0], ws_ffn_k[0]
    transposed = args.weights != "plain"
    fwd_t, bwd_t = args.weights == "fwd-transposed", args.weights == "bwd-transposed"
    WgT = torch.empty((E, h, hff), dtype=torch.bfloat16, device=dev) if transposed else None
    WuT = torch.empty_like(WgT) if transposed else None
    WdT = torch.empty((E, hff, h), dtype=torch.bfloat16, device=dev) if transposed else None

    def upload(plan):
        return {key: torch.from_numpy(plan[key]).to(dev, non_blocking=True) for key in TABLES}

    def layer(mb, tabs, first):
        X, dOut = tok[mb]
        i = mb if batched else 0
        dYr, Ar, ws = (None if gate_fused else dYrows_k[i]), A_k[i], ws_ffn_k[i]
        fw = (WgT, WuT, WdT) if fwd_t else (Wg, Wu, Wd)
        fwd_flags = rl.FWD_TRANSPOSED_WEIGHTS if fwd_t else 0
        if fused_gather:                        # the GEMMs fetch token rows through row_tok: no gathered copy
            Xr = None
            rl.relibra_permute(ids_all[mb], tabs["inst_ptr"][mb], tabs["inst_rows"][mb], tabs["inst_group"][mb],
                               tabs["group_offset"][mb], None, E, tabs["group_expert"].shape[1], row_of=row_of, src_of=src_of,
                               workspace=ws_perm, err_flag=err)
            rl.relibra_row_tokens(src_of, k, T, row_tok=row_tok_k[i], err_flag=err)
            if gate_fused:
                rl.relibra_row_gates(src_of, gates_all[mb], row_gate=row_gate, err_flag=err)
                # gated in place: A = gate * A, the rows come out gate-scaled and the combine below is a plain sum
                rl.relibra_moe_ffn_fwd_gated(X, row_tok_k[i], row_gate, tabs["group_offset"][mb], tabs["group_expert"][mb], *fw,
                                             Gt=Gt, U=U, A=Ag_k[i], Ag=Ag_k[i], Yrows=Yrows, workspace=ws, err_flag=err, flags=fwd_flags)
            else:
                rl.relibra_moe_ffn_fwd_gather(X, row_tok_k[i], tabs["group_offset"][mb], tabs["group_expert"][mb], *fw,
                                              Gt=Gt, U=U, A=Ar, Yrows=Yrows, workspace=ws, err_flag=err, flags=fwd_flags)
        else:
            Xr = Xrows_k[i]
            rl.relibra_permute(ids_all[mb], tabs["inst_ptr"][mb], tabs["inst_rows"][mb], tabs["inst_group"][mb],
                               tabs["group_offset"][mb], X, E, tabs["group_expert"].shape[1], row_of=row_of, src_of=src_of,
                               Xrows=Xr, workspace=ws_perm, err_flag=err)
            rl.relibra_moe_ffn_fwd(Xr, tabs["group_offset"][mb], tabs["group_expert"][mb], *fw,
                                   Gt=Gt, U=U, A=Ar, Yrows=Yrows, workspace=ws, err_flag=err, flags=fwd_flags)
        if gate_fused:
            rl.relibra_unpermute_combine(rl.COMBINE_SUM, Yrows, row_of, T, k, out_tok=Out, err_flag=err)
        else:
            rl.relibra_unpermute_combine(rl.COMBINE_FWD, Yrows, row_of, T, k, gates=gates_all[mb], out_tok=Out, err_flag=err)
        bw = (WgT, WuT, WdT) if bwd_t else (Wg, Wu, Wd)
        if gate_fused:
            rl.relibra_moe_ffn_bwd_gated(dOut, row_tok_k[i], row_gate, Gt, U, tabs["group_offset"][mb], tabs["group_expert"][mb],
                                         tabs["group_dw_slot"][mb], *bw, src_of=src_of, E=E,
                                         flags=rl.BWD_TRANSPOSED_WEIGHTS if bwd_t else 0, dXrows=dXrows, dgate=dgate,
                                         workspace=ws, dgate_scratch=dgate_scratch, err_flag=err)
        else:
            rl.relibra_unpermute_combine(rl.COMBINE_BWD, Yrows, row_of, T, k, gates=gates_all[mb], tok=dOut,
                                         out_rows=dYr, dgate=dgate, err_flag=err)
            flags = rl.BWD_DEFER_WGRAD if batched else (0 if first else rl.BWD_ACCUMULATE)
            rl.relibra_moe_ffn_bwd(dYr, Xr, Gt, U, Ar, tabs["group_offset"][mb], tabs["group_expert"][mb],
                                   tabs["group_dw_slot"][mb], *bw, dWg, dWu, dWd, E=E,
                                   flags=flags | (rl.BWD_TRANSPOSED_WEIGHTS if bwd_t else 0), dXrows=dXrows,
                                   workspace=ws, err_flag=err)
        rl.relibra_unpermute_combine(rl.COMBINE_SUM, dXrows, row_of, T, k, out_tok=dX, err_flag=err)

    def weight_gradients(tabs):
        mbs = [dict(bwd_workspace=ws_ffn_k[mb],
                    inst_ptr=tabs["inst_ptr"][mb], inst_group=tabs["inst_group"][mb], group_offset=tabs["group_offset"][mb],
                    **(dict(dOut=tok[mb][1], A=Ag_k[mb]) if gate_fused else dict(dYrows=dYrows_k[mb], A=A_k[mb])),
                    **(dict(X=tok[mb][0], row_tok=row_tok_k[mb]) if fused_gather else dict(Xrows=Xrows_k[mb])))
               for mb in range(n_mb)]
        rl.relibra_moe_ffn_wgrad_batched(mbs, E, dWg, dWu, dWd, workspace=ws_wgrad, err_flag=err,
                                         tile=None if args.wgrad_tile == "auto" else args.wgrad_tile)

    plan_ms = []

    # The plan of a batch needs only its replayed routing, which is known before the batch trains
    # (Section 3: the control plane solves while earlier work still runs, off the critical path).
    # --plan ahead: the histogram of the NEXT batch is launched at the start of a step, copied to pinned
    # host memory asynchronously, and a host thread plans it while this step's kernels run; every step
    # still launches one histogram, makes one device->host crossing and computes one plan.
    # --plan inline: histogram, crossing and plan at the head of the step that uses them.
    counts_pin = torch.empty((n_mb, E), dtype=torch.int32, pin_memory=True)
    ahead = {"thread": None, "plan": None}
    planner_pool = concurrent.futures.ThreadPoolExecutor(max_workers=1)        # one resident host thread

    def plan_from(counts_h):
        tp = time.perf_counter()
        plan = rl.relibra_plan(counts_h, k, EP, cfg.rpn, r)
        plan_ms.append((time.perf_counter() - tp) * 1e3)
        return plan

    def launch_planning():
        rl.relibra_route_hist(ids_all, E, counts=counts_d, err_flag=err)
        counts_pin.copy_(counts_d, non_blocking=True)           # the path's one device->host crossing
        ev = torch.cuda.Event()
        ev.record()

        def work():
            ev.synchronize()
            ahead["plan"] = plan_from(counts_pin.numpy())
        ahead["thread"] = planner_pool.submit(work)

    def step():
        if args.plan == "ahead":
            if ahead["thread"] is None:                         # very first step: nothing was prepared
                launch_planning()
            ahead["thread"].result()
            plan = ahead["plan"]
            launch_planning()                                   # for the step after this one
        else:
            rl.relibra_route_hist(ids_all, E, counts=counts_d, err_flag=err)
            counts_h = counts_d.cpu().numpy()                   # the path's one device->host crossing
        if transposed:          # this step's parameters in the transposed layout, once per step
            rl.relibra_transpose_experts(Wg, WgT)
            rl.relibra_transpose_experts(Wu, WuT)
            rl.relibra_transpose_experts(Wd, WdT)
        if args.plan != "ahead":
            plan = plan_from(counts_h)
        tabs = upload(plan)
        for mb in range(n_mb):
            layer(mb, tabs, first=(mb == 0))
        if batched:
            weight_gradients(tabs)
        return plan, tabs

    # ---------------- warmup, then the timed region
    for _ in range(max(warmup, 0)):
        plan, tabs = step()
    torch.cuda.synchronize()
    assert err.item() == 0, f"device error flag {err.item()} during warmup"
    plan_ms.clear()
    rl.prof_start(level=1, max_records=steps * n_mb * 6 + 64)
    torch.cuda.synchronize()
    t_begin = time.perf_counter()
    for _ in range(steps):
        plan, tabs = step()
    if ahead["thread"] is not None:
        ahead["thread"].result()        # the plan prepared during the last step belongs to the timed work
    torch.cuda.synchronize()
    t_end = time.perf_counter()
    prof = rl.prof_stop()
    assert err.item() == 0, f"device error flag {err.item()}"
    ms_per_step = (t_end - t_begin) * 1e3 / steps
    flops_step = cfg.flops_per_mb * n_mb
    value = flops_step / (ms_per_step * 1e-3) / 1e12

    # Algorithmic HBM bytes per launch: every tensor read or written once,
    # a group's weights once per live group, weight gradients written per live group and, when
    # accumulating, the home slots read first.  Averaged over the micro-batches of the step.
    def alg_bytes(name):
        w1 = 2.0 * h * hff                       # one bf16 weight matrix
        act_h, act_ff = 2.0 * h * N, 2.0 * hff * N
        act_x = 2.0 * h * T + 4.0 * N if fused_gather else act_h      # the layer's input rows: tokens + row table, or the gathered copy
        act_dy = 2.0 * h * T + 4.0 * N if gate_fused else act_h       # the upstream rows: dOut tokens + row table, or gate * dOut rows
        gate_rows = 4.0 * N if gate_fused else 0.0                    # the per-row gates
        if batched and name.startswith("wgrad"):   # one launch per batch: every micro-batch's rows read once, dW written once
            return n_mb * (act_dy + act_ff) + 2 * w1 * E if name == "wgrad_down" else n_mb * (2 * act_ff + act_x) + 4 * w1 * E
        tot = 0.0
        for mb in range(n_mb):
            rows_g = np.diff(plan["group_offset"][mb])
            live = int((rows_g > 0).sum())
            home_live = int(((rows_g > 0) & (plan["group_dw_slot"][mb] < E)).sum())
            acc_mode = mb > 0
            tot += {
                "fwd_gate_up": act_x + 2 * w1 * live + 3 * act_ff + gate_rows,
                "fwd_down": act_ff + w1 * live + act_h,
                "bwd_act": act_dy + w1 * live + 2 * act_ff + 2 * act_ff + 2 * gate_rows,      # + the row sums of dgate
                "bwd_dx": 2 * act_ff + 2 * w1 * live + act_h,
                "wgrad_down": act_h + act_ff + 2 * w1 * live + (2 * w1 * home_live if acc_mode else 0.0),
                "wgrad_gate_up": 2 * act_ff + act_x + 4 * w1 * live + (4 * w1 * home_live if acc_mode else 0.0),
            }[name]
        return tot / n_mb

    traffic_file = os.path.join(ROOT, "profiles", f"bench_config{config_index + 1}_hbm_traffic.json")
    measured = json.load(open(traffic_file))["kernels"] if os.path.exists(traffic_file) else {}
    util_file = os.path.join(ROOT, "profiles", f"bench_config{config_index + 1}_mfma_util.json")
    util = json.load(open(util_file))["kernels"] if os.path.exists(util_file) else {}

    kernels = {}
    for name, (ms, n) in prof.items():
        fl = GEMM_FLOP_FACTOR[name] * h * hff * N * (n_mb if batched and name.startswith("wgrad") else 1)
        by = alg_bytes(name)
        t_s = ms / n * 1e-3
        kernels[name] = {"avg_ms": ms / n, "launches": n, "tflops": fl / t_s / 1e12, "alg_GBps": by / t_s / 1e9,
                         "bound": "hbm" if by / (PEAK_HBM_GBS * 1e9) > fl / (PEAK_BF16_TFLOPS * 1e12) else "mfma",
                         "flops_per_launch": fl, "alg_bytes_per_launch": by}
    gemm_ms_step = sum(ms for ms, _ in prof.values()) / steps
    dominant = max(prof, key=lambda nm: prof[nm][0])
    kd = kernels[dominant]
    tr = measured.get(dominant)
    if kd["bound"] == "hbm":
        roofline = {"bound": "hbm", "kernel": dominant, "achieved": kd["alg_GBps"], "peak": PEAK_HBM_GBS, "unit": "GB/s",
                    "frac": kd["alg_GBps"] / PEAK_HBM_GBS}
    else:
        roofline = {"bound": "mfma", "kernel": dominant, "achieved": kd["tflops"], "peak": PEAK_BF16_TFLOPS,
                    "unit": "TFLOP/s", "frac": kd["tflops"] / PEAK_BF16_TFLOPS}
    roofline.update({"traffic": (tr["read_bytes"] + tr["write_bytes"]) if tr else None, "avg_launch_ms": kd["avg_ms"],
                     "flops_per_launch": kd["flops_per_launch"], "alg_bytes_per_launch": kd["alg_bytes_per_launch"],
                     "mfma_frac": kd["tflops"] / PEAK_BF16_TFLOPS,
                     # from a committed rocprofv3 counter run of this command (profiles/): the matrix pipes' busy share
                     # of the cycles the chip actually ran, and that clock (the published peak assumes 2.4 GHz)
                     "mfma_util_counter": util.get(dominant)})
    # mixed roofline of all six GEMM kernels: sum over kernels of max(flops/peak, bytes/bandwidth)
    floor_ms = sum(max(v["flops_per_launch"] / (PEAK_BF16_TFLOPS * 1e12), v["alg_bytes_per_launch"] / (PEAK_HBM_GBS * 1e9))
                   * v["launches"] / steps for v in kernels.values()) * 1e3          # per step
    gemm_tflops = flops_step / (gemm_ms_step * 1e-3) / 1e12
    log(f"{cfg.name}: step {ms_per_step:.2f} ms  value {value:.1f} TFLOP/s  grouped GEMMs alone {gemm_tflops:.1f} TFLOP/s")

    extras = {}
    if extras_level >= 1:
        # ---- every kernel of a step once more, untimed, then the unfused bandwidth kernels the default step does
        # not launch (row gather of the permutation, gated combine, combine backward), once per micro-batch
        rl.prof_start(level=2, max_records=n_mb * 48 + 64)
        step()
        if ahead["thread"] is not None:
            ahead["thread"].result()
        dY_x = dYrows_k[0] if dYrows_k else bf(N, h)
        for mb in range(n_mb):
            X, dOut = tok[mb]
            rl.relibra_permute(ids_all[mb], tabs["inst_ptr"][mb], tabs["inst_rows"][mb], tabs["inst_group"][mb],
                               tabs["group_offset"][mb], X, E, G, row_of=row_of, src_of=src_of, Xrows=Xrows,
                               workspace=ws_perm, err_flag=err)
            rl.relibra_unpermute_combine(rl.COMBINE_FWD, Yrows, row_of, T, k, gates=gates_all[mb], out_tok=Out, err_flag=err)
            rl.relibra_unpermute_combine(rl.COMBINE_BWD, Yrows, row_of, T, k, gates=gates_all[mb], tok=dOut,
                                         out_rows=dY_x, dgate=dgate, err_flag=err)
        torch.cuda.synchronize()
        p2 = rl.prof_stop()
        del dY_x
        n_units = (N + 127) // 128
        parts = 4 * ((hff + 255) // 256)
        small_bytes = {        # algorithmic bytes per launch of the bandwidth-bound and index kernels
            "hist": 4.0 * N * n_mb + 4.0 * E * n_mb,
            "gather": 2.0 * h * N + 2.0 * h * T + 4.0 * N,
            "combine_fwd": 2.0 * h * N + 2.0 * h * T + 8.0 * N,
            "combine_bwd": 2.0 * h * T + 4.0 * h * N + 12.0 * N,
            "combine_sum": 2.0 * h * N + 2.0 * h * T + 4.0 * N,
            "perm_count": 8.0 * N + 4.0 * n_units * E,
            "perm_scan": 8.0 * n_units * E,
            "perm_rank": 12.0 * N + 4.0 * n_units * E,
            "row_tokens": 8.0 * N,
            "row_gates": 12.0 * N,
            "dgate_reduce": 4.0 * parts * N + 8.0 * N,
            "transpose": 4.0 * h * hff * E,
        }
        hbm = {}
        for name, b in small_bytes.items():
            if name in p2:
                avg = p2[name][0] / p2[name][1]
                hbm[name] = {"avg_ms": avg, "launches": p2[name][1], "alg_bytes_per_launch": b, "GBps": b / (avg * 1e-3) / 1e9,
                             "frac_of_8TBps": b / (avg * 1e-3) / 1e9 / PEAK_HBM_GBS}
        # the histogram at the size where it is bandwidth-bound: the replayed routing of every layer of a model is
        # known before the batch trains (Section 3), so one launch covers [layers * n_mb] micro-batches
        layers = max(1, min(64, (1 << 30) // max(ids_all.numel() * 4, 1)))
        ids_layers = ids_all.repeat(layers, 1, 1)
        counts_layers = i32(layers * n_mb, E)
        rl.relibra_route_hist(ids_layers, E, counts=counts_layers, err_flag=err)
        rl.prof_start(level=2, max_records=16)
        for _ in range(5):
            rl.relibra_route_hist(ids_layers, E, counts=counts_layers, err_flag=err)
        torch.cuda.synchronize()
        p3 = rl.prof_stop()
        assert torch.equal(counts_layers[:n_mb], counts_d) and torch.equal(counts_layers[-n_mb:], counts_d)
        b = 4.0 * N * n_mb * layers + 4.0 * E * n_mb * layers
        avg = p3["hist"][0] / p3["hist"][1]
        hbm["hist_all_layers"] = {"layers": layers, "avg_ms": avg, "launches": p3["hist"][1], "alg_bytes_per_launch": b,
                                  "GBps": b / (avg * 1e-3) / 1e9, "frac_of_8TBps": b / (avg * 1e-3) / 1e9 / PEAK_HBM_GBS}
        del ids_layers, counts_layers
        extras["hbm_kernels"] = hbm
        # what this machine's memory system sustains for plain streams (torch's own copy and fill kernels, calibration
        # only): a 1 GiB copy (read + write) and a 2 GiB fill (write only); the read-only stream is hist_all_layers
        src_c = torch.empty(1 << 30, dtype=torch.uint8, device=dev).fill_(1)
        dst_c = torch.empty(2 << 30, dtype=torch.uint8, device=dev)
        best = {"copy": 1e9, "fill": 1e9}
        for _ in range(5):
            e0, e1, e2 = (torch.cuda.Event(enable_timing=True) for _ in range(3))
            e0.record()
            dst_c[:1 << 30].copy_(src_c)
            e1.record()
            dst_c.zero_()
            e2.record()
            e2.synchronize()
            best["copy"], best["fill"] = min(best["copy"], e0.elapsed_time(e1)), min(best["fill"], e1.elapsed_time(e2))
        extras["measured_stream_GBps"] = {"copy_read_plus_write": 2.0 * (1 << 30) / (best["copy"] * 1e-3) / 1e9,
                                          "fill_write_only": 2.0 * (1 << 30) / (best["fill"] * 1e-3) / 1e9,
                                          "read_only": hbm["hist_all_layers"]["GBps"]}
        del src_c, dst_c
        extras["index_kernels_ms"] = {nm: p2[nm][0] / p2[nm][1] for nm in ("sched", "wgrad_order", "replica_sum") if nm in p2}
        assert err.item() == 0

    if extras_level >= 2:
        # ---- straggler rank: FFN fwd+bwd on the most loaded rank's groups, before / after the plan
        M = cfg.M
        un = {  # unplanned layout: expert e is group e on rank e // M, no replicas
            "inst_ptr": np.tile(np.arange(E + 1, dtype=np.int32), (n_mb, 1)),
            "inst_rows": counts_d.cpu().numpy().astype(np.int32),
            "inst_group": np.tile(np.arange(E, dtype=np.int32), (n_mb, 1)),
            "group_expert": np.tile(np.arange(E, dtype=np.int32), (n_mb, 1)),
            "group_dw_slot": np.tile(np.arange(E, dtype=np.int32), (n_mb, 1)),
        }
        un["group_offset"] = np.concatenate([np.zeros((n_mb, 1), np.int32), np.cumsum(un["inst_rows"], 1, dtype=np.int32)], 1)
        un_d = upload(un)

        def straggler_ms(tabs_d, host, per_rank, mb):
            go = host["group_offset"][mb]
            loads = [(go[(g + 1) * per_rank] - go[g * per_rank]) for g in range(EP)]
            g_star = int(np.argmax(loads))
            X, dOut = tok[mb]
            rl.relibra_permute(ids_all[mb], tabs_d["inst_ptr"][mb], tabs_d["inst_rows"][mb], tabs_d["inst_group"][mb],
                               tabs_d["group_offset"][mb], X, E, tabs_d["group_expert"].shape[1], row_of=row_of,
                               src_of=src_of, Xrows=Xrows, workspace=ws_perm, err_flag=err)
            rng = (g_star * per_rank, (g_star + 1) * per_rank)
            times = []
            for it in range(3):
                e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                e0.record()
                rl.relibra_moe_ffn_fwd(Xrows, tabs_d["group_offset"][mb], tabs_d["group_expert"][mb], Wg, Wu, Wd,
                                       g_begin=rng[0], g_end=rng[1], Gt=Gt, U=U, A=A, Yrows=Yrows, workspace=ws_ffn, err_flag=err)
                rl.relibra_moe_ffn_bwd(Yrows, Xrows, Gt, U, A, tabs_d["group_offset"][mb], tabs_d["group_expert"][mb],
                                       tabs_d["group_dw_slot"][mb], Wg, Wu, Wd, dWg, dWu, dWd, g_begin=rng[0], g_end=rng[1],
                                       flags=rl.BWD_NO_REPLICA_SUM, dXrows=dXrows, workspace=ws_ffn, err_flag=err)
                e1.record()
                e1.synchronize()
                times.append(e0.elapsed_time(e1))
            return min(times), int(max(loads))

        sb, sa = [], []
        for mb in range(min(n_mb, 4)):
            sb.append(straggler_ms(un_d, un, M, mb))
            sa.append(straggler_ms(tabs, plan, M + r, mb))
        extras["straggler"] = {
            "micro_batches": len(sb),
            "ms_before": float(np.mean([x[0] for x in sb])), "ms_after": float(np.mean([x[0] for x in sa])),
            "rows_before": float(np.mean([x[1] for x in sb])), "rows_after": float(np.mean([x[1] for x in sa])),
            "balanced_rows": N / EP,
        }
        assert err.item() == 0

        # ---- layer-shared replica buffer (Section 5.1): the forward push of micro-batch 0's replicas and the
        # gradient pull-back, alone and on a second stream beside the FFN forward (the paper hides both behind
        # attention, which is outside this path; the expert forward stands in as the compute they compete with)
        if r > 0:
            rep0 = torch.from_numpy(np.ascontiguousarray(plan["replica_expert"][0].reshape(-1))).to(dev)
            live_slots = int((plan["replica_expert"][0] >= 0).sum())
            pad = lambda W: torch.cat([W, torch.empty((EP * r, *W.shape[1:]), dtype=W.dtype, device=dev)])
            Wb = [pad(W) for W in (Wg, Wu, Wd)]
            side = torch.cuda.Stream()
            ev = lambda: torch.cuda.Event(enable_timing=True)
            mb = 0

            def fwd():
                rl.relibra_moe_ffn_fwd(Xrows, tabs["group_offset"][mb], tabs["group_expert"][mb], Wg, Wu, Wd,
                                       Gt=Gt, U=U, A=A, Yrows=Yrows, workspace=ws_ffn, err_flag=err)

            def timed(side_fn, run_fwd):
                best = [1e9, 1e9]
                for _ in range(3):
                    torch.cuda.synchronize()
                    p0, p1, f0, f1 = ev(), ev(), ev(), ev()
                    if side_fn:
                        with torch.cuda.stream(side):
                            p0.record()
                            side_fn()
                            p1.record()
                    if run_fwd:
                        f0.record()
                        fwd()
                        f1.record()
                    torch.cuda.synchronize()
                    if side_fn:
                        best[0] = min(best[0], p0.elapsed_time(p1))
                    if run_fwd:
                        best[1] = min(best[1], f0.elapsed_time(f1))
                return best

            X0, _ = tok[mb]
            rl.relibra_permute(ids_all[mb], tabs["inst_ptr"][mb], tabs["inst_rows"][mb], tabs["inst_group"][mb],
                               tabs["group_offset"][mb], X0, E, G, row_of=row_of, src_of=src_of, Xrows=Xrows,
                               workspace=ws_perm, err_flag=err)
            fwd_alone = timed(None, True)[1]
            push_bytes = live_slots * 3 * 2.0 * h * hff * 2          # read + write of three bf16 blocks per slot
            pull_bytes = live_slots * 3 * 4.0 * h * hff * 3          # fp32: read slot, read home, write home
            rows, rows_pull = [], []
            for n_wg in (8, 32, 128):
                push = lambda: rl.relibra_replica_push(*Wb, rep0, E, EP, r, n_workgroups=n_wg, err_flag=err)
                pull = lambda: rl.relibra_replica_pull(dWg, dWu, dWd, rep0, E, EP, r, n_workgroups=n_wg, err_flag=err)
                alone = timed(push, False)[0]
                both = timed(push, True)
                rows.append({"n_workgroups": n_wg, "push_ms_alone": alone, "push_GBps_alone": push_bytes / (alone * 1e-3) / 1e9,
                             "push_ms_beside_fwd": both[0], "fwd_ms_beside_push": both[1]})
                alone = timed(pull, False)[0]
                both = timed(pull, True)
                rows_pull.append({"n_workgroups": n_wg, "pull_ms_alone": alone, "pull_GBps_alone": pull_bytes / (alone * 1e-3) / 1e9,
                                  "pull_ms_beside_fwd": both[0], "fwd_ms_beside_pull": both[1]})
            extras["replica_push"] = {"live_slots": live_slots, "bytes": push_bytes, "fwd_ms_alone": fwd_alone, "runs": rows}
            extras["replica_pull"] = {"live_slots": live_slots, "bytes": pull_bytes, "fwd_ms_alone": fwd_alone, "runs": rows_pull}
            del Wb
            assert err.item() == 0

        # ---- communication-aware model (Section 4.1) and Algorithm 1 on this batch: per-source
        # histogram on the GPU, modelled T_MoE of the unplanned layout, of the plan's placement and of
        # the annealed placement.  Model constants are MI355X-flavoured assumptions, not measurements:
        # F = 0.5 PFLOP/s effective, intra-node 7 x 153.6 GB/s xGMI links, 50 GB/s (400 Gb/s) per NIC.
        if T % EP == 0:
            x_h = rl.relibra_route_hist_src(ids_all, E, EP, err_flag=err).sum(0).cpu().numpy().astype(np.int64)
            cm = rl.cost_model(EP, cfg.rpn, h, hff, 5e14, 7 * 153.6e9, 50e9)
            t_sa = time.perf_counter()
            sa_rank, sa_stats = rl.relibra_reorder_sa(x_h, cm, n_seeds=8, seed=0)
            t_sa = (time.perf_counter() - t_sa) * 1e3
            placed = plan["expert_to_slot"] // cfg.M
            ident = np.arange(E, dtype=np.int32) // cfg.M
            extras["comm_model"] = {
                "assumed": {"F": 5e14, "B_intra": 7 * 153.6e9, "B_inter": 50e9, "ranks_per_node": cfg.rpn},
                "T_unplanned_ms": rl.relibra_moe_time(x_h, ident, cm)["T"] * 1e3,
                "T_plan_placement_ms": rl.relibra_moe_time(x_h, placed, cm)["T"] * 1e3,
                "T_lpt_ms": sa_stats["T_start"] * 1e3, "T_annealed_ms": sa_stats["T"] * 1e3,
                "sa_iterations_per_seed": sa_stats["iterations"], "sa_seeds": 8, "sa_solve_ms": t_sa,
            }
            # source-aware token split of micro-batch 0 (Section 5.2, y_{j,e,g}) against the split in
            # token order that the plain permutation makes: modelled link loads and times (Eq. 1-6)
            x0 = rl.relibra_route_hist_src(ids_all[:1], E, EP, err_flag=err)[0].cpu().numpy().astype(np.int64)
            ptr0, rank0, rows0_ = plan["inst_ptr"][0], plan["inst_rank"][0], plan["inst_rows"][0]
            n_inst = int(ptr0[E])
            t_as = time.perf_counter()
            split = rl.relibra_assign_sources(x0, cfg.rpn, ptr0, rank0, rows0_)
            t_as = (time.perf_counter() - t_as) * 1e3
            y_order = np.zeros_like(split["inst_src_rows"])
            for e in range(E):
                i, room = int(ptr0[e]), int(rows0_[ptr0[e]])
                for j in range(EP):
                    n = int(x0[j, e])
                    while n:
                        while room == 0:
                            i += 1
                            room = int(rows0_[i])
                        m = min(n, room)
                        y_order[i, j] += m
                        n, room = n - m, room - m
            ms = {}
            for name, yy in (("token_order", y_order), ("source_aware", split["inst_src_rows"])):
                t = rl.relibra_moe_time_split(yy[:n_inst], rank0[:n_inst], cm, with_loads=True)
                ms[name] = {"T_comm_ms": t["T_comm"] * 1e3, "T_ms": t["T"] * 1e3,
                            "intra_node_tokens": int(t["loads"][1].sum()), "rdma_tokens": int(t["loads"][3].sum())}
            d_tabs = {key: torch.from_numpy(v).to(dev) for key, v in split.items()}
            perm_args = (ids_all[0], tabs["inst_ptr"][0], tabs["inst_group"][0], tabs["group_offset"][0], EP,
                         d_tabs["src_first"], d_tabs["inst_src_rows"], d_tabs["inst_src_base"], None, E, tabs["group_expert"].shape[1])
            ev = [torch.cuda.Event(enable_timing=True) for _ in range(3)]
            rl.relibra_permute_src(*perm_args, row_of=row_of, src_of=src_of, workspace=ws_perm, err_flag=err)
            ev[0].record()
            for _ in range(10):
                rl.relibra_permute_src(*perm_args, row_of=row_of, src_of=src_of, workspace=ws_perm, err_flag=err)
            ev[1].record()
            for _ in range(10):
                rl.relibra_permute(ids_all[0], tabs["inst_ptr"][0], tabs["inst_rows"][0], tabs["inst_group"][0],
                                   tabs["group_offset"][0], None, E, tabs["group_expert"].shape[1], row_of=row_of, src_of=src_of,
                                   workspace=ws_perm, err_flag=err)
            ev[2].record()
            torch.cuda.synchronize()
            # Algorithm 2 driven by T_MoE,g (Section 5.2 as printed) against the load-only plan the step uses:
            # modelled T_MoE per micro-batch, both with the source-aware split
            x_all = rl.relibra_route_hist_src(ids_all, E, EP, err_flag=err).cpu().numpy().astype(np.int64)
            t_tp = time.perf_counter()
            timed_plan = rl.relibra_plan_timed(x_all, k, cm, r, placed)
            t_tp = (time.perf_counter() - t_tp) * 1e3
            t_load_only = []
            for mb in range(n_mb):
                n_i = int(plan["inst_ptr"][mb][E])
                sp = rl.relibra_assign_sources(x_all[mb], cfg.rpn, plan["inst_ptr"][mb], plan["inst_rank"][mb], plan["inst_rows"][mb])
                t_load_only.append(rl.relibra_moe_time_split(sp["inst_src_rows"][:n_i], plan["inst_rank"][mb][:n_i], cm)["T"])
            extras["timed_plan"] = {"host_ms": t_tp, "T_no_replicas_ms": float(np.mean(timed_plan["t_before"]) * 1e3),
                                    "T_load_only_plan_ms": float(np.mean(t_load_only) * 1e3),
                                    "T_timed_plan_ms": float(np.mean(timed_plan["t_after"]) * 1e3),
                                    "max_load_load_only": int(plan["max_load_after"].max()),
                                    "max_load_timed": int(timed_plan["max_load_after"].max())}
            extras["source_aware_split"] = {"micro_batch": 0, "assign_host_ms": t_as, **ms,
                                            "permute_src_ms": ev[0].elapsed_time(ev[1]) / 10,
                                            "permute_ms": ev[1].elapsed_time(ev[2]) / 10}
            assert err.item() == 0

    # ---------------- the CPU oracle on a bounded sample of this workload, on this machine's host cores
    cpu_baseline = None
    if cpu_seconds > 0:
        cpu_baseline = oracle_leg(cfg, ids_h, gates_h, tok, (Wg, Wu, Wd), plan, cpu_seconds)

    planner_pool.shutdown()
    out = {
        "value": value, "ms_per_step": ms_per_step,
        "config": {"workload": f"{cfg.name}: E={E} top-{k} h={h} h'={hff} {n_mb}x{T} tokens, simulated EP={EP}, r={r}; "
                               "whole path per step (hist, plan on host, permute, FFN fwd, combine, combine bwd, FFN bwd, gather bwd); "
                               + ("combine backward folded into the expert backward (gate-fused); " if gate_fused else "")
                               + ("weight gradients once per batch over all resident micro-batches" if batched
                                  else "weight gradients accumulated micro-batch by micro-batch")
                               + ("; row gather fused into the GEMMs" if fused_gather else "")
                               + ("; histogram and host plan of the next batch overlapped with the step" if args.plan == "ahead"
                                  else "; histogram and host plan at the head of the step")
                               + {"fwd-transposed": "; forward GEMMs on transposed weight copies made once per step",
                                  "bwd-transposed": "; data gradients on transposed weight copies made once per step",
                                  "plain": ""}[args.weights],
                   "flops_per_step": flops_step},
        "roofline": roofline, "cpu_baseline": cpu_baseline,
        "gemm_kernels": kernels, "gemm_only_tflops": gemm_tflops,
        "gemm_mixed_roofline": {"floor_ms_per_step": floor_ms, "achieved_ms_per_step": gemm_ms_step,
                                "frac": floor_ms / gemm_ms_step}, "plan_host_ms": float(np.mean(plan_ms)),
        "skew_before": float(np.mean(plan["max_load_before"]) / (N / EP)),
        "skew_after": float(np.mean(plan["max_load_after"]) / (N / EP)),
    }
    out.update(extras)
    return out


def oracle_leg(cfg, ids_h, gates_h, tok, weights, plan, cpu_seconds):
    """The CPU oracle, as it stands, on this machine's host cores: the integer path (histogram, plan, permutation) on
    every micro-batch in full, and the floating-point expert FFN forward + backward on the straggler rank's share
    before (unplanned layout) and after the plan for micro-batch 0 and a mid-batch one, on the real token rows,
    upstream gradients and weights.  The FFN legs are bounded to about cpu_seconds in total: every leg takes the
    same fraction f of each of its groups' rows (their first rows), so the before/after ratio is that of the full
    shares, and the full-share time is the measured one divided by f."""
    import numpy as np
    import torch
    import oracle

    E, k, h, hff, T, n_mb, EP, r, N, M = cfg.E, cfg.k, cfg.h, cfg.hff, cfg.T, cfg.n_mb, cfg.EP, cfg.r, cfg.N, cfg.M
    threads = oracle.num_threads()
    affinity = len(os.sched_getaffinity(0))
    # ---- integer path, every micro-batch
    t = time.perf_counter()
    counts_o, _ = oracle.route_hist(ids_h, E)
    hist_ms = (time.perf_counter() - t) * 1e3
    t = time.perf_counter()
    po = oracle.plan(counts_o, EP, cfg.rpn, r)
    plan_ms = (time.perf_counter() - t) * 1e3
    t = time.perf_counter()
    perms = [oracle.permute(ids_h[mb], E, po["inst_ptr"][mb], po["inst_rows"][mb], po["inst_group"][mb], po["group_offset"][mb])
             for mb in range(n_mb)]
    permute_ms = (time.perf_counter() - t) * 1e3
    for key in ("group_offset", "group_expert", "inst_rows"):
        assert np.array_equal(po[key], plan[key]), key          # the timed GPU step ran under the plan the oracle makes

    # ---- floating point: straggler rank's share, before / after, two micro-batches
    def share(mb, planned):
        """(rows of the most loaded rank, list of (expert, assignment indices of the group's rows))"""
        if planned:
            go, ge, per_rank = po["group_offset"][mb], po["group_expert"][mb], M + r
            src_of = perms[mb][1]
            loads = [int(go[(g + 1) * per_rank] - go[g * per_rank]) for g in range(EP)]
            g_star = int(np.argmax(loads))
            groups = [(int(ge[g]), src_of[go[g]:go[g + 1]]) for g in range(g_star * per_rank, (g_star + 1) * per_rank)
                      if ge[g] >= 0 and go[g + 1] > go[g]]
        else:           # expert e on rank e // M, rows of an expert in ascending assignment order
            flat = ids_h[mb].reshape(-1)
            loads = [int(counts_o[mb][g * M:(g + 1) * M].sum()) for g in range(EP)]
            g_star = int(np.argmax(loads))
            groups = [(e, np.flatnonzero(flat == e).astype(np.int32)) for e in range(g_star * M, (g_star + 1) * M)
                      if counts_o[mb][e] > 0]
        return max(loads), groups

    def run(mb, groups, frac):
        X, dOut = (x.cpu() for x in tok[mb])
        experts = sorted(set(e for e, _ in groups))
        remap = {e: i for i, e in enumerate(experts)}
        idx = torch.tensor(experts, device=weights[0].device)
        w = [W[idx].cpu() for W in weights]
        taken = [(e, a[:max(1, int(round(len(a) * frac)))]) for e, a in groups]
        sub_go = np.concatenate([[0], np.cumsum([len(a) for _, a in taken])]).astype(np.int32)
        sub_ge = np.array([remap[e] for e, _ in taken], np.int32)
        asg = np.concatenate([a for _, a in taken]).astype(np.int64)
        Xs = X[torch.from_numpy(asg // k)]
        g = torch.from_numpy(gates_h[mb].reshape(-1)[asg])
        dYs = (g[:, None] * dOut[torch.from_numpy(asg // k)].float()).to(torch.bfloat16)     # the combine's backward, row by row
        t0 = time.perf_counter()
        oracle.ffn_fwd(Xs, sub_go, sub_ge, *w)
        oracle.ffn_bwd(Xs, dYs, sub_go, sub_ge, *w)
        return int(sub_go[-1]), time.perf_counter() - t0

    mbs = sorted(set([0, n_mb // 2]))
    legs = [(mb, planned, *share(mb, planned)) for mb in mbs for planned in (False, True)]
    # probe the oracle's rate on 64 rows, then size the fraction so that all legs together take about cpu_seconds
    probe_rows, probe_dt = run(legs[0][0], [(e, a[:16]) for e, a in legs[0][3][:4]], 1.0)
    rate = probe_rows / probe_dt
    total_rows = sum(l[2] for l in legs)
    frac = min(1.0, max(rate * cpu_seconds / total_rows, 64.0 * len(legs) / total_rows))
    log(f"oracle probe: {probe_rows} rows in {probe_dt:.2f}s; taking {frac:.4f} of each straggler share ({total_rows} rows in {len(legs)} legs)")
    res, rows_sum, dt_sum = [], 0, 0.0
    for mb, planned, share_rows, groups in legs:
        rows, dt = run(mb, groups, frac)
        rows_sum, dt_sum = rows_sum + rows, dt_sum + dt
        res.append({"micro_batch": mb, "plan": "after" if planned else "before", "share_rows": share_rows, "sample_rows": rows,
                    "sample_s": dt, "full_share_ms_extrapolated": dt / rows * share_rows * 1e3})
        log(f"oracle FFN fwd+bwd, micro-batch {mb} {'after' if planned else 'before'} the plan: {rows} of {share_rows} rows in {dt:.1f}s")
    return {"value": 18.0 * h * hff * rows_sum / dt_sum / 1e12, "unit": "TFLOP/s", "cores": threads, "kind": "oracle",
            "sched_getaffinity_cores": affinity, "seconds": dt_sum,
            "sample": f"expert FFN fwd+bwd (double precision, plain loops) on the first {frac:.4f} of every group of the straggler "
                      f"rank's share of {cfg.name}, before (unplanned layout) and after the plan, micro-batches {mbs}: "
                      f"{rows_sum} routed rows in all, real token rows, gradients and weights",
            "straggler_share": res,
            "integer_path_ms": {"route_hist_all_micro_batches": hist_ms, "plan_batch": plan_ms,
                                "permute_all_micro_batches": permute_ms, "micro_batches": n_mb}}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=3)
    ap.add_argument("--warmup", type=int, default=1)
    ap.add_argument("--config", type=int, default=4,
                    help="index into workloads.CONFIGS (default 4: the largest workload that fits one GPU)")
    ap.add_argument("--also-config", type=int, default=None,
                    help="a second workload timed after the first and reported under its own key (default: 1, the "
                         "Qwen3-30B-A3B-shaped layer, when --config is 4; -1: none)")
    ap.add_argument("--cpu-seconds", type=float, default=40.0, help="target length of the oracle's FFN sample (0 = skip the oracle leg)")
    ap.add_argument("--no-extras", action="store_true", help="skip the bandwidth-kernel, straggler, replica and model sections")
    ap.add_argument("--wgrad", choices=("batched", "per-mb"), default="batched",
                    help="weight gradients once per batch over all resident micro-batches (default), or "
                         "accumulated into dW micro-batch by micro-batch")
    ap.add_argument("--wgrad-tile", choices=("auto", "narrow", "wide"), default="auto",
                    help="output tile of the batched weight gradients (auto: by contraction length)")
    ap.add_argument("--gathered-copy", action="store_true",
                    help="materialise the group-ordered rows in the permutation (default with batched weight gradients: "
                         "the GEMMs gather token rows themselves)")
    ap.add_argument("--weights", choices=("fwd-transposed", "bwd-transposed", "plain"), default="fwd-transposed",
                    help="which GEMMs read transposed weight copies (made once per step inside the timed region) so that "
                         "their weight operand is contraction-strided: the forward ones (default; the data gradients "
                         "read the stored layout that way already), the data gradients (both passes then read "
                         "contraction-contiguous weights), or none")
    ap.add_argument("--backward", choices=("auto", "gate-fused", "plain"), default="auto",
                    help="gate-fused (needs batched weight gradients and the fused row gather): the combine's backward "
                         "folded into the expert backward (dOut rows read from the token tensor, the gate applied to dA, dgate "
                         "reduced in the same epilogue, dWd from dOut rows against gate * A); plain: the combine-backward pass "
                         "writes gate * dOut rows first.  auto (default): gate-fused when h' < 4096 - the fused form saves a "
                         "bandwidth pass over N x h and costs the dWd GEMM (N x h x h') about a tenth for its gathered operand")
    ap.add_argument("--plan", choices=("ahead", "inline"), default="ahead",
                    help="histogram and host plan of the next batch overlapped with this step's kernels (default: replayed "
                         "routing is known before a batch trains), or at the head of the step that uses them")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="also run three plain 1 GiB device copies (reference for scaling rocprofv3 byte counters)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU (each simulated EP rank's share executes on it); "
              "--gpus above 1 is not supported", file=sys.stderr)
        sys.exit(2)

    import torch
    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)

    if args.copy_calibration:
        src = torch.empty(1 << 30, dtype=torch.uint8, device="cuda").fill_(1)
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    main_res = run_config(args, args.config, args.steps, args.warmup, 0 if args.no_extras else 2, args.cpu_seconds)
    also = args.also_config if args.also_config is not None else (1 if args.config == 4 else -1)
    second = None
    if also >= 0 and also != args.config:
        import gc
        gc.collect()
        torch.cuda.empty_cache()
        second = run_config(args, also, max(args.steps, 5), args.warmup, 0 if args.no_extras else 1, 0.0)

    out = {"metric": "MoE expert-layer fwd+bwd TFLOP/s (bf16)", "value": main_res.pop("value"), "unit": "TFLOP/s",
           "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": main_res.pop("ms_per_step"),
           "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic"}
    out.update(main_res)
    if second is not None:
        second.pop("cpu_baseline")
        out[f"config{also + 1}"] = second
    print(json.dumps(out))


if __name__ == "__main__":
    main()

#!/usr/bin/env python3
"""Benchmark of the LRQK decode-step hot path on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload c3] [--r 32]
                    [--mode staged|direct] [--layers N] [--no-cpu-baseline]

A *step* is one pass of the whole hot path (proxy scores -> top-k -> hit/miss ->
fetch -> exact attention, i.e. one lrqk_decode_step call) for one layer.  The
default workload is the 128K-context LLaMA-3-8B-shaped decode (32 layers, 32 query /
8 KV heads, d = 128, l = 131072, r = 32, k = 2048, 64 lite tokens, 4096 cache slots per
head, batch 1); consecutive steps walk through the 32 layers, so the data touched
between two visits of a layer (> 5 GB) is far larger than any on-chip cache.  All
inputs are seeded synthetic tensors already resident (A_K, caches in HBM; K/V store in
pinned host memory) when the timed region starts.  The caches are primed with two
untimed passes over all layers ("seeded from the previous steps' selections").

Prints ONE JSON line: metric/value = layer-steps per second, plus
  roofline      achieved HBM bandwidth of the dominant kernel (the proxy-score stream
                over A_K) from HIP-event timing of that kernel alone on the same layers;
  cpu_baseline  the plain CPU oracle timed on the host cores on a bounded sample.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0

# HBM traffic of one proxy-score launch measured with rocprofv3 --pmc (FETCH_SIZE, then
# WRITE_SIZE, each scaled by what the same counter reads for lrqk_calib_copy), bytes per launch:
# profiles/proxy_scores_c3_r32_hbm_traffic.md.  Only for the workload it was measured on.
MEASURED_TRAFFIC = {"c3_r32": 130637 * 1024 + 2611 * 1024}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=256)
    ap.add_argument("--warmup", type=int, default=32)
    ap.add_argument("--workload", default="c3")
    ap.add_argument("--r", type=int, default=32)
    ap.add_argument("--layers", type=int, default=None)
    ap.add_argument("--mode", choices=["staged", "direct"], default="direct")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-seconds", type=float, default=12.0)
    ap.add_argument("--no-alg2", action="store_true",
                    help="skip the extra section that times the whole of Alg. 2 (factor update, "
                         "append, then the step)")
    ap.add_argument("--alg2-steps", type=int, default=64)
    ap.add_argument("--no-prefill", action="store_true",
                    help="skip the extra section that times the prefill factorisation (Alg. 1)")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs on one GPU only (no collectives, no sharding); "
              "run with --gpus 1", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    import paper_2510_23649_amd as L
    from paper_2510_23649_amd import build as hip_build
    from gen import get_config, make_layer, QueryStream, as_numpy

    if not hip_build.is_built():
        hip_build.build()
    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)
    dev = "cuda"

    cfg = get_config(args.workload, r=args.r)
    if args.layers:
        cfg = cfg.with_(layers=args.layers)
    nl = cfg.layers
    shape = L.Shape.make(B=cfg.B, Hq=cfg.Hq, Hkv=cfg.Hkv, l=cfg.l, r=cfg.r, k=cfg.k, w=cfg.w,
                         C_slots=cfg.C, d=cfg.d, scale=cfg.scale,
                         kv_dtype=L.LRQK_KV_BF16 if cfg.kv_dtype == "bf16" else L.LRQK_KV_F32)
    mode = L.LRQK_FETCH_STAGED if args.mode == "staged" else L.LRQK_FETCH_DIRECT
    with_alg2 = not args.no_alg2 and cfg.r in (8, 16, 32, 64)
    if with_alg2:      # room for the tokens the Alg. 2 section appends after the timed region
        alg2_per_layer = -(-args.alg2_steps // cfg.layers) + 1
        shape.l_cap = cfg.l + alg2_per_layer

    def log(msg):
        print(f"[bench] {msg}", file=sys.stderr, flush=True)

    # ---------------------------------------------------------------- inputs (untimed)
    t0 = time.time()
    layers, streams, bmats = [], [], []
    oracle_layer = None
    for li in range(nl):
        data = make_layer(cfg, li, device=dev)
        layers.append(L.LayerBuffers(shape, data.A_K, data.K, data.V))
        streams.append(QueryStream(data))
        bmats.append(data.Bmat)
        if li == 0 and not args.no_cpu_baseline:
            oracle_layer = dict(A_K=as_numpy(data.A_K), K=as_numpy(data.K), V=as_numpy(data.V))
        data.K = data.V = data.A_K = None
        if li % 8 == 7:
            log(f"generated {li + 1}/{nl} layers ({time.time() - t0:.1f}s)")
    torch.cuda.synchronize()
    plan = L.Plan(shape.with_l(shape.rows))
    out = torch.empty((cfg.B, cfg.Hq, cfg.d), device=dev)
    n_miss = torch.zeros((cfg.B, cfg.Hq), dtype=torch.int32, device=dev)
    dbg = dict(n_miss=n_miss)
    step_no = [0] * nl

    def run_step(li, q, q_hat, debug=None):
        step_no[li] += 1
        # a layer's first step estimates its candidate thresholds from a sample; later steps
        # carry them over
        flags = L.LRQK_SELECT_FRESH if step_no[li] == 1 else 0
        return L.lrqk_decode_step(plan, shape, step_no[li], layers[li].struct, q_hat, q, out,
                                  mode | flags, debug)

    # prime the caches: two untimed passes over all layers
    oracle_queries = []
    for p in range(2):
        for li in range(nl):
            q, q_hat = streams[li].next()
            if li == 0:
                oracle_queries.append((as_numpy(q), as_numpy(q_hat)))
            run_step(li, q, q_hat)
    torch.cuda.synchronize()
    log(f"caches primed ({time.time() - t0:.1f}s)")

    # queries of the warm-up and timed steps, resident before timing starts
    n_pre = args.warmup + 2 * args.steps
    queries = []
    for i in range(n_pre):
        q, q_hat = streams[i % nl].next()
        queries.append((q, q_hat))
    torch.cuda.synchronize()

    # ---------------------------------------------------------------- timed region
    for i in range(args.warmup):
        run_step(i % nl, *queries[i])
    torch.cuda.synchronize()
    tot_miss = 0
    t_start = time.perf_counter()
    for i in range(args.warmup, args.warmup + args.steps):
        tm = run_step(i % nl, *queries[i])
        tot_miss += max(tm, 0)
    torch.cuda.synchronize()
    t_end = time.perf_counter()
    elapsed = t_end - t_start
    ms_per_step = 1e3 * elapsed / args.steps
    value = args.steps / elapsed
    log(f"timed {args.steps} steps: {ms_per_step * 1e3:.1f} us/step")

    # ---------------------------------------------------------------- per-phase breakdown
    plan.profile(args.steps)
    for i in range(args.warmup + args.steps, args.warmup + 2 * args.steps):
        run_step(i % nl, *queries[i], debug=dbg)
    phases_ms, n_prof = plan.profile_read()
    plan.profile(0)
    phases_us = {k: 1e3 * v / max(n_prof, 1) for k, v in phases_ms.items()}
    torch.cuda.synchronize()
    last_nmiss = n_miss.clamp(min=0).sum().item()
    miss_rate = (tot_miss / (args.steps * cfg.B * cfg.Hq * cfg.k) if args.mode == "staged"
                 else last_nmiss / (cfg.B * cfg.Hq * cfg.k))

    # ---------------------------------------------------------------- dominant kernel alone
    # the proxy-score pass exactly as the fused step launches it, n_k launches back to back
    # over the layers' A_K, bracketed by HIP events on the launch stream inside the library
    # (a Python loop of single launches would be bound by the interpreter, not by the GPU)
    n_k = max(args.steps, 64)
    k1_us = plan.time_proxy_pass(shape, [lb.A_K for lb in layers], queries[0][1], n_k,
                                  sel_thr=layers[0].sel_thr)
    a_k_bytes = cfg.B * cfg.Hkv * cfg.l * cfg.r * 4 + cfg.B * cfg.Hq * cfg.r * 4
    k1_gbs = a_k_bytes / (k1_us * 1e-6) / 1e9

    # a plain copy of known traffic (2 x A_K bytes per launch): calibrates the HBM byte counters
    # when this script runs under rocprofv3 --pmc; it is outside every timed region
    calib_dst = torch.empty_like(layers[0].A_K)
    for i in range(4):
        L.lrqk_calib_copy(calib_dst, layers[(i + 1) % nl].A_K)
    torch.cuda.synchronize()
    del calib_dst

    step_bytes = (a_k_bytes + 2 * 2 * cfg.d * (cfg.B * cfg.Hq * cfg.k + cfg.B * cfg.Hkv * cfg.w)
                  + 2 * cfg.B * cfg.Hq * cfg.d * 4 + 2 * cfg.B * cfg.Hq * cfg.k * 4)
    gpu_us = sum(phases_us.values())
    row_kv_bytes = 2 * cfg.d * (2 if cfg.kv_dtype == "bf16" else 4)   # one K row + one V row

    # ---------------------------------------------------------------- the whole of Alg. 2
    # (outside the headline metric) factor update -> append -> the step at length l + 1, on the
    # same layers; B_K starts at the generator's basis, B_Q at its dual basis, k_t, v_t random
    alg2 = None
    if with_alg2:
        i32 = dict(dtype=torch.int32, device=dev)
        sel_idx = [torch.zeros((cfg.B, cfg.Hq, cfg.k), **i32) for _ in range(nl)]
        sel_slot = [torch.zeros((cfg.B, cfg.Hq, cfg.k), **i32) for _ in range(nl)]
        B_Q, B_K = [], []
        for li in range(nl):
            Bm = bmats[li]
            dual = torch.linalg.solve(Bm @ Bm.transpose(-1, -2), Bm)
            B_Q.append(dual.repeat_interleave(cfg.G, dim=1).contiguous())
            B_K.append(Bm.clone().contiguous())
            q, q_hat = streams[li].next()       # leaves this layer's previous selection
            run_step(li, q, q_hat, debug=dict(sel_idx=sel_idx[li], sel_slot=sel_slot[li]))
        ws_u = torch.empty(L.lrqk_workspace_bytes(shape.with_l(shape.rows), L.LRQK_WS_UPDATE),
                           dtype=torch.uint8, device=dev)
        q_hat_u = torch.zeros((cfg.B, cfg.Hq, cfg.r), device=dev)
        k_hat_u = torch.zeros((cfg.B, cfg.Hkv, cfg.r), device=dev)
        n2 = args.alg2_steps
        kvdt = torch.bfloat16 if cfg.kv_dtype == "bf16" else torch.float32
        qs2 = [streams[i % nl].next()[0] for i in range(n2)]
        kn = [torch.randn(cfg.B, cfg.Hkv, cfg.d, device=dev).to(kvdt) for _ in range(n2)]
        vn = [torch.randn(cfg.B, cfg.Hkv, cfg.d, device=dev).to(kvdt) for _ in range(n2)]
        l_now = [cfg.l] * nl
        ev = [[torch.cuda.Event(enable_timing=True) for _ in range(4)] for _ in range(n2)]
        torch.cuda.synchronize()
        t_a = time.perf_counter()
        for i in range(n2):
            li = i % nl
            shp = shape.with_l(l_now[li])
            ev[i][0].record()
            L.lrqk_factor_update(shp, layers[li].struct, sel_idx[li], sel_slot[li], qs2[i], kn[i],
                                 B_Q[li], B_K[li], 1.0, 1.0, 2, q_hat_u, k_hat_u, ws_u)
            ev[i][1].record()
            L.lrqk_append_token(shp, layers[li].struct, k_hat_u, kn[i], vn[i])
            ev[i][2].record()
            l_now[li] += 1
            step_no[li] += 1
            L.lrqk_decode_step(plan, shape.with_l(l_now[li]), step_no[li], layers[li].struct,
                               q_hat_u, qs2[i], out, mode,
                               dict(sel_idx=sel_idx[li], sel_slot=sel_slot[li]))
            ev[i][3].record()
        torch.cuda.synchronize()
        t_b = time.perf_counter()
        skip = min(8, n2 // 2)
        seg = np.array([[ev[i][j].elapsed_time(ev[i][j + 1]) * 1e3 for j in range(3)]
                        for i in range(skip, n2)])
        alg2 = {"steps": n2, "us_per_step_wall": (t_b - t_a) / n2 * 1e6,
                "factor_update_us": float(seg[:, 0].mean()),
                "append_token_us": float(seg[:, 1].mean()),
                "decode_step_us": float(seg[:, 2].mean()),
                "lambda_d1": 1.0, "lambda_d2": 1.0, "rounds": 2,
                "note": "HIP-event time of each call on the launch stream; the wall figure "
                        "includes the Python launch loop"}
        log(f"Alg. 2: update {alg2['factor_update_us']:.1f} us, append "
            f"{alg2['append_token_us']:.1f} us, step {alg2['decode_step_us']:.1f} us")

    # ---------------------------------------------------------------- prefill factorisation
    # (outside the headline metric) Alg. 1 for one layer of the same shape: Q, K near rank r,
    # N(0,1) initial factors, lambda_pQ = lambda_pK = 1, 2 rounds
    prefill = None
    if not args.no_prefill and cfg.r in (8, 16, 32, 64):
        from gen import make_prefill_inputs
        pdata = make_layer(cfg, 0, device=dev)
        Qp, A_Q0, A_K0 = make_prefill_inputs(cfg, pdata)
        Kp = pdata.K
        pdata.V = pdata.A_K = None
        pshape = shape.with_l(cfg.l)
        pshape.l_cap = 0
        ws_p = torch.empty(L.lrqk_workspace_bytes(pshape, L.LRQK_WS_PREFILL), dtype=torch.uint8,
                           device=dev)
        B_Qp = torch.empty((cfg.B, cfg.Hq, cfg.r, cfg.d), device=dev)
        B_Kp = torch.empty((cfg.B, cfg.Hkv, cfg.r, cfg.d), device=dev)
        times = []
        for rep in range(4):
            A_Qp, A_Kp = A_Q0.clone(), A_K0.clone()
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            torch.cuda.synchronize()
            e0.record()
            L.lrqk_prefill_factorize(pshape, Qp, Kp, A_Qp, A_Kp, B_Qp, B_Kp, 1.0, 1.0, 2, ws_p)
            e1.record()
            torch.cuda.synchronize()
            times.append(e0.elapsed_time(e1))
        ms = float(np.median(times[1:]))
        rows_q, rows_k, r_, d_ = cfg.B * cfg.Hq * cfg.l, cfg.B * cfg.Hkv * cfg.l, cfg.r, cfg.d
        # initial sums on both sides; per round: fused apply + sums on K, then on Q (the last
        # round's Q pass only applies)
        flops = (2 * r_ * (d_ + r_) * (rows_q + rows_k)
                 + 2 * 2 * r_ * (2 * d_ + r_) * rows_k
                 + 2 * r_ * (2 * d_ + r_) * rows_q + 2 * r_ * d_ * rows_q)
        prefill = {"ms_per_layer": ms, "rounds": 2, "lambda_pQ": 1.0, "lambda_pK": 1.0,
                   "algorithmic_flops": flops, "achieved_TFLOPs": flops / (ms * 1e-3) / 1e12,
                   "peak_TFLOPs_fp32_mfma": 157.3,
                   "frac": flops / (ms * 1e-3) / 1e12 / 157.3,
                   "note": "HIP-event time of one lrqk_prefill_factorize call (all its launches, "
                           "r x r solves included) on one layer of the same shape"}
        log(f"prefill factorisation: {ms:.3f} ms per layer, "
            f"{prefill['achieved_TFLOPs']:.1f} TFLOP/s")
        del Qp, A_Q0, A_K0, Kp, ws_p, pdata

    # ---------------------------------------------------------------- CPU oracle baseline
    cpu = None
    if oracle_layer is not None:
        from oracle import lrqk_oracle as orc
        st = orc.CacheState(cfg.B, cfg.Hq, cfg.l, cfg.C)
        cK = np.zeros((cfg.B, cfg.Hq, cfg.C, cfg.d), oracle_layer["K"].dtype)
        cV = np.zeros_like(cK)
        done, t_cpu = 0, 0.0
        qi = 0
        while t_cpu < args.cpu_seconds and done < 2048:
            qn, qhn = oracle_queries[qi % len(oracle_queries)]
            qi += 1
            tc = time.perf_counter()
            orc.decode_step(oracle_layer["A_K"], qhn, qn, oracle_layer["K"], oracle_layer["V"], st,
                            cK, cV, done + 1, cfg.k, cfg.w, cfg.scale)
            t_cpu += time.perf_counter() - tc
            done += 1
        cpu = {"value": done / t_cpu, "unit": "layer-steps/s", "cores": orc.num_threads(),
               "kind": "oracle",
               "sample": f"{done} consecutive steps of layer 0 of the same workload "
                         f"({t_cpu:.1f} s of CPU time, gcc -O2 + OpenMP over heads)"}

    result = {
        "metric": "LRQK decode steps/sec per layer at 128K ctx; achieved HBM GB/s vs peak",
        "value": value, "unit": "layer-steps/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": ms_per_step, "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": "f32", "data": "synthetic",
        "config": {"workload": f"{cfg.name}: LLaMA-3-8B-shaped decode, {nl} layers, "
                               f"{cfg.Hq}q/{cfg.Hkv}kv heads, d={cfg.d}, l={cfg.l}, r={cfg.r}, "
                               f"k={cfg.k}, w={cfg.w}, C={cfg.C}, batch {cfg.B}, bf16 K/V, "
                               f"fp32 factors",
                   "fetch_mode": args.mode, "step": "one layer's lrqk_decode_step",
                   "layers_rotated": nl, "miss_rate": miss_rate},
        "roofline": {"bound": "hbm", "achieved": k1_gbs, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": k1_gbs / HBM_PEAK_GBS,
                     "traffic": MEASURED_TRAFFIC.get(f"{cfg.name}_r{cfg.r}"),
                     "kernel": "proxy_scores_kernel", "us_per_launch": k1_us,
                     "algorithmic_bytes_per_launch": a_k_bytes},
        "cpu_baseline": cpu,
        "phases_us": phases_us,
        "host_link": {"rows_per_step": miss_rate * cfg.B * cfg.Hq * cfg.k,
                      "MB_per_step": miss_rate * cfg.B * cfg.Hq * cfg.k * row_kv_bytes / 1e6,
                      "attend_phase_us": phases_us.get("attend"),
                      "GBs_if_the_attend_phase_were_all_link_time":
                          miss_rate * cfg.B * cfg.Hq * cfg.k * row_kv_bytes
                          / max(phases_us.get("attend", 0.0), 1e-9) / 1e3,
                      "note": "missing K and V rows cross the host link inside the attention "
                              "kernel (direct mode); the step is bound by this leg"},
        "alg2": alg2,
        "prefill": prefill,
        "step_roofline": {"algorithmic_bytes_per_step": step_bytes,
                          "gpu_us_per_step_sum_of_phases": gpu_us,
                          "achieved_GBs_end_to_end": step_bytes / (ms_per_step * 1e-3) / 1e9,
                          "frac_end_to_end": step_bytes / (ms_per_step * 1e-3) / 1e9 / HBM_PEAK_GBS},
    }
    plan.close()
    print(json.dumps(result))


if __name__ == "__main__":
    main()

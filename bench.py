#!/usr/bin/env python3
"""Benchmark of the LRQK decode-step hot path on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload c3] [--r 32]
                    [--mode staged|direct] [--layers N] [--no-cpu-baseline] [--no-alg2]
                    [--no-prefill] [--no-workloads]

A *step* is one pass of the whole hot path (proxy scores -> top-k -> hit/miss ->
fetch -> exact attention, i.e. one lrqk_decode_step call) for one layer.  The
default workload is the 128K-context LLaMA-3-8B-shaped decode (32 layers, 32 query /
8 KV heads, d = 128, l = 131072, r = 32, k = 2048, 64 lite tokens, 4096 cache slots per
head, batch 1); consecutive steps walk through the 32 layers, so the data touched
between two visits of a layer (> 5 GB) is far larger than any on-chip cache.  All
inputs are seeded synthetic tensors already resident (A_K, caches in HBM; K/V store in
pinned host memory) when the timed region starts.  The caches are primed with eight
untimed passes over all layers ("seeded from the previous steps' selections": after them the
miss rate no longer drifts); a layer's
first step estimates its selection thresholds from a sample, later steps carry them.

Prints ONE JSON line: metric/value = layer-steps per second of the headline workload, plus
  roofline      achieved HBM bandwidth of the dominant kernel (the proxy-score stream over
                A_K) from HIP events attached to that kernel, and under "stages" the same
                for every kernel of the step (events attached to each kernel inside real
                steps), with the attention also measured on steps in which nothing misses;
  cpu_baseline  the plain CPU oracle timed on the host cores on a bounded sample;
  staged        the same workload with the fetch leg staged through the host;
  workloads     the other workloads of the measurement plan (rank 16 / 64, the Qwen-shaped
                batch-8 layer, the miss-heavy batch-16 layer over 64 steps), each with its
                time per step, miss rate and proxy-score kernel figures;
  alg2, prefill the factor update / append and the prefill factorisation (not in `value`).
"""
from __future__ import annotations

import argparse
import json
import os
import re
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0


def log(msg):
    print(f"[bench] {msg}", file=sys.stderr, flush=True)


def measured_traffic(cfg):
    """HBM bytes of one proxy-score launch from the rocprofv3 --pmc summary kept under
    profiles/ for this workload (FETCH_SIZE + WRITE_SIZE, scaled by what the same counters
    read for the plain copy kernel); None where no summary exists for the workload."""
    path = os.path.join(ROOT, "profiles", f"proxy_scores_{cfg.name}_r{cfg.r}_hbm_traffic.md")
    try:
        m = re.search(r"traffic_bytes_per_launch:\s*(\d+)", open(path).read())
    except OSError:
        return None
    return int(m.group(1)) if m else None


class Workload:
    """One workload resident on the GPU: its layers, query streams, plan and step counters."""

    def __init__(self, L, cfg, mode, extra_rows=0, keep_oracle_layer=False):
        import torch
        from gen import make_layer, QueryStream, as_numpy
        self.L, self.cfg, self.torch = L, cfg, torch
        self.nl = cfg.layers
        self.mode = mode
        self.shape = L.Shape.make(B=cfg.B, Hq=cfg.Hq, Hkv=cfg.Hkv, l=cfg.l, r=cfg.r, k=cfg.k,
                                  w=cfg.w, C_slots=cfg.C, d=cfg.d, scale=cfg.scale,
                                  kv_dtype=L.LRQK_KV_BF16 if cfg.kv_dtype == "bf16"
                                  else L.LRQK_KV_F32)
        if extra_rows:
            self.shape.l_cap = cfg.l + extra_rows
        t0 = time.time()
        self.layers, self.streams, self.bmats = [], [], []
        self.oracle_layer = None
        for li in range(self.nl):
            data = make_layer(cfg, li, device="cuda")
            self.layers.append(L.LayerBuffers(self.shape, data.A_K, data.K, data.V))
            self.streams.append(QueryStream(data))
            self.bmats.append(data.Bmat)
            if li == 0 and keep_oracle_layer:
                self.oracle_layer = dict(A_K=as_numpy(data.A_K), K=as_numpy(data.K),
                                         V=as_numpy(data.V))
            data.K = data.V = data.A_K = None
        torch.cuda.synchronize()
        log(f"{cfg.name} r={cfg.r}: {self.nl} layer(s) generated ({time.time() - t0:.1f}s)")
        self.plan = L.Plan(self.shape.with_l(self.shape.rows))
        self.out = torch.empty((cfg.B, cfg.Hq, cfg.d), device="cuda")
        self.n_miss = torch.zeros((cfg.B, cfg.Hq), dtype=torch.int32, device="cuda")
        self.step_no = [0] * self.nl
        self._next_layer = 0
        self.oracle_queries = []

    def step(self, li, q, q_hat, debug=None, mode=None, shape=None):
        L = self.L
        self.step_no[li] += 1
        # a layer's first step estimates its candidate thresholds from a sample; later steps
        # carry them over
        flags = L.LRQK_SELECT_FRESH if self.step_no[li] == 1 else 0
        return L.lrqk_decode_step(self.plan, shape or self.shape, self.step_no[li],
                                  self.layers[li].struct, q_hat, q, self.out,
                                  (self.mode if mode is None else mode) | flags, debug)

    def prime(self, passes=8):
        from gen import as_numpy
        for _ in range(passes):
            for li in range(self.nl):
                q, q_hat = self.streams[li].next()
                if li == 0 and self.oracle_layer is not None:
                    self.oracle_queries.append((as_numpy(q), as_numpy(q_hat)))
                self.step(li, q, q_hat)
        self.torch.cuda.synchronize()

    def queries(self, n):
        """The next n queries of the rotation over the layers, as (layer, q, q_hat)."""
        qs = []
        for _ in range(n):
            li = self._next_layer
            self._next_layer = (li + 1) % self.nl
            qs.append((li, *self.streams[li].next()))
        self.torch.cuda.synchronize()
        return qs

    def timed(self, queries, warmup, mode=None):
        """Wall-clock time of len(queries) - warmup consecutive steps, layers in rotation."""
        torch = self.torch
        for i in range(warmup):
            self.step(*queries[i], mode=mode)
        torch.cuda.synchronize()
        tot_miss = 0
        t0 = time.perf_counter()
        for i in range(warmup, len(queries)):
            tot_miss += max(self.step(*queries[i], mode=mode), 0)
        torch.cuda.synchronize()
        return (time.perf_counter() - t0) / (len(queries) - warmup), tot_miss

    def kernel_times(self, queries, repeat_each=False):
        """Microseconds per step of every kernel of the step (events attached to the kernels).
        repeat_each: the queries are stepped in rounds over the layers, every round twice, and
        only the second time is timed -- its selections are the ones just made, so nothing
        misses, while a whole round over the other layers lies between the two visits of a
        layer (no cache holds its rows)."""
        cfg = self.cfg
        self.plan.profile(len(queries))
        miss = counted = 0
        for r0 in range(0, len(queries), self.nl):
            chunk = queries[r0:r0 + self.nl]          # at most one visit of every layer
            if repeat_each:
                for li, q, q_hat in chunk:
                    self._untimed_step(li, q, q_hat)
            for li, q, q_hat in chunk:
                self.step(li, q, q_hat, debug=dict(n_miss=self.n_miss))
                if repeat_each or counted < 8:
                    miss += int(self.n_miss.clamp(min=0).sum().item())
                    counted += 1
        ms, n = self.plan.profile_read()
        self.plan.profile(0)
        us = {k: 1e3 * v / max(n, 1) for k, v in ms.items() if v > 0.0}
        return us, miss / (max(counted, 1) * cfg.B * cfg.Hq * cfg.k)

    def _untimed_step(self, li, q, q_hat):
        # a step that takes no slot of the armed profile: it runs on a second plan
        if not hasattr(self, "_plan2"):
            self._plan2 = self.L.Plan(self.shape.with_l(self.shape.rows))
        self.step_no[li] += 1
        self.L.lrqk_decode_step(self._plan2, self.shape, self.step_no[li],
                                self.layers[li].struct, q_hat, q, self.out, self.mode, None)

    def bytes(self):
        cfg = self.cfg
        esz = 2 if cfg.kv_dtype == "bf16" else 4
        a1 = cfg.B * cfg.Hkv * cfg.l * cfg.r * 4 + cfg.B * cfg.Hq * cfg.r * 4
        a5 = (2 * esz * cfg.d * (cfg.B * cfg.Hq * cfg.k + cfg.B * cfg.Hkv * cfg.w)
              + 2 * cfg.B * cfg.Hq * cfg.d * 4)
        a23 = 2 * cfg.B * cfg.Hq * cfg.k * 4            # k positions out, k slot look-ups
        return dict(a1=a1, a23=a23, a5=a5, step=a1 + a23 + a5, row=2 * cfg.d * esz)

    def close(self):
        self.plan.close()
        if hasattr(self, "_plan2"):
            self._plan2.close()
        self.layers = self.streams = None
        self.torch.cuda.empty_cache()


def stage(us, nbytes):
    gbs = nbytes / (us * 1e-6) / 1e9
    return {"us": us, "algorithmic_bytes": nbytes, "GBs": gbs, "frac_of_hbm_peak": gbs / HBM_PEAK_GBS}


def measure(wl, steps, warmup, with_all_hit):
    """Time per step, per-kernel times and the roofline figures of one resident workload."""
    cfg, by = wl.cfg, wl.bytes()
    n_prof = min(steps, 64)
    qs = wl.queries(warmup + steps + n_prof + (n_prof if with_all_hit else 0))
    sec, tot_miss = wl.timed(qs[:warmup + steps], warmup)
    k_us, miss_rate = wl.kernel_times(qs[warmup + steps:warmup + steps + n_prof])
    if wl.mode == wl.L.LRQK_FETCH_STAGED:
        miss_rate = tot_miss / (steps * cfg.B * cfg.Hq * cfg.k)
    # the proxy-score pass exactly as the step launches it, back to back over the layers' A_K,
    # events attached to every kernel (a Python loop of single launches is interpreter-bound)
    li0, _, q_hat0 = qs[0]
    k1_us = wl.plan.time_proxy_pass(wl.shape, [lb.A_K for lb in wl.layers], q_hat0,
                                    max(steps, 64), sel_thr=wl.layers[li0].sel_thr)
    res = {
        "ms_per_step": 1e3 * sec, "layer_steps_per_s": 1.0 / sec, "steps": steps,
        "layers_rotated": wl.nl, "miss_rate": miss_rate,
        "host_link_MB_per_step": miss_rate * cfg.B * cfg.Hq * cfg.k * by["row"] / 1e6,
        "kernels_us": k_us,
        "proxy_scores_kernel": stage(k1_us, by["a1"]),
        "step_algorithmic_bytes": by["step"],
        "frac_of_hbm_peak_end_to_end": by["step"] / sec / 1e9 / HBM_PEAK_GBS,
    }
    if with_all_hit:
        hit_us, hit_miss = wl.kernel_times(qs[warmup + steps + n_prof:], repeat_each=True)
        res["all_hit_kernels_us"] = hit_us
        res["all_hit_miss_rate"] = hit_miss
    return res


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
                    help="skip the section that times the whole of Alg. 2 (factor update, append, "
                         "then the step)")
    ap.add_argument("--alg2-steps", type=int, default=64)
    ap.add_argument("--no-prefill", action="store_true",
                    help="skip the section that times the prefill factorisation (Alg. 1)")
    ap.add_argument("--no-workloads", action="store_true",
                    help="skip the other workloads (rank sweep, batch-8 and batch-16 layers) and "
                         "the staged-fetch figure")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs on one GPU only (no collectives, no sharding); "
              "run with --gpus 1", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    import paper_2510_23649_amd as L
    from paper_2510_23649_amd import build as hip_build
    from gen import get_config

    if not hip_build.is_built():
        hip_build.build()
    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)
    dev = "cuda"
    t_begin = time.time()

    cfg = get_config(args.workload, r=args.r)
    if args.layers:
        cfg = cfg.with_(layers=args.layers)
    nl = cfg.layers
    mode = L.LRQK_FETCH_STAGED if args.mode == "staged" else L.LRQK_FETCH_DIRECT
    with_alg2 = not args.no_alg2 and cfg.r in (8, 16, 32, 64)
    extra_rows = (-(-args.alg2_steps // nl) + 1) if with_alg2 else 0

    # ---------------------------------------------------------------- headline workload
    wl = Workload(L, cfg, mode, extra_rows=extra_rows, keep_oracle_layer=not args.no_cpu_baseline)
    wl.prime()
    log(f"caches primed ({time.time() - t_begin:.1f}s)")
    head = measure(wl, args.steps, args.warmup, with_all_hit=True)
    by = wl.bytes()
    log(f"timed {args.steps} steps: {head['ms_per_step'] * 1e3:.1f} us/step; kernels "
        + ", ".join(f"{k} {v:.1f}" for k, v in head["kernels_us"].items()))
    shape, layers, streams, plan, out = wl.shape, wl.layers, wl.streams, wl.plan, wl.out
    step_no = wl.step_no

    # a plain copy of known traffic (2 x A_K bytes per launch): calibrates the HBM byte counters
    # when this script runs under rocprofv3 --pmc; it is outside every timed region
    calib_dst = torch.empty_like(layers[0].A_K)
    for i in range(4):
        L.lrqk_calib_copy(calib_dst, layers[(i + 1) % nl].A_K)
    torch.cuda.synchronize()
    del calib_dst

    # the same workload with the fetch leg staged through the host (the design the task states:
    # miss list -> host gather -> hipMemcpyAsync on a side stream, overlapped with hit rows)
    staged = None
    if not args.no_workloads and args.mode == "direct":
        n_st = 32
        qs = wl.queries(8 + n_st)
        sec, tot = wl.timed(qs, 8, mode=L.LRQK_FETCH_STAGED)
        staged = {"ms_per_step": 1e3 * sec, "layer_steps_per_s": 1.0 / sec, "steps": n_st,
                  "miss_rate": tot / (n_st * cfg.B * cfg.Hq * cfg.k)}
        log(f"staged fetch: {sec * 1e6:.1f} us/step")

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
            Bm = wl.bmats[li]
            dual = torch.linalg.solve(Bm @ Bm.transpose(-1, -2), Bm)
            B_Q.append(dual.repeat_interleave(cfg.G, dim=1).contiguous())
            B_K.append(Bm.clone().contiguous())
            q, q_hat = streams[li].next()       # leaves this layer's previous selection
            wl.step(li, q, q_hat, debug=dict(sel_idx=sel_idx[li], sel_slot=sel_slot[li]))
        wl._next_layer = 0
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
            wl.step(li, qs2[i], q_hat_u, debug=dict(sel_idx=sel_idx[li], sel_slot=sel_slot[li]),
                    shape=shape.with_l(l_now[li]))
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

    oracle_layer, oracle_queries = wl.oracle_layer, wl.oracle_queries
    wl.close()
    del wl, layers, streams, plan

    # ---------------------------------------------------------------- prefill factorisation
    # (outside the headline metric) Alg. 1 for one layer of the same shape: Q, K near rank r,
    # N(0,1) initial factors, lambda_pQ = lambda_pK = 1, 2 rounds
    prefill = None
    if not args.no_prefill and cfg.r in (8, 16, 32, 64):
        from gen import make_layer, make_prefill_inputs
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
        del Qp, A_Q0, A_K0, Kp, ws_p, pdata, A_Qp, A_Kp
        torch.cuda.empty_cache()

    # ---------------------------------------------------------------- the other workloads
    workloads = None
    if not args.no_workloads:
        workloads = {}
        plan_list = [("c3_r16", get_config("c3", r=16, layers=8), 64),
                     ("c3_r64", get_config("c3", r=64, layers=8), 64),
                     ("c4", get_config("c4", layers=2), 64),
                     ("c5", get_config("c5"), 64)]
        for name, wcfg, n_steps in plan_list:
            w2 = Workload(L, wcfg, L.LRQK_FETCH_DIRECT)
            w2.prime()
            res = measure(w2, n_steps, 8, with_all_hit=False)
            res["workload"] = (f"{wcfg.Hq}q/{wcfg.Hkv}kv heads, l={wcfg.l}, r={wcfg.r}, k={wcfg.k}, "
                               f"w={wcfg.w}, C={wcfg.C}, batch {wcfg.B}, fetch direct")
            workloads[name] = res
            log(f"{name}: {res['ms_per_step'] * 1e3:.1f} us/step, miss rate "
                f"{res['miss_rate']:.3f}, proxy kernel {res['proxy_scores_kernel']['us']:.1f} us "
                f"({res['proxy_scores_kernel']['frac_of_hbm_peak']:.2f} of peak)")
            w2.close()
            del w2

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

    k_us, hit_us = head["kernels_us"], head["all_hit_kernels_us"]
    k1 = head["proxy_scores_kernel"]
    sel_us = k_us.get("select", 0.0) + k_us.get("resolve", 0.0)
    att_hit = hit_us.get("attend", 0.0) + hit_us.get("combine", 0.0)
    chain_hit = (hit_us.get("proxy_scores", 0.0) + hit_us.get("select", 0.0)
                 + hit_us.get("resolve", 0.0) + att_hit)
    result = {
        "metric": "LRQK decode steps/sec per layer at 128K ctx; achieved HBM GB/s vs peak",
        "value": head["layer_steps_per_s"], "unit": "layer-steps/s", "n_gpus": 1,
        "steps": args.steps, "warmup": args.warmup, "ms_per_step": head["ms_per_step"],
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "f32",
        "data": "synthetic",
        "config": {"workload": f"{cfg.name}: LLaMA-3-8B-shaped decode, {nl} layers, "
                               f"{cfg.Hq}q/{cfg.Hkv}kv heads, d={cfg.d}, l={cfg.l}, r={cfg.r}, "
                               f"k={cfg.k}, w={cfg.w}, C={cfg.C}, batch {cfg.B}, bf16 K/V, "
                               f"fp32 factors",
                   "fetch_mode": args.mode, "step": "one layer's lrqk_decode_step",
                   "layers_rotated": nl, "miss_rate": head["miss_rate"]},
        "roofline": {
            "bound": "hbm", "achieved": k1["GBs"], "peak": HBM_PEAK_GBS, "unit": "GB/s",
            "frac": k1["frac_of_hbm_peak"], "traffic": measured_traffic(cfg),
            "kernel": "proxy_scores_kernel", "us_per_launch": k1["us"],
            "algorithmic_bytes_per_launch": by["a1"],
            "stages": {
                "a1_proxy_scores": stage(k_us.get("proxy_scores", k1["us"]), by["a1"]),
                "a2_a3_select_resolve": dict(stage(max(sel_us, 1e-9), by["a23"]),
                                             note="latency-bound: one workgroup per head works "
                                                  "on a few KB; the fraction is not meaningful"),
                "a5_attend_with_fetch": dict(
                    stage(k_us.get("attend", 0.0) + k_us.get("combine", 0.0) or 1e-9, by["a5"]),
                    note="the missing rows cross the host link inside this kernel: it is bound "
                         "by that link, not by HBM",
                    host_link_GBs=head["host_link_MB_per_step"] * 1e-3
                                  / max(k_us.get("attend", 0.0), 1e-9) * 1e6),
                "a5_attend_all_hit": stage(max(att_hit, 1e-9), by["a5"]),
                "a1_a2_a3_a5_all_hit": stage(max(chain_hit, 1e-9), by["step"]),
            }},
        "cpu_baseline": cpu,
        "kernels_us": k_us,
        "all_hit_kernels_us": hit_us,
        "host_link": {"rows_per_step": head["miss_rate"] * cfg.B * cfg.Hq * cfg.k,
                      "MB_per_step": head["host_link_MB_per_step"]},
        "step_roofline": {"algorithmic_bytes_per_step": by["step"],
                          "gpu_us_per_step_sum_of_kernels": sum(k_us.values()),
                          "achieved_GBs_end_to_end": by["step"] / (head["ms_per_step"] * 1e-3) / 1e9,
                          "frac_end_to_end": head["frac_of_hbm_peak_end_to_end"]},
        "staged": staged,
        "workloads": workloads,
        "alg2": alg2,
        "prefill": prefill,
    }
    log(f"done ({time.time() - t_begin:.1f}s)")
    print(json.dumps(result))


if __name__ == "__main__":
    main()

"""Hit/miss ablation and miss-rate grid on the synthetic workloads (needs a GPU).

    python -m paper_2510_23649_amd.ablation [--grid] [--no-hit-miss] [--group-fetch]
                                             [--end-to-end] [--steps N] [--drift F]

Two experiments of the paper, re-run on seeded synthetic inputs (its prompts and models are
not available; the generator's query drift is what sets the level of the miss rate, so the
numbers show how the mechanism responds to r, the number of active tokens and the number of
lite tokens, not what a language model would produce):

  --grid         Sec. 5.3: rank r in {8, 16, 32, 64} x active tokens in {128, 256, 512} x lite
                 tokens in {4, 8}, cache of exactly k slots (the paper's cache), miss rate =
                 fetched rows / selected rows per step; mean and standard deviation per cell,
                 and a histogram over all cells and steps.
  --no-hit-miss  App. C.2, "LRQK no hit/miss": the same decode steps with the cache emptied
                 before every step, so that every selected row crosses the host link, against
                 the default (only the missing rows do).
  --group-fetch  the fetch leg per head against the fetch shared by the query heads of a KV
                 group (a row missed by several heads crosses the host link once), for heads
                 that want the same tokens to different degrees.
  --attend-all-hit  step a5 alone (lrqk_sparse_attend) on caches that hold every selected row,
                 for profiling the attention kernels with nothing to fetch.
  --end-to-end   the whole method in sequence: prefill factorisation of a synthetic prompt,
                 then decode steps (factor update, append, proxy top-k, fetch, attention) on
                 the factors it produced; reports the recall of the exact top-k and the
                 distance of the output from dense attention.

Everything runs through the library's entry points; this module only generates inputs,
launches and tabulates.
"""
from __future__ import annotations

import argparse
import os
import sys
import time

import numpy as np
import torch

from . import binding as L
from .state import LayerBuffers

# the seeded workload generators live beside the package, at the repository root
sys.path.insert(0, os.path.dirname(os.path.dirname(os.path.abspath(__file__))))


def _shape(cfg, **kw):
    return L.Shape.make(B=cfg.B, Hq=cfg.Hq, Hkv=cfg.Hkv, l=cfg.l, r=cfg.r, k=cfg.k, w=cfg.w,
                        C_slots=cfg.C, d=cfg.d, scale=cfg.scale, **kw)


def miss_rate_grid(steps: int, warm: int, drift: float, out=sys.stdout):
    from gen import get_config, make_layer, QueryStream
    rates_all = []
    print("| r | active k | lite w | mean miss rate | std | min | max |", file=out)
    print("|---|---|---|---|---|---|---|", file=out)
    for r in (8, 16, 32, 64):
        for k in (128, 256, 512):
            for w in (4, 8):
                cfg = get_config("c2").with_(l=4096, r=r, k=k, w=w, C=k, n_heavy=k // 4,
                                             pool_mult=4, drift=drift)
                data = make_layer(cfg, 0, device="cuda")
                shape = _shape(cfg)
                lb = LayerBuffers(shape, data.A_K, data.K, data.V)
                plan = L.Plan(shape)
                qs = QueryStream(data)
                out_t = torch.empty((cfg.B, cfg.Hq, cfg.d), device="cuda")
                n_miss = torch.zeros((cfg.B, cfg.Hq), dtype=torch.int32, device="cuda")
                rates = []
                for step in range(1, warm + steps + 1):
                    q, q_hat = qs.next()
                    L.lrqk_decode_step(plan, shape, step, lb.struct, q_hat, q, out_t,
                                       L.LRQK_FETCH_DIRECT | (L.LRQK_SELECT_FRESH if step == 1 else 0),
                                       dict(n_miss=n_miss))
                    if step > warm:
                        rates.append(n_miss.clamp(min=0).sum().item() / (cfg.B * cfg.Hq * k))
                plan.close()
                rates = np.array(rates)
                rates_all.append(rates)
                print(f"| {r} | {k} | {w} | {rates.mean():.3f} | {rates.std():.3f} | "
                      f"{rates.min():.3f} | {rates.max():.3f} |", file=out)
    allr = np.concatenate(rates_all)
    print(f"\nAll cells and steps: mean {allr.mean():.3f}, std {allr.std():.3f} "
          f"({allr.size} step measurements).  Histogram (bin width 0.1):", file=out)
    hist, edges = np.histogram(allr, bins=10, range=(0.0, 1.0))
    for h, e in zip(hist, edges[:-1]):
        print(f"    {e:.1f}-{e + 0.1:.1f}  {h:5d}  {'#' * int(round(60 * h / max(hist.max(), 1)))}",
              file=out)


def no_hit_miss(steps: int, layers: int, out=sys.stdout):
    from gen import get_config, make_layer, QueryStream
    cfg = get_config("c3").with_(layers=layers)
    shape = _shape(cfg)
    lbs, streams = [], []
    for li in range(layers):
        data = make_layer(cfg, li, device="cuda")
        lbs.append(LayerBuffers(shape, data.A_K, data.K, data.V))
        streams.append(QueryStream(data))
    plan = L.Plan(shape)
    out_t = torch.empty((cfg.B, cfg.Hq, cfg.d), device="cuda")
    n_miss = torch.zeros((cfg.B, cfg.Hq), dtype=torch.int32, device="cuda")
    step_no = [0] * layers
    row_bytes = 2 * cfg.d * 2   # K and V row, bf16

    def run(reset: bool, n: int, timed: bool):
        qs = [streams[i % layers].next() for i in range(n)]
        torch.cuda.synchronize()
        fetched = 0
        t0 = time.perf_counter()
        for i in range(n):
            li = i % layers
            lb = lbs[li]
            if reset:
                L.lrqk_cache_init(shape, lb.slot_of, lb.token_of, lb.last_used)
            step_no[li] += 1
            L.lrqk_decode_step(plan, shape, step_no[li], lb.struct, qs[i][1], qs[i][0], out_t,
                               L.LRQK_FETCH_DIRECT | (L.LRQK_SELECT_FRESH if step_no[li] == 1 else 0),
                               None if timed else dict(n_miss=n_miss))
            if not timed:
                fetched += n_miss.clamp(min=0).sum().item()
        torch.cuda.synchronize()
        return (time.perf_counter() - t0) / n * 1e6, fetched / n

    run(False, 2 * layers, True)                      # warm the caches
    print("| variant | us per layer-step | rows fetched per step | MB over the host link per step |",
          file=out)
    print("|---|---|---|---|", file=out)
    for name, reset in (("default (hit/miss cache)", False), ("no hit/miss (cache emptied before "
                                                              "every step)", True)):
        _, rows = run(reset, steps, False)
        us, _ = run(reset, steps, True)
        print(f"| {name} | {us:.1f} | {rows:.0f} | {rows * row_bytes / 1e6:.2f} |", file=out)
        if reset:
            run(False, 2 * layers, True)
    plan.close()


def group_fetch_ab(steps: int, layers: int, out=sys.stdout):
    """Per-head fetch (LRQK_FETCH_DIRECT) against the fetch shared inside a KV group
    (LRQK_FETCH_GROUP) on workload 3, for query heads of a group that want the same tokens to
    different degrees (the generator's group_share): time per layer-step and rows / MB over the
    host link per step (DIRECT: every head's misses; GROUP: the union per KV head)."""
    from gen import get_config, make_layer, QueryStream
    print("| group_share | fetch | us per layer-step | rows missed per step | rows over the host "
          "link per step | MB over the link per step |", file=out)
    print("|---|---|---|---|---|---|", file=out)
    for share in (0.0, 0.5, 1.0):
        cfg = get_config("c3").with_(layers=layers, group_share=share)
        shape = _shape(cfg)
        row_bytes = 2 * cfg.d * 2
        for name, mode in (("per head (DIRECT)", L.LRQK_FETCH_DIRECT),
                           ("shared in the group (GROUP)", L.LRQK_FETCH_GROUP)):
            lbs, streams = [], []
            for li in range(layers):
                data = make_layer(cfg, li, device="cuda")
                lbs.append(LayerBuffers(shape, data.A_K, data.K, data.V))
                streams.append(QueryStream(data))
            plan = L.Plan(shape)
            out_t = torch.empty((cfg.B, cfg.Hq, cfg.d), device="cuda")
            n_miss = torch.zeros((cfg.B, cfg.Hq), dtype=torch.int32, device="cuda")
            link = torch.zeros((cfg.B, cfg.Hkv), dtype=torch.int32, device="cuda")
            step_no = [0] * layers

            def run(n, dbg):
                qs = [streams[i % layers].next() for i in range(n)]
                torch.cuda.synchronize()
                missed = linked = 0
                t0 = time.perf_counter()
                for i in range(n):
                    li = i % layers
                    step_no[li] += 1
                    flags = L.LRQK_SELECT_FRESH if step_no[li] == 1 else 0
                    L.lrqk_decode_step(plan, shape, step_no[li], lbs[li].struct, qs[i][1], qs[i][0],
                                       out_t, mode | flags,
                                       dict(n_miss=n_miss, link_rows=link) if dbg else None)
                    if dbg:
                        missed += n_miss.clamp(min=0).sum().item()
                        linked += link.sum().item()
                torch.cuda.synchronize()
                return (time.perf_counter() - t0) / n * 1e6, missed / n, linked / n

            run(2 * layers, False)                    # warm the caches
            _, missed, linked = run(steps, True)
            us, _, _ = run(steps, False)
            if mode == L.LRQK_FETCH_DIRECT:
                linked = missed                       # every head fetches its own misses
            print(f"| {share} | {name} | {us:.1f} | {missed:.0f} | {linked:.0f} | "
                  f"{linked * row_bytes / 1e6:.2f} |", file=out)
            plan.close()
            del lbs, streams


def attend_all_hit(steps: int, layers: int, out=sys.stdout):
    """Step a5 alone on caches that hold every selected row (lrqk_sparse_attend on the slots of
    each layer's last selection, layers in rotation): the attention kernels with nothing to
    fetch, e.g. to profile them."""
    from gen import get_config, make_layer, QueryStream
    cfg = get_config("c3").with_(layers=layers)
    shape = _shape(cfg)
    lbs, sel, qs = [], [], []
    plan = L.Plan(shape)
    out_t = torch.empty((cfg.B, cfg.Hq, cfg.d), device="cuda")
    for li in range(layers):
        data = make_layer(cfg, li, device="cuda")
        lb = LayerBuffers(shape, data.A_K, data.K, data.V)
        stream = QueryStream(data)
        sel_slot = torch.zeros((cfg.B, cfg.Hq, cfg.k), dtype=torch.int32, device="cuda")
        for step in range(1, 3):
            q, q_hat = stream.next()
            L.lrqk_decode_step(plan, shape, step, lb.struct, q_hat, q, out_t,
                               L.LRQK_FETCH_DIRECT | (L.LRQK_SELECT_FRESH if step == 1 else 0),
                               dict(sel_slot=sel_slot))
        lbs.append(lb)
        sel.append(sel_slot)
        qs.append(q)
    ws = torch.empty(L.lrqk_workspace_bytes(shape, L.LRQK_WS_ATTEND), dtype=torch.uint8,
                     device="cuda")
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(steps):
        li = i % layers
        L.lrqk_sparse_attend(shape, qs[li], lbs[li].cacheK, lbs[li].cacheV, sel[li], lbs[li].liteK,
                             lbs[li].liteV, out_t, ws)
    torch.cuda.synchronize()
    us = (time.perf_counter() - t0) / steps * 1e6
    nbytes = 2 * 2 * cfg.d * (cfg.B * cfg.Hq * cfg.k + cfg.B * cfg.Hkv * cfg.w)
    print(f"{steps} calls of lrqk_sparse_attend, {layers} layers in rotation: {us:.1f} us per call "
          f"(host loop included), {nbytes / 1e6:.1f} MB of K/V rows per call", file=out)
    plan.close()


def end_to_end(steps: int, out=sys.stdout):
    """Prefill factorisation, then Alg. 2 decode steps on the factors it produced; reports how
    much of the exact top-k of q K^T the proxy selects and how far the sparse attention output
    is from dense attention.  The exact scores and the dense attention are evaluation code
    (torch), not part of the path."""
    from gen import get_config, make_layer, QueryStream
    cfg = get_config("c2").with_(B=1, Hq=8, Hkv=2, l=8192, r=32, k=512, w=16, C=1024,
                                 n_heavy=128, pool_mult=4)
    dev = "cuda"
    data = make_layer(cfg, 0, device=dev)
    G, l, k, w, r, d = cfg.G, cfg.l, cfg.k, cfg.w, cfg.r, cfg.d
    # the prompt's queries: l draws of the same query process the decode steps continue
    qs = QueryStream(data)
    Q = torch.empty((cfg.B, cfg.Hq, l, d), device=dev, dtype=data.K.dtype)
    for i in range(l):
        Q[:, :, i, :] = qs.next()[0].to(data.K.dtype)
    gen = torch.Generator(device=dev).manual_seed(1234)
    n_new = steps
    shape = _shape(cfg, l_cap=l + n_new)
    A_Q = torch.randn((cfg.B, cfg.Hq, l, r), generator=gen, device=dev)
    A_K0 = torch.randn((cfg.B, cfg.Hkv, l, r), generator=gen, device=dev)
    lb = LayerBuffers(shape, A_K0, data.K, data.V)       # A_K is overwritten by the prefill
    B_Q = torch.empty((cfg.B, cfg.Hq, r, d), device=dev)
    B_K = torch.empty((cfg.B, cfg.Hkv, r, d), device=dev)
    ws = torch.empty(L.lrqk_workspace_bytes(shape, L.LRQK_WS_PREFILL), dtype=torch.uint8,
                     device=dev)
    L.lrqk_prefill_factorize(shape, Q, data.K, A_Q, lb.A_K, B_Q, B_K, 1.0, 1.0, 2, ws)
    Kf = data.K.float()
    rel_fit = ((lb.A_K[:, :, :l] @ B_K - Kf).norm() / Kf.norm()).item()
    print(f"prefill: |K - A_K B_K| / |K| = {rel_fit:.3f} (rank {r}, keys = rank-{r} part + "
          f"{cfg.noise} noise)", file=out)
    plan = L.Plan(shape.with_l(l + n_new))
    ws_u = torch.empty(L.lrqk_workspace_bytes(shape.with_l(l + n_new), L.LRQK_WS_UPDATE),
                       dtype=torch.uint8, device=dev)
    i32 = dict(dtype=torch.int32, device=dev)
    sel_idx = torch.zeros((cfg.B, cfg.Hq, k), **i32)
    sel_slot = torch.full((cfg.B, cfg.Hq, k), -1, **i32)
    q_hat = torch.zeros((cfg.B, cfg.Hq, r), device=dev)
    k_hat = torch.zeros((cfg.B, cfg.Hkv, r), device=dev)
    out_t = torch.empty((cfg.B, cfg.Hq, d), device=dev)
    Kall = torch.zeros((cfg.B, cfg.Hkv, l + n_new, d), device=dev)
    Vall = torch.zeros_like(Kall)
    Kall[:, :, :l], Vall[:, :, :l] = Kf, data.V.float()
    recalls, errs, mass = [], [], []
    lcur = l
    for t in range(1, n_new + 1):
        q = qs.next()[0]
        k_new = torch.einsum("bhr,bhrd->bhd",
                             torch.randn((cfg.B, cfg.Hkv, r), generator=gen, device=dev),
                             data.Bmat).to(data.K.dtype)
        v_new = torch.randn((cfg.B, cfg.Hkv, d), generator=gen, device=dev).to(data.K.dtype)
        shp = shape.with_l(lcur)
        # the first step has no previous selection: lambda_d2 = 0 leaves Omega out
        lam2 = 0.0 if t == 1 else 1.0
        L.lrqk_factor_update(shp, lb.struct, sel_idx, sel_slot, q, k_new, B_Q, B_K, 1.0, lam2, 2,
                             q_hat, k_hat, ws_u)
        L.lrqk_append_token(shp, lb.struct, k_hat, k_new, v_new)
        Kall[:, :, lcur], Vall[:, :, lcur] = k_new.float(), v_new.float()
        lcur += 1
        L.lrqk_decode_step(plan, shape.with_l(lcur), t, lb.struct, q_hat, q, out_t,
                           L.LRQK_FETCH_DIRECT | (L.LRQK_SELECT_FRESH if t == 1 else 0),
                           dict(sel_idx=sel_idx, sel_slot=sel_slot))
        # evaluation: exact scores, exact top-k over [0, l - w), dense attention
        Krep = Kall[:, :, :lcur].repeat_interleave(G, dim=1)
        Vrep = Vall[:, :, :lcur].repeat_interleave(G, dim=1)
        s = torch.einsum("bhd,bhld->bhl", q, Krep)
        top = s[:, :, :lcur - w].topk(k, dim=-1).indices
        hit = torch.zeros_like(s, dtype=torch.bool)
        hit.scatter_(2, sel_idx.long(), True)
        recalls.append(hit.gather(2, top).float().mean().item())
        p = torch.softmax(s * cfg.scale, dim=-1)
        dense = torch.einsum("bhl,bhld->bhd", p, Vrep)
        hit[:, :, lcur - w:] = True
        mass.append((p * hit).sum(-1).mean().item())
        errs.append(((out_t - dense).norm() / dense.norm()).item())
    plan.close()
    print("| steps | recall of the exact top-k | attention mass covered by the k + w rows | "
          "|out - dense| / |dense| |", file=out)
    print("|---|---|---|---|", file=out)
    for name, sl in (("step 1 (no previous selection)", slice(0, 1)),
                     (f"steps 2..{n_new}", slice(1, None))):
        print(f"| {name} | {np.mean(recalls[sl]):.3f} | {np.mean(mass[sl]):.3f} | "
              f"{np.mean(errs[sl]):.3f} |", file=out)


def main():
    ap = argparse.ArgumentParser(description=__doc__.split("\n")[0])
    ap.add_argument("--grid", action="store_true")
    ap.add_argument("--no-hit-miss", action="store_true")
    ap.add_argument("--end-to-end", action="store_true")
    ap.add_argument("--group-fetch", action="store_true")
    ap.add_argument("--attend-all-hit", action="store_true")
    ap.add_argument("--steps", type=int, default=64)
    ap.add_argument("--warm", type=int, default=8)
    ap.add_argument("--layers", type=int, default=8)
    ap.add_argument("--drift", type=float, default=0.1,
                    help="fraction of the heavy window the planted query direction moves per "
                         "step in the grid (the generator's knob for the miss rate)")
    args = ap.parse_args()
    if not torch.cuda.is_available():
        sys.exit("ablation: needs a GPU")
    both = not (args.grid or args.no_hit_miss or args.end_to_end or args.group_fetch
                or args.attend_all_hit)
    if args.attend_all_hit:
        attend_all_hit(args.steps, args.layers)
    if args.grid or both:
        print("## Miss-rate grid (Sec. 5.3), l = 4096, 32 q / 8 kv heads, cache of k slots, "
              f"query drift {args.drift} of the heavy window per step\n")
        miss_rate_grid(args.steps, args.warm, args.drift)
    if args.no_hit_miss or both:
        print("\n## Hit/miss ablation (App. C.2), workload 3 (l = 131072, r = 32, k = 2048), "
              f"{args.layers} layers rotated\n")
        no_hit_miss(args.steps, args.layers)
    if args.group_fetch or both:
        print("\n## Fetch per head against fetch shared inside a KV group, workload 3, "
              f"{args.layers} layers rotated\n")
        group_fetch_ab(args.steps, args.layers)
    if args.end_to_end or both:
        print("\n## Prefill factorisation, then Alg. 2 decode steps on its factors: 8 q / 2 kv "
              "heads, l = 8192, r = 32, k = 512, w = 16\n")
        end_to_end(min(args.steps, 32))


if __name__ == "__main__":
    main()

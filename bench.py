#!/usr/bin/env python3
"""Benchmark of one worker's Kimad+ compression step on one MI355X.

A "step" is one pass of the whole hot path over one synthetic gradient set that is already
resident in HBM: kimad_profile -> kimad_allocate -> kimad_compress_ef (thresholds reused).
Prints ONE JSON line.  The metric is gradient GB/s = 4 * d / t_step.

The estimator h is restored from a device copy before every step, outside the timed
intervals: every step then compresses the same x = g - h, as the first round of training
would.  Each step is timed with a pair of events on the stream the library launches on;
`ms_per_step` is the mean of those intervals, `wall_ms_per_step` the host clock around all
K steps including the restores.
"""
from __future__ import annotations

import argparse
import json
import re
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0           # MI355X HBM3E, published peak

STREAMING_KERNELS = ("k_main", "k_hist1", "k_hist2", "k_candidates")


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--workload", default="gpt2", choices=["mlp", "resnet18", "resnet50", "gpt2", "llama"])
    ap.add_argument("--D", type=int, default=None, help="cost discretisation factor (default: the workload's)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--also-D", type=int, default=4096,
                    help="also time the step with this discretisation factor, reported beside the headline (0 = skip)")
    ap.add_argument("--block-min", type=int, default=0,
                    help="also time the step with tensors below this many elements merged into blocks (Section 6 remark)")
    ap.add_argument("--compare-allocators", action="store_true",
                    help="also report the total error of Kimad+, uniform-ratio Kimad and whole-model TopK (Section 4.3)")
    ap.add_argument("--single-draw", action="store_true",
                    help="repeat one gradient draw instead of alternating between two")
    ap.add_argument("--no-overlap", action="store_true",
                    help="skip the measurement of the allocation overlapped with the next round (Section 5 remark)")
    ap.add_argument("--no-settled", action="store_true",
                    help="skip the extra steps timed with the last-level cache emptied first (inputs_settled_in_hbm)")
    ap.add_argument("--server-workers", type=int, default=4,
                    help="workers of the server-step measurement reported beside the headline (0 = skip)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build measures one worker on one GPU; --gpus must be 1 "
              "(one worker's step has no exchange between workers: M GPUs run M independent instances)", file=sys.stderr)
        return 2

    import numpy as np
    import torch
    import kimad_synth as ks
    import paper_2312_08053_amd as kimad

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        return 3
    kimad.lib()   # fails loudly when the HIP library is missing

    t0 = time.time()
    kw = {} if args.D is None else {"D": args.D}
    work = ks.make_workload(args.workload, **kw)
    t_gen = time.time() - t0
    d, L, J = work.d, work.L, len(work.ratios)
    g = torch.from_numpy(work.g).cuda()
    h = torch.from_numpy(work.h).cuda()
    h0 = h.clone()
    # Successive rounds see different gradients: from its second profile on the plan predicts from the previous
    # round's histogram, which a repeated input would make a perfect prediction.  The steps alternate between two
    # draws of the set (same per-layer scales, independent values), copied into g outside the timed intervals.
    draws = [g.clone()]
    if not args.single_draw and work.name in ("gpt2", "llama"):
        kw2 = dict(kw, step=1)
        if work.name == "gpt2":
            kw2["scales_of_step"] = 0
        t0 = time.time()
        draws.append(torch.from_numpy(ks.make_workload(args.workload, **kw2).g).cuda())
        t_gen += time.time() - t0
    nload = [0]

    def load_round():
        g.copy_(draws[nload[0] % len(draws)])
        h.copy_(h0)
        nload[0] += 1
    plan = kimad.Plan(g, h, work.sizes.tolist(), work.ratios.tolist(), pair_bytes=work.pair_bytes,
                      D=work.cost_units_D, max_budget_bytes=work.budget_bytes,
                      capacity_pairs=work.budget_bytes // work.pair_bytes + 1)
    stream = torch.cuda.current_stream()

    def one_step():
        plan.step(work.budget_bytes)

    sumKs = []
    for k in range(max(args.warmup, len(draws))):
        load_round()
        one_step()
        if k < len(draws):
            sumKs.append(int(plan.offsets[-1].item()))
    torch.cuda.synchronize()
    status = plan.status.cpu().tolist()
    if status != [0, 0]:
        print(f"bench.py: step failed with device status {status}", file=sys.stderr)
        return 4
    sumK = int(round(float(np.mean(sumKs))))

    # ---- timed region: K steps, each bracketed by events; h restored between the intervals
    starts = [torch.cuda.Event(enable_timing=True) for _ in range(args.steps)]
    ends = [torch.cuda.Event(enable_timing=True) for _ in range(args.steps)]
    torch.cuda.synchronize()
    w0 = time.perf_counter()
    for k in range(args.steps):
        load_round()
        starts[k].record(stream)
        one_step()
        ends[k].record(stream)
    torch.cuda.synchronize()
    wall_ms = (time.perf_counter() - w0) * 1e3 / args.steps
    per_step = [starts[k].elapsed_time(ends[k]) for k in range(args.steps)]
    ms = float(np.mean(per_step))

    # ---- the metric's own composition, timed directly: kimad_profile + kimad_compress_ef(thresholds reused) with
    # the sizes K fixed by an allocation done beforehand (outside the intervals), and each call on its own
    def timed_calls(what, reps):
        ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(reps)]
        for a, b in ev:
            load_round()
            if what == "compress":                        # its thresholds come from a profile outside the interval
                plan.profile(budget_hint_bytes=work.budget_bytes)
            a.record(stream)
            if what in ("profile", "profile+compress"):
                plan.profile(budget_hint_bytes=work.budget_bytes)
            if what == "allocate":
                plan.allocate(work.budget_bytes)
            if what in ("compress", "profile+compress"):
                plan.compress_ef(reuse_profile=True)
            b.record(stream)
        torch.cuda.synchronize()
        return float(np.mean([a.elapsed_time(b) for a, b in ev]))

    load_round()
    plan.profile(budget_hint_bytes=work.budget_bytes)
    plan.allocate(work.budget_bytes)                      # K, offsets stay in the plan's tensors from here on
    torch.cuda.synchronize()
    call_ms = {name: timed_calls(name, args.steps) for name in ("profile+compress", "profile", "allocate", "compress")}
    if plan.status.cpu().tolist() != [0, 0]:
        print(f"bench.py: separate calls failed with device status {plan.status.cpu().tolist()}", file=sys.stderr)
        return 4

    # ---- the same steps again with an event after every kernel: per-kernel durations
    plan.set_timing(True)
    agg: dict = {}
    order = []
    for k in range(args.steps):
        load_round()
        one_step()
        for name, t in plan.get_timings():
            if name not in agg:
                agg[name] = []
                order.append(name)
            agg[name].append(t)
    plan.set_timing(False)
    kern = {n: {"launches_per_step": len(v) / args.steps, "avg_ms": float(np.mean(v)),
                "ms_per_step": float(np.sum(v)) / args.steps} for n, v in agg.items()}

    # ---- beside it: the same steps with the inputs settled in HBM.  The copies that load a round leave their last
    # 256 MB in the last-level cache as dirty lines, which are written back while the streaming pass reads (as
    # after a backward pass that has just written the gradient: the headline keeps that).  Here 1 GiB of unrelated
    # memory is read between the copies and the interval, so that g and h come from HBM and nothing is pending.
    settled_dom, settled_ms = [], 0.0
    if not args.no_settled:
        settle = torch.empty(1 << 28, dtype=torch.float32, device="cuda").fill_(1.0)
        s_start = [torch.cuda.Event(enable_timing=True) for _ in range(args.steps)]
        s_end = [torch.cuda.Event(enable_timing=True) for _ in range(args.steps)]
        for k in range(args.steps):
            load_round()
            settle.sum()
            s_start[k].record(stream)
            one_step()
            s_end[k].record(stream)
        torch.cuda.synchronize()
        settled_ms = float(np.mean([a.elapsed_time(b) for a, b in zip(s_start, s_end)]))
        plan.set_timing(True)
        for k in range(args.steps):
            load_round()
            settle.sum()
            one_step()
            settled_dom += [t for name, t in plan.get_timings() if name == "k_main"]
        plan.set_timing(False)
        del settle
    stage_ms = {"profile": 0.0, "allocate": 0.0, "compress": 0.0}
    for n, v in kern.items():
        if n.startswith("k_dp"):
            stage_ms["allocate"] += v["ms_per_step"]
        elif n in ("k_sample", "k_predict", "k_main", "k_scan1x", "k_hist2c", "k_hist1", "k_scan1", "k_hist2",
                   "k_scan2", "k_hist3p", "k_scan3p", "k_small_profile"):
            stage_ms["profile"] += v["ms_per_step"]
        elif n != "k_zero16":
            stage_ms["compress"] += v["ms_per_step"]

    d_big = int(sum(int(n) for n in work.sizes if int(n) > 8192))
    # algorithmic bytes of a streaming kernel: it must read g and h of the tiled layers once
    alg_bytes = {"k_main": 8 * d_big, "k_hist1": 8 * d_big, "k_hist2": 8 * d_big, "k_candidates": 8 * d_big}
    dom = max((n for n in STREAMING_KERNELS if n in kern), key=lambda n: kern[n]["ms_per_step"])
    ach = alg_bytes[dom] / (kern[dom]["avg_ms"] * 1e-3) / 1e9
    # HBM bytes per launch from rocprofv3 counter runs, recorded under profiles/ (None if there is no record for
    # this kernel and workload)
    traffic = None
    rec = os.path.join(ROOT, "profiles", f"hbm_traffic_{dom}_{work.name}.txt")
    if os.path.exists(rec):
        with open(rec) as f:
            m = re.search(r"traffic_bytes_per_launch\s*=\s*(\d+)", f.read())
        traffic = float(m.group(1)) if m else None
    roofline = {"bound": "hbm", "kernel": dom, "achieved": round(ach, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s",
                "frac": round(ach / HBM_PEAK_GBS, 4), "traffic": traffic,
                "algorithmic_bytes_per_launch": alg_bytes[dom],
                "avg_launch_ms": round(kern[dom]["avg_ms"], 5)}

    bytes_min = 8 * d + (work.pair_bytes + 4) * sumK + 8 * L * J + 8 * (L + 1)
    value = 4.0 * d / (ms * 1e-3) / 1e9
    t_no_alloc = call_ms["profile+compress"]               # measured: the two calls back to back, K fixed beforehand
    out = {
        "metric": "gradient GB/s compressed per step (profile+select+EF)",
        "value": round(value, 2), "unit": "GB/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms, 4), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32", "data": "synthetic",
        "config": {"workload": f"{work.name}-shaped gradient set ({L} tensors, {d} elements)",
                   "ratios": J, "budget_bytes": work.budget_bytes, "cost_units_D": work.cost_units_D,
                   "also_timed_cost_units_D": args.also_D if args.also_D != work.cost_units_D else 0,
                   "payload_pairs": sumK, "gradient_draws": len(draws),
                   "prediction": "previous round's histogram (sampled on a plan's first profile)", "estimator": "zero" if not work.h.any() else "nonzero",
                   "tile_elems": None},
        "wall_ms_per_step": round(wall_ms, 4),
        "min_ms_per_step": round(float(np.min(per_step)), 4),
        "median_ms_per_step": round(float(np.median(per_step)), 4),
        "path_roofline": {"bytes_min": bytes_min, "frac_of_hbm_peak": round(bytes_min / (ms * 1e-3) / 1e9 / HBM_PEAK_GBS, 4),
                          "ms_without_allocate": round(t_no_alloc, 4),
                          "frac_without_allocate": round(bytes_min / (t_no_alloc * 1e-3) / 1e9 / HBM_PEAK_GBS, 4),
                          "gradient_GBs_without_allocate": round(4.0 * d / (t_no_alloc * 1e-3) / 1e9, 2)},
        "call_ms": {k: round(v, 4) for k, v in call_ms.items()},
        "stage_ms_from_kernel_events": {k: round(v, 4) for k, v in stage_ms.items()},
        "kernels": {n: {k: round(v, 5) for k, v in kern[n].items()} for n in order},
        "roofline": roofline,
        "allocation_band": plan.allocate_diagnostics(),
        "input_generation_s": round(t_gen, 1),
    }
    if settled_dom and dom == "k_main":
        t_dom = float(np.mean(settled_dom))
        out["inputs_settled_in_hbm"] = {
            "what": "1 GiB of unrelated memory read between the loading copies and each interval",
            "ms_per_step": round(settled_ms, 4),
            "frac_of_hbm_peak": round(bytes_min / (settled_ms * 1e-3) / 1e9 / HBM_PEAK_GBS, 4),
            "k_main_avg_launch_ms": round(t_dom, 5),
            "k_main_frac": round(alg_bytes[dom] / (t_dom * 1e-3) / 1e9 / HBM_PEAK_GBS, 4)}

    # ---- beside the headline: the paper's remark that the allocation "can be overlapped with communication"
    # (Section 5): round k is compressed with the sizes that round k-1's table chose, and round k's allocation
    # runs on a second stream beside that compression and the next round's profile.  Error table and K are double
    # buffered; the profile leaves 8 compute units to the second stream.  Not part of `value`: the sizes are one
    # round old, a variant of the method, not the same result sooner.
    if not args.no_overlap:
        oplan = kimad.Plan(g, h, work.sizes.tolist(), work.ratios.tolist(), pair_bytes=work.pair_bytes,
                           D=work.cost_units_D, max_budget_bytes=work.budget_bytes,
                           capacity_pairs=work.budget_bytes // work.pair_bytes + 1,
                           max_workgroups=max(1, torch.cuda.get_device_properties(0).multi_processor_count - 8))
        side = torch.cuda.Stream()
        errs = [torch.empty_like(oplan.err_table) for _ in range(2)]
        Ks = [torch.empty_like(oplan.K) for _ in range(2)]
        offs = [torch.empty_like(oplan.offsets) for _ in range(2)]
        js = [torch.empty_like(oplan.j) for _ in range(2)]
        ast = torch.zeros(2, dtype=torch.int32, device="cuda")
        ev_prof = [torch.cuda.Event() for _ in range(2)]
        ev_alloc = [torch.cuda.Event() for _ in range(2)]
        # round -1: a table and sizes to start from
        oplan.profile(errs[1], budget_hint_bytes=work.budget_bytes)
        kimad.kimad_allocate(oplan.handle, errs[1], work.budget_bytes, js[1], Ks[1], offs[1], ast[1:2])
        ev_alloc[1].record(stream)
        rounds = args.steps + args.warmup
        o_start = [torch.cuda.Event(enable_timing=True) for _ in range(rounds)]
        o_end = [torch.cuda.Event(enable_timing=True) for _ in range(rounds)]
        for k in range(rounds):
            cur, prev = k % 2, (k + 1) % 2
            load_round()
            o_start[k].record(stream)
            oplan.profile(errs[cur], budget_hint_bytes=work.budget_bytes)
            ev_prof[cur].record(stream)
            side.wait_event(ev_prof[cur])
            with torch.cuda.stream(side):
                kimad.kimad_allocate(oplan.handle, errs[cur], work.budget_bytes, js[cur], Ks[cur], offs[cur], ast[cur:cur + 1])
                ev_alloc[cur].record(side)
            stream.wait_event(ev_alloc[prev])
            oplan.compress_ef(Ks[prev], offs[prev], reuse_profile=True)
            o_end[k].record(stream)
            # the next round's profile overwrites errs[prev], which round k-1's allocation has long read
        torch.cuda.synchronize()
        oms = float(np.mean([o_start[k].elapsed_time(o_end[k]) for k in range(args.warmup, rounds)]))
        out["allocation_overlapped"] = {"what": "sizes from the previous round's table; allocation on a second stream",
                                        "ms_per_round_profile_to_payload": round(oms, 4),
                                        "status": ast.cpu().tolist() + oplan.status[1:2].cpu().tolist(),
                                        "gradient_GBs": round(4.0 * d / (oms * 1e-3) / 1e9, 2)}
        del oplan

    # ---- beside the headline: the server's step of the same round (decode M payloads into M estimators,
    # x <- x - gamma * sum_m w_m u_hat_m), timed with events on the same stream.  Not part of `value`.
    if args.server_workers > 0:
        M = args.server_workers
        hats = [h0.clone() for _ in range(M)]
        xm = torch.zeros(d, dtype=torch.float32, device="cuda")
        starts_dev = torch.from_numpy(np.asarray(work.starts, dtype=np.int64)).cuda()
        pl = [(plan.idx, plan.val, plan.offsets)] * M
        wts = [1.0 / M] * M

        def timed(fn, reps=10):
            for _ in range(2):
                fn()
            ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(reps)]
            for a, b in ev:
                a.record(stream); fn(); b.record(stream)
            torch.cuda.synchronize()
            return float(np.mean([a.elapsed_time(b) for a, b in ev]))

        sstat = torch.zeros(M, dtype=torch.int32, device="cuda")
        t_dec = timed(lambda: kimad.kimad_server_apply(pl, hats, wts, starts_dev, d, None, 0.0, status_out=sstat))
        t_all = timed(lambda: kimad.kimad_server_apply(pl, hats, wts, starts_dev, d, xm, 1e-3, status_out=sstat))
        assert sstat.cpu().tolist() == [0] * M
        t_step = max(t_all - t_dec, 1e-6)
        step_bytes = 4 * (M + 2) * d
        out["server_step"] = {"workers": M, "decode_ms": round(t_dec, 4), "model_step_ms": round(t_step, 4),
                              "model_step_algorithmic_bytes": step_bytes,
                              "model_step_GBs": round(step_bytes / (t_step * 1e-3) / 1e9, 1),
                              "model_step_frac_of_hbm_peak": round(step_bytes / (t_step * 1e-3) / 1e9 / HBM_PEAK_GBS, 4)}
        del hats, xm

    if args.also_D > 0 and args.also_D != work.cost_units_D:
        # beside the headline: the same step with another discretisation factor of the allocation (rows of
        # also_D + 1 cost cells).  Not part of `value`.
        dplan = kimad.Plan(g, h, work.sizes.tolist(), work.ratios.tolist(), pair_bytes=work.pair_bytes, D=args.also_D,
                           max_budget_bytes=work.budget_bytes, capacity_pairs=work.budget_bytes // work.pair_bytes + 1)
        for _ in range(max(2, args.warmup)):
            load_round()
            dplan.step(work.budget_bytes)
        torch.cuda.synchronize()
        ds_ = [torch.cuda.Event(enable_timing=True) for _ in range(args.steps)]
        de_ = [torch.cuda.Event(enable_timing=True) for _ in range(args.steps)]
        for k in range(args.steps):
            load_round()
            ds_[k].record(stream)
            dplan.step(work.budget_bytes)
            de_[k].record(stream)
        torch.cuda.synchronize()
        dms = float(np.mean([ds_[k].elapsed_time(de_[k]) for k in range(args.steps)]))
        out["other_D"] = {"cost_units_D": args.also_D, "status": dplan.status.cpu().tolist(), "ms_per_step": round(dms, 4),
                          "gradient_GBs": round(4.0 * d / (dms * 1e-3) / 1e9, 2),
                          "payload_pairs": int(dplan.offsets[-1].item()),
                          "allocation_band": dplan.allocate_diagnostics()}
        del dplan

    if args.block_min > 0:
        # beside the headline: block granularity (one block = a run of consecutive tensors).  Not part of `value`.
        from paper_2312_08053_amd.blocks import merge_small
        bsizes = merge_small(work.sizes.tolist(), args.block_min)
        bplan = kimad.Plan(g, h, bsizes, work.ratios.tolist(), pair_bytes=work.pair_bytes, D=work.cost_units_D,
                           max_budget_bytes=work.budget_bytes, capacity_pairs=work.budget_bytes // work.pair_bytes + 1)
        for _ in range(max(2, args.warmup)):
            load_round()
            bplan.step(work.budget_bytes)
        torch.cuda.synchronize()
        bs = [torch.cuda.Event(enable_timing=True) for _ in range(args.steps)]
        be = [torch.cuda.Event(enable_timing=True) for _ in range(args.steps)]
        for k in range(args.steps):
            load_round()
            bs[k].record(stream)
            bplan.step(work.budget_bytes)
            be[k].record(stream)
        torch.cuda.synchronize()
        bms = float(np.mean([bs[k].elapsed_time(be[k]) for k in range(args.steps)]))
        out["blocked"] = {"min_elems": args.block_min, "blocks": len(bsizes), "status": bplan.status.cpu().tolist(),
                          "ms_per_step": round(bms, 4), "gradient_GBs": round(4.0 * d / (bms * 1e-3) / 1e9, 2),
                          "payload_pairs": int(bplan.offsets[-1].item())}
        del bplan

    if args.compare_allocators:
        from paper_2312_08053_amd.baselines import allocator_errors
        g.copy_(draws[0])
        h.copy_(h0)
        out["allocator_comparison"] = allocator_errors(g, h, work.sizes.tolist(), work.ratios.tolist(), work.budget_bytes,
                                                       work.pair_bytes, work.cost_units_D)

    # ---- the CPU oracle on a bounded sample of the same workload (rank 0, reported baseline)
    if not args.no_cpu_baseline:
        from oracle import kimad_oracle as ko
        gL, hL = work.layer_views(work.g), work.layer_views(work.h)
        if work.name == "llama":
            sel = list(range(1, 1 + 9 * 2))        # 9 tensors per block, after the embedding
            what = "first 2 transformer blocks"
        else:
            sel = list(range(L))
            what = "the benchmark's own inputs, all tensors"
        gs, hs = [gL[i] for i in sel], [hL[i].copy() for i in sel]
        ds = int(sum(len(x) for x in gs))
        budget_s = work.budget_bytes if ds == d else int(work.budget_bytes * ds / d)
        c0 = time.perf_counter()
        res = ko.step(gs, hs, work.ratios, budget_s, work.pair_bytes, work.cost_units_D)
        cpu_s = time.perf_counter() - c0
        out["cpu_baseline"] = {"value": round(4.0 * ds / cpu_s / 1e9, 5), "unit": "GB/s", "cores": 1,
                               "kind": "oracle", "seconds": round(cpu_s, 2),
                               "sample": f"{what}: {len(sel)} tensors, {ds} elements, budget {budget_s} B"
                                         f"{'' if ds == d else ' (scaled)'}, one step; numpy sorts on one thread; "
                                         f"status {res['status']}"}
    print(json.dumps(out))
    return 0


if __name__ == "__main__":
    sys.exit(main())

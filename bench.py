#!/usr/bin/env python3
"""Benchmark of the shared-pool MoE layer, forward + backward, on one MI355X.

One step = forward of all L layers that share the pool (route, permute, expert FFN, combine),
the pool auxiliary loss, and the backward of all L layers (combine-bwd, expert dgrad, dispatch-bwd,
router-bwd) with the pool weight gradient.  Inputs are synthetic, drawn on the device before the
timed region.  Prints ONE JSON line.

  python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload C5] [--wgrad pool|layer]
                  [--recompute] [--lagged]
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0     # MI355X dense bf16 MFMA
PEAK_HBM_GBS = 8000.0         # MI355X HBM3E

# HBM bytes per gemm_xw launch from rocprofv3 counter runs of this command (FETCH_SIZE x 2.0 + WRITE_SIZE x 1.0,
# the factors of the 1 GiB copy below), averaged over the four expert-FFN launches of a layer.  A run of
# bench.py cannot collect counters itself: the value is the one recorded in the profile named below.
PROFILED_XW_TRAFFIC_BYTES = {"C5": 5.5e9}
PROFILED_XW_TRAFFIC_SOURCE = ("profiles/gemm_counters_C5.txt: rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs of "
                              "`bench.py --workload C5`, recorded there; not measured in this run")


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=5)
    ap.add_argument("--warmup", type=int, default=2)
    ap.add_argument("--workload", default="C5")
    ap.add_argument("--wgrad", default="pool", choices=["pool", "layer"])
    ap.add_argument("--recompute", action="store_true",
                    help="keep one shared pair of A/B buffers and rebuild them before each layer's backward")
    ap.add_argument("--lagged", action="store_true", help="one-step-behind usage statistic across steps")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--step-only", action="store_true",
                    help="whole steps only: no CPU baseline, no side measurements (analysis entry points, "
                         "forward-only dispatch comparison), no other workloads; for profiler runs")
    ap.add_argument("--oracle-tokens", type=int, default=4096)
    ap.add_argument("--other-workloads", default="C2,C3,C4,C4z",
                    help="comma-separated workloads summarised after the headline one ('' for none)")
    ap.add_argument("--other-steps", type=int, default=3)
    a = ap.parse_args()
    if a.step_only:
        a.no_cpu_baseline = True
        a.other_workloads = ""
    return a


def cpu_baseline(w, xs0, wr0, g0, wg, wu, wd, n_tok, n_tok_1thread=512):
    """The oracle as it stands, timed on the host: one layer, the first n_tok tokens, fwd + bwd, with the BLAS
    threads numpy has by default; and the same on the first n_tok_1thread tokens with one thread."""
    import numpy as np
    from oracle import unipool_oracle as O
    try:
        from threadpoolctl import threadpool_info, threadpool_limits
        cores = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
    except Exception:
        threadpool_limits = None
        cores = 1
    wr = wr0.float().cpu().numpy()
    wg_h, wu_h, wd_h = (t.float().cpu().numpy() for t in (wg, wu, wd))

    def run(n):
        x = xs0[:n].float().cpu().numpy()
        g = g0[:n].float().cpu().numpy()
        t0 = time.perf_counter()
        fw = O.moe_layer_fwd(x, wr, wg_h, wu_h, wd_h, w.k, w.sigma, w.c, w.eps)
        _, _, _, coef = O.pool_aux_loss(fw["counts"][None], fw["psum"][None], n, w.k, w.alpha)
        O.moe_layer_bwd(fw, x, wr, wg_h, wu_h, wd_h, g, coef, w.k, w.sigma, w.c, w.eps)
        return time.perf_counter() - t0
    dt = run(n_tok)
    out = {"value": n_tok / dt, "unit": "tokens/s", "cores": int(cores), "kind": "oracle",
           "sample": "one layer, first %d tokens of %s, fwd+bwd in float64 numpy, %.1f s; work is linear "
                     "in tokens at fixed shape" % (n_tok, w.name, dt)}
    if threadpool_limits is not None and n_tok_1thread > 0:
        with threadpool_limits(limits=1):
            dt1 = run(n_tok_1thread)
        out["value_1_thread"] = n_tok_1thread / dt1
        out["sample_1_thread"] = "the same on the first %d tokens with one BLAS thread, %.1f s" % (n_tok_1thread, dt1)
    return out


def roofline_of(w, a, ps, agg, steps):
    """Per-entry-point figures of one workload from the HIP-event times in agg."""
    S = w.S
    gemm_flops_third = 6.0 * S * w.d * w.f            # one of fwd / dgrad / wgrad, per layer
    n_per_layer = 5 if a.recompute else 4             # gate-up, down, dH, dX (and gate-up again) launches
    n_xw = n_per_layer * w.L * steps
    t_xw_ms = (sum(agg.get("expert_ffn_fwd", [])) + sum(agg.get("expert_ffn_bwd", []))
               + sum(agg.get("expert_ffn_recompute", [])))
    xw_flops_per_launch = (2.0 * gemm_flops_third + (4.0 * S * w.d * w.f if a.recompute else 0.0)) / n_per_layer
    avg_xw_ms = t_xw_ms / n_xw
    xw_tflops = xw_flops_per_launch / (avg_xw_ms * 1e-3) / 1e12
    t_wg_ms = sum(agg.get("expert_wgrad", []))
    gemm_flops_layer = 3.0 * gemm_flops_third + (4.0 * S * w.d * w.f if a.recompute else 0.0)
    all_gemm_tflops = gemm_flops_layer * w.L * steps / ((t_xw_ms + t_wg_ms) * 1e-3) / 1e12 \
        if a.wgrad == "pool" else gemm_flops_layer * w.L * steps / (t_xw_ms * 1e-3) / 1e12
    act_b = 2 if w.dtype == "bf16" else 4

    def hbm(name, nbytes):
        ts = agg.get(name, [])
        if not ts:
            return None
        avg = sum(ts) / len(ts)
        return {"GB/s": nbytes / (avg * 1e-3) / 1e9, "frac": nbytes / (avg * 1e-3) / 1e9 / PEAK_HBM_GBS,
                "avg_ms": avg, "algorithmic_bytes": nbytes}
    others = {
        "grouped_gemm_all": {"TFLOP/s": all_gemm_tflops, "frac": all_gemm_tflops / PEAK_BF16_TFLOPS,
                             "wgrad": a.wgrad, "gemm_ms_per_step": (t_xw_ms + t_wg_ms) / steps},
        "route": hbm("route", act_b * w.T * w.d + 4 * w.T * w.E + 8 * w.T * w.k),
        "permute": hbm("permute", act_b * w.T * w.d + act_b * S * w.d + 12 * S),
        "combine": hbm("combine", act_b * S * w.d + act_b * w.T * w.d + 8 * S),
        "combine_bwd": hbm("combine_bwd", act_b * w.T * w.d + 2 * act_b * S * w.d + 12 * S),
        # x and logits read, dx read and written (the expert path's dx is already there), router gradient written
        "route_bwd": hbm("route_bwd", 3 * act_b * w.T * w.d + 4 * w.T * w.E + 12 * S + 4 * w.E * w.d),
    }
    if a.wgrad == "pool" and t_wg_ms > 0:
        wg_tflops = gemm_flops_third * w.L * steps / (t_wg_ms * 1e-3) / 1e12
        others["wgrad_pool"] = {"TFLOP/s": wg_tflops, "frac": wg_tflops / PEAK_BF16_TFLOPS}
    # The floor of the average gemm_xw launch: the longer of its MFMA time and its HBM time at the published
    # peaks (algorithmic bytes: weights once, activations in and out).  Below the ridge of 312 FLOP per byte
    # the HBM time is the longer one even though the kernel is a contraction.
    xw_bytes_per_launch = (12.0 * w.E * w.d * w.f + 8.0 * S * w.d + 20.0 * S * w.f) / 4.0
    t_mfma_ms = xw_flops_per_launch / (PEAK_BF16_TFLOPS * 1e12) * 1e3
    t_hbm_ms = xw_bytes_per_launch / (PEAK_HBM_GBS * 1e9) * 1e3
    floor = {"t_mfma_ms": t_mfma_ms, "t_hbm_ms": t_hbm_ms, "longer": "hbm" if t_hbm_ms > t_mfma_ms else "mfma",
             "frac_of_longer": max(t_mfma_ms, t_hbm_ms) / avg_xw_ms}
    xw = {"achieved": xw_tflops, "frac": xw_tflops / PEAK_BF16_TFLOPS, "avg_launch_ms": avg_xw_ms,
          "launches": n_xw, "flops_per_launch": xw_flops_per_launch,
          "algorithmic_bytes_per_launch": xw_bytes_per_launch, "floor": floor}
    return xw, others


def xw_roofline(xw, workload):
    """The roofline object of the gemm_xw launch, on the roof that binds it."""
    ms = xw["avg_launch_ms"]
    mfma = {"achieved": xw["achieved"], "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s", "frac": xw["frac"]}
    gbs = xw["algorithmic_bytes_per_launch"] / (ms * 1e-3) / 1e9
    hbm = {"achieved": gbs, "peak": PEAK_HBM_GBS, "unit": "GB/s", "frac": gbs / PEAK_HBM_GBS}
    bound = xw["floor"]["longer"]
    top = dict(hbm if bound == "hbm" else mfma)
    out = {"bound": bound}
    out.update(top)
    out.update({
        "traffic": PROFILED_XW_TRAFFIC_BYTES.get(workload),
        "traffic_source": PROFILED_XW_TRAFFIC_SOURCE if workload in PROFILED_XW_TRAFFIC_BYTES else None,
        "algorithmic_bytes_per_launch": xw["algorithmic_bytes_per_launch"],
        "flops_per_launch": xw["flops_per_launch"],
        "mfma": mfma, "hbm": hbm, "floor": xw["floor"],
        "kernel": "gemm_xw (grouped bf16 GEMM: gate-up, down, dH, dX)",
        "avg_launch_ms": ms, "launches": xw["launches"]})
    return out


def run_workload(name, a, steps, warmup, keep=False):
    """Allocates the synthetic inputs of one workload on the device, times `steps` whole steps."""
    import torch
    import paper_2605_06665_amd as U
    from paper_2605_06665_amd.pipeline import PoolStep
    from synth import workloads as W
    w = W.WORKLOADS[name]
    dev = torch.device("cuda:0")
    dtype = U.BF16 if w.dtype == "bf16" else U.F32
    xs = [W.gen_x_torch(w, l, dev) for l in range(w.L)]
    wrs = [W.gen_w_router_torch(w, l, dev) for l in range(w.L)]
    gs = [W.gen_grad_out_torch(w, l, dev) for l in range(w.L)]
    wg, wu, wd = W.gen_pool_weights_torch(w, dev)
    wgu = torch.cat([wg, wu], dim=1).contiguous()
    sigmas = [w.sigma] * w.L
    ps = PoolStep(w.T, w.d, w.f, w.E, w.k, w.L, dtype, w.c, w.eps, w.alpha, device=dev, wgrad=a.wgrad,
                  recompute=a.recompute, lagged=a.lagged)
    for _ in range(warmup):
        ps.step(xs, wrs, sigmas, wgu, wd, gs)
    torch.cuda.synchronize()
    ps.timing = True                      # HIP events around the entry points, on the launch stream
    ps.events = []
    t0 = time.perf_counter()
    for _ in range(steps):
        ps.step(xs, wrs, sigmas, wgu, wd, gs)
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    agg = {}
    for ename, e0, e1 in ps.events:
        agg.setdefault(ename, []).append(e0.elapsed_time(e1))
    ps.events = []
    ps.timing = False
    res = dict(w=w, ms_step=dt / steps * 1e3, agg=agg, ps=ps)
    if not a.step_only and not a.lagged:
        # the same step recorded once into a HIP graph and replayed: what the launches cost on the host side
        # (a side figure: if recording fails the headline stands and the reason is reported in its place)
        try:
            graph = ps.capture(xs, wrs, sigmas, wgu, wd, gs)
            graph.replay()
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            for _ in range(steps):
                graph.replay()
            torch.cuda.synchronize()
            res["ms_step_graph"] = (time.perf_counter() - t0) / steps * 1e3
            del graph
        except Exception as exc:          # noqa: BLE001
            res["graph_error"] = "%s: %s" % (type(exc).__name__, exc)
            torch.cuda.synchronize()
    if keep:
        res.update(xs=xs, wrs=wrs, gs=gs, wg=wg, wu=wu, wd=wd, wgu=wgu)
    return res


def main():
    a = parse()
    if a.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs on one GPU only (no collectives, no sharding); use --gpus 1",
              file=sys.stderr)
        sys.exit(2)
    import torch
    import __graft_entry__ as entry
    entry.ensure_built()
    import paper_2605_06665_amd as U
    from synth import workloads as W

    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    # one plain device-to-device copy of known size (1 GiB read + 1 GiB write): the reference
    # against which the HBM byte counters of a profiler run are scaled
    cal_src = torch.empty(1 << 28, dtype=torch.float32, device=dev).fill_(1.0)
    cal_dst = torch.empty_like(cal_src)
    cal_dst.copy_(cal_src)
    del cal_src, cal_dst
    torch.cuda.synchronize()

    r = run_workload(a.workload, a, a.steps, a.warmup, keep=True)
    w, ps, ms_step = r["w"], r["ps"], r["ms_step"]
    xw, others = roofline_of(w, a, ps, r["agg"], a.steps)

    # ---- analysis observables (outside the timed step): Alg. 1 on 1e5 draws, distinct experts per token
    def timed(fn, reps=5):
        fn()
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(reps):
            fn()
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) / reps
    if not a.step_only:
        n_draws = 100000
        gen = torch.Generator(device=dev)
        gen.manual_seed(1)
        draws = torch.randn((n_draws, w.E), generator=gen, device=dev, dtype=torch.float32)
        c_out = torch.zeros(1, dtype=torch.float32, device=dev)
        c_used = torch.zeros(1, dtype=torch.int32, device=dev)
        ms_c = timed(lambda: U.estimate_c(w.E, w.k, draws, c_out, c_used, ps.ws))
        idx_tab = torch.tensor([st.topk_idx.data_ptr() for st in ps.layers], dtype=torch.int64, device=dev)
        dist = torch.zeros(w.T, dtype=torch.int32, device=dev)
        dist_mean = torch.zeros(1, dtype=torch.float32, device=dev)
        ms_u = timed(lambda: U.distinct_experts(ps.shape(1.0), w.L, idx_tab, dist, dist_mean, ps.ws))
        by_c, by_u = 4.0 * n_draws * w.E, 4.0 * w.L * w.T * w.k + 4.0 * w.T
        others["estimate_c"] = {"GB/s": by_c / (ms_c * 1e-3) / 1e9, "frac": by_c / (ms_c * 1e-3) / 1e9 / PEAK_HBM_GBS,
                                "avg_ms": ms_c, "algorithmic_bytes": by_c, "draws": n_draws, "c": float(c_out.item())}
        others["distinct_experts"] = {"GB/s": by_u / (ms_u * 1e-3) / 1e9, "frac": by_u / (ms_u * 1e-3) / 1e9 / PEAK_HBM_GBS,
                                      "avg_ms": ms_u, "algorithmic_bytes": by_u,
                                      "mean_distinct_per_token": float(dist_mean.item())}

    # ---- forward pass alone, with the permuted copy and with the dispatch fused into the first GEMM
    if not a.step_only:
        fwd = {}
        for mode, gather in (("materialised", False), ("gathered", True)):
            def fwd_all(gather=gather):
                for l in range(w.L):
                    ps.forward_layer(l, r["xs"][l], r["wrs"][l], w.sigma, r["wgu"], r["wd"], gather=gather)
            fwd[mode + "_ms_per_forward"] = timed(fwd_all, reps=3)
        fwd["gather_speedup"] = fwd["materialised_ms_per_forward"] / fwd["gathered_ms_per_forward"]
        others["forward_only_dispatch"] = fwd

    if "graph_error" in r:
        others["step_as_graph"] = {"error": r["graph_error"]}
    if "ms_step_graph" in r:
        others["step_as_graph"] = {"ms_per_step": r["ms_step_graph"], "eager_ms_per_step": ms_step,
                                   "note": "the same step replayed from a HIP graph; `value` is the eager step"}
    out = {
        "metric": "shared-pool MoE layer fwd+bwd tokens/s; grouped-GEMM % bf16 MFMA peak",
        "value": w.L * w.T / (ms_step * 1e-3), "unit": "tokens/s", "n_gpus": 1, "steps": a.steps,
        "warmup": a.warmup, "ms_per_step": ms_step, "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": w.dtype, "data": "synthetic",
        "config": {"workload": w.name, "L": w.L, "E": w.E, "d_model": w.d, "d_ff": w.f, "top_k": w.k,
                   "tokens_per_layer": w.T, "skew": w.skew, "wgrad": a.wgrad, "recompute": a.recompute,
                   "lagged_statistic": a.lagged,
                   "tokens_counted": "L*T token-layer evaluations per step"},
        # gemm_xw is a bf16 contraction below the ridge point at these group sizes: the roof that binds it is the
        # longer of its MFMA time and its HBM time at the published peaks ("floor").  The headline figures are
        # those of that roof; "mfma" and "hbm" give the launch against each roof.
        "roofline": xw_roofline(xw, a.workload),
        "roofline_others": others,
    }
    if not a.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(w, r["xs"][0], r["wrs"][0], r["gs"][0], r["wg"], r["wu"], r["wd"],
                                           a.oracle_tokens)
    # ---- the other workloads: a few steps each, same library, no CPU baseline
    if a.other_workloads:
        del r, ps
        torch.cuda.empty_cache()
        summary = {}
        for name in a.other_workloads.split(","):
            if name == a.workload:
                continue
            ro = run_workload(name, a, a.other_steps, 1)
            wo = ro["w"]
            xo, oo = roofline_of(wo, a, ro["ps"], ro["agg"], a.other_steps)
            summary[name] = {
                "workload": wo.name, "ms_per_step": ro["ms_step"], "tokens/s": wo.L * wo.T / (ro["ms_step"] * 1e-3),
                "steps": a.other_steps, "ms_per_step_as_graph": ro.get("ms_step_graph"),
                "gemm_xw_frac_mfma": xo["frac"], "gemm_xw_avg_launch_ms": xo["avg_launch_ms"],
                "gemm_xw_floor": xo["floor"],
                "gemm_all_frac_mfma": oo["grouped_gemm_all"]["frac"],
                "wgrad_pool_frac_mfma": oo.get("wgrad_pool", {}).get("frac"),
                "route_frac_hbm": oo["route"]["frac"], "route_ms": oo["route"]["avg_ms"],
                "permute_frac_hbm": oo["permute"]["frac"], "permute_ms": oo["permute"]["avg_ms"],
                "combine_frac_hbm": oo["combine"]["frac"], "combine_bwd_frac_hbm": oo["combine_bwd"]["frac"],
                "route_bwd_frac_hbm": oo["route_bwd"]["frac"], "route_bwd_ms": oo["route_bwd"]["avg_ms"],
            }
            del ro
            torch.cuda.empty_cache()
        out["workloads"] = summary
    print(json.dumps(out))


if __name__ == "__main__":
    main()

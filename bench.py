#!/usr/bin/env python3
"""Benchmark of the Switch FFN layer (forward + backward) on one MI355X.

A step is one pass of the whole hot path -- router, dispatch, two grouped
expert GEMMs, combine, and the full backward -- over one synthetic batch that
is already resident in HBM.  Prints ONE JSON line:

  value        tokens/s = T / (time of one forward + backward), all T input
               tokens counted (dropped ones included)
  roofline     the kernel with the largest share of the step: algorithmic
               FLOPs (or bytes) per launch / its average duration, measured
               with HIP events on the launch stream, against the MI355X peak
  kernels      the same figures for every kernel of the path
  cpu_baseline the fp64 CPU oracle timed on this machine's host cores on a bounded
               sample of the same workload (reported baseline, not a target)
  other_workloads  the other layer shapes of the paper's model table, timed after
               the headline measurement (ms per step, tokens/s, GEMM share of peak)

Usage: python bench.py [--gpus 1] [--steps K] [--warmup W] [--config base_cf1.0]
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_MFMA_BF16 = 2.5e15      # dense bf16 MFMA, FLOP/s
PEAK_FP32 = 157.3e12         # fp32 vector / matrix, FLOP/s
PEAK_HBM = 8.0e12            # bytes/s


def kernel_work(shape, kept, elt):
    """Algorithmic work per launch: name -> (flops, bytes, bound).  `kept` is
    the number of tokens that fit their expert's capacity; padding slots and
    dropped tokens are neither computed nor counted."""
    T, d, f, E = shape.T, shape.d_model, shape.d_ff, shape.E
    gemm = 2.0 * kept * d * f
    w_bytes = float(E) * d * f * elt
    f1 = 2 * f if shape.ffn == "geglu" else f          # columns of W_in
    gemm_in = 2.0 * kept * d * f1
    w_in_bytes = float(E) * d * f1 * elt
    geglu = {
        # gated-GELU FFN: plain first-layer product, streaming activation kernels
        "gemm1_fwd": (gemm_in, w_in_bytes + kept * (d + f1) * elt, "mfma"),
        "geglu_fwd": (0.0, kept * (f1 + f) * elt, "hbm"),
        "gemm2_dgrad": (gemm, w_bytes + kept * (d + f) * elt, "mfma"),
        "geglu_bwd": (0.0, kept * (f1 + f + f1) * elt, "hbm"),
        "gemm1_dgrad": (gemm_in, w_in_bytes + kept * (f1 + d) * elt, "mfma"),
        "gemm1_wgrad": (gemm_in, w_in_bytes + kept * (d + f1) * elt, "mfma"),
    } if shape.ffn == "geglu" else {}
    jit = shape.jitter_eps > 0
    zero_with_positions = (shape.dtype == "bf16" and shape.fused_dispatch and
                           shape.ntlb_rounds == 0)
    dpad = -(-d // 32) * 32
    x_router = T * 3 * dpad * 2 if jit else T * d * elt     # bytes of the router's input operand
    return {**{
        "router_jitter_split": (0.0, T * d * elt + T * 3 * dpad * 2, "hbm"),
        "router_dx_jitter": (0.0, 2.0 * T * d * elt + kept * d * elt + T * 4, "hbm"),
        "router_split_weights": (0.0, d * E * 4 + 3 * 128 * d * 2 + d * 512, "hbm"),
        "router_fwd_mfma": (6.0 * T * d * E, x_router + T * E * 4 + T * 12, "hbm"),
        "router_logits": (2.0 * T * d * E, T * d * elt + T * E * 4 + d * E * 4, "hbm"),
        "router_softmax_top1": (0.0, 2.0 * T * E * 4 + T * 8, "hbm"),
        "route_scan_aux": (0.0, 3.0 * (T / 256.0) * E * 4, "hbm"),
        # (with dispatch / combine inside the GEMMs and no re-routing stages it also clears the
        # rows of y of the tokens without a slot)
        "positions": (0.0, T * (4 + 4 + 4 + 4 + 1 + 4 + 1) +
                      ((T - kept) * d * elt if zero_with_positions else 0), "hbm"),
        "dispatch_gather": (0.0, 2.0 * kept * d * elt, "hbm"),
        # dispatch / combine inside the GEMMs: what is left of the two passes
        "zero_dropped": (0.0, T * 4.0 + (T - kept) * d * elt, "hbm"),
        "gate_grad": (0.0, 2.0 * kept * d * elt + T * 12.0, "hbm"),
        "gemm1_fwd_relu": (gemm, w_bytes + kept * (d + f) * elt + kept * f / 8.0, "mfma"),
        "gemm2_fwd": (gemm, w_bytes + kept * (f + d) * elt, "mfma"),
        "combine_scatter": (0.0, kept * d * elt + T * d * elt + T * 4, "hbm"),
        "combine_bwd": (0.0, 3.0 * kept * d * elt + T * 8, "hbm"),
        "gemm2_dgrad_relumask": (gemm, w_bytes + kept * (d + f) * elt + kept * f / 8.0, "mfma"),
        "gemm2_wgrad": (gemm, w_bytes + kept * (f + d) * elt, "mfma"),
        "gemm1_dgrad": (gemm, w_bytes + kept * (f + d) * elt, "mfma"),
        "gemm1_wgrad": (gemm, w_bytes + kept * (d + f) * elt, "mfma"),
        "router_dlogits": (0.0, T * E * 4 + T * 512 + T * 8, "hbm"),
        "router_dx_mfma": (6.0 * T * d * E, T * 512 + kept * d * elt + T * d * elt, "hbm"),
        "router_dWr_mfma": (4.0 * T * d * E, (T * 2 * dpad * 2 if jit else T * d * elt) + T * 512, "hbm"),
        "router_dWr_reduce": (0.0, -(-T // (-(-(-(-T // 85)) // 64) * 64)) * d * 256 * 4.0 + d * E * 4.0, "hbm"),
        "router_dx": (2.0 * T * d * E, T * E * 4 + kept * d * elt + T * d * elt, "hbm"),
        "router_dWr": (2.0 * T * d * E, T * d * elt + T * E * 4, "hbm"),
        "router_dbr": (0.0, T * E * 4.0, "hbm"),
        # per stage: the logits rows of the waiting tokens are not known in advance; priced
        # with the token-sized tables the four kernels always stream
        "ntlb_stages": (0.0, shape.ntlb_rounds * T * 4.0 * 6, "hbm"),
    }, **geglu}


def cpu_baseline(shape, inp, every):
    """Time the oracle on the workload's own configuration (all T tokens routed, the true
    capacity), with the expert FFN forward + backward evaluated for every `every`-th expert
    only; the whole-job rate is the routing time plus the expert time scaled to all kept
    tokens."""
    import numpy as np
    import oracle
    to_np = lambda t: None if t is None else t.float().cpu().numpy()
    x, dy = to_np(inp["x"]), to_np(inp["dy"])
    W_r, b_r, W_in, W_out = (to_np(inp[k]) for k in ("W_r", "b_r", "W_in", "W_out"))
    threads = oracle.max_threads()
    noise = None
    if shape.expert_dropout or shape.jitter_eps:
        noise = (shape.expert_dropout, shape.jitter_eps, shape.noise_seed)
    t0 = time.perf_counter()
    fwd = oracle.forward(x, W_r, W_in, W_out, shape.capacity_factor, shape.alpha, b_r=b_r,
                         n_groups=shape.n_groups, noise=noise, ffn=shape.ffn,
                         ntlb_rounds=shape.ntlb_rounds, skip_ffn=True)
    t_route = time.perf_counter() - t0
    sel = list(range(0, shape.E, max(1, every)))
    kept = fwd["dropped"] == 0
    kept_all = int(kept.sum())
    kept_sel = int((kept & np.isin(fwd["expert_index"], sel)).sum())
    t0 = time.perf_counter()
    fwd["y"] = oracle.expert_ffn(x, W_in, W_out, fwd["expert_index"], fwd["dropped"], fwd["gate"],
                                 expert_sel=sel, noise=noise, ffn=shape.ffn)
    oracle.backward(x, W_r, W_in, W_out, dy, fwd, shape.alpha, 1.0, expert_sel=sel)
    t_expert = time.perf_counter() - t0
    est = t_route + t_expert * (kept_all / max(1, kept_sel))
    return {"value": shape.T / est, "unit": "tokens/s", "cores": threads, "kind": "oracle",
            "sample": "all %d tokens routed at capacity %d (%.1f s); expert FFN forward + backward and "
                      "the router backward over all tokens for %d of %d experts = %d of %d kept "
                      "tokens (%.1f s); value = T / (routing + expert time x %d / %d), extrapolated"
                      % (shape.T, fwd["capacity"], t_route, len(sel), shape.E, kept_sel, kept_all,
                         t_expert, kept_all, kept_sel)}


def measure(shape, steps, warmup, dev="cuda:0"):
    """K timed steps (forward + backward, inputs resident in HBM), then the same K steps with
    every kernel bracketed by HIP events.  Returns (ms per step, ms per step with events,
    per-kernel dict, layer facts, inputs)."""
    import torch
    import paper_2101_03961_amd as sw
    from paper_2101_03961_amd.layer import SwitchLayer
    from synth_inputs import make_inputs
    inp = make_inputs(shape, dev)
    layer = SwitchLayer(shape.T, shape.d_model, shape.d_ff, shape.E, shape.capacity_factor,
                        shape.alpha, shape.dtype, device=dev, n_groups=shape.n_groups,
                        expert_dropout=shape.expert_dropout, jitter_eps=shape.jitter_eps,
                        seed=shape.noise_seed, ffn=shape.ffn, ntlb_rounds=shape.ntlb_rounds,
                        fused_dispatch=shape.fused_dispatch)
    layer.alloc_grads(with_bias=inp["b_r"] is not None)

    def step():
        layer.forward(inp["x"], inp["W_r"], inp["W_in"], inp["W_out"], inp["b_r"])
        layer.backward(inp["dy"], inp["x"], inp["W_r"], inp["W_in"], inp["W_out"], inp["b_r"], 1.0)

    for _ in range(warmup):
        step()
    torch.cuda.synchronize()
    # timed region: K steps, no per-kernel events
    t0 = time.perf_counter()
    for _ in range(steps):
        step()
    torch.cuda.synchronize()
    ms_per_step = (time.perf_counter() - t0) / steps * 1e3
    # same K steps again with every kernel bracketed by HIP events on the launch stream
    sw.switch_profile_enable(True)
    t0 = time.perf_counter()
    for _ in range(steps):
        step()
    torch.cuda.synchronize()
    ms_prof = (time.perf_counter() - t0) / steps * 1e3
    sw.switch_profile_collect()
    prof = sw.switch_profile_read()
    sw.switch_profile_enable(False)

    counts = layer.expert_counts.cpu().numpy().astype("int64")
    kept = shape.T - int(layer.dropped.sum().item())
    elt = 2 if shape.dtype == "bf16" else 4
    work = kernel_work(shape, kept, elt)
    kernels = {}
    for name, (total_ms, launches) in prof.items():
        avg_s = total_ms / launches * 1e-3
        flops, nbytes, bound = work.get(name, (0.0, 0.0, "hbm"))
        entry = {"avg_us": round(avg_s * 1e6, 2), "launches_per_step": launches / steps,
                 "bound": bound}
        if bound == "mfma":
            # a contraction is priced against the matrix peak; its HBM share is given beside it
            # (at 512 tokens per expert these GEMMs need ~0.7 of HBM peak to reach 0.6 of MFMA peak)
            entry.update(achieved=flops / avg_s / 1e12, peak=PEAK_MFMA_BF16 / 1e12,
                         unit="TFLOP/s", frac=flops / avg_s / PEAK_MFMA_BF16,
                         hbm_gbs=nbytes / avg_s / 1e9, hbm_frac=nbytes / avg_s / PEAK_HBM)
        else:
            entry.update(achieved=nbytes / avg_s / 1e9, peak=PEAK_HBM / 1e9, unit="GB/s",
                         frac=nbytes / avg_s / PEAK_HBM)
        kernels[name] = entry
    gemm_names = [k for k in kernels if kernels[k]["bound"] == "mfma"]
    gemm_s = sum(kernels[k]["avg_us"] * kernels[k]["launches_per_step"] for k in gemm_names) * 1e-6
    gemm_flops = sum(work[k][0] for k in gemm_names)
    facts = {"capacity": layer.capacity, "kept_tokens": kept, "dropped_frac": 1.0 - kept / shape.T,
             "count_min_mean_max": [int(counts.min()), float(counts.mean()), int(counts.max())],
             "gemm_tflops": gemm_flops / gemm_s / 1e12 if gemm_s else None,
             "gemm_frac": gemm_flops / gemm_s / PEAK_MFMA_BF16 if gemm_s else None,
             "gemm_ms": gemm_s * 1e3}
    del layer
    return ms_per_step, ms_prof, kernels, facts, inp


OTHER_WORKLOADS = ("base_cf1.25", "base_zipf", "large", "xxl", "c_share")


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--config", default="base_cf1.0")
    ap.add_argument("--cpu-every", type=int, default=8,
                    help="the oracle evaluates every N-th expert's FFN (routing on all tokens)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-other-workloads", action="store_true",
                    help="skip the other model shapes (timed only after the default workload)")
    ap.add_argument("--n-groups", type=int, default=1,
                    help="routing groups (1 = the benchmark's workload; >1 for experiments)")
    ap.add_argument("--expert-dropout", type=float, default=0.0,
                    help="expert dropout rate (0 = the benchmark's workload; >0 for experiments)")
    ap.add_argument("--jitter-eps", type=float, default=0.0,
                    help="input jitter on the router (0 = the benchmark's workload)")
    ap.add_argument("--fused-dispatch", action="store_true",
                    help="dispatch / combine inside the expert GEMMs (for experiments)")
    ap.add_argument("--ntlb-rounds", type=int, default=0,
                    help="No-Token-Left-Behind re-routing stages (0 = the benchmark's workload)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py measures one GPU: this build has no multi-GPU path "
              "(--gpus %d refused; run with --gpus 1)" % args.gpus, file=sys.stderr)
        return 2

    import torch
    from synth_inputs import CONFIGS

    if not torch.cuda.is_available():
        print("bench.py needs a GPU", file=sys.stderr)
        return 2
    shape = CONFIGS[args.config]
    if args.n_groups != 1:
        shape = shape.with_(name="%s_x%dgroups" % (shape.name, args.n_groups), n_groups=args.n_groups)
    if args.expert_dropout or args.jitter_eps:
        shape = shape.with_(name="%s_drop%g_jit%g" % (shape.name, args.expert_dropout, args.jitter_eps),
                            expert_dropout=args.expert_dropout, jitter_eps=args.jitter_eps,
                            noise_seed=2101)
    if args.ntlb_rounds:
        shape = shape.with_(name="%s_ntlb%d" % (shape.name, args.ntlb_rounds),
                            ntlb_rounds=args.ntlb_rounds)
    if args.fused_dispatch:
        shape = shape.with_(name="%s_fused_dispatch" % shape.name, fused_dispatch=True)
    ms_per_step, ms_prof, kernels, facts, inp = measure(shape, args.steps, args.warmup)

    dominant = max(kernels, key=lambda k: kernels[k]["avg_us"] * kernels[k]["launches_per_step"])
    dk = kernels[dominant]
    roofline = {"kernel": dominant, "bound": dk["bound"], "achieved": dk["achieved"],
                "peak": dk["peak"], "unit": dk["unit"], "frac": dk["frac"], "traffic": None,
                "avg_us": dk["avg_us"]}
    if "hbm_frac" in dk:
        roofline["hbm_frac"] = dk["hbm_frac"]
    # HBM bytes per launch measured with rocprofv3 FETCH_SIZE + WRITE_SIZE (see profiles/):
    # lines "<config> <kernel> <bytes>"
    traffic_file = os.path.join(ROOT, "profiles", "hbm_traffic.txt")
    if os.path.exists(traffic_file):
        with open(traffic_file) as fh:
            for ln in fh:
                parts = ln.split("#")[0].split()
                if len(parts) == 3 and parts[0] == shape.name and parts[1] == dominant:
                    roofline["traffic"] = float(parts[2])
                    roofline["traffic_source"] = ("profiles/hbm_traffic.txt: rocprofv3 FETCH_SIZE + "
                                                  "WRITE_SIZE of an earlier run of this command, "
                                                  "not measured in this run")

    line = {
        "metric": "Switch-layer fwd+bwd tokens/sec at Switch-Base shape",
        "value": shape.T / (ms_per_step * 1e-3),
        "unit": "tokens/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_per_step,
        "ms_per_step_with_kernel_events": ms_prof,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": shape.dtype, "data": "synthetic",
        "config": {"workload": shape.name, "T": shape.T, "d_model": shape.d_model,
                   "d_ff": shape.d_ff, "ffn": shape.ffn, "E": shape.E,
                   "capacity_factor": shape.capacity_factor,
                   "n_groups": shape.n_groups, "expert_dropout": shape.expert_dropout,
                   "jitter_eps": shape.jitter_eps, "ntlb_rounds": shape.ntlb_rounds,
                   "capacity": facts["capacity"], "kept_tokens": facts["kept_tokens"],
                   "dropped_frac": facts["dropped_frac"],
                   "count_min_mean_max": facts["count_min_mean_max"]},
        "roofline": roofline,
        "expert_gemms": {"tflops": facts["gemm_tflops"],
                         "frac_of_bf16_mfma_peak": facts["gemm_frac"], "ms": facts["gemm_ms"]},
        "kernels": kernels,
    }
    if not args.no_cpu_baseline:
        line["cpu_baseline"] = cpu_baseline(shape, inp, args.cpu_every)
    del inp
    torch.cuda.empty_cache()
    if shape.name == "base_cf1.0" and not args.no_other_workloads:
        # the other layer shapes of the model table: 5 warm-up + 20 timed steps each
        others = {}
        for name in OTHER_WORKLOADS:
            s2 = CONFIGS[name]
            ms2, _, k2, f2, inp2 = measure(s2, 20, 5)
            del inp2
            torch.cuda.empty_cache()
            slowest = max(k2, key=lambda k: k2[k]["avg_us"] * k2[k]["launches_per_step"])
            others[name] = {"T": s2.T, "d_model": s2.d_model, "d_ff": s2.d_ff, "E": s2.E,
                            "capacity_factor": s2.capacity_factor, "capacity": f2["capacity"],
                            "kept_tokens": f2["kept_tokens"], "ms_per_step": ms2,
                            "tokens_per_s": s2.T / (ms2 * 1e-3),
                            "expert_gemms_frac_of_bf16_mfma_peak": f2["gemm_frac"],
                            "expert_gemms_ms": f2["gemm_ms"], "slowest_kernel": slowest,
                            "slowest_kernel_us": k2[slowest]["avg_us"],
                            "slowest_kernel_frac": k2[slowest]["frac"]}
        line["other_workloads"] = others
    print(json.dumps(line))
    return 0


if __name__ == "__main__":
    sys.exit(main())

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
        "positions": (0.0, T * (4 + 4 + 4 + 4 + 1 + 4 + 1), "hbm"),
        "dispatch_gather": (0.0, 2.0 * kept * d * elt, "hbm"),
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


def cpu_baseline(shape, inp, sample_tokens):
    """Time the oracle (forward + backward) on the first `sample_tokens` tokens of
    the batch with the full set of expert weights."""
    import numpy as np
    import oracle
    n = min(sample_tokens, shape.T)
    n -= n % shape.n_groups
    to_np = lambda t: None if t is None else t.float().cpu().numpy()
    x, dy = to_np(inp["x"][:n]), to_np(inp["dy"][:n])
    W_r, b_r, W_in, W_out = (to_np(inp[k]) for k in ("W_r", "b_r", "W_in", "W_out"))
    threads = oracle.max_threads()
    t0 = time.perf_counter()
    noise = None
    if shape.expert_dropout or shape.jitter_eps:
        noise = (shape.expert_dropout, shape.jitter_eps, shape.noise_seed)
    fwd = oracle.forward(x, W_r, W_in, W_out, shape.capacity_factor, shape.alpha, b_r=b_r,
                         n_groups=shape.n_groups, noise=noise, ffn=shape.ffn,
                         ntlb_rounds=shape.ntlb_rounds)
    oracle.backward(x, W_r, W_in, W_out, dy, fwd, shape.alpha, 1.0)
    dt = time.perf_counter() - t0
    return {"value": n / dt, "unit": "tokens/s", "cores": threads, "kind": "oracle",
            "sample": "first %d tokens of the batch (capacity %d), all %d experts' weights, "
                      "forward + backward, %.1f s" % (n, fwd["capacity"], shape.E, dt)}


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--config", default="base_cf1.0")
    ap.add_argument("--cpu-sample-tokens", type=int, default=8192)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--n-groups", type=int, default=1,
                    help="routing groups (1 = the benchmark's workload; >1 for experiments)")
    ap.add_argument("--expert-dropout", type=float, default=0.0,
                    help="expert dropout rate (0 = the benchmark's workload; >0 for experiments)")
    ap.add_argument("--jitter-eps", type=float, default=0.0,
                    help="input jitter on the router (0 = the benchmark's workload)")
    ap.add_argument("--ntlb-rounds", type=int, default=0,
                    help="No-Token-Left-Behind re-routing stages (0 = the benchmark's workload)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py measures one GPU: this build has no multi-GPU path "
              "(--gpus %d refused; run with --gpus 1)" % args.gpus, file=sys.stderr)
        return 2

    import torch
    import paper_2101_03961_amd as sw
    from paper_2101_03961_amd.layer import SwitchLayer
    from synth_inputs import CONFIGS, make_inputs

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
    dev = "cuda:0"
    inp = make_inputs(shape, dev)
    layer = SwitchLayer(shape.T, shape.d_model, shape.d_ff, shape.E, shape.capacity_factor,
                        shape.alpha, shape.dtype, device=dev, n_groups=shape.n_groups,
                        expert_dropout=shape.expert_dropout, jitter_eps=shape.jitter_eps,
                        seed=shape.noise_seed, ffn=shape.ffn, ntlb_rounds=shape.ntlb_rounds)
    layer.alloc_grads(with_bias=inp["b_r"] is not None)

    def step():
        layer.forward(inp["x"], inp["W_r"], inp["W_in"], inp["W_out"], inp["b_r"])
        layer.backward(inp["dy"], inp["x"], inp["W_r"], inp["W_in"], inp["W_out"], inp["b_r"], 1.0)

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()

    # timed region: K steps, no per-kernel events
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    ms_per_step = elapsed / args.steps * 1e3

    # same K steps again with every kernel bracketed by HIP events on the launch stream
    sw.switch_profile_enable(True)
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    elapsed_prof = time.perf_counter() - t0
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
        entry = {"avg_us": round(avg_s * 1e6, 2), "launches_per_step": launches / args.steps,
                 "bound": bound}
        if bound == "mfma":
            entry.update(achieved=flops / avg_s / 1e12, peak=PEAK_MFMA_BF16 / 1e12,
                         unit="TFLOP/s", frac=flops / avg_s / PEAK_MFMA_BF16)
        else:
            entry.update(achieved=nbytes / avg_s / 1e9, peak=PEAK_HBM / 1e9, unit="GB/s",
                         frac=nbytes / avg_s / PEAK_HBM)
        kernels[name] = entry
    dominant = max(kernels, key=lambda k: kernels[k]["avg_us"] * kernels[k]["launches_per_step"])
    dk = kernels[dominant]
    roofline = {"kernel": dominant, "bound": dk["bound"], "achieved": dk["achieved"],
                "peak": dk["peak"], "unit": dk["unit"], "frac": dk["frac"], "traffic": None,
                "avg_us": dk["avg_us"]}
    # HBM bytes per launch measured with rocprofv3 FETCH_SIZE + WRITE_SIZE (see profiles/):
    # lines "<config> <kernel> <bytes>"
    traffic_file = os.path.join(ROOT, "profiles", "hbm_traffic.txt")
    if os.path.exists(traffic_file):
        with open(traffic_file) as fh:
            for ln in fh:
                parts = ln.split("#")[0].split()
                if len(parts) == 3 and parts[0] == args.config and parts[1] == dominant:
                    roofline["traffic"] = float(parts[2])
    gemm_names = [k for k in kernels if kernels[k]["bound"] == "mfma"]
    gemm_s = sum(kernels[k]["avg_us"] * kernels[k]["launches_per_step"] for k in gemm_names) * 1e-6
    gemm_flops = sum(work[k][0] for k in gemm_names)

    line = {
        "metric": "Switch-layer fwd+bwd tokens/sec at Switch-Base shape",
        "value": shape.T / (ms_per_step * 1e-3),
        "unit": "tokens/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_per_step,
        "ms_per_step_with_kernel_events": elapsed_prof / args.steps * 1e3,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": shape.dtype, "data": "synthetic",
        "config": {"workload": shape.name, "T": shape.T, "d_model": shape.d_model,
                   "d_ff": shape.d_ff, "ffn": shape.ffn, "E": shape.E,
                   "capacity_factor": shape.capacity_factor,
                   "n_groups": shape.n_groups, "expert_dropout": shape.expert_dropout,
                   "jitter_eps": shape.jitter_eps, "ntlb_rounds": shape.ntlb_rounds,
                   "capacity": layer.capacity, "kept_tokens": kept,
                   "dropped_frac": 1.0 - kept / shape.T,
                   "count_min_mean_max": [int(counts.min()), float(counts.mean()), int(counts.max())]},
        "roofline": roofline,
        "expert_gemms": {"tflops": gemm_flops / gemm_s / 1e12 if gemm_s else None,
                         "frac_of_bf16_mfma_peak": gemm_flops / gemm_s / PEAK_MFMA_BF16 if gemm_s else None,
                         "ms": gemm_s * 1e3},
        "kernels": kernels,
    }
    if not args.no_cpu_baseline:
        line["cpu_baseline"] = cpu_baseline(shape, inp, args.cpu_sample_tokens)
    print(json.dumps(line))
    return 0


if __name__ == "__main__":
    sys.exit(main())
